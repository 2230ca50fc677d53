"""Are the pins sharp?  Plant one plausible mistake at a time in a copy of the
oracle's source and check that the pin suite rejects every one of them.  The
mistakes are planted in the oracle, on the CPU; nothing here touches a GPU."""

import os
import sys
import types

import pytest

import test_oracle_pins as pins
import test_oracle_mailbox as mailbox
import test_oracle_mpich_paths as paths
import test_oracle_smp as smp

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                   "oracle", "bcast_oracle.py")

MUTANTS = {
    "chunk size rounded down": (
        "return (n + P - 1) // P", "return max(1, n // P)"),
    "negative chunk count not clamped": (
        "    if count < 0:\n        count = 0\n", ""),
    "relative rank measured the wrong way round": (
        "return rank - root if rank >= root else rank - root + P",
        "return root - rank if root >= rank else root - rank + P"),
    "scatter hands over the lower half": (
        "disp, _ = chunk_extent(child, n, P)\n            length = sum(chunk_extent(c, n, P)[1] for c in range(child, upper_end))",
        "disp, _ = chunk_extent(rho, n, P)\n            length = sum(chunk_extent(c, n, P)[1] for c in range(rho, child))"),
    "scatter levels smallest distance first": (
        "    mask = ceil_pow2(P) // 2\n    while mask >= 1:\n        rows: List[Row] = []",
        "    for mask in [1 << k for k in range(ceil_log2(P))]:\n        rows: List[Row] = []"),
    "switch: own subtree tested before the neighbour's": (
        "    if right % 2 == 0:\n        return len(owned_after_scatter(right, P)), RECV_ONLY\n    return len(owned_after_scatter(rel, P)), SEND_ONLY",
        "    if rel % 2 == 0:\n        return len(owned_after_scatter(rel, P)), SEND_ONLY\n    return len(owned_after_scatter(right, P)), RECV_ONLY"),
    "switch: subtree size not clipped": (
        "    return range(rel, min(rel + span, P))", "    return range(rel, rel + span)"),
    "switch: directions swapped": (
        "    return len(owned_after_scatter(rel, P)), SEND_ONLY", "    return len(owned_after_scatter(rel, P)), RECV_ONLY"),
    "switch: the root not counted as ahead": (
        "    if right % 2 == 0:\n        return len(owned_after_scatter(right, P)), RECV_ONLY",
        "    if right % 2 == 0 and right != 0:\n        return len(owned_after_scatter(right, P)), RECV_ONLY"),
    "switch: span of a subtree head one level short": (
        "    while rel % (2 * span) == 0:\n        span *= 2\n    return range(rel, min(rel + span, P))",
        "    while rel % (4 * span) == 0:\n        span *= 2\n    return range(rel, min(rel + span, P))"),
    "ring: one-direction phase starts a step late": (
        "if i > P - step:", "if i > P - step + 1:"),
    "ring: one-direction phase starts a step early": (
        "if i > P - step:", "if i >= P - step:"),
    "ring: chunks counted to the right": (
        "passing = (r - (i - 1)) % P", "passing = (r + (i - 1)) % P"),
    "ring: first chunk sent is the left neighbour's": (
        "passing = (r - (i - 1)) % P      # rank whose chunk this rank passes on\n            awaiting = (r - i) % P ",
        "passing = (r - i) % P      # rank whose chunk this rank passes on\n            awaiting = (r - i - 1) % P "),
    "ring: chunk looked up by absolute rank": (
        "out_extent = chunk_extent(relative_rank(passing, root, P), n, P)",
        "out_extent = chunk_extent(passing, n, P)"),
    "ring: sends go to the left neighbour": (
        "sends[(r, right)] = out_extent", "sends[(r, left)] = out_extent"),
    "delivery lands at the wrong offset": (
        "bufs[dst][off:off + length] = data", "bufs[dst][off - length:off] = data[:len(bufs[dst][off - length:off])]"),
    "delivery reads the receiver's buffer": (
        "payloads = [bufs[src][off:off + length].copy() for (src, _dst, off, length) in rows]",
        "payloads = [bufs[_dst][off:off + length].copy() for (src, _dst, off, length) in rows]"),
    "binomial: children sent a chunk instead of the message": (
        "rows.append((absolute_rank(rho, root, P), absolute_rank(child, root, P), 0, n))",
        "rows.append((absolute_rank(rho, root, P), absolute_rank(child, root, P), 0, scatter_size(n, P)))"),
    "binomial: levels smallest distance first": (
        "    posted: List[int] = []\n    mask = ceil_pow2(P) // 2\n    while mask >= 1:",
        "    posted: List[int] = []\n    for mask in [1 << k for k in range(ceil_log2(P))]:"),
    "doubling: partner one rank away instead of one bit away": (
        "partner = rho ^ dist", "partner = (rho + dist) % P"),
    "doubling: only the own chunk is swapped": (
        "s_count = sum(chunk_extent(c, n, P)[1] for c in range(mine, mine + dist))",
        "s_count = chunk_extent(rho, n, P)[1]"),
    "doubling: block start not aligned": (
        "mine = (rho // dist) * dist          # block gathered so far", "mine = rho"),
    "selection: long threshold off by one": (
        "if n < LONG_MSG_BYTES and P & (P - 1) == 0:", "if n <= LONG_MSG_BYTES and P & (P - 1) == 0:"),
    "selection: short threshold off by one": (
        "if n < SHORT_MSG_BYTES:", "if n <= SHORT_MSG_BYTES:"),
    "selection: power-of-two test inverted": (
        "if n < LONG_MSG_BYTES and P & (P - 1) == 0:", "if n < LONG_MSG_BYTES and P & (P - 1) != 0:"),
    "census: nodes counted by relative rank": (
        'kind = "inter" if src // ranks_per_node != dst // ranks_per_node else "intra"',
        'kind = "inter" if ((src - sched.root) % sched.P) // ranks_per_node != ((dst - sched.root) % sched.P) // ranks_per_node else "intra"'),
    "census: ranks dealt round-robin to nodes": (
        'kind = "inter" if src // ranks_per_node != dst // ranks_per_node else "intra"',
        'kind = "inter" if src % ranks_per_node != dst % ranks_per_node else "intra"'),
    "three-phase: middle phase starts at node 0": (
        "build_schedule(len(leaders), root_node, n, ring_algo)", "build_schedule(len(leaders), 0, n, ring_algo)"),
    "three-phase: first phase starts at the node's lowest rank": (
        "build_schedule(len(home), home.index(root), n, BINOMIAL)", "build_schedule(len(home), 0, n, BINOMIAL)"),
    "three-phase: nodes represented by their highest rank": (
        "leaders = [nd[0] for nd in nodes]", "leaders = [nd[-1] for nd in nodes]"),
    "three-phase: the root's node is broadcast to twice": (
        "        if j != root_node:\n            out.append(SubSchedule(3,", "        if True:\n            out.append(SubSchedule(3,"),
    "zero-length rows kept": (
        "for (src, dst), (disp, cnt) in sends.items() if cnt > 0]",
        "for (src, dst), (disp, cnt) in sends.items()]"),
}


def load_mutant(old, new):
    text = open(SRC).read()
    assert text.count(old) >= 1, "mutation site not found - keep this test in step with the oracle"
    mod = types.ModuleType("bcast_oracle_mutant")
    mod.__file__ = SRC
    sys.modules[mod.__name__] = mod      # dataclasses look their module up by name
    exec(compile(text.replace(old, new), SRC, "exec"), mod.__dict__)
    return mod


def run_pin_suite():
    """A compact pass over the pin tests (same functions pytest collects)."""
    pins.test_chunking()
    pins.test_switch_point_values()
    pins.test_scatter_tree_8_processes()
    pins.test_scatter_tree_10_processes()
    for P in (5, 6, 10, 12):
        pins.test_scatter_matches_recursive_halving(P)
    for case in [(10, 3, 1000), (10, 0, 12), (7, 2, 5)]:
        pins.test_state_after_scatter_is_own_subtree_only(*case)
    pins.test_native_ring_forwards_what_arrived(10, 7)
    pins.test_native_ring_count_paper_examples()
    pins.test_tuned_ring_8_processes_narrative()
    pins.test_tuned_ring_10_processes_narrative()
    pins.test_tuned_saving_power_of_two(4)
    for P in (6, 9, 10, 16):
        pins.test_tuned_rule_equals_only_missing_chunks(P)
    for case in [(10, 9, 9), (10, 3, 32), (13, 4, 14), (5, 0, 1000)]:
        pins.test_final_state_is_the_broadcast(*case)
    pins.test_tuned_writes_every_missing_byte_exactly_once(10, 4, 1003)
    pins.test_byte_counts_closed_form(10, 0, 12)
    pins.test_byte_counts_closed_form(33, 7, 20)
    pins.test_degenerate_cases()
    mailbox.test_async_execution_agrees_with_the_tables(10, 5, 32)
    mailbox.test_async_execution_agrees_with_the_tables(9, 8, 10)
    for P in (5, 8, 13):
        paths.test_binomial_broadcast_tree_and_counts(P)
    paths.test_binomial_tree_is_the_scatter_tree_of_the_paper()
    for k in (0, 2, 3):
        paths.test_recursive_doubling_matches_the_set_model(k)
    paths.test_final_state_and_independent_rows(8, 7, 1000)
    paths.test_async_execution(8, 7, 200)
    paths.test_selection_thresholds()
    pins.test_node_census_closed_forms(64, 17, 999_983, 24)
    pins.test_node_census_closed_forms(10, 3, 1000, 4)
    pins.test_node_census_paper_sizes()
    for case in [(9, 4, 5, 4), (17, 16, 12_288, 4), (25, 12, 5, 24), (7, 6, 5, 3)]:
        smp.test_three_phases(*case)


def test_unmutated_oracle_passes_the_compact_suite():
    run_pin_suite()


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_reject_mutant(name, monkeypatch):
    old, new = MUTANTS[name]
    mutant = load_mutant(old, new)
    monkeypatch.setattr(pins, "O", mutant)
    monkeypatch.setattr(mailbox, "O", mutant)
    monkeypatch.setattr(paths, "O", mutant)
    monkeypatch.setattr(smp, "O", mutant)
    with pytest.raises(BaseException) as info:
        run_pin_suite()
    assert not isinstance(info.value, (KeyboardInterrupt, SystemExit))
