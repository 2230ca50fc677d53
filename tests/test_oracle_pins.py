"""Pins for the CPU oracle: what the paper prints and what the mathematics
fixes, none of it computed by the oracle itself.  CPU only."""

import os

import numpy as np
import pytest

from oracle import bcast_oracle as O
import pin_models as M

HERE = os.path.dirname(os.path.abspath(__file__))


def load_paper_numbers():
    out = {}
    with open(os.path.join(HERE, "golden", "paper_worked_examples.txt")) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            k, v = [x.strip() for x in line.split("=")]
            vals = [int(x) for x in v.split()]
            out[k] = vals[0] if len(vals) == 1 else vals
    return out


PAPER = load_paper_numbers()


def chunks_of(row, n, P):
    """Relative chunk indices a row covers (rows move whole chunks)."""
    _src, _dst, off, length = row
    ss = O.scatter_size(n, P)
    assert off % ss == 0
    return list(range(off // ss, (off + length + ss - 1) // ss))


def make_bufs(P, root, n, extra=5, seed=1):
    rng = np.random.default_rng(seed)
    bufs = [rng.integers(0, 256, n + extra, dtype=np.uint8) for _ in range(P)]
    return bufs


# ---------------------------------------------------------------- scatter tree

def test_scatter_tree_8_processes():
    """Sec. III-A, Fig. 1: 0 sends {4,5,6,7} to 4; then 2 and 6 become subtree
    roots; after the third step everyone has its chunk."""
    P, n = 8, 8 * 11
    lv = O.scatter_levels(P, 0, n)
    assert len(lv) == PAPER["scatter_levels_P8"]
    as_sets = [[(s, d, chunks_of((s, d, o, l), n, P)) for (s, d, o, l) in rows] for rows in lv]
    assert as_sets[0] == [(0, 4, [4, 5, 6, 7])]
    assert as_sets[1] == [(0, 2, [2, 3]), (4, 6, [6, 7])]
    assert as_sets[2] == [(0, 1, [1]), (2, 3, [3]), (4, 5, [5]), (6, 7, [7])]


def test_scatter_tree_10_processes():
    """Sec. III-A, Fig. 2: same paths as for 8 plus one more branch rooted at 8;
    ceil(log2 10) = 4 steps."""
    P, n = 10, 10 * 7
    lv = O.scatter_levels(P, 0, n)
    assert len(lv) == PAPER["scatter_levels_P10"]
    as_sets = [[(s, d, chunks_of((s, d, o, l), n, P)) for (s, d, o, l) in rows] for rows in lv]
    assert as_sets[0] == [(0, 8, [8, 9])]
    assert as_sets[1] == [(0, 4, [4, 5, 6, 7])]
    assert as_sets[2] == [(0, 2, [2, 3]), (4, 6, [6, 7])]
    assert as_sets[3] == [(0, 1, [1]), (2, 3, [3]), (4, 5, [5]), (6, 7, [7]), (8, 9, [9])]


@pytest.mark.parametrize("P", list(range(1, 41)) + [63, 64, 65, 127, 129])
def test_scatter_matches_recursive_halving(P):
    """The level loop and a recursive-halving construction of the binomial
    tree give the same edges at the same depth (any root, by rotation)."""
    levels, _ = M.prose_model(P, tuned=False)
    for root in {0, 1, P // 2, P - 1}:
        n = P * 3
        lv = O.scatter_levels(P, root, n)
        assert len(lv) == len(levels) == O.ceil_log2(P)
        for rows, ref in zip(lv, levels):
            got = sorted(((s - root) % P, (d - root) % P, set(chunks_of((s, d, o, l), n, P)))
                         for (s, d, o, l) in rows)
            assert got == ref


@pytest.mark.parametrize("P,root,n", [(8, 0, 80), (10, 3, 1000), (10, 0, 12), (13, 12, 1301),
                                      (24, 3, 4099), (33, 32, 33), (7, 2, 5), (16, 5, 0)])
def test_state_after_scatter_is_own_subtree_only(P, root, n):
    """Sec. III-A: after the scatter a rank holds its own chunk and those of
    its descendants - and, with poisoned buffers, nothing else."""
    bufs = make_bufs(P, root, n)
    init = [b.copy() for b in bufs]
    sched = O.build_schedule(P, root, n, O.NATIVE)
    O.run_steps(bufs, sched, 0, sched.n_scatter_steps)
    subtree = {}
    for (s, r, a, b, h) in M.binomial_tree_messages(P):
        subtree[r] = range(a, b)
    subtree[0] = range(0, P)
    ss = O.scatter_size(n, P)
    for rank in range(P):
        rel = (rank - root) % P
        expect = init[rank].copy()
        lo = min(subtree[rel].start * ss, n)
        hi = min(subtree[rel].stop * ss, n)
        expect[lo:hi] = init[root][lo:hi]
        assert np.array_equal(bufs[rank], expect), (rank, rel)
        assert list(O.owned_after_scatter(rel, P)) == list(subtree[rel])


# ---------------------------------------------------------------- native ring

@pytest.mark.parametrize("P,root", [(8, 0), (10, 0), (10, 7), (17, 4), (2, 1), (3, 0)])
def test_native_ring_forwards_what_arrived(P, root):
    """Sec. III-A, Fig. 3: step 1 sends the own chunk to the right; later steps
    forward what came from the left one step earlier; P transfers per step,
    P (P - 1) in total."""
    n = P * 5
    ring = O.ring_steps(P, root, n, O.NATIVE)
    assert len(ring.steps) == P - 1
    got_last = {}
    for i, rows in enumerate(ring.steps, start=1):
        assert len(rows) == P
        now = {}
        for (src, dst, off, length) in rows:
            assert dst == (src + 1) % P
            (c,) = chunks_of((src, dst, off, length), n, P)
            own = (src - root) % P
            assert c == (own if i == 1 else got_last[src])
            now[dst] = c
        got_last = now
    assert sum(len(r) for r in ring.steps) == P * (P - 1)
    assert sum(ring.posted_sends) == P * (P - 1)


def test_native_ring_count_paper_examples():
    for P, key in [(8, "native_ring_transfers_P8"), (10, "native_ring_transfers_P10")]:
        s = O.build_schedule(P, 0, P * 9, O.NATIVE)
        assert s.ring_rows == PAPER[key] == s.ring_msgs_issued


# ---------------------------------------------------------------- tuned ring, worked examples

def recv_sequence(ring, rank, n, P):
    seq = []
    for rows in ring.steps:
        got = [chunks_of(r, n, P)[0] for r in rows if r[1] == rank]
        assert len(got) <= 1
        seq.append(got[0] if got else None)
    return seq


def test_tuned_ring_8_processes_narrative():
    """Sec. IV, Fig. 4."""
    P, n = 8, 8 * 13
    ring = O.ring_steps(P, 0, n, O.TUNED)
    assert len(ring.steps) == PAPER["ring_steps_P8"]
    # the root does not receive anything from process 7
    assert recv_sequence(ring, 0, n, P) == [None] * 7
    # process 4 gets 3, 2, 1, 0 in the first four steps and nothing afterwards
    want = PAPER["tuned_recv_seq_rank4_P8"]
    assert recv_sequence(ring, 4, n, P) == want + [None] * (7 - len(want))
    # processes 2 and 6 have everything by the seventh step
    for r in PAPER["tuned_done_before_last_P8"]:
        seq = recv_sequence(ring, r, n, P)
        assert None not in seq[:6] and seq[6] is None
    total = sum(len(r) for r in ring.steps)
    assert total == PAPER["native_ring_transfers_P8"] - PAPER["tuned_ring_saving_P8"]


def test_tuned_ring_10_processes_narrative():
    """Sec. IV, Fig. 5."""
    P, n = 10, 10 * 13
    ring = O.ring_steps(P, 0, n, O.TUNED)
    assert len(ring.steps) == 9
    want = PAPER["tuned_recv_seq_rank4_P10"]
    assert recv_sequence(ring, 4, n, P) == want + [None] * (9 - len(want))
    for r in PAPER["tuned_done_before_last_P10"]:
        seq = recv_sequence(ring, r, n, P)
        assert None not in seq[:8] and seq[8] is None
    total = sum(len(r) for r in ring.steps)
    assert total == PAPER["tuned_ring_transfers_P10"]
    assert PAPER["native_ring_transfers_P10"] - total == PAPER["tuned_ring_saving_P10"]


@pytest.mark.parametrize("k", range(1, 11))
def test_tuned_saving_power_of_two(k):
    """Sec. IV (remark on power-of-two process counts): the tuned ring sends
    (P / 2) log2 P fewer chunks."""
    P = 1 << k
    nat = O.ring_steps(P, 0, P, O.NATIVE)
    tun = O.ring_steps(P, 0, P, O.TUNED)
    saved = sum(map(len, nat.steps)) - sum(map(len, tun.steps))
    assert saved == (P // 2) * k


# ---------------------------------------------------------------- prose model == listing rule

@pytest.mark.parametrize("P", range(1, 41))
def test_tuned_rule_equals_only_missing_chunks(P):
    """Sec. IV: a rank receives a chunk only if it still lacks it.  The
    (step, flag) rule must drop exactly the transfers whose receiver already
    holds the chunk, in every step, for every root."""
    for tuned in (False, True):
        _, ring_ref = M.prose_model(P, tuned)
        for root in range(P):
            n = 4 * P - (1 if P > 4 else 0)   # last chunk short, none empty
            ring = O.ring_steps(P, root, n, O.TUNED if tuned else O.NATIVE)
            assert len(ring.steps) == len(ring_ref) == P - 1
            assert ring.posted_sends == [len(ref) for ref in ring_ref]
            for rows, ref in zip(ring.steps, ring_ref):
                got = [((s - root) % P, (d - root) % P, chunks_of((s, d, o, l), n, P)[0])
                       for (s, d, o, l) in rows]
                assert got == ref


@pytest.mark.parametrize("P", [129, 256, 513])
def test_tuned_rule_equals_only_missing_chunks_large(P):
    _, ring_ref = M.prose_model(P, True)
    root = P // 2
    n = 2 * P
    ring = O.ring_steps(P, root, n, O.TUNED)
    for rows, ref in zip(ring.steps, ring_ref):
        got = [((s - root) % P, (d - root) % P, chunks_of((s, d, o, l), n, P)[0])
               for (s, d, o, l) in rows]
        assert got == ref


# ---------------------------------------------------------------- definition of broadcast, per-step state

GRID = [(P, root, n) for P in (1, 2, 3, 5, 8, 10, 13, 16, 24)
        for root in sorted({0, P // 3, P - 1})
        for n in sorted({0, 1, P - 1, P, P + 1, 3 * P + 2, 1000})]


@pytest.mark.parametrize("P,root,n", GRID)
def test_final_state_is_the_broadcast(P, root, n):
    """Sec. III-A: after the call every rank holds the root's message; bytes
    beyond the message are untouched."""
    for algo in (O.NATIVE, O.TUNED):
        bufs = make_bufs(P, root, n, seed=P * 1000 + root)
        want = O.broadcast_definition(bufs, root, n)
        O.run_steps(bufs, O.build_schedule(P, root, n, algo))
        for a, b in zip(bufs, want):
            assert np.array_equal(a, b)


@pytest.mark.parametrize("threads", [1, 3, 8])
@pytest.mark.parametrize("P,root,n", [(1, 0, 5), (2, 1, 9), (8, 0, 800), (10, 4, 1003), (24, 3, 4099), (13, 12, 11)])
def test_rows_of_a_step_over_several_cores(P, root, n, threads):
    """The C byte execution behind the benchmark's all-cores CPU figure
    (oracle/csrc/run_rows.c), in its literal two-phase form and in its direct
    form: after every range of steps the buffers are the ones the plain numpy
    execution leaves, and the end is the definition of broadcast.  The direct
    form is only claimed for schedules whose rows are independent within a step,
    which the C check confirms for both rings and denies for a planted overlap."""
    from oracle import native_rows as N
    for algo in (O.NATIVE, O.TUNED):
        sched = O.build_schedule(P, root, n, algo)
        assert N.rows_independent(sched.steps)
        plain = make_bufs(P, root, n, seed=P * 77 + threads)
        staged = [x.copy() for x in plain]
        direct = [x.copy() for x in plain]
        want = O.broadcast_definition(plain, root, n)
        cuts = sorted({0, sched.n_scatter_steps, sched.n_steps // 2, sched.n_steps})
        for a, b in zip(cuts, cuts[1:]):
            O.run_steps(plain, sched, a, b)
            N.run_rows(staged, sched.steps[a:b], threads, staged=True)
            N.run_rows(direct, sched.steps[a:b], threads, staged=False)
            for x, y, z in zip(plain, staged, direct):
                assert np.array_equal(x, y) and np.array_equal(x, z)
        for x, y in zip(direct, want):
            assert np.array_equal(x, y)
    # a step in which one row reads what another writes is not independent, and
    # only the two-phase form then agrees with the plain execution
    swap = [[(0, 1, 0, 8), (1, 0, 0, 8)]]
    assert not N.rows_independent(swap)
    bufs = [np.arange(16, dtype=np.uint8) + 16 * r for r in range(2)]
    ref = [x.copy() for x in bufs]
    O.apply_step(ref, swap[0])
    N.run_rows(bufs, swap, 2, staged=True)
    assert all(np.array_equal(x, y) for x, y in zip(bufs, ref))


@pytest.mark.parametrize("P,root,n", [(8, 0, 800), (10, 4, 1003), (24, 3, 4099), (13, 12, 11), (16, 1, 4096)])
def test_native_and_tuned_state_identical_after_every_step(P, root, n):
    """The tuned ring only leaves out deliveries of bytes the receiver already
    has, so both variants pass through the same states."""
    a = make_bufs(P, root, n)
    b = [x.copy() for x in a]
    sa = O.build_schedule(P, root, n, O.NATIVE)
    sb = O.build_schedule(P, root, n, O.TUNED)
    assert sa.n_steps == sb.n_steps == O.ceil_log2(P) + P - 1
    for s in range(sa.n_steps):
        O.apply_step(a, sa.steps[s])
        O.apply_step(b, sb.steps[s])
        for x, y in zip(a, b):
            assert np.array_equal(x, y)


@pytest.mark.parametrize("P,root,n", [(8, 0, 800), (10, 4, 1003), (24, 3, 4099), (13, 12, 11), (2, 0, 7), (96, 17, 12345)])
def test_tuned_writes_every_missing_byte_exactly_once(P, root, n):
    """Tuned: every byte of the message is written exactly once into every
    non-root rank and never into the root; native additionally rewrites what
    the scatter delivered."""
    for algo in (O.NATIVE, O.TUNED):
        sched = O.build_schedule(P, root, n, algo)
        writes = np.zeros((P, n), dtype=np.int32)
        for rows in sched.steps:
            for (_s, d, off, length) in rows:
                writes[d, off:off + length] += 1
        if algo == O.TUNED:
            for r in range(P):
                assert (writes[r] == (0 if r == root else 1)).all()
            assert sched.bytes_moved == (P - 1) * n
        else:
            assert sched.bytes_moved == (P - 1) * n + sched.scatter_bytes


@pytest.mark.parametrize("P,root,n", [(8, 0, 800), (10, 4, 1003), (24, 3, 4099), (7, 6, 3)])
def test_rows_of_a_step_never_read_what_another_row_writes(P, root, n):
    for algo in (O.NATIVE, O.TUNED):
        sched = O.build_schedule(P, root, n, algo)
        for rows in sched.steps:
            written = [(d, off, off + ln) for (_s, d, off, ln) in rows]
            for (s, _d, off, ln) in rows:
                for (wd, a, b) in written:
                    assert not (wd == s and a < off + ln and off < b)
            for i, (d1, a1, b1) in enumerate(written):
                for (d2, a2, b2) in written[i + 1:]:
                    assert not (d1 == d2 and a1 < b2 and a2 < b1)


@pytest.mark.parametrize("P,root,n", [(8, 0, 800), (10, 4, 1003), (24, 3, 4099), (13, 12, 11)])
def test_ownership_form_matches_byte_state(P, root, n):
    for algo in (O.NATIVE, O.TUNED):
        sched = O.build_schedule(P, root, n, algo)
        bufs = make_bufs(P, root, n)
        init = [b.copy() for b in bufs]
        for k in range(sched.n_steps + 1):
            if k:
                O.apply_step(bufs, sched.steps[k - 1])
            has = O.ownership_after(sched, k)
            for r in range(P):
                expect = init[r].copy()
                for c in range(P):
                    if has[r, c]:
                        d, cnt = O.chunk_extent(c, n, P)
                        expect[d:d + cnt] = init[root][d:d + cnt]
                assert np.array_equal(bufs[r], expect)


# ---------------------------------------------------------------- closed forms

def popcount(x):
    return bin(x).count("1")


CLOSED = [(10, 0, 524_288), (24, 3, 4_194_304), (64, 0, 16_777_216), (96, 17, 12_345_677),
          (513, 256, 134_217_728), (9, 2, 12_288), (17, 0, 524_287), (129, 5, 2_560_000),
          (10, 0, 12), (33, 7, 20), (256, 255, 30_000_000)]


@pytest.mark.parametrize("P,root,n", CLOSED)
def test_byte_counts_closed_form(P, root, n):
    ss = -(-n // P)
    clen = [max(0, min(ss, n - c * ss)) for c in range(P)]
    assert sum(clen) == n
    # a chunk travels down the tree once per set bit of its relative index
    scatter_bytes = sum(popcount(c) * clen[c] for c in range(P))
    nat = O.build_schedule(P, root, n, O.NATIVE)
    tun = O.build_schedule(P, root, n, O.TUNED)
    assert nat.scatter_bytes == tun.scatter_bytes == scatter_bytes
    # native ring: every rank sends every chunk but its right neighbour's
    assert nat.ring_bytes == (P - 1) * n
    assert nat.ring_msgs_issued == P * (P - 1)
    sent = {}
    for rows in nat.steps[nat.n_scatter_steps:]:
        for (s, _d, _o, ln) in rows:
            sent[s] = sent.get(s, 0) + ln
    for r in range(P):
        rel = (r - root) % P
        assert sent.get(r, 0) == n - clen[(rel + 1) % P]
    # tuned: what the ring leaves out is exactly what the scatter delivered
    assert tun.bytes_moved == (P - 1) * n
    assert nat.bytes_moved == (P - 1) * n + scatter_bytes
    if n >= P:
        assert tun.bytes_moved < nat.bytes_moved
    # messages saved: a subtree of s chunks saves its head s - 1 receives
    def span(rel):
        if rel == 0:
            return P
        return min(rel & -rel, P - rel)
    assert nat.ring_msgs_issued - tun.ring_msgs_issued == sum(span(r) - 1 for r in range(P))
    assert nat.n_steps == tun.n_steps == (P - 1).bit_length() + P - 1


def test_counts_do_not_depend_on_root():
    for P in (8, 10, 24, 33):
        for algo in (O.NATIVE, O.TUNED):
            ref = None
            for root in range(P):
                s = O.build_schedule(P, root, 7 * P + 3, algo)
                sig = (s.step_rows(), s.step_bytes(), s.ring_msgs_issued)
                ref = ref or sig
                assert sig == ref
                # and the tables are the root-0 tables with ranks rotated
                s0 = O.build_schedule(P, 0, 7 * P + 3, algo)
                for rows, rows0 in zip(s.steps, s0.steps):
                    assert rows == [((a + root) % P, (b + root) % P, o, l) for (a, b, o, l) in rows0]


def test_degenerate_cases():
    # one rank: nothing to do
    for algo in (O.NATIVE, O.TUNED):
        s = O.build_schedule(1, 0, 100, algo)
        assert s.n_steps == 0 and s.bytes_moved == 0
    # two ranks: scatter hands chunk 1 over; the one ring step sends chunk 0
    # to rank 1 and - only in the native ring - chunk 1 back to the root
    nat = O.build_schedule(2, 0, 10, O.NATIVE)
    tun = O.build_schedule(2, 0, 10, O.TUNED)
    assert nat.steps == [[(0, 1, 5, 5)], [(0, 1, 0, 5), (1, 0, 5, 5)]]
    assert tun.steps == [[(0, 1, 5, 5)], [(0, 1, 0, 5)]]
    # empty message: steps exist, nothing moves, but the ring calls are still issued
    for P in (1, 2, 5, 8):
        for algo in (O.NATIVE, O.TUNED):
            s = O.build_schedule(P, P - 1, 0, algo)
            assert all(len(r) == 0 for r in s.steps)
            assert s.n_steps == (0 if P == 1 else O.ceil_log2(P) + P - 1)
    assert O.build_schedule(8, 0, 0, O.NATIVE).ring_msgs_issued == 56
    assert O.build_schedule(8, 0, 0, O.TUNED).ring_msgs_issued == 44
    # fewer bytes than ranks: trailing chunks are empty and never travel
    s = O.build_schedule(10, 0, 12, O.TUNED)   # ss = 2, chunks 6..9 empty
    assert [O.chunk_extent(c, 12, 10)[1] for c in range(10)] == [2] * 6 + [0] * 4
    assert s.ring_msgs_issued == 75 and s.ring_rows < 75


def test_switch_point_values():
    """(step, flag) for the paper's 8-process example, read off Fig. 4: the
    root and ranks 2, 4, 6 head subtrees of 8, 2, 4, 2 chunks (send-only
    tails); their left neighbours 7, 1, 3, 5 get the matching receive-only
    tails."""
    got = [O.tuned_switch(r, 8) for r in range(8)]
    assert got == [(8, O.SEND_ONLY), (2, O.RECV_ONLY), (2, O.SEND_ONLY), (4, O.RECV_ONLY),
                   (4, O.SEND_ONLY), (2, O.RECV_ONLY), (2, O.SEND_ONLY), (8, O.RECV_ONLY)]
    assert O.tuned_switch(0, 1) is None
    # 10 processes: rank 8 heads a clipped subtree {8, 9}
    assert O.tuned_switch(8, 10) == (2, O.SEND_ONLY)
    assert O.tuned_switch(7, 10) == (2, O.RECV_ONLY)
    assert O.tuned_switch(9, 10) == (10, O.RECV_ONLY)


def test_chunking():
    assert O.scatter_size(524_288, 10) == 52_429
    assert O.chunk_extent(9, 524_288, 10) == (471_861, 52_427)
    assert O.chunk_extent(5, 12, 10) == (10, 2)
    assert O.chunk_extent(6, 12, 10) == (12, 0)
    assert O.chunk_extent(9, 12, 10) == (18, 0)
    assert [O.ceil_pow2(p) for p in (1, 2, 3, 8, 9, 10, 513)] == [1, 2, 4, 8, 16, 16, 1024]
    assert [O.relative_rank(r, 3, 5) for r in range(5)] == [2, 3, 4, 0, 1]
    assert [O.absolute_rank(O.relative_rank(r, 3, 5), 3, 5) for r in range(5)] == list(range(5))


# ---------------------------------------------------------------- node census

@pytest.mark.parametrize("P,root,n,rpn", [(16, 0, 524_288, 24), (64, 0, 3_000_000, 24), (64, 17, 999_983, 24),
                                          (256, 5, 524_288, 24), (129, 128, 12_288, 24), (10, 3, 1000, 4),
                                          (48, 47, 4800, 24), (50, 0, 77, 7)])
def test_node_census_closed_forms(P, root, n, rpn):
    """Sec. V-A: ranks are placed on the nodes in blocks (24 per node on the
    paper's cluster), so 16 processes never leave their node.  Closed forms for
    the ring: a step uses every ring edge once, an edge (r -> r+1) carries every
    chunk but the receiver's own, and the tuned ring drops the receiver's last
    span - 1 receives."""
    ss = -(-n // P)
    clen = [max(0, min(ss, n - c * ss)) for c in range(P)]
    rel = lambda r: (r - root) % P
    crossing = [r for r in range(P) if r // rpn != ((r + 1) % P) // rpn]
    nodes = -(-P // rpn)
    assert len(crossing) == (nodes if nodes > 1 else 0)

    def span(c):
        return P if c == 0 else min(c & -c, P - c)

    nat = O.node_census(O.build_schedule(P, root, n, O.NATIVE), rpn)
    tun = O.node_census(O.build_schedule(P, root, n, O.TUNED), rpn)
    empty = sum(1 for c in range(P) if clen[c] == 0)
    # native: every crossing edge carries P - 1 chunks, the empty ones excepted
    want_msgs = sum((P - 1) - (empty - (1 if clen[rel((r + 1) % P)] == 0 else 0)) for r in crossing)
    want_bytes = sum(n - clen[rel((r + 1) % P)] for r in crossing)
    assert nat["ring_inter_msgs"] == want_msgs and nat["ring_inter_bytes"] == want_bytes
    assert nat["ring_inter_bytes"] + nat["ring_intra_bytes"] == (P - 1) * n
    # tuned: the receiver behind a crossing edge already holds its subtree's chunks
    t_bytes = 0
    for r in crossing:
        c = rel((r + 1) % P)
        held = sum(clen[(c + k) % P] for k in range(span(c)))
        t_bytes += n - held
    assert tun["ring_inter_bytes"] == t_bytes
    assert tun["ring_inter_msgs"] <= nat["ring_inter_msgs"]
    assert tun["scatter_inter_bytes"] == nat["scatter_inter_bytes"]
    total = sum(v for k, v in tun.items() if k.endswith("bytes"))
    assert total == (P - 1) * n
    if P <= rpn:
        assert nat["ring_inter_msgs"] == nat["scatter_inter_msgs"] == 0   # one node only


def test_node_census_paper_sizes():
    """16 processes stay inside one node; with 64 and 256 the tuned ring sends
    fewer messages between nodes than the native one (Sec. V-A)."""
    one = O.node_census(O.build_schedule(16, 0, 524_288, O.TUNED), 24)
    assert one["ring_inter_msgs"] == 0 and one["scatter_inter_msgs"] == 0
    for P in (64, 256):
        nat = O.node_census(O.build_schedule(P, 0, 1_048_576, O.NATIVE), 24)
        tun = O.node_census(O.build_schedule(P, 0, 1_048_576, O.TUNED), 24)
        nodes = -(-P // 24)
        assert nat["ring_inter_msgs"] == nodes * (P - 1)
        assert tun["ring_inter_msgs"] < nat["ring_inter_msgs"]
