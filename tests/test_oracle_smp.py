"""Pins for the oracle's multi-core-aware three-phase broadcast [Sec. I]: the
state at the phase boundaries, the definition of broadcast, closed-form byte
counts, and that only the middle phase crosses nodes.  CPU only."""

import numpy as np
import pytest

from oracle import bcast_oracle as O

CASES = [(P, root, n, rpn) for (P, rpn) in [(1, 4), (4, 4), (5, 4), (9, 4), (17, 4), (24, 24), (25, 24),
                                            (33, 8), (65, 24), (129, 24), (10, 1), (7, 3)]
         for root in sorted({0, P // 2, P - 1}) for n in (0, 5, 12_288)]


def bufs_for(P, n, seed):
    rng = np.random.default_rng(seed)
    return [rng.integers(0, 256, n + 2, dtype=np.uint8) for _ in range(P)]


@pytest.mark.parametrize("P,root,n,rpn", CASES)
def test_three_phases(P, root, n, rpn):
    for ring in (O.NATIVE, O.TUNED):
        subs = O.smp_schedule(P, root, n, rpn, ring)
        n_nodes = -(-P // rpn)
        root_node = root // rpn
        assert [s.phase for s in subs] == [1, 2] + [3] * (n_nodes - 1)
        node_of = lambda r: r // rpn
        # phase 1 and 3 stay inside a node, phase 2 only touches one rank per node
        for sub in subs:
            nodes = {node_of(r) for r in sub.members}
            if sub.phase == 2:
                assert sub.members == [j * rpn for j in range(n_nodes)]
                assert sub.sched.root == root_node and sub.sched.algo == ring
            else:
                assert len(nodes) == 1 and sub.sched.algo == O.BINOMIAL
                assert sub.members == list(range(min(sub.members), max(sub.members) + 1))
                if sub.phase == 1:
                    assert sub.members[sub.sched.root] == root and nodes == {root_node}
                else:
                    assert sub.sched.root == 0 and root_node not in nodes
        # state at the phase boundaries
        bufs = bufs_for(P, n, P + n)
        init = [b.copy() for b in bufs]
        have = lambda r: np.array_equal(bufs[r][:n], init[root][:n])
        untouched = lambda r: np.array_equal(bufs[r], init[r])
        O.run_smp(bufs, subs, phases=(1,))
        for r in range(P):
            assert have(r) if node_of(r) == root_node else untouched(r)
        O.run_smp(bufs, subs, phases=(2,))
        for r in range(P):
            if node_of(r) == root_node or r % rpn == 0:
                assert have(r)
            else:
                assert untouched(r)
        O.run_smp(bufs, subs, phases=(3,))
        want = O.broadcast_definition(init, root, n)
        for a, b in zip(bufs, want):
            assert np.array_equal(a, b)
        # bytes: a binomial broadcast over m ranks moves (m - 1) n; the middle phase is the
        # ring broadcast over the node representatives
        sizes = [min(rpn, P - j * rpn) for j in range(n_nodes)]
        got = {ph: sum(s.sched.bytes_moved for s in subs if s.phase == ph) for ph in (1, 2, 3)}
        assert got[1] == (sizes[root_node] - 1) * n
        assert got[3] == sum((m - 1) * n for j, m in enumerate(sizes) if j != root_node)
        mid = O.build_schedule(n_nodes, root_node, n, ring)
        assert got[2] == mid.bytes_moved
        if ring == O.TUNED:
            assert got[2] == (n_nodes - 1) * n
        # every rank but the root receives the whole message at least once
        assert sum(got.values()) >= (P - 1) * n


def test_fewer_messages_between_nodes_than_the_flat_ring():
    """What multi-core awareness buys: only the middle phase crosses nodes."""
    P, n, rpn = 129, 100_000, 24
    flat = O.node_census(O.build_schedule(P, 5, n, O.TUNED), rpn)
    subs = O.smp_schedule(P, 5, n, rpn, O.TUNED)
    inter = 0
    for sub in subs:
        for s in range(sub.sched.n_steps):
            for (a, b, _o, _l) in sub.rows_absolute(s):
                crosses = a // rpn != b // rpn
                assert crosses == (sub.phase == 2)
                inter += crosses
    assert inter < flat["ring_inter_msgs"] + flat["scatter_inter_msgs"]
