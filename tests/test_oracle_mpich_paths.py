"""Pins for the oracle's neighbouring algorithms (binomial-tree broadcast,
scatter + recursive-doubling allgather) and for the rule that selects among the
algorithms.  The paper names these and gives the thresholds [Abstract, Sec. I,
Sec. V] but prints no worked numbers, so the pins are closed forms, invariants,
brute-force models that do not import the oracle, and the definition of
broadcast.  CPU only."""

import random

import numpy as np
import pytest

from oracle import bcast_oracle as O
import pin_models as M


def bufs_for(P, n, seed):
    rng = np.random.default_rng(seed)
    return [rng.integers(0, 256, n + 4, dtype=np.uint8) for _ in range(P)]


# ------------------------------------------------------------------ binomial broadcast

@pytest.mark.parametrize("P", list(range(1, 34)) + [64, 65, 127, 128, 513])
def test_binomial_broadcast_tree_and_counts(P):
    edges = M.binomial_tree_messages(P)          # recursive halving, root 0
    by_dist = {}
    for (s, r, _a, _b, h) in edges:
        by_dist.setdefault(h, []).append((s, r))
    for root in sorted({0, P // 2, P - 1}):
        n = 37
        sched = O.build_schedule(P, root, n, O.BINOMIAL)
        assert sched.n_steps == O.ceil_log2(P) and sched.n_scatter_steps == 0
        dist = O.ceil_pow2(P) // 2
        has = {root}
        for rows in sched.steps:
            got = sorted(((s - root) % P, (d - root) % P) for (s, d, _o, _l) in rows)
            assert got == sorted(by_dist.get(dist, []))
            for (s, d, off, ln) in rows:
                assert (off, ln) == (0, n)
                assert s in has and d not in has      # sender has it, receiver gets it once
            has |= {d for (_s, d, _o, _l) in rows}
            dist //= 2
        assert has == set(range(P))
        assert sched.bytes_moved == (P - 1) * n
        assert sched.ring_msgs_issued == P - 1
    # an empty message still posts the P - 1 sends but moves nothing
    empty = O.build_schedule(P, 0, 0, O.BINOMIAL)
    assert empty.bytes_moved == 0 and empty.ring_msgs_issued == P - 1
    assert all(len(r) == 0 for r in empty.steps)


def test_binomial_tree_is_the_scatter_tree_of_the_paper():
    """Sec. III-A: the scatter follows a binomial tree from the root - 0 to 4,
    then 0 to 2 and 4 to 6, then the leaves; the broadcast uses the same tree."""
    rows = O.build_schedule(8, 0, 5, O.BINOMIAL).steps
    assert [[(s, d) for (s, d, _o, _l) in lvl] for lvl in rows] == \
        [[(0, 4)], [(0, 2), (4, 6)], [(0, 1), (2, 3), (4, 5), (6, 7)]]


# ------------------------------------------------------------------ recursive doubling

def doubling_model(P):
    """Chunk sets: everyone starts with its own chunk and, at distance 1, 2, 4,
    ..., swaps all it has with the rank whose number differs in that bit."""
    own = {r: {r} for r in range(P)}
    steps = []
    d = 1
    while d < P:
        steps.append([(r, r ^ d, frozenset(own[r])) for r in range(P)])
        own = {r: own[r] | own[r ^ d] for r in range(P)}
        d *= 2
    assert all(own[r] == set(range(P)) for r in range(P))
    return steps


@pytest.mark.parametrize("k", range(0, 8))
def test_recursive_doubling_matches_the_set_model(k):
    P = 1 << k
    model = doubling_model(P)
    for root in sorted({0, P // 3, P - 1}):
        for n in sorted({4 * P, 4 * P - 1, 40 * P - 3}):     # last chunk short, none empty
            ss = -(-n // P)
            steps, posted = O.recursive_doubling_steps(P, root, n)
            assert len(steps) == k and posted == [P] * k
            for rows, ref in zip(steps, model):
                got = []
                for (s, d, off, ln) in rows:
                    assert off % ss == 0
                    chunks = frozenset(range(off // ss, (off + ln + ss - 1) // ss))
                    got.append(((s - root) % P, (d - root) % P, chunks))
                assert got == [(a, b, c) for (a, b, c) in ref]
            sched = O.build_schedule(P, root, n, O.SCATTER_RDB)
            # every rank receives every chunk but its own exactly once after the scatter
            assert sched.ring_bytes == (P - 1) * n
            assert sched.bytes_moved == (P - 1) * n + sched.scatter_bytes
            assert sched.n_steps == 2 * k and sched.n_scatter_steps == k
            assert sched.ring_msgs_issued == P * k
            O.ownership_after(sched, sched.n_steps)     # raises if a rank sends what it lacks


def test_recursive_doubling_needs_a_power_of_two():
    for P in (3, 6, 10, 24, 513):
        with pytest.raises(ValueError):
            O.recursive_doubling_steps(P, 0, 100)


# ------------------------------------------------------------------ definition of broadcast, races, async

CASES = [(P, root, n) for P in (1, 2, 3, 4, 7, 8, 16, 21, 32)
         for root in sorted({0, P - 1}) for n in sorted({0, 1, P - 1, P + 1, 1000})]


@pytest.mark.parametrize("P,root,n", CASES)
def test_final_state_and_independent_rows(P, root, n):
    algos = [O.BINOMIAL] + ([O.SCATTER_RDB] if P & (P - 1) == 0 else [])
    for algo in algos:
        sched = O.build_schedule(P, root, n, algo)
        bufs = bufs_for(P, n, P * 100 + n)
        want = O.broadcast_definition(bufs, root, n)
        O.run_steps(bufs, sched)
        for a, b in zip(bufs, want):
            assert np.array_equal(a, b)
        for rows in sched.steps:           # no row reads or writes what another row writes
            wr = [(d, o, o + l) for (_s, d, o, l) in rows]
            for (s, _d, o, l) in rows:
                assert not any(wd == s and a < o + l and o < b for (wd, a, b) in wr)
            for i, (d1, a1, b1) in enumerate(wr):
                assert not any(d1 == d2 and a1 < b2 and a2 < b1 for (d2, a2, b2) in wr[i + 1:])


def binomial_program(rank, P, root, n):
    rel = O.relative_rank(rank, root, P)
    span = O.ceil_pow2(P) if rel == 0 else rel & -rel
    if rel:
        yield ("recv", O.absolute_rank(rel - span, root, P), 0, n)
    m = span // 2
    while m >= 1:
        if rel + m < P:
            yield ("send", O.absolute_rank(rel + m, root, P), 0, n)
        m //= 2


def doubling_program(rank, P, root, n):
    rel = O.relative_rank(rank, root, P)
    ext = lambda a, b: (O.chunk_extent(a, n, P)[0], sum(O.chunk_extent(c, n, P)[1] for c in range(a, b)))
    # scatter part, as in the ring broadcast
    span = O.ceil_pow2(P) if rel == 0 else rel & -rel
    if rel:
        d, l = ext(rel, min(rel + span, P))
        if l:
            yield ("recv", O.absolute_rank(rel - span, root, P), d, l)
    m = span // 2
    while m >= 1:
        if rel + m < P:
            d, l = ext(rel + m, min(rel + 2 * m, P))
            if l:
                yield ("send", O.absolute_rank(rel + m, root, P), d, l)
        m //= 2
    dist = 1
    while dist < P:
        partner = O.absolute_rank(rel ^ dist, root, P)
        mine, theirs = (rel // dist) * dist, ((rel ^ dist) // dist) * dist
        sd, sl = ext(mine, mine + dist)
        rd, rl = ext(theirs, theirs + dist)
        yield ("sendrecv", partner, sd, sl, partner, rd, rl)
        dist *= 2


@pytest.mark.parametrize("P,root,n", [(P, r, n) for P in (1, 2, 4, 5, 8, 13, 16) for r in (0, P - 1)
                                      for n in (0, 3, 200)])
def test_async_execution(P, root, n):
    for algo, prog in ((O.BINOMIAL, binomial_program), (O.SCATTER_RDB, doubling_program)):
        if algo == O.SCATTER_RDB and P & (P - 1):
            continue
        if algo == O.BINOMIAL and n == 0:
            continue        # the mailbox world would carry P - 1 empty messages; nothing to compare
        bufs = bufs_for(P, n, 5 + P)
        ref = [b.copy() for b in bufs]
        world = M.MailboxWorld(bufs)
        order = list(range(P))
        random.Random(P * 7 + n).shuffle(order)
        world.run([prog(r, P, root, n) for r in range(P)], order)
        sched = O.build_schedule(P, root, n, algo)
        O.run_steps(ref, sched)
        for a, b in zip(bufs, ref):
            assert np.array_equal(a, b)
        assert world.bytes == sched.bytes_moved


# ------------------------------------------------------------------ the selection rule

def test_selection_thresholds():
    """Sec. V: short below 12288 bytes, long from 524288 bytes; Abstract / Sec. I:
    binomial for short, recursive doubling for medium on a power of two, scatter
    + ring for long and for medium on other process counts."""
    assert O.SHORT_MSG_BYTES == 12288 and O.LONG_MSG_BYTES == 524288
    for tuned, ring in ((False, O.NATIVE), (True, O.TUNED)):
        assert O.select_algorithm(0, 8, tuned) == O.BINOMIAL
        assert O.select_algorithm(12287, 9, tuned) == O.BINOMIAL
        assert O.select_algorithm(12288, 8, tuned) == O.SCATTER_RDB
        assert O.select_algorithm(12288, 9, tuned) == ring            # mmsg-npof2
        assert O.select_algorithm(524287, 256, tuned) == O.SCATTER_RDB
        assert O.select_algorithm(524287, 129, tuned) == ring
        assert O.select_algorithm(524288, 256, tuned) == ring         # lmsg
        assert O.select_algorithm(30_000_000, 16, tuned) == ring
        assert O.select_algorithm(12288, 1, tuned) == O.SCATTER_RDB   # 1 = 2**0
