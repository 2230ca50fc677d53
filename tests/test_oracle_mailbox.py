"""Asynchronous execution of the broadcast as P per-rank programs with
rendezvous matching, against the oracle's level-synchronous tables.  CPU only.

The per-rank program below is what one MPI process would run: receive its
subtree's chunks from its parent, pass the upper halves on to its children,
then walk the ring.  It takes the oracle's per-rank rules (chunk extents and
the tuned switch point) but none of its table generation, matching or
stepping; message matching, byte movement and deadlock detection are the
mailbox world's."""

import random

import numpy as np
import pytest

from oracle import bcast_oracle as O
import pin_models as M


def rank_program(rank, P, root, n, tuned):
    rel = O.relative_rank(rank, root, P)

    def extent(first, last):           # bytes of chunks [first, last)
        disp = O.chunk_extent(first, n, P)[0]
        return disp, sum(O.chunk_extent(c, n, P)[1] for c in range(first, last))

    # ---- scatter: the span of chunks this rank is handed, then its children
    if rel == 0:
        span = O.ceil_pow2(P)
    else:
        span = rel & -rel
        parent = O.absolute_rank(rel - span, root, P)
        disp, length = extent(rel, min(rel + span, P))
        if length > 0:
            yield ("recv", parent, disp, length)
    mask = span // 2
    while mask >= 1:
        if rel + mask < P:
            disp, length = extent(rel + mask, min(rel + 2 * mask, P))
            if length > 0:
                yield ("send", O.absolute_rank(rel + mask, root, P), disp, length)
        mask //= 2

    # ---- ring: a chunk moves one rank to the right per step, so in step i this
    # rank hands on the chunk that started i - 1 ranks to its left and is handed
    # the one that started i ranks to its left
    left, right = (rank - 1) % P, (rank + 1) % P
    sw = O.tuned_switch(rel, P)
    for i in range(1, P):
        give = O.chunk_extent(O.relative_rank((rank - i + 1) % P, root, P), n, P)
        take = O.chunk_extent(O.relative_rank((rank - i) % P, root, P), n, P)
        in_tail = tuned and i > P - sw[0]
        if not in_tail:
            yield ("sendrecv", right, *give, left, *take)
        elif sw[1] == O.RECV_ONLY:
            yield ("recv", left, *take)
        else:
            yield ("send", right, *give)


CASES = [(P, root, n)
         for P in list(range(1, 21)) + [24, 31, 32, 33, 40]
         for root in sorted({0, P // 2, P - 1})
         for n in sorted({0, 1, P - 1, P + 1, 3 * P + 2, 257})]


@pytest.mark.parametrize("P,root,n", CASES)
def test_async_execution_agrees_with_the_tables(P, root, n):
    for tuned in (False, True):
        rng = np.random.default_rng(P * 7919 + root * 31 + n)
        bufs = [rng.integers(0, 256, n + 3, dtype=np.uint8) for _ in range(P)]
        ref = [b.copy() for b in bufs]
        world = M.MailboxWorld(bufs)
        order = list(range(P))
        random.Random(P + n).shuffle(order)   # progress order must not matter
        world.run([rank_program(r, P, root, n, tuned) for r in range(P)], order)

        sched = O.build_schedule(P, root, n, O.TUNED if tuned else O.NATIVE)
        O.run_steps(ref, sched)
        for a, b in zip(bufs, ref):
            assert np.array_equal(a, b)
        for b in bufs:
            assert np.array_equal(b[:n], bufs[root][:n])
        assert world.bytes == sched.bytes_moved
        scatter_msgs = sum(sched.step_rows()[: sched.n_scatter_steps])
        assert world.messages == scatter_msgs + sched.ring_msgs_issued


def test_mailbox_world_detects_a_broken_pairing():
    """The harness itself must notice an unmatched receive."""
    P, n = 4, 16

    def broken(rank):
        # rank 1 skips its last send: its right neighbour waits forever
        prog = list(rank_program(rank, P, 0, n, False))
        return iter(prog[:-1] + [("recv", (rank - 1) % P, 0, 4)] if rank == 1 else prog)

    bufs = [np.zeros(n, dtype=np.uint8) for _ in range(P)]
    with pytest.raises((M.Deadlock, AssertionError)):
        M.MailboxWorld(bufs).run([broken(r) for r in range(P)])
