"""Two small models that are independent of the oracle's schedule generator and
are used to pin it.  Neither imports the oracle.

1. ``prose_model``: the broadcast as the paper *describes* it in words, on sets
   of chunk numbers: a binomial tree built by recursive halving, a ring in
   which every rank forwards what it got one step earlier, and - for the tuned
   variant - a transfer happens only if the receiver still lacks the chunk
   [Sec. III-A, Sec. IV prose and Figs. 1-5].  No mask loop, no step/flag.

2. ``MailboxWorld``: an asynchronous execution of P per-rank programs that
   issue blocking send / recv / sendrecv calls, matched through rendezvous
   (a send completes only together with the receive it meets).  It moves real
   bytes and detects deadlock, unmatched or mismatched messages.
"""

from __future__ import annotations

from typing import Dict, Generator, List, Optional, Set, Tuple

import numpy as np


# --------------------------------------------------------------------------
# 1. the prose model, on chunk sets (relative ranks; the root is 0)
# --------------------------------------------------------------------------

def binomial_tree_messages(P: int) -> List[Tuple[int, int, int, int, int]]:
    """(sender, receiver, first chunk, one-past-last chunk, distance) for every
    edge of the binomial scatter tree over ranks 0..P-1, root 0, built by
    recursive halving: the holder of chunks [lo, hi) hands the part above the
    largest power of two below the range size to the rank at its start."""
    edges = []

    def hand_off(lo: int, hi: int) -> None:
        size = hi - lo
        if size <= 1:
            return
        h = 1
        while h * 2 < size:
            h *= 2
        edges.append((lo, lo + h, lo + h, hi, h))
        hand_off(lo, lo + h)
        hand_off(lo + h, hi)

    hand_off(0, P)
    return edges


def prose_model(P: int, tuned: bool):
    """Return (levels, ring) where ``levels[d]`` is the list of scatter edges
    (sender, receiver, set of chunks) whose distance is the d-th largest power
    of two, and ``ring[i-1]`` is the list of (sender, receiver, chunk) moved in
    ring step i."""
    edges = binomial_tree_messages(P)
    top = 1
    while top < P:
        top *= 2
    levels: List[List[Tuple[int, int, Set[int]]]] = []
    dist = top // 2
    while dist >= 1:
        levels.append(sorted((s, r, set(range(a, b)))
                             for (s, r, a, b, h) in edges if h == dist))
        dist //= 2

    owns: Dict[int, Set[int]] = {r: set() for r in range(P)}
    owns[0] = set(range(P))
    for lvl in levels:
        for (_s, r, chunks) in lvl:
            owns[r] |= chunks
    # each rank now holds its own chunk and its descendants'
    in_hand = {r: r for r in range(P)}  # the chunk a rank forwards next
    ring = []
    for _i in range(1, P):
        moved = []
        arriving = {}
        for r in range(P):
            dst = (r + 1) % P
            c = in_hand[r]
            arriving[dst] = c
            if tuned and c in owns[dst]:
                continue          # the receiver is not missing this chunk
            moved.append((r, dst, c))
        for dst, c in arriving.items():
            owns[dst].add(c)
            in_hand[dst] = c
        ring.append(moved)
    assert all(owns[r] == set(range(P)) for r in range(P))
    return levels, ring


# --------------------------------------------------------------------------
# 2. asynchronous rendezvous execution of per-rank programs
# --------------------------------------------------------------------------

Op = Tuple  # ("send", dst, off, len) | ("recv", src, off, len) | ("sendrecv", dst, soff, slen, src, roff, rlen)


class Deadlock(Exception):
    pass


class MailboxWorld:
    def __init__(self, bufs: List[np.ndarray]):
        self.bufs = bufs
        self.P = len(bufs)
        self.messages = 0          # matched messages, zero-length ones included
        self.bytes = 0

    def run(self, programs: List[Generator[Op, None, None]], order: Optional[List[int]] = None) -> None:
        P = self.P
        # per rank: the halves of its current call that are still open
        open_send: List[Optional[Tuple[int, int, int]]] = [None] * P   # (dst, off, len)
        open_recv: List[Optional[Tuple[int, int, int]]] = [None] * P   # (src, off, len)
        done = [False] * P
        visit = order if order is not None else list(range(P))

        def fetch(r: int) -> None:
            try:
                op = next(programs[r])
            except StopIteration:
                done[r] = True
                return
            if op[0] == "send":
                open_send[r] = (op[1], op[2], op[3])
            elif op[0] == "recv":
                open_recv[r] = (op[1], op[2], op[3])
            elif op[0] == "sendrecv":
                open_send[r] = (op[1], op[2], op[3])
                open_recv[r] = (op[4], op[5], op[6])
            else:
                raise ValueError(op)

        for r in visit:
            fetch(r)
        while not all(done):
            progressed = False
            for s in visit:
                if open_send[s] is None:
                    continue
                dst, off, length = open_send[s]
                want = open_recv[dst]
                if want is None or want[0] != s:
                    continue
                if want[1:] != (off, length):
                    raise AssertionError(
                        f"rank {s} sends (off={off}, len={length}) but rank {dst} "
                        f"expects (off={want[1]}, len={want[2]})")
                # payload is taken when the pair meets
                self.bufs[dst][off:off + length] = self.bufs[s][off:off + length].copy()
                self.messages += 1
                self.bytes += length
                open_send[s] = None
                open_recv[dst] = None
                progressed = True
            for r in visit:
                if not done[r] and open_send[r] is None and open_recv[r] is None:
                    fetch(r)
                    progressed = True
            if not progressed:
                stuck = [r for r in range(P) if not done[r]]
                raise Deadlock(f"ranks {stuck} wait forever")
