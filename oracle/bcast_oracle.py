"""CPU oracle for the scatter + ring-allgather broadcast of P virtual ranks.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain reference that the
GPU library is checked against.  It is imported by the tests, by the smoke
check and by the benchmark's CPU-baseline leg, never by the product path, and
it shares no code with the HIP sources.

What it models (paper sections in brackets):

* every rank views its n-byte buffer as P chunks of ``ceil(n / P)`` bytes laid
  out in relative-rank order, the last ones short or empty        [Sec. IV, listing]
* a binomial scatter from the root: in ``ceil(log2 P)`` levels every subtree
  root hands the upper half of its chunk range to the rank ``mask`` above it
                                                          [Sec. III-A, Figs. 1-2]
* the native ("enclosed") ring allgather: P-1 steps, every rank sends one
  chunk to its right neighbour and receives one from its left    [Sec. III-A, Fig. 3]
* the tuned ("non-enclosed") ring: every rank derives a pair (step, flag) from
  its relative rank and, for the last ``step - 1`` ring steps, only sends or
  only receives                                          [Sec. IV, listing, Figs. 4-5]

The ring is written as P little per-rank programs advanced in lock step: each
rank decides from its own variables what it sends and what it expects, and the
oracle then checks that every posted send meets a posted receive with the same
extent before delivering it.  Nothing is blocked, fused or reordered.

* the two neighbouring algorithms of the same MPI_Bcast that the paper names
  without describing them - binomial-tree broadcast and scatter + recursive-
  doubling allgather, in their textbook form - and the size / process-count
  rule that selects among the three                    [Abstract, Sec. I, Sec. V]

Parity pins: every function here is pinned by tests/test_oracle_*.py against
the paper's worked examples (P = 8 and P = 10), closed forms, the definition of
broadcast, independent ownership-set models and an asynchronous mailbox
execution.  No function is "parity unpinned"; for the two neighbouring
algorithms the paper prints no numbers, so their pins are the mathematics only
(closed forms, invariants, brute force, the definition of broadcast).
"""

from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

NATIVE = "native"            # scatter + native ring allgather
TUNED = "tuned"              # scatter + tuned ring allgather
BINOMIAL = "binomial"        # binomial-tree broadcast of the whole message
SCATTER_RDB = "scatter_rdb"  # scatter + recursive-doubling allgather (power-of-two P)

SHORT_MSG_BYTES = 12288      # below: short message            [Sec. V]
LONG_MSG_BYTES = 524288      # from here on: long message      [Sec. V]

RECV_ONLY = 1  # the listing's flag = 1
SEND_ONLY = 0  # the listing's flag = 0

Row = Tuple[int, int, int, int]  # (src rank, dst rank, byte offset, byte length)


# --------------------------------------------------------------------------
# rank and chunk arithmetic                                   [Sec. IV, listing]
# --------------------------------------------------------------------------

def relative_rank(rank: int, root: int, P: int) -> int:
    """Distance of ``rank`` above ``root`` on the ring of P ranks."""
    return rank - root if rank >= root else rank - root + P


def absolute_rank(rel: int, root: int, P: int) -> int:
    """Inverse of :func:`relative_rank`."""
    return (rel + root) % P


def scatter_size(n: int, P: int) -> int:
    """Chunk size: n bytes divided over P ranks, rounded up."""
    return (n + P - 1) // P


def chunk_extent(c: int, n: int, P: int) -> Tuple[int, int]:
    """(displacement, count) of the chunk with relative index ``c``.

    The count is what is left of the message at that displacement, at most one
    scatter size and never negative.
    """
    ss = scatter_size(n, P)
    disp = c * ss
    count = min(ss, n - disp)
    if count < 0:
        count = 0
    return disp, count


def ceil_pow2(P: int) -> int:
    """2 ** ceil(log2 P), in integers."""
    m = 1
    while m < P:
        m *= 2
    return m


def ceil_log2(P: int) -> int:
    k = 0
    while (1 << k) < P:
        k += 1
    return k


# --------------------------------------------------------------------------
# binomial scatter                                      [Sec. III-A, Figs. 1-2]
# --------------------------------------------------------------------------

def scatter_levels(P: int, root: int, n: int) -> List[List[Row]]:
    """One list of messages per level of the binomial tree.

    At the level with distance ``mask`` every relative rank that is a multiple
    of ``2 * mask`` is a subtree root holding the chunks ``[rho, rho + 2*mask)``
    (clipped to P); it keeps the lower half and sends the upper half, as one
    contiguous message, to relative rank ``rho + mask`` if that rank exists.
    Levels run from the largest distance down to 1, so the root's first
    message is the one that spawns the largest subtree.  Empty messages are
    not sent.
    """
    levels: List[List[Row]] = []
    mask = ceil_pow2(P) // 2
    while mask >= 1:
        rows: List[Row] = []
        for rho in range(0, P, 2 * mask):
            child = rho + mask
            if child >= P:
                continue
            upper_end = min(rho + 2 * mask, P)
            disp, _ = chunk_extent(child, n, P)
            length = sum(chunk_extent(c, n, P)[1] for c in range(child, upper_end))
            if length > 0:
                rows.append((absolute_rank(rho, root, P),
                             absolute_rank(child, root, P), disp, length))
        levels.append(rows)
        mask //= 2
    return levels


def owned_after_scatter(rel: int, P: int) -> range:
    """Relative chunk indices a rank holds once the scatter is over: its own
    chunk and those of all its descendants in the tree."""
    if rel == 0:
        return range(0, P)
    span = 1
    while rel % (2 * span) == 0:
        span *= 2
    return range(rel, min(rel + span, P))


# --------------------------------------------------------------------------
# the tuned ring's per-rank switch point                      [Sec. IV, listing]
# --------------------------------------------------------------------------

def tuned_switch(rel: int, P: int) -> Optional[Tuple[int, int]]:
    """(step, flag) of the rank with relative rank ``rel``; None for P = 1.

    After the scatter some ranks are ahead of the others: the root holds the
    whole message, and a rank whose relative rank is even heads a subtree and
    holds its ``span`` chunks (`owned_after_scatter`).  A rank that is ahead needs
    only ``P - span`` chunks from the ring, so it has everything ``span - 1`` steps
    before the ring ends; from then on it takes nothing more, and its left
    neighbour has nothing left to give it.

    Seen from one rank this gives exactly one of two tails.  Of two consecutive
    relative ranks only one is even; at the ring's seam, where the root (0)
    follows rank P - 1, the root counts, whatever the parity of P - 1.  So:

    * the right neighbour is ahead (its relative rank is even, 0 included): this
      rank stops sending when the neighbour is complete and only receives for
      the rest - flag RECV_ONLY, step = the neighbour's span;
    * otherwise the rank is ahead itself: it stops receiving and only sends -
      flag SEND_ONLY, step = its own span.

    The listing of Sec. IV reaches the same pair by trying power-of-two distances
    from 2**ceil(log2 P) down to 2, at each distance first on the right
    neighbour, then on the rank itself; the distance at which it stops, clipped
    at the last rank, is the span above, and the order of its two tests is what
    gives the seam to the root.
    """
    if P < 2:
        return None
    right = (rel + 1) % P
    if right % 2 == 0:
        return len(owned_after_scatter(right, P)), RECV_ONLY
    return len(owned_after_scatter(rel, P)), SEND_ONLY


# --------------------------------------------------------------------------
# ring allgather, native and tuned          [Sec. III-A Fig. 3; Sec. IV listing]
# --------------------------------------------------------------------------

@dataclass
class RingResult:
    steps: List[List[Row]]          # delivered messages with len > 0, per ring step
    posted_sends: List[int]         # sends posted per step, zero-length ones included
    posted_recvs: List[int]         # receives posted per step


def ring_steps(P: int, root: int, n: int, algo: str) -> RingResult:
    """Advance P per-rank programs through the P-1 ring steps.

    A chunk travels one rank to the right per step [Sec. III-A, Fig. 3: a rank
    forwards what it received one step earlier]: in step i every rank passes on
    the chunk that started i - 1 ranks to its left (its own in step 1) and
    expects the chunk that started i ranks to its left.  Each rank decides for
    itself what it posts; whether the posts of neighbours fit is checked below.

    native: every rank sends and receives in every step.
    tuned : a rank does both for the first ``P - step`` steps; in the remaining
            ``step - 1`` it only receives (flag RECV_ONLY) or only sends (SEND_ONLY).
    """
    if algo not in (NATIVE, TUNED):
        raise ValueError(algo)
    order = [absolute_rank(rho, root, P) for rho in range(P)]  # by relative rank
    switch = {r: tuned_switch(relative_rank(r, root, P), P) for r in range(P)}

    out = RingResult([], [], [])
    for i in range(1, P):
        sends = {}   # (src, dst) -> (disp, count), posted by the sender
        recvs = {}   # (src, dst) -> (disp, count), posted by the receiver
        for r in order:
            left = (r - 1) % P
            right = (r + 1) % P
            passing = (r - (i - 1)) % P      # rank whose chunk this rank passes on
            awaiting = (r - i) % P           # rank whose chunk it expects from the left
            out_extent = chunk_extent(relative_rank(passing, root, P), n, P)
            in_extent = chunk_extent(relative_rank(awaiting, root, P), n, P)

            sending = receiving = True
            if algo == TUNED:
                step, flag = switch[r]
                if i > P - step:             # the rank's one-direction tail
                    sending = flag == SEND_ONLY
                    receiving = flag == RECV_ONLY

            if sending:
                sends[(r, right)] = out_extent
            if receiving:
                recvs[(left, r)] = in_extent

        # Blocking point-to-point calls complete only in matched pairs.
        if sends != recvs:
            raise AssertionError(
                f"ring step {i}: posted sends and receives do not pair up "
                f"(P={P}, root={root}, n={n}, algo={algo})")
        out.posted_sends.append(len(sends))
        out.posted_recvs.append(len(recvs))
        rows = [(src, dst, disp, cnt)
                for (src, dst), (disp, cnt) in sends.items() if cnt > 0]
        out.steps.append(rows)
    return out


# --------------------------------------------------------------------------
# the neighbouring algorithms of the same MPI_Bcast          [Abstract, Sec. I]
#
# The paper names them (binomial dissemination for short messages,
# recursive-doubling exchange for medium messages on a power-of-two process
# count) and gives the size thresholds that select between them [Sec. V], but
# does not describe them; they are written here in their textbook form, the
# one of the MPICH collectives paper this paper cites.
# --------------------------------------------------------------------------

def binomial_levels(P: int, root: int, n: int):
    """Binomial-tree broadcast: the same tree as the scatter, but every edge
    carries the whole message.  Level by level from the largest distance, a
    rank that already has the message hands it to the rank ``mask`` above.
    Returns (levels, posted): rows with len > 0 per level, and the number of
    sends posted per level (zero-length ones included)."""
    levels: List[List[Row]] = []
    posted: List[int] = []
    mask = ceil_pow2(P) // 2
    while mask >= 1:
        rows: List[Row] = []
        count = 0
        for rho in range(0, P, 2 * mask):
            child = rho + mask
            if child < P:
                count += 1
                if n > 0:
                    rows.append((absolute_rank(rho, root, P), absolute_rank(child, root, P), 0, n))
        levels.append(rows)
        posted.append(count)
        mask //= 2
    return levels, posted


def recursive_doubling_steps(P: int, root: int, n: int):
    """Recursive-doubling allgather after the scatter, for a power-of-two P.

    Every rank acts as if it held only its own chunk.  In exchange k (distance
    2**k) the rank with relative rank rho swaps with rho XOR 2**k everything it
    has gathered so far: the 2**k chunks of the aligned block that contains
    rho.  After log2 P exchanges every rank has all P chunks.
    Returns (steps, posted): rows with len > 0 per exchange, and the number of
    sends posted per exchange (zero-length ones included).
    """
    if P & (P - 1):
        raise ValueError("recursive doubling needs a power-of-two process count")
    steps, posted = [], []
    dist = 1
    while dist < P:
        sends, recvs = {}, {}
        for rho in range(P):
            partner = rho ^ dist
            mine = (rho // dist) * dist          # block gathered so far
            theirs = (partner // dist) * dist
            s_disp = chunk_extent(mine, n, P)[0]
            s_count = sum(chunk_extent(c, n, P)[1] for c in range(mine, mine + dist))
            r_disp = chunk_extent(theirs, n, P)[0]
            r_count = sum(chunk_extent(c, n, P)[1] for c in range(theirs, theirs + dist))
            a, b = absolute_rank(rho, root, P), absolute_rank(partner, root, P)
            sends[(a, b)] = (s_disp, s_count)
            recvs[(b, a)] = (r_disp, r_count)
        if sends != recvs:
            raise AssertionError("recursive doubling: sends and receives do not pair up")
        posted.append(len(sends))
        steps.append([(src, dst, d, cnt) for (src, dst), (d, cnt) in sends.items() if cnt > 0])
        dist *= 2
    return steps, posted


def select_algorithm(n: int, P: int, tuned: bool) -> str:
    """Which algorithm MPICH's broadcast takes for n bytes on P processes, as
    the paper states it [Abstract; Sec. I; thresholds in Sec. V]: short messages
    go down a binomial tree; medium messages on a power-of-two process count
    use scatter + recursive doubling; long messages, and medium messages on any
    other process count, use scatter + ring allgather - the native ring, or the
    paper's tuned one."""
    if n < SHORT_MSG_BYTES:
        return BINOMIAL
    if n < LONG_MSG_BYTES and P & (P - 1) == 0:
        return SCATTER_RDB
    return TUNED if tuned else NATIVE


# --------------------------------------------------------------------------
# the whole schedule
# --------------------------------------------------------------------------

@dataclass
class Schedule:
    P: int
    root: int
    n: int
    algo: str
    ss: int
    n_scatter_steps: int
    steps: List[List[Row]] = field(default_factory=list)  # scatter levels, then ring steps
    ring_msgs_issued: int = 0   # sends posted after the scatter, zero-length ones included

    @property
    def n_steps(self) -> int:
        return len(self.steps)

    def step_bytes(self) -> List[int]:
        return [sum(r[3] for r in rows) for rows in self.steps]

    def step_rows(self) -> List[int]:
        return [len(rows) for rows in self.steps]

    @property
    def scatter_bytes(self) -> int:
        return sum(self.step_bytes()[: self.n_scatter_steps])

    @property
    def ring_bytes(self) -> int:
        return sum(self.step_bytes()[self.n_scatter_steps:])

    @property
    def bytes_moved(self) -> int:
        return sum(self.step_bytes())

    @property
    def ring_rows(self) -> int:
        return sum(self.step_rows()[self.n_scatter_steps:])


def build_schedule(P: int, root: int, n: int, algo: str) -> Schedule:
    """Scatter levels followed by ring steps (or recursive-doubling exchanges),
    or the levels of the binomial broadcast; one level / ring step / exchange =
    one step.  Rows inside a step are ordered by the sender's relative rank.
    """
    if P < 1 or not (0 <= root < P) or n < 0:
        raise ValueError("bad (P, root, n)")
    if algo == BINOMIAL:
        tree, posted = binomial_levels(P, root, n)
        return Schedule(P=P, root=root, n=n, algo=algo, ss=scatter_size(n, P),
                        n_scatter_steps=0, steps=tree, ring_msgs_issued=sum(posted))
    levels = scatter_levels(P, root, n)
    if algo == SCATTER_RDB:
        steps, posted = recursive_doubling_steps(P, root, n)
        return Schedule(P=P, root=root, n=n, algo=algo, ss=scatter_size(n, P),
                        n_scatter_steps=len(levels), steps=levels + steps,
                        ring_msgs_issued=sum(posted))
    ring = ring_steps(P, root, n, algo)
    return Schedule(P=P, root=root, n=n, algo=algo, ss=scatter_size(n, P),
                    n_scatter_steps=len(levels),
                    steps=levels + ring.steps,
                    ring_msgs_issued=sum(ring.posted_sends))


# --------------------------------------------------------------------------
# the multi-core-aware three-phase broadcast                         [Sec. I]
#
# The paper describes it in one sentence and does not implement it: a binomial
# broadcast inside the root's node, then the scatter-ring-allgather between the
# nodes, then a binomial broadcast inside every other node.  Readings taken
# where the sentence is silent: ranks sit on nodes in blocks of
# ``ranks_per_node`` [Sec. V-A]; a node is represented between the nodes by
# its lowest rank; the inter-node phase starts from the root node's
# representative, which holds the message after the first phase.
# --------------------------------------------------------------------------

@dataclass
class SubSchedule:
    phase: int                 # 1, 2 or 3
    members: List[int]         # absolute ranks of the sub-communicator, in its rank order
    sched: Schedule            # schedule in the sub-communicator's own rank numbers

    def rows_absolute(self, s: int) -> List[Row]:
        m = self.members
        return [(m[a], m[b], off, ln) for (a, b, off, ln) in self.sched.steps[s]]


def smp_schedule(P: int, root: int, n: int, ranks_per_node: int, ring_algo: str) -> List[SubSchedule]:
    """The three phases as schedules over sub-communicators, in execution
    order: phase 1 (one), phase 2 (one), phase 3 (one per node other than the
    root's; they are independent of each other)."""
    if ring_algo not in (NATIVE, TUNED):
        raise ValueError(ring_algo)
    if P < 1 or not (0 <= root < P) or ranks_per_node < 1:
        raise ValueError("bad arguments")
    nodes = [list(range(a, min(a + ranks_per_node, P))) for a in range(0, P, ranks_per_node)]
    root_node = root // ranks_per_node
    out: List[SubSchedule] = []
    home = nodes[root_node]
    out.append(SubSchedule(1, home, build_schedule(len(home), home.index(root), n, BINOMIAL)))
    leaders = [nd[0] for nd in nodes]
    out.append(SubSchedule(2, leaders, build_schedule(len(leaders), root_node, n, ring_algo)))
    for j, nd in enumerate(nodes):
        if j != root_node:
            out.append(SubSchedule(3, nd, build_schedule(len(nd), 0, n, BINOMIAL)))
    return out


def run_smp(bufs: Sequence[np.ndarray], subs: Sequence[SubSchedule], phases=(1, 2, 3)) -> None:
    """Execute the sub-schedules of the given phases, in order."""
    for sub in subs:
        if sub.phase in phases:
            for s in range(sub.sched.n_steps):
                apply_step(bufs, sub.rows_absolute(s))


# --------------------------------------------------------------------------
# inter-node / intra-node census                                  [Sec. V-A]
# --------------------------------------------------------------------------

def node_census(sched: Schedule, ranks_per_node: int) -> dict:
    """Messages and bytes that cross a node boundary when the ranks sit on
    nodes in blocks of ``ranks_per_node`` (rank r on node r // ranks_per_node;
    the paper's cluster holds 24 processes per node and places them this way).
    Counted separately for the scatter and for the steps after it; only rows
    with len > 0 count."""
    out = {"scatter_inter_msgs": 0, "scatter_inter_bytes": 0,
           "scatter_intra_msgs": 0, "scatter_intra_bytes": 0,
           "ring_inter_msgs": 0, "ring_inter_bytes": 0,
           "ring_intra_msgs": 0, "ring_intra_bytes": 0}
    for s, rows in enumerate(sched.steps):
        phase = "scatter" if s < sched.n_scatter_steps else "ring"
        for (src, dst, _off, length) in rows:
            kind = "inter" if src // ranks_per_node != dst // ranks_per_node else "intra"
            out[f"{phase}_{kind}_msgs"] += 1
            out[f"{phase}_{kind}_bytes"] += length
    return out


# --------------------------------------------------------------------------
# executing a schedule on byte buffers
# --------------------------------------------------------------------------

def apply_step(bufs: Sequence[np.ndarray], rows: Sequence[Row]) -> None:
    """Deliver all messages of one step.

    All sends of a step read the state from before the step: payloads are
    taken first, then written at the same offset in the receiver's buffer.
    """
    payloads = [bufs[src][off:off + length].copy() for (src, _dst, off, length) in rows]
    for (_src, dst, off, length), data in zip(rows, payloads):
        bufs[dst][off:off + length] = data


def run_steps(bufs: Sequence[np.ndarray], sched: Schedule,
              first: int = 0, last: Optional[int] = None) -> None:
    """Apply steps ``[first, last)`` of the schedule, in order."""
    if last is None:
        last = sched.n_steps
    for s in range(first, last):
        apply_step(bufs, sched.steps[s])


def broadcast_definition(bufs: Sequence[np.ndarray], root: int, n: int) -> List[np.ndarray]:
    """What MPI requires of any broadcast: on return the first n bytes of every
    rank's buffer equal the root's; nothing else changes.       [Sec. III-A]"""
    out = [b.copy() for b in bufs]
    for b in out:
        b[:n] = bufs[root][:n]
    return out


# --------------------------------------------------------------------------
# chunk-ownership form of the state (no byte buffers needed)
# --------------------------------------------------------------------------

def ownership_after(sched: Schedule, k: int) -> np.ndarray:
    """has[rank, c] after the first k steps: does ``rank`` hold valid (root's)
    data in the chunk with relative index ``c``?

    Every message moves whole chunks at unchanged offsets, so the byte state
    is: root's bytes where has[...] is set, the rank's initial bytes elsewhere.
    A message that would carry a chunk its sender does not hold is an error.
    """
    P, root, n = sched.P, sched.root, sched.n
    has = np.zeros((P, P), dtype=bool)
    has[root, :] = True
    ss = scatter_size(n, P)
    for s in range(k):
        before = has.copy()
        for (src, dst, off, length) in sched.steps[s]:
            # walk the chunks the message covers, starting at the one at `off`
            c = off // ss
            covered = []
            remaining = length
            while remaining > 0:
                disp, cnt = chunk_extent(c, n, P)
                if cnt == 0 or cnt > remaining or (not covered and disp != off):
                    raise AssertionError("message does not consist of whole chunks")
                covered.append(c)
                remaining -= cnt
                c += 1
            for c in covered:
                if not before[src, c]:
                    raise AssertionError(
                        f"step {s}: rank {src} sends chunk {c} it does not hold")
                has[dst, c] = True
    return has
