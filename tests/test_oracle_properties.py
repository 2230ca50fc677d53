"""Property tests (hypothesis) for the oracle over random (P, root, n): the
definition of broadcast, the byte and message closed forms, tuned never moving
more than native.  CPU only."""

import numpy as np
from hypothesis import given, settings, strategies as st

from oracle import bcast_oracle as O


@st.composite
def shapes(draw):
    P = draw(st.integers(1, 70))
    root = draw(st.integers(0, P - 1))
    n = draw(st.one_of(st.integers(0, 3 * P), st.integers(0, 5000)))
    return P, root, n


@settings(max_examples=120, deadline=None, derandomize=True, database=None)
@given(shapes(), st.sampled_from([O.NATIVE, O.TUNED, O.BINOMIAL, O.SCATTER_RDB]))
def test_any_schedule_is_a_broadcast(shape, algo):
    P, root, n = shape
    if algo == O.SCATTER_RDB and P & (P - 1):
        return
    sched = O.build_schedule(P, root, n, algo)
    rng = np.random.default_rng(P * 7 + n)
    bufs = [rng.integers(0, 256, n + 3, dtype=np.uint8) for _ in range(P)]
    want = O.broadcast_definition(bufs, root, n)
    O.run_steps(bufs, sched)
    for a, b in zip(bufs, want):
        assert np.array_equal(a, b)
    O.ownership_after(sched, sched.n_steps)          # no rank ever sends what it lacks
    for rows in sched.steps:
        for (s, d, off, ln) in rows:
            assert 0 <= s < P and 0 <= d < P and s != d and ln > 0 and off + ln <= n


@settings(max_examples=120, deadline=None, derandomize=True, database=None)
@given(shapes())
def test_byte_and_message_counts(shape):
    P, root, n = shape
    nat = O.build_schedule(P, root, n, O.NATIVE)
    tun = O.build_schedule(P, root, n, O.TUNED)
    ss = -(-n // P) if P else 0
    clen = [max(0, min(ss, n - c * ss)) for c in range(P)]
    scatter = sum(bin(c).count("1") * clen[c] for c in range(P))
    assert nat.scatter_bytes == tun.scatter_bytes == scatter
    assert nat.ring_bytes == (P - 1) * n
    assert tun.bytes_moved == (P - 1) * n <= nat.bytes_moved
    assert nat.ring_msgs_issued == P * (P - 1)
    span = lambda c: P if c == 0 else min(c & -c, P - c)
    assert tun.ring_msgs_issued == P * (P - 1) - sum(span(c) - 1 for c in range(P))
    assert nat.n_steps == tun.n_steps == (O.ceil_log2(P) + P - 1 if P > 1 else 0)
    assert O.build_schedule(P, root, n, O.BINOMIAL).bytes_moved == (P - 1) * n
