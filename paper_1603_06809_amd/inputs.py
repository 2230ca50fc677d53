"""Seeded synthetic inputs: workloads, root messages and per-rank poison.

This module holds no broadcast arithmetic.  It only names the workloads and
turns (seed, stream, index) into bytes with a counter-based generator, so the
CPU oracle's tests and the GPU path's tests can be fed the same bytes without
either side importing the other.

Generator: SplitMix64 (Steele, Lea, Flood 2014; the published finaliser with
constants 0xBF58476D1CE4E5B9 and 0x94D049BB133111EB and increment
0x9E3779B97F4A7C15), used as a hash of a counter: word k of a stream is
``mix(key + (k + 1) * GOLDEN)``, and the byte string is the little-endian
concatenation of those 64-bit words.  Two implementations are given, numpy
(uint64) and torch (int64, any device); a CPU test holds them to each other and
to values computed with plain Python integers.

The paper broadcasts opaque bytes (MPI_BYTE) and uses no dataset, so uniform
random bytes stand in for its messages [Sec. V].  Buffers of non-root ranks
start as "poison": bytes of a different stream per rank, so that a byte that
was never delivered, or delivered to the wrong place, is visible.
"""

from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np

_GOLDEN = 0x9E3779B97F4A7C15
_MIX1 = 0xBF58476D1CE4E5B9
_MIX2 = 0x94D049BB133111EB
_MASK64 = (1 << 64) - 1


@dataclass(frozen=True)
class Workload:
    name: str
    P: int        # virtual ranks
    root: int
    n: int        # message bytes
    seed: int


# The five workloads: process counts and sizes in the range the paper sweeps
# (long messages from 524288 bytes up, power-of-two and other process counts),
# plus one large case that fills a good part of one GPU's memory.
WORKLOADS: List[Workload] = [
    Workload("P10_n512K", P=10, root=0, n=524_288, seed=160306809),
    Workload("P24_n4M", P=24, root=3, n=4_194_304, seed=160306810),
    Workload("P64_n16M", P=64, root=0, n=16_777_216, seed=160306811),
    Workload("P96_n12M_ragged", P=96, root=17, n=12_345_677, seed=160306812),
    Workload("P513_n128M", P=513, root=256, n=134_217_728, seed=160306813),
]


def workload(name: str) -> Workload:
    for w in WORKLOADS:
        if w.name == name:
            return w
    raise KeyError(name)


def stream_key(seed: int, stream: int) -> int:
    """Key of a byte stream: stream 0 is the root's message, stream r + 1 the
    poison of rank r."""
    return (seed ^ (stream * _GOLDEN)) & _MASK64


def splitmix64_word(key: int, k: int) -> int:
    """Word k of the stream with the given key, in plain Python integers."""
    z = (key + (k + 1) * _GOLDEN) & _MASK64
    z = ((z ^ (z >> 30)) * _MIX1) & _MASK64
    z = ((z ^ (z >> 27)) * _MIX2) & _MASK64
    return z ^ (z >> 31)


def bytes_numpy(seed: int, stream: int, nbytes: int, start: int = 0) -> np.ndarray:
    """Bytes ``[start, start + nbytes)`` of a stream as a numpy uint8 array."""
    if start:
        first = start // 8
        head = start - first * 8
        words = bytes_numpy_words(seed, stream, first, (head + nbytes + 7) // 8)
        return words.view(np.uint8)[head:head + nbytes].copy()
    return bytes_numpy_words(seed, stream, 0, (nbytes + 7) // 8).view(np.uint8)[:nbytes].copy()


def bytes_numpy_words(seed: int, stream: int, first_word: int, nwords: int) -> np.ndarray:
    """Words ``[first_word, first_word + nwords)`` of a stream, little-endian."""
    key = np.uint64(stream_key(seed, stream))
    with np.errstate(over="ignore"):
        k = np.arange(first_word + 1, first_word + nwords + 1, dtype=np.uint64)
        z = key + k * np.uint64(_GOLDEN)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(_MIX1)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(_MIX2)
        z = z ^ (z >> np.uint64(31))
    return z.astype("<u8")


def _s64(x: int) -> int:
    """Reinterpret an unsigned 64-bit value as a signed one."""
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


def bytes_torch(seed: int, stream: int, nbytes: int, device="cpu"):
    """Same bytes as :func:`bytes_numpy`, produced with torch int64 arithmetic
    on ``device`` (two's-complement wrap-around; logical shifts are emulated by
    masking after the arithmetic shift)."""
    import torch

    nwords = (nbytes + 7) // 8
    key = _s64(stream_key(seed, stream))
    k = torch.arange(1, nwords + 1, dtype=torch.int64, device=device)
    z = k * _s64(_GOLDEN) + key

    def lsr(v, s):
        return (v >> s) & ((1 << (64 - s)) - 1)

    z = (z ^ lsr(z, 30)) * _s64(_MIX1)
    z = (z ^ lsr(z, 27)) * _s64(_MIX2)
    z = z ^ lsr(z, 31)
    return z.view(torch.uint8)[:nbytes].clone()


def message_numpy(w: Workload) -> np.ndarray:
    return bytes_numpy(w.seed, 0, w.n)


def poison_numpy(w: Workload, rank: int, nbytes: int) -> np.ndarray:
    return bytes_numpy(w.seed, rank + 1, nbytes)


def message_torch(w: Workload, device="cpu"):
    return bytes_torch(w.seed, 0, w.n, device)


def poison_torch(w: Workload, rank: int, nbytes: int, device="cpu"):
    return bytes_torch(w.seed, rank + 1, nbytes, device)
