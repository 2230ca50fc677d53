"""Shared by the GPU parity tests: the same seeded bytes as device buffers for
the library and as numpy buffers for the oracle."""

from __future__ import annotations

import numpy as np

from paper_1603_06809_amd import inputs as I


def stride_of(n: int, pad: int = 64) -> int:
    return (n + pad + 255) // 256 * 256


def host_row(w: I.Workload, rank: int, stride: int) -> np.ndarray:
    """Initial buffer of one rank: the message (root) or that rank's poison,
    followed by poison up to the stride."""
    row = I.poison_numpy(w, rank, stride)
    if rank == w.root:
        row[: w.n] = I.message_numpy(w)
    return row


def host_tail(w: I.Workload, rank: int, stride: int) -> np.ndarray:
    """Bytes [n, stride) of a rank's initial buffer (never part of a message)."""
    return I.bytes_numpy(w.seed, rank + 1, stride - w.n, start=w.n)


def host_buffers(w: I.Workload, pad: int = 64):
    stride = stride_of(w.n, pad)
    return [host_row(w, r, stride) for r in range(w.P)]


def device_buffers(w: I.Workload, pad: int = 64, device="cuda"):
    """One [P, stride] uint8 tensor; row r is rank r's buffer."""
    import torch

    stride = stride_of(w.n, pad)
    state = torch.empty((w.P, stride), dtype=torch.uint8, device=device)
    refill(state, w)
    return state


def refill(state, w: I.Workload) -> None:
    stride = state.shape[1]
    for r in range(w.P):
        state[r].copy_(I.poison_torch(w, r, stride, state.device))
    state[w.root, : w.n].copy_(I.message_torch(w, state.device))
