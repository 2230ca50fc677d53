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


# ---- other layouts the library admits: rank bases that are 16-byte aligned but
# ---- not on 256-byte boundaries, and one allocation per rank in any address order

def device_rows(w: I.Workload, layout, pad: int = 64, device="cuda"):
    """P rank buffers as a list of 1-D uint8 tensors of equal size (the stride),
    filled like :func:`device_buffers`, plus whatever keeps their memory alive.

    layout
      int k        one block; every base sits k bytes past a 256-byte boundary
                   (k a multiple of 16), consecutive ranks one stride apart
      "mixed"      one block; the stride is a multiple of 16 but not of 256, so
                   the bases sit at different places inside their 256-byte
                   windows (all still congruent modulo 16)
      "per_rank"   one allocation per rank, handed to the ranks in a seeded
                   shuffled order (rank order and address order differ)
    """
    import torch

    stride = stride_of(w.n, pad)
    if layout == "per_rank":
        owned = [torch.empty(stride, dtype=torch.uint8, device=device) for _ in range(w.P)]
        order = np.random.default_rng(w.seed).permutation(w.P)
        rows = [owned[int(k)] for k in order]
        keep = owned
    else:
        if layout == "mixed":
            stride += 48
            first = 0
        else:
            first = int(layout)
            assert first % 16 == 0 and 0 <= first < 256
        block = torch.empty(first + w.P * stride + 256, dtype=torch.uint8, device=device)
        assert block.data_ptr() % 256 == 0
        rows = [block[first + r * stride: first + (r + 1) * stride] for r in range(w.P)]
        keep = block
    refill_rows(rows, w)
    return rows, keep


def refill_rows(rows, w: I.Workload) -> None:
    stride = rows[0].numel()
    for r in range(w.P):
        rows[r].copy_(I.poison_torch(w, r, stride, rows[r].device))
    rows[w.root][: w.n].copy_(I.message_torch(w, rows[w.root].device))


def host_rows(w: I.Workload, stride: int):
    return [host_row(w, r, stride) for r in range(w.P)]


def rows_to_numpy(rows) -> np.ndarray:
    import torch

    return torch.stack(list(rows)).cpu().numpy()
