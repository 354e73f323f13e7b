"""Helpers for the GPU tests: host <-> device moves and the fragment-order layout of the split output.
No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np


def to_device(store: np.ndarray):
    """Column-major (ld, cols) Fortran array -> torch CUDA tensor over the same bytes."""
    import torch
    assert store.flags.f_contiguous and store.dtype == np.float32
    return torch.from_numpy(np.ascontiguousarray(store.T)).cuda()


def to_host(t, ld: int, cols: int) -> np.ndarray:
    """Inverse of to_device: (ld, cols) Fortran array."""
    return t.cpu().numpy().reshape(cols, ld).T


def empty_colmajor(ld: int, cols: int, fill=None):
    import torch
    t = torch.empty((cols, ld), dtype=torch.float32, device="cuda")
    if fill is not None:
        t.fill_(fill)
    return t


def round_up(v: int, m: int) -> int:
    return (v + m - 1) // m * m


def pack_fragment_order(parts, row_pad: int = 256, depth_pad: int = 32) -> np.ndarray:
    """Places `parts` (a list of rows x depth uint16 arrays, high part first) in the layout
    ecgemm_split documents: [row_block][k_step][part][lane][8] with lane = ((k % 16) / 8) * 32 + r % 32."""
    rows, depth = parts[0].shape
    Rp, Kp = round_up(rows, row_pad), round_up(depth, depth_pad)
    out = []
    for p in parts:
        full = np.zeros((Rp, Kp), dtype=np.uint16)
        full[:rows, :depth] = p
        # (row_block, r, k_step, half, e) -> (row_block, k_step, half, r, e)
        out.append(full.reshape(Rp // 32, 32, Kp // 16, 2, 8).transpose(0, 2, 3, 1, 4))
    stacked = np.stack(out, axis=2)  # (row_block, k_step, part, half, r, e)
    return np.ascontiguousarray(stacked).reshape(-1)


def pack_fp32_fragment_order(X: np.ndarray, row_pad: int = 256, depth_pad: int = 32) -> np.ndarray:
    """Layout of ecgemm_split for ECGEMM_MODE_FP32_MFMA: 1 KiB chunks [row_block][k_step][half][lane][4] of float32,
    half = (k % 16) / 8, lane = (k % 2) * 32 + r % 32, float (k % 8) / 2: what v_mfma_f32_32x32x2_f32 takes, four
    2-deep steps per 16-byte lane entry.  Returned as the uint16 view the other layouts are compared in."""
    rows, depth = X.shape
    Rp, Kp = round_up(rows, row_pad), round_up(depth, depth_pad)
    full = np.zeros((Rp, Kp), dtype=np.float32)
    full[:rows, :depth] = X
    # (row_block, r, k_step, half, slot, parity) -> (row_block, k_step, half, parity, r, slot)
    v = full.reshape(Rp // 32, 32, Kp // 16, 2, 4, 2).transpose(0, 2, 3, 5, 1, 4)
    return np.ascontiguousarray(v).reshape(-1).view(np.uint16)
