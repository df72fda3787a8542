"""Helpers shared by the GPU parity tests: move generator output to the device,
run the C-ABI calls through the binding, and compare with the CPU oracle."""
from __future__ import annotations

import numpy as np


def to_dev(bits: np.ndarray):
    """uint16 bf16 bit patterns [N][H][d] -> torch bf16 device tensor [1][N][H][d]."""
    import torch
    t = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16)
    return t.unsqueeze(0).cuda()


def bf16_dev_to_f32(t) -> np.ndarray:
    return t.float().cpu().numpy()


def alloc_layer(sp, cfg, q, k, n_dense):
    """Output / pattern / workspace buffers for one layer."""
    import torch
    nqb = cfg.seq // cfg.block
    shape = sp.shape_of(q, k, None, cfg.block)
    o = torch.empty_like(q)
    ws = torch.empty(sp.sp_workspace_bytes(shape, n_dense), dtype=torch.uint8, device="cuda")
    scores = torch.empty((1, n_dense, nqb, nqb), dtype=torch.float32, device="cuda")
    kb_idx = torch.empty((1, n_dense, nqb, nqb), dtype=torch.int32, device="cuda")
    kb_cnt = torch.empty((1, n_dense, nqb), dtype=torch.int32, device="cuda")
    return shape, o, ws, scores, kb_idx, kb_cnt


def err_stats(got: np.ndarray, want: np.ndarray):
    d = np.abs(got.astype(np.float64) - want.astype(np.float64))
    return float(d.max()), float(d.mean())
