"""Test-side helpers: move seeded NumPy bundles to the device and drive the C-ABI calls
through the Python binding.  Holds no arithmetic of the method."""
from __future__ import annotations

import numpy as np
import torch


def dev(a: np.ndarray, dtype: str | None = None) -> torch.Tensor:
    """NumPy -> device tensor.  dtype "bf16"/"f32" for feature tensors (the values are already
    representable, so the cast is exact); None keeps integer / float32 arrays as they are."""
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
    elif dtype == "f32":
        t = t.to(torch.float32)
    return t.contiguous()


def host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        t = t.to(torch.float32)
    return t.detach().cpu().numpy()


def tdtype(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


class Forward:
    """Runs gate_select -> pack(qkv) [-> pack(x, gate-scaled)] -> attention -> unpack on the GPU."""

    def __init__(self, spa, B, N, C, H, dtype, container_len=0, use_counts=True, want_lse=True):
        self.spa, self.B, self.N, self.C, self.H, self.dtype = spa, B, N, C, H, dtype
        self.Dh = C // H
        self.container_len = container_len
        self.use_counts = use_counts
        td = tdtype(dtype)
        cap = B * N
        rows = cap + max(container_len - 1, 0)
        z = dict(device="cuda")
        self.scores = torch.empty(B, N, dtype=torch.float32, **z)
        self.mask = torch.empty(B, N, dtype=torch.uint8, **z)
        self.counts = torch.empty(B, dtype=torch.int32, **z) if use_counts else None
        self.packed_qkv = torch.full((rows, 3 * C), float("nan"), dtype=td, **z)
        self.cu = torch.empty(B + 1, dtype=torch.int32, **z)
        self.gidx = torch.full((cap,), -7, dtype=torch.int32, **z)
        self.inv = torch.empty(cap, dtype=torch.int32, **z)
        self.total = torch.empty(1, dtype=torch.int32, **z)
        self.out = torch.full((cap, C), float("nan"), dtype=td, **z)
        self.lse = torch.full((H, cap), float("nan"), dtype=torch.float32, **z) if want_lse else None
        self.y = torch.empty(B, N, C, dtype=td, **z)

    def run(self, x, w, bias, qkv, tau, s_up=None, base=None):
        spa, C = self.spa, self.C
        spa.spa_gate_select(x, w, bias, s_up, tau, self.scores, self.mask, self.counts)
        spa.spa_pack(qkv, self.mask, self.counts, None, self.container_len, self.packed_qkv, self.cu,
                     self.gidx, self.inv, self.total)
        p = self.packed_qkv
        spa.spa_packed_attention(p[:, :C], p[:, C:2 * C], p[:, 2 * C:], self.cu, self.B, self.N,
                                 self.H, self.Dh, self.out, self.lse)
        spa.spa_unpack(self.out, self.inv, base, self.y)
        return self
