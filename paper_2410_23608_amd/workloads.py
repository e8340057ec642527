"""Seeded synthetic inputs for the Select-and-Pack Attention (SPA) hot path.

This module only *draws inputs*: token features, gate weights, projected q/k/v
stand-ins, foreground masks, labels and upstream gradients.  It contains none of
the method's steps (no scoring, selection, packing, attention or unpacking) and is
the only code shared by the CPU oracle's tests and the HIP path's tests/bench.

Every bundle is a pure function of (workload, seed); the generator is NumPy's
counter-based Philox.  Values handed out for a bf16 workload are float32 arrays
that are exactly representable in bf16 (round-to-nearest-even is applied here), so
both sides start from identical bits.

The shapes and sparsity follow the paper's workloads: ViT / Swin-like token grids,
foreground given by object blobs (segmentation-style) or stacked boxes
(detection-style, Section 3.2 "Multi-Scale Supervised Selection"), select ratios
in the range the paper reports (Tables 4-6).  They stand in for the paper's
datasets, which are not used.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional, Tuple

import numpy as np

__all__ = [
    "Workload", "WORKLOADS", "HIER_STAGES", "generate", "generate_hierarchy",
    "round_bf16", "foreground_masks",
]


@dataclass(frozen=True)
class Workload:
    name: str
    B: int                      # images per batch
    grid: Tuple[int, int]       # token grid (h, w); N = h*w
    C: int                      # embedding dim
    H: int                      # heads (C = H*Dh)
    dtype: str                  # "f32" or "bf16"
    frac: Tuple[float, float]   # per-image selected fraction ~ U[lo, hi]
    mask_kind: str              # "disc" (blobs) or "rect" (stacked boxes)
    train: bool = False         # forward+backward workload
    tau: float = 0.5            # selection threshold on sigmoid(score)
    bias: float = 0.0

    @property
    def N(self) -> int:
        return self.grid[0] * self.grid[1]

    @property
    def Dh(self) -> int:
        return self.C // self.H


WORKLOADS: Dict[str, Workload] = {
    # tiny fp32 case the oracle finishes in well under a second
    "tiny": Workload("tiny", 2, (14, 14), 64, 2, "f32", (0.20, 0.40), "disc"),
    # ViT-S-shaped classification, forward
    "vit_s": Workload("vit_s", 64, (14, 14), 384, 6, "bf16", (0.10, 0.90), "disc"),
    # ViT-B-shaped training step, forward + backward
    "vit_b_train": Workload("vit_b_train", 64, (14, 14), 768, 12, "bf16", (0.05, 0.95), "disc", train=True),
    # detection-shaped high resolution: 800x1344 at stride 16
    "det": Workload("det", 8, (50, 84), 256, 8, "bf16", (0.05, 0.40), "rect"),
}

# Swin-like four-stage hierarchy (batch 16); selection is recomputed per stage.
HIER_STAGES = (
    Workload("hier_s1", 16, (56, 56), 96, 3, "bf16", (0.10, 0.60), "disc", train=True),
    Workload("hier_s2", 16, (28, 28), 192, 6, "bf16", (0.10, 0.60), "disc", train=True),
    Workload("hier_s3", 16, (14, 14), 384, 12, "bf16", (0.10, 0.60), "disc", train=True),
    Workload("hier_s4", 16, (7, 7), 768, 24, "bf16", (0.10, 0.60), "disc", train=True),
)


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(stream)]))


def round_bf16(a: np.ndarray) -> np.ndarray:
    """float32 -> nearest bf16 (ties to even), returned as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    out = ((u + r) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return out.view(np.float32).reshape(a.shape)


def _to_dtype(a: np.ndarray, dtype: str) -> np.ndarray:
    a = np.asarray(a, dtype=np.float32)
    return round_bf16(a) if dtype == "bf16" else a


def _disc_field(rng: np.random.Generator, h: int, w: int) -> np.ndarray:
    """Higher = closer to the centre of one of 1-3 random discs (scaled by radius)."""
    k = int(rng.integers(1, 4))
    cy = rng.uniform(0, h, size=k)
    cx = rng.uniform(0, w, size=k)
    rad = rng.uniform(0.6, 1.0, size=k)
    yy, xx = np.meshgrid(np.arange(h) + 0.5, np.arange(w) + 0.5, indexing="ij")
    d = np.sqrt((yy[None] - cy[:, None, None]) ** 2 + (xx[None] - cx[:, None, None]) ** 2)
    return (-d / rad[:, None, None]).max(axis=0)


def _rect_field(rng: np.random.Generator, h: int, w: int) -> np.ndarray:
    """Higher = deeper inside one of 3-20 random axis-aligned boxes (stacked boxes)."""
    k = int(rng.integers(3, 21))
    cy = rng.uniform(0, h, size=k)
    cx = rng.uniform(0, w, size=k)
    ay = rng.uniform(0.3, 1.0, size=k)
    ax = rng.uniform(0.3, 1.0, size=k)
    yy, xx = np.meshgrid(np.arange(h) + 0.5, np.arange(w) + 0.5, indexing="ij")
    d = np.maximum(np.abs(yy[None] - cy[:, None, None]) / ay[:, None, None],
                   np.abs(xx[None] - cx[:, None, None]) / ax[:, None, None])
    return (-d).max(axis=0)


def foreground_masks(wl: Workload, seed: int) -> np.ndarray:
    """Planted foreground mask [B, N] uint8 with the workload's per-image ratios.

    disc: blobs grown until exactly round(f_b * N) tokens are covered.
    rect: boxes grown (common scale) to the coverage closest to f_b * N, so that
          the foreground stays a union of exact rectangles.
    """
    h, w = wl.grid
    N = h * w
    rng = _rng(seed, 1)
    out = np.zeros((wl.B, N), dtype=np.uint8)
    for b in range(wl.B):
        f = rng.uniform(wl.frac[0], wl.frac[1])
        target = int(min(N, max(1, round(f * N))))
        if wl.mask_kind == "disc":
            field = _disc_field(rng, h, w).reshape(-1)
            field = field + rng.uniform(0, 1e-6, size=N)       # seeded tie-break
            order = np.argsort(-field, kind="stable")
            out[b, order[:target]] = 1
        elif wl.mask_kind == "rect":
            field = _rect_field(rng, h, w).reshape(-1)
            sf = np.sort(field)[::-1]                           # descending
            last = np.flatnonzero(np.append(sf[1:] != sf[:-1], True))
            counts = last + 1                                   # tokens with field >= level
            t = sf[last[int(np.argmin(np.abs(counts - target)))]]
            out[b, field >= t] = 1
        else:
            raise ValueError(wl.mask_kind)
    return out


def _planted_features(rng: np.random.Generator, wl: Workload, sign_mask: np.ndarray,
                      w: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Token features ~ N(0, I) whose component along the gate weight is replaced so
    that the linear gate's logit equals a planted value with |logit - theta| >= 0.5:
    positive where sign_mask is set, negative elsewhere.  Only the 1-D component along
    w changes, so the marginals stay close to N(0, 1)."""
    B, N, C = wl.B, wl.N, wl.C
    theta = float(np.log(wl.tau / (1.0 - wl.tau)))
    z = rng.standard_normal((B, N, C), dtype=np.float32)
    mag = 0.5 + np.abs(rng.standard_normal((B, N)))
    logit = theta + np.where(sign_mask.astype(bool), mag, -mag)
    w64 = w.astype(np.float64)
    wn2 = float(w64 @ w64)
    proj = (z.reshape(-1, C).astype(np.float64) @ w64).reshape(B, N)
    coef = ((logit - wl.bias - proj) / wn2).astype(np.float32)
    x = z + coef[:, :, None] * w[None, None, :].astype(np.float32)
    return _to_dtype(x, wl.dtype), logit


def generate(wl: Workload, seed: int = 0, planted_mask: Optional[np.ndarray] = None,
             with_qkv: bool = True) -> Dict[str, np.ndarray]:
    """One seeded input bundle for a workload.

    keys: planted_mask [B,N] u8, planted_logit [B,N] f64, w [C] f32, bias float,
          x [B,N,C] f32, qkv [B,N,3C] f32 (q | k | v, each [H,Dh]; stand-ins for the
          projected tokens), labels [B,N] u8 (mask with 5% flips), dy [B,N,C] f32
          (upstream gradient; training workloads only).
    All float arrays hold values exactly representable in wl.dtype.
    """
    if planted_mask is None:
        planted_mask = foreground_masks(wl, seed)
    rng = _rng(seed, 2)
    C = wl.C
    w = _to_dtype(rng.standard_normal(C, dtype=np.float32) / np.sqrt(np.float32(C)), wl.dtype)
    x, logit = _planted_features(rng, wl, planted_mask, w)
    out = {
        "planted_mask": planted_mask, "planted_logit": logit,
        "w": w, "bias": float(wl.bias), "x": x,
    }
    if with_qkv:
        rq = _rng(seed, 3)
        out["qkv"] = _to_dtype(rq.standard_normal((wl.B, wl.N, 3 * C), dtype=np.float32), wl.dtype)
    rl = _rng(seed, 4)
    flips = rl.uniform(size=planted_mask.shape) < 0.05
    out["labels"] = (planted_mask.astype(bool) ^ flips).astype(np.uint8)
    if wl.train:
        out["dy"] = _to_dtype(rl.standard_normal((wl.B, wl.N, C), dtype=np.float32), wl.dtype)
    return out


def _pool_mask(m: np.ndarray, h: int, w: int) -> np.ndarray:
    B = m.shape[0]
    return m.reshape(B, h // 2, 2, w // 2, 2).max(axis=(2, 4)).reshape(B, -1)


def generate_hierarchy(seed: int = 0, stages=HIER_STAGES, B: Optional[int] = None):
    """Bundles for the four-stage hierarchy.  The finest stage's foreground is a blob
    mask; each coarser stage's foreground is the 2x2 max-pool of the finer one.  A
    stage's own gate is planted to fire on a seeded ~85% subset of its foreground, so
    the up-scale scores handed down from the finer stage (Eq. for s = Max(gate, s_up))
    genuinely add tokens."""
    bundles = []
    mask = None
    for i, wl in enumerate(stages):
        if B is not None:
            wl = replace(wl, B=B)
        h, w = wl.grid
        if i == 0:
            mask = foreground_masks(wl, seed)
            own = mask
        else:
            ph, pw = stages[i - 1].grid
            mask = _pool_mask(mask, ph, pw)
            keep = _rng(seed, 10 + i).uniform(size=mask.shape) < 0.85
            own = (mask.astype(bool) & keep).astype(np.uint8)
        bun = generate(wl, seed * 16 + i, planted_mask=own)
        bun["stage_foreground"] = mask
        bun["workload"] = wl
        bundles.append(bun)
    return bundles
