"""Randomised shapes through every form of the attention step: the packed, gathered and
from-the-mask forward forms must agree bit for bit with each other and with the oracle within
tolerance; the backward at token positions must agree with the oracle.  Shapes are drawn so that
segments straddle every tile size of the kernels (32, 64, 128, 256 keys; one, several and many
tiles; empty and full images; batches on both sides of the in-kernel ranking limits; seeds 40-43:
17 to 64 long images)."""
import numpy as np
import pytest
import torch

from oracle import spa_oracle as orc
from paper_2410_23608_amd import workloads as wlmod
from spa_harness import dev, host, tdtype

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def spa():
    from paper_2410_23608_amd import spa as mod
    return mod


def _draw(seed):
    """(B, N, H, Dh, dtype, per-image lengths): small N with many images or large N with few."""
    rng = np.random.default_rng(7000 + seed)
    dtype = "f32" if seed % 5 == 4 else "bf16"
    Dh = [32, 64][seed % 2]
    H = int(rng.integers(1, 4))
    kind = seed % 4
    if seed >= 40:       # 17 to 64 long images: the long-segment kernels number their blocks per workgroup, ranking
        B, N = ((40, 500), (20, 2600), (64, 300), (33, 1100))[seed - 40]      # by block count (B > blocks) or pairwise
        dtype, H = "bf16", 2
        lens = rng.integers(0, N + 1, size=B)
        lens[rng.integers(0, B)] = N
        lens[rng.integers(0, B)] = 0
        return rng, B, N, H, Dh, dtype, lens
    if kind == 0:        # many short images (the one-wave kernels, ranking of up to 64 images and beyond)
        B, N = int(rng.integers(40, 90)), int(rng.integers(20, 257))
    elif kind == 1:      # a few long images (the tiled kernels, several 128-key tiles and a ragged tail)
        B, N = int(rng.integers(1, 5)), int(rng.integers(300, 1400))
    elif kind == 2:      # lengths exactly on and next to tile edges
        B, N = 8, int(rng.choice([128, 256, 384, 512])) + int(rng.integers(0, 2))
    else:
        B, N = int(rng.integers(2, 12)), int(rng.integers(1, 300))
    if dtype == "f32":
        B, N = min(B, 6), min(N, 300)
    lens = rng.integers(0, N + 1, size=B)
    if kind == 2:
        edges = np.array([0, 1, 31, 32, 33, 64, 127, 128, 129, 255, 256, 257, N - 1, N])
        lens = rng.choice(edges[edges <= N], size=B)
    lens[rng.integers(0, B)] = N                      # one image keeps every token
    return rng, B, N, H, Dh, dtype, lens


@pytest.mark.parametrize("seed", range(44))
def test_random_shapes_all_forward_forms_and_backward(spa, seed):
    rng, B, N, H, Dh, dtype, lens = _draw(seed)
    C, cap, td = H * Dh, B * N, tdtype(dtype)
    mk = wlmod.round_bf16 if dtype == "bf16" else (lambda a: a)
    qkv = mk(rng.standard_normal((B, N, 3 * C)).astype(np.float32))
    base = mk(rng.standard_normal((B, N, C)).astype(np.float32)) if seed % 3 == 0 else None
    mask = np.zeros((B, N), np.uint8)
    for b, n in enumerate(lens):
        mask[b, rng.permutation(N)[:n]] = 1
    ref_cu, ref_gidx, ref_inv, T = orc.pack_indices(mask)
    ref_out, ref_lse = orc.attention_per_image(qkv[..., :C], qkv[..., C:2 * C], qkv[..., 2 * C:], mask, H)
    ref_y = orc.unpack(ref_out, ref_inv, B, N, base)
    print(f"seed {seed}: B {B} N {N} H {H} Dh {Dh} {dtype} T {T} base {base is not None}", flush=True)

    d_qkv, d_mask = dev(qkv, dtype), dev(mask)
    d_base = None if base is None else dev(base, dtype)
    flat = d_qkv.view(cap, 3 * C)
    packed = torch.zeros(cap, 3 * C, dtype=td, device="cuda")
    cu = torch.empty(B + 1, dtype=torch.int32, device="cuda")
    gidx = torch.empty(cap, dtype=torch.int32, device="cuda")
    inv = torch.empty(cap, dtype=torch.int32, device="cuda")
    tot = torch.empty(1, dtype=torch.int32, device="cuda")
    spa.spa_pack(d_qkv, d_mask, None, None, 0, packed, cu, gidx, inv, tot)
    torch.cuda.synchronize()
    assert np.array_equal(host(cu), ref_cu) and int(host(tot)[0]) == T
    assert np.array_equal(host(gidx)[:T], ref_gidx) and np.array_equal(host(inv), ref_inv)

    tol = 1e-5 if dtype == "f32" else 2e-2
    ytol = tol if base is None else 2 * tol          # base + out is rounded once more
    ys = {}
    out = torch.zeros(cap, C, dtype=td, device="cuda")
    lse = torch.zeros(H, cap, dtype=torch.float32, device="cuda")
    y = torch.full((B, N, C), float("nan"), dtype=td, device="cuda")
    spa.spa_packed_attention_unpack(packed[:, :C], packed[:, C:2 * C], packed[:, 2 * C:], cu, gidx, inv, d_base,
                                    H, Dh, y, out, lse)
    ys["packed"] = y
    y = torch.full((B, N, C), float("nan"), dtype=td, device="cuda")
    spa.spa_gathered_attention_unpack(flat[:, :C], flat[:, C:2 * C], flat[:, 2 * C:], cu, gidx, inv, d_base, H, Dh, y)
    ys["gathered"] = y
    if N <= 256:
        y = torch.full((B, N, C), float("nan"), dtype=td, device="cuda")
        spa.spa_selected_attention_unpack(flat[:, :C], flat[:, C:2 * C], flat[:, 2 * C:], d_mask, d_base, H, Dh, y)
        ys["selected"] = y
    torch.cuda.synchronize()
    assert np.max(np.abs(host(out)[:T] - ref_out), initial=0.0) <= tol
    assert np.max(np.abs(host(lse)[:, :T] - ref_lse), initial=0.0) <= (1e-4 if dtype == "f32" else 1e-3)
    for form, y in ys.items():
        assert np.max(np.abs(host(y) - ref_y)) <= ytol, form
        assert torch.equal(y, ys["packed"]), form

    # backward at token positions against the oracle (gradients of the packed rows, scattered)
    dy = mk(rng.standard_normal((B, N, C)).astype(np.float32))
    ref_dout = dy.reshape(cap, C)[ref_gidx]
    rdq, rdk, rdv = orc.attention_backward_per_image(qkv[..., :C], qkv[..., C:2 * C], qkv[..., 2 * C:], mask,
                                                     ref_dout, H)
    ws = torch.empty(spa.spa_attention_bwd_workspace_bytes(B, N, H, Dh, spa.dtype_code(out)), dtype=torch.uint8,
                     device="cuda")
    got = torch.full((cap, 3 * C), float("nan"), dtype=td, device="cuda")
    spa.spa_packed_attention_bwd_tokens(packed[:, :C], packed[:, C:2 * C], packed[:, 2 * C:], out, dev(dy, dtype), lse,
                                        cu, B, N, H, Dh, gidx, inv, got[:, :C], got[:, C:2 * C], got[:, 2 * C:], ws)
    torch.cuda.synchronize()
    g = host(got)
    sel = mask.reshape(-1) != 0
    assert not np.isnan(g).any() and not g[~sel].any()
    gtol = 2e-5 if dtype == "f32" else 2e-2
    for name, part, ref in (("dq", g[:, :C], rdq), ("dk", g[:, C:2 * C], rdk), ("dv", g[:, 2 * C:], rdv)):
        scale = max(1.0, float(np.max(np.abs(ref), initial=0.0)))
        assert np.max(np.abs(part[sel] - ref), initial=0.0) / scale <= gtol, name
