"""Parity at the large end of the documented limits: batches beyond the sizes for which the kernels
rank the images (64 / 256 / 512), one very long segment, and half a million tokens through the
gate and the packing index.  Every value is compared with the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import spa_oracle as orc
from paper_2410_23608_amd import workloads as wlmod
from spa_harness import dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def spa():
    from paper_2410_23608_amd import spa as mod
    return mod


def _fwd_bwd(spa, qkv, mask, dy, H, Dh):
    """pack -> attention -> token-position backward on bf16 inputs; returns host arrays."""
    B, N, C3 = qkv.shape
    C, cap = C3 // 3, B * N
    td = torch.bfloat16
    packed = torch.zeros(cap, 3 * C, dtype=td, device="cuda")
    cu = torch.empty(B + 1, dtype=torch.int32, device="cuda")
    gidx = torch.zeros(cap, dtype=torch.int32, device="cuda")
    inv = torch.empty(cap, dtype=torch.int32, device="cuda")
    tot = torch.empty(1, dtype=torch.int32, device="cuda")
    spa.spa_pack(dev(qkv, "bf16"), dev(mask), None, None, 0, packed, cu, gidx, inv, tot)
    pq, pk, pv = packed[:, :C], packed[:, C:2 * C], packed[:, 2 * C:]
    out = torch.zeros(cap, C, dtype=td, device="cuda")
    lse = torch.zeros(H, cap, dtype=torch.float32, device="cuda")
    spa.spa_packed_attention(pq, pk, pv, cu, B, N, H, Dh, out, lse)
    ws = torch.empty(max(spa.spa_attention_bwd_workspace_bytes(B, N, H, Dh, spa.SPA_BF16), 256), dtype=torch.uint8,
                     device="cuda")
    grads = torch.full((cap, 3 * C), float("nan"), dtype=td, device="cuda")
    spa.spa_packed_attention_bwd_tokens(pq, pk, pv, out, dev(dy, "bf16"), lse, cu, B, N, H, Dh, gidx, inv, grads[:, :C],
                                        grads[:, C:2 * C], grads[:, 2 * C:], ws)
    torch.cuda.synchronize()
    return host(cu), host(gidx), host(inv), host(out), host(lse), host(grads)


def _check(spa, B, N, H, Dh, dens, seed):
    C = H * Dh
    rng = np.random.default_rng(seed)
    qkv = wlmod.round_bf16(rng.standard_normal((B, N, 3 * C)).astype(np.float32))
    dy = wlmod.round_bf16(rng.standard_normal((B, N, C)).astype(np.float32))
    mask = (rng.uniform(size=(B, N)) < rng.uniform(0, 2 * dens, size=(B, 1))).astype(np.uint8)
    mask[B // 2] = 0                                          # an image with nothing selected in the middle
    cu, gidx, inv, out, lse, grads = _fwd_bwd(spa, qkv, mask, dy, H, Dh)
    cu_r, g_r, inv_r, T = orc.pack_indices(mask)
    assert np.array_equal(cu, cu_r) and np.array_equal(gidx[:T], g_r) and np.array_equal(inv, inv_r)
    q, k, v = qkv[..., :C], qkv[..., C:2 * C], qkv[..., 2 * C:]
    ref_out, ref_lse = orc.attention_per_image(q, k, v, mask, H)
    assert np.max(np.abs(out[:T] - ref_out)) <= 2e-2
    assert np.max(np.abs(lse[:, :T] - ref_lse)) <= 1e-3
    refs = orc.attention_backward_per_image(q, k, v, mask, dy.reshape(-1, C)[g_r], H)
    sel = mask.reshape(-1).astype(bool)
    assert np.all(grads[~sel] == 0.0)                         # unselected tokens: zero gradient rows
    for i, r in enumerate(refs):
        err = np.max(np.abs(grads[g_r, i * C:(i + 1) * C] - r)) / max(1.0, np.max(np.abs(r)))
        assert err <= 2e-2, (i, err)


@pytest.mark.parametrize("B,N,H,Dh", [(300, 40, 2, 64),      # one-wave forward without the weight numbering (B > 64), backward ranked through LDS
                                      (600, 40, 2, 32),      # backward beyond 512 images: launch order = image order
                                      (300, 300, 1, 32),     # long-segment kernels beyond 256 images
                                      (100, 300, 2, 32),     # long-segment kernels, 65 to 256 images: ranked through LDS, blocks not compacted
                                      (48, 300, 12, 32),     # the same with at most 64 images but more than 512 (image, head) pairs
                                      (70, 196, 3, 64)])     # ViT-shaped, just past one wave of images
def test_many_images(spa, B, N, H, Dh):
    _check(spa, B, N, H, Dh, 0.5, seed=B + N)


def test_one_very_long_segment(spa):
    """4096 selected tokens in ONE image (32 key tiles of 128, 64-token backward tiles), next to a short one."""
    B, N, H, Dh = 2, 4096, 2, 32
    C = H * Dh
    rng = np.random.default_rng(4096)
    qkv = wlmod.round_bf16(rng.standard_normal((B, N, 3 * C)).astype(np.float32))
    dy = wlmod.round_bf16(rng.standard_normal((B, N, C)).astype(np.float32))
    mask = np.zeros((B, N), dtype=np.uint8)
    mask[0] = 1
    mask[1, ::37] = 1
    cu, gidx, inv, out, lse, grads = _fwd_bwd(spa, qkv, mask, dy, H, Dh)
    cu_r, g_r, inv_r, T = orc.pack_indices(mask)
    assert np.array_equal(cu, cu_r) and np.array_equal(gidx[:T], g_r) and np.array_equal(inv, inv_r)
    q, k, v = qkv[..., :C], qkv[..., C:2 * C], qkv[..., 2 * C:]
    ref_out, ref_lse = orc.attention_per_image(q, k, v, mask, H)
    assert np.max(np.abs(out[:T] - ref_out)) <= 2e-2
    assert np.max(np.abs(lse[:, :T] - ref_lse)) <= 1e-3
    refs = orc.attention_backward_per_image(q, k, v, mask, dy.reshape(-1, C)[g_r], H)
    for i, r in enumerate(refs):
        err = np.max(np.abs(grads[g_r, i * C:(i + 1) * C] - r)) / max(1.0, np.max(np.abs(r)))
        assert err <= 2e-2, (i, err)


def test_half_a_million_tokens_through_gate_and_index(spa):
    """2048 images x 256 tokens: scores within tolerance, mask / counts / cu_seqlens / gather_idx / inv_pos
    bit for bit (tokens whose logit is within 1e-3 of the threshold are left out of the mask check and
    the index is compared for the device's own mask), by the two-launch and the one-launch form."""
    B, N, C = 2048, 256, 64
    rng = np.random.default_rng(5)
    x = wlmod.round_bf16(rng.standard_normal((B, N, C)).astype(np.float32))
    w = wlmod.round_bf16((rng.standard_normal(C) / 8).astype(np.float32))
    tau, bias = 0.5, 0.0
    s_ref = orc.gate_only(x, w, bias)
    xd, wd = dev(x, "bf16"), dev(w, "bf16")
    cap = B * N
    ints = lambda n: torch.full((n,), -3, dtype=torch.int32, device="cuda")
    for fused in (False, True):
        scores = torch.empty(B, N, dtype=torch.float32, device="cuda")
        mask = torch.empty(B, N, dtype=torch.uint8, device="cuda")
        counts, cu, gidx, inv, tot = ints(B), ints(B + 1), ints(cap), ints(cap), ints(1)
        if fused:
            ws = torch.zeros(17 * 1088, dtype=torch.int32, device="cuda")
            spa.spa_gate_select_index(xd, wd, bias, None, tau, scores, mask, counts, cu, gidx, inv, tot, ws)
        else:
            spa.spa_gate_select(xd, wd, bias, None, tau, scores, mask, counts)
            spa.spa_pack(None, mask, counts, None, 0, None, cu, gidx, inv, tot)
        torch.cuda.synchronize()
        s, m = host(scores), host(mask)
        assert np.max(np.abs(s - s_ref) / (1 + np.abs(s_ref))) <= 1e-3
        m_ref, _ = orc.select(s_ref, tau)
        clear = np.abs(s_ref - orc.threshold_logit(tau)) > 1e-3
        assert np.array_equal(m[clear], m_ref[clear])
        cu_r, g_r, inv_r, T = orc.pack_indices(m)
        assert int(host(tot)[0]) == T
        assert np.array_equal(host(counts), m.reshape(B, N).sum(1).astype(np.int32))
        assert np.array_equal(host(cu), cu_r) and np.array_equal(host(gidx)[:T], g_r) and np.array_equal(host(inv), inv_r)
        if fused:
            assert int(ws.abs().sum().item()) == 0            # the arrival counters are left zero
