"""Parity of the HIP backward path (attention backward, gate backward + selection loss,
and the transposes of pack / unpack) against the CPU oracle, through the C-ABI binding."""
import dataclasses

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


def _rel(got, ref):
    """max abs error relative to max(1, |ref|_inf) — the bound used for gradients."""
    return float(np.max(np.abs(got - ref)) / max(1.0, np.max(np.abs(ref)))) if ref.size else 0.0


def _attention_fwd_bwd(spa, q, k, v, mask, dout_packed, H, dtype):
    B, N, C = q.shape
    Dh = C // H
    cap = B * N
    td = tdtype(dtype)
    qkv = np.concatenate([q, k, v], axis=2).astype(np.float32)
    packed = torch.zeros(cap, 3 * C, dtype=td, device="cuda")
    cu = torch.empty(B + 1, dtype=torch.int32, device="cuda")
    out = torch.zeros(cap, C, dtype=td, device="cuda")
    lse = torch.zeros(H, cap, dtype=torch.float32, device="cuda")
    spa.spa_pack(dev(qkv, dtype), dev(mask), None, None, 0, packed, cu, None, None, None)
    pq, pk, pv = packed[:, :C], packed[:, C:2 * C], packed[:, 2 * C:]
    spa.spa_packed_attention(pq, pk, pv, cu, B, N, H, Dh, out, lse)
    T = dout_packed.shape[0]
    dout = torch.zeros(cap, C, dtype=td, device="cuda")
    dout[:T] = dev(dout_packed, dtype)
    grads = torch.full((cap, 3 * C), float("nan"), dtype=td, device="cuda")
    ws = torch.empty(spa.spa_attention_bwd_workspace_bytes(B, N, H, Dh, spa.dtype_code(out)), dtype=torch.uint8,
                     device="cuda")
    spa.spa_packed_attention_bwd(pq, pk, pv, out, dout, lse, cu, B, N, H, Dh,
                                 grads[:, :C], grads[:, C:2 * C], grads[:, 2 * C:], ws)
    torch.cuda.synchronize()
    g = host(grads)
    return g[:, :C], g[:, C:2 * C], g[:, 2 * C:]


@pytest.mark.parametrize("N", [257, 256, 224, 100, 40])      # > 256: the long-segment kernels; else the one-kernel form
@pytest.mark.parametrize("dtype,Dh", [("f32", 32), ("f32", 64), ("bf16", 32), ("bf16", 64)])
def test_attention_backward_matches_oracle(spa, dtype, Dh, N):
    H = 2
    C = H * Dh
    lens = [n for n in [0, 1, 5, 31, 32, 33, 64, 65, 96, 127, 129, 200, 224, 225] if n < N] + [N]
    B = len(lens)
    rng = np.random.default_rng(21)
    mk = wlmod.round_bf16 if dtype == "bf16" else (lambda a: a)
    q, k, v = (mk(rng.standard_normal((B, N, C)).astype(np.float32)) for _ in range(3))
    mask = np.zeros((B, N), np.uint8)
    for b, n in enumerate(lens):
        mask[b, rng.permutation(N)[:n]] = 1
    T = int(mask.sum())
    dO = mk(rng.standard_normal((T, C)).astype(np.float32))
    rdq, rdk, rdv = orc.attention_backward_per_image(q, k, v, mask, dO, H)
    dq, dk, dv = _attention_fwd_bwd(spa, q, k, v, mask, dO, H, dtype)
    tol = 2e-5 if dtype == "f32" else 2e-2
    for name, got, ref in (("dq", dq, rdq), ("dk", dk, rdk), ("dv", dv, rdv)):
        assert np.all(np.isnan(got[T:])), name              # rows past T untouched
        assert _rel(got[:T], ref) <= tol, (name, _rel(got[:T], ref))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("Dh,H,N", [(64, 2, 256), (64, 3, 196), (32, 4, 100), (32, 2, 40), (32, 3, 700), (64, 2, 300)])
def test_attention_backward_at_token_positions_equals_three_calls(spa, Dh, H, N, dtype):
    """spa_packed_attention_bwd_tokens = unpack_bwd + attention backward + pack_bwd (x3): same bits at the
    selected tokens, zeros elsewhere, nothing else written."""
    C = H * Dh
    lens = [n for n in [0, 1, 31, 33, 64, 97, 130, 200, 257, 513] if n < N] + [N, 0]
    B, cap = len(lens), len(lens) * N
    rng = np.random.default_rng(N + Dh)
    qkv = wlmod.round_bf16(rng.standard_normal((B, N, 3 * C)).astype(np.float32))
    mask = np.zeros((B, N), np.uint8)
    for b, n in enumerate(lens):
        mask[b, rng.permutation(N)[:n]] = 1
    dy = dev(wlmod.round_bf16(rng.standard_normal((B, N, C)).astype(np.float32)), dtype)
    td = tdtype(dtype)
    packed = torch.zeros(cap, 3 * C, dtype=td, device="cuda")
    cu = torch.empty(B + 1, dtype=torch.int32, device="cuda")
    gidx = torch.empty(cap, dtype=torch.int32, device="cuda")
    inv = torch.empty(cap, dtype=torch.int32, device="cuda")
    tot = torch.empty(1, dtype=torch.int32, device="cuda")
    spa.spa_pack(dev(qkv, dtype), dev(mask), None, None, 0, packed, cu, gidx, inv, tot)
    pq, pk, pv = packed[:, :C], packed[:, C:2 * C], packed[:, 2 * C:]
    out = torch.zeros(cap, C, dtype=td, device="cuda")
    lse = torch.zeros(H, cap, dtype=torch.float32, device="cuda")
    spa.spa_packed_attention(pq, pk, pv, cu, B, N, H, Dh, out, lse)
    # three calls
    dout = torch.zeros(cap, C, dtype=td, device="cuda")
    gp = torch.zeros(cap, 3 * C, dtype=td, device="cuda")
    ws = torch.empty(spa.spa_attention_bwd_workspace_bytes(B, N, H, Dh, spa.dtype_code(out)), dtype=torch.uint8,
                     device="cuda")
    ref = torch.full((B, N, 3 * C), float("nan"), dtype=td, device="cuda")
    spa.spa_unpack_bwd(dy, gidx, tot, dout)
    spa.spa_packed_attention_bwd(pq, pk, pv, out, dout, lse, cu, B, N, H, Dh, gp[:, :C], gp[:, C:2 * C], gp[:, 2 * C:], ws)
    spa.spa_pack_bwd(gp, inv, ref)
    # one call, into a wider buffer whose extra columns must stay untouched
    got = torch.full((cap, 3 * C + 8), float("nan"), dtype=td, device="cuda")
    spa.spa_packed_attention_bwd_tokens(pq, pk, pv, out, dy, lse, cu, B, N, H, Dh, gidx, inv,
                                        got[:, :C], got[:, C:2 * C], got[:, 2 * C:3 * C],
                                        ws if N > 256 or dtype == "f32" else None)
    torch.cuda.synchronize()
    assert torch.equal(got[:, :3 * C], ref.view(cap, 3 * C))
    assert bool(torch.isnan(got[:, 3 * C:]).all())


@pytest.mark.parametrize("fill", [0, 1])
def test_attention_backward_at_token_positions_degenerate_masks(spa, fill):
    """Nothing selected: all gradients zero.  Everything selected: the plain backward, row for row."""
    B, N, H, Dh = 3, 70, 2, 32
    C, cap = H * Dh, B * N
    rng = np.random.default_rng(5)
    qkv = dev(wlmod.round_bf16(rng.standard_normal((B, N, 3 * C)).astype(np.float32)), "bf16")
    dy = dev(wlmod.round_bf16(rng.standard_normal((B, N, C)).astype(np.float32)), "bf16")
    mask = torch.full((B, N), fill, dtype=torch.uint8, device="cuda")
    td = torch.bfloat16
    packed = torch.zeros(cap, 3 * C, dtype=td, device="cuda")
    cu = torch.empty(B + 1, dtype=torch.int32, device="cuda")
    gidx = torch.zeros(cap, dtype=torch.int32, device="cuda")
    inv = torch.empty(cap, dtype=torch.int32, device="cuda")
    tot = torch.empty(1, dtype=torch.int32, device="cuda")
    spa.spa_pack(qkv, mask, None, None, 0, packed, cu, gidx, inv, tot)
    pq, pk, pv = packed[:, :C], packed[:, C:2 * C], packed[:, 2 * C:]
    out = torch.zeros(cap, C, dtype=td, device="cuda")
    lse = torch.zeros(H, cap, dtype=torch.float32, device="cuda")
    spa.spa_packed_attention(pq, pk, pv, cu, B, N, H, Dh, out, lse)
    got = torch.full((cap, 3 * C), float("nan"), dtype=td, device="cuda")
    spa.spa_packed_attention_bwd_tokens(pq, pk, pv, out, dy, lse, cu, B, N, H, Dh, gidx, inv,
                                        got[:, :C], got[:, C:2 * C], got[:, 2 * C:])
    torch.cuda.synchronize()
    if fill == 0:
        assert int(tot.item()) == 0 and bool((got == 0).all())
    else:
        ref = torch.full((cap, 3 * C), float("nan"), dtype=td, device="cuda")
        ws = torch.empty(spa.spa_attention_bwd_workspace_bytes(B, N, H, Dh, spa.SPA_BF16), dtype=torch.uint8, device="cuda")
        spa.spa_packed_attention_bwd(pq, pk, pv, out, dy.view(cap, C), lse, cu, B, N, H, Dh,
                                     ref[:, :C], ref[:, C:2 * C], ref[:, 2 * C:], ws)
        torch.cuda.synchronize()
        assert int(tot.item()) == cap and torch.equal(got, ref)


@pytest.mark.parametrize("N", [300, 190])
def test_attention_backward_is_bit_stable(spa, N):
    B, H, Dh = 4, 2, 64
    C = H * Dh
    rng = np.random.default_rng(22)
    q, k, v = (wlmod.round_bf16(rng.standard_normal((B, N, C)).astype(np.float32)) for _ in range(3))
    mask = (rng.uniform(size=(B, N)) < 0.6).astype(np.uint8)
    dO = wlmod.round_bf16(rng.standard_normal((int(mask.sum()), C)).astype(np.float32))
    a = _attention_fwd_bwd(spa, q, k, v, mask, dO, H, "bf16")
    b = _attention_fwd_bwd(spa, q, k, v, mask, dO, H, "bf16")
    T = int(mask.sum())
    for x, y in zip(a, b):
        assert np.array_equal(x[:T], y[:T])


@pytest.mark.parametrize("dtype,C", [("f32", 64), ("bf16", 96), ("bf16", 384), ("bf16", 768), ("f32", 1040)])
@pytest.mark.parametrize("with_up,scaled", [(False, False), (True, True)])
def test_gate_backward_matches_oracle(spa, dtype, C, with_up, scaled):
    B, N = 3, 201
    rng = np.random.default_rng(23)
    mk = wlmod.round_bf16 if dtype == "bf16" else (lambda a: a)
    x = mk(rng.standard_normal((B, N, C)).astype(np.float32))
    w = mk((rng.standard_normal(C) / np.sqrt(C)).astype(np.float32))
    bias = 0.125
    labels = (rng.uniform(size=(B, N)) < 0.4).astype(np.uint8)
    s_up = (rng.standard_normal((B, N)) * 1.5).astype(np.float32) if with_up else None
    d_rg = mk((rng.standard_normal((B, N, C)) * (rng.uniform(size=(B, N, 1)) < 0.5)).astype(np.float32))
    lam = 0.01 / (B * N)
    td = tdtype(dtype)
    xd, wd = dev(x, dtype), dev(w, dtype)
    scores = torch.empty(B, N, dtype=torch.float32, device="cuda")
    mask = torch.empty(B, N, dtype=torch.uint8, device="cuda")
    sup_d = None if s_up is None else dev(s_up)
    spa.spa_gate_select(xd, wd, bias, sup_d, 0.5, scores, mask)
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    dx = torch.empty(B, N, C, dtype=td, device="cuda")
    dw = torch.empty(C, dtype=torch.float32, device="cuda")
    db = torch.empty(1, dtype=torch.float32, device="cuda")
    ws = torch.empty(spa.spa_gate_bwd_workspace_bytes(B, N, C, spa.dtype_code(xd)), dtype=torch.uint8, device="cuda")
    spa.spa_gate_bwd(xd, wd, bias, scores, sup_d, dev(labels), dev(d_rg, dtype) if scaled else None, scaled, lam,
                     loss, dx, dw, db, ws)
    torch.cuda.synchronize()
    ref = orc.gate_backward(x, w, bias, s_up, labels, d_rg if scaled else None, scaled, lam)
    if with_up:
        g = orc.gate_only(x, w, bias)
        assert np.min(np.abs(g - s_up)) > 1e-4            # which side won the max is unambiguous
    assert abs(float(host(loss)[0]) - ref["loss"]) <= 1e-3 * abs(ref["loss"])
    tol = 1e-5 if dtype == "f32" else 2e-2
    assert _rel(host(dx), ref["dx"]) <= tol
    assert _rel(host(dw), ref["dw"]) <= 1e-3
    assert abs(float(host(db)[0]) - ref["db"]) <= 1e-3 * max(1.0, abs(ref["db"]))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_pack_and_unpack_transposes(spa, dtype):
    B, N, C = 5, 77, 48
    rng = np.random.default_rng(24)
    mk = wlmod.round_bf16 if dtype == "bf16" else (lambda a: a)
    mask = (rng.uniform(size=(B, N)) < 0.45).astype(np.uint8)
    mask[2] = 0
    cu, gidx, inv, T = orc.pack_indices(mask)
    td = tdtype(dtype)
    cap = B * N
    # unpack_bwd: dout[j] = dy[gather_idx[j]]
    dy = mk(rng.standard_normal((B, N, C)).astype(np.float32))
    gidx_d = torch.zeros(cap, dtype=torch.int32, device="cuda")
    gidx_d[:T] = dev(gidx)
    dout = torch.full((cap, C), float("nan"), dtype=td, device="cuda")
    spa.spa_unpack_bwd(dev(dy, dtype), gidx_d, dev(np.array([T], np.int32)), dout)
    # pack_bwd: d_rg[i] = dpacked[inv_pos[i]] or 0
    dpacked = mk(rng.standard_normal((cap, C)).astype(np.float32))
    d_rg = torch.full((B, N, C), float("nan"), dtype=td, device="cuda")
    spa.spa_pack_bwd(dev(dpacked, dtype), dev(inv), d_rg)
    torch.cuda.synchronize()
    got = host(dout)
    assert np.array_equal(got[:T], dy.reshape(-1, C)[gidx]) and np.all(np.isnan(got[T:]))
    ref = orc.unpack(dpacked[:T], inv, B, N)
    assert np.array_equal(host(d_rg).astype(np.float64), ref)


def test_training_chain_matches_oracle(spa):
    """Forward + backward of the ViT-B-shaped training step on a reduced batch: q, k are
    seeded stand-ins for projected tokens, v is the packed gated representation
    r_g = Sigmoid(s) . r, so the gate receives a real gradient through the attention."""
    wl = dataclasses.replace(wlmod.WORKLOADS["vit_b_train"], B=3)
    B, N, C, H, Dh = wl.B, wl.N, wl.C, wl.H, wl.Dh
    bun = wlmod.generate(wl, 7)
    lam = 0.01 / (B * N)
    x, w, bias = bun["x"], bun["w"], bun["bias"]
    qk = bun["qkv"][:, :, :2 * C]
    # ---- oracle
    s = orc.gate_scores(x, w, bias)
    mask, margin = orc.select(s, wl.tau)
    assert margin > 1e-3
    cu, gidx, inv, T = orc.pack_indices(mask)
    s32 = s.astype(np.float32).astype(np.float64)
    rg = orc.round_to_dtype(orc.sigmoid(s32)[:, :, None] * x, "bf16")
    out_ref, _ = orc.attention_per_image(qk[:, :, :C], qk[:, :, C:], rg, mask, H)
    y_ref = orc.unpack(out_ref, inv, B, N)
    dO = bun["dy"].reshape(-1, C)[gidx]
    rdq, rdk, rdv = orc.attention_backward_per_image(qk[:, :, :C], qk[:, :, C:], rg, mask, dO, H)
    d_rg_ref = orc.unpack(rdv, inv, B, N)
    gref = orc.gate_backward(x, w, bias, None, bun["labels"], d_rg_ref, True, lam)
    # ---- device
    td, cap = torch.bfloat16, B * N
    xd, wd = dev(x, "bf16"), dev(w, "bf16")
    scores = torch.empty(B, N, dtype=torch.float32, device="cuda")
    mask_d = torch.empty(B, N, dtype=torch.uint8, device="cuda")
    spa.spa_gate_select(xd, wd, bias, None, wl.tau, scores, mask_d)
    pqk = torch.zeros(cap, 2 * C, dtype=td, device="cuda")
    pv = torch.zeros(cap, C, dtype=td, device="cuda")
    cu_d = torch.empty(B + 1, dtype=torch.int32, device="cuda")
    gidx_d = torch.empty(cap, dtype=torch.int32, device="cuda")
    inv_d = torch.empty(cap, dtype=torch.int32, device="cuda")
    total = torch.empty(1, dtype=torch.int32, device="cuda")
    spa.spa_pack(dev(qk, "bf16"), mask_d, None, None, 0, pqk, cu_d, gidx_d, inv_d, total)
    spa.spa_pack(xd, mask_d, None, scores, 0, pv, None, None, None, None)
    out = torch.zeros(cap, C, dtype=td, device="cuda")
    lse = torch.zeros(H, cap, dtype=torch.float32, device="cuda")
    spa.spa_packed_attention(pqk[:, :C], pqk[:, C:], pv, cu_d, B, N, H, Dh, out, lse)
    y = torch.empty(B, N, C, dtype=td, device="cuda")
    spa.spa_unpack(out, inv_d, None, y)
    dout = torch.zeros(cap, C, dtype=td, device="cuda")
    spa.spa_unpack_bwd(dev(bun["dy"], "bf16"), gidx_d, total, dout)
    dqk = torch.zeros(cap, 2 * C, dtype=td, device="cuda")
    dv = torch.zeros(cap, C, dtype=td, device="cuda")
    ws = torch.empty(spa.spa_attention_bwd_workspace_bytes(B, N, H, Dh, spa.SPA_BF16), dtype=torch.uint8, device="cuda")
    spa.spa_packed_attention_bwd(pqk[:, :C], pqk[:, C:], pv, out, dout, lse, cu_d, B, N, H, Dh,
                                 dqk[:, :C], dqk[:, C:], dv, ws)
    d_rg = torch.empty(B, N, C, dtype=td, device="cuda")
    spa.spa_pack_bwd(dv, inv_d, d_rg)
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    dx = torch.empty(B, N, C, dtype=td, device="cuda")
    dw = torch.empty(C, dtype=torch.float32, device="cuda")
    db = torch.empty(1, dtype=torch.float32, device="cuda")
    ws2 = torch.empty(spa.spa_gate_bwd_workspace_bytes(B, N, C, spa.SPA_BF16), dtype=torch.uint8, device="cuda")
    spa.spa_gate_bwd(xd, wd, bias, scores, None, dev(bun["labels"]), d_rg, True, lam, loss, dx, dw, db, ws2)
    torch.cuda.synchronize()
    # ---- compare
    assert np.array_equal(host(mask_d), mask) and np.array_equal(host(cu_d), cu)
    assert np.array_equal(host(gidx_d)[:T], gidx) and np.array_equal(host(inv_d), inv)
    assert np.max(np.abs(host(y) - y_ref)) <= 2e-2
    assert _rel(host(dqk)[:T, :C], rdq) <= 2e-2 and _rel(host(dqk)[:T, C:], rdk) <= 2e-2
    assert _rel(host(dv)[:T], rdv) <= 2e-2
    assert _rel(host(dx), gref["dx"]) <= 2e-2
    assert _rel(host(dw), gref["dw"]) <= 2e-2            # dw sums bf16-rounded attention gradients
    assert abs(float(host(db)[0]) - gref["db"]) <= 2e-2 * max(1.0, abs(gref["db"]))
    assert abs(float(host(loss)[0]) - gref["loss"]) <= 1e-3 * abs(gref["loss"])
