"""Projection of packed tokens (gather and gate scaling folded into the operand load) against
the CPU oracle, and a whole SPA block: gate -> select -> indices -> QKV projection of the
selected, gated tokens -> per-image attention -> scatter back."""
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
    return float(np.max(np.abs(got - ref)) / max(1.0, np.max(np.abs(ref)))) if ref.size else 0.0


@pytest.mark.parametrize("dtype,B,N,K,No", [("bf16", 3, 100, 64, 96), ("bf16", 8, 196, 384, 1152),
                                            ("bf16", 2, 777, 96, 288), ("bf16", 4, 129, 32, 8), ("bf16", 2, 150, 200, 64), ("bf16", 40, 196, 96, 1280),
                                            ("f32", 2, 60, 64, 192)])
@pytest.mark.parametrize("mode", ["plain", "gather", "gather_scale_bias"])
def test_linear_packed_matches_oracle(spa, dtype, B, N, K, No, mode):
    rng = np.random.default_rng(41)
    mk = wlmod.round_bf16 if dtype == "bf16" else (lambda a: a)
    x = mk(rng.standard_normal((B, N, K)).astype(np.float32))
    W = mk((rng.standard_normal((No, K)) / np.sqrt(K)).astype(np.float32))
    bias = mk(rng.standard_normal(No).astype(np.float32)) if mode == "gather_scale_bias" else None
    s = rng.standard_normal((B, N)).astype(np.float32) if mode == "gather_scale_bias" else None
    mask = (rng.uniform(size=(B, N)) < 0.55).astype(np.uint8)
    cu, gidx, inv, T = orc.pack_indices(mask)
    cap = B * N
    td = tdtype(dtype)
    if mode == "plain":
        rows = np.arange(cap, dtype=np.int32)
        T_used, gi_d, tot_d = cap, None, None
    else:
        rows = gidx
        T_used = T
        gi = np.zeros(cap, np.int32)
        gi[:T] = gidx
        gi_d, tot_d = dev(gi), dev(np.array([T], np.int32))
    ref = orc.linear_packed(x, rows, W, bias, s, dtype)
    out = torch.full((cap, No + 16), float("nan"), dtype=td, device="cuda")     # a column-slice view: row stride > N_out
    spa.spa_linear_packed(dev(x, dtype), gi_d, None if s is None else dev(s), tot_d, dev(W, dtype),
                          None if bias is None else dev(bias, dtype), out[:, :No])
    torch.cuda.synchronize()
    got = host(out)
    assert np.all(np.isnan(got[:, No:])) and np.all(np.isnan(got[T_used:]))       # nothing outside the result
    tol = 1e-5 if dtype == "f32" else 1e-2
    assert _rel(got[:T_used, :No], ref) <= tol


def test_spa_block_with_projection(spa):
    """gate_select -> pack (indices only) -> spa_linear_packed(x gathered and gate-scaled, W_qkv)
    -> spa_packed_attention_unpack, against the oracle's composition of the same steps."""
    wl = dataclasses.replace(wlmod.WORKLOADS["vit_s"], B=6)
    B, N, C, H, Dh = wl.B, wl.N, wl.C, wl.H, wl.Dh
    bun = wlmod.generate(wl, 9, with_qkv=False)
    rng = np.random.default_rng(9)
    Wqkv = wlmod.round_bf16((rng.standard_normal((3 * C, C)) / np.sqrt(C)).astype(np.float32))
    bqkv = wlmod.round_bf16((rng.standard_normal(3 * C) * 0.1).astype(np.float32))
    x, w, bias = bun["x"], bun["w"], bun["bias"]
    # oracle
    s = orc.gate_scores(x, w, bias)
    mask, margin = orc.select(s, wl.tau)
    assert margin > 1e-3
    cu, gidx, inv, T = orc.pack_indices(mask)
    qkv_packed = orc.round_to_dtype(orc.linear_packed(x, gidx, Wqkv, bqkv, s.astype(np.float32), "bf16"), "bf16")
    # the oracle's attention takes un-packed tensors: scatter the packed projections back to [B,N,3C]
    qkv_full = orc.unpack(qkv_packed, inv, B, N)
    out_ref, _ = orc.attention_per_image(qkv_full[..., :C], qkv_full[..., C:2 * C], qkv_full[..., 2 * C:], mask, H)
    y_ref = orc.unpack(out_ref, inv, B, N)
    # device
    td, cap = torch.bfloat16, B * N
    xd, wd = dev(x, "bf16"), dev(w, "bf16")
    scores = torch.empty(B, N, dtype=torch.float32, device="cuda")
    mask_d = torch.empty(B, N, dtype=torch.uint8, device="cuda")
    cu_d = torch.empty(B + 1, dtype=torch.int32, device="cuda")
    gidx_d = torch.zeros(cap, dtype=torch.int32, device="cuda")
    inv_d = torch.empty(cap, dtype=torch.int32, device="cuda")
    total = torch.empty(1, dtype=torch.int32, device="cuda")
    pqkv = torch.zeros(cap, 3 * C, dtype=td, device="cuda")
    y = torch.empty(B, N, C, dtype=td, device="cuda")
    spa.spa_gate_select(xd, wd, bias, None, wl.tau, scores, mask_d)
    spa.spa_pack(None, mask_d, None, None, 0, None, cu_d, gidx_d, inv_d, total)
    spa.spa_linear_packed(xd, gidx_d, scores, total, dev(Wqkv, "bf16"), dev(bqkv, "bf16"), pqkv)
    spa.spa_packed_attention_unpack(pqkv[:, :C], pqkv[:, C:2 * C], pqkv[:, 2 * C:], cu_d, gidx_d, inv_d, None, H, Dh, y)
    torch.cuda.synchronize()
    assert np.array_equal(host(mask_d), mask) and np.array_equal(host(cu_d), cu)
    assert np.array_equal(host(gidx_d)[:T], gidx) and np.array_equal(host(inv_d), inv)
    assert _rel(host(pqkv)[:T], qkv_packed) <= 1e-2
    # the device attention runs on its own (slightly different) bf16 projections
    assert np.max(np.abs(host(y) - y_ref)) <= 4e-2


def test_block_pass_with_both_projections(spa):
    """BlockPass (six launches: gate, indices, QKV projection, attention, output projection,
    scatter with x as the bypass) against the oracle's composition of the same steps."""
    from paper_2410_23608_amd.pipeline import BlockPass
    wl = dataclasses.replace(wlmod.WORKLOADS["vit_s"], B=5)
    B, N, C, H = wl.B, wl.N, wl.C, wl.H
    bun = wlmod.generate(wl, 21, with_qkv=False)
    rng = np.random.default_rng(21)
    mkw = lambda *shape: wlmod.round_bf16((rng.standard_normal(shape) / np.sqrt(C)).astype(np.float32))
    Wqkv, bqkv, Wo, bo = mkw(3 * C, C), mkw(3 * C), mkw(C, C), mkw(C)
    x, w, bias = bun["x"], bun["w"], bun["bias"]
    s = orc.gate_scores(x, w, bias)
    mask, margin = orc.select(s, wl.tau)
    assert margin > 1e-3
    cu, gidx, inv, T = orc.pack_indices(mask)
    qkv_packed = orc.round_to_dtype(orc.linear_packed(x, gidx, Wqkv, bqkv, s.astype(np.float32), "bf16"), "bf16")
    qkv_full = orc.unpack(qkv_packed, inv, B, N)
    attn_ref, _ = orc.attention_per_image(qkv_full[..., :C], qkv_full[..., C:2 * C], qkv_full[..., 2 * C:], mask, H)
    attn_ref = orc.round_to_dtype(attn_ref, "bf16")                       # packed rows, [T, C]
    proj_ref = orc.linear_packed(attn_ref, np.arange(T), Wo, bo, None, "bf16")
    y_ref = orc.unpack(proj_ref, inv, B, N, base=x)
    bp = BlockPass(B, N, C, H, "bf16", wl.tau, bias)
    y = bp.run(dev(x, "bf16"), dev(w, "bf16"), dev(Wqkv, "bf16"), dev(bqkv, "bf16"), dev(Wo, "bf16"), dev(bo, "bf16"))
    torch.cuda.synchronize()
    assert np.array_equal(host(bp.mask), mask) and int(bp.total.item()) == T
    got = host(y)
    assert np.array_equal(got[mask == 0], x[mask == 0])                   # bypassing tokens are x, bit for bit
    assert np.max(np.abs(got - y_ref)) <= 5e-2


def test_linear_packed_empty_and_capped_totals(spa):
    """*total = 0 writes nothing; *total above the capacity is clamped to it."""
    rng = np.random.default_rng(5)
    cap, K, No = 300, 64, 128
    x = wlmod.round_bf16(rng.standard_normal((cap, K)).astype(np.float32))
    W = wlmod.round_bf16((rng.standard_normal((No, K)) / 8).astype(np.float32))
    gi = torch.arange(cap, dtype=torch.int32, device="cuda")
    for tot, rows in ((0, 0), (10 ** 6, cap), (1, 1), (129, 129)):
        out = torch.full((cap, No), float("nan"), dtype=torch.bfloat16, device="cuda")
        spa.spa_linear_packed(dev(x, "bf16"), gi, None, dev(np.array([tot], np.int32)), dev(W, "bf16"), None, out)
        torch.cuda.synchronize()
        got = host(out)
        assert np.all(np.isnan(got[rows:])) and not np.any(np.isnan(got[:rows]))
        if rows:
            ref = orc.linear_packed(x, np.arange(rows), W)
            assert _rel(got[:rows], ref) <= 1e-2


def test_linear_packed_rejects_bad_arguments(spa):
    x = torch.zeros(16, 64, dtype=torch.bfloat16, device="cuda")
    W = torch.zeros(32, 64, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(16, 32, dtype=torch.bfloat16, device="cuda")
    sc = torch.zeros(16, device="cuda")
    with pytest.raises(spa.SpaError):
        spa.spa_linear_packed(x, None, sc, None, W, None, out)                      # scores without gather_idx
    with pytest.raises(spa.SpaError):
        spa.spa_linear_packed(x[:, :60].contiguous(), None, None, None, W[:, :60].contiguous(), None, out)   # K % 8 != 0


@pytest.mark.parametrize("dtype,K,No", [("bf16", 384, 384), ("bf16", 96, 200), ("f32", 64, 48)])
@pytest.mark.parametrize("with_residual", [False, True])
def test_linear_packed_scatter_matches_oracle(spa, dtype, K, No, with_residual):
    """y[scatter_idx[j]] = residual[...] + x[j] W^T + bias against the oracle's projection followed
    by its scatter back; rows that no j names stay as they were."""
    rng = np.random.default_rng(K + No)
    B, N = 3, 150
    mk = wlmod.round_bf16 if dtype == "bf16" else (lambda a: a)
    mask = (rng.random((B, N)) < 0.5).astype(np.uint8)
    cu, gidx, inv, T = orc.pack_indices(mask)
    cap = B * N
    xp = mk(rng.standard_normal((cap, K)).astype(np.float32))                 # packed rows (first T used)
    W = mk((rng.standard_normal((No, K)) / np.sqrt(K)).astype(np.float32))
    b = mk((rng.standard_normal(No) * 0.1).astype(np.float32))
    res = mk(rng.standard_normal((B, N, No)).astype(np.float32))
    proj = orc.linear_packed(xp, np.arange(T), W, b)
    if dtype == "bf16":
        proj = orc.round_to_dtype(proj, "bf16")                               # the kernel rounds before the add
    y_ref = orc.unpack(proj, inv, B, N, base=res if with_residual else None)
    td = tdtype(dtype)
    gi = torch.zeros(cap, dtype=torch.int32, device="cuda")
    gi[:T] = dev(gidx)
    tot = dev(np.array([T], np.int32))
    canary = 123.0
    y = torch.full((B, N, No), canary, dtype=td, device="cuda")
    spa.spa_linear_packed_scatter(dev(xp, dtype), tot, dev(W, dtype), dev(b, dtype), gi,
                                  dev(res, dtype) if with_residual else None, y)
    torch.cuda.synchronize()
    got = host(y)
    sel = mask.astype(bool)
    assert np.all(got[~sel] == canary)                                        # untouched rows
    tol = 1e-4 if dtype == "f32" else 2e-2
    assert np.max(np.abs(got[sel] - y_ref[sel])) <= tol * max(1.0, np.max(np.abs(y_ref)))
    if with_residual:                                                         # in place on the residual stream
        y2 = dev(res, dtype).clone()
        spa.spa_linear_packed_scatter(dev(xp, dtype), tot, dev(W, dtype), dev(b, dtype), gi, y2, y2)
        torch.cuda.synchronize()
        g2 = host(y2)
        assert np.array_equal(g2[sel], got[sel]) and np.array_equal(g2[~sel], res[~sel])


def test_block_pass_in_place_equals_six_launch_form(spa):
    """BlockPass(in_place=True) (output projection scatters into the residual stream) gives the
    same bits as the six-launch form with its separate scatter."""
    from paper_2410_23608_amd.pipeline import BlockPass
    wl = dataclasses.replace(wlmod.WORKLOADS["vit_s"], B=7)
    B, N, C, H = wl.B, wl.N, wl.C, wl.H
    bun = wlmod.generate(wl, 33, with_qkv=False)
    rng = np.random.default_rng(33)
    mkw = lambda *shape: wlmod.round_bf16((rng.standard_normal(shape) / np.sqrt(C)).astype(np.float32))
    Wqkv, bqkv, Wo, bo = (dev(a, "bf16") for a in (mkw(3 * C, C), mkw(3 * C), mkw(C, C), mkw(C)))
    x, w = dev(bun["x"], "bf16"), dev(bun["w"], "bf16")
    y6 = BlockPass(B, N, C, H, "bf16", wl.tau, bun["bias"]).run(x, w, Wqkv, bqkv, Wo, bo).clone()
    x5 = x.clone()
    y5 = BlockPass(B, N, C, H, "bf16", wl.tau, bun["bias"], in_place=True).run(x5, w, Wqkv, bqkv, Wo, bo)
    torch.cuda.synchronize()
    assert y5.data_ptr() == x5.data_ptr() and torch.equal(y5, y6)


# ----------------------------------------------------------------------------- backward
def _bwd_case(dtype, B, N, K, No, mode, seed=43, select=0.55):
    rng = np.random.default_rng(seed)
    mk = wlmod.round_bf16 if dtype == "bf16" else (lambda a: a)
    cap = B * N
    x_tok = mk(rng.standard_normal((B, N, K)).astype(np.float32))
    W = mk((rng.standard_normal((No, K)) / np.sqrt(K)).astype(np.float32))
    s = rng.standard_normal((B, N)).astype(np.float32)
    mask = (rng.uniform(size=(B, N)) < select).astype(np.uint8)
    cu, gidx, inv, T = orc.pack_indices(mask)
    g_rows = mk(rng.standard_normal((cap, No)).astype(np.float32))
    return dict(x_tok=x_tok, W=W, s=s, gidx=gidx, inv=inv, T=T, g_rows=g_rows, cap=cap)


@pytest.mark.parametrize("dtype,B,N,K,No", [("bf16", 3, 100, 64, 96), ("bf16", 8, 196, 384, 1152),
                                            ("bf16", 2, 777, 96, 288), ("bf16", 4, 129, 32, 8), ("bf16", 2, 150, 200, 72),
                                            ("bf16", 40, 196, 96, 1280), ("bf16", 2, 300, 136, 264),
                                            ("bf16", 64, 196, 64, 96),      # token chunks longer than one LDS table of rows
                                            ("f32", 2, 60, 64, 192)])
@pytest.mark.parametrize("mode", ["plain", "qkv", "out_proj"])
def test_linear_backward_matches_oracle(spa, dtype, B, N, K, No, mode):
    """plain: rows in order, no index arrays, no row count on the device.
    qkv: the backward of spa_linear_packed(x, gather_idx, scores): upstream rows packed (a
    column-slice view), x read at token positions and gate-scaled, d_rg written at token
    positions with the unselected rows cleared.
    out_proj: the backward of spa_linear_packed_scatter: upstream gradient gathered from token
    positions, x and dx packed."""
    c = _bwd_case(dtype, B, N, K, No, mode)
    cap, T, gidx, td = c["cap"], c["T"], c["gidx"], tdtype(dtype)
    gi = np.zeros(cap, np.int32)
    gi[:T] = gidx
    gi_d, tot_d, inv_d = dev(gi), dev(np.array([T], np.int32)), dev(c["inv"])
    x_flat = c["x_tok"].reshape(cap, K)
    W_d = dev(c["W"], dtype)
    dW = torch.full((No, K), float("nan"), dtype=torch.float32, device="cuda")
    db = torch.full((No,), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(spa.spa_linear_bwd_weight_workspace_bytes(cap, K, No, dtype), 256), dtype=torch.uint8, device="cuda")
    if mode == "plain":
        M = cap
        ref = orc.linear_packed_backward(c["g_rows"], x_flat, np.arange(cap), c["W"])
        g_d = dev(c["g_rows"], dtype)
        dx = torch.full((cap, K), float("nan"), dtype=td, device="cuda")
        spa.spa_linear_packed_bwd_input(g_d, None, None, W_d, cap, None, None, dx)
        spa.spa_linear_packed_bwd_weight(g_d, None, dev(x_flat, dtype), None, None, None, cap, dW, db, ws)
        dx_rows = host(dx)
    elif mode == "qkv":
        M = T
        ref = orc.linear_packed_backward(c["g_rows"], x_flat, gidx, c["W"], c["s"], None, dtype)
        wide = torch.full((cap, No + 24), float("nan"), dtype=td, device="cuda")
        wide[:, 8:8 + No] = dev(c["g_rows"], dtype)
        g_d = wide[:, 8:8 + No]                                   # row stride No + 24, offset 8 columns
        dx = torch.full((cap, K), float("nan"), dtype=td, device="cuda")
        spa.spa_linear_packed_bwd_input(g_d, None, tot_d, W_d, cap, gi_d, inv_d, dx)
        spa.spa_linear_packed_bwd_weight(g_d, None, dev(x_flat, dtype), gi_d, dev(c["s"]), tot_d, cap, dW, db, ws)
        got = host(dx)
        assert not np.any(np.isnan(got))                          # every row written: a result or zero
        assert np.all(got[c["inv"] < 0] == 0)
        dx_rows = got[gidx]
    else:
        M = T
        packed_x = np.zeros((cap, K), np.float32)
        packed_x[:T] = x_flat[gidx]                               # any packed rows will do as the forward input
        ref = orc.linear_packed_backward(c["g_rows"], packed_x, np.arange(T), c["W"], None, gidx)
        g_d = dev(c["g_rows"], dtype)
        dx = torch.full((cap, K), float("nan"), dtype=td, device="cuda")
        spa.spa_linear_packed_bwd_input(g_d, gi_d, tot_d, W_d, cap, None, None, dx)
        spa.spa_linear_packed_bwd_weight(g_d, gi_d, dev(packed_x, dtype), None, None, tot_d, cap, dW, db, ws)
        got = host(dx)
        assert np.all(np.isnan(got[T:]))                          # rows past the total untouched
        dx_rows = got[:T]
    torch.cuda.synchronize()
    tol_x, tol_w = (1e-5, 1e-5) if dtype == "f32" else (1e-2, 2e-3)
    assert _rel(dx_rows[:M], ref["d_rows"]) <= tol_x
    assert _rel(host(dW), ref["dW"]) <= tol_w
    assert _rel(host(db), ref["dbias"]) <= tol_w
    # the sums run in a fixed order
    dW2, db2 = torch.empty_like(dW), torch.empty_like(db)
    if mode == "plain":
        spa.spa_linear_packed_bwd_weight(g_d, None, dev(x_flat, dtype), None, None, None, cap, dW2, db2, ws)
    elif mode == "qkv":
        spa.spa_linear_packed_bwd_weight(g_d, None, dev(x_flat, dtype), gi_d, dev(c["s"]), tot_d, cap, dW2, db2, ws)
    else:
        spa.spa_linear_packed_bwd_weight(g_d, gi_d, dev(packed_x, dtype), None, None, tot_d, cap, dW2, db2, ws)
    assert torch.equal(dW, dW2) and torch.equal(db, db2)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("T", [0, 1, 63, 65])
def test_linear_backward_few_or_no_rows(spa, dtype, T):
    """No selected token: dW and dbias are zero and d_rg is all zeros; a handful of rows: one
    ragged contraction step on the weight side, one ragged tile on the input side."""
    B, N, K, No = 2, 96, 72, 40
    rng = np.random.default_rng(47)
    mk = wlmod.round_bf16 if dtype == "bf16" else (lambda a: a)
    cap, td = B * N, tdtype(dtype)
    x = mk(rng.standard_normal((cap, K)).astype(np.float32))
    W = mk((rng.standard_normal((No, K)) / np.sqrt(K)).astype(np.float32))
    g = mk(rng.standard_normal((cap, No)).astype(np.float32))
    mask = np.zeros(cap, np.uint8)
    mask[rng.permutation(cap)[:T]] = 1
    cu, gidx, inv, T_ = orc.pack_indices(mask.reshape(B, N))
    assert T_ == T
    gi = np.zeros(cap, np.int32)
    gi[:T] = gidx
    ref = orc.linear_packed_backward(g, x, gidx, W)
    dx = torch.full((cap, K), float("nan"), dtype=td, device="cuda")
    dW = torch.full((No, K), float("nan"), dtype=torch.float32, device="cuda")
    db = torch.full((No,), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(spa.spa_linear_bwd_weight_workspace_bytes(cap, K, No, dtype), 256), dtype=torch.uint8, device="cuda")
    tot = dev(np.array([T], np.int32))
    spa.spa_linear_packed_bwd_input(dev(g, dtype), None, tot, dev(W, dtype), cap, dev(gi), dev(inv), dx)
    spa.spa_linear_packed_bwd_weight(dev(g, dtype), None, dev(x, dtype), dev(gi), None, tot, cap, dW, db, ws)
    torch.cuda.synchronize()
    got = host(dx)
    assert np.all(got[inv < 0] == 0) and not np.any(np.isnan(got))
    tol_x, tol_w = (1e-5, 1e-5) if dtype == "f32" else (1e-2, 2e-3)
    if T == 0:
        assert np.all(host(dW) == 0) and np.all(host(db) == 0)
    else:
        assert _rel(got[gidx], ref["d_rows"]) <= tol_x
        assert _rel(host(dW), ref["dW"]) <= tol_w and _rel(host(db), ref["dbias"]) <= tol_w


def test_linear_backward_rejects_bad_arguments(spa):
    x = torch.zeros(64, 64, dtype=torch.bfloat16, device="cuda")
    W = torch.zeros(32, 64, dtype=torch.bfloat16, device="cuda")
    g = torch.zeros(64, 32, dtype=torch.bfloat16, device="cuda")
    dW = torch.zeros(32, 64, dtype=torch.float32, device="cuda")
    inv = torch.zeros(64, dtype=torch.int32, device="cuda")
    sc = torch.zeros(64, dtype=torch.float32, device="cuda")
    with pytest.raises(spa.SpaError, match="dx_idx"):
        spa.spa_linear_packed_bwd_input(g, None, None, W, 64, None, inv, x)              # zero fill without dx_idx
    with pytest.raises(spa.SpaError, match="workspace"):
        spa.spa_linear_packed_bwd_weight(g, None, x, None, None, None, 64, dW, None, None)
    with pytest.raises(spa.SpaError, match="x_idx"):
        spa.spa_linear_packed_bwd_weight(g, None, x, None, sc, None, 64, dW, None, torch.empty(1 << 20, dtype=torch.uint8, device="cuda"))


@pytest.mark.parametrize("overlap,dtype", [(True, "bf16"), (False, "bf16"), (True, "f32"), (False, "f32")])
def test_block_train_pass_with_both_projections(spa, overlap, dtype):
    """BlockTrainPass (forward + backward of the block with its projections and the selection
    loss) against the oracle, in bf16 (ViT-S shape, reduced batch) and in fp32 (the tiny
    workload's shape).  Every backward stage is checked against the oracle applied to the
    device's own inputs of that stage (so each link of the chain is held to a tight bound), and
    the end of the chain against the oracle's own chain.  overlap: the weight-side GEMMs on a
    second stream (as benchmarked) or everything on one stream."""
    from paper_2410_23608_amd.pipeline import BlockTrainPass
    bf = dtype == "bf16"
    wl = dataclasses.replace(wlmod.WORKLOADS["vit_s"], B=6) if bf else dataclasses.replace(wlmod.WORKLOADS["tiny"], B=3)
    B, N, C, H = wl.B, wl.N, wl.C, wl.H
    cap = B * N
    bun = wlmod.generate(wl, 23, with_qkv=False)
    rng = np.random.default_rng(23)
    rnd = wlmod.round_bf16 if bf else (lambda a: a)
    mkw = lambda *shape: rnd((rng.standard_normal(shape) / np.sqrt(C)).astype(np.float32))
    Wqkv, bqkv, Wo, bo = mkw(3 * C, C), mkw(3 * C), mkw(C, C), mkw(C)
    x, w, bias, labels = bun["x"], bun["w"], bun["bias"], bun["labels"]
    dy = rnd(rng.standard_normal((B, N, C)).astype(np.float32))
    # bounds per stage: bf16 (one or two bf16 roundings of O(1) values per link) | fp32 (accumulation order only)
    t_proj, t_attn, t_y, t_gin, t_gw, t_gattn, t_gate = ((1e-2, 2e-2, 4e-2, 1e-2, 2e-3, 2e-2, 1e-2) if bf else
                                                         (2e-5, 1e-5, 2e-5, 2e-5, 2e-5, 2e-5, 2e-5))
    tp = BlockTrainPass(B, N, C, H, dtype, wl.tau, bias, overlap_weight_grads=overlap)
    tp.d_rg.fill_(float("nan"))
    tp.run(dev(x, dtype), dev(w, dtype), dev(Wqkv, dtype), dev(bqkv, dtype), dev(Wo, dtype), dev(bo, dtype),
           dev(labels), dev(dy, dtype))
    torch.cuda.synchronize()
    # forward
    s = orc.gate_scores(x, w, bias)
    mask, margin = orc.select(s, wl.tau)
    assert margin > 1e-3
    cu, gidx, inv, T = orc.pack_indices(mask)
    assert np.array_equal(host(tp.mask), mask) and int(tp.total.item()) == T
    s32 = host(tp.scores)
    qkv_ref = orc.linear_packed(x, gidx, Wqkv, bqkv, s32, dtype)
    assert _rel(host(tp.packed_qkv)[:T], qkv_ref) <= t_proj
    qkv_dev = host(tp.packed_qkv)[:T].astype(np.float64)
    full = orc.unpack(qkv_dev, inv, B, N)
    qf, kf, vf = full[..., :C], full[..., C:2 * C], full[..., 2 * C:]
    attn_ref, _ = orc.attention_per_image(qf, kf, vf, mask, H)
    attn_dev = host(tp.attn)[:T].astype(np.float64)
    assert np.max(np.abs(attn_dev - attn_ref)) <= t_attn
    y_ref = orc.unpack(orc.linear_packed(attn_dev, np.arange(T), Wo, bo), inv, B, N, base=x)
    assert np.max(np.abs(host(tp.y) - y_ref)) <= t_y
    assert np.array_equal(host(tp.y)[mask == 0], x[mask == 0])
    # backward, stage by stage on the device's own intermediates
    bo_ = orc.linear_packed_backward(dy.reshape(cap, C), attn_dev, np.arange(T), Wo, None, gidx)
    d_attn_dev = host(tp.d_attn)[:T].astype(np.float64)
    assert _rel(d_attn_dev, bo_["d_rows"]) <= t_gin
    assert _rel(host(tp.dW_o), bo_["dW"]) <= t_gw and _rel(host(tp.db_o), bo_["dbias"]) <= t_gw
    rdq, rdk, rdv = orc.attention_backward_per_image(qf, kf, vf, mask, d_attn_dev, H)
    dqkv_dev = host(tp.d_qkv)[:T].astype(np.float64)
    assert _rel(dqkv_dev, np.concatenate([rdq, rdk, rdv], axis=1)) <= t_gattn
    bq = orc.linear_packed_backward(dqkv_dev, x, gidx, Wqkv, s32, None, dtype)
    d_rg_dev = host(tp.d_rg).reshape(cap, C)
    assert _rel(d_rg_dev[gidx], bq["d_rows"]) <= t_gin
    assert np.all(d_rg_dev[inv < 0] == 0)
    assert _rel(host(tp.dW_qkv), bq["dW"]) <= t_gw and _rel(host(tp.db_qkv), bq["dbias"]) <= t_gw
    g = orc.gate_backward(x, w, bias, None, labels, d_rg_dev.reshape(B, N, C).astype(np.float64), True, tp.loss_scale)
    assert _rel(host(tp.dx), g["dx"]) <= t_gate
    assert _rel(host(tp.dw), g["dw"]) <= t_gate
    assert abs(float(host(tp.loss)[0]) - g["loss"]) <= 1e-3 * abs(g["loss"])
    # the whole chain in the oracle, from its own forward intermediates
    qkv_o = orc.round_to_dtype(qkv_ref, dtype)
    full_o = orc.unpack(qkv_o, inv, B, N)
    attn_o, _ = orc.attention_per_image(full_o[..., :C], full_o[..., C:2 * C], full_o[..., 2 * C:], mask, H)
    attn_o = orc.round_to_dtype(attn_o, dtype)
    co = orc.linear_packed_backward(dy.reshape(cap, C), attn_o, np.arange(T), Wo, None, gidx)
    cdq, cdk, cdv = orc.attention_backward_per_image(full_o[..., :C], full_o[..., C:2 * C], full_o[..., 2 * C:], mask,
                                                      orc.round_to_dtype(co["d_rows"], dtype), H)
    cq = orc.linear_packed_backward(orc.round_to_dtype(np.concatenate([cdq, cdk, cdv], axis=1), dtype), x, gidx, Wqkv,
                                    s32, None, dtype)
    cg = orc.gate_backward(x, w, bias, None, labels, orc.unpack(orc.round_to_dtype(cq["d_rows"], dtype), inv, B, N),
                           True, tp.loss_scale)
    t_cw, t_cq, t_cx = (1e-2, 2e-2, 3e-2) if bf else (1e-4, 1e-4, 1e-4)
    assert _rel(host(tp.dW_o), co["dW"]) <= t_cw and _rel(host(tp.dW_qkv), cq["dW"]) <= t_cq
    assert _rel(host(tp.dx), cg["dx"]) <= t_cx and _rel(host(tp.dw), cg["dw"]) <= t_cx
