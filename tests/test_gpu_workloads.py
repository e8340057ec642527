"""Full-size parity of the HIP path in the launch configuration bench.py times (through
paper_2410_23608_amd.pipeline), the multi-stage hierarchy with up-scale scores, property
tests over random shapes, and run-to-run determinism."""
import dataclasses
import itertools

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


@pytest.fixture(scope="module")
def pipeline():
    from paper_2410_23608_amd import pipeline as mod
    return mod


def _hier_cfg(bundles):
    return [(b["workload"].B, *b["workload"].grid, b["workload"].C, b["workload"].H, b["workload"].dtype,
             b["workload"].tau, b["bias"]) for b in bundles]


def _rel(got, ref):
    return float(np.max(np.abs(got - ref)) / max(1.0, np.max(np.abs(ref))))


def _gate_backward_candidates(x, w, bias, s_up, labels, d_rg, loss_scale):
    """The oracle's gate backward for every admissible reading of near-ties between the gate's own
    score and the up-scale score.  Which of the two wins the max decides whether the token's score
    gradient reaches (w, b); the kernel takes that decision on its fp32 sum, the oracle on its fp64
    sum, so for a token whose two scores lie within 1e-4 of each other (far above the fp32
    reassociation error, far below anything that matters to the values) both outcomes are valid.
    Yields the oracle result with each such token forced to either side."""
    if s_up is None:
        yield orc.gate_backward(x, w, bias, None, labels, d_rg, True, loss_scale)
        return
    g = orc.gate_only(x, w, bias)
    near = np.argwhere(np.abs(g - s_up) < 1e-4)
    assert len(near) <= 4, "too many near-ties for an exhaustive check"
    for signs in itertools.product((-1.0, 1.0), repeat=len(near)):
        su = s_up.astype(np.float64).copy()
        for (b, n), sg in zip(near, signs):
            su[b, n] = g[b, n] + sg * 2e-4
        yield orc.gate_backward(x, w, bias, su, labels, d_rg, True, loss_scale)


def _sampled_attention_reference(q, k, v, mask, H, rows):
    """Oracle attention for a sample of packed rows only, one row at a time: row j of image b
    attends to all selected tokens of b.  Plain definition, fp64."""
    B, N, C = q.shape
    Dh = C // H
    cu, gidx, inv, T = orc.pack_indices(mask)
    out = np.zeros((len(rows), C))
    for t, j in enumerate(rows):
        b = int(np.searchsorted(cu, j, side="right") - 1)
        sel = np.flatnonzero(mask[b])
        n = gidx[j] - b * N
        for h in range(H):
            sl = slice(h * Dh, (h + 1) * Dh)
            s = k[b, sel, sl].astype(np.float64) @ q[b, n, sl].astype(np.float64) / np.sqrt(Dh)
            p = np.exp(s - s.max())
            out[t, sl] = (p / p.sum()) @ v[b, sel, sl].astype(np.float64)
    return out


@pytest.mark.parametrize("name", ["vit_s", "det"])
def test_full_size_forward_as_benchmarked(spa, pipeline, name):
    """The exact batch and launch path of bench.py: integers bit-exact, packed rows bit-exact,
    attention checked on EVERY packed row of the full batch (vit_s: 64 images, det: 8 images of
    4200 tokens), and on det also row by row on a sample computed one query at a time."""
    wl = wlmod.WORKLOADS[name]
    bun = wlmod.generate(wl, 0)
    C = wl.C
    fp = pipeline.ForwardPass(wl.B, wl.N, C, wl.H, wl.dtype, wl.tau, wl.bias)
    fp.run(dev(bun["x"], wl.dtype), dev(bun["w"], wl.dtype), dev(bun["qkv"], wl.dtype))
    torch.cuda.synchronize()
    s = orc.gate_scores(bun["x"], bun["w"], bun["bias"])
    mask, margin = orc.select(s, wl.tau)
    assert margin > 1e-3
    cu, gidx, inv, T = orc.pack_indices(mask)
    assert np.array_equal(host(fp.mask), mask)
    assert np.array_equal(host(fp.cu_seqlens), cu) and int(host(fp.total)[0]) == T
    assert np.array_equal(host(fp.gather_idx)[:T], gidx) and np.array_equal(host(fp.inv_pos), inv)
    assert np.array_equal(host(fp.packed_qkv)[:T], bun["qkv"].reshape(-1, 3 * C)[gidx])
    q, k, v = bun["qkv"][..., :C], bun["qkv"][..., C:2 * C], bun["qkv"][..., 2 * C:]
    out = host(fp.out)
    ref, lse_ref = orc.attention_per_image(q, k, v, mask, wl.H)
    assert np.max(np.abs(out[:T] - ref)) <= 2e-2
    assert np.max(np.abs(host(fp.lse)[:, :T] - lse_ref)) <= 2e-2
    if name == "det":
        rng = np.random.default_rng(0)
        rows = np.unique(np.concatenate([rng.integers(0, T, 48), cu[:-1][np.diff(cu) > 0], cu[1:][np.diff(cu) > 0] - 1]))
        ref = _sampled_attention_reference(q, k, v, mask, wl.H, rows)
        assert np.max(np.abs(out[rows] - ref)) <= 2e-2
    # scatter back: exact copies at selected positions, zeros elsewhere (a property at any size)
    y = host(fp.y).reshape(-1, C)
    assert np.array_equal(y[gidx], out[:T]) and np.all(y[inv < 0] == 0)


@pytest.mark.parametrize("fused_bwd,pack_pair", [(True, True), (True, False), (False, False)])
def test_full_size_training_step_as_benchmarked(spa, pipeline, fused_bwd, pack_pair):
    """ViT-B-shaped forward+backward step at full batch through pipeline.TrainPass, with the
    gather / scatter of the gradients inside the attention backward (as benchmarked) and as
    separate launches."""
    wl = wlmod.WORKLOADS["vit_b_train"]
    B, N, C, H = wl.B, wl.N, wl.C, wl.H
    bun = wlmod.generate(wl, 0)
    tp = pipeline.TrainPass(B, N, C, H, wl.dtype, wl.tau, wl.bias, fused_bwd=fused_bwd, pack_pair=pack_pair)
    tp.dqk.fill_(float("nan"))
    tp.d_rg.fill_(float("nan"))
    qk = bun["qkv"][:, :, :2 * C]
    tp.run(dev(bun["x"], "bf16"), dev(bun["w"], "bf16"), dev(qk, "bf16"), dev(bun["labels"]), dev(bun["dy"], "bf16"))
    torch.cuda.synchronize()
    x, w, bias = bun["x"], bun["w"], bun["bias"]
    s = orc.gate_scores(x, w, bias)
    mask, margin = orc.select(s, wl.tau)
    assert margin > 1e-3
    cu, gidx, inv, T = orc.pack_indices(mask)
    assert np.array_equal(host(tp.mask), mask) and np.array_equal(host(tp.cu_seqlens), cu)
    rg = orc.round_to_dtype(orc.sigmoid(s.astype(np.float32).astype(np.float64))[:, :, None] * x, "bf16")
    out_ref, _ = orc.attention_per_image(qk[:, :, :C], qk[:, :, C:], rg, mask, H)
    assert np.max(np.abs(host(tp.out)[:T] - out_ref)) <= 2e-2
    dO = bun["dy"].reshape(-1, C)[gidx]
    rdq, rdk, rdv = orc.attention_backward_per_image(qk[:, :, :C], qk[:, :, C:], rg, mask, dO, H)

    def rel(got, ref):
        return float(np.max(np.abs(got - ref)) / max(1.0, np.max(np.abs(ref))))

    # gradients w.r.t. the un-packed q|k and r_g: at the selected positions, zero elsewhere
    dqk_full = host(tp.dqk).reshape(-1, 2 * C)
    d_rg = host(tp.d_rg).reshape(-1, C)
    assert rel(dqk_full[gidx][:, :C], rdq) <= 2e-2 and rel(dqk_full[gidx][:, C:], rdk) <= 2e-2
    assert rel(d_rg[gidx], rdv) <= 2e-2
    assert np.all(dqk_full[inv < 0] == 0) and np.all(d_rg[inv < 0] == 0)
    if not fused_bwd:
        dqk = host(tp.dqk_packed)
        assert np.array_equal(dqk_full[gidx], dqk[:T]) and np.array_equal(d_rg[gidx], host(tp.dv_packed)[:T])
    g = orc.gate_backward(x, w, bias, None, bun["labels"], orc.unpack(rdv, inv, B, N), True, tp.loss_scale)
    assert rel(host(tp.dx), g["dx"]) <= 2e-2
    assert rel(host(tp.dw), g["dw"]) <= 2e-2
    assert abs(float(host(tp.loss)[0]) - g["loss"]) <= 1e-3 * abs(g["loss"])


def test_maxpool_matches_oracle(spa):
    rng = np.random.default_rng(3)
    for B, h, w in ((3, 8, 6), (2, 56, 56), (1, 2, 2)):
        s = rng.standard_normal((B, h * w)).astype(np.float32)
        out = torch.empty(B, (h // 2) * (w // 2), dtype=torch.float32, device="cuda")
        spa.spa_maxpool2x2(dev(s), h, w, out)
        torch.cuda.synchronize()
        assert np.array_equal(host(out).astype(np.float64), orc.maxpool2x2(s, h, w))


def test_hierarchy_forward_with_upscale_scores(spa, pipeline):
    """Four Swin-like stages (reduced batch): each stage's scores are max-merged with the
    2x2 max-pooled scores of the finer stage; selection, packing and attention per stage."""
    bundles = wlmod.generate_hierarchy(seed=1, B=3)
    s_up_ref, s_up_dev = None, None
    for i, bun in enumerate(bundles):
        wl = bun["workload"]
        h, w = wl.grid
        C = wl.C
        ref = orc.spa_forward(bun["x"], bun["w"], bun["bias"], bun["qkv"], wl.H, wl.tau, wl.dtype, s_up=s_up_ref)
        assert ref["margin"] > 1e-3
        fp = pipeline.ForwardPass(wl.B, wl.N, C, wl.H, wl.dtype, wl.tau, wl.bias)
        fp.run(dev(bun["x"], wl.dtype), dev(bun["w"], wl.dtype), dev(bun["qkv"], wl.dtype), s_up=s_up_dev)
        torch.cuda.synchronize()
        T = ref["total"]
        assert np.array_equal(host(fp.mask), ref["mask"])
        assert np.array_equal(host(fp.cu_seqlens), ref["cu_seqlens"])
        assert np.array_equal(host(fp.gather_idx)[:T], ref["gather_idx"])
        assert np.max(np.abs(host(fp.out)[:T] - ref["out"])) <= 2e-2
        assert np.max(np.abs(host(fp.y) - ref["y"])) <= 2e-2
        if i > 0:
            # the up-scale scores added tokens the stage's own gate would have dropped,
            # and the stage covers the pooled foreground of the finer stage
            own, _ = orc.select(orc.gate_scores(bun["x"], bun["w"], bun["bias"]), wl.tau)
            assert ref["mask"].sum() > own.sum()
            assert np.all(ref["mask"] >= bun["stage_foreground"])
        if i + 1 < len(bundles):
            # hand the post-max scores to the next (2x coarser) stage
            s_up_ref = orc.maxpool2x2(ref["scores"].astype(np.float32), h, w).astype(np.float32)
            pooled = torch.empty(wl.B, (h // 2) * (w // 2), dtype=torch.float32, device="cuda")
            spa.spa_maxpool2x2(fp.scores, h, w, pooled)
            s_up_dev = pooled
            torch.cuda.synchronize()
            assert np.max(np.abs(host(pooled) - s_up_ref)) <= 1e-3


def test_hierarchy_backward_stage_with_upscale_scores(spa, pipeline):
    """Backward of a coarse stage whose scores were partly taken from s_up: no gradient to
    (w, b) where the up-scale score won the max."""
    bundles = wlmod.generate_hierarchy(seed=2, B=2)
    b2, b3 = bundles[1], bundles[2]
    wl2, wl3 = b2["workload"], b3["workload"]
    s2 = orc.gate_scores(b2["x"], b2["w"], b2["bias"])
    s_up = orc.maxpool2x2(s2.astype(np.float32), *wl2.grid).astype(np.float32)
    B, N, C = wl3.B, wl3.N, wl3.C
    x, w = b3["x"], b3["w"]
    g_own = orc.gate_only(x, w, b3["bias"])
    assert np.min(np.abs(g_own - s_up)) > 1e-4 and (g_own < s_up).any() and (g_own > s_up).any()
    rng = np.random.default_rng(5)
    d_rg = wlmod.round_bf16(rng.standard_normal((B, N, C)).astype(np.float32))
    lam = 0.01 / (B * N)
    ref = orc.gate_backward(x, w, b3["bias"], s_up, b3["labels"], d_rg, True, lam)
    xd, wd, sup_d = dev(x, "bf16"), dev(w, "bf16"), dev(s_up)
    scores = torch.empty(B, N, dtype=torch.float32, device="cuda")
    mask = torch.empty(B, N, dtype=torch.uint8, device="cuda")
    spa.spa_gate_select(xd, wd, b3["bias"], sup_d, wl3.tau, scores, mask)
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    dx = torch.empty(B, N, C, dtype=torch.bfloat16, device="cuda")
    dw = torch.empty(C, dtype=torch.float32, device="cuda")
    db = torch.empty(1, dtype=torch.float32, device="cuda")
    ws = torch.empty(spa.spa_gate_bwd_workspace_bytes(B, N, C, spa.SPA_BF16), dtype=torch.uint8, device="cuda")
    spa.spa_gate_bwd(xd, wd, b3["bias"], scores, sup_d, dev(b3["labels"]), dev(d_rg, "bf16"), True, lam, loss, dx, dw, db, ws)
    torch.cuda.synchronize()
    assert np.max(np.abs(host(scores) - ref["scores"])) <= 1e-3 * (1 + np.abs(ref["scores"]).max())
    assert np.max(np.abs(host(dx) - ref["dx"])) / max(1.0, np.abs(ref["dx"]).max()) <= 2e-2
    assert np.max(np.abs(host(dw) - ref["dw"])) / max(1.0, np.abs(ref["dw"]).max()) <= 1e-3
    assert abs(float(host(db)[0]) - ref["db"]) <= 1e-3 * max(1.0, abs(ref["db"]))


@pytest.mark.parametrize("seed", range(6))
def test_random_shapes_forward(spa, seed):
    """Random B, N, H, head dim, dtype, selection density (including empty and full images,
    N not a multiple of any tile): integers bit-exact, values within tolerance."""
    rng = np.random.default_rng(100 + seed)
    dtype = ["f32", "bf16"][seed % 2]
    Dh = [32, 64][(seed // 2) % 2]
    H = int(rng.integers(1, 5))
    C = H * Dh
    B = int(rng.integers(1, 7))
    N = int(rng.integers(1, 400))
    mk = wlmod.round_bf16 if dtype == "bf16" else (lambda a: a)
    x = mk(rng.standard_normal((B, N, C)).astype(np.float32))
    w = mk((rng.standard_normal(C) / np.sqrt(C)).astype(np.float32))
    qkv = mk(rng.standard_normal((B, N, 3 * C)).astype(np.float32))
    bias = float(rng.normal() * 0.5)
    ref = orc.spa_forward(x, w, bias, qkv, H, 0.5, dtype)
    near = np.abs(ref["scores"]) < 1e-3        # tokens whose decision is a rounding tie are excluded
    td = tdtype(dtype)
    cap = B * N
    scores = torch.empty(B, N, dtype=torch.float32, device="cuda")
    mask = torch.empty(B, N, dtype=torch.uint8, device="cuda")
    spa.spa_gate_select(dev(x, dtype), dev(w, dtype), bias, None, 0.5, scores, mask)
    torch.cuda.synchronize()
    got_mask = host(mask)
    assert np.array_equal(got_mask[~near], ref["mask"][~near])
    # continue from the device's own mask so a near-tie cannot change the rest of the check
    ref_cu, ref_gidx, ref_inv, T = orc.pack_indices(got_mask)
    packed = torch.zeros(cap, 3 * C, dtype=td, device="cuda")
    cu = torch.empty(B + 1, dtype=torch.int32, device="cuda")
    gidx = torch.empty(cap, dtype=torch.int32, device="cuda")
    inv = torch.empty(cap, dtype=torch.int32, device="cuda")
    total = torch.empty(1, dtype=torch.int32, device="cuda")
    out = torch.zeros(cap, C, dtype=td, device="cuda")
    lse = torch.zeros(H, cap, dtype=torch.float32, device="cuda")
    y = torch.empty(B, N, C, dtype=td, device="cuda")
    spa.spa_pack(dev(qkv, dtype), mask, None, None, 0, packed, cu, gidx, inv, total)
    spa.spa_packed_attention(packed[:, :C], packed[:, C:2 * C], packed[:, 2 * C:], cu, B, N, H, Dh, out, lse)
    spa.spa_unpack(out, inv, None, y)
    torch.cuda.synchronize()
    assert np.array_equal(host(cu), ref_cu) and int(host(total)[0]) == T
    assert np.array_equal(host(gidx)[:T], ref_gidx) and np.array_equal(host(inv), ref_inv)
    ref_out, _ = orc.attention_per_image(qkv[..., :C], qkv[..., C:2 * C], qkv[..., 2 * C:], got_mask, H)
    tol = 1e-5 if dtype == "f32" else 2e-2
    assert np.max(np.abs(host(out)[:T] - ref_out), initial=0.0) <= tol
    assert np.max(np.abs(host(y) - orc.unpack(ref_out, ref_inv, B, N))) <= tol


@pytest.mark.parametrize("form", ["packed", "gathered", "fused"])
def test_forward_is_run_to_run_bit_stable(spa, pipeline, form):
    """20 runs of the forward chain (each of its three forms) on the same inputs: every output bit for bit."""
    wl = dataclasses.replace(wlmod.WORKLOADS["vit_s"], B=16)
    bun = wlmod.generate(wl, 4)
    fp = pipeline.ForwardPass(wl.B, wl.N, wl.C, wl.H, wl.dtype, wl.tau, wl.bias, gathered=form != "packed",
                              fused_index=form == "fused")
    x, w, qkv = dev(bun["x"], "bf16"), dev(bun["w"], "bf16"), dev(bun["qkv"], "bf16")
    first = None
    for _ in range(20):
        fp.run(x, w, qkv)
        torch.cuda.synchronize()
        snap = [host(t).copy() for t in (fp.scores, fp.mask, fp.cu_seqlens, fp.gather_idx, fp.inv_pos, fp.y)]
        if first is None:
            first = snap
        else:
            for a, b in zip(first, snap):
                assert np.array_equal(a, b)


def test_training_step_is_run_to_run_bit_stable(spa, pipeline):
    """20 runs of forward + backward with the selection loss: loss, dx, dw, db and dq|dk bit for bit
    (every reduction of the path has a fixed order; there are no atomics on floating point)."""
    wl = dataclasses.replace(wlmod.WORKLOADS["vit_b_train"], B=16)
    bun = wlmod.generate(wl, 5)
    C = wl.C
    tp = pipeline.TrainPass(wl.B, wl.N, C, wl.H, wl.dtype, wl.tau, wl.bias)
    x, w, dy = dev(bun["x"], "bf16"), dev(bun["w"], "bf16"), dev(bun["dy"], "bf16")
    qk = dev(np.ascontiguousarray(bun["qkv"][:, :, :2 * C]), "bf16")
    labels = dev(bun["labels"])
    stages = tp.stages(x, w, qk, labels, dy)
    first = None
    for _ in range(20):
        for _, fn in stages:
            fn()
        torch.cuda.synchronize()
        snap = [host(t).copy() for t in (tp.loss, tp.dx, tp.dw, tp.db, tp.dqk, tp.y)]
        if first is None:
            first = snap
        else:
            for a, b in zip(first, snap):
                assert np.array_equal(a, b, equal_nan=True)


def test_gate_select_pooled_equals_pool_then_gate(spa):
    """The gate with the 2x2 max-pool folded in against the oracle's composition
    (maxpool2x2 then gate_scores / select), and bit for bit against the two separate launches."""
    rng = np.random.default_rng(41)
    for dtype, (gh, gw), C in (("bf16", (14, 14), 384), ("f32", (5, 9), 64), ("bf16", (7, 7), 768)):
        B, N = 3, gh * gw
        mk = wlmod.round_bf16 if dtype == "bf16" else (lambda a: a)
        x = mk(rng.standard_normal((B, N, C)).astype(np.float32))
        w = mk((rng.standard_normal(C) * 2 / np.sqrt(C)).astype(np.float32))
        s_fine = (rng.standard_normal((B, 4 * N)) * 1.5).astype(np.float32)
        s_up = orc.maxpool2x2(s_fine, 2 * gh, 2 * gw)
        s_ref = orc.gate_scores(x, w, 0.1, s_up)
        mask_ref, _ = orc.select(s_ref, 0.4)
        near = np.abs(s_ref - orc.threshold_logit(0.4)) < (1e-3 if dtype == "bf16" else 1e-5)
        xd, wd = dev(x, dtype), dev(w, dtype)
        sc = torch.empty(B, N, dtype=torch.float32, device="cuda")
        m = torch.empty(B, N, dtype=torch.uint8, device="cuda")
        cnt = torch.empty(B, dtype=torch.int32, device="cuda")
        pooled = torch.empty(B, N, dtype=torch.float32, device="cuda")
        spa.spa_gate_select_pooled(xd, wd, 0.1, dev(s_fine), gh, gw, 0.4, sc, m, cnt, pooled)
        sc2, m2, pooled2 = torch.empty_like(sc), torch.empty_like(m), torch.empty_like(pooled)
        spa.spa_maxpool2x2(dev(s_fine), 2 * gh, 2 * gw, pooled2)
        spa.spa_gate_select(xd, wd, 0.1, pooled2, 0.4, sc2, m2)
        torch.cuda.synchronize()
        assert np.array_equal(host(pooled), s_up.astype(np.float32))         # a max of fp32 values is exact
        assert np.max(np.abs(host(sc) - s_ref)) <= (1e-3 if dtype == "bf16" else 1e-5)
        assert np.array_equal(host(m)[~near], mask_ref[~near])
        assert torch.equal(sc, sc2) and torch.equal(m, m2) and torch.equal(pooled, pooled2)
        assert np.array_equal(host(cnt), host(m).sum(1).astype(np.int32))


def test_hierarchy_pass_matches_stagewise_oracle(spa, pipeline):
    """HierarchyPass (three launches per stage, pooling inside the gate) against the oracle run
    stage by stage with max-pooled up-scale scores."""
    bundles = wlmod.generate_hierarchy(seed=3, B=2)
    cfg = [(b["workload"].B, *b["workload"].grid, b["workload"].C, b["workload"].H, b["workload"].dtype,
            b["workload"].tau, b["bias"]) for b in bundles]
    hp = pipeline.HierarchyPass(cfg)
    ys = hp.run([dev(b["x"], "bf16") for b in bundles], [dev(b["w"], "bf16") for b in bundles],
                [dev(b["qkv"], "bf16") for b in bundles])
    torch.cuda.synchronize()
    s_up = None
    for i, bun in enumerate(bundles):
        wl = bun["workload"]
        ref = orc.spa_forward(bun["x"], bun["w"], bun["bias"], bun["qkv"], wl.H, wl.tau, wl.dtype, s_up=s_up)
        assert ref["margin"] > 1e-3
        fp = hp.passes[i]
        assert np.array_equal(host(fp.mask), ref["mask"]) and np.array_equal(host(fp.cu_seqlens), ref["cu_seqlens"])
        assert np.max(np.abs(host(ys[i]) - ref["y"])) <= 2e-2
        s_up = orc.maxpool2x2(ref["scores"].astype(np.float32), *wl.grid).astype(np.float32)


@pytest.mark.parametrize("concurrent", [False, True])
def test_hierarchy_training_chain_matches_stagewise_oracle(spa, pipeline, concurrent):
    """Forward + backward over the four stages (reduced batch) through HierarchyTrainPass:
    every stage's selection, attention gradients and gate gradients against the oracle run stage
    by stage with max-pooled up-scale scores; on one stream and with a stream per stage."""
    bundles = wlmod.generate_hierarchy(seed=4, B=2)
    cfg = [(b["workload"].B, *b["workload"].grid, b["workload"].C, b["workload"].H, b["workload"].dtype,
            b["workload"].tau, b["bias"]) for b in bundles]
    hp = pipeline.HierarchyTrainPass(cfg, concurrent=concurrent)
    qks = [b["qkv"][:, :, :2 * b["workload"].C] for b in bundles]
    hp.run([dev(b["x"], "bf16") for b in bundles], [dev(b["w"], "bf16") for b in bundles],
           [dev(q, "bf16") for q in qks], [dev(b["labels"]) for b in bundles], [dev(b["dy"], "bf16") for b in bundles])
    torch.cuda.synchronize()

    def rel(got, ref):
        return float(np.max(np.abs(got - ref)) / max(1.0, np.max(np.abs(ref))))

    s_up = None
    for i, bun in enumerate(bundles):
        wl, tp = bun["workload"], hp.passes[i]
        B, N, C, H = wl.B, wl.N, wl.C, wl.H
        x, w, bias, qk = bun["x"], bun["w"], bun["bias"], qks[i]
        s = orc.gate_scores(x, w, bias, s_up)
        mask, margin = orc.select(s, wl.tau)
        assert margin > 1e-3
        cu, gidx, inv, T = orc.pack_indices(mask)
        assert np.array_equal(host(tp.mask), mask) and np.array_equal(host(tp.cu_seqlens), cu)
        rg = orc.round_to_dtype(orc.sigmoid(s.astype(np.float32).astype(np.float64))[:, :, None] * x, "bf16")
        dO = bun["dy"].reshape(-1, C)[gidx]
        rdq, rdk, rdv = orc.attention_backward_per_image(qk[:, :, :C], qk[:, :, C:], rg, mask, dO, H)
        dqk, d_rg = host(tp.dqk).reshape(-1, 2 * C), host(tp.d_rg).reshape(-1, C)     # at token positions
        assert rel(dqk[gidx][:, :C], rdq) <= 2e-2 and rel(dqk[gidx][:, C:], rdk) <= 2e-2
        assert rel(d_rg[gidx], rdv) <= 2e-2
        assert np.all(dqk[inv < 0] == 0) and np.all(d_rg[inv < 0] == 0)
        if s_up is not None:
            assert np.min(np.abs(orc.gate_only(x, w, bias) - s_up)) > 1e-4      # which side won the max is unambiguous
        g = orc.gate_backward(x, w, bias, s_up, bun["labels"], orc.unpack(rdv, inv, B, N), True, tp.loss_scale)
        assert rel(host(tp.dx), g["dx"]) <= 2e-2 and rel(host(tp.dw), g["dw"]) <= 2e-2
        assert abs(float(host(tp.loss)[0]) - g["loss"]) <= 1e-3 * abs(g["loss"])
        s_up = orc.maxpool2x2(s.astype(np.float32), *wl.grid).astype(np.float32)


def test_independent_batches_on_four_streams_match_their_own_results(spa, pipeline):
    """Four different batches in flight on four HIP streams (as the benchmark runs the forward
    chain): every batch's outputs equal, bit for bit, what the same batch gives alone on one
    stream, so the calls share no hidden state."""
    wl = dataclasses.replace(wlmod.WORKLOADS["vit_s"], B=16)
    bundles = [wlmod.generate(wl, seed) for seed in (11, 12, 13, 14)]
    ins = [(dev(b["x"], "bf16"), dev(b["w"], "bf16"), dev(b["qkv"], "bf16")) for b in bundles]
    alone = []
    for (x, w, qkv), b in zip(ins, bundles):
        fp = pipeline.ForwardPass(wl.B, wl.N, wl.C, wl.H, wl.dtype, wl.tau, b["bias"], keep_packed_out=False)
        alone.append((fp.run(x, w, qkv).clone(), fp.gather_idx.clone(), int(fp.total.item())))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in bundles]
    passes, chains = [], []
    for st, (x, w, qkv), b in zip(streams, ins, bundles):
        with torch.cuda.stream(st):
            fp = pipeline.ForwardPass(wl.B, wl.N, wl.C, wl.H, wl.dtype, wl.tau, b["bias"], keep_packed_out=False)
            passes.append(fp)
            chains.append([fn for _, fn in fp.stages(x, w, qkv)])
    torch.cuda.synchronize()
    for _ in range(20):                      # steps dealt round-robin to the streams, launches interleaved
        for k in range(3):
            for chain in chains:
                chain[k]()
    torch.cuda.synchronize()
    for fp, (y, gidx, T) in zip(passes, alone):
        assert int(fp.total.item()) == T
        assert torch.equal(fp.gather_idx[:T], gidx[:T]) and torch.equal(fp.y, y)


@pytest.mark.parametrize("lean", [False, True])
def test_hierarchy_full_batch_forward_matches_stagewise_oracle(spa, pipeline, lean):
    """The four-stage hierarchy at its stated size (batch 16, 56^2 .. 7^2 tokens, C 96 .. 768)
    through HierarchyPass: every stage's mask, cu_seqlens, gather_idx, inv_pos and total bit-exact,
    packed attention output and y within the bf16 bound, the score map handed down within the score
    bound.  lean = the form bench.py times (no row copies, no packed output; the two coarse stages
    take their packing order from the mask and write no index): what that form does write is checked."""
    bundles = wlmod.generate_hierarchy(0)
    assert [b["workload"].B for b in bundles] == [16] * 4 and bundles[0]["workload"].N == 3136
    hp = pipeline.HierarchyPass(_hier_cfg(bundles), lean=lean)
    ys = hp.run([dev(b["x"], "bf16") for b in bundles], [dev(b["w"], "bf16") for b in bundles],
                [dev(b["qkv"], "bf16") for b in bundles])
    torch.cuda.synchronize()
    s_up = None
    for i, bun in enumerate(bundles):
        wl, fp = bun["workload"], hp.passes[i]
        ref = orc.spa_forward(bun["x"], bun["w"], bun["bias"], bun["qkv"], wl.H, wl.tau, wl.dtype, s_up=s_up)
        assert ref["margin"] > 1e-3
        T = ref["total"]
        assert np.array_equal(host(fp.mask), ref["mask"])
        assert fp.from_mask == (lean and wl.N <= 256)
        if not fp.from_mask:
            assert np.array_equal(host(fp.cu_seqlens), ref["cu_seqlens"]) and int(host(fp.total)[0]) == T
            assert np.array_equal(host(fp.gather_idx)[:T], ref["gather_idx"])
            assert np.array_equal(host(fp.inv_pos), ref["inv_pos"])
        assert np.max(np.abs(host(fp.scores) - ref["scores"])) <= 1e-3 * (1 + np.abs(ref["scores"]).max())
        if not lean:
            assert np.max(np.abs(host(fp.out)[:T] - ref["out"])) <= 2e-2
        assert np.max(np.abs(host(ys[i]) - ref["y"])) <= 2e-2
        if i > 0:      # the pooled score map the gate kernel handed to the backward pass
            assert np.max(np.abs(host(hp.s_up[i]) - s_up)) <= 1e-3 * (1 + np.abs(s_up).max())
        s_up = orc.maxpool2x2(ref["scores"].astype(np.float32), *wl.grid).astype(np.float32)


@pytest.mark.parametrize("concurrent", [False, True])
def test_hierarchy_full_batch_training_chain_matches_stagewise_oracle(spa, pipeline, concurrent):
    """Forward + backward of the four-stage hierarchy at its stated size (batch 16) through
    HierarchyTrainPass as bench.py runs it (one stream, and a stream per stage): every stage's
    integers bit-exact; y, dq | dk, d_rg, dx, dw, db and the loss against the oracle run stage by
    stage with the max-pooled up-scale scores."""
    bundles = wlmod.generate_hierarchy(0)
    hp = pipeline.HierarchyTrainPass(_hier_cfg(bundles), concurrent=concurrent)
    qks = [b["qkv"][:, :, :2 * b["workload"].C] for b in bundles]
    hp.run([dev(b["x"], "bf16") for b in bundles], [dev(b["w"], "bf16") for b in bundles],
           [dev(q, "bf16") for q in qks], [dev(b["labels"]) for b in bundles], [dev(b["dy"], "bf16") for b in bundles])
    torch.cuda.synchronize()
    s_up = None
    for i, bun in enumerate(bundles):
        wl, tp = bun["workload"], hp.passes[i]
        B, N, C, H = wl.B, wl.N, wl.C, wl.H
        assert B == 16
        x, w, bias, qk = bun["x"], bun["w"], bun["bias"], qks[i]
        s = orc.gate_scores(x, w, bias, s_up)
        mask, margin = orc.select(s, wl.tau)
        assert margin > 1e-3
        cu, gidx, inv, T = orc.pack_indices(mask)
        assert np.array_equal(host(tp.mask), mask) and np.array_equal(host(tp.cu_seqlens), cu)
        assert np.array_equal(host(tp.gather_idx)[:T], gidx) and np.array_equal(host(tp.inv_pos), inv)
        assert int(host(tp.total)[0]) == T
        rg = orc.round_to_dtype(orc.sigmoid(s.astype(np.float32).astype(np.float64))[:, :, None] * x, "bf16")
        out_ref, _ = orc.attention_per_image(qk[:, :, :C], qk[:, :, C:], rg, mask, H)
        assert np.max(np.abs(host(tp.out)[:T] - out_ref)) <= 2e-2
        assert np.max(np.abs(host(tp.y) - orc.unpack(out_ref, inv, B, N))) <= 2e-2
        dO = bun["dy"].reshape(-1, C)[gidx]
        rdq, rdk, rdv = orc.attention_backward_per_image(qk[:, :, :C], qk[:, :, C:], rg, mask, dO, H)
        dqk, d_rg = host(tp.dqk).reshape(-1, 2 * C), host(tp.d_rg).reshape(-1, C)     # at token positions
        assert _rel(dqk[gidx][:, :C], rdq) <= 2e-2 and _rel(dqk[gidx][:, C:], rdk) <= 2e-2
        assert _rel(d_rg[gidx], rdv) <= 2e-2
        assert np.all(dqk[inv < 0] == 0) and np.all(d_rg[inv < 0] == 0)
        dx_d, dw_d, db_d, loss_d = host(tp.dx), host(tp.dw), float(host(tp.db)[0]), float(host(tp.loss)[0])
        ok = [(_rel(dx_d, g["dx"]) <= 2e-2 and _rel(dw_d, g["dw"]) <= 2e-2
               and abs(db_d - g["db"]) <= 2e-2 * max(1.0, abs(g["db"]))
               and abs(loss_d - g["loss"]) <= 1e-3 * abs(g["loss"]))
              for g in _gate_backward_candidates(x, w, bias, s_up, bun["labels"], orc.unpack(rdv, inv, B, N),
                                                 tp.loss_scale)]
        assert any(ok), f"stage {i + 1}: gate backward matches no admissible reading of the near-ties"
        s_up = orc.maxpool2x2(s.astype(np.float32), *wl.grid).astype(np.float32)


@pytest.mark.parametrize("fused_index", [False, True])
@pytest.mark.parametrize("name", ["tiny", "vit_s", "det"])
def test_full_size_gathered_forward_as_benchmarked(spa, pipeline, name, fused_index):
    """The forward step bench.py times (gate_select [+ index in the same launch | index-only pack],
    attention on gathered rows + scatter) on the full batch: integers bit-exact, y against the oracle on every row, and
    bit-equal to the form that copies the rows first."""
    wl = wlmod.WORKLOADS[name]
    bun = wlmod.generate(wl, 0)
    ins = (dev(bun["x"], wl.dtype), dev(bun["w"], wl.dtype), dev(bun["qkv"], wl.dtype))
    fg = pipeline.ForwardPass(wl.B, wl.N, wl.C, wl.H, wl.dtype, wl.tau, wl.bias, gathered=True, keep_packed_out=False,
                              fused_index=fused_index)
    fp = pipeline.ForwardPass(wl.B, wl.N, wl.C, wl.H, wl.dtype, wl.tau, wl.bias, keep_packed_out=False)
    yg, yp = fg.run(*ins), fp.run(*ins)
    torch.cuda.synchronize()
    assert len(fg.stages(*ins)) == (2 if fused_index else 3)
    ref = orc.spa_forward(bun["x"], bun["w"], bun["bias"], bun["qkv"], wl.H, wl.tau, wl.dtype)
    assert ref["margin"] > 1e-3
    T = ref["total"]
    assert np.array_equal(host(fg.mask), ref["mask"]) and np.array_equal(host(fg.cu_seqlens), ref["cu_seqlens"])
    assert np.array_equal(host(fg.gather_idx)[:T], ref["gather_idx"]) and np.array_equal(host(fg.inv_pos), ref["inv_pos"])
    assert int(host(fg.total)[0]) == T
    assert torch.equal(yg, yp)
    assert np.max(np.abs(host(yg) - ref["y"])) <= (1e-5 if wl.dtype == "f32" else 2e-2)
