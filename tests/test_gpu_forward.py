"""Parity of the HIP forward path against the CPU oracle, through the C-ABI binding.
Integers (mask, counts, cu_seqlens, gather_idx, inv_pos, total) bit-exact; unscaled row
copies bit-exact; fp32 values max-abs <= 1e-5; bf16 attention outputs max-abs <= 2e-2."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import spa_oracle as orc
from paper_2410_23608_amd import workloads as wlmod
from spa_harness import Forward, dev, host, tdtype

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}
SCORE_TOL = {"f32": 1e-5, "bf16": 1e-3}


@pytest.fixture(scope="module")
def spa():
    from paper_2410_23608_amd import spa as mod
    return mod


def small(wl, B):
    return dataclasses.replace(wl, B=B)


CASES = [
    ("tiny", None),          # fp32, Dh 32, the whole tiny workload
    ("vit_s", 8),            # bf16, Dh 64, N=196 (ragged 64/32 tails)
    ("vit_b_train", 4),      # bf16, Dh 64, C=768
    ("det", 2),              # bf16, Dh 32, N=4200, long segments (many key tiles)
]


def run_case(spa, wl, seed, container_len=0, use_counts=True, s_up=None, base=None):
    bun = wlmod.generate(wl, seed)
    ref = orc.spa_forward(bun["x"], bun["w"], bun["bias"], bun["qkv"], wl.H, wl.tau, wl.dtype,
                          s_up=s_up, container_len=container_len, base=base)
    f = Forward(spa, wl.B, wl.N, wl.C, wl.H, wl.dtype, container_len, use_counts)
    f.run(dev(bun["x"], wl.dtype), dev(bun["w"], wl.dtype), bun["bias"], dev(bun["qkv"], wl.dtype), wl.tau,
          s_up=None if s_up is None else dev(s_up.astype(np.float32)),
          base=None if base is None else dev(base, wl.dtype))
    torch.cuda.synchronize()
    return bun, ref, f


def check_forward(wl, bun, ref, f, container_len=0):
    T = ref["total"]
    assert ref["margin"] > 1e-3                      # bit-exact masks are well defined
    s = host(f.scores)
    assert np.max(np.abs(s - ref["scores"]) / (1 + np.abs(ref["scores"]))) <= SCORE_TOL[wl.dtype]
    assert np.array_equal(host(f.mask), ref["mask"])
    if f.counts is not None:
        assert np.array_equal(host(f.counts), ref["counts"])
    assert np.array_equal(host(f.cu), ref["cu_seqlens"])
    assert int(host(f.total)[0]) == T
    assert np.array_equal(host(f.gidx)[:T], ref["gather_idx"])
    assert np.all(host(f.gidx)[T:] == -7)            # nothing written past T
    assert np.array_equal(host(f.inv), ref["inv_pos"])
    pq = host(f.packed_qkv)
    t_pad = ref["packed_qkv"].shape[0]
    assert np.array_equal(pq[:t_pad].astype(np.float64), ref["packed_qkv"])     # bit-exact copies, zero pad rows
    assert np.all(np.isnan(pq[t_pad:]))              # canary rows untouched
    out = host(f.out)
    assert np.all(np.isnan(out[T:]))
    err = np.max(np.abs(out[:T] - ref["out"])) if T else 0.0
    assert err <= TOL[wl.dtype], err
    lse = host(f.lse)
    assert np.max(np.abs(lse[:, :T] - ref["lse"])) <= 1e-3 if T else True
    y = host(f.y)
    assert np.max(np.abs(y - ref["y"])) <= TOL[wl.dtype]
    return err


@pytest.mark.parametrize("name,B", CASES)
def test_forward_chain_matches_oracle(spa, name, B):
    wl = wlmod.WORKLOADS[name]
    if B is not None:
        wl = small(wl, B)
    bun, ref, f = run_case(spa, wl, seed=0)
    check_forward(wl, bun, ref, f)
    # unselected rows of y are exactly zero, selected rows are exact copies of the packed output
    y, out, inv = host(f.y).reshape(-1, wl.C), host(f.out), ref["inv_pos"]
    assert np.all(y[inv < 0] == 0)
    assert np.array_equal(y[inv >= 0], out[inv[inv >= 0]])


@pytest.mark.parametrize("name,B", [("tiny", None), ("vit_s", 4)])
def test_forward_without_counts_and_with_containers(spa, name, B):
    wl = wlmod.WORKLOADS[name]
    if B is not None:
        wl = small(wl, B)
    bun, ref, f = run_case(spa, wl, seed=1, container_len=49, use_counts=False)
    check_forward(wl, bun, ref, f, 49)
    T = ref["total"]
    assert ref["packed_qkv"].shape[0] == -(-T // 49) * 49


def test_forward_with_upscale_scores_and_base(spa):
    wl = small(wlmod.WORKLOADS["vit_s"], 4)
    rng = np.random.default_rng(5)
    # up-scale scores: mostly far below, sometimes well above the threshold (adds tokens)
    s_up = np.where(rng.uniform(size=(wl.B, wl.N)) < 0.2, 3.0, -9.0) + rng.uniform(0, 1, size=(wl.B, wl.N))
    s_up = s_up.astype(np.float32)
    base = wlmod.round_bf16(rng.standard_normal((wl.B, wl.N, wl.C)).astype(np.float32))
    bun, ref, f = run_case(spa, wl, seed=2, s_up=s_up, base=base)
    assert ref["mask"].sum() > bun["planted_mask"].sum()
    # y = base (+ out): compare against the oracle evaluated on the device's own bf16 out
    T = ref["total"]
    assert np.array_equal(host(f.mask), ref["mask"])
    assert np.array_equal(host(f.inv), ref["inv_pos"])
    assert np.max(np.abs(host(f.out)[:T] - ref["out"])) <= TOL["bf16"]
    y = host(f.y)
    sel = ref["mask"].astype(bool)
    assert np.array_equal(y[~sel], base[~sel])
    assert np.max(np.abs(y - ref["y"])) <= 2 * TOL["bf16"]      # two bf16 roundings (out, then the sum)


def test_gate_scaled_pack(spa):
    # r_g = Sigmoid(s) . r on the packed rows
    for name, B in (("tiny", None), ("vit_s", 4)):
        wl = wlmod.WORKLOADS[name]
        if B is not None:
            wl = small(wl, B)
        bun = wlmod.generate(wl, 3, with_qkv=False)
        s = orc.gate_scores(bun["x"], bun["w"], bun["bias"])
        mask, _ = orc.select(s, wl.tau)
        cu, gidx, inv, T = orc.pack_indices(mask)
        ref = orc.pack_rows(bun["x"], gidx, s.astype(np.float32), 0, wl.dtype)
        cap = wl.B * wl.N
        packed = torch.full((cap, wl.C), float("nan"), dtype=tdtype(wl.dtype), device="cuda")
        cu_d = torch.empty(wl.B + 1, dtype=torch.int32, device="cuda")
        spa.spa_pack(dev(bun["x"], wl.dtype), dev(mask), None, dev(s.astype(np.float32)), 0, packed, cu_d,
                     None, None, None)
        torch.cuda.synchronize()
        got = host(packed)
        assert np.array_equal(host(cu_d), cu)
        tol = 1e-6 if wl.dtype == "f32" else 2.0 ** -7       # one bf16 ulp at |x| < 4 ... rounding of the product
        assert np.max(np.abs(got[:T] - ref) / np.maximum(1.0, np.abs(ref))) <= tol
        assert np.all(np.isnan(got[T:]))


def _attention_only(spa, q, k, v, mask, H, dtype, want_lse=True):
    """Packs q|k|v with a given mask on the device and runs the packed attention."""
    B, N, C = q.shape
    qkv = np.concatenate([q, k, v], axis=2).astype(np.float32)
    cap = B * N
    td = tdtype(dtype)
    packed = torch.zeros(cap, 3 * C, dtype=td, device="cuda")
    cu = torch.empty(B + 1, dtype=torch.int32, device="cuda")
    inv = torch.empty(cap, dtype=torch.int32, device="cuda")
    out = torch.full((cap, C), float("nan"), dtype=td, device="cuda")
    lse = torch.full((H, cap), float("nan"), dtype=torch.float32, device="cuda")
    spa.spa_pack(dev(qkv, dtype), dev(mask), None, None, 0, packed, cu, None, inv, None)
    spa.spa_packed_attention(packed[:, :C], packed[:, C:2 * C], packed[:, 2 * C:], cu, B, N, H, C // H,
                             out, lse if want_lse else None)
    torch.cuda.synchronize()
    return host(out), host(lse), host(cu), host(inv)


@pytest.mark.parametrize("dtype,Dh", [("f32", 32), ("f32", 64), ("bf16", 32), ("bf16", 64)])
def test_attention_edge_cases(spa, dtype, Dh):
    """empty images, single-token segments, all selected, lengths around the 32/64/128 tile edges."""
    H = 2
    C = H * Dh
    lens = [0, 1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 200, 0, 257]
    B, N = len(lens), 257
    rng = np.random.default_rng(11)
    mk = wlmod.round_bf16 if dtype == "bf16" else (lambda a: a)
    q, k, v = (mk(rng.standard_normal((B, N, C)).astype(np.float32)) for _ in range(3))
    mask = np.zeros((B, N), np.uint8)
    for b, n in enumerate(lens):
        mask[b, rng.permutation(N)[:n]] = 1
    assert mask[-1].all()                                     # last image: every token selected
    ref_out, ref_lse = orc.attention_per_image(q, k, v, mask, H)
    out, lse, cu, inv = _attention_only(spa, q, k, v, mask, H, dtype)
    T = int(mask.sum())
    assert np.array_equal(cu, orc.pack_indices(mask)[0])
    assert np.max(np.abs(out[:T] - ref_out)) <= TOL[dtype]
    assert np.max(np.abs(lse[:, :T] - ref_lse)) <= (1e-5 if dtype == "f32" else 1e-3) * (1 + np.abs(ref_lse).max())
    assert np.all(np.isnan(out[T:]))
    # single-token segment: O = v exactly
    j = cu[1]
    assert np.array_equal(out[j], v[1, mask[1].astype(bool)][0])
    # all selected == ordinary full self-attention of that image (library softmax)
    import scipy.special
    b = B - 1
    for h in range(H):
        sl = slice(h * Dh, (h + 1) * Dh)
        S = q[b, :, sl].astype(np.float64) @ k[b, :, sl].astype(np.float64).T / np.sqrt(Dh)
        full = scipy.special.softmax(S, axis=1) @ v[b, :, sl].astype(np.float64)
        assert np.max(np.abs(out[cu[b]:cu[b + 1], sl] - full)) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_attention_no_cross_image_leakage(spa, dtype):
    """Poisoning every other image and every unselected token leaves an image's outputs
    bit-identical (segments never mix)."""
    B, N, H, Dh = 3, 150, 2, 32
    C = H * Dh
    rng = np.random.default_rng(12)
    mk = wlmod.round_bf16 if dtype == "bf16" else (lambda a: a)
    q, k, v = (mk(rng.standard_normal((B, N, C)).astype(np.float32)) for _ in range(3))
    mask = (rng.uniform(size=(B, N)) < 0.5).astype(np.uint8)
    out0, _, cu, _ = _attention_only(spa, q, k, v, mask, H, dtype)
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    for t in (q2, k2, v2):
        t[0] = 1e30
        t[2] = -1e30
        t[1, mask[1] == 0] = 1e30
    out1, _, _, _ = _attention_only(spa, q2, k2, v2, mask, H, dtype)
    assert np.array_equal(out0[cu[1]:cu[2]], out1[cu[1]:cu[2]])


def test_all_unselected_batch_is_noop(spa):
    wl = wlmod.WORKLOADS["tiny"]
    bun = wlmod.generate(wl, 0)
    f = Forward(spa, wl.B, wl.N, wl.C, wl.H, wl.dtype)
    # bias far below the threshold: nothing selected
    f.run(dev(bun["x"], "f32"), dev(bun["w"], "f32"), -1e4, dev(bun["qkv"], "f32"), wl.tau)
    torch.cuda.synchronize()
    assert int(host(f.total)[0]) == 0 and np.all(host(f.cu) == 0) and np.all(host(f.inv) == -1)
    assert np.all(host(f.y) == 0) and np.all(np.isnan(host(f.out)))


@pytest.mark.parametrize("dtype,Dh", [("bf16", 64), ("bf16", 32), ("f32", 32), ("f32", 64)])
def test_padded_baseline_matches_oracle(spa, dtype, Dh):
    """The padded-to-max baseline computes the same attention on the valid rows (bf16 and fp32:
    the benchmark runs it in the workload's dtype)."""
    B, H = 5, 2
    C = H * Dh
    lens = np.array([40, 97, 1, 0, 130], np.int32)
    n_pad = int(lens.max())
    rng = np.random.default_rng(13)
    mk = wlmod.round_bf16 if dtype == "bf16" else (lambda a: a)
    q, k, v = (mk(rng.standard_normal((B, n_pad, C)).astype(np.float32)) for _ in range(3))
    mask = (np.arange(n_pad)[None, :] < lens[:, None]).astype(np.uint8)
    ref, _ = orc.attention_per_image(q, k, v, mask, H)
    qkv = dev(np.concatenate([q, k, v], axis=2), dtype)
    out = torch.empty(B, n_pad, C, dtype=tdtype(dtype), device="cuda")
    flat = qkv.view(B * n_pad, 3 * C)
    spa.spa_padded_attention(flat[:, :C], flat[:, C:2 * C], flat[:, 2 * C:], dev(lens), B, n_pad, H, Dh, out)
    torch.cuda.synchronize()
    got = host(out)
    assert np.all(np.isfinite(got))
    row = 0
    for b in range(B):
        n = int(lens[b])
        assert np.max(np.abs(got[b, :n] - ref[row:row + n]), initial=0.0) <= TOL[dtype]
        row += n


def test_argument_validation_returns_errors_before_launch(spa):
    x = torch.zeros(2, 8, 64, device="cuda")
    w = torch.zeros(64, device="cuda")
    scores = torch.empty(2, 8, device="cuda")
    mask = torch.empty(2, 8, dtype=torch.uint8, device="cuda")
    with pytest.raises(spa.SpaError) as e:
        spa.spa_gate_select(x, w, 0.0, None, 1.5, scores, mask)
    assert e.value.code == -1 and "tau" in str(e.value)
    out = torch.empty(16, 48, device="cuda")
    cu = torch.zeros(3, dtype=torch.int32, device="cuda")
    with pytest.raises(spa.SpaError) as e:
        spa.spa_packed_attention(out, out, out, cu, 2, 8, 2, 24, out)
    assert e.value.code == -2
    torch.cuda.synchronize()


@pytest.fixture
def short_option(spa):
    """Selects the short-segment forward kernel for one test and restores the default after it."""
    yield lambda value: spa.spa_set_option("attn_fwd_short", value)
    spa.spa_set_option("attn_fwd_short", None)


@pytest.mark.parametrize("dtype,Dh,N,short", [("f32", 32, 150, ""), ("bf16", 64, 196, ""), ("bf16", 64, 196, "wave"),
                                              ("bf16", 64, 196, "wave plain"), ("bf16", 32, 250, "wave"),
                                              ("bf16", 32, 49, ""), ("bf16", 32, 700, ""), ("bf16", 64, 300, "")])
@pytest.mark.parametrize("with_base,keep_out", [(False, True), (True, False)])
def test_fused_attention_unpack_equals_separate_calls(spa, short_option, dtype, Dh, N, short, with_base, keep_out):
    """spa_packed_attention_unpack == spa_packed_attention followed by spa_unpack, bit for bit,
    for the short-segment kernels (whole / wave with blocks numbered by weight / wave numbered
    blindly), the tiled kernel and the fp32 kernel; and both equal the oracle within tolerance."""
    short_option(short if short else "whole")
    B, H = 5, 2
    C = H * Dh
    rng = np.random.default_rng(31)
    mk = wlmod.round_bf16 if dtype == "bf16" else (lambda a: a)
    qkv = mk(rng.standard_normal((B, N, 3 * C)).astype(np.float32))
    base = mk(rng.standard_normal((B, N, C)).astype(np.float32)) if with_base else None
    mask = (rng.uniform(size=(B, N)) < rng.uniform(0.1, 0.9, size=(B, 1))).astype(np.uint8)
    mask[1] = 0                                   # an image with nothing selected
    mask[2] = 1                                   # an image with everything selected
    td, cap = tdtype(dtype), B * N
    packed = torch.zeros(cap, 3 * C, dtype=td, device="cuda")
    cu = torch.empty(B + 1, dtype=torch.int32, device="cuda")
    gidx = torch.zeros(cap, dtype=torch.int32, device="cuda")
    inv = torch.empty(cap, dtype=torch.int32, device="cuda")
    spa.spa_pack(dev(qkv, dtype), dev(mask), None, None, 0, packed, cu, gidx, inv, None)
    pq, pk, pv = packed[:, :C], packed[:, C:2 * C], packed[:, 2 * C:]
    base_d = None if base is None else dev(base, dtype)
    out1 = torch.zeros(cap, C, dtype=td, device="cuda")
    lse1 = torch.zeros(H, cap, dtype=torch.float32, device="cuda")
    y1 = torch.full((B, N, C), float("nan"), dtype=td, device="cuda")
    spa.spa_packed_attention(pq, pk, pv, cu, B, N, H, Dh, out1, lse1)
    spa.spa_unpack(out1, inv, base_d, y1)
    out2 = torch.zeros(cap, C, dtype=td, device="cuda") if keep_out else None
    lse2 = torch.zeros(H, cap, dtype=torch.float32, device="cuda")
    y2 = torch.full((B, N, C), float("nan"), dtype=td, device="cuda")
    spa.spa_packed_attention_unpack(pq, pk, pv, cu, gidx, inv, base_d, H, Dh, y2, out2, lse2)
    torch.cuda.synchronize()
    assert np.array_equal(host(y1), host(y2))
    assert np.array_equal(host(lse1), host(lse2))
    if keep_out:
        assert np.array_equal(host(out1), host(out2))
    ref_out, _ = orc.attention_per_image(qkv[..., :C], qkv[..., C:2 * C], qkv[..., 2 * C:], mask, H)
    ref_y = orc.unpack(ref_out, orc.pack_indices(mask)[2], B, N, base)
    tol = TOL[dtype] * (2 if with_base and dtype == "bf16" else 1)
    assert np.max(np.abs(host(y2) - ref_y)) <= tol


@pytest.mark.parametrize("dtype,Dh,N,short", [("f32", 32, 150, ""), ("f32", 64, 77, ""), ("bf16", 64, 196, ""),
                                              ("bf16", 64, 196, "plain"), ("bf16", 64, 196, "whole"),
                                              ("bf16", 32, 250, "64"), ("bf16", 32, 49, ""), ("bf16", 32, 700, ""),
                                              ("bf16", 64, 300, ""), ("bf16", 32, 1337, "")])
@pytest.mark.parametrize("with_base,keep_out", [(False, True), (True, False)])
def test_gathered_attention_equals_packed_form(spa, short_option, dtype, Dh, N, short, with_base, keep_out):
    """spa_gathered_attention_unpack (rows fetched through gather_idx from the un-packed q | k | v,
    index-only packing) == spa_pack of the rows + spa_packed_attention_unpack, bit for bit, for
    every forward kernel (one-wave numbered by weight / blindly / 64-key steps, whole-segment,
    tiled, fp32), and both equal the oracle within tolerance."""
    short_option(short)
    B, H = 5, 2
    C = H * Dh
    rng = np.random.default_rng(77)
    mk = wlmod.round_bf16 if dtype == "bf16" else (lambda a: a)
    qkv = mk(rng.standard_normal((B, N, 3 * C)).astype(np.float32))
    base = mk(rng.standard_normal((B, N, C)).astype(np.float32)) if with_base else None
    mask = (rng.uniform(size=(B, N)) < rng.uniform(0.1, 0.9, size=(B, 1))).astype(np.uint8)
    mask[1] = 0                                   # an image with nothing selected
    mask[2] = 1                                   # an image with everything selected
    td, cap = tdtype(dtype), B * N
    qkv_d, mask_d = dev(qkv, dtype), dev(mask)
    base_d = None if base is None else dev(base, dtype)
    new = lambda *shape, t=td: torch.full(shape, float("nan"), dtype=t, device="cuda")
    ints = lambda n: torch.full((n,), -9, dtype=torch.int32, device="cuda")
    # packed form: rows copied, then attention + scatter
    packed = torch.zeros(cap, 3 * C, dtype=td, device="cuda")
    cu1, g1, inv1 = ints(B + 1), ints(cap), ints(cap)
    spa.spa_pack(qkv_d, mask_d, None, None, 0, packed, cu1, g1, inv1, None)
    out1, lse1, y1 = new(cap, C), new(H, cap, t=torch.float32), new(B, N, C)
    spa.spa_packed_attention_unpack(packed[:, :C], packed[:, C:2 * C], packed[:, 2 * C:], cu1, g1, inv1, base_d, H, Dh,
                                    y1, out1, lse1)
    # gathered form: indices only, rows fetched where they lie
    cu2, g2, inv2, tot2 = ints(B + 1), ints(cap), ints(cap), ints(1)
    spa.spa_pack(None, mask_d, None, None, 0, None, cu2, g2, inv2, tot2)
    flat = qkv_d.view(cap, 3 * C)
    out2 = new(cap, C) if keep_out else None
    lse2 = new(H, cap, t=torch.float32) if keep_out else None
    y2 = new(B, N, C)
    spa.spa_gathered_attention_unpack(flat[:, :C], flat[:, C:2 * C], flat[:, 2 * C:], cu2, g2, inv2, base_d, H, Dh, y2,
                                      out2, lse2)
    torch.cuda.synchronize()
    T = int(mask.sum())
    assert int(host(tot2)[0]) == T and torch.equal(cu1, cu2) and torch.equal(g1[:T], g2[:T]) and torch.equal(inv1, inv2)
    assert np.array_equal(host(y1), host(y2)) and not np.any(np.isnan(host(y2)))
    if keep_out:
        assert np.array_equal(host(out1)[:T], host(out2)[:T]) and np.array_equal(host(lse1)[:, :T], host(lse2)[:, :T])
        assert np.all(np.isnan(host(out2)[T:]))                  # rows past T untouched
    ref_out, _ = orc.attention_per_image(qkv[..., :C], qkv[..., C:2 * C], qkv[..., 2 * C:], mask, H)
    ref_y = orc.unpack(ref_out, orc.pack_indices(mask)[2], B, N, base)
    tol = TOL[dtype] * (2 if with_base and dtype == "bf16" else 1)
    assert np.max(np.abs(host(y2) - ref_y)) <= tol


@pytest.mark.parametrize("dtype,B,N,C", [("bf16", 64, 196, 384), ("bf16", 8, 4200, 256), ("f32", 2, 196, 64),
                                         ("bf16", 3, 37, 64), ("f32", 1, 1, 8), ("bf16", 5, 4099, 96),
                                         ("bf16", 16, 3136, 96), ("f32", 7, 16, 32)])
def test_gate_select_index_equals_gate_then_pack(spa, dtype, B, N, C):
    """spa_gate_select_index (the gate launch builds the packing index itself) against the oracle's
    indices, and bit for bit against spa_gate_select followed by the index-only spa_pack; shapes
    whose token count is and is not a multiple of the 16-token groups the index builder reads, an
    empty and a full image, up-scale scores; three calls in a row on one arrival counter."""
    rng = np.random.default_rng(B * 1000 + N)
    mk = wlmod.round_bf16 if dtype == "bf16" else (lambda a: a)
    x = mk(rng.standard_normal((B, N, C)).astype(np.float32))
    w = mk((rng.standard_normal(C) * 3 / np.sqrt(C)).astype(np.float32))
    s_up = (rng.standard_normal((B, N)) * 2 - 1).astype(np.float32)
    if B > 2:
        s_up[1] = -50.0
        x[1] = 0                                   # an image with nothing selected (bias below the threshold)
        s_up[2] = 50.0                             # an image with everything selected
    bias = -0.25
    xd, wd, sd = dev(x, dtype), dev(w, dtype), dev(s_up)
    cap = B * N
    ints = lambda n: torch.full((n,), -9, dtype=torch.int32, device="cuda")
    ws = torch.zeros(17 * 1088, dtype=torch.int32, device="cuda")
    for call, sup in enumerate((sd, None, sd)):
        sc1, m1 = torch.empty(B, N, device="cuda"), torch.empty(B, N, dtype=torch.uint8, device="cuda")
        cnt1, cu1, g1, inv1, tot1 = ints(B), ints(B + 1), ints(cap), ints(cap), ints(1)
        spa.spa_gate_select_index(xd, wd, bias, sup, 0.5, sc1, m1, cnt1, cu1, g1, inv1, tot1, ws)
        sc2, m2 = torch.empty(B, N, device="cuda"), torch.empty(B, N, dtype=torch.uint8, device="cuda")
        cnt2, cu2, g2, inv2, tot2 = ints(B), ints(B + 1), ints(cap), ints(cap), ints(1)
        spa.spa_gate_select(xd, wd, bias, sup, 0.5, sc2, m2, cnt2)
        spa.spa_pack(None, m2, None, None, 0, None, cu2, g2, inv2, tot2)
        torch.cuda.synchronize()
        assert not host(ws).any()                                   # the arrival counters are left zero
        T = int(host(tot1)[0])
        assert torch.equal(sc1, sc2) and torch.equal(m1, m2) and torch.equal(cnt1, cnt2)
        assert torch.equal(cu1, cu2) and T == int(host(tot2)[0]) and torch.equal(inv1, inv2)
        assert torch.equal(g1[:T], g2[:T]) and bool((g1[T:] == -9).all())
        # against the oracle, from the device's own mask (near-ties of the threshold aside)
        ref_cu, ref_g, ref_inv, ref_T = orc.pack_indices(host(m1))
        assert np.array_equal(host(cu1), ref_cu) and T == ref_T
        assert np.array_equal(host(g1)[:T], ref_g) and np.array_equal(host(inv1), ref_inv)
        s_ref = orc.gate_scores(x, w, bias, s_up if sup is not None else None)
        mask_ref, _ = orc.select(s_ref, 0.5)
        near = np.abs(s_ref) < (1e-3 if dtype == "bf16" else 1e-5)
        assert np.array_equal(host(m1)[~near], mask_ref[~near])


@pytest.mark.parametrize("B", [64, 70])
def test_short_segments_many_images(spa, B):
    """The one-wave kernel with as many images as lanes (blocks numbered by weight) and with
    more (numbered blindly): same results as the oracle, fused scatter equal to separate calls."""
    N, H, Dh = 40, 3, 32
    C, cap = H * Dh, B * N
    rng = np.random.default_rng(B)
    qkv = wlmod.round_bf16(rng.standard_normal((B, N, 3 * C)).astype(np.float32))
    mask = (rng.uniform(size=(B, N)) < rng.uniform(0.0, 1.0, size=(B, 1))).astype(np.uint8)
    mask[3] = 0
    mask[B - 1] = 1
    td = torch.bfloat16
    packed = torch.zeros(cap, 3 * C, dtype=td, device="cuda")
    cu = torch.empty(B + 1, dtype=torch.int32, device="cuda")
    gidx = torch.zeros(cap, dtype=torch.int32, device="cuda")
    inv = torch.empty(cap, dtype=torch.int32, device="cuda")
    spa.spa_pack(dev(qkv, "bf16"), dev(mask), None, None, 0, packed, cu, gidx, inv, None)
    pq, pk, pv = packed[:, :C], packed[:, C:2 * C], packed[:, 2 * C:]
    out1 = torch.zeros(cap, C, dtype=td, device="cuda")
    y1 = torch.full((B, N, C), float("nan"), dtype=td, device="cuda")
    y2 = torch.full((B, N, C), float("nan"), dtype=td, device="cuda")
    spa.spa_packed_attention(pq, pk, pv, cu, B, N, H, Dh, out1, None)
    spa.spa_unpack(out1, inv, None, y1)
    spa.spa_packed_attention_unpack(pq, pk, pv, cu, gidx, inv, None, H, Dh, y2, None, None)
    torch.cuda.synchronize()
    assert np.array_equal(host(y1), host(y2))
    ref_out, _ = orc.attention_per_image(qkv[..., :C], qkv[..., C:2 * C], qkv[..., 2 * C:], mask, H)
    T = int(mask.sum())
    assert np.max(np.abs(host(out1)[:T] - ref_out)) <= TOL["bf16"]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("B,N,C,C2,dens,use_counts", [(3, 100, 64, 32, 0.5, False), (64, 196, 768, 384, 0.5, False),
                                                     (2, 777, 96, 48, 0.9, True), (5, 33, 16, 200, 0.0, False),
                                                     (4, 257, 128, 64, 1.0, True)])
def test_pack_pair_equals_two_packs(spa, dtype, B, N, C, C2, dens, use_counts):
    """spa_pack_pair against spa_pack(x) + spa_pack(x2, gate-scaled): every output bit for bit."""
    rng = np.random.default_rng(5)
    mk = wlmod.round_bf16 if dtype == "bf16" else (lambda a: a)
    td = tdtype(dtype)
    x = dev(mk(rng.standard_normal((B, N, C)).astype(np.float32)), dtype)
    x2 = dev(mk(rng.standard_normal((B, N, C2)).astype(np.float32)), dtype)
    scores = dev(rng.standard_normal((B, N)).astype(np.float32))
    mask_h = (rng.uniform(size=(B, N)) < dens).astype(np.uint8)
    mask = dev(mask_h)
    counts = dev(mask_h.sum(1).astype(np.int32)) if use_counts else None
    cap = B * N

    def bufs():
        return (torch.full((cap, C), float("nan"), dtype=td, device="cuda"),
                torch.full((cap, C2), float("nan"), dtype=td, device="cuda"),
                torch.full((B + 1,), -5, dtype=torch.int32, device="cuda"), torch.full((cap,), -5, dtype=torch.int32, device="cuda"),
                torch.full((cap,), -5, dtype=torch.int32, device="cuda"), torch.full((1,), -5, dtype=torch.int32, device="cuda"))

    pa, pb, cu, gi, inv, tot = bufs()
    spa.spa_pack(x, mask, counts, None, 0, pa, cu, gi, inv, tot)
    spa.spa_pack(x2, mask, counts, scores, 0, pb, None, None, None, None)
    qa, qb, cu2, gi2, inv2, tot2 = bufs()
    spa.spa_pack_pair(x, x2, mask, counts, scores, qa, qb, cu2, gi2, inv2, tot2)
    torch.cuda.synchronize()
    T = int(tot.item())
    assert T == int(mask_h.sum()) == int(tot2.item())
    assert torch.equal(cu, cu2) and torch.equal(inv, inv2) and torch.equal(gi[:T], gi2[:T])
    eq = lambda a, b: torch.equal(a[:T].view(torch.uint8), b[:T].view(torch.uint8))
    assert eq(pa, qa) and eq(pb, qb)
    assert torch.isnan(qa[T:]).all() and torch.isnan(qb[T:]).all()       # rows past the total untouched


@pytest.mark.parametrize("dtype,Dh,N,B", [("bf16", 64, 196, 5), ("bf16", 32, 49, 9), ("bf16", 32, 256, 3), ("bf16", 64, 100, 70),
                                          ("bf16", 32, 7, 4), ("f32", 32, 196, 3), ("f32", 64, 77, 4), ("f32", 32, 256, 3)])
@pytest.mark.parametrize("with_base", [False, True])
def test_selected_attention_from_the_mask_equals_the_indexed_form(spa, dtype, Dh, N, B, with_base):
    """spa_selected_attention_unpack (no packing launch: every wave derives its image's packing order from
    the mask bytes) == index-only spa_pack + spa_gathered_attention_unpack, bit for bit, and both equal the
    oracle; images with nothing and with everything selected included."""
    H = 2
    C = H * Dh
    rng = np.random.default_rng(500 + N + B)
    mk = wlmod.round_bf16 if dtype == "bf16" else (lambda a: a)
    qkv = mk(rng.standard_normal((B, N, 3 * C)).astype(np.float32))
    base = mk(rng.standard_normal((B, N, C)).astype(np.float32)) if with_base else None
    mask = (rng.uniform(size=(B, N)) < rng.uniform(0.05, 0.95, size=(B, 1))).astype(np.uint8)
    mask[1] = 0
    mask[2] = 1
    cap = B * N
    qkv_d, mask_d = dev(qkv, dtype), dev(mask)
    base_d = None if base is None else dev(base, dtype)
    flat = qkv_d.view(cap, 3 * C)
    ints = lambda n: torch.full((n,), -9, dtype=torch.int32, device="cuda")
    cu, gidx, inv, tot = ints(B + 1), ints(cap), ints(cap), ints(1)
    spa.spa_pack(None, mask_d, None, None, 0, None, cu, gidx, inv, tot)
    y1 = torch.full((B, N, C), float("nan"), dtype=tdtype(dtype), device="cuda")
    y2 = torch.full((B, N, C), float("nan"), dtype=tdtype(dtype), device="cuda")
    spa.spa_gathered_attention_unpack(flat[:, :C], flat[:, C:2 * C], flat[:, 2 * C:], cu, gidx, inv, base_d, H, Dh, y1)
    spa.spa_selected_attention_unpack(flat[:, :C], flat[:, C:2 * C], flat[:, 2 * C:], mask_d, base_d, H, Dh, y2)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)
    ref_out, _ = orc.attention_per_image(qkv[..., :C], qkv[..., C:2 * C], qkv[..., 2 * C:], mask, H)
    _, _, inv_r, _ = orc.pack_indices(mask)
    ref_y = orc.unpack(ref_out, inv_r, B, N, base)
    assert np.max(np.abs(host(y2) - ref_y)) <= (2 * TOL[dtype] if with_base and dtype == "bf16" else TOL[dtype])


def test_selected_attention_refuses_what_it_does_not_cover(spa):
    B, N, H, Dh = 2, 300, 2, 32
    C = H * Dh
    qkv = torch.zeros(B * N, 3 * C, dtype=torch.bfloat16, device="cuda")
    mask = torch.ones(B, N, dtype=torch.uint8, device="cuda")
    y = torch.empty(B, N, C, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(spa.SpaError):                      # more than 256 tokens per image
        spa.spa_selected_attention_unpack(qkv[:, :C], qkv[:, C:2 * C], qkv[:, 2 * C:], mask, None, H, Dh, y)
