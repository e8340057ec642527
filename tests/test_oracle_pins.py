"""Pins for the CPU oracle: each function is checked against something other than itself —
closed forms, library routines on special cases, brute force on tiny inputs, invariants
the paper fixes (Section 3.2), finite differences.  No GPU needed."""
import math

import numpy as np
import pytest
import scipy.special

from oracle import spa_oracle as orc
from paper_2410_23608_amd import workloads as wlmod


def rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------------------ gate
def test_gate_unit_rows_closed_form():
    C = 16
    w = rng(0).standard_normal(C)
    x = np.eye(C)[None]                       # token c is the unit vector e_c
    s = orc.gate_scores(x, w, 0.25)
    np.testing.assert_allclose(s[0], w + 0.25, rtol=0, atol=1e-15)


def test_gate_zero_weight_gives_bias():
    x = rng(1).standard_normal((2, 5, 8))
    s = orc.gate_scores(x, np.zeros(8), -1.5)
    assert np.all(s == -1.5)


def test_gate_matches_library_matvec():
    x = rng(2).standard_normal((3, 7, 33))
    w = rng(3).standard_normal(33)
    np.testing.assert_allclose(orc.gate_scores(x, w, 0.1), x @ w + 0.1, rtol=1e-13, atol=1e-13)


def test_gate_max_with_upscale_scores_is_monotone():
    # Eq. s = Max(f_g(r), s_up): adding s_up can only raise scores / add selected tokens
    x = rng(4).standard_normal((2, 9, 8))
    w = rng(5).standard_normal(8)
    s0 = orc.gate_scores(x, w, 0.0)
    s_up = rng(6).standard_normal((2, 9))
    s1 = orc.gate_scores(x, w, 0.0, s_up)
    assert np.all(s1 >= s0) and np.all(s1 >= s_up)
    assert np.all((s1 == s0) | (s1 == s_up))
    m0, _ = orc.select(s0, 0.5)
    m1, _ = orc.select(s1, 0.5)
    assert np.all(m1 >= m0)
    assert np.all(m1[s_up > 0] == 1)


@pytest.mark.parametrize("name", ["tiny", "vit_s", "det"])
def test_planted_logits_and_mask_recovered(name):
    wl = wlmod.WORKLOADS[name]
    if name != "tiny":
        wl = wlmod.replace(wl, B=2)
    bun = wlmod.generate(wl, seed=3, with_qkv=False)
    s = orc.gate_scores(bun["x"], bun["w"], bun["bias"])
    # the generator plants the logit; storage rounding moves it only slightly
    tol = 1e-4 if wl.dtype == "f32" else 0.06
    assert np.max(np.abs(s - bun["planted_logit"])) < tol
    mask, margin = orc.select(s, wl.tau)
    assert margin > 0.4
    assert np.array_equal(mask, bun["planted_mask"])
    # select ratio = selected / total (the paper's definition) equals the planted ratio
    assert mask.mean() == bun["planted_mask"].mean()


def test_select_threshold_and_strict_tie():
    theta = orc.threshold_logit(0.01)
    assert math.isclose(1.0 / (1.0 + math.exp(-theta)), 0.01, rel_tol=1e-12)
    assert orc.threshold_logit(0.5) == 0.0
    s = np.array([[0.0, 1e-300, -1e-300, 5.0, -5.0]])
    mask, margin = orc.select(s, 0.5)
    assert mask.tolist() == [[0, 1, 0, 1, 0]] and margin == 0.0
    # decision agrees with the sigmoid form wherever it is not a rounding tie
    s = rng(7).standard_normal((4, 50)) * 3
    for tau in (0.01, 0.3, 0.5, 0.9):
        mask, _ = orc.select(s, tau)
        assert np.array_equal(mask, (scipy.special.expit(s) > tau).astype(np.uint8))


def test_maxpool_matches_reshape_max():
    s = rng(8).standard_normal((3, 8 * 6))
    ref = s.reshape(3, 4, 2, 3, 2).max(axis=(2, 4)).reshape(3, -1)
    assert np.array_equal(orc.maxpool2x2(s, 8, 6), ref)


def test_sigmoid_matches_library():
    s = np.array([-800.0, -30.0, -1.0, 0.0, 1.0, 30.0, 800.0])
    np.testing.assert_allclose(orc.sigmoid(s), scipy.special.expit(s), rtol=1e-15, atol=0)


def test_round_to_bf16_known_values():
    # 1 + 2^-8 is a tie between 1.0 and 1+2^-7 -> even (1.0); 1 + 3*2^-8 ties up to 1+2^-6
    vals = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 3 * 2.0 ** -8, -2.5, 0.0])
    want = np.array([1.0, 1.0, 1.0 + 2.0 ** -7, 1.0 + 2.0 ** -6, -2.5, 0.0])
    assert np.array_equal(orc.round_to_dtype(vals, "bf16"), want)
    # agrees with the input generator's own, separately written rounding
    a = rng(9).standard_normal(10000).astype(np.float32)
    assert np.array_equal(orc.round_to_dtype(a, "bf16"), wlmod.round_bf16(a).astype(np.float64))
    # and with torch's bf16 cast
    import torch
    t = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(orc.round_to_dtype(a, "bf16"), t.astype(np.float64))


# ------------------------------------------------------------------------------ pack
def _random_mask(seed, B, N, p=0.4):
    m = (rng(seed).uniform(size=(B, N)) < p).astype(np.uint8)
    return m


def test_pack_indices_equal_flatnonzero_and_invariants():
    B, N = 5, 37
    mask = _random_mask(10, B, N)
    mask[2] = 0                                             # an empty image
    mask[3] = 1                                             # a full image
    cu, gidx, inv, T = orc.pack_indices(mask)
    assert np.array_equal(gidx, np.flatnonzero(mask.reshape(-1)).astype(np.int32))
    assert cu[0] == 0 and cu[-1] == T == mask.sum()
    assert np.array_equal(np.diff(cu), mask.sum(axis=1))
    assert np.all(np.diff(gidx) > 0)
    for b in range(B):
        seg = gidx[cu[b]:cu[b + 1]]
        assert np.all((seg >= b * N) & (seg < (b + 1) * N))
    assert np.array_equal(inv[gidx], np.arange(T))
    assert np.array_equal(inv == -1, mask.reshape(-1) == 0)


def test_pack_all_and_none_selected():
    cu, gidx, inv, T = orc.pack_indices(np.zeros((3, 4), np.uint8))
    assert T == 0 and len(gidx) == 0 and np.all(cu == 0) and np.all(inv == -1)
    cu, gidx, inv, T = orc.pack_indices(np.ones((3, 4), np.uint8))
    assert T == 12 and np.array_equal(gidx, np.arange(12)) and np.array_equal(cu, [0, 4, 8, 12])


def test_pack_container_padding():
    # B' = ceil(T / L); only the last container is padded, with zeros
    B, N, C, L = 3, 20, 4, 7
    mask = _random_mask(11, B, N)
    x = rng(12).standard_normal((B, N, C))
    cu, gidx, inv, T = orc.pack_indices(mask)
    p = orc.pack_rows(x, gidx, None, L)
    assert p.shape[0] == math.ceil(T / L) * L and p.shape[0] - T < L
    assert np.all(p[T:] == 0)
    assert np.array_equal(p[:T], x.reshape(-1, C)[np.flatnonzero(mask.reshape(-1))])
    assert orc.packed_rows(0, 7) == 0 and orc.packed_rows(14, 7) == 14 and orc.packed_rows(15, 7) == 21


def test_unpack_of_pack_is_identity_on_selected():
    B, N, C = 4, 23, 6
    mask = _random_mask(13, B, N)
    x = rng(14).standard_normal((B, N, C))
    cu, gidx, inv, T = orc.pack_indices(mask)
    y = orc.unpack(orc.pack_rows(x, gidx), inv, B, N)
    sel = mask.astype(bool)
    assert np.array_equal(y[sel], x[sel])
    assert np.all(y[~sel] == 0)
    base = rng(15).standard_normal((B, N, C))
    y2 = orc.unpack(orc.pack_rows(x, gidx), inv, B, N, base)
    assert np.array_equal(y2[~sel], base[~sel])
    np.testing.assert_allclose(y2[sel], base[sel] + x[sel], rtol=0, atol=0)


def test_pack_gate_scaling():
    # Eq. r_g = Sigmoid(s) . r
    B, N, C = 2, 9, 5
    mask = _random_mask(16, B, N, 0.6)
    x = rng(17).standard_normal((B, N, C))
    s = rng(18).standard_normal((B, N))
    cu, gidx, inv, T = orc.pack_indices(mask)
    p = orc.pack_rows(x, gidx, s)
    ref = (scipy.special.expit(s)[:, :, None] * x).reshape(-1, C)[gidx]
    np.testing.assert_allclose(p, ref, rtol=1e-15, atol=0)


# ------------------------------------------------------------------------- attention
def _full_msa_library(q, k, v, H):
    """Ordinary multi-head self-attention via einsum + scipy softmax (textbook routine)."""
    B, N, C = q.shape
    Dh = C // H
    qh, kh, vh = (t.reshape(B, N, H, Dh) for t in (q, k, v))
    S = np.einsum("bnhd,bmhd->bhnm", qh, kh) / math.sqrt(Dh)
    P = scipy.special.softmax(S, axis=-1)
    O = np.einsum("bhnm,bmhd->bnhd", P, vh).reshape(B, N, C)
    return O, scipy.special.logsumexp(S, axis=-1)          # lse [B,H,N]


def _qkv(seed, B, N, C):
    r = rng(seed)
    return r.standard_normal((B, N, C)), r.standard_normal((B, N, C)), r.standard_normal((B, N, C))


def test_attention_all_selected_equals_full_msa():
    B, N, C, H = 3, 19, 24, 3
    q, k, v = _qkv(20, B, N, C)
    out, lse = orc.attention_per_image(q, k, v, np.ones((B, N), np.uint8), H)
    ref, ref_lse = _full_msa_library(q, k, v, H)
    np.testing.assert_allclose(out.reshape(B, N, C), ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse.reshape(H, B, N).transpose(1, 0, 2), ref_lse, rtol=1e-12, atol=1e-13)


def test_attention_equals_per_image_dense_on_subset():
    # packed result == dense attention run separately on each image's selected subset
    B, N, C, H = 4, 17, 16, 2
    q, k, v = _qkv(21, B, N, C)
    mask = _random_mask(22, B, N, 0.5)
    mask[1] = 0
    out, lse = orc.attention_per_image(q, k, v, mask, H)
    cu, gidx, inv, T = orc.pack_indices(mask)
    for b in range(B):
        sel = np.flatnonzero(mask[b])
        if len(sel) == 0:
            continue
        ref, ref_lse = _full_msa_library(q[b:b + 1, sel], k[b:b + 1, sel], v[b:b + 1, sel], H)
        np.testing.assert_allclose(out[cu[b]:cu[b + 1]], ref[0], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(lse[:, cu[b]:cu[b + 1]], ref_lse[0], rtol=1e-12, atol=1e-13)


def test_attention_brute_force_tiny():
    B, N, C, H = 2, 6, 4, 2
    Dh = C // H
    q, k, v = _qkv(23, B, N, C)
    mask = np.array([[1, 0, 1, 1, 0, 1], [0, 1, 1, 0, 0, 0]], np.uint8)
    out, lse = orc.attention_per_image(q, k, v, mask, H)
    j = 0
    for b in range(B):
        sel = [n for n in range(N) if mask[b, n]]
        for n in sel:
            for h in range(H):
                sc = [sum(q[b, n, h * Dh + d] * k[b, m, h * Dh + d] for d in range(Dh)) / math.sqrt(Dh)
                      for m in sel]
                z = sum(math.exp(t) for t in sc)
                for d in range(Dh):
                    o = sum(math.exp(t) / z * v[b, m, h * Dh + d] for t, m in zip(sc, sel))
                    assert abs(out[j, h * Dh + d] - o) < 1e-13
                assert abs(lse[h, j] - math.log(z)) < 1e-13
            j += 1
    assert j == out.shape[0]


def test_attention_special_cases():
    B, N, C, H = 2, 11, 8, 2
    q, k, v = _qkv(24, B, N, C)
    # single selected token: O = v of that token, lse = its own score
    mask = np.zeros((B, N), np.uint8)
    mask[0, 4] = 1
    mask[1, 9] = 1
    out, lse = orc.attention_per_image(q, k, v, mask, H)
    np.testing.assert_allclose(out[0], v[0, 4], rtol=1e-15)
    np.testing.assert_allclose(out[1], v[1, 9], rtol=1e-15)
    Dh = C // H
    assert abs(lse[1, 0] - q[0, 4, Dh:] @ k[0, 4, Dh:] / math.sqrt(Dh)) < 1e-13
    # q = 0: uniform weights -> mean of the segment's v rows, lse = ln n_b
    mask = _random_mask(25, B, N, 0.6)
    out, lse = orc.attention_per_image(np.zeros_like(q), k, v, mask, H)
    cu, _, _, _ = orc.pack_indices(mask)
    for b in range(B):
        sel = np.flatnonzero(mask[b])
        np.testing.assert_allclose(out[cu[b]:cu[b + 1]], np.tile(v[b, sel].mean(0), (len(sel), 1)), rtol=1e-13)
        np.testing.assert_allclose(lse[:, cu[b]:cu[b + 1]], math.log(len(sel)), rtol=1e-13)
    # v = 1: O = 1
    out, _ = orc.attention_per_image(q, k, np.ones_like(v), mask, H)
    np.testing.assert_allclose(out, 1.0, rtol=1e-14)


def test_attention_permutation_equivariance_and_no_leakage():
    B, N, C, H = 3, 13, 8, 2
    q, k, v = _qkv(26, B, N, C)
    mask = _random_mask(27, B, N, 0.6)
    out, _ = orc.attention_per_image(q, k, v, mask, H)
    cu, gidx, inv, T = orc.pack_indices(mask)
    # permute tokens of image 1 (and its mask): outputs permute with them
    perm = rng(28).permutation(N)
    q2, k2, v2, m2 = q.copy(), k.copy(), v.copy(), mask.copy()
    q2[1], k2[1], v2[1], m2[1] = q[1, perm], k[1, perm], v[1, perm], mask[1, perm]
    out2, _ = orc.attention_per_image(q2, k2, v2, m2, H)
    y = orc.unpack(out, inv, B, N)
    _, _, inv2, _ = orc.pack_indices(m2)
    y2 = orc.unpack(out2, inv2, B, N)
    np.testing.assert_allclose(y2[1], y[1, perm], rtol=1e-12, atol=1e-13)
    # poison another image and every unselected token: image 0's outputs are bit-identical
    q3, k3, v3 = q.copy(), k.copy(), v.copy()
    for t in (q3, k3, v3):
        t[1:] = 1e30
        t[0, mask[0] == 0] = -1e30
    out3, _ = orc.attention_per_image(q3, k3, v3, mask, H)
    assert np.array_equal(out3[cu[0]:cu[1]], out[cu[0]:cu[1]])


# -------------------------------------------------------------------------- backward
def _fd(f, a, h=1e-6):
    g = np.zeros_like(a)
    it = np.nditer(a, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = a[i]
        a[i] = old + h
        fp = f()
        a[i] = old - h
        fm = f()
        a[i] = old
        g[i] = (fp - fm) / (2 * h)
    return g


def test_attention_backward_finite_differences():
    B, N, C, H = 2, 5, 4, 2
    q, k, v = _qkv(30, B, N, C)
    mask = np.array([[1, 1, 0, 1, 0], [0, 1, 0, 1, 1]], np.uint8)
    cu, gidx, inv, T = orc.pack_indices(mask)
    dO = rng(31).standard_normal((T, C))

    def loss():
        out, _ = orc.attention_per_image(q, k, v, mask, H)
        return float((out * dO).sum())

    dq, dk, dv = orc.attention_backward_per_image(q, k, v, mask, dO, H)
    for arr, grad in ((q, dq), (k, dk), (v, dv)):
        fd = _fd(loss, arr).reshape(B * N, C)
        np.testing.assert_allclose(grad, fd[gidx], rtol=1e-6, atol=1e-8)
        unsel = np.setdiff1d(np.arange(B * N), gidx)
        assert np.all(np.abs(fd[unsel]) < 1e-9)          # unselected tokens get no gradient


def test_attention_backward_identities():
    B, N, C, H = 2, 9, 8, 2
    q, k, v = _qkv(32, B, N, C)
    mask = _random_mask(33, B, N, 0.7)
    T = int(mask.sum())
    dO = rng(34).standard_normal((T, C))
    # v constant within each head column => O does not depend on q, k => dq = dk = 0
    vc = np.tile(rng(35).standard_normal((1, 1, C)), (B, N, 1))
    dq, dk, dv = orc.attention_backward_per_image(q, k, vc, mask, dO, H)
    assert np.max(np.abs(dq)) < 1e-13 and np.max(np.abs(dk)) < 1e-13
    # sum over a segment of dV equals the segment sum of dO (columns of P sum... rows of P sum to 1)
    dq, dk, dv = orc.attention_backward_per_image(q, k, v, mask, dO, H)
    cu, _, _, _ = orc.pack_indices(mask)
    for b in range(B):
        np.testing.assert_allclose(dv[cu[b]:cu[b + 1]].sum(0), dO[cu[b]:cu[b + 1]].sum(0), rtol=1e-12, atol=1e-12)


def test_selection_loss_closed_forms():
    # s = 0 => ln 2 per token regardless of the label
    y = np.array([[0, 1, 1, 0]], np.uint8)
    assert math.isclose(orc.selection_loss(np.zeros((1, 4)), y, 1.0), 4 * math.log(2), rel_tol=1e-14)
    # equals -(y log p + (1-y) log(1-p)) written with the library sigmoid
    s = rng(36).standard_normal((3, 8)) * 4
    y = (rng(37).uniform(size=(3, 8)) < 0.5).astype(np.uint8)
    p = scipy.special.expit(s)
    ref = -(y * np.log(p) + (1 - y) * np.log1p(-p)).sum()
    assert math.isclose(orc.selection_loss(s, y, 0.01), 0.01 * ref, rel_tol=1e-12)
    # stable at extreme logits
    assert math.isclose(orc.selection_loss(np.array([[800.0, -800.0]]), np.array([[0, 1]]), 1.0), 1600.0)


@pytest.mark.parametrize("with_up,scaled", [(False, False), (False, True), (True, True)])
def test_gate_backward_finite_differences(with_up, scaled):
    B, N, C = 2, 4, 3
    r = rng(40)
    x = r.standard_normal((B, N, C))
    w = r.standard_normal(C)
    bias = np.array([0.3])
    s_up = r.standard_normal((B, N)) if with_up else None
    y = (r.uniform(size=(B, N)) < 0.5).astype(np.uint8)
    d_rg = r.standard_normal((B, N, C))
    lam = 0.7

    def loss():
        s = orc.gate_scores(x, w, bias[0], s_up)
        L = orc.selection_loss(s, y, lam)
        if scaled:
            L += float((orc.sigmoid(s)[:, :, None] * x * d_rg).sum())
        return L

    g = orc.gate_backward(x, w, bias[0], s_up, y, d_rg, scaled, lam)
    np.testing.assert_allclose(g["dx"], _fd(loss, x), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(g["dw"], _fd(loss, w), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(g["db"], _fd(loss, bias)[0], rtol=1e-6, atol=1e-8)
    assert math.isclose(g["loss"], orc.selection_loss(orc.gate_scores(x, w, bias[0], s_up), y, lam))
    if with_up:
        s = orc.gate_scores(x, w, bias[0], s_up)
        assert (s == s_up).any() and (s != s_up).any()      # both branches of the max exercised
    if not scaled:
        # dL/ds = lam * (sigmoid(s) - y), and dw = X^T ds via the library
        s = orc.gate_scores(x, w, bias[0], s_up)
        np.testing.assert_allclose(g["ds"], lam * (scipy.special.expit(s) - y), rtol=1e-13)
        np.testing.assert_allclose(g["dw"], x.reshape(-1, C).T @ g["ds"].reshape(-1), rtol=1e-12)


# ------------------------------------------------------------------------ whole path
def test_forward_path_on_tiny_workload():
    wl = wlmod.WORKLOADS["tiny"]
    bun = wlmod.generate(wl, seed=0)
    r = orc.spa_forward(bun["x"], bun["w"], bun["bias"], bun["qkv"], wl.H, wl.tau, wl.dtype)
    frac = r["mask"].mean(axis=1)
    assert np.all((frac > 0.15) & (frac < 0.45))
    assert np.array_equal(r["mask"], bun["planted_mask"])
    C = wl.C
    q, k, v = bun["qkv"][..., :C], bun["qkv"][..., C:2 * C], bun["qkv"][..., 2 * C:]
    for b in range(wl.B):
        sel = np.flatnonzero(r["mask"][b])
        ref, _ = _full_msa_library(q[b:b + 1, sel].astype(np.float64), k[b:b + 1, sel].astype(np.float64),
                                   v[b:b + 1, sel].astype(np.float64), wl.H)
        np.testing.assert_allclose(r["y"][b, sel], ref[0], rtol=1e-12, atol=1e-13)
        unsel = np.flatnonzero(r["mask"][b] == 0)
        assert np.all(r["y"][b, unsel] == 0)


def test_linear_packed_matches_library_and_bruteforce():
    B, N, K, No = 2, 7, 5, 3
    r = rng(50)
    x = r.standard_normal((B, N, K))
    W = r.standard_normal((No, K))
    bias = r.standard_normal(No)
    s = r.standard_normal((B, N))
    mask = _random_mask(51, B, N, 0.6)
    cu, gidx, inv, T = orc.pack_indices(mask)
    y = orc.linear_packed(x, gidx, W, bias, s)
    ref = (scipy.special.expit(s)[:, :, None] * x).reshape(-1, K)[gidx] @ W.T + bias
    np.testing.assert_allclose(y, ref, rtol=1e-13, atol=1e-13)
    # brute force, no gate scaling, no bias
    y0 = orc.linear_packed(x, gidx, W)
    for j in range(T):
        for n in range(No):
            acc = sum(x.reshape(-1, K)[gidx[j], c] * W[n, c] for c in range(K))
            assert abs(y0[j, n] - acc) < 1e-13
    # identity weights return the packed rows themselves
    np.testing.assert_array_equal(orc.linear_packed(x, gidx, np.eye(K)), x.reshape(-1, K)[gidx])


def test_linear_packed_backward_matches_finite_differences_and_bruteforce():
    """The projection is linear in W, bias and the rows, so central differences of the scalar
    L = sum_j <g_j, out_j> through linear_packed (the forward oracle) are exact up to rounding;
    with scores, the chain through r_g = Sigmoid(s) . r fixes what d_rows is the gradient of."""
    B, N, K, No = 2, 6, 5, 3
    r = rng(60)
    x = r.standard_normal((B, N, K))
    W = r.standard_normal((No, K))
    bias = r.standard_normal(No)
    s = r.standard_normal((B, N))
    mask = _random_mask(61, B, N, 0.6)
    cu, gidx, inv, T = orc.pack_indices(mask)
    assert 2 <= T < B * N
    dy = r.standard_normal((B * N, No))           # upstream gradient at token positions
    didx = gidx[::-1].copy()                      # row j of the gradient is dy[didx[j]] (any index map)
    g = dy[didx]
    eps = 1e-6

    def L(x_=x, W_=W, b_=bias, s_=None):
        return float((g * orc.linear_packed(x_, gidx, W_, b_, s_)).sum())

    for scores in (None, s):
        bw = orc.linear_packed_backward(dy, x, gidx, W, scores, didx)
        for n in range(No):
            e = np.zeros(No); e[n] = eps
            assert abs((L(b_=bias + e, s_=scores) - L(b_=bias - e, s_=scores)) / (2 * eps) - bw["dbias"][n]) < 1e-8
            for c in range(K):
                E = np.zeros((No, K)); E[n, c] = eps
                fd = (L(W_=W + E, s_=scores) - L(W_=W - E, s_=scores)) / (2 * eps)
                assert abs(fd - bw["dW"][n, c]) < 1e-8
        p = scipy.special.expit(s).reshape(-1)
        for j in range(T):
            tok = gidx[j]
            scale = 1.0 if scores is None else p[tok]
            for c in range(K):
                E = np.zeros((B * N, K)); E[tok, c] = eps
                fd = (L(x_=(x.reshape(-1, K) + E).reshape(B, N, K), s_=scores) -
                      L(x_=(x.reshape(-1, K) - E).reshape(B, N, K), s_=scores)) / (2 * eps)
                assert abs(fd - scale * bw["d_rows"][j, c]) < 1e-8           # dL/dx = Sigmoid(s) dL/dr_g
            if scores is not None:
                E = np.zeros(B * N); E[tok] = eps
                fd = (L(s_=(s.reshape(-1) + E).reshape(B, N)) - L(s_=(s.reshape(-1) - E).reshape(B, N))) / (2 * eps)
                assert abs(fd - p[tok] * (1 - p[tok]) * float(bw["d_rows"][j] @ x.reshape(-1, K)[tok])) < 1e-8
    # brute force with explicit loops, no scores, rows of dout taken in order
    bw = orc.linear_packed_backward(dy, x, gidx, W)
    xf = x.reshape(-1, K)
    for n in range(No):
        assert abs(bw["dbias"][n] - sum(dy[j, n] for j in range(T))) < 1e-13
        for c in range(K):
            assert abs(bw["dW"][n, c] - sum(dy[j, n] * xf[gidx[j], c] for j in range(T))) < 1e-12
    for j in range(T):
        for c in range(K):
            assert abs(bw["d_rows"][j, c] - sum(dy[j, n] * W[n, c] for n in range(No))) < 1e-12
    # identity weights hand the gradient through unchanged
    dyk = r.standard_normal((B * N, K))
    np.testing.assert_array_equal(orc.linear_packed_backward(dyk, x, gidx, np.eye(K))["d_rows"], dyk[:T])


# ------------------------------------------------ cyclic shift and container-local attention
def test_shift_order_is_a_roll_of_the_index_grid():
    """The shifted map's raster order equals numpy's roll of the position grid by (-sh, -sw)
    (the torch.roll convention of the Swin window shift), and zero shift is the identity."""
    for (gh, gw, sh, sw) in [(3, 4, 1, 1), (7, 7, 3, 3), (5, 9, 0, 4), (6, 2, 5, 1), (4, 4, 0, 0)]:
        grid = np.arange(gh * gw).reshape(gh, gw)
        ref = np.roll(grid, shift=(-sh, -sw), axis=(0, 1)).ravel()
        assert np.array_equal(orc.shift_order(gh, gw, sh, sw), ref)
    assert np.array_equal(orc.shift_order(4, 5, 0, 0), np.arange(20))
    # a shift by the full extent is the identity again
    assert np.array_equal(orc.shift_order(4, 5, 4, 5), np.arange(20))


def test_shifted_pack_indices_invariants():
    rng = np.random.default_rng(3)
    gh, gw, B = 6, 5, 4
    mask = (rng.random((B, gh * gw)) < 0.4).astype(np.uint8)
    order = orc.shift_order(gh, gw, 2, 3)
    cu, gidx, inv, T = orc.pack_indices(mask, order)
    cu0, gidx0, inv0, T0 = orc.pack_indices(mask)
    assert T == T0 and np.array_equal(cu, cu0)                    # a shift moves nothing between images
    assert sorted(gidx.tolist()) == sorted(gidx0.tolist())        # same tokens, other order
    assert np.array_equal(inv[gidx], np.arange(T))
    # inside an image the packed order is the order of the rolled map
    rank_in_rolled = np.empty(gh * gw, dtype=np.int64)
    rank_in_rolled[order] = np.arange(gh * gw)
    for b in range(B):
        seg = gidx[cu[b]:cu[b + 1]] - b * gh * gw
        assert np.all(np.diff(rank_in_rolled[seg]) > 0)
    # rolling the mask itself and packing without an order selects the same tokens in the same sequence
    rolled = np.stack([np.roll(m.reshape(gh, gw), shift=(-2, -3), axis=(0, 1)).ravel() for m in mask])
    _, g_rolled, _, _ = orc.pack_indices(rolled)
    for b in range(B):
        pos_rolled = g_rolled[cu[b]:cu[b + 1]] - b * gh * gw
        assert np.array_equal(order[pos_rolled], gidx[cu[b]:cu[b + 1]] - b * gh * gw)


def test_container_segments_examples_and_invariants():
    # worked example: images of 5, 0, 7 and 8 tokens, containers of 7
    assert orc.container_segments(np.array([0, 5, 5, 12, 20]), 7).tolist() == [0, 5, 7, 12, 14, 20]
    # containers at least as long as the stream change nothing but drop empty images
    assert orc.container_segments(np.array([0, 3, 3, 9]), 100).tolist() == [0, 3, 9]
    # L = 1: every token is its own segment
    assert orc.container_segments(np.array([0, 2, 4]), 1).tolist() == [0, 1, 2, 3, 4]
    rng = np.random.default_rng(0)
    for _ in range(20):
        lens = rng.integers(0, 30, size=6)
        cu = np.concatenate([[0], np.cumsum(lens)])
        L = int(rng.integers(1, 12))
        seg = orc.container_segments(cu, L)
        assert seg[0] == 0 and seg[-1] == cu[-1] and np.all(np.diff(seg) > 0) if cu[-1] > 0 else True
        for a, b in zip(seg[:-1], seg[1:]):
            assert b - a <= L and a // L == (b - 1) // L                                   # inside one container
            assert np.searchsorted(cu, a, side="right") == np.searchsorted(cu, b - 1, side="right")  # one image


def _packed_qkv(rng, T, C):
    return tuple(rng.standard_normal((T, C)) for _ in range(3))


def test_container_attention_reduces_to_per_image_attention():
    """With a container longer than the stream the mask is 'same image' alone, which the
    per-image oracle (written separately, on un-packed tensors) computes."""
    rng = np.random.default_rng(5)
    B, N, C, H = 3, 17, 16, 2
    mask = (rng.random((B, N)) < 0.6).astype(np.uint8)
    q, k, v = (rng.standard_normal((B, N, C)) for _ in range(3))
    cu, gidx, inv, T = orc.pack_indices(mask)
    flat = lambda a: a.reshape(B * N, C)[gidx]
    out, lse = orc.attention_container_local(flat(q), flat(k), flat(v), cu, 10 ** 6, H)
    ref, lse_ref = orc.attention_per_image(q, k, v, mask, H)
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(lse, lse_ref, rtol=1e-12, atol=1e-12)


def test_container_attention_equals_attention_on_each_piece():
    """Cutting the stream at the oracle's own segment boundaries and running plain softmax
    attention (scipy) on each piece gives the same rows; L = 1 returns v itself."""
    rng = np.random.default_rng(6)
    C, H, L = 8, 2, 5
    cu = np.array([0, 7, 7, 18, 21])
    T, Dh = int(cu[-1]), C // H
    qp, kp, vp = _packed_qkv(rng, T, C)
    out, lse = orc.attention_container_local(qp, kp, vp, cu, L, H)
    seg = orc.container_segments(cu, L)
    for a, b in zip(seg[:-1], seg[1:]):
        for h in range(H):
            sl = slice(h * Dh, (h + 1) * Dh)
            S = qp[a:b, sl] @ kp[a:b, sl].T / math.sqrt(Dh)
            P = scipy.special.softmax(S, axis=1)
            np.testing.assert_allclose(out[a:b, sl], P @ vp[a:b, sl], rtol=1e-12, atol=1e-12)
            np.testing.assert_allclose(lse[h, a:b], scipy.special.logsumexp(S, axis=1), rtol=1e-12, atol=1e-12)
    out1, lse1 = orc.attention_container_local(qp, kp, vp, cu, 1, H)
    np.testing.assert_allclose(out1, vp, rtol=1e-13, atol=1e-13)
    for h in range(H):
        sl = slice(h * Dh, (h + 1) * Dh)
        np.testing.assert_allclose(lse1[h], (qp[:, sl] * kp[:, sl]).sum(1) / math.sqrt(Dh), rtol=1e-12, atol=1e-12)


def test_container_attention_no_leakage_across_containers_or_images():
    rng = np.random.default_rng(7)
    C, H, L = 8, 2, 4
    cu = np.array([0, 6, 13])
    T = 13
    qp, kp, vp = _packed_qkv(rng, T, C)
    out, _ = orc.attention_container_local(qp, kp, vp, cu, L, H)
    # rows 4..5 form the segment (image 0, container 1); changing k, v anywhere else leaves them unchanged
    k2, v2 = kp.copy(), vp.copy()
    others = np.r_[0:4, 6:13]
    k2[others] += rng.standard_normal((len(others), C))
    v2[others] += rng.standard_normal((len(others), C))
    out2, _ = orc.attention_container_local(qp, k2, v2, cu, L, H)
    np.testing.assert_array_equal(out2[4:6], out[4:6])
    assert not np.allclose(out2[0:4], out[0:4])


def test_container_attention_backward_finite_differences_and_reduction():
    rng = np.random.default_rng(8)
    C, H, L = 6, 2, 3
    cu = np.array([0, 4, 9])
    T = 9
    qp, kp, vp = _packed_qkv(rng, T, C)
    dout = rng.standard_normal((T, C))
    dq, dk, dv = orc.attention_container_local_backward(qp, kp, vp, cu, L, dout, H)
    f = lambda a, b, c: float((orc.attention_container_local(a, b, c, cu, L, H)[0] * dout).sum())
    eps = 1e-6
    for arr, grad, which in ((qp, dq, 0), (kp, dk, 1), (vp, dv, 2)):
        for idx in [(0, 0), (3, 5), (5, 2), (8, 1)]:
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += eps
            lo[idx] -= eps
            args_hi = [qp, kp, vp]
            args_lo = [qp, kp, vp]
            args_hi[which], args_lo[which] = hi, lo
            num = (f(*args_hi) - f(*args_lo)) / (2 * eps)
            assert abs(num - grad[idx]) <= 1e-6 * max(1.0, abs(num))
    # one long container: the per-image backward oracle on un-packed tensors
    B, N = 2, 7
    mask = (rng.random((B, N)) < 0.7).astype(np.uint8)
    q, k, v = (rng.standard_normal((B, N, C)) for _ in range(3))
    cu2, gidx, inv, T2 = orc.pack_indices(mask)
    flat = lambda a: a.reshape(B * N, C)[gidx]
    do2 = rng.standard_normal((T2, C))
    got = orc.attention_container_local_backward(flat(q), flat(k), flat(v), cu2, 10 ** 6, do2, H)
    ref = orc.attention_backward_per_image(q, k, v, mask, do2, H)
    for g, r in zip(got, ref):
        np.testing.assert_allclose(g, r, rtol=1e-11, atol=1e-12)


# ------------------------------------------------ stochastic selection, straight-through
def test_select_gumbel_reduces_to_select_without_noise():
    rng = np.random.default_rng(11)
    s = rng.standard_normal((3, 50)) * 3
    for tau in (0.5, 0.01, 0.9):
        m0, _ = orc.select(s, tau)
        m1, pt, _ = orc.select_gumbel(s, np.zeros_like(s), 1.0, tau)
        assert np.array_equal(m0, m1)
        np.testing.assert_allclose(pt, scipy.special.expit(s), rtol=1e-13)
        assert np.array_equal(m1, (pt > tau).astype(np.uint8))          # the decision is p~ > tau


def test_select_gumbel_is_the_two_class_gumbel_softmax():
    """p~ equals the first component of softmax(([s, 0] + [g1, g2]) / T) with Gumbel draws,
    and the frequency of selection under Logistic noise matches sigmoid(s - T logit(tau))."""
    rng = np.random.default_rng(12)
    s = rng.standard_normal((2, 40)) * 2
    g1, g2 = rng.gumbel(size=s.shape), rng.gumbel(size=s.shape)
    for T in (1.0, 0.5, 2.0):
        mask, pt, _ = orc.select_gumbel(s, g1 - g2, T, 0.3)
        logits = np.stack([s + g1, g2], axis=-1) / T
        ref = scipy.special.softmax(logits, axis=-1)[..., 0]
        np.testing.assert_allclose(pt, ref, rtol=1e-12, atol=1e-15)
        assert np.array_equal(mask, (ref > 0.3).astype(np.uint8))
    # selection frequency: P(s + e > T theta) = sigmoid(s - T theta) for e ~ Logistic(0, 1)
    n, T, tau = 200000, 0.7, 0.2
    for s0 in (-1.5, 0.0, 0.8):
        e = rng.logistic(size=n)
        mask, _, _ = orc.select_gumbel(np.full(n, s0), e, T, tau)
        p = scipy.special.expit(s0 - T * scipy.special.logit(tau))
        assert abs(mask.mean() - p) <= 5 * math.sqrt(p * (1 - p) / n)
    # a lower threshold selects a superset (the paper lowers the threshold to keep more tokens)
    e = rng.logistic(size=s.shape)
    m_lo, _, _ = orc.select_gumbel(s, e, 1.0, 0.01)
    m_hi, _, _ = orc.select_gumbel(s, e, 1.0, 0.5)
    assert np.all(m_lo >= m_hi) and m_lo.sum() > m_hi.sum()


def test_straight_through_term_is_the_derivative_of_the_relaxed_selection():
    """Replace the hard mask by the relaxed weight p~(s) in r_p = m . r_g and differentiate
    numerically with respect to the gate bias: the extra term of gate_backward (db with minus
    without the flag) equals that derivative restricted to the selected tokens."""
    rng = np.random.default_rng(13)
    B, N, C, T = 2, 9, 8, 0.6
    x = rng.standard_normal((B, N, C))
    w = rng.standard_normal(C) * 0.5
    bias = 0.1
    noise = rng.logistic(size=(B, N))
    up = rng.standard_normal((B, N, C))                         # d L / d r_p
    labels = (rng.random((B, N)) < 0.5).astype(np.uint8)
    s = orc.gate_scores(x, w, bias)
    mask, _, _ = orc.select_gumbel(s, noise, T, 0.4)
    d_rg = up * mask[:, :, None]                                # what pack_bwd hands over: zero rows where unselected
    with_st = orc.gate_backward(x, w, bias, None, labels, d_rg, True, 0.0, st_mask=mask, st_noise=noise, st_temperature=T)
    without = orc.gate_backward(x, w, bias, None, labels, d_rg, True, 0.0)

    def relaxed_only(b):                                        # sum_i m_i <up_i, p~_i(b) * r_g_i>, r_g held fixed
        sb = orc.gate_scores(x, w, b)
        pt = scipy.special.expit((sb + noise) / T)
        r_g = scipy.special.expit(s)[:, :, None] * x
        return float((mask[:, :, None] * up * pt[:, :, None] * r_g).sum())

    eps = 1e-6
    num = (relaxed_only(bias + eps) - relaxed_only(bias - eps)) / (2 * eps)
    assert abs((with_st["db"] - without["db"]) - num) <= 1e-6 * max(1.0, abs(num))
    # per token: the term vanishes where the mask is 0 and has the sign of <d_rg, r_g>
    extra = with_st["ds"] - without["ds"]
    assert np.all(extra[mask == 0] == 0)
    dots = (d_rg * scipy.special.expit(s)[:, :, None] * x).sum(axis=2)
    assert np.all(np.sign(extra[mask == 1]) == np.sign(dots[mask == 1]))
    # dw picks the same term up through ds
    np.testing.assert_allclose(with_st["dw"] - without["dw"], (extra[:, :, None] * x).sum(axis=(0, 1)), rtol=1e-10)


def test_attention_work_matches_the_papers_complexity_terms():
    """The score counts that the segment boundaries imply reproduce the attention terms of the
    paper's complexity formulas on the hand-evaluated example in tests/golden: container
    segments -> B' 2 L^2 C, all tokens selected with per-image segments -> B 2 N^2 C."""
    import os
    golden = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "complexity_worked_example.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                golden[k] = int(v)
    C, L = 64, 49
    cu = np.array([0, 98, 196])                      # two images with 98 selected tokens each: 4 full containers
    seg = orc.container_segments(cu, L)
    assert len(seg) - 1 == 4
    assert int((np.diff(seg).astype(np.int64) ** 2).sum()) * 2 * C == golden["spa_attention_macs"]
    mask = np.ones((2, 196), np.uint8)               # everything selected: ordinary self-attention per image
    cu_all, _, _, _ = orc.pack_indices(mask)
    assert int((np.diff(cu_all).astype(np.int64) ** 2).sum()) * 2 * C == golden["msa_attention_macs"]
    # bench.py's algorithmic flop count, 4 C sum n^2, is two flops per multiply-accumulate of these terms
    assert 4 * C * int((np.diff(cu_all).astype(np.int64) ** 2).sum()) == 2 * golden["msa_attention_macs"]


# ------------------------------------------------------------ the block with its projections
def test_block_chain_of_oracle_steps_matches_finite_differences():
    """The backward of a whole block, assembled from the oracle's steps in the order the GPU
    pipeline runs them (output projection -> attention -> QKV projection of the gated rows ->
    gate with the selection loss), against central differences of the block's forward value
    L = sum(dy * y) + loss_scale * BCE.  The hard mask is a constant (perturbations are far
    smaller than the selection margin).  Pins the composition itself: which gradient feeds which
    step, and that the gradient reaching x is dy (residual and bypass) plus the gate's dx."""
    B, N, C, H = 2, 6, 4, 2
    r = rng(70)
    x = r.standard_normal((B, N, C))
    w = r.standard_normal(C)
    bias = 0.1
    Wqkv, bqkv = r.standard_normal((3 * C, C)) / 2, r.standard_normal(3 * C) / 4
    Wo, bo = r.standard_normal((C, C)) / 2, r.standard_normal(C) / 4
    labels = (r.uniform(size=(B, N)) < 0.5).astype(np.uint8)
    dy = r.standard_normal((B, N, C))
    lam = 0.3
    s0 = orc.gate_scores(x, w, bias)
    mask, margin = orc.select(s0, 0.5)
    assert margin > 1e-3 and 2 <= mask.sum() < B * N
    cu, gidx, inv, T = orc.pack_indices(mask)

    def forward(x_=x, w_=w, Wqkv_=Wqkv, bqkv_=bqkv, Wo_=Wo, bo_=bo):
        s = orc.gate_scores(x_, w_, bias)
        qkv = orc.unpack(orc.linear_packed(x_, gidx, Wqkv_, bqkv_, s), inv, B, N)
        attn, _ = orc.attention_per_image(qkv[..., :C], qkv[..., C:2 * C], qkv[..., 2 * C:], mask, H)
        y = orc.unpack(orc.linear_packed(attn, np.arange(T), Wo_, bo_), inv, B, N, base=x_)
        return float((dy * y).sum()) + orc.selection_loss(s, labels, lam), (s, qkv, attn)

    _, (s, qkv, attn) = forward()
    # backward, step by step
    g_o = orc.linear_packed_backward(dy.reshape(-1, C), attn, np.arange(T), Wo, None, gidx)
    dq, dk, dv = orc.attention_backward_per_image(qkv[..., :C], qkv[..., C:2 * C], qkv[..., 2 * C:], mask,
                                                  g_o["d_rows"], H)
    g_q = orc.linear_packed_backward(np.concatenate([dq, dk, dv], axis=1), x, gidx, Wqkv, s)
    g_g = orc.gate_backward(x, w, bias, None, labels, orc.unpack(g_q["d_rows"], inv, B, N), True, lam)
    dx_total = dy + g_g["dx"]

    eps = 1e-6

    def fd(name, arr, idx):
        e = np.zeros_like(arr)
        e[idx] = eps
        return (forward(**{name: arr + e})[0] - forward(**{name: arr - e})[0]) / (2 * eps)

    for idx in [(0, 0), (5, 3), (11, 2)]:
        assert abs(fd("Wqkv_", Wqkv, idx) - g_q["dW"][idx]) < 1e-6
    for idx in [(0,), (7,)]:
        assert abs(fd("bqkv_", bqkv, idx) - g_q["dbias"][idx]) < 1e-6
    for idx in [(0, 0), (3, 1)]:
        assert abs(fd("Wo_", Wo, idx) - g_o["dW"][idx]) < 1e-6
    assert abs(fd("bo_", bo, (2,)) - g_o["dbias"][2]) < 1e-6
    for c in range(C):
        assert abs(fd("w_", w, (c,)) - g_g["dw"][c]) < 1e-6
    sel = np.argwhere(mask == 1)[0]
    uns = np.argwhere(mask == 0)[0]
    for b, n in (sel, uns):
        for c in range(C):
            assert abs(fd("x_", x, (b, n, c)) - dx_total[b, n, c]) < 1e-6
