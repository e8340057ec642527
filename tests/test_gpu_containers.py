"""Container-local attention and the cyclic shift (Section 3.2 "Token Packing", Section 1 on
shifting the feature maps) on the GPU against the CPU oracle: index work bit-exact, fp32
values max-abs <= 1e-5, bf16 attention outputs max-abs <= 2e-2, bf16 gradients <= 2e-2
relative to the largest reference entry."""
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


def _ints(n, **kw):
    return torch.zeros(n, dtype=torch.int32, device="cuda", **kw)


@pytest.mark.parametrize("gh,gw,sh,sw", [(14, 14, 3, 3), (14, 14, 0, 5), (7, 9, 6, 1), (60, 70, 3, 3), (5, 4, -1, 9),
                                         (14, 14, 0, 0)])
@pytest.mark.parametrize("use_counts", [False, True])
def test_pack_shifted_matches_oracle(spa, gh, gw, sh, sw, use_counts):
    rng = np.random.default_rng(gh * 100 + gw + sh)
    B, N, C = 5, gh * gw, 24
    mask = (rng.random((B, N)) < 0.45).astype(np.uint8)
    mask[1] = 0
    mask[3] = 1
    x = wlmod.round_bf16(rng.standard_normal((B, N, C)).astype(np.float32))
    s = rng.standard_normal((B, N)).astype(np.float32)
    order = orc.shift_order(gh, gw, sh % gh, sw % gw)
    cu, gidx, inv, T = orc.pack_indices(mask, order)
    rows_ref = orc.pack_rows(x, gidx, None, 0, None)
    scaled_ref = orc.pack_rows(x, gidx, s, 0, "bf16")
    cap = B * N
    counts = dev(mask.sum(1).astype(np.int32)) if use_counts else None
    cu_d, g_d, inv_d, tot = _ints(B + 1), _ints(cap), _ints(cap), _ints(1)
    packed = torch.zeros(cap, C, dtype=torch.bfloat16, device="cuda")
    spa.spa_pack_shifted(dev(x, "bf16"), dev(mask), counts, None, gh, gw, sh, sw, 0, packed, cu_d, g_d, inv_d, tot)
    torch.cuda.synchronize()
    assert int(tot.item()) == T
    assert np.array_equal(host(cu_d), cu) and np.array_equal(host(g_d)[:T], gidx) and np.array_equal(host(inv_d), inv)
    assert np.array_equal(host(packed)[:T], rows_ref)                     # plain row copies are bit-exact
    # gate-scaled rows, indices only, fp32
    spa.spa_pack_shifted(dev(x, "bf16"), dev(mask), counts, dev(s), gh, gw, sh, sw, 0, packed, None, None, None, None)
    torch.cuda.synchronize()
    assert np.max(np.abs(host(packed)[:T] - scaled_ref)) <= 2 ** -7 * np.max(np.abs(scaled_ref))
    g2 = _ints(cap)
    spa.spa_pack_shifted(None, dev(mask), counts, None, gh, gw, sh, sw, 0, None, None, g2, None, None)
    xf = rng.standard_normal((B, N, 8)).astype(np.float32)
    pf = torch.zeros(cap, 8, dtype=torch.float32, device="cuda")
    spa.spa_pack_shifted(dev(xf, "f32"), dev(mask), counts, None, gh, gw, sh, sw, 0, pf, None, None, None, None)
    torch.cuda.synchronize()
    assert np.array_equal(host(g2)[:T], gidx)
    assert np.array_equal(host(pf)[:T], xf.reshape(cap, 8)[gidx])


@pytest.mark.parametrize("lens,L", [([5, 0, 7, 8], 7), ([3, 0, 6], 100), ([2, 2], 1), ([0, 0, 0], 4), ([49] * 9, 49),
                                    ([130, 1, 0, 77, 300], 49)])
def test_container_segments_matches_oracle(spa, lens, L):
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    B, max_total = len(lens), int(cu[-1]) + 5
    ref = orc.container_segments(cu, L)
    cap = spa.spa_container_segments_capacity(B, max_total, L)
    assert cap == B + max_total // L and cap >= len(ref) - 1
    seg = torch.full((cap + 1,), -7, dtype=torch.int32, device="cuda")
    n = _ints(1)
    spa.spa_container_segments(dev(cu), L, max_total, seg, n)
    torch.cuda.synchronize()
    nseg = int(n.item())
    got = host(seg)
    if cu[-1] == 0:
        assert nseg == 0 and np.all(got == 0)
        return
    assert nseg == len(ref) - 1
    assert np.array_equal(got[:nseg + 1], ref) and np.all(got[nseg:] == cu[-1])


def test_container_segments_many_images_and_capacity_check(spa):
    rng = np.random.default_rng(1)
    lens = rng.integers(0, 120, size=700)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    L, B = 49, 700
    ref = orc.container_segments(cu, L)
    cap = spa.spa_container_segments_capacity(B, int(cu[-1]), L)
    seg, n = _ints(cap + 1), _ints(1)
    spa.spa_container_segments(dev(cu), L, int(cu[-1]), seg, n)
    torch.cuda.synchronize()
    assert int(n.item()) == len(ref) - 1 and np.array_equal(host(seg)[:len(ref)], ref)
    with pytest.raises(spa.SpaError):
        spa.spa_container_segments(dev(cu), L, int(cu[-1]), _ints(cap), n)     # one boundary short


def _container_case(spa, dtype, B, gh, gw, C, H, L, shift, seed, frac=(0.2, 0.9), backward=False):
    """gate mask (random) -> shifted pack of q|k|v -> container segments -> attention on the
    segments [-> backward] -> unpack, against the oracle's masked attention on the packed stream."""
    rng = np.random.default_rng(seed)
    N, Dh, cap = gh * gw, C // H, B * gh * gw
    mk = (lambda a: wlmod.round_bf16(a.astype(np.float32))) if dtype == "bf16" else (lambda a: a.astype(np.float32))
    qkv = mk(rng.standard_normal((B, N, 3 * C)))
    fr = rng.uniform(*frac, size=B)
    mask = (rng.random((B, N)) < fr[:, None]).astype(np.uint8)
    order = orc.shift_order(gh, gw, shift[0], shift[1])
    cu, gidx, inv, T = orc.pack_indices(mask, order)
    pk = qkv.reshape(cap, 3 * C)[gidx].astype(np.float64)
    out_ref, lse_ref = orc.attention_container_local(pk[:, :C], pk[:, C:2 * C], pk[:, 2 * C:], cu, L, H)
    y_ref = orc.unpack(out_ref, inv, B, N)
    td = tdtype(dtype)
    cu_d, g_d, inv_d, tot = _ints(B + 1), _ints(cap), _ints(cap), _ints(1)
    packed = torch.zeros(cap, 3 * C, dtype=td, device="cuda")
    seg_cap = spa.spa_container_segments_capacity(B, cap, L)
    seg, nseg = _ints(seg_cap + 1), _ints(1)
    out = torch.zeros(cap, C, dtype=td, device="cuda")
    n_max = min(L, N)
    lse = torch.zeros(H, seg_cap * n_max, dtype=torch.float32, device="cuda")   # [H, segments * max_seqlen]
    y = torch.empty(B, N, C, dtype=td, device="cuda")
    spa.spa_pack_shifted(dev(qkv, dtype), dev(mask), None, None, gh, gw, shift[0], shift[1], 0, packed, cu_d, g_d,
                         inv_d, tot)
    spa.spa_container_segments(cu_d, L, cap, seg, nseg)
    q, k, v = packed[:, :C], packed[:, C:2 * C], packed[:, 2 * C:]
    spa.spa_packed_attention(q, k, v, seg, seg_cap, n_max, H, Dh, out, lse)
    spa.spa_unpack(out, inv_d, None, y)
    torch.cuda.synchronize()
    assert np.array_equal(host(seg)[:int(nseg.item()) + 1], orc.container_segments(cu, L))
    tol = 1e-5 if dtype == "f32" else 2e-2
    assert np.max(np.abs(host(out)[:T] - out_ref)) <= tol
    assert np.max(np.abs(host(lse)[:, :T] - lse_ref)) <= (1e-5 if dtype == "f32" else 2e-2)
    assert np.max(np.abs(host(y) - y_ref)) <= tol
    assert np.all(host(y)[mask == 0] == 0)
    if not backward:
        return
    dout = mk(rng.standard_normal((T, C)) * 0.5)
    dq_ref, dk_ref, dv_ref = orc.attention_container_local_backward(pk[:, :C], pk[:, C:2 * C], pk[:, 2 * C:], cu, L,
                                                                     dout, H)
    dout_d = torch.zeros(cap, C, dtype=td, device="cuda")
    dout_d[:T] = dev(dout, dtype)
    dqkv = torch.zeros(cap, 3 * C, dtype=td, device="cuda")
    code = spa.SPA_BF16 if dtype == "bf16" else spa.SPA_F32
    ws = torch.empty(max(spa.spa_attention_bwd_workspace_bytes(seg_cap, n_max, H, Dh, code), 256), dtype=torch.uint8,
                     device="cuda")
    spa.spa_packed_attention_bwd(q, k, v, out, dout_d, lse, seg, seg_cap, n_max, H, Dh, dqkv[:, :C], dqkv[:, C:2 * C],
                                 dqkv[:, 2 * C:], ws)
    torch.cuda.synchronize()
    got = host(dqkv)[:T]
    for name, g, r in (("dq", got[:, :C], dq_ref), ("dk", got[:, C:2 * C], dk_ref), ("dv", got[:, 2 * C:], dv_ref)):
        err = np.max(np.abs(g - r)) / max(np.max(np.abs(r)), 1e-30)
        assert err <= (1e-4 if dtype == "f32" else 2e-2), (name, err)
    if dtype == "bf16":
        # the same backward with the gradients at token positions (shifted packing order included)
        dy = torch.zeros(cap, C, dtype=td, device="cuda")
        dy[g_d[:T].long()] = dout_d[:T]
        tok = torch.full((cap, 3 * C), float("nan"), dtype=td, device="cuda")
        spa.spa_packed_attention_bwd_tokens(q, k, v, out, dy.view(B, N, C), lse, seg, seg_cap, n_max, H, Dh, g_d, inv_d,
                                            tok[:, :C], tok[:, C:2 * C], tok[:, 2 * C:])
        torch.cuda.synchronize()
        assert torch.equal(tok[g_d[:T].long()], dqkv[:T])
        assert bool((tok[inv_d < 0] == 0).all())


@pytest.mark.parametrize("dtype,B,gh,gw,C,H,L,shift", [
    ("f32", 3, 6, 7, 64, 2, 9, (0, 0)),
    ("f32", 3, 6, 7, 64, 2, 9, (3, 2)),
    ("bf16", 6, 14, 14, 384, 6, 49, (0, 0)),       # vit_s-shaped, the paper's L = M^2 with M = 7
    ("bf16", 6, 14, 14, 384, 6, 49, (3, 3)),
    ("bf16", 2, 20, 30, 256, 8, 49, (3, 3)),       # Dh 32
    ("bf16", 4, 14, 14, 128, 2, 144, (6, 6)),      # L = 12^2
    ("bf16", 3, 10, 10, 64, 1, 1000, (0, 0)),      # one container holds everything: per-image attention
])
def test_container_attention_forward(spa, dtype, B, gh, gw, C, H, L, shift):
    _container_case(spa, dtype, B, gh, gw, C, H, L, shift, seed=L + C)


@pytest.mark.parametrize("dtype,B,gh,gw,C,H,L,shift", [
    ("f32", 2, 6, 7, 64, 2, 9, (3, 2)),
    ("bf16", 5, 14, 14, 384, 6, 49, (3, 3)),
    ("bf16", 2, 20, 30, 256, 8, 49, (0, 0)),
])
def test_container_attention_backward(spa, dtype, B, gh, gw, C, H, L, shift):
    _container_case(spa, dtype, B, gh, gw, C, H, L, shift, seed=7 * L + C, backward=True)


def test_shift_changes_container_partners_but_not_membership(spa):
    """With and without the shift every selected token is processed exactly once and lands at
    its own position; the sets of tokens that share a segment differ."""
    rng = np.random.default_rng(2)
    B, gh, gw = 3, 14, 14
    N, cap = gh * gw, B * gh * gw
    mask = (rng.random((B, N)) < 0.5).astype(np.uint8)
    res = {}
    for shift in ((0, 0), (3, 3)):
        cu_d, g_d, inv_d, tot = _ints(B + 1), _ints(cap), _ints(cap), _ints(1)
        spa.spa_pack_shifted(None, dev(mask), None, None, gh, gw, shift[0], shift[1], 0, None, cu_d, g_d, inv_d, tot)
        torch.cuda.synchronize()
        T = int(tot.item())
        res[shift] = (host(cu_d), host(g_d)[:T], host(inv_d))
    (cu0, g0, inv0), (cu1, g1, inv1) = res[(0, 0)], res[(3, 3)]
    assert np.array_equal(cu0, cu1) and np.array_equal(np.sort(g0), np.sort(g1))
    assert np.array_equal(inv0 >= 0, inv1 >= 0) and not np.array_equal(g0, g1)
    same_container = lambda inv, a, b: inv[a] // 49 == inv[b] // 49
    sel = np.flatnonzero(inv0[:N] >= 0)
    pairs = [(a, b) for a in sel[:40] for b in sel[:40] if a < b]
    assert any(same_container(inv0, a, b) != same_container(inv1, a, b) for a, b in pairs)


@pytest.mark.parametrize("dtype,B,gh,gw,C,H,L", [("bf16", 6, 14, 14, 384, 6, 49), ("bf16", 2, 20, 30, 256, 8, 49),
                                                 ("f32", 3, 6, 7, 64, 2, 9), ("bf16", 2, 30, 30, 64, 2, 400)])
@pytest.mark.parametrize("with_base", [False, True])
def test_segment_attention_unpack_equals_two_calls(spa, dtype, B, gh, gw, C, H, L, with_base):
    """Attention on container segments + scatter back in one launch gives the bits of
    spa_packed_attention on the segments followed by spa_unpack."""
    rng = np.random.default_rng(L + C + B)
    N, Dh, cap = gh * gw, C // H, B * gh * gw
    mk = (lambda a: wlmod.round_bf16(a.astype(np.float32))) if dtype == "bf16" else (lambda a: a.astype(np.float32))
    qkv = dev(mk(rng.standard_normal((B, N, 3 * C))), dtype)
    base = dev(mk(rng.standard_normal((B, N, C))), dtype) if with_base else None
    mask = (rng.random((B, N)) < rng.uniform(0.1, 0.9, size=(B, 1))).astype(np.uint8)
    mask[0] = 0
    td = tdtype(dtype)
    cu_d, g_d, inv_d, tot = _ints(B + 1), _ints(cap), _ints(cap), _ints(1)
    packed = torch.zeros(cap, 3 * C, dtype=td, device="cuda")
    seg_cap = spa.spa_container_segments_capacity(B, cap, L)
    seg, nseg = _ints(seg_cap + 1), _ints(1)
    n_max = min(L, N)
    spa.spa_pack_shifted(qkv, dev(mask), None, None, gh, gw, 2, 1, 0, packed, cu_d, g_d, inv_d, tot)
    spa.spa_container_segments(cu_d, L, cap, seg, nseg)
    q, k, v = packed[:, :C], packed[:, C:2 * C], packed[:, 2 * C:]
    out2 = torch.zeros(cap, C, dtype=td, device="cuda")
    lse2 = torch.zeros(H, seg_cap * n_max, dtype=torch.float32, device="cuda")
    y2 = torch.empty(B, N, C, dtype=td, device="cuda")
    spa.spa_packed_attention(q, k, v, seg, seg_cap, n_max, H, Dh, out2, lse2)
    spa.spa_unpack(out2, inv_d, base, y2)
    out1, lse1 = torch.zeros_like(out2), torch.zeros_like(lse2)
    y1 = torch.full((B, N, C), float("nan"), dtype=td, device="cuda")
    spa.spa_segment_attention_unpack(q, k, v, seg, n_max, g_d, inv_d, base, H, Dh, y1, out1, lse1)
    torch.cuda.synchronize()
    T = int(tot.item())
    assert torch.equal(y1, y2) and torch.equal(out1[:T], out2[:T]) and torch.equal(lse1, lse2)
    y3 = torch.full((B, N, C), float("nan"), dtype=td, device="cuda")
    spa.spa_segment_attention_unpack(q, k, v, seg, n_max, g_d, inv_d, base, H, Dh, y3)      # y only
    torch.cuda.synchronize()
    assert torch.equal(y3, y2)
