"""spa_gate_bwd_static (the gate backward for callers that cannot allocate: its scratch is a
device array built into the library) against spa_gate_bwd with a caller workspace, through the
C-ABI: two calls in a row on the same GPU, the second with a smaller input, results bit for bit."""
import numpy as np
import pytest
import torch

from paper_2410_23608_amd import workloads as wlmod
from spa_harness import dev, host, tdtype

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def spa():
    from paper_2410_23608_amd import spa as mod
    return mod


def _case(spa, B, N, C, dtype, seed, with_s_up):
    rng = np.random.default_rng(seed)
    mk = wlmod.round_bf16 if dtype == "bf16" else (lambda a: a)
    td = tdtype(dtype)
    x = dev(mk(rng.standard_normal((B, N, C)).astype(np.float32)), dtype)
    w = dev(mk((rng.standard_normal(C) / np.sqrt(C)).astype(np.float32)), dtype)
    d_rg = dev(mk(rng.standard_normal((B, N, C)).astype(np.float32)), dtype)
    labels = dev((rng.uniform(size=(B, N)) < 0.4).astype(np.uint8))
    s_up = dev(rng.standard_normal((B, N)).astype(np.float32)) if with_s_up else None
    scores = torch.empty(B, N, dtype=torch.float32, device="cuda")
    mask = torch.empty(B, N, dtype=torch.uint8, device="cuda")
    spa.spa_gate_select(x, w, 0.1, s_up, 0.5, scores, mask)
    outs = []
    for static in (False, True):
        loss = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
        dx = torch.full((B, N, C), float("nan"), dtype=td, device="cuda")
        dw = torch.full((C,), float("nan"), dtype=torch.float32, device="cuda")
        db = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
        if static:
            spa.spa_gate_bwd_static(x, w, 0.1, scores, s_up, labels, d_rg, True, 0.01 / (B * N), loss, dx, dw, db)
        else:
            code = spa.SPA_BF16 if dtype == "bf16" else spa.SPA_F32
            ws = torch.empty(spa.spa_gate_bwd_workspace_bytes(B, N, C, code), dtype=torch.uint8, device="cuda")
            spa.spa_gate_bwd(x, w, 0.1, scores, s_up, labels, d_rg, True, 0.01 / (B * N), loss, dx, dw, db, ws)
        torch.cuda.synchronize()
        outs.append([host(t).copy() for t in (loss, dx, dw, db)])
    for a, b in zip(*outs):
        assert not np.any(np.isnan(b))
        assert np.array_equal(a, b)


def test_static_scratch_gate_backward_equals_workspace_form(spa):
    # two calls in a row on this GPU's one scratch array; the second is smaller (fewer partial rows,
    # narrower rows), so stale contents of the first would show if anything read them
    _case(spa, 64, 196, 768, "bf16", 1, False)
    _case(spa, 3, 50, 96, "bf16", 2, True)
    _case(spa, 2, 196, 64, "f32", 3, False)
    _case(spa, 1, 7, 8, "f32", 4, True)


def test_static_scratch_rejects_sizes_beyond_its_limit(spa):
    B, N, C = 1, 4, 2048
    x = torch.zeros(B, N, C, dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(C, dtype=torch.bfloat16, device="cuda")
    f = lambda *s: torch.zeros(*s, dtype=torch.float32, device="cuda")
    with pytest.raises(spa.SpaError) as e:
        spa.spa_gate_bwd_static(x, w, 0.0, f(B, N), None, torch.zeros(B, N, dtype=torch.uint8, device="cuda"), None,
                                False, 1.0, f(1), torch.empty_like(x), f(C), f(1))
    assert e.value.code == -3 and "1024" in str(e.value)
