"""The Python binding refuses calls whose tensors would be read or written with the wrong
element size or past their end.  The C-ABI takes void* and ONE dtype code per call, so these
checks are the only place a dtype mix can be caught; they run before any pointer is taken and
therefore need no GPU (the tensors here live on the host and are never dereferenced)."""
import pytest
import torch

from paper_2410_23608_amd import spa


def _t(shape, dtype):
    return torch.zeros(shape, dtype=dtype)


B, N, C, H, Dh = 2, 16, 64, 2, 32
CAP = B * N
bf, f32, i32, u8 = torch.bfloat16, torch.float32, torch.int32, torch.uint8


def test_fp32_rows_into_bf16_packed_buffers_are_refused():
    """The case that once ended in a GPU memory fault: fp32 feature tensors handed to a chain whose
    packed buffers are bf16.  spa_pack_pair would have written T*(C+C2)*4 bytes into buffers of
    CAP*(C+C2)*2 bytes."""
    x, x2 = _t((B, N, 2 * C), f32), _t((B, N, C), f32)
    packed, packed2 = _t((CAP, 2 * C), bf), _t((CAP, C), bf)
    assert x.numel() * x.element_size() == 2 * packed.numel() * packed.element_size()   # twice the bytes
    with pytest.raises(ValueError, match="share one dtype"):
        spa.spa_pack_pair(x, x2, _t((B, N), u8), None, _t((B, N), f32), packed, packed2, _t(B + 1, i32), _t(CAP, i32),
                          _t(CAP, i32), _t(1, i32))


def test_fp32_gradient_into_bf16_dx_is_refused():
    x, w = _t((B, N, C), f32), _t(C, f32)
    args = dict(scores=_t((B, N), f32), s_up=None, labels=_t((B, N), u8), loss=_t(1, f32), dw=_t(C, f32), db=_t(1, f32))
    with pytest.raises(ValueError, match="share one dtype"):
        spa.spa_gate_bwd(x, w, 0.0, args["scores"], None, args["labels"], _t((B, N, C), bf), True, 1.0, args["loss"],
                         _t((B, N, C), bf), args["dw"], args["db"], _t(4096, u8))
    with pytest.raises(ValueError, match="share one dtype"):
        spa.spa_gate_bwd(x, w, 0.0, args["scores"], None, args["labels"], _t((B, N, C), f32), True, 1.0, args["loss"],
                         _t((B, N, C), bf), args["dw"], args["db"], _t(4096, u8))


def test_every_feature_tensor_of_a_call_is_compared():
    q = _t((CAP, 3 * C), bf)
    with pytest.raises(ValueError, match="share one dtype"):
        spa.spa_packed_attention(q[:, :C], q[:, C:2 * C], q[:, 2 * C:], _t(B + 1, i32), B, N, H, Dh, _t((CAP, C), f32))
    with pytest.raises(ValueError, match="share one dtype"):
        spa.spa_packed_attention_unpack(q[:, :C], q[:, C:2 * C], q[:, 2 * C:], _t(B + 1, i32), _t(CAP, i32),
                                        _t(CAP, i32), _t((B, N, C), f32), H, Dh, _t((B, N, C), bf))
    with pytest.raises(ValueError, match="share one dtype"):
        spa.spa_gate_select(_t((B, N, C), bf), _t(C, f32), 0.0, None, 0.5, _t((B, N), f32), _t((B, N), u8))
    with pytest.raises(ValueError, match="share one dtype"):
        spa.spa_pack(_t((B, N, C), f32), _t((B, N), u8), None, None, 0, _t((CAP, C), bf), None, None, None, None)
    with pytest.raises(ValueError, match="share one dtype"):
        spa.spa_unpack(_t((CAP, C), bf), _t(CAP, i32), None, _t((B, N, C), f32))
    with pytest.raises(ValueError, match="share one dtype"):
        spa.spa_linear_packed(_t((B, N, C), f32), None, None, None, _t((C, C), bf), None, _t((CAP, C), bf))
    with pytest.raises(ValueError, match="share one dtype"):
        spa.spa_packed_attention_bwd(q[:, :C], q[:, C:2 * C], q[:, 2 * C:], _t((CAP, C), bf), _t((CAP, C), bf),
                                     _t((H, CAP), f32), _t(B + 1, i32), B, N, H, Dh, _t((CAP, C), f32),
                                     _t((CAP, C), bf), _t((CAP, C), bf), None)


def test_index_score_and_mask_types_are_fixed():
    x, w = _t((B, N, C), bf), _t(C, bf)
    with pytest.raises(ValueError, match="scores must be torch.float32"):
        spa.spa_gate_select(x, w, 0.0, None, 0.5, _t((B, N), bf), _t((B, N), u8))
    with pytest.raises(ValueError, match="mask must be torch.uint8"):
        spa.spa_gate_select(x, w, 0.0, None, 0.5, _t((B, N), f32), _t((B, N), torch.bool))
    with pytest.raises(ValueError, match="gather_idx must be torch.int32"):
        spa.spa_pack(None, _t((B, N), u8), None, None, 0, None, _t(B + 1, i32), _t(CAP, torch.int64), None, None)
    with pytest.raises(ValueError, match="feature tensors are float32 or bfloat16"):
        spa.spa_unpack(_t((CAP, C), torch.float16), _t(CAP, i32), None, _t((B, N, C), torch.float16))


def test_outputs_that_are_too_small_are_refused():
    x, w = _t((B, N, C), bf), _t(C, bf)
    with pytest.raises(ValueError, match="scores holds"):
        spa.spa_gate_select(x, w, 0.0, None, 0.5, _t((B, N - 1), f32), _t((B, N), u8))
    with pytest.raises(ValueError, match="packed holds"):
        spa.spa_pack(x, _t((B, N), u8), None, None, 0, _t((CAP - 1, C), bf), None, None, None, None)
    with pytest.raises(ValueError, match="packed holds"):        # the zero tail of the last container
        spa.spa_pack(x, _t((B, N), u8), None, None, 8, _t((CAP, C), bf), None, None, None, None)
    with pytest.raises(ValueError, match="inv_pos holds"):
        spa.spa_pack(None, _t((B, N), u8), None, None, 0, None, None, None, _t(CAP - 1, i32), None)
    with pytest.raises(ValueError, match="dx holds"):
        spa.spa_gate_bwd(x, w, 0.0, _t((B, N), f32), None, _t((B, N), u8), None, False, 1.0, _t(1, f32),
                         _t((B, N, C // 2), bf), _t(C, f32), _t(1, f32), _t(4096, u8))
    q = _t((CAP, 3 * C), bf)
    with pytest.raises(ValueError, match="lse holds"):
        spa.spa_packed_attention(q[:, :C], q[:, C:2 * C], q[:, 2 * C:], _t(B + 1, i32), B, N, H, Dh, _t((CAP, C), bf),
                                 _t((H, CAP - 1), f32))
    with pytest.raises(ValueError, match="dq must be"):
        spa.spa_packed_attention_bwd_tokens(q[:, :C], q[:, C:2 * C], q[:, 2 * C:], _t((CAP, C), bf), _t((B, N, C), bf),
                                            _t((H, CAP), f32), _t(B + 1, i32), B, N, H, Dh, _t(CAP, i32), _t(CAP, i32),
                                            _t((CAP - 1, C), bf), _t((CAP, C), bf), _t((CAP, C), bf))


def test_a_consistent_call_gets_past_the_checks_to_the_device_test():
    """With consistent host tensors the next thing that fails is the device check: the dtype and
    size checks come first and pass."""
    with pytest.raises(ValueError, match="device tensors"):
        spa.spa_gate_select(_t((B, N, C), bf), _t(C, bf), 0.0, None, 0.5, _t((B, N), f32), _t((B, N), u8))
