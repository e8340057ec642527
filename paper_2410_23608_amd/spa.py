"""ctypes binding over libspa.so: same names as the C entry points in include/spa.h.

Argument marshalling only — torch tensors supply device memory and the current stream;
every step of the path runs in the library's HIP kernels.  There is no fallback: if the
shared library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import c_char_p, c_double, c_float, c_int, c_int64, c_size_t, c_void_p
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SPA_LIB_PATH", os.path.join(_HERE, "libspa.so"))

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2410_23608_amd.build` "
        "(the SPA path has no CPU or PyTorch fallback)")

lib = ctypes.CDLL(LIB_PATH)

SPA_OK, SPA_F32, SPA_BF16 = 0, 0, 1

_P = c_void_p
_SIGNATURES = {
    "spa_version": (c_int, []),
    "spa_last_error": (c_char_p, []),
    "spa_set_option": (c_int, [c_char_p, c_char_p]),
    "spa_workspace_bytes": (c_size_t, [c_int, c_int, c_int, c_int, c_int, c_int]),
    "spa_gate_select": (c_int, [_P, _P, c_float, _P, c_float, c_int, c_int, c_int, c_int, _P, _P, _P, _P]),
    "spa_gate_select_index": (c_int, [_P, _P, c_float, _P, c_float, c_int, c_int, c_int, c_int, _P, _P, _P, _P, _P, _P, _P,
                                      _P, c_size_t, _P]),
    "spa_gate_select_pooled": (c_int, [_P, _P, c_float, _P, c_float, c_int, c_int, c_int, c_int, c_int, _P, _P, _P, _P,
                                       _P]),
    "spa_gate_select_gumbel": (c_int, [_P, _P, c_float, _P, _P, c_float, c_float, c_int, c_int, c_int, c_int, _P, _P,
                                       _P, _P]),
    "spa_gate_bwd_straight_through": (c_int, [_P, _P, c_float, _P, _P, _P, _P, c_float, _P, _P, c_float, c_int, c_int,
                                              c_int, c_int, _P, _P, _P, _P, _P, c_size_t, _P]),
    "spa_maxpool2x2": (c_int, [_P, c_int, c_int, c_int, _P, _P]),
    "spa_pack": (c_int, [_P, _P, _P, _P, c_int, c_int, c_int, c_int, c_int, _P, _P, _P, _P, _P, _P]),
    "spa_pack_pair": (c_int, [_P, c_int, _P, c_int, _P, _P, _P, c_int, c_int, c_int, _P, _P, _P, _P, _P, _P, _P]),
    "spa_pack_shifted": (c_int, [_P, _P, _P, _P, c_int, c_int, c_int, c_int, c_int, c_int, c_int, c_int, _P, _P, _P,
                                 _P, _P, _P]),
    "spa_container_segments_capacity": (c_int64, [c_int, c_int64, c_int]),
    "spa_container_segments": (c_int, [_P, c_int, c_int, c_int64, c_int, _P, _P, _P]),
    "spa_packed_attention": (c_int, [_P, _P, _P, c_int64, c_int64, c_int64, _P, c_int, c_int, c_int, c_int, c_int, c_float, _P, _P, _P]),
    "spa_packed_attention_unpack": (c_int, [_P, _P, _P, c_int64, c_int64, c_int64, _P, _P, _P, _P, c_int, c_int, c_int,
                                            c_int, c_int, c_float, _P, _P, _P, _P]),
    "spa_gathered_attention_unpack": (c_int, [_P, _P, _P, c_int64, c_int64, c_int64, _P, _P, _P, _P, c_int, c_int, c_int,
                                              c_int, c_int, c_float, _P, _P, _P, _P]),
    "spa_selected_attention_unpack": (c_int, [_P, _P, _P, c_int64, c_int64, c_int64, _P, _P, c_int, c_int, c_int, c_int,
                                              c_int, c_float, _P, _P]),
    "spa_segment_attention_unpack": (c_int, [_P, _P, _P, c_int64, c_int64, c_int64, _P, c_int, c_int, _P, _P, _P, c_int64,
                                             c_int, c_int, c_int, c_float, _P, _P, _P, _P]),
    "spa_ceiling_copy": (c_int, [_P, _P, c_size_t, _P]),
    "spa_ceiling_mfma": (c_double, [_P, c_int, c_int, _P]),
    "spa_linear_packed": (c_int, [_P, _P, _P, _P, _P, _P, c_int, c_int, c_int, c_int, _P, c_int64, _P]),
    "spa_linear_packed_scatter": (c_int, [_P, _P, _P, _P, c_int, c_int, c_int, c_int, _P, _P, _P, c_int64, _P]),
    "spa_linear_packed_bwd_input": (c_int, [_P, _P, c_int64, _P, _P, c_int, c_int, c_int, c_int, _P, _P, c_int64, _P,
                                            c_int64, _P]),
    "spa_linear_bwd_weight_workspace_bytes": (c_size_t, [c_int, c_int, c_int, c_int]),
    "spa_linear_packed_bwd_weight": (c_int, [_P, _P, c_int64, _P, _P, _P, _P, c_int, c_int, c_int, c_int, _P, _P, _P,
                                             c_size_t, _P]),
    "spa_unpack": (c_int, [_P, _P, _P, c_int, c_int, c_int, c_int, _P, _P]),
    "spa_unpack_bwd": (c_int, [_P, _P, _P, c_int, c_int, c_int, c_int, _P, _P]),
    "spa_pack_bwd": (c_int, [_P, _P, c_int, c_int, c_int, c_int, _P, _P]),
    "spa_attention_bwd_workspace_bytes": (c_size_t, [c_int, c_int, c_int, c_int, c_int]),
    "spa_packed_attention_bwd": (c_int, [_P, _P, _P, c_int64, c_int64, c_int64, _P, _P, _P, _P, c_int, c_int, c_int,
                                         c_int, c_int, c_float, _P, _P, _P, c_int64, c_int64, c_int64, _P,
                                         c_size_t, _P]),
    "spa_packed_attention_bwd_tokens": (c_int, [_P, _P, _P, c_int64, c_int64, c_int64, _P, _P, _P, _P, c_int, c_int,
                                                c_int, c_int, c_int, c_float, _P, _P, c_int64, _P, _P, _P, c_int64,
                                                c_int64, c_int64, _P, c_size_t, _P]),
    "spa_gate_bwd_workspace_bytes": (c_size_t, [c_int, c_int, c_int, c_int]),
    "spa_gate_bwd": (c_int, [_P, _P, c_float, _P, _P, _P, _P, c_int, c_float, c_int, c_int, c_int, c_int,
                             _P, _P, _P, _P, _P, c_size_t, _P]),
    "spa_gate_bwd_static": (c_int, [_P, _P, c_float, _P, _P, _P, _P, c_int, c_float, c_int, c_int, c_int, c_int,
                                    _P, _P, _P, _P, _P]),
    "spa_padded_attention": (c_int, [_P, _P, _P, c_int64, _P, c_int, c_int, c_int, c_int, c_int, c_float, _P, _P]),
}
for _name, (_res, _args) in _SIGNATURES.items():
    _fn = getattr(lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args

EXPORTS = tuple(_SIGNATURES)


class SpaError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libspa error {code}: {msg}")
        self.code = code


def _check(rc: int) -> None:
    if rc != SPA_OK:
        raise SpaError(rc, lib.spa_last_error().decode())


class Prepared:
    """A C-ABI call with its arguments already marshalled (pointers, sizes and the stream that
    was current at preparation).  Calling it enqueues the work again with no per-call
    conversion cost; the tensors it refers to are kept alive by the object."""
    __slots__ = ("_fn", "_args", "_keep")

    def __init__(self, fn, args, keep):
        self._fn = fn
        self._args = tuple(a if not isinstance(a, int) or t is not _P else _P(a)
                           for a, t in zip(args, fn.argtypes))
        self._keep = keep

    def __call__(self):
        rc = self._fn(*self._args)
        if rc != SPA_OK:
            raise SpaError(rc, lib.spa_last_error().decode())


def _dispatch(fn, args, keep, prepare):
    if prepare:
        return Prepared(fn, args, keep)
    _check(fn(*args))
    return None


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("libspa takes device tensors")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return SPA_F32
    if t.dtype == torch.bfloat16:
        return SPA_BF16
    raise ValueError(f"unsupported dtype {t.dtype}")


def _contig(*ts):
    for t in ts:
        if t is not None and not t.is_contiguous():
            raise ValueError("libspa takes contiguous tensors")


# The C-ABI sees void* and ONE dtype code per call, so a tensor of another type would be read
# or written with the wrong element size (twice the bytes for fp32 in a bf16 buffer).  Every
# binding function therefore checks, BEFORE any pointer is taken, that the feature tensors of
# the call share one dtype, that index / score / mask tensors have their fixed types, and that
# every output holds at least what the call can write.
def _features(fn: str, **named) -> int:
    """All given feature tensors share one dtype (fp32 or bf16); returns its SPA_* code."""
    first = None
    for name, t in named.items():
        if t is None:
            continue
        if t.dtype not in (torch.float32, torch.bfloat16):
            raise ValueError(f"{fn}: {name} has dtype {t.dtype}; feature tensors are float32 or bfloat16")
        if first is None:
            first = (name, t.dtype)
        elif t.dtype != first[1]:
            raise ValueError(f"{fn}: {name} is {t.dtype} but {first[0]} is {first[1]}: the feature tensors of a "
                             "call must share one dtype")
    if first is None:
        raise ValueError(f"{fn}: no feature tensor given")
    return SPA_F32 if first[1] == torch.float32 else SPA_BF16


def _typed(fn: str, dtype, **named) -> None:
    for name, t in named.items():
        if t is not None and t.dtype != dtype:
            raise ValueError(f"{fn}: {name} must be {dtype}, got {t.dtype}")


def _holds(fn: str, **named) -> None:
    """named: name = (tensor or None, elements the call may touch)."""
    for name, (t, need) in named.items():
        if t is not None and t.numel() < need:
            raise ValueError(f"{fn}: {name} holds {t.numel()} elements, the call needs {need}")


def _rows(fn: str, width: int, **named) -> None:
    """named: name = (2-D tensor or column-slice view or None, rows the call may touch)."""
    for name, (t, need) in named.items():
        if t is None:
            continue
        if t.dim() != 2 or t.shape[1] != width or t.shape[0] < need:
            raise ValueError(f"{fn}: {name} must be [>= {need}, {width}], got {tuple(t.shape)}")


def spa_version() -> int:
    return lib.spa_version()


SPA_OP_GATE_SELECT, SPA_OP_PACK, SPA_OP_PACKED_ATTENTION, SPA_OP_UNPACK = 0, 1, 2, 3
SPA_OP_PACKED_ATTENTION_BWD, SPA_OP_GATE_BWD = 4, 5
SPA_OP_QKV_PROJECTION_BWD_WEIGHT, SPA_OP_OUT_PROJECTION_BWD_WEIGHT = 6, 7


def spa_set_option(name: str, value: Optional[str] = None) -> None:
    """Process-wide launch option (kernel selection for tests and tuning); None / "" = default."""
    _check(lib.spa_set_option(name.encode(), (value or "").encode()))


def spa_workspace_bytes(op: int, B: int, N: int, C: int, H: int, dtype: int) -> int:
    return int(lib.spa_workspace_bytes(int(op), int(B), int(N), int(C), int(H), int(dtype)))


def _gate_select_checks(fn, x, w, s_up, noise, scores, mask, counts):
    B, N, C = x.shape
    code = _features(fn, x=x, w=w)
    _typed(fn, torch.float32, s_up=s_up, noise=noise, scores=scores)
    _typed(fn, torch.uint8, mask=mask)
    _typed(fn, torch.int32, counts=counts)
    _holds(fn, w=(w, C), s_up=(s_up, B * N), noise=(noise, B * N), scores=(scores, B * N), mask=(mask, B * N),
           counts=(counts, B))
    return B, N, C, code


def spa_gate_select(x, w, bias, s_up, tau, scores, mask, counts=None, prepare=False):
    """x [B,N,C]; w [C]; s_up [B,N] f32 or None -> scores [B,N] f32, mask [B,N] u8, counts [B] i32."""
    B, N, C, code = _gate_select_checks("spa_gate_select", x, w, s_up, None, scores, mask, counts)
    _keep = (x, w, s_up, scores, mask, counts,)
    _contig(*_keep)
    return _dispatch(lib.spa_gate_select, (_ptr(x), _ptr(w), float(bias), _ptr(s_up), float(tau), B, N, C, code,
                               _ptr(scores), _ptr(mask), _ptr(counts), _stream(),), _keep, prepare)


def spa_gate_select_index(x, w, bias, s_up, tau, scores, mask, counts, cu_seqlens, gather_idx, inv_pos, total, workspace,
                          prepare=False):
    """spa_gate_select + the index-only spa_pack in one launch.  workspace: >= 73984 bytes, zero before the
    first call (every call leaves it zero)."""
    fn = "spa_gate_select_index"
    B, N, C, code = _gate_select_checks(fn, x, w, s_up, None, scores, mask, counts)
    _typed(fn, torch.int32, cu_seqlens=cu_seqlens, gather_idx=gather_idx, inv_pos=inv_pos, total=total)
    _holds(fn, cu_seqlens=(cu_seqlens, B + 1), gather_idx=(gather_idx, B * N), inv_pos=(inv_pos, B * N), total=(total, 1))
    _keep = (x, w, s_up, scores, mask, counts, cu_seqlens, gather_idx, inv_pos, total, workspace,)
    _contig(*_keep)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    return _dispatch(lib.spa_gate_select_index,
                     (_ptr(x), _ptr(w), float(bias), _ptr(s_up), float(tau), B, N, C, code, _ptr(scores), _ptr(mask),
                      _ptr(counts), _ptr(cu_seqlens), _ptr(gather_idx), _ptr(inv_pos), _ptr(total), _ptr(workspace),
                      ws_bytes, _stream(),), _keep, prepare)


def spa_gate_select_gumbel(x, w, bias, s_up, noise, temperature, tau, scores, mask, counts=None, prepare=False):
    """spa_gate_select with caller-supplied logistic noise [B,N] f32 and a temperature:
    selected when sigmoid((s + noise) / temperature) > tau."""
    B, N, C, code = _gate_select_checks("spa_gate_select_gumbel", x, w, s_up, noise, scores, mask, counts)
    _keep = (x, w, s_up, noise, scores, mask, counts,)
    _contig(*_keep)
    return _dispatch(lib.spa_gate_select_gumbel,
                     (_ptr(x), _ptr(w), float(bias), _ptr(s_up), _ptr(noise), float(temperature), float(tau), B, N, C,
                      code, _ptr(scores), _ptr(mask), _ptr(counts), _stream(),), _keep, prepare)


def spa_gate_select_pooled(x, w, bias, s_fine, grid_h, grid_w, tau, scores, mask, counts=None, s_up_pooled=None,
                           prepare=False):
    """spa_gate_select whose up-scale scores are the 2x2 max-pool of s_fine [B, 2*grid_h*2*grid_w],
    pooled inside the kernel."""
    fn = "spa_gate_select_pooled"
    B, N, C, code = _gate_select_checks(fn, x, w, None, None, scores, mask, counts)
    if N != grid_h * grid_w or s_fine.numel() != 4 * B * N:
        raise ValueError("x must be [B, grid_h*grid_w, C] and s_fine [B, 4*grid_h*grid_w]")
    _typed(fn, torch.float32, s_fine=s_fine, s_up_pooled=s_up_pooled)
    _holds(fn, s_up_pooled=(s_up_pooled, B * N))
    _keep = (x, w, s_fine, scores, mask, counts, s_up_pooled,)
    _contig(*_keep)
    return _dispatch(lib.spa_gate_select_pooled,
                     (_ptr(x), _ptr(w), float(bias), _ptr(s_fine), float(tau), B, int(grid_h), int(grid_w), C,
                      code, _ptr(scores), _ptr(mask), _ptr(counts), _ptr(s_up_pooled), _stream(),), _keep, prepare)


def spa_maxpool2x2(s, h, w, pooled, prepare=False):
    B = s.shape[0]
    _typed("spa_maxpool2x2", torch.float32, s=s, pooled=pooled)
    _holds("spa_maxpool2x2", s=(s, B * h * w), pooled=(pooled, B * (h // 2) * (w // 2)))
    _keep = (s, pooled,)
    _contig(*_keep)
    return _dispatch(lib.spa_maxpool2x2, (_ptr(s), B, h, w, _ptr(pooled), _stream(),), _keep, prepare)


def _pack_checks(fn, x, mask, counts, gate_scores, container_len, packed, cu_seqlens, gather_idx, inv_pos, total):
    B, N = mask.shape
    if (x is None) != (packed is None):
        raise ValueError(f"{fn}: x and packed are given together or not at all")
    C = x.shape[-1] if x is not None else 8
    code = _features(fn, x=x, packed=packed) if x is not None else SPA_BF16
    _typed(fn, torch.uint8, mask=mask)
    _typed(fn, torch.int32, counts=counts, cu_seqlens=cu_seqlens, gather_idx=gather_idx, inv_pos=inv_pos, total=total)
    _typed(fn, torch.float32, gate_scores=gate_scores)
    cap = B * N
    _holds(fn, x=(x, cap * C), packed=(packed, (cap + max(int(container_len) - 1, 0)) * C), counts=(counts, B),
           gate_scores=(gate_scores, cap), cu_seqlens=(cu_seqlens, B + 1), gather_idx=(gather_idx, cap),
           inv_pos=(inv_pos, cap), total=(total, 1))
    return B, N, C, code


def spa_pack(x, mask, counts, gate_scores, container_len, packed, cu_seqlens, gather_idx, inv_pos, total,
             prepare=False):
    """x [B,N,C] (C may be a fused q|k|v row) -> packed [cap,C], cu_seqlens [B+1], gather_idx, inv_pos, total.
    x = packed = None computes the indices only."""
    B, N, C, code = _pack_checks("spa_pack", x, mask, counts, gate_scores, container_len, packed, cu_seqlens,
                                 gather_idx, inv_pos, total)
    _keep = (x, mask, counts, gate_scores, packed, cu_seqlens, gather_idx, inv_pos, total,)
    _contig(*_keep)
    return _dispatch(lib.spa_pack, (_ptr(x), _ptr(mask), _ptr(counts), _ptr(gate_scores), B, N, C, code,
                        int(container_len), _ptr(packed), _ptr(cu_seqlens), _ptr(gather_idx), _ptr(inv_pos),
                        _ptr(total), _stream(),), _keep, prepare)


def spa_pack_pair(x, x2, mask, counts, gate_scores, packed, packed2, cu_seqlens, gather_idx, inv_pos, total,
                  prepare=False):
    """spa_pack of x [B,N,C] (unscaled) and x2 [B,N,C2] (scaled by sigmoid(gate_scores) if given) in one launch."""
    fn = "spa_pack_pair"
    B, N, C, code = _pack_checks(fn, x, mask, counts, gate_scores, 0, packed, cu_seqlens, gather_idx, inv_pos, total)
    C2 = x2.shape[-1]
    _features(fn, x=x, x2=x2, packed=packed, packed2=packed2)
    _holds(fn, x2=(x2, B * N * C2), packed2=(packed2, B * N * C2))
    _keep = (x, x2, mask, counts, gate_scores, packed, packed2, cu_seqlens, gather_idx, inv_pos, total,)
    _contig(*_keep)
    return _dispatch(lib.spa_pack_pair,
                     (_ptr(x), C, _ptr(x2), C2, _ptr(mask), _ptr(counts), _ptr(gate_scores), B, N, code,
                      _ptr(packed), _ptr(packed2), _ptr(cu_seqlens), _ptr(gather_idx), _ptr(inv_pos), _ptr(total),
                      _stream(),), _keep, prepare)


def spa_pack_shifted(x, mask, counts, gate_scores, grid_h, grid_w, shift_h, shift_w, container_len, packed,
                     cu_seqlens, gather_idx, inv_pos, total, prepare=False):
    """spa_pack in the raster order of the feature map cyclically shifted by (shift_h, shift_w);
    mask [B, grid_h*grid_w].  gather_idx / inv_pos name positions of the original layout."""
    B, N, C, code = _pack_checks("spa_pack_shifted", x, mask, counts, gate_scores, container_len, packed, cu_seqlens,
                                 gather_idx, inv_pos, total)
    if N != grid_h * grid_w:
        raise ValueError("mask.shape[1] != grid_h * grid_w")
    _keep = (x, mask, counts, gate_scores, packed, cu_seqlens, gather_idx, inv_pos, total,)
    _contig(*_keep)
    return _dispatch(lib.spa_pack_shifted,
                     (_ptr(x), _ptr(mask), _ptr(counts), _ptr(gate_scores), B, int(grid_h), int(grid_w), int(shift_h),
                      int(shift_w), C, code, int(container_len), _ptr(packed),
                      _ptr(cu_seqlens), _ptr(gather_idx), _ptr(inv_pos), _ptr(total), _stream(),), _keep, prepare)


def spa_container_segments_capacity(B, max_total, container_len) -> int:
    return int(lib.spa_container_segments_capacity(int(B), int(max_total), int(container_len)))


def spa_container_segments(cu_seqlens, container_len, max_total, seg_cu_seqlens, n_segments, prepare=False):
    """cu_seqlens [B+1] -> seg_cu_seqlens [seg_cap+1] (boundaries of image x container segments,
    padded with empty segments), n_segments [1]."""
    B = cu_seqlens.numel() - 1
    _typed("spa_container_segments", torch.int32, cu_seqlens=cu_seqlens, seg_cu_seqlens=seg_cu_seqlens,
           n_segments=n_segments)
    _keep = (cu_seqlens, seg_cu_seqlens, n_segments,)
    _contig(*_keep)
    return _dispatch(lib.spa_container_segments,
                     (_ptr(cu_seqlens), B, int(container_len), int(max_total), seg_cu_seqlens.numel() - 1,
                      _ptr(seg_cu_seqlens), _ptr(n_segments), _stream(),), _keep, prepare)


def _row_stride(t) -> int:
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError("expected a 2-D [rows, H*Dh] tensor or column-slice view with unit inner stride")
    return int(t.stride(0))


def spa_packed_attention(q, k, v, cu_seqlens, B, max_seqlen, H, Dh, out, lse=None, softmax_scale=0.0,
                         prepare=False):
    """q, k, v: [rows, H*Dh] tensors or column-slice views of fused packed buffers; the row
    strides are taken from the views."""
    fn = "spa_packed_attention"
    code = _features(fn, q=q, k=k, v=v, out=out)
    _typed(fn, torch.int32, cu_seqlens=cu_seqlens)
    _typed(fn, torch.float32, lse=lse)
    _rows(fn, H * Dh, q=(q, 1), k=(k, 1), v=(v, 1), out=(out, 1))
    _holds(fn, cu_seqlens=(cu_seqlens, B + 1), lse=(lse, H * B * max_seqlen))
    _keep = (q, k, v, out, lse, cu_seqlens,)
    _contig(out, lse, cu_seqlens)
    return _dispatch(lib.spa_packed_attention, (_ptr(q), _ptr(k), _ptr(v), _row_stride(q), _row_stride(k), _row_stride(v),
                                    _ptr(cu_seqlens), B, max_seqlen,
                                    H, Dh, code, float(softmax_scale), _ptr(out), _ptr(lse), _stream(),), _keep, prepare)


def _scatter_checks(fn, q, k, v, seg, n_seg, max_seqlen, gather_idx, inv_pos, base, H, Dh, y, out, lse):
    C = H * Dh
    rows = y.numel() // y.shape[-1]
    if y.shape[-1] != C:
        raise ValueError(f"{fn}: y must be [..., H*Dh]")
    code = _features(fn, q=q, k=k, v=v, y=y, base=base, out=out)
    _typed(fn, torch.int32, cu_seqlens=seg, gather_idx=gather_idx, inv_pos=inv_pos)
    _typed(fn, torch.float32, lse=lse)
    _rows(fn, C, q=(q, 1), k=(k, 1), v=(v, 1), out=(out, 1))
    _holds(fn, cu_seqlens=(seg, n_seg + 1), gather_idx=(gather_idx, rows), inv_pos=(inv_pos, rows),
           base=(base, rows * C), lse=(lse, H * n_seg * max_seqlen))
    return rows, code


def spa_packed_attention_unpack(q, k, v, cu_seqlens, gather_idx, inv_pos, base, H, Dh, y, out=None, lse=None,
                                softmax_scale=0.0, prepare=False):
    """Attention on the packed rows + scatter back to y [B,N,C] in one launch."""
    B, N, C = y.shape
    _, code = _scatter_checks("spa_packed_attention_unpack", q, k, v, cu_seqlens, B, N, gather_idx, inv_pos, base, H,
                              Dh, y, out, lse)
    _keep = (q, k, v, cu_seqlens, gather_idx, inv_pos, base, y, out, lse,)
    _contig(cu_seqlens, gather_idx, inv_pos, base, y, out, lse)
    return _dispatch(lib.spa_packed_attention_unpack,
                     (_ptr(q), _ptr(k), _ptr(v), _row_stride(q), _row_stride(k), _row_stride(v), _ptr(cu_seqlens),
                      _ptr(gather_idx), _ptr(inv_pos), _ptr(base), B, N, H, Dh, code, float(softmax_scale),
                      _ptr(out), _ptr(lse), _ptr(y), _stream(),), _keep, prepare)


def spa_gathered_attention_unpack(q, k, v, cu_seqlens, gather_idx, inv_pos, base, H, Dh, y, out=None, lse=None,
                                  softmax_scale=0.0, prepare=False):
    """spa_packed_attention_unpack on un-packed q, k, v ([B*N, H*Dh] tensors or column-slice views at
    token positions): the kernel fetches packed row j from row gather_idx[j]."""
    fn = "spa_gathered_attention_unpack"
    B, N, C = y.shape
    _, code = _scatter_checks(fn, q, k, v, cu_seqlens, B, N, gather_idx, inv_pos, base, H, Dh, y, out, lse)
    _rows(fn, C, q=(q, B * N), k=(k, B * N), v=(v, B * N))
    _keep = (q, k, v, cu_seqlens, gather_idx, inv_pos, base, y, out, lse,)
    _contig(cu_seqlens, gather_idx, inv_pos, base, y, out, lse)
    return _dispatch(lib.spa_gathered_attention_unpack,
                     (_ptr(q), _ptr(k), _ptr(v), _row_stride(q), _row_stride(k), _row_stride(v), _ptr(cu_seqlens),
                      _ptr(gather_idx), _ptr(inv_pos), _ptr(base), B, N, H, Dh, code, float(softmax_scale),
                      _ptr(out), _ptr(lse), _ptr(y), _stream(),), _keep, prepare)


def spa_selected_attention_unpack(q, k, v, mask, base, H, Dh, y, softmax_scale=0.0, prepare=False):
    """Attention over the selected tokens of every image straight from the mask (no packing index), scatter
    and bypass included: q, k, v [B*N, H*Dh] tensors or column-slice views at token positions, mask [B,N]
    uint8, y [B,N,C].  N <= 256."""
    fn = "spa_selected_attention_unpack"
    B, N, C = y.shape
    if C != H * Dh:
        raise ValueError(f"{fn}: y must be [B, N, H*Dh]")
    code = _features(fn, q=q, k=k, v=v, base=base, y=y)
    _typed(fn, torch.uint8, mask=mask)
    _rows(fn, C, q=(q, B * N), k=(k, B * N), v=(v, B * N))
    _holds(fn, mask=(mask, B * N), base=(base, B * N * C))
    _keep = (q, k, v, mask, base, y,)
    _contig(mask, base, y)
    return _dispatch(lib.spa_selected_attention_unpack,
                     (_ptr(q), _ptr(k), _ptr(v), _row_stride(q), _row_stride(k), _row_stride(v), _ptr(mask), _ptr(base),
                      B, N, H, Dh, code, float(softmax_scale), _ptr(y), _stream(),), _keep, prepare)


def spa_segment_attention_unpack(q, k, v, seg_cu_seqlens, max_seqlen, gather_idx, inv_pos, base, H, Dh, y, out=None,
                                 lse=None, softmax_scale=0.0, prepare=False):
    """Attention inside the segments of seg_cu_seqlens (not necessarily whole images) + scatter
    back to y [B,N,C] in one launch."""
    n_segments = seg_cu_seqlens.numel() - 1
    rows, code = _scatter_checks("spa_segment_attention_unpack", q, k, v, seg_cu_seqlens, n_segments, max_seqlen,
                                 gather_idx, inv_pos, base, H, Dh, y, out, lse)
    _keep = (q, k, v, seg_cu_seqlens, gather_idx, inv_pos, base, y, out, lse,)
    _contig(seg_cu_seqlens, gather_idx, inv_pos, base, y, out, lse)
    return _dispatch(lib.spa_segment_attention_unpack,
                     (_ptr(q), _ptr(k), _ptr(v), _row_stride(q), _row_stride(k), _row_stride(v), _ptr(seg_cu_seqlens),
                      n_segments, int(max_seqlen), _ptr(gather_idx), _ptr(inv_pos), _ptr(base), rows, H, Dh,
                      code, float(softmax_scale), _ptr(out), _ptr(lse), _ptr(y), _stream(),), _keep, prepare)


def spa_linear_packed(x, gather_idx, gate_scores, total, W, bias, out, prepare=False):
    """out[j] = (sigmoid(score) * x[gather_idx[j]]) W^T + bias for j < *total.  x [*, K] (any leading
    shape), W [N_out, K], out a [rows, N_out] tensor or column-slice view."""
    fn = "spa_linear_packed"
    K = x.shape[-1]
    N_out = W.shape[0]
    code = _features(fn, x=x, W=W, bias=bias, out=out)
    _typed(fn, torch.int32, gather_idx=gather_idx, total=total)
    _typed(fn, torch.float32, gate_scores=gate_scores)
    if W.shape[1] != K:
        raise ValueError(f"{fn}: W must be [N_out, K = {K}], got {tuple(W.shape)}")
    _rows(fn, N_out, out=(out, 1))
    _holds(fn, bias=(bias, N_out), gather_idx=(gather_idx, out.shape[0]), total=(total, 1))
    _keep = (x, gather_idx, gate_scores, total, W, bias,)
    _contig(*_keep)
    return _dispatch(lib.spa_linear_packed,
                     (_ptr(x), _ptr(gather_idx), _ptr(gate_scores), _ptr(total), _ptr(W), _ptr(bias), out.shape[0], K,
                      N_out, code, _ptr(out), _row_stride(out), _stream(),), _keep + (out,), prepare)


def spa_linear_packed_scatter(x, total, W, bias, scatter_idx, residual, y, prepare=False):
    """y[scatter_idx[j]] = residual[scatter_idx[j]] + x[j] W^T + bias for j < *total.  x [rows, K] packed,
    y / residual [*, N_out] (any leading shape, contiguous); y may be residual itself."""
    fn = "spa_linear_packed_scatter"
    K, N_out = x.shape[-1], W.shape[0]
    if y.shape[-1] != N_out or (residual is not None and residual.shape != y.shape):
        raise ValueError("y (and residual) must be [..., N_out]")
    code = _features(fn, x=x, W=W, bias=bias, residual=residual, y=y)
    _typed(fn, torch.int32, scatter_idx=scatter_idx, total=total)
    if W.shape[1] != K:
        raise ValueError(f"{fn}: W must be [N_out, K = {K}], got {tuple(W.shape)}")
    _holds(fn, bias=(bias, N_out), scatter_idx=(scatter_idx, min(x.shape[0], y.numel() // N_out)), total=(total, 1))
    _keep = (x, total, W, bias, scatter_idx, residual, y,)
    _contig(*_keep)
    return _dispatch(lib.spa_linear_packed_scatter,
                     (_ptr(x), _ptr(total), _ptr(W), _ptr(bias), x.shape[0], K, N_out, code, _ptr(scatter_idx),
                      _ptr(residual), _ptr(y), N_out, _stream(),), _keep, prepare)


def spa_linear_packed_bwd_input(dout, dout_idx, total, W, M_cap, dx_idx, inv_pos, dx, prepare=False):
    """dx[dx_idx[j] or j] = dout[dout_idx[j] or j] W for j < min(*total, M_cap).  dout [*, N_out] and dx
    [*, K] may be column-slice views; W [N_out, K].  inv_pos given: the rows of dx (all of its leading
    shape) that no packed row maps to are zeroed."""
    fn = "spa_linear_packed_bwd_input"
    N_out, K = W.shape
    rows = dx.numel() // dx.shape[-1] if inv_pos is not None else 0
    code = _features(fn, dout=dout, W=W, dx=dx)
    _typed(fn, torch.int32, dout_idx=dout_idx, total=total, dx_idx=dx_idx, inv_pos=inv_pos)
    _rows(fn, N_out, dout=(dout, 1 if dout_idx is not None else min(int(M_cap), dout.shape[0])))
    _rows(fn, K, dx=(dx, 1 if dx_idx is not None else int(M_cap)))
    _holds(fn, dout_idx=(dout_idx, int(M_cap)), dx_idx=(dx_idx, int(M_cap)), inv_pos=(inv_pos, rows), total=(total, 1))
    _keep = (dout_idx, total, W, dx_idx, inv_pos,)
    _contig(*_keep)
    return _dispatch(lib.spa_linear_packed_bwd_input,
                     (_ptr(dout), _ptr(dout_idx), _row_stride(dout), _ptr(total), _ptr(W), int(M_cap), K, N_out,
                      code, _ptr(dx_idx), _ptr(inv_pos), rows, _ptr(dx), _row_stride(dx), _stream(),),
                     _keep + (dout, dx,), prepare)


def spa_linear_bwd_weight_workspace_bytes(M_cap, K, N_out, dtype) -> int:
    return int(lib.spa_linear_bwd_weight_workspace_bytes(int(M_cap), int(K), int(N_out),
                                                          SPA_F32 if dtype in (torch.float32, "f32") else SPA_BF16))


def spa_linear_packed_bwd_weight(dout, dout_idx, x, x_idx, gate_scores, total, M_cap, dW, dbias, workspace=None,
                                 prepare=False):
    """dW [N_out, K] f32 = sum_j dout[dout_idx[j] or j]^T (sigmoid(score) x[x_idx[j] or j]), dbias [N_out] f32 =
    sum_j dout[...] over j < min(*total, M_cap).  dout may be a column-slice view; x [*, K] contiguous."""
    fn = "spa_linear_packed_bwd_weight"
    N_out, K = dW.shape
    code = _features(fn, dout=dout, x=x)
    _typed(fn, torch.int32, dout_idx=dout_idx, x_idx=x_idx, total=total)
    _typed(fn, torch.float32, gate_scores=gate_scores, dW=dW, dbias=dbias)
    if x.shape[-1] != K:
        raise ValueError(f"{fn}: x must be [*, K = {K}], got {tuple(x.shape)}")
    _rows(fn, N_out, dout=(dout, 1))
    _holds(fn, dout_idx=(dout_idx, int(M_cap)), x_idx=(x_idx, int(M_cap)), dbias=(dbias, N_out), total=(total, 1))
    _keep = (dout_idx, x, x_idx, gate_scores, total, dW, dbias, workspace,)
    _contig(*_keep)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    return _dispatch(lib.spa_linear_packed_bwd_weight,
                     (_ptr(dout), _ptr(dout_idx), _row_stride(dout), _ptr(x), _ptr(x_idx), _ptr(gate_scores), _ptr(total),
                      int(M_cap), K, N_out, code, _ptr(dW), _ptr(dbias), _ptr(workspace), ws_bytes, _stream(),),
                     _keep + (dout,), prepare)


def spa_ceiling_copy(src, dst, prepare=False):
    """Yardstick: dst = src with the library's plain copy kernel (uint8 / any dtype tensors of equal byte size)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() < nbytes:
        raise ValueError("spa_ceiling_copy: dst is smaller than src")
    _keep = (src, dst,)
    _contig(*_keep)
    return _dispatch(lib.spa_ceiling_copy, (_ptr(src), _ptr(dst), nbytes, _stream(),), _keep, prepare)


def spa_ceiling_mfma(sink, waves_per_simd, iters) -> float:
    """Yardstick: launches the MFMA-only loop; returns the flops issued."""
    fl = float(lib.spa_ceiling_mfma(_ptr(sink), int(waves_per_simd), int(iters), _stream()))
    if fl < 0:
        raise SpaError(-1, lib.spa_last_error().decode())
    return fl


def spa_unpack(packed_out, inv_pos, base, y, prepare=False):
    B, N, C = y.shape
    code = _features("spa_unpack", packed_out=packed_out, base=base, y=y)
    _typed("spa_unpack", torch.int32, inv_pos=inv_pos)
    _rows("spa_unpack", C, packed_out=(packed_out, 1))
    _holds("spa_unpack", inv_pos=(inv_pos, B * N), base=(base, B * N * C))
    _keep = (packed_out, inv_pos, base, y,)
    _contig(*_keep)
    return _dispatch(lib.spa_unpack, (_ptr(packed_out), _ptr(inv_pos), _ptr(base), B, N, C, code, _ptr(y), _stream(),), _keep, prepare)


def spa_unpack_bwd(dy, gather_idx, total, dout, prepare=False):
    B, N, C = dy.shape
    code = _features("spa_unpack_bwd", dy=dy, dout=dout)
    _typed("spa_unpack_bwd", torch.int32, gather_idx=gather_idx, total=total)
    _rows("spa_unpack_bwd", C, dout=(dout, B * N))
    _holds("spa_unpack_bwd", gather_idx=(gather_idx, B * N), total=(total, 1))
    _keep = (dy, gather_idx, total, dout,)
    _contig(*_keep)
    return _dispatch(lib.spa_unpack_bwd, (_ptr(dy), _ptr(gather_idx), _ptr(total), B, N, C, code, _ptr(dout), _stream(),), _keep, prepare)


def spa_pack_bwd(dpacked, inv_pos, d_rg, prepare=False):
    B, N, C = d_rg.shape
    code = _features("spa_pack_bwd", dpacked=dpacked, d_rg=d_rg)
    _typed("spa_pack_bwd", torch.int32, inv_pos=inv_pos)
    _rows("spa_pack_bwd", C, dpacked=(dpacked, 1))
    _holds("spa_pack_bwd", inv_pos=(inv_pos, B * N))
    _keep = (dpacked, inv_pos, d_rg,)
    _contig(*_keep)
    return _dispatch(lib.spa_pack_bwd, (_ptr(dpacked), _ptr(inv_pos), B, N, C, code, _ptr(d_rg), _stream(),), _keep, prepare)


def spa_attention_bwd_workspace_bytes(B, max_seqlen, H, Dh, dtype) -> int:
    return int(lib.spa_attention_bwd_workspace_bytes(B, max_seqlen, H, Dh, dtype))


def spa_packed_attention_bwd(q, k, v, out, dout, lse, cu_seqlens, B, max_seqlen, H, Dh,
                             dq, dk, dv, workspace, softmax_scale=0.0, prepare=False):
    fn = "spa_packed_attention_bwd"
    C = H * Dh
    code = _features(fn, q=q, k=k, v=v, out=out, dout=dout, dq=dq, dk=dk, dv=dv)
    _typed(fn, torch.int32, cu_seqlens=cu_seqlens)
    _typed(fn, torch.float32, lse=lse)
    _rows(fn, C, q=(q, 1), k=(k, 1), v=(v, 1), out=(out, 1), dout=(dout, 1), dq=(dq, 1), dk=(dk, 1), dv=(dv, 1))
    _holds(fn, cu_seqlens=(cu_seqlens, B + 1), lse=(lse, H * B * max_seqlen))
    _keep = (q, k, v, dq, dk, dv, out, dout, lse, cu_seqlens, workspace,)
    _contig(out, dout, lse, cu_seqlens, workspace)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    return _dispatch(lib.spa_packed_attention_bwd, (_ptr(q), _ptr(k), _ptr(v), _row_stride(q), _row_stride(k), _row_stride(v),
                                        _ptr(out), _ptr(dout), _ptr(lse), _ptr(cu_seqlens), B, max_seqlen, H, Dh,
                                        code, float(softmax_scale), _ptr(dq), _ptr(dk), _ptr(dv),
                                        _row_stride(dq), _row_stride(dk), _row_stride(dv), _ptr(workspace),
                                        ws_bytes, _stream(),), _keep, prepare)


def spa_packed_attention_bwd_tokens(q, k, v, out, dy, lse, cu_seqlens, B, max_seqlen, H, Dh, gather_idx, inv_pos,
                                    dq, dk, dv, workspace=None, softmax_scale=0.0, prepare=False):
    """unpack_bwd + attention backward + pack_bwd in one call: dy and dq, dk, dv at token positions
    (workspace: only for max_seqlen > 256)."""
    fn = "spa_packed_attention_bwd_tokens"
    C = H * Dh
    rows = dy.numel() // dy.shape[-1]
    code = _features(fn, q=q, k=k, v=v, out=out, dy=dy, dq=dq, dk=dk, dv=dv)
    _typed(fn, torch.int32, cu_seqlens=cu_seqlens, gather_idx=gather_idx, inv_pos=inv_pos)
    _typed(fn, torch.float32, lse=lse)
    if dy.shape[-1] != C:
        raise ValueError(f"{fn}: dy must be [..., H*Dh]")
    _rows(fn, C, q=(q, 1), k=(k, 1), v=(v, 1), out=(out, 1), dq=(dq, rows), dk=(dk, rows), dv=(dv, rows))
    _holds(fn, cu_seqlens=(cu_seqlens, B + 1), lse=(lse, H * B * max_seqlen), gather_idx=(gather_idx, rows),
           inv_pos=(inv_pos, rows))
    _keep = (q, k, v, dq, dk, dv, out, dy, lse, cu_seqlens, gather_idx, inv_pos, workspace,)
    _contig(out, dy, lse, cu_seqlens, gather_idx, inv_pos, workspace)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    return _dispatch(lib.spa_packed_attention_bwd_tokens,
                     (_ptr(q), _ptr(k), _ptr(v), _row_stride(q), _row_stride(k), _row_stride(v), _ptr(out), _ptr(dy),
                      _ptr(lse), _ptr(cu_seqlens), B, max_seqlen, H, Dh, code, float(softmax_scale),
                      _ptr(gather_idx), _ptr(inv_pos), rows, _ptr(dq), _ptr(dk), _ptr(dv), _row_stride(dq),
                      _row_stride(dk), _row_stride(dv), _ptr(workspace), ws_bytes, _stream(),), _keep, prepare)


def spa_gate_bwd_workspace_bytes(B, N, C, dtype) -> int:
    return int(lib.spa_gate_bwd_workspace_bytes(B, N, C, dtype))


def _gate_bwd_checks(fn, x, w, scores, s_up, labels, d_rg, mask, noise, loss, dx, dw, db):
    B, N, C = x.shape
    code = _features(fn, x=x, w=w, d_rg=d_rg, dx=dx)
    _typed(fn, torch.float32, scores=scores, s_up=s_up, noise=noise, loss=loss, dw=dw, db=db)
    _typed(fn, torch.uint8, labels=labels, mask=mask)
    cap = B * N
    _holds(fn, w=(w, C), scores=(scores, cap), s_up=(s_up, cap), noise=(noise, cap), labels=(labels, cap),
           mask=(mask, cap), d_rg=(d_rg, cap * C), dx=(dx, cap * C), dw=(dw, C), db=(db, 1), loss=(loss, 1))
    return B, N, C, code


def spa_gate_bwd(x, w, bias, scores, s_up, labels, d_rg, gate_scaled, loss_scale, loss, dx, dw, db, workspace,
                 prepare=False):
    B, N, C, code = _gate_bwd_checks("spa_gate_bwd", x, w, scores, s_up, labels, d_rg, None, None, loss, dx, dw, db)
    _keep = (x, w, scores, s_up, labels, d_rg, loss, dx, dw, db, workspace,)
    _contig(*_keep)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    return _dispatch(lib.spa_gate_bwd, (_ptr(x), _ptr(w), float(bias), _ptr(scores), _ptr(s_up), _ptr(labels), _ptr(d_rg),
                            int(bool(gate_scaled)), float(loss_scale), B, N, C, code, _ptr(loss), _ptr(dx),
                            _ptr(dw), _ptr(db), _ptr(workspace), ws_bytes, _stream(),), _keep, prepare)


def spa_gate_bwd_static(x, w, bias, scores, s_up, labels, d_rg, gate_scaled, loss_scale, loss, dx, dw, db,
                        prepare=False):
    """spa_gate_bwd without a workspace argument: the reduction's scratch is a device array built
    into the library (C <= 1024); the call allocates nothing."""
    B, N, C, code = _gate_bwd_checks("spa_gate_bwd_static", x, w, scores, s_up, labels, d_rg, None, None, loss, dx,
                                     dw, db)
    _keep = (x, w, scores, s_up, labels, d_rg, loss, dx, dw, db,)
    _contig(*_keep)
    return _dispatch(lib.spa_gate_bwd_static,
                     (_ptr(x), _ptr(w), float(bias), _ptr(scores), _ptr(s_up), _ptr(labels), _ptr(d_rg),
                      int(bool(gate_scaled)), float(loss_scale), B, N, C, code, _ptr(loss), _ptr(dx), _ptr(dw),
                      _ptr(db), _stream(),), _keep, prepare)


def spa_gate_bwd_straight_through(x, w, bias, scores, s_up, labels, d_rg, loss_scale, mask, noise, temperature,
                                  loss, dx, dw, db, workspace, prepare=False):
    B, N, C, code = _gate_bwd_checks("spa_gate_bwd_straight_through", x, w, scores, s_up, labels, d_rg, mask, noise,
                                     loss, dx, dw, db)
    _keep = (x, w, scores, s_up, labels, d_rg, mask, noise, loss, dx, dw, db, workspace,)
    _contig(*_keep)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    return _dispatch(lib.spa_gate_bwd_straight_through,
                     (_ptr(x), _ptr(w), float(bias), _ptr(scores), _ptr(s_up), _ptr(labels), _ptr(d_rg),
                      float(loss_scale), _ptr(mask), _ptr(noise), float(temperature), B, N, C, code,
                      _ptr(loss), _ptr(dx), _ptr(dw), _ptr(db), _ptr(workspace), ws_bytes, _stream(),), _keep, prepare)


def spa_padded_attention(q, k, v, seqlens, B, n_pad, H, Dh, out, softmax_scale=0.0, prepare=False):
    fn = "spa_padded_attention"
    code = _features(fn, q=q, k=k, v=v, out=out)
    _typed(fn, torch.int32, seqlens=seqlens)
    _rows(fn, H * Dh, q=(q, B * n_pad), k=(k, B * n_pad), v=(v, B * n_pad))
    _holds(fn, seqlens=(seqlens, B), out=(out, B * n_pad * H * Dh))
    _keep = (q, k, v, out, seqlens,)
    _contig(out, seqlens)
    if not (_row_stride(q) == _row_stride(k) == _row_stride(v)):
        raise ValueError("spa_padded_attention takes one row stride for q, k, v")
    return _dispatch(lib.spa_padded_attention, (_ptr(q), _ptr(k), _ptr(v), _row_stride(q), _ptr(seqlens), B, n_pad, H, Dh,
                                    code, float(softmax_scale), _ptr(out), _stream(),), _keep, prepare)
