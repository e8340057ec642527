"""Buffer owners for the SPA hot path: they allocate the device tensors once and issue the
C-ABI calls of one forward (or forward + backward) pass in order.  No arithmetic happens
here; every step runs in libspa's HIP kernels on the current stream, without host syncs.

Order of the forward pass (Section 3.2): gate score -> hard selection -> pack ->
per-image attention on the packed tokens -> scatter back.  The projected q | k | v of every
token are supplied by the caller as one fused [B, N, 3C] tensor (the projections are not
part of this path) and are packed with the gate's mask.
"""
from __future__ import annotations

from typing import Callable, List, Optional, Tuple

import torch

from . import spa


def _td(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


class ForwardPass:
    """gate_select(x) -> pack(qkv) -> packed_attention -> unpack.

    fused_unpack=True (default) issues the last two steps as ONE launch
    (spa_packed_attention_unpack: the attention kernel scatters its rows back itself and
    fills the bypassing rows); the results are bit-identical to the two separate calls.
    gathered=True (fused form only): packing builds the index only and the attention kernel
    fetches the q | k | v rows through gather_idx from where they lie, so no row is copied
    (spa_pack with x = NULL, then spa_gathered_attention_unpack); same results, bit for bit.
    from_mask=True (with gathered; N <= 256, forward only): no packing launch at all, the attention
    kernel derives each image's packing order from the mask (spa_selected_attention_unpack): two launches
    per step, same y bit for bit; cu_seqlens, gather_idx, inv_pos and total are NOT produced."""

    def __init__(self, B: int, N: int, C: int, H: int, dtype: str, tau: float = 0.5, bias: float = 0.0,
                 container_len: int = 0, fused_unpack: bool = True, keep_packed_out: bool = True,
                 gathered: bool = False, fused_index: bool = False, from_mask: bool = False):
        """keep_packed_out=False (fused form only): the packed attention output and the
        log-sum-exp rows, which only a backward pass reads, are not written; y is the result.
        fused_index=True (with gathered): the gate launch builds the packing index itself
        (spa_gate_select_index), two launches per step."""
        if gathered and (not fused_unpack or container_len):
            raise ValueError("gathered=True needs the fused form and no container padding")
        if fused_index and not gathered:
            raise ValueError("fused_index=True needs gathered=True")
        if from_mask and not (gathered and not fused_index and not keep_packed_out and N <= 256):
            raise ValueError("from_mask=True needs gathered=True, keep_packed_out=False and N <= 256")
        self.gathered, self.fused_index, self.from_mask = gathered, fused_index, from_mask
        self.ws_index = torch.zeros(17 * 1088, dtype=torch.int32, device="cuda") if fused_index else None
        self.B, self.N, self.C, self.H, self.Dh = B, N, C, H, C // H
        self.tau, self.bias, self.container_len = tau, bias, container_len
        self.fused_unpack = fused_unpack
        self.keep_packed_out = keep_packed_out or not fused_unpack
        td, cap = _td(dtype), B * N
        dv = dict(device="cuda")
        self.scores = torch.empty(B, N, dtype=torch.float32, **dv)
        self.mask = torch.empty(B, N, dtype=torch.uint8, **dv)
        self.packed_qkv = None if gathered else torch.zeros(cap + max(container_len - 1, 0), 3 * C, dtype=td, **dv)
        self.cu_seqlens = torch.zeros(B + 1, dtype=torch.int32, **dv)
        self.gather_idx = torch.zeros(cap, dtype=torch.int32, **dv)
        self.inv_pos = torch.zeros(cap, dtype=torch.int32, **dv)
        self.total = torch.zeros(1, dtype=torch.int32, **dv)
        self.out = torch.zeros(cap, C, dtype=td, **dv) if self.keep_packed_out else None
        self.lse = torch.zeros(H, cap, dtype=torch.float32, **dv) if self.keep_packed_out else None
        self.y = torch.empty(B, N, C, dtype=td, **dv)

    def stages(self, x, w, qkv, s_up=None, base=None) -> List[Tuple[str, Callable[[], None]]]:
        """The pass as named, prepared launches (bound to the stream that is current now), so a
        caller can time each of them or replay them with no marshalling cost."""
        C, p = self.C, self.packed_qkv
        if self.from_mask:
            t = qkv.view(self.B * self.N, 3 * C)
            return [
                ("gate_select", spa.spa_gate_select(x, w, self.bias, s_up, self.tau, self.scores, self.mask, None,
                                                    prepare=True)),
                ("selected_attention_unpack", spa.spa_selected_attention_unpack(
                    t[:, :C], t[:, C:2 * C], t[:, 2 * C:], self.mask, base, self.H, self.Dh, self.y, prepare=True)),
            ]
        if self.gathered:
            t = qkv.view(self.B * self.N, 3 * C)
            head = [
                ("gate_select_index", spa.spa_gate_select_index(x, w, self.bias, s_up, self.tau, self.scores, self.mask,
                                                                None, self.cu_seqlens, self.gather_idx, self.inv_pos,
                                                                self.total, self.ws_index, prepare=True)),
            ] if self.fused_index else [
                ("gate_select", spa.spa_gate_select(x, w, self.bias, s_up, self.tau, self.scores, self.mask, None,
                                                    prepare=True)),
                ("pack_indices", spa.spa_pack(None, self.mask, None, None, 0, None, self.cu_seqlens, self.gather_idx,
                                              self.inv_pos, self.total, prepare=True)),
            ]
            return head + [
                ("gathered_attention_unpack", spa.spa_gathered_attention_unpack(
                    t[:, :C], t[:, C:2 * C], t[:, 2 * C:], self.cu_seqlens, self.gather_idx, self.inv_pos, base,
                    self.H, self.Dh, self.y, self.out, self.lse, prepare=True)),
            ]
        q, k, v = p[:, :C], p[:, C:2 * C], p[:, 2 * C:]
        head = [
            ("gate_select", spa.spa_gate_select(x, w, self.bias, s_up, self.tau, self.scores, self.mask, None,
                                                prepare=True)),
            ("pack", spa.spa_pack(qkv, self.mask, None, None, self.container_len, p, self.cu_seqlens,
                                  self.gather_idx, self.inv_pos, self.total, prepare=True)),
        ]
        if self.fused_unpack:
            return head + [
                ("packed_attention_unpack", spa.spa_packed_attention_unpack(
                    q, k, v, self.cu_seqlens, self.gather_idx, self.inv_pos, base, self.H, self.Dh, self.y,
                    self.out if self.keep_packed_out else None, self.lse if self.keep_packed_out else None,
                    prepare=True)),
            ]
        return head + [
            ("packed_attention", spa.spa_packed_attention(q, k, v, self.cu_seqlens, self.B, self.N, self.H,
                                                          self.Dh, self.out, self.lse, prepare=True)),
            ("unpack", spa.spa_unpack(self.out, self.inv_pos, base, self.y, prepare=True)),
        ]

    def run(self, x, w, qkv, s_up=None, base=None):
        for _, fn in self.stages(x, w, qkv, s_up, base):
            fn()
        return self.y


class TrainPass:
    """Forward + backward of one SPA block with the selection loss (Section 3.3).

    q | k are supplied ([B, N, 2C], stand-ins for projected tokens); v is the packed gated
    representation r_g = Sigmoid(s) . r, so the gate receives the attention's gradient:
      fwd: gate_select(x) -> pack(qk) -> pack(x, scaled by sigmoid(s)) -> attention + unpack (one launch)
      bwd: unpack_bwd(dy) -> attention_bwd -> pack_bwd(dv) [-> pack_bwd(dq|dk)] -> gate_bwd
    fused_bwd (default): the gather of dy and the scatters of dq, dk, dv run inside the
    attention backward, 6 calls instead of 9.
    pack_pair (default): q|k and the gated x are packed by one launch (the survivors are counted
    and ranked once), 5 calls.
    """

    def __init__(self, B: int, N: int, C: int, H: int, dtype: str, tau: float = 0.5, bias: float = 0.0,
                 loss_scale: Optional[float] = None, fused_bwd: Optional[bool] = None, pack_pair: bool = True):
        self.B, self.N, self.C, self.H, self.Dh = B, N, C, H, C // H
        self.fused_bwd = True if fused_bwd is None else fused_bwd
        self.pack_pair = pack_pair
        self.tau, self.bias = tau, bias
        self.loss_scale = 0.01 / (B * N) if loss_scale is None else loss_scale
        td, cap = _td(dtype), B * N
        code = spa.SPA_BF16 if dtype == "bf16" else spa.SPA_F32
        dv = dict(device="cuda")
        self.scores = torch.empty(B, N, dtype=torch.float32, **dv)
        self.mask = torch.empty(B, N, dtype=torch.uint8, **dv)
        self.packed_qk = torch.zeros(cap, 2 * C, dtype=td, **dv)
        self.packed_v = torch.zeros(cap, C, dtype=td, **dv)
        self.cu_seqlens = torch.zeros(B + 1, dtype=torch.int32, **dv)
        self.gather_idx = torch.zeros(cap, dtype=torch.int32, **dv)
        self.inv_pos = torch.zeros(cap, dtype=torch.int32, **dv)
        self.total = torch.zeros(1, dtype=torch.int32, **dv)
        self.out = torch.zeros(cap, C, dtype=td, **dv)
        self.lse = torch.zeros(H, cap, dtype=torch.float32, **dv)
        self.y = torch.empty(B, N, C, dtype=td, **dv)
        self.dout = torch.zeros(cap, C, dtype=td, **dv)
        self.dqk_packed = torch.zeros(cap, 2 * C, dtype=td, **dv)
        self.dv_packed = torch.zeros(cap, C, dtype=td, **dv)
        self.d_rg = torch.empty(B, N, C, dtype=td, **dv)
        self.dqk = torch.empty(B, N, 2 * C, dtype=td, **dv)
        self.dx = torch.empty(B, N, C, dtype=td, **dv)
        self.dw = torch.empty(C, dtype=torch.float32, **dv)
        self.db = torch.empty(1, dtype=torch.float32, **dv)
        self.loss = torch.empty(1, dtype=torch.float32, **dv)
        self.ws_attn = torch.empty(max(spa.spa_attention_bwd_workspace_bytes(B, N, H, self.Dh, code), 256),
                                   dtype=torch.uint8, **dv)
        self.ws_gate = torch.empty(max(spa.spa_gate_bwd_workspace_bytes(B, N, C, code), 256), dtype=torch.uint8, **dv)

    def stages(self, x, w, qk, labels, dy, noise=None, temperature: float = 1.0, s_fine=None, grid=None
               ) -> List[Tuple[str, Callable[[], None]]]:
        """noise [B,N] f32 (logistic variates) switches the selection to the stochastic
        Gumbel-Softmax form and the gate backward to its straight-through estimator.
        s_fine [B, 4N] f32 with grid = (grid_h, grid_w): the score map of the 2x finer stage of a
        hierarchy; it is max-pooled inside the gate kernel and the pooled map is the s_up of the
        gate backward (no gradient to this stage's gate where the up-scale score won)."""
        st = self._stages(x, w, qk, labels, dy)
        if s_fine is not None:
            if noise is not None:
                raise ValueError("s_fine and noise together are not wired up")
            self.s_up = torch.empty(self.B, self.N, dtype=torch.float32, device="cuda")
            st[0] = ("gate_select_pooled", spa.spa_gate_select_pooled(
                x, w, self.bias, s_fine, grid[0], grid[1], self.tau, self.scores, self.mask, None, self.s_up,
                prepare=True))
            st[-1] = ("gate_bwd", spa.spa_gate_bwd(x, w, self.bias, self.scores, self.s_up, labels, self.d_rg, True,
                                                   self.loss_scale, self.loss, self.dx, self.dw, self.db, self.ws_gate,
                                                   prepare=True))
            return st
        if noise is None:
            return st
        st[0] = ("gate_select_gumbel", spa.spa_gate_select_gumbel(x, w, self.bias, None, noise, temperature, self.tau,
                                                                  self.scores, self.mask, None, prepare=True))
        st[-1] = ("gate_bwd_straight_through", spa.spa_gate_bwd_straight_through(
            x, w, self.bias, self.scores, None, labels, self.d_rg, self.loss_scale, self.mask, noise, temperature,
            self.loss, self.dx, self.dw, self.db, self.ws_gate, prepare=True))
        return st

    def _stages(self, x, w, qk, labels, dy) -> List[Tuple[str, Callable[[], None]]]:
        C = self.C
        pq, pk, pv = self.packed_qk[:, :C], self.packed_qk[:, C:], self.packed_v
        dq, dk = self.dqk_packed[:, :C], self.dqk_packed[:, C:]
        B, N, H, Dh = self.B, self.N, self.H, self.Dh
        if self.fused_bwd:
            dqk_tok = self.dqk.view(B * N, 2 * C)
            attention_bwd = [("packed_attention_bwd_tokens", spa.spa_packed_attention_bwd_tokens(
                pq, pk, pv, self.out, dy, self.lse, self.cu_seqlens, B, N, H, Dh, self.gather_idx, self.inv_pos,
                dqk_tok[:, :C], dqk_tok[:, C:], self.d_rg.view(B * N, C), self.ws_attn, prepare=True))]
        else:
            attention_bwd = [
                ("unpack_bwd", spa.spa_unpack_bwd(dy, self.gather_idx, self.total, self.dout, prepare=True)),
                ("packed_attention_bwd", spa.spa_packed_attention_bwd(
                    pq, pk, pv, self.out, self.dout, self.lse, self.cu_seqlens, B, N, H, Dh, dq, dk, self.dv_packed,
                    self.ws_attn, prepare=True)),
                ("pack_bwd_v", spa.spa_pack_bwd(self.dv_packed, self.inv_pos, self.d_rg, prepare=True)),
                ("pack_bwd_qk", spa.spa_pack_bwd(self.dqk_packed, self.inv_pos, self.dqk, prepare=True)),
            ]
        return [
            ("gate_select", spa.spa_gate_select(x, w, self.bias, None, self.tau, self.scores, self.mask, None, prepare=True)),
            *([("pack_qk_rg", spa.spa_pack_pair(qk, x, self.mask, None, self.scores, self.packed_qk, self.packed_v,
                                                self.cu_seqlens, self.gather_idx, self.inv_pos, self.total,
                                                prepare=True))] if self.pack_pair else [
                ("pack_qk", spa.spa_pack(qk, self.mask, None, None, 0, self.packed_qk, self.cu_seqlens,
                                         self.gather_idx, self.inv_pos, self.total, prepare=True)),
                ("pack_rg", spa.spa_pack(x, self.mask, None, self.scores, 0, self.packed_v, None, None, None, None,
                                         prepare=True))]),
            ("packed_attention_unpack", spa.spa_packed_attention_unpack(
                pq, pk, pv, self.cu_seqlens, self.gather_idx, self.inv_pos, None, H, Dh, self.y, self.out, self.lse,
                prepare=True)),
            *attention_bwd,
            ("gate_bwd", spa.spa_gate_bwd(x, w, self.bias, self.scores, None, labels, self.d_rg, True,
                                                  self.loss_scale, self.loss, self.dx, self.dw, self.db, self.ws_gate,
                                          prepare=True)),
        ]

    def run(self, x, w, qk, labels, dy):
        for _, fn in self.stages(x, w, qk, labels, dy):
            fn()
        return self.loss


class BlockPass:
    """One SPA attention block with its projections (Section 3.2), six launches:

      gate_select(x) -> pack (indices only) -> QKV projection of the selected, gated tokens
      (gather and Sigmoid(s) scaling folded into the GEMM's operand load) -> packed attention
      -> output projection on the packed rows -> scatter back as a residual on x (unselected tokens keep x unchanged).

    Only selected tokens are ever projected, which is where the method saves its FLOPs.

    in_place=True: five launches.  The output projection scatters its rows straight into the
    residual stream x (x[token] += projection), so there is no scatter launch and no copy of the
    bypassing tokens; run() then returns x itself."""

    def __init__(self, B: int, N: int, C: int, H: int, dtype: str, tau: float = 0.5, bias: float = 0.0,
                 in_place: bool = False):
        self.B, self.N, self.C, self.H, self.Dh = B, N, C, H, C // H
        self.tau, self.bias, self.in_place = tau, bias, in_place
        td, cap = _td(dtype), B * N
        dv = dict(device="cuda")
        self.scores = torch.empty(B, N, dtype=torch.float32, **dv)
        self.mask = torch.empty(B, N, dtype=torch.uint8, **dv)
        self.cu_seqlens = torch.zeros(B + 1, dtype=torch.int32, **dv)
        self.gather_idx = torch.zeros(cap, dtype=torch.int32, **dv)
        self.inv_pos = torch.zeros(cap, dtype=torch.int32, **dv)
        self.total = torch.zeros(1, dtype=torch.int32, **dv)
        self.packed_qkv = torch.zeros(cap, 3 * C, dtype=td, **dv)
        self.attn = torch.zeros(cap, C, dtype=td, **dv)
        self.proj = torch.zeros(cap, C, dtype=td, **dv)
        self.y = torch.empty(B, N, C, dtype=td, **dv)

    def stages(self, x, w, W_qkv, b_qkv, W_o, b_o) -> List[Tuple[str, Callable[[], None]]]:
        C, p = self.C, self.packed_qkv
        return [
            ("gate_select", spa.spa_gate_select(x, w, self.bias, None, self.tau, self.scores, self.mask, None,
                                                prepare=True)),
            ("pack_indices", spa.spa_pack(None, self.mask, None, None, 0, None, self.cu_seqlens, self.gather_idx,
                                          self.inv_pos, self.total, prepare=True)),
            ("qkv_projection", spa.spa_linear_packed(x, self.gather_idx, self.scores, self.total, W_qkv, b_qkv, p,
                                                     prepare=True)),
            ("packed_attention", spa.spa_packed_attention(p[:, :C], p[:, C:2 * C], p[:, 2 * C:], self.cu_seqlens,
                                                          self.B, self.N, self.H, self.Dh, self.attn, None,
                                                          prepare=True)),
        ] + ([
            ("out_projection_scatter", spa.spa_linear_packed_scatter(self.attn, self.total, W_o, b_o, self.gather_idx,
                                                                     x, x, prepare=True)),
        ] if self.in_place else [
            ("out_projection", spa.spa_linear_packed(self.attn, None, None, self.total, W_o, b_o, self.proj,
                                                     prepare=True)),
            ("unpack", spa.spa_unpack(self.proj, self.inv_pos, x, self.y, prepare=True)),
        ])

    def run(self, x, w, W_qkv, b_qkv, W_o, b_o):
        for _, fn in self.stages(x, w, W_qkv, b_qkv, W_o, b_o):
            fn()
        return x if self.in_place else self.y


class BlockTrainPass:
    """Forward + backward of one SPA attention block WITH its projections (Section 3.2) and the
    selection loss (Section 3.3), twelve launches:

      fwd: gate_select(x) -> pack (indices only) -> QKV projection of the selected, gated tokens
           -> packed attention -> output projection of the packed rows -> scatter back as a
           residual on x (y[token] = x[token] + projection, bypassing tokens y = x; x stays
           intact for the backward pass)
      bwd: (dy at token positions) -> input side and weight side of the output projection (dy
           gathered inside the GEMMs) -> attention backward on the packed rows -> input side of
           the QKV projection, scattering d_rg to token positions with the unselected rows
           cleared, and its weight side (x gathered and gate-scaled inside the GEMM) -> gate
           backward with the selection loss.
    Results: dW_qkv, db_qkv, dW_o, db_o, dw, db (fp32), loss, and dx = the gradient that reaches x
    through the gate and the gated representation; the residual path adds dy itself to it, which
    is left to the caller (it is the upstream gradient, unchanged).

    overlap_weight_grads (default): nothing downstream in the step reads dW / dbias, so the two
    weight-side GEMMs are enqueued on a second HIP stream (default priority) and run beside the
    attention backward, the input-side GEMM and the gate backward; events order them after
    their inputs and the step's last stage joins the streams."""

    def __init__(self, B: int, N: int, C: int, H: int, dtype: str, tau: float = 0.5, bias: float = 0.0,
                 loss_scale: Optional[float] = None, overlap_weight_grads: bool = True):
        self.overlap = overlap_weight_grads
        self.side = torch.cuda.Stream() if overlap_weight_grads else None
        self.B, self.N, self.C, self.H, self.Dh = B, N, C, H, C // H
        self.tau, self.bias = tau, bias
        self.loss_scale = 0.01 / (B * N) if loss_scale is None else loss_scale
        td, cap = _td(dtype), B * N
        code = spa.SPA_BF16 if dtype == "bf16" else spa.SPA_F32
        dv = dict(device="cuda")
        f32 = dict(dtype=torch.float32, device="cuda")
        self.scores = torch.empty(B, N, **f32)
        self.mask = torch.empty(B, N, dtype=torch.uint8, **dv)
        self.cu_seqlens = torch.zeros(B + 1, dtype=torch.int32, **dv)
        self.gather_idx = torch.zeros(cap, dtype=torch.int32, **dv)
        self.inv_pos = torch.zeros(cap, dtype=torch.int32, **dv)
        self.total = torch.zeros(1, dtype=torch.int32, **dv)
        self.packed_qkv = torch.zeros(cap, 3 * C, dtype=td, **dv)
        self.attn = torch.zeros(cap, C, dtype=td, **dv)
        self.lse = torch.zeros(H, cap, **f32)
        self.proj = torch.zeros(cap, C, dtype=td, **dv)
        self.y = torch.empty(B, N, C, dtype=td, **dv)
        self.d_attn = torch.zeros(cap, C, dtype=td, **dv)
        self.d_qkv = torch.zeros(cap, 3 * C, dtype=td, **dv)
        self.d_rg = torch.empty(B, N, C, dtype=td, **dv)
        self.dx = torch.empty(B, N, C, dtype=td, **dv)
        self.dW_qkv, self.db_qkv = torch.empty(3 * C, C, **f32), torch.empty(3 * C, **f32)
        self.dW_o, self.db_o = torch.empty(C, C, **f32), torch.empty(C, **f32)
        self.dw, self.db, self.loss = torch.empty(C, **f32), torch.empty(1, **f32), torch.empty(1, **f32)
        u8 = lambda n: torch.empty(max(n, 256), dtype=torch.uint8, **dv)
        self.ws_attn = u8(spa.spa_attention_bwd_workspace_bytes(B, N, H, self.Dh, code))
        self.ws_gate = u8(spa.spa_gate_bwd_workspace_bytes(B, N, C, code))
        self.ws_qkv = u8(spa.spa_linear_bwd_weight_workspace_bytes(cap, C, 3 * C, dtype))
        self.ws_o = u8(spa.spa_linear_bwd_weight_workspace_bytes(cap, C, C, dtype))

    def stages(self, x, w, W_qkv, b_qkv, W_o, b_o, labels, dy) -> List[Tuple[str, Callable[[], None]]]:
        B, N, C, H, Dh = self.B, self.N, self.C, self.H, self.Dh
        cap, p, dp = B * N, self.packed_qkv, self.d_qkv
        dy2 = dy.view(cap, C)
        main = torch.cuda.current_stream()

        def weight_side():
            return (spa.spa_linear_packed_bwd_weight(dy2, self.gather_idx, self.attn, None, None, self.total, cap,
                                                     self.dW_o, self.db_o, self.ws_o, prepare=True),
                    spa.spa_linear_packed_bwd_weight(dp, None, x, self.gather_idx, self.scores, self.total, cap,
                                                     self.dW_qkv, self.db_qkv, self.ws_qkv, prepare=True))

        if self.overlap:
            with torch.cuda.stream(self.side):             # the prepared calls keep the stream they were made on
                w_o, w_qkv = weight_side()
            events = [torch.cuda.Event() for _ in range(3)]

            def on_side(ev, call):
                def go():
                    ev.record(main)                        # inputs of the GEMM are complete on the main stream
                    self.side.wait_event(ev)
                    call()
                return go

            def join():
                events[2].record(self.side)
                main.wait_event(events[2])

            w_o, w_qkv = on_side(events[0], w_o), on_side(events[1], w_qkv)
        else:
            w_o, w_qkv = weight_side()
        return [
            ("gate_select", spa.spa_gate_select(x, w, self.bias, None, self.tau, self.scores, self.mask, None,
                                                prepare=True)),
            ("pack_indices", spa.spa_pack(None, self.mask, None, None, 0, None, self.cu_seqlens, self.gather_idx,
                                          self.inv_pos, self.total, prepare=True)),
            ("qkv_projection", spa.spa_linear_packed(x, self.gather_idx, self.scores, self.total, W_qkv, b_qkv, p,
                                                     prepare=True)),
            ("packed_attention", spa.spa_packed_attention(p[:, :C], p[:, C:2 * C], p[:, 2 * C:], self.cu_seqlens, B, N,
                                                          H, Dh, self.attn, self.lse, prepare=True)),
            ("out_projection", spa.spa_linear_packed(self.attn, None, None, self.total, W_o, b_o, self.proj,
                                                     prepare=True)),
            ("unpack", spa.spa_unpack(self.proj, self.inv_pos, x, self.y, prepare=True)),
            ("out_projection_bwd_weight", w_o),
            ("out_projection_bwd_input", spa.spa_linear_packed_bwd_input(dy2, self.gather_idx, self.total, W_o, cap,
                                                                         None, None, self.d_attn, prepare=True)),
            ("packed_attention_bwd", spa.spa_packed_attention_bwd(
                p[:, :C], p[:, C:2 * C], p[:, 2 * C:], self.attn, self.d_attn, self.lse, self.cu_seqlens, B, N, H, Dh,
                dp[:, :C], dp[:, C:2 * C], dp[:, 2 * C:], self.ws_attn, prepare=True)),
            ("qkv_projection_bwd_weight", w_qkv),
            ("qkv_projection_bwd_input", spa.spa_linear_packed_bwd_input(dp, None, self.total, W_qkv, cap,
                                                                         self.gather_idx, self.inv_pos,
                                                                         self.d_rg.view(cap, C), prepare=True)),
            ("gate_bwd", spa.spa_gate_bwd(x, w, self.bias, self.scores, None, labels, self.d_rg, True, self.loss_scale,
                                          self.loss, self.dx, self.dw, self.db, self.ws_gate, prepare=True)),
        ] + ([("join_streams", join)] if self.overlap else [])

    def run(self, x, w, W_qkv, b_qkv, W_o, b_o, labels, dy):
        for _, fn in self.stages(x, w, W_qkv, b_qkv, W_o, b_o, labels, dy):
            fn()
        return self.loss


class ContainerForwardPass:
    """The forward pass with the paper's container mask (Section 3.2 "Token Packing"): the
    packed stream is cut into containers of length L and a token attends to the tokens of its
    own image inside its own container; shift = (sh, sw) packs the cyclically shifted map.

      gate_select(x) -> pack_shifted(qkv) -> container_segments -> attention on the image x
      container segments + scatter back (one launch; fused_unpack=False: two).  No host sync."""

    def __init__(self, B: int, grid_h: int, grid_w: int, C: int, H: int, dtype: str, container_len: int,
                 shift: Tuple[int, int] = (0, 0), tau: float = 0.5, bias: float = 0.0, fused_unpack: bool = True):
        self.fused_unpack = fused_unpack
        N = grid_h * grid_w
        self.B, self.N, self.C, self.H, self.Dh = B, N, C, H, C // H
        self.grid, self.shift, self.L, self.tau, self.bias = (grid_h, grid_w), shift, container_len, tau, bias
        td, cap = _td(dtype), B * N
        dv = dict(device="cuda")
        self.scores = torch.empty(B, N, dtype=torch.float32, **dv)
        self.mask = torch.empty(B, N, dtype=torch.uint8, **dv)
        self.packed_qkv = torch.zeros(cap + container_len - 1, 3 * C, dtype=td, **dv)
        self.cu_seqlens = torch.zeros(B + 1, dtype=torch.int32, **dv)
        self.gather_idx = torch.zeros(cap, dtype=torch.int32, **dv)
        self.inv_pos = torch.zeros(cap, dtype=torch.int32, **dv)
        self.total = torch.zeros(1, dtype=torch.int32, **dv)
        self.seg_cap = spa.spa_container_segments_capacity(B, cap, container_len)
        self.max_seqlen = min(container_len, N)
        self.seg_cu_seqlens = torch.zeros(self.seg_cap + 1, dtype=torch.int32, **dv)
        self.n_segments = torch.zeros(1, dtype=torch.int32, **dv)
        self.out = torch.zeros(cap, C, dtype=td, **dv)
        self.y = torch.empty(B, N, C, dtype=td, **dv)

    def stages(self, x, w, qkv, base=None) -> List[Tuple[str, Callable[[], None]]]:
        C, p = self.C, self.packed_qkv
        return [
            ("gate_select", spa.spa_gate_select(x, w, self.bias, None, self.tau, self.scores, self.mask, None,
                                                prepare=True)),
            ("pack_shifted", spa.spa_pack_shifted(qkv, self.mask, None, None, self.grid[0], self.grid[1],
                                                  self.shift[0], self.shift[1], self.L, p, self.cu_seqlens,
                                                  self.gather_idx, self.inv_pos, self.total, prepare=True)),
            ("container_segments", spa.spa_container_segments(self.cu_seqlens, self.L, self.B * self.N,
                                                              self.seg_cu_seqlens, self.n_segments, prepare=True)),
        ] + ([
            ("segment_attention_unpack", spa.spa_segment_attention_unpack(
                p[:, :C], p[:, C:2 * C], p[:, 2 * C:], self.seg_cu_seqlens, self.max_seqlen, self.gather_idx,
                self.inv_pos, base, self.H, self.Dh, self.y, None, None, prepare=True)),
        ] if self.fused_unpack else [
            ("packed_attention", spa.spa_packed_attention(p[:, :C], p[:, C:2 * C], p[:, 2 * C:], self.seg_cu_seqlens,
                                                          self.seg_cap, self.max_seqlen, self.H, self.Dh, self.out,
                                                          None, prepare=True)),
            ("unpack", spa.spa_unpack(self.out, self.inv_pos, base, self.y, prepare=True)),
        ])

    def run(self, x, w, qkv, base=None):
        for _, fn in self.stages(x, w, qkv, base):
            fn()
        return self.y


def _on_streams(per_stage, streams, stream_of):
    """Chains of prepared launches, one chain per stage, stage i prepared on streams[stream_of[i]],
    as one list for a host thread to issue in order.  per_stage[i] = list of (name, call); the
    FIRST call of stage i reads what the first call of stage i - 1 wrote (the score map handed
    down): stages that share a stream are ordered by the stream, across streams by one event.
    The host issues stage after stage, finest (largest) first: its long kernels start at once and
    the small coarser stages fill in beside them (alternating between the streams measured no
    gain over one stream).  The first entry forks the streams off the stream that is current when
    the list is built, the last one joins them back."""
    main = torch.cuda.current_stream()
    start = torch.cuda.Event()
    done = [torch.cuda.Event() for _ in streams]
    n = len(per_stage)
    crossing = [i + 1 < n and stream_of[i + 1] != stream_of[i] for i in range(n)]
    handed = [torch.cuda.Event() if c else None for c in crossing]

    def fork():
        start.record(main)
        for st in streams:
            st.wait_event(start)

    def join():
        for ev, st in zip(done, streams):
            ev.record(st)
            main.wait_event(ev)

    queues = [[] for _ in streams]
    for i, chain in enumerate(per_stage):
        for j, (name, call) in enumerate(chain):
            st = streams[stream_of[i]]
            if j == 0 and (crossing[i] or (i > 0 and crossing[i - 1])):
                def go(call=call, st=st, wait=handed[i - 1] if i > 0 and crossing[i - 1] else None,
                       signal=handed[i] if crossing[i] else None):
                    if wait is not None:
                        st.wait_event(wait)
                    call()
                    if signal is not None:
                        signal.record(st)
                queues[stream_of[i]].append((name, go))
            else:
                queues[stream_of[i]].append((name, call))
    out = [("fork_streams", fork)]
    for q in queues:
        out += q
    return out + [("join_streams", join)]


class HierarchyPass:
    """A multi-stage hierarchy (Section 3.1, Section 3.2 on multi-scale scores): every stage
    runs gate -> pack -> attention + scatter, and from the second stage on the gate takes the
    previous (2x finer) stage's score map, max-pooled inside the gate kernel, as s_up.
    Three launches per stage (lean form: two for the coarse stages), no host sync anywhere in the chain.  (Everything on one stream:
    spreading the stages over two or four streams was measured and is slower for the forward
    chain, 129 and 166 us against 102 us; the events and the fork / join per chain cost more
    than the overlap of the small coarse stages brings.)"""

    def __init__(self, stages, lean: bool = False):
        """stages: one (B, grid_h, grid_w, C, H, dtype, tau, bias) tuple per stage, finest
        first; consecutive grids halve.
        lean=True (forward only; y is the same bit for bit): no stage copies rows or keeps the packed
        output and lse; stages of at most 256 tokens per image take their packing order from the mask
        (two launches, no index arrays), the others fetch gathered rows through the index."""
        self.cfg = list(stages)
        for (a, b) in zip(self.cfg[:-1], self.cfg[1:]):
            if a[1] != 2 * b[1] or a[2] != 2 * b[2] or a[0] != b[0]:
                raise ValueError("consecutive stages must share B and halve the grid")
        if lean:
            self.passes = [ForwardPass(B, gh * gw, C, H, dtype, tau, bias, keep_packed_out=False, gathered=True,
                                       from_mask=gh * gw <= 256)
                           for (B, gh, gw, C, H, dtype, tau, bias) in self.cfg]
        else:
            self.passes = [ForwardPass(B, gh * gw, C, H, dtype, tau, bias)
                           for (B, gh, gw, C, H, dtype, tau, bias) in self.cfg]
        self.s_up = [None] + [torch.empty(c[0], c[1] * c[2], dtype=torch.float32, device="cuda") for c in self.cfg[1:]]

    def stages(self, xs, ws, qkvs, bases=None) -> List[Tuple[str, Callable[[], None]]]:
        """xs, ws, qkvs: one tensor per stage.  Returns the chain as named prepared launches."""
        out = []
        for i, (fp, cfg) in enumerate(zip(self.passes, self.cfg)):
            st = fp.stages(xs[i], ws[i], qkvs[i], None, None if bases is None else bases[i])
            if i > 0:
                st[0] = ("gate_select_pooled", spa.spa_gate_select_pooled(
                    xs[i], ws[i], fp.bias, self.passes[i - 1].scores, cfg[1], cfg[2], fp.tau, fp.scores, fp.mask,
                    None, self.s_up[i], prepare=True))
            out += [(f"s{i + 1}.{name}", fn) for name, fn in st]
        return out

    def run(self, xs, ws, qkvs, bases=None):
        for _, fn in self.stages(xs, ws, qkvs, bases):
            fn()
        return [fp.y for fp in self.passes]


class HierarchyTrainPass:
    """Forward + backward of every stage of a hierarchy (TrainPass per stage); from the second
    stage on the gate takes the finer stage's score map (pooled in the gate kernel).  All
    forwards run first (a stage's gate needs the finer stage's scores), then all backwards.
    The score map handed down is treated as a constant by the coarser stage's backward.

    concurrent=True: every stage runs forward and backward on a HIP stream of its own (default
    priority); the only coupling is the score map a gate reads from the finer stage (one event).
    Measured on the four-stage workload: 228 us per chain against 293 us on one stream (263 us
    with the finest stage on one stream and the three coarser ones on a second)."""

    def __init__(self, stages, concurrent: bool = False):
        self.concurrent = concurrent
        self.streams = [torch.cuda.Stream() for _ in stages] if concurrent else None
        self.stream_of = list(range(len(stages)))
        self.cfg = list(stages)
        self.passes = [TrainPass(B, gh * gw, C, H, dtype, tau, bias) for (B, gh, gw, C, H, dtype, tau, bias) in self.cfg]

    def stages(self, xs, ws, qks, labels, dys) -> List[Tuple[str, Callable[[], None]]]:
        fwd, bwd, chains = [], [], []
        for i, (tp, cfg) in enumerate(zip(self.passes, self.cfg)):
            with torch.cuda.stream(self.streams[self.stream_of[i]] if self.concurrent else torch.cuda.current_stream()):
                st = tp.stages(xs[i], ws[i], qks[i], labels[i], dys[i],
                               s_fine=self.passes[i - 1].scores if i > 0 else None, grid=(cfg[1], cfg[2]))
            n_fwd = 3 if tp.pack_pair else 4      # gate, pack (one or two launches), attention + scatter
            fwd += [(f"s{i + 1}.{n}", f) for n, f in st[:n_fwd]]
            bwd += [(f"s{i + 1}.{n}", f) for n, f in st[n_fwd:]]
            chains.append([(f"s{i + 1}.{n}", f) for n, f in st])
        return _on_streams(chains, self.streams, self.stream_of) if self.concurrent else fwd + bwd

    def run(self, xs, ws, qks, labels, dys):
        for _, fn in self.stages(xs, ws, qks, labels, dys):
            fn()
        return [tp.loss for tp in self.passes]
