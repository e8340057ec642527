"""CPU oracle for the Select-and-Pack Attention (SPA) hot path.  TEST INFRASTRUCTURE.

This file is a plain, slow, fp64 NumPy statement of what the path computes, written
from the paper (Section 3.2 "Select and Pack Attention", Eqs. for s / r_g / r_p,
"Token Packing", and the selection loss of Section 3.3).  It exists only so that
tests, the smoke check and the benchmark's cpu_baseline leg can compare the HIP
kernels against it.  It shares no code with the HIP path, is never imported by the
product package, and is not tuned for speed.

Given the selection mask, SPA reaches exactly the plain result "softmax self-attention
of each image restricted to that image's selected tokens" (packing is a re-arrangement,
the attention mask keeps images apart).  So the attention oracle is that definition,
evaluated per image directly on the un-packed [B, N, .] tensors: it never looks at the
packed layout.

Readings taken where the paper is silent (each listed in the design notes):
  * gate = one linear map w in R^C plus a scalar bias (Section 3.2: "linear gating layer",
    scores of shape B x N x 1);
  * selection = noise-free hard decision of the two-class Gumbel-Softmax on [s, 0]:
    sigmoid(s) > tau, i.e. s > ln(tau / (1 - tau)), strict, ties not selected;
  * packed order = images in batch order, tokens in ascending position (stable);
  * attention scale 1/sqrt(Dh), no bias, no dropout;
  * the post-max score s feeds the sigmoid scale and the loss; where s_up wins the max,
    no gradient reaches (w, b); a tie goes to the gate;
  * the hard mask is a constant in the backward pass.

Pins: every function below is checked in tests/test_oracle_*.py against closed forms,
library routines on special cases, brute force and finite differences.
"""
from __future__ import annotations

import math
from typing import Optional, Tuple

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------- dtype
def round_to_dtype(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp64 values to the storage type of the workload ("f32" or "bf16"),
    returned as fp64.  bf16 = keep the top 16 bits of the fp32 pattern, nearest-even."""
    f = np.asarray(a, dtype=np.float32)
    if dtype == "f32":
        return f.astype(F64)
    if dtype != "bf16":
        raise ValueError(dtype)
    bits = np.ascontiguousarray(f).view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    bits = (bits + 0x7FFF + lsb) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32).reshape(f.shape).astype(F64)


# ---------------------------------------------------------------------------- gate
def gate_scores(x: np.ndarray, w: np.ndarray, bias: float,
                s_up: Optional[np.ndarray] = None) -> np.ndarray:
    """Eq. s = Max(f_g(r), s_up) (Section 3.2).  f_g(r)_i = bias + sum_c w_c x_ic, summed
    left to right in fp64.  x [B,N,C], w [C], s_up [B,N] or None.  Returns logits [B,N]."""
    x = np.asarray(x, dtype=F64)
    w = np.asarray(w, dtype=F64)
    B, N, C = x.shape
    g = np.full((B, N), float(bias), dtype=F64)
    for c in range(C):
        g = g + w[c] * x[:, :, c]
    if s_up is not None:
        g = np.maximum(g, np.asarray(s_up, dtype=F64))
    return g


def gate_only(x, w, bias) -> np.ndarray:
    """The linear gate alone, f_g(r), before the max with the up-scale scores."""
    return gate_scores(x, w, bias, None)


def threshold_logit(tau: float) -> float:
    """sigmoid(s) > tau  <=>  s > ln(tau / (1 - tau))."""
    if not (0.0 < tau < 1.0):
        raise ValueError("tau must lie in (0, 1)")
    return math.log(tau / (1.0 - tau))


def select(s: np.ndarray, tau: float) -> Tuple[np.ndarray, float]:
    """Hard selection (Eq. r_p = Gumbel-Softmax(s) . r_g, noise-free): mask_i = [s_i > theta].
    Returns (mask [B,N] uint8, margin = min_i |s_i - theta|)."""
    theta = threshold_logit(tau)
    s = np.asarray(s, dtype=F64)
    mask = (s > theta).astype(np.uint8)
    margin = float(np.min(np.abs(s - theta))) if s.size else float("inf")
    return mask, margin


def select_gumbel(s: np.ndarray, noise: np.ndarray, temperature: float, tau: float):
    """Stochastic hard selection (Eq. r_p = Gumbel-Softmax(s) . r_g, Gumbel-Softmax of the
    two-class logits [s, 0]): with g1, g2 independent Gumbel(0,1) draws the relaxed weight
    of the 'select' class is
        p~_i = exp((s_i + g1)/T) / (exp((s_i + g1)/T) + exp(g2/T)) = sigmoid((s_i + e_i) / T),
    e_i = g1 - g2 (a Logistic(0,1) variate, passed in as `noise`), and the token is selected
    when p~_i exceeds the threshold tau, i.e. when s_i + e_i > T * logit(tau) (strict).
    Returns (mask [B,N] uint8, p~ [B,N], margin = min_i |s_i + e_i - T logit(tau)|)."""
    s = np.asarray(s, dtype=F64)
    e = np.asarray(noise, dtype=F64)
    z = s + e
    bound = temperature * threshold_logit(tau)
    mask = (z > bound).astype(np.uint8)
    margin = float(np.min(np.abs(z - bound))) if s.size else float("inf")
    return mask, sigmoid(z / temperature), margin


def maxpool2x2(s: np.ndarray, h: int, w: int) -> np.ndarray:
    """Up-scale scores resized to the next (2x coarser) stage by 2x2 stride-2 max-pooling
    (Section 3.2: scores from up-scaled features are "adjusted via max-pooling").
    s [B, h*w] -> [B, (h/2)*(w/2)]."""
    s = np.asarray(s, dtype=F64)
    B = s.shape[0]
    out = np.empty((B, (h // 2) * (w // 2)), dtype=F64)
    for b in range(B):
        g = s[b].reshape(h, w)
        for i in range(h // 2):
            for j in range(w // 2):
                out[b, i * (w // 2) + j] = max(g[2 * i, 2 * j], g[2 * i, 2 * j + 1],
                                               g[2 * i + 1, 2 * j], g[2 * i + 1, 2 * j + 1])
    return out


def sigmoid(s: np.ndarray) -> np.ndarray:
    s = np.asarray(s, dtype=F64)
    e = np.exp(-np.abs(s))
    return np.where(s >= 0, 1.0 / (1.0 + e), e / (1.0 + e))


# ---------------------------------------------------------------------------- pack
def shift_order(grid_h: int, grid_w: int, shift_h: int, shift_w: int) -> np.ndarray:
    """Cyclic shift of the feature map (Section 1, the paragraph on shifting the feature maps
    every two blocks; the amount and direction follow the window shift of the Swin design the
    paper builds on): the shifted map holds at (r', c') the token that sits at
    ((r' + shift_h) mod grid_h, (c' + shift_w) mod grid_w) in the original map.
    Returns order [N] i32: order[p'] = original position of the p'-th token of the shifted map
    in raster order."""
    order = np.zeros(grid_h * grid_w, dtype=np.int32)
    for r in range(grid_h):
        for c in range(grid_w):
            order[r * grid_w + c] = ((r + shift_h) % grid_h) * grid_w + (c + shift_w) % grid_w
    return order


def pack_indices(mask: np.ndarray, order: Optional[np.ndarray] = None):
    """Token Packing (Section 3.2): walk images in batch order and tokens in ascending
    position (of the shifted map when `order` is given, see shift_order), appending
    survivors.  Returns
      cu_seqlens [B+1] i32 (segment of image b is [cu[b], cu[b+1])),
      gather_idx [T] i32  (flat token id b*N+n, in the ORIGINAL layout, of the j-th packed row),
      inv_pos [B*N] i32   (packed row of a token, -1 if not selected),
      total T."""
    mask = np.asarray(mask)
    B, N = mask.shape
    cu = np.zeros(B + 1, dtype=np.int32)
    gather = []
    inv = np.full(B * N, -1, dtype=np.int32)
    for b in range(B):
        for p in range(N):
            n = p if order is None else int(order[p])
            if mask[b, n]:
                inv[b * N + n] = len(gather)
                gather.append(b * N + n)
        cu[b + 1] = len(gather)
    return cu, np.asarray(gather, dtype=np.int32), inv, len(gather)


def container_segments(cu_seqlens: np.ndarray, container_len: int) -> np.ndarray:
    """Boundaries of the attention segments when the packed stream is cut into containers of
    length L (Section 3.2 "Token Packing" and the 2 L^2 C term of the complexity formula): a
    token attends to the tokens of its own image inside its own container, so a segment ends
    wherever an image ends or a container ends.  Returns the sorted distinct boundaries
    [S+1] i32, from 0 to T."""
    cu = np.asarray(cu_seqlens).astype(np.int64)
    T = int(cu[-1])
    cuts = set(int(c) for c in cu)
    cuts.update(range(0, T, container_len))
    cuts.add(T)
    cuts.add(0)
    return np.asarray(sorted(cuts), dtype=np.int32)


def packed_rows(total: int, container_len: int) -> int:
    """Rows of the packed buffer: T rounded up to whole containers of length L; only
    the last container is padded (Section 3.2 "Token Packing").  L = 0: no padding."""
    if container_len <= 0:
        return total
    return -(-total // container_len) * container_len


def pack_rows(x: np.ndarray, gather_idx: np.ndarray, scores: Optional[np.ndarray] = None,
              container_len: int = 0, dtype: Optional[str] = None) -> np.ndarray:
    """packed[j] = x[gather_idx[j]], times sigmoid(s) of that token when scores are given
    (Eq. r_g = Sigmoid(s) . r); pad rows up to whole containers are zero.  If dtype is
    given the scaled rows are rounded to it (what a kernel storing that type can hold)."""
    x = np.asarray(x, dtype=F64)
    C = x.shape[-1]
    flat = x.reshape(-1, C)
    T = len(gather_idx)
    out = np.zeros((packed_rows(T, container_len), C), dtype=F64)
    for j in range(T):
        row = flat[gather_idx[j]]
        if scores is not None:
            row = row * sigmoid(np.asarray(scores, dtype=F64).reshape(-1)[gather_idx[j]])
        out[j] = row
    if dtype is not None:
        out = round_to_dtype(out, dtype)
    return out


def unpack(o: np.ndarray, inv_pos: np.ndarray, B: int, N: int,
           base: Optional[np.ndarray] = None) -> np.ndarray:
    """Scatter back (Section 3.2 / SPA-block figure): selected tokens receive their
    attention output at their original position; the others keep `base` (the tokens that
    bypass attention) or zero.  With base given, selected rows get base + o."""
    o = np.asarray(o, dtype=F64)
    C = o.shape[-1]
    y = np.zeros((B * N, C), dtype=F64) if base is None else np.array(base, dtype=F64).reshape(B * N, C)
    for i in range(B * N):
        j = inv_pos[i]
        if j >= 0:
            y[i] = y[i] + o[j]
    return y.reshape(B, N, C)


# ----------------------------------------------------------------------- attention
def _split_heads(t: np.ndarray, H: int) -> np.ndarray:
    B, N, C = t.shape
    return np.asarray(t, dtype=F64).reshape(B, N, H, C // H)


def attention_per_image(q: np.ndarray, k: np.ndarray, v: np.ndarray, mask: np.ndarray,
                        H: int, scale: Optional[float] = None):
    """Multi-head self-attention in which a token attends only to the selected tokens of
    its own image (Section 3.2, last paragraph).  q, k, v are the UN-packed [B,N,C]
    tensors; for each image the selected rows are taken with the mask, the full n_b x n_b
    score matrix is formed, and softmax(QK^T * scale) V is evaluated row by row.
    Returns out [T, C] in packed order and lse [H, T] (log-sum-exp of the scaled scores)."""
    qh, kh, vh = _split_heads(q, H), _split_heads(k, H), _split_heads(v, H)
    B, N, _, Dh = qh.shape
    if scale is None:
        scale = 1.0 / math.sqrt(Dh)
    mask = np.asarray(mask).astype(bool)
    T = int(mask.sum())
    out = np.zeros((T, H * Dh), dtype=F64)
    lse = np.zeros((H, T), dtype=F64)
    row0 = 0
    for b in range(B):
        sel = np.flatnonzero(mask[b])
        n = len(sel)
        if n == 0:
            continue
        for h in range(H):
            Q, K, V = qh[b, sel, h], kh[b, sel, h], vh[b, sel, h]
            S = (Q @ K.T) * scale
            m = S.max(axis=1, keepdims=True)
            E = np.exp(S - m)
            Z = E.sum(axis=1, keepdims=True)
            P = E / Z
            out[row0:row0 + n, h * Dh:(h + 1) * Dh] = P @ V
            lse[h, row0:row0 + n] = (m + np.log(Z))[:, 0]
        row0 += n
    return out, lse


def attention_container_local(qp: np.ndarray, kp: np.ndarray, vp: np.ndarray, cu_seqlens: np.ndarray,
                              container_len: int, H: int, scale: Optional[float] = None):
    """Attention over the packed stream [T, C] with the paper's full mask written out
    (Section 3.2: containers of length L, tokens attend only to tokens of the same image
    inside their container): row i may attend to row j iff both lie in the same image
    segment of cu_seqlens and floor(i / L) == floor(j / L).  The T x T score matrix is
    formed whole, disallowed entries are set to -inf, and softmax(S) V is evaluated.
    Returns out [T, C] and lse [H, T]."""
    qp, kp, vp = (np.asarray(a, dtype=F64) for a in (qp, kp, vp))
    T, C = qp.shape
    Dh = C // H
    if scale is None:
        scale = 1.0 / math.sqrt(Dh)
    cu = np.asarray(cu_seqlens)
    image = np.zeros(T, dtype=np.int64)
    for b in range(len(cu) - 1):
        image[cu[b]:cu[b + 1]] = b
    container = np.arange(T) // container_len
    allowed = (image[:, None] == image[None, :]) & (container[:, None] == container[None, :])
    out = np.zeros((T, C), dtype=F64)
    lse = np.zeros((H, T), dtype=F64)
    for h in range(H):
        Q, K, V = (a[:, h * Dh:(h + 1) * Dh] for a in (qp, kp, vp))
        S = np.where(allowed, (Q @ K.T) * scale, -np.inf)
        m = S.max(axis=1, keepdims=True)
        E = np.exp(S - m)
        Z = E.sum(axis=1, keepdims=True)
        out[:, h * Dh:(h + 1) * Dh] = (E / Z) @ V
        lse[h] = (m + np.log(Z))[:, 0]
    return out, lse


def attention_container_local_backward(qp, kp, vp, cu_seqlens, container_len: int, dout: np.ndarray, H: int,
                                       scale: Optional[float] = None):
    """Gradient of attention_container_local with respect to qp, kp, vp: the textbook
    softmax-attention calculus on the whole T x T matrices with the same mask
    (P = 0 where disallowed): dV = P^T dO, dP = dO V^T, dS = P * (dP - rowsum(P * dP)),
    dQ = dS K * scale, dK = dS^T Q * scale."""
    qp, kp, vp, dout = (np.asarray(a, dtype=F64) for a in (qp, kp, vp, dout))
    T, C = qp.shape
    Dh = C // H
    if scale is None:
        scale = 1.0 / math.sqrt(Dh)
    cu = np.asarray(cu_seqlens)
    image = np.zeros(T, dtype=np.int64)
    for b in range(len(cu) - 1):
        image[cu[b]:cu[b + 1]] = b
    container = np.arange(T) // container_len
    allowed = (image[:, None] == image[None, :]) & (container[:, None] == container[None, :])
    dq, dk, dv = np.zeros_like(qp), np.zeros_like(kp), np.zeros_like(vp)
    for h in range(H):
        sl = slice(h * Dh, (h + 1) * Dh)
        Q, K, V, dO = qp[:, sl], kp[:, sl], vp[:, sl], dout[:, sl]
        S = np.where(allowed, (Q @ K.T) * scale, -np.inf)
        E = np.exp(S - S.max(axis=1, keepdims=True))
        P = E / E.sum(axis=1, keepdims=True)
        dv[:, sl] = P.T @ dO
        dP = dO @ V.T
        dS = P * (dP - (P * dP).sum(axis=1, keepdims=True))
        dq[:, sl] = dS @ K * scale
        dk[:, sl] = dS.T @ Q * scale
    return dq, dk, dv


def attention_backward_per_image(q, k, v, mask, dout_packed, H: int,
                                 scale: Optional[float] = None):
    """Gradient of attention_per_image with respect to the selected rows of q, k, v.
    dout_packed [T, C] is the gradient of the packed output.  Textbook softmax-attention
    calculus with explicit n_b x n_b matrices:
      P = softmax(S), dV = P^T dO, dP = dO V^T, dS = P * (dP - rowsum(P * dP)),
      dQ = dS K * scale, dK = dS^T Q * scale.
    Returns dq, dk, dv, each [T, C] in packed order."""
    qh, kh, vh = _split_heads(q, H), _split_heads(k, H), _split_heads(v, H)
    B, N, _, Dh = qh.shape
    if scale is None:
        scale = 1.0 / math.sqrt(Dh)
    mask = np.asarray(mask).astype(bool)
    T = int(mask.sum())
    dO = np.asarray(dout_packed, dtype=F64).reshape(T, H, Dh)
    dq = np.zeros((T, H * Dh), dtype=F64)
    dk = np.zeros_like(dq)
    dv = np.zeros_like(dq)
    row0 = 0
    for b in range(B):
        sel = np.flatnonzero(mask[b])
        n = len(sel)
        if n == 0:
            continue
        for h in range(H):
            Q, K, V = qh[b, sel, h], kh[b, sel, h], vh[b, sel, h]
            G = dO[row0:row0 + n, h]
            S = (Q @ K.T) * scale
            E = np.exp(S - S.max(axis=1, keepdims=True))
            P = E / E.sum(axis=1, keepdims=True)
            dP = G @ V.T
            dS = P * (dP - (P * dP).sum(axis=1, keepdims=True))
            sl = slice(h * Dh, (h + 1) * Dh)
            dv[row0:row0 + n, sl] = P.T @ G
            dq[row0:row0 + n, sl] = (dS @ K) * scale
            dk[row0:row0 + n, sl] = (dS.T @ Q) * scale
        row0 += n
    return dq, dk, dv


# ------------------------------------------------------------------ loss / gate bwd
def selection_loss(s: np.ndarray, labels: np.ndarray, loss_scale: float) -> float:
    """Selection loss (Section 3.3): binary cross-entropy between sigmoid(s) and the
    label, summed over tokens and multiplied by loss_scale.  Evaluated in the stable
    form  max(s,0) - y s + log(1 + exp(-|s|))  which equals
    -(y log sigma(s) + (1-y) log(1 - sigma(s)))."""
    s = np.asarray(s, dtype=F64)
    y = np.asarray(labels, dtype=F64)
    per = np.maximum(s, 0.0) - y * s + np.log1p(np.exp(-np.abs(s)))
    return float(loss_scale * per.sum())


def gate_backward(x, w, bias, s_up, labels, d_rg, gate_scaled: bool, loss_scale: float,
                  st_mask: Optional[np.ndarray] = None, st_noise: Optional[np.ndarray] = None,
                  st_temperature: float = 1.0):
    """Backward of the gate: scores s = Max(x.w + b, s_up); optional gated representation
    r_g = sigmoid(s) . x whose gradient d_rg [B,N,C] arrives from the packed path (zero
    rows for unselected tokens); selection loss = loss_scale * BCE(sigmoid(s), labels).

      ds_i = loss_scale * (sigmoid(s_i) - y_i) + [gate_scaled] p_i (1 - p_i) <d_rg_i, x_i>
      dx_i = [gate_scaled] p_i * d_rg_i + own_i * ds_i * w
      dw   = sum_i own_i * ds_i * x_i,   db = sum_i own_i * ds_i
    where own_i = 1 when the gate's own logit produced s_i (g_i >= s_up_i) and 0 where the
    up-scale score won the max.  Returns dict(loss, ds, dx, dw, db).

    Straight-through estimator of the hard selection (Gumbel-Softmax with hard samples: the
    forward pass multiplies r_g by the 0/1 mask m_i, the backward pass differentiates the
    relaxed weight p~_i = sigmoid((s_i + e_i)/T) in its place).  With st_mask given, selected
    tokens add   ds_i += <d_rg_i, r_g_i> * p~_i (1 - p~_i) / T,   r_g_i = p_i x_i,
    where d_rg_i (the gradient that reached r_g through the packed row) equals d r_p_i there."""
    x = np.asarray(x, dtype=F64)
    w = np.asarray(w, dtype=F64)
    B, N, C = x.shape
    g = gate_only(x, w, bias)
    if s_up is None:
        s = g
        own = np.ones((B, N), dtype=F64)
    else:
        su = np.asarray(s_up, dtype=F64)
        s = np.maximum(g, su)
        own = (g >= su).astype(F64)
    p = sigmoid(s)
    y = np.asarray(labels, dtype=F64)
    ds = loss_scale * (p - y)
    dx = np.zeros_like(x)
    if gate_scaled and d_rg is not None:
        d_rg = np.asarray(d_rg, dtype=F64)
        ds = ds + p * (1.0 - p) * (d_rg * x).sum(axis=2)
        dx = dx + p[:, :, None] * d_rg
        if st_mask is not None:
            e = np.zeros_like(s) if st_noise is None else np.asarray(st_noise, dtype=F64)
            pt = sigmoid((s + e) / st_temperature)
            r_g = p[:, :, None] * x
            ds = ds + np.asarray(st_mask, dtype=F64) * (d_rg * r_g).sum(axis=2) * pt * (1.0 - pt) / st_temperature
    dsg = ds * own
    dx = dx + dsg[:, :, None] * w[None, None, :]
    dw = (dsg[:, :, None] * x).sum(axis=(0, 1))
    db = float(dsg.sum())
    return {"loss": selection_loss(s, labels, loss_scale), "ds": ds, "dx": dx, "dw": dw, "db": db,
            "scores": s}


# ------------------------------------------------------------------------ projections
def linear_packed(x, gather_idx, W, bias=None, scores=None, dtype: Optional[str] = None) -> np.ndarray:
    """Projection of the packed tokens (the 3LC^2 / NC^2 terms of the complexity formula of
    Section 3.2): row j of the result is a_j W^T + bias with a_j = x[gather_idx[j]], first
    multiplied by sigmoid(score) of that token (r_g = Sigmoid(s) . r) and rounded to the
    storage type when scores are given.  x [..., K], W [N_out, K].  Plain fp64 matmul."""
    rows = pack_rows(np.asarray(x, dtype=F64).reshape(-1, np.shape(x)[-1])[None], np.asarray(gather_idx),
                     None if scores is None else np.asarray(scores, dtype=F64).reshape(1, -1), 0,
                     dtype if scores is not None else None)
    y = rows @ np.asarray(W, dtype=F64).T
    if bias is not None:
        y = y + np.asarray(bias, dtype=F64)[None, :]
    return y


def linear_packed_backward(dout, x, gather_idx, W, scores=None, dout_idx=None, dtype: Optional[str] = None):
    """Gradients of the projection out_j = r_j W^T + bias, with r_j = x[gather_idx[j]]
    (times sigmoid(score) of that token when scores are given: the gated row of Eq.
    r_g = Sigmoid(s) . r), for an upstream gradient whose row j is dout[dout_idx[j]]
    (dout[j] without dout_idx).  The chain rule of a linear map, written out:
      d_rows[j,:] = dout_j W           gradient with respect to the row r_j that was multiplied
      dW          = sum_j dout_j^T r_j
      dbias       = sum_j dout_j
    When scores are given r_j is the gated row, so d_rows is the gradient of r_g (what the
    gate backward takes), not of x.  dtype: the gated rows are rounded to it first, as in
    linear_packed.  x [..., K], W [N_out, K], dout [*, N_out]."""
    gather_idx = np.asarray(gather_idx)
    rows = pack_rows(np.asarray(x, dtype=F64).reshape(-1, np.shape(x)[-1])[None], gather_idx,
                     None if scores is None else np.asarray(scores, dtype=F64).reshape(1, -1), 0,
                     dtype if scores is not None else None)
    g = np.asarray(dout, dtype=F64).reshape(-1, np.shape(dout)[-1])
    g = g[np.asarray(dout_idx)] if dout_idx is not None else g[:len(gather_idx)]
    return {"d_rows": g @ np.asarray(W, dtype=F64), "dW": g.T @ rows, "dbias": g.sum(axis=0)}


# ------------------------------------------------------------------------ whole path
def spa_forward(x, w, bias, qkv, H: int, tau: float, dtype: str,
                s_up: Optional[np.ndarray] = None, container_len: int = 0,
                base: Optional[np.ndarray] = None):
    """The forward hot path in the paper's order: score (Eq. s) -> select (Eq. r_p) ->
    pack -> per-image attention on the selected tokens -> scatter back.
    qkv [B,N,3C] holds the (already projected) q | k | v of every token.
    Returns a dict of every intermediate the HIP path exposes."""
    x = np.asarray(x, dtype=F64)
    B, N, C = x.shape
    s = gate_scores(x, w, bias, s_up)
    mask, margin = select(s, tau)
    cu, gidx, inv, T = pack_indices(mask)
    qkv = np.asarray(qkv, dtype=F64)
    q, k, v = qkv[:, :, :C], qkv[:, :, C:2 * C], qkv[:, :, 2 * C:]
    packed_qkv = pack_rows(qkv, gidx, None, container_len)
    packed_rg = pack_rows(x, gidx, s, container_len, dtype)
    out, lse = attention_per_image(q, k, v, mask, H)
    y = unpack(out, inv, B, N, base)
    return {"scores": s, "mask": mask, "margin": margin, "counts": mask.sum(axis=1).astype(np.int32),
            "cu_seqlens": cu, "gather_idx": gidx, "inv_pos": inv, "total": T,
            "packed_qkv": packed_qkv, "packed_rg": packed_rg, "out": out, "lse": lse, "y": y}
