"""Unsliced reference forward of a video-UNet transformer block (float64 NumPy).

TEST INFRASTRUCTURE ONLY -- see the package docstring.

The paper (Sec. 4.1, 4.2.1, Eq. 1) states that slicing plus operator grouping
reproduces the unsliced result exactly, so the oracle is the plain definition
of the unsliced block, applied operator by operator to the whole tensor.  The
paper names the operator types only (GroupNorm, LayerNorm, Attention, Linear;
Sec. 4.1); the block wiring below is the reading fixed for this build:

  1. GroupNorm per (batch, frame, group) over (C/G) x H x W, biased variance.
  2. tokens = channel vectors; h = tokens W_in + b_in.
  3. sequences: temporal block = one per (batch, position) over F frames;
     spatial block = one per (batch, frame) over H*W positions.
  4. h += Attn(LN1(h) [+ sinusoidal frame embedding]) W_o + b_o.
  5. spatial only: h += CrossAttn(LN2(h), context) W_o2 + b_o2.
  6. h += GEGLU-FFN(LN3(h)).
  7. out = x + (h W_out + b_out) scattered back to [B,C,F,H,W].

Parameters are a dict of arrays (row-major [in, out] matrices) named like the
fields of the C-ABI weight struct, plus a hyper-parameter object with
attributes kind, heads, dim_head, gn_groups, gn_eps, ln_eps, add_sin_pe.
"""
from __future__ import annotations

import math
from typing import Iterator, Optional, Tuple

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64


def group_norm_ref(x, groups: int, eps: float, gamma, beta):
    """GroupNorm with statistics per (b, f, group) over (C/G)*H*W values.

    x: [B,C,F,H,W].  mean and *biased* variance of x[b, g*n:(g+1)*n, f, :, :];
    result (x-mean)/sqrt(var+eps)*gamma[c]+beta[c]."""
    x = np.asarray(x, F64)
    B, C, Fr, H, W = x.shape
    n = C // groups
    assert n * groups == C
    xg = x.reshape(B, groups, n, Fr, H, W)
    mean = xg.mean(axis=(2, 4, 5), keepdims=True)
    var = ((xg - mean) ** 2).mean(axis=(2, 4, 5), keepdims=True)
    xh = ((xg - mean) / np.sqrt(var + eps)).reshape(B, C, Fr, H, W)
    g = np.asarray(gamma, F64).reshape(1, C, 1, 1, 1)
    b = np.asarray(beta, F64).reshape(1, C, 1, 1, 1)
    return xh * g + b


def layer_norm_ref(h, gamma, beta, eps: float):
    """LayerNorm over the last axis, biased variance, affine."""
    h = np.asarray(h, F64)
    mean = h.mean(axis=-1, keepdims=True)
    var = ((h - mean) ** 2).mean(axis=-1, keepdims=True)
    return (h - mean) / np.sqrt(var + eps) * np.asarray(gamma, F64) + np.asarray(beta, F64)


def sinusoidal_pe_ref(frames: int, width: int):
    """PE[f, 2i] = sin(f / 10000^(2i/width)), PE[f, 2i+1] = cos(same angle)."""
    pe = np.zeros((frames, width), F64)
    for f in range(frames):
        for i in range(0, width, 2):
            angle = f / (10000.0 ** (i / width))
            pe[f, i] = math.sin(angle)
            if i + 1 < width:
                pe[f, i + 1] = math.cos(angle)
    return pe


def gelu_erf_ref(u):
    """Exact GELU: 0.5 u (1 + erf(u / sqrt 2))."""
    u = np.asarray(u, F64)
    return 0.5 * u * (1.0 + _erf(u / math.sqrt(2.0)))


def softmax_rows_ref(s):
    s = np.asarray(s, F64)
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def attention_ref(q, k, v, heads: int):
    """Multi-head scaled dot-product attention, no mask.

    q: [S, Nq, D]; k, v: [S, Nk, D]; D split into `heads` contiguous chunks of
    d; per head softmax_rows(q k^T / sqrt d) v; heads concatenated."""
    q, k, v = (np.asarray(t, F64) for t in (q, k, v))
    S, Nq, D = q.shape
    d = D // heads
    out = np.empty((S, Nq, D), F64)
    for s in range(S):
        for hd in range(heads):
            cs = slice(hd * d, (hd + 1) * d)
            scores = q[s, :, cs] @ k[s, :, cs].T / math.sqrt(d)
            out[s, :, cs] = softmax_rows_ref(scores) @ v[s, :, cs]
    return out


def tokens_from_feature_ref(xh, kind: str):
    """[B,C,F,H,W] -> sequences [S, N, C]: temporal S=B*P, N=F; spatial S=B*F, N=P."""
    B, C, Fr, H, W = xh.shape
    P = H * W
    t = xh.reshape(B, C, Fr, P)
    if kind == "temporal":
        return t.transpose(0, 3, 2, 1).reshape(B * P, Fr, C)
    return t.transpose(0, 2, 3, 1).reshape(B * Fr, P, C)


def feature_from_tokens_ref(y, kind: str, shape):
    """Inverse of tokens_from_feature_ref."""
    B, C, Fr, H, W = shape
    P = H * W
    if kind == "temporal":
        return y.reshape(B, P, Fr, C).transpose(0, 3, 2, 1).reshape(B, C, Fr, H, W)
    return y.reshape(B, Fr, P, C).transpose(0, 3, 1, 2).reshape(B, C, Fr, H, W)


def transformer_ref(t, w, hp, ctx_per_seq=None):
    """Steps 2-7 (up to y = h W_out + b_out) on sequences t [S, N, C].

    ctx_per_seq: [S, M, Cc] context of each sequence (spatial blocks).  Row n of a temporal
    sequence is frame n (the frame embedding's index)."""
    W = {k: np.asarray(v, F64) for k, v in w.items()}
    t = np.asarray(t, F64)
    h = t @ W["w_in"] + W["b_in"]
    D = h.shape[-1]
    a = layer_norm_ref(h, W["ln1_g"], W["ln1_b"], hp.ln_eps)
    if hp.kind == "temporal" and hp.add_sin_pe:
        a = a + sinusoidal_pe_ref(h.shape[1], D)[None, :, :]
    o = attention_ref(a @ W["wq"], a @ W["wk"], a @ W["wv"], hp.heads)
    h = h + o @ W["wo"] + W["bo"]
    if hp.kind == "spatial":
        a = layer_norm_ref(h, W["ln2_g"], W["ln2_b"], hp.ln_eps)
        c = np.asarray(ctx_per_seq, F64)
        o = attention_ref(a @ W["wq2"], c @ W["wk2"], c @ W["wv2"], hp.heads)
        h = h + o @ W["wo2"] + W["bo2"]
    a = layer_norm_ref(h, W["ln3_g"], W["ln3_b"], hp.ln_eps)
    u = a @ W["w1"] + W["b1"]
    inner = u.shape[-1] // 2
    g = u[..., :inner] * gelu_erf_ref(u[..., inner:])
    h = h + g @ W["w2"] + W["b2"]
    return h @ W["w_out"] + W["b_out"]


def block_forward_ref(x, w, hp, ctx=None, xhat=None):
    """Unsliced block forward.  x: [B,C,F,H,W]; ctx: [B,M,Cc] or None.

    `xhat` optionally supplies the GroupNorm output (used by the sliced wrapper
    and by sampled-position checks, where statistics come from the full tensor
    but only a window of positions is evaluated)."""
    x = np.asarray(x, F64)
    B, C, Fr, H, Wd = x.shape
    if xhat is None:
        xhat = group_norm_ref(x, hp.gn_groups, hp.gn_eps, w["gn_g"], w["gn_b"])
    t = tokens_from_feature_ref(xhat, hp.kind)
    cps = None
    if hp.kind == "spatial":
        cps = np.repeat(np.asarray(ctx, F64), Fr, axis=0)          # sequence index = b*F + f
    y = transformer_ref(t, w, hp, ctx_per_seq=cps)
    return x + feature_from_tokens_ref(y, hp.kind, x.shape)


def slice_windows_ref(extent: int, slice_len: int) -> Iterator[Tuple[int, int]]:
    """Feature Slicer windows (Sec. 4.1): k = ceil(extent/len) windows of `len`,
    the last one ragged."""
    k = -(-extent // slice_len)
    for i in range(k):
        yield i * slice_len, min((i + 1) * slice_len, extent)


def sliced_block_forward_ref(x, w, hp, ctx=None, axis: str = "HW", slice_len: int = 1,
                             local_stats: bool = False):
    """Eq. (1): X^o = Concat(GroupOP(X_1), ..., GroupOP(X_k)).

    axis "F" slices frames, axis "HW" slices flattened positions.  GroupNorm
    statistics come from the whole tensor (they are the one dependency that
    crosses position slices) unless local_stats=True, which recomputes them per
    slice -- exact for frame slices, lossy for position slices."""
    x = np.asarray(x, F64)
    B, C, Fr, H, Wd = x.shape
    P = H * Wd
    out = np.empty_like(x)
    xhat_full = group_norm_ref(x, hp.gn_groups, hp.gn_eps, w["gn_g"], w["gn_b"])
    if axis == "F":
        for f0, f1 in slice_windows_ref(Fr, slice_len):
            xs = x[:, :, f0:f1]
            xh = None if local_stats else xhat_full[:, :, f0:f1]
            if hp.kind == "temporal" and hp.add_sin_pe:
                raise ValueError("frame slices of a temporal block lose the frame index")
            out[:, :, f0:f1] = block_forward_ref(xs, w, hp, ctx, xhat=xh)
    else:
        xf = x.reshape(B, C, Fr, 1, P)
        of = out.reshape(B, C, Fr, 1, P)
        xhf = xhat_full.reshape(B, C, Fr, 1, P)
        for p0, p1 in slice_windows_ref(P, slice_len):
            xh = None if local_stats else xhf[..., p0:p1]
            of[..., p0:p1] = block_forward_ref(xf[..., p0:p1], w, hp, ctx, xhat=xh)
    return out
