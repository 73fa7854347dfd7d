"""Unsliced reference forward of the Spatial ResBlock operator group (float64 NumPy).

TEST INFRASTRUCTURE ONLY -- see the package docstring.

Sec. 4.2.1 gives the Spatial ResBlock's consecutive GroupNorm, Conv2D and SiLU
operators as its example of a spatial operator group, sliced along the merged
batch x frame axis (Sec. 4.1, spatial layers slicer) and concatenated (Eq. 1).
The paper names the operator types only; the wiring fixed for this build is the
pre-activation residual block of the latent-diffusion U-Net family:

  1. a = SiLU(GroupNorm1(x)), statistics per (batch, frame, group) over (C/G) x H x W.
  2. h = Conv3x3(a) + b1, zero padding 1, stride 1 ("convolution" in the
     deep-learning sense: a cross-correlation, no kernel flip).
  3. optional: h[b, :, f] += (SiLU(temb[b]) W_t + b_t) broadcast over frames and positions.
  4. h = Conv3x3(SiLU(GroupNorm2(h))) + b2.
  5. out = skip(x) + h    skip = identity when C_out = C_in, else the 1x1 convolution
     skip(x)[b, o, f, p] = sum_c w_skip[o, c] * x[b, c, f, p] + b_skip[o]  (used whenever the
     parameter dict holds "w_skip").

Every frame is independent, so slicing along frames reproduces the unsliced
result exactly.  Parameters: dict of arrays named like the fields of the C-ABI
weight struct; convolution kernels in [C_out, C_in, 3, 3] order (conv1 maps C_in to C_out,
conv2 C_out to C_out), w_skip [C_out, C_in], W_t row-major [temb_dim, C_out].
"""
from __future__ import annotations

from typing import Optional

import numpy as np

from .block_ref import group_norm_ref, slice_windows_ref

F64 = np.float64


def silu_ref(v):
    """SiLU / swish: v * sigmoid(v) = v / (1 + exp(-v))."""
    v = np.asarray(v, F64)
    return v / (1.0 + np.exp(-v))


def conv3x3_ref(a, weight, bias=None):
    """out[n, o, y, x] = bias[o] + sum_{c, i, j} weight[o, c, i, j] * a[n, c, y + i - 1, x + j - 1]
    with a = 0 outside the image.  a: [N, C, H, W]; weight: [O, C, 3, 3]."""
    a = np.asarray(a, F64)
    weight = np.asarray(weight, F64)
    N, C, H, W = a.shape
    O = weight.shape[0]
    assert weight.shape == (O, C, 3, 3)
    padded = np.zeros((N, C, H + 2, W + 2), F64)
    padded[:, :, 1:H + 1, 1:W + 1] = a
    out = np.zeros((N, O, H, W), F64)
    for i in range(3):
        for j in range(3):
            out += np.einsum("oc,nchw->nohw", weight[:, :, i, j], padded[:, :, i:i + H, j:j + W])
    if bias is not None:
        out += np.asarray(bias, F64).reshape(1, O, 1, 1)
    return out


def _frames_first(x5):
    """[B,C,F,H,W] -> [B*F, C, H, W] (the reshape of the spatial layers slicer)."""
    B, C, Fr, H, W = x5.shape
    return np.transpose(x5, (0, 2, 1, 3, 4)).reshape(B * Fr, C, H, W)


def _frames_back(x4, B, Fr):
    N, C, H, W = x4.shape
    return np.transpose(x4.reshape(B, Fr, C, H, W), (0, 2, 1, 3, 4))


def resblock_forward_ref(x, w: dict, hp, temb: Optional[np.ndarray] = None):
    """Steps 1-5 above on the whole tensor.  x: [B,C,F,H,W]; hp has gn_groups, gn_eps;
    temb: [B, temb_dim] or None (step 3 skipped)."""
    x = np.asarray(x, F64)
    B, C, Fr, H, W = x.shape
    a = silu_ref(group_norm_ref(x, hp.gn_groups, hp.gn_eps, w["gn1_g"], w["gn1_b"]))
    h = _frames_back(conv3x3_ref(_frames_first(a), w["w_conv1"], w["b_conv1"]), B, Fr)
    if temb is not None:
        e = silu_ref(np.asarray(temb, F64)) @ np.asarray(w["w_temb"], F64) + np.asarray(w["b_temb"], F64)
        h = h + e.reshape(B, -1, 1, 1, 1)
    a2 = silu_ref(group_norm_ref(h, hp.gn_groups, hp.gn_eps, w["gn2_g"], w["gn2_b"]))
    h2 = _frames_back(conv3x3_ref(_frames_first(a2), w["w_conv2"], w["b_conv2"]), B, Fr)
    if w.get("w_skip") is not None:
        skip = np.einsum("oc,bcfhw->bofhw", np.asarray(w["w_skip"], F64), x)
        if w.get("b_skip") is not None:
            skip = skip + np.asarray(w["b_skip"], F64).reshape(1, -1, 1, 1, 1)
        return skip + h2
    return x + h2


def sliced_resblock_forward_ref(x, w: dict, hp, temb, slice_len: int):
    """Eq. 1 along frames: every window of frames goes through the whole group on its own and lands
    in its window of the preallocated output."""
    x = np.asarray(x, F64)
    parts = [resblock_forward_ref(x[:, :, f0:f1], w, hp, temb) for f0, f1 in slice_windows_ref(x.shape[2], slice_len)]
    return np.concatenate(parts, axis=2)


def downsample_ref(x, weight, bias=None):
    """Spatial DownSample of the group (Sec. 4.2.1 names the operator only; reading: the strided
    convolution of the latent-diffusion U-Nets): 3x3 convolution with zero padding 1 and stride 2,
    out[n, o, y, x] = bias[o] + sum weight[o, c, i, j] * a[n, c, 2y + i - 1, 2x + j - 1], i.e. the
    stride-1 convolution sampled at even pixels.  x: [B,C,F,H,W] -> [B,O,F,ceil(H/2),ceil(W/2)]."""
    x = np.asarray(x, F64)
    B, C, Fr, H, W = x.shape
    full = conv3x3_ref(_frames_first(x), weight, bias)
    return _frames_back(full[:, :, ::2, ::2], B, Fr)


def upsample_ref(x, weight, bias=None):
    """Spatial UpSample (reading: nearest-neighbour doubling followed by a 3x3 convolution, zero
    padding 1): u[n, c, Y, X] = a[n, c, Y // 2, X // 2]; out = Conv3x3(u) + bias.
    x: [B,C,F,H,W] -> [B,O,F,2H,2W]."""
    x = np.asarray(x, F64)
    B, C, Fr, H, W = x.shape
    u = np.repeat(np.repeat(_frames_first(x), 2, axis=2), 2, axis=3)
    return _frames_back(conv3x3_ref(u, weight, bias), B, Fr)


def sliced_resample_ref(x, weight, bias, kind: str, slice_len: int):
    """Eq. 1 along frames for the resampling operators (each frame is independent)."""
    x = np.asarray(x, F64)
    fn = downsample_ref if kind == "down" else upsample_ref
    parts = [fn(x[:, :, f0:f1], weight, bias) for f0, f1 in slice_windows_ref(x.shape[2], slice_len)]
    return np.concatenate(parts, axis=2)
