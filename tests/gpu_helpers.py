"""GPU-side test helpers: move seeded NumPy inputs to the device and call the C-ABI binding."""
from __future__ import annotations

import numpy as np
import torch

import paper_2411_01171_amd as si
import si_workloads as wl

from paper_2411_01171_amd.devio import AXIS, KIND, TORCH_DTYPE, device_res_weights, device_weights, to_dev  # noqa: F401


GUARD_BYTES = 4096


def guarded(nbytes_or_like, dtype=None):
    """Device buffer with GUARD_BYTES of 0xFF bytes (NaN in bf16 / fp32) before and after it.

    Returns (whole uint8 buffer, view of the middle).  With a tensor argument the middle has its
    shape and dtype and is filled with NaN; with a byte count it is raw uint8."""
    if isinstance(nbytes_or_like, int):
        n, like = nbytes_or_like, None
    else:
        like = nbytes_or_like
        n = like.numel() * like.element_size()
    pad = (-n) % 256
    buf = torch.full((GUARD_BYTES + n + pad + GUARD_BYTES,), 0xFF, dtype=torch.uint8, device="cuda")
    mid = buf[GUARD_BYTES:GUARD_BYTES + n]
    if like is not None:
        mid = mid.view(like.dtype).view(like.shape)
    return buf, mid


def guards_intact(buf, n) -> bool:
    """True when the bytes before and after the n-byte middle of a guarded() buffer still hold 0xFF."""
    head = buf[:GUARD_BYTES]
    tail = buf[GUARD_BYTES + n:]
    return bool((head == 0xFF).all().item()) and bool((tail == 0xFF).all().item())


def run_block(spec: wl.BlockSpec, x: np.ndarray, w: dict, ctx, slice_len=None, return_torch=False):
    """One si_block_forward call; `out` starts as NaN and both `out` and the workspace sit between
    guard bands that the call must leave untouched."""
    xd = to_dev(x, spec.dtype)
    cd = None if ctx is None else to_dev(ctx, spec.dtype)
    wd = device_weights(spec, w)
    axis = AXIS[spec.slice_axis]
    sl = spec.slice_len if slice_len is None else slice_len
    nbytes = si.si_workspace_bytes(xd, wd, cd, axis, sl)
    assert nbytes > 0, "si_workspace_bytes rejected the arguments"
    ws_buf, ws = guarded(nbytes)
    out_buf, out = guarded(xd)
    si.si_block_forward(xd, wd, cd, out, axis, sl, ws)
    torch.cuda.synchronize()
    assert guards_intact(out_buf, out.numel() * out.element_size()), "write outside `out`"
    assert guards_intact(ws_buf, nbytes), "write outside the workspace"
    if return_torch:
        return out.clone()
    return out.float().cpu().numpy().astype(np.float64)


def errors(out: np.ndarray, ref: np.ndarray, x: np.ndarray):
    out = np.asarray(out, np.float64); ref = np.asarray(ref, np.float64); x = np.asarray(x, np.float64)
    d = out - ref
    branch = ref - x
    return {
        "max_abs": float(np.max(np.abs(d))),
        "rel_l2": float(np.linalg.norm(d) / np.linalg.norm(ref)),
        "rel_l2_branch": float(np.linalg.norm(d) / max(np.linalg.norm(branch), 1e-300)),
        "max_ref": float(np.max(np.abs(ref))),
    }


def run_resblock(spec: wl.ResSpec, x: np.ndarray, w: dict, temb, slice_len=None) -> np.ndarray:
    xd = to_dev(x, spec.dtype)
    td = None if temb is None else to_dev(temb, spec.dtype)
    wd = device_res_weights(spec, w)
    sl = spec.slice_len if slice_len is None else slice_len
    nbytes = si.si_resblock_workspace_bytes(xd, wd, sl)
    assert nbytes > 0, "si_resblock_workspace_bytes rejected the arguments"
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    B, C, F, H, W = xd.shape
    out = torch.full((B, spec.C_out or C, F, H, W), float("nan"), dtype=xd.dtype, device="cuda")
    si.si_resblock_forward(xd, wd, td, out, sl, ws)
    torch.cuda.synchronize()
    return out.float().cpu().numpy().astype(np.float64)
