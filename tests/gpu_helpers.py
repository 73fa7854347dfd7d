"""GPU-side test helpers: move seeded NumPy inputs to the device and call the C-ABI binding."""
from __future__ import annotations

import numpy as np
import torch

import paper_2411_01171_amd as si
import si_workloads as wl

TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}
AXIS = {wl.AXIS_F: si.SI_AXIS_F, wl.AXIS_HW: si.SI_AXIS_HW}
KIND = {wl.TEMPORAL: si.SI_BLOCK_TEMPORAL, wl.SPATIAL: si.SI_BLOCK_SPATIAL}


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    """fp32 array holding storage-rounded values -> device tensor of the storage type (exact)."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda").to(TORCH_DTYPE[dtype]).contiguous()


def device_weights(spec: wl.BlockSpec, w: dict) -> si.BlockWeights:
    tensors = {k: to_dev(v, spec.dtype) for k, v in w.items()}
    return si.BlockWeights(KIND[spec.kind], spec.heads, spec.dim_head, spec.gn_groups, tensors,
                           gn_eps=spec.gn_eps, ln_eps=spec.ln_eps, add_sin_pe=spec.add_sin_pe)


def run_block(spec: wl.BlockSpec, x: np.ndarray, w: dict, ctx, slice_len=None, return_torch=False):
    xd = to_dev(x, spec.dtype)
    cd = None if ctx is None else to_dev(ctx, spec.dtype)
    wd = device_weights(spec, w)
    axis = AXIS[spec.slice_axis]
    sl = spec.slice_len if slice_len is None else slice_len
    nbytes = si.si_workspace_bytes(xd, wd, cd, axis, sl)
    assert nbytes > 0, "si_workspace_bytes rejected the arguments"
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    out = torch.full_like(xd, float("nan"))
    si.si_block_forward(xd, wd, cd, out, axis, sl, ws)
    torch.cuda.synchronize()
    if return_torch:
        return out
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


def device_res_weights(spec: wl.ResSpec, w: dict) -> si.ResBlockWeights:
    tensors = {k: to_dev(v, spec.dtype) for k, v in w.items()}
    return si.ResBlockWeights(spec.gn_groups, tensors, gn_eps=spec.gn_eps, temb_dim=spec.temb_dim, c_out=spec.C_out)


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
