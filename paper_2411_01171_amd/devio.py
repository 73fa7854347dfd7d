"""Host arrays -> device tensors for the binding's callers (tests, benchmark).

Marshalling only: seeded NumPy arrays that already hold storage-rounded values
are moved to the GPU in the storage type (exact), and the weight structs of the
binding are filled from dictionaries of such arrays."""
from __future__ import annotations

import numpy as np
import torch

import si_workloads as wl

from . import binding as si

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


def device_res_weights(spec: wl.ResSpec, w: dict) -> si.ResBlockWeights:
    tensors = {k: to_dev(v, spec.dtype) for k, v in w.items()}
    return si.ResBlockWeights(spec.gn_groups, tensors, gn_eps=spec.gn_eps, temb_dim=spec.temb_dim, c_out=spec.C_out)
