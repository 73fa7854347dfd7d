"""Test-side helpers: hyper-parameter objects and small random blocks."""
from __future__ import annotations

import numpy as np

import si_workloads as wl


def tiny_spec(kind, *, B=1, C=8, F=3, H=2, W=2, heads=2, dim_head=4, groups=2, pe=False,
              M=3, Cc=5, dtype="f32", seed=7, **kw):
    return wl.BlockSpec("tiny", kind, dtype, B, C, F, H, W, heads, dim_head, gn_groups=groups,
                        add_sin_pe=pe, ctx_tokens=M if kind == wl.SPATIAL else 0,
                        ctx_dim=Cc if kind == wl.SPATIAL else 0,
                        slice_axis=wl.AXIS_F if kind == wl.SPATIAL else wl.AXIS_HW,
                        slice_len=1, seed=seed, **kw)


def random_block(spec, *, std=0.3, affine=True, seed=None):
    w = wl.make_weights(spec, seed=seed, randomize_affine=affine, matrix_std=std)
    x = wl.make_x(spec, seed=seed)
    ctx = wl.make_context(spec, seed=seed)
    return x, w, ctx


def rel_l2(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))
