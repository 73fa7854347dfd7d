"""Seeded synthetic workloads: shapes, slicing plans and random tensors.

This module is the only code shared by the CPU oracle's tests and the HIP
path's tests / benchmark.  It holds no arithmetic of the method: it names the
five workload shapes, draws seeded Gaussian tensors with NumPy's PCG64, and
rounds them to the storage type (bf16 round-to-nearest-even, kept in fp32
containers so that both sides read identical values).

The shapes stand in for the paper's workloads (AnimateDiff 512x512x16f with a
64x64 latent and 320 channels at the top level; SVD-XT 576x1024x25f with a
72x128 latent; classifier-free guidance doubling the batch, Sec. 3 and Sec. 5
"Experimental setup"); trained weights and video datasets are not used.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Optional

import numpy as np

TEMPORAL = "temporal"
SPATIAL = "spatial"
AXIS_F = "F"
AXIS_HW = "HW"


@dataclasses.dataclass(frozen=True)
class BlockSpec:
    """One transformer block workload (shape + hyper-parameters + slice plan)."""
    name: str
    kind: str                # TEMPORAL | SPATIAL
    dtype: str               # "f32" | "bf16"
    B: int
    C: int
    F: int
    H: int
    W: int
    heads: int
    dim_head: int
    gn_groups: int = 32
    gn_eps: float = 1e-6
    ln_eps: float = 1e-5
    add_sin_pe: bool = False
    ctx_tokens: int = 0      # M (spatial only)
    ctx_dim: int = 0         # Cc (spatial only)
    slice_axis: str = AXIS_HW
    slice_len: int = 0
    seed: int = 0

    @property
    def D(self) -> int:
        return self.heads * self.dim_head

    @property
    def tokens(self) -> int:
        return self.B * self.F * self.H * self.W

    def flops(self) -> float:
        """Algorithmic FLOPs of one block forward: GEMMs (2mnk) plus attention
        (4*Nq*Nk*d per head); norms, softmax, GELU and padding are not counted."""
        T, C, D = self.tokens, self.C, self.D
        P = self.H * self.W
        gemm = 2.0 * T * (C * D + 3 * D * D + D * D + D * 8 * D + 4 * D * D + D * C)
        if self.kind == TEMPORAL:
            attn = 4.0 * T * self.F * D
        else:
            attn = 4.0 * T * P * D
            gemm += 2.0 * T * (D * D + D * D)                      # q2, o2
            gemm += 2.0 * self.B * self.ctx_tokens * self.ctx_dim * 2 * D  # ctx k,v once
            attn += 4.0 * T * self.ctx_tokens * D
        return gemm + attn


CONFIGS: Dict[str, BlockSpec] = {
    "cfg1": BlockSpec("cfg1", TEMPORAL, "f32", 1, 64, 8, 8, 8, 1, 64,
                      slice_axis=AXIS_HW, slice_len=16, seed=1000),
    "cfg2": BlockSpec("cfg2", TEMPORAL, "bf16", 2, 320, 16, 64, 64, 8, 40, add_sin_pe=True,
                      slice_axis=AXIS_HW, slice_len=1024, seed=2000),
    "cfg3": BlockSpec("cfg3", SPATIAL, "bf16", 2, 640, 16, 32, 32, 10, 64,
                      ctx_tokens=77, ctx_dim=768, slice_axis=AXIS_F, slice_len=1, seed=3000),
    "cfg4s": BlockSpec("cfg4s", SPATIAL, "bf16", 2, 320, 25, 72, 128, 5, 64,
                       ctx_tokens=1, ctx_dim=1024, slice_axis=AXIS_F, slice_len=1, seed=4000),
    "cfg4t": BlockSpec("cfg4t", TEMPORAL, "bf16", 2, 320, 25, 72, 128, 5, 64,
                       slice_axis=AXIS_HW, slice_len=1152, seed=4500),
    "cfg5s": BlockSpec("cfg5s", SPATIAL, "bf16", 2, 1280, 16, 16, 16, 20, 64,
                       ctx_tokens=77, ctx_dim=768, slice_axis=AXIS_F, slice_len=4, seed=5000),
    "cfg5t": BlockSpec("cfg5t", TEMPORAL, "bf16", 2, 1280, 16, 16, 16, 20, 64,
                       slice_axis=AXIS_HW, slice_len=64, seed=5500),
}

CFG5_PAIRS = 4
CFG5_STEPS = 10
CFG5_GAMMA = 0.95

MATRIX_NAMES_COMMON = ("w_in", "wq", "wk", "wv", "wo", "w1", "w2", "w_out")
MATRIX_NAMES_SPATIAL = ("wq2", "wk2", "wv2", "wo2")


def round_to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round an fp32 array to the storage type and return it as fp32.

    "f32": unchanged.  "bf16": round-to-nearest-even on the upper 16 bits."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return a
    if dtype != "bf16":
        raise ValueError(dtype)
    bits = a.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def _normal(seed: int, shape, std: float, dtype: str) -> np.ndarray:
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(size=shape, dtype=np.float32) * np.float32(std)
    return round_to_storage(a, dtype)


def weight_shapes(spec: BlockSpec) -> Dict[str, tuple]:
    """Shape of every parameter; matrices are row-major [in, out]."""
    C, D = spec.C, spec.D
    shapes = {
        "gn_g": (C,), "gn_b": (C,),
        "w_in": (C, D), "b_in": (D,),
        "ln1_g": (D,), "ln1_b": (D,),
        "wq": (D, D), "wk": (D, D), "wv": (D, D), "wo": (D, D), "bo": (D,),
        "ln3_g": (D,), "ln3_b": (D,),
        "w1": (D, 8 * D), "b1": (8 * D,), "w2": (4 * D, D), "b2": (D,),
        "w_out": (D, C), "b_out": (C,),
    }
    if spec.kind == SPATIAL:
        shapes.update({
            "ln2_g": (D,), "ln2_b": (D,),
            "wq2": (D, D), "wk2": (spec.ctx_dim, D), "wv2": (spec.ctx_dim, D),
            "wo2": (D, D), "bo2": (D,),
        })
    return shapes


def make_weights(spec: BlockSpec, seed: Optional[int] = None, *, randomize_affine: bool = False,
                 matrix_std: float = 0.02) -> Dict[str, np.ndarray]:
    """Parameters of one block as fp32 arrays holding storage-rounded values.

    Default recipe: matrices ~ N(0, matrix_std^2), biases 0, norm gains 1 and
    shifts 0.  `randomize_affine` draws gains ~ N(1, 0.1^2) and shifts / biases
    ~ N(0, 0.1^2) instead, to exercise the affine and bias paths."""
    seed = spec.seed if seed is None else seed
    out: Dict[str, np.ndarray] = {}
    for k, (name, shape) in enumerate(weight_shapes(spec).items()):
        s = seed + 2 + k
        if len(shape) == 2:
            out[name] = _normal(s, shape, matrix_std, spec.dtype)
        elif name.endswith("_g"):
            if randomize_affine:
                out[name] = round_to_storage(1.0 + _normal(s, shape, 0.1, "f32"), spec.dtype)
            else:
                out[name] = np.ones(shape, np.float32)
        else:
            if randomize_affine:
                out[name] = _normal(s, shape, 0.1, spec.dtype)
            else:
                out[name] = np.zeros(shape, np.float32)
    return out


def make_x(spec: BlockSpec, seed: Optional[int] = None, mean: float = 0.0) -> np.ndarray:
    seed = spec.seed if seed is None else seed
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(size=(spec.B, spec.C, spec.F, spec.H, spec.W), dtype=np.float32)
    if mean:
        a += np.float32(mean)
    return round_to_storage(a, spec.dtype)


def make_context(spec: BlockSpec, seed: Optional[int] = None) -> Optional[np.ndarray]:
    if spec.kind != SPATIAL:
        return None
    seed = spec.seed if seed is None else seed
    return _normal(seed + 1, (spec.B, spec.ctx_tokens, spec.ctx_dim), 1.0, spec.dtype)


def cfg5_sigma(t: int) -> float:
    """Noise scale added at step t (1..9): linear from 0.2 down to 0.01."""
    return 0.2 - (t - 1) * (0.19 / 8.0)


def cfg5_step_input(prev: np.ndarray, t: int, dtype: str = "bf16") -> np.ndarray:
    """x_t = x_{t-1} + sigma_t * N(0,1), noise seeded per step, rounded once."""
    rng = np.random.default_rng(5000 + 100 + t)
    noise = rng.standard_normal(size=prev.shape, dtype=np.float32)
    return round_to_storage(prev + np.float32(cfg5_sigma(t)) * noise, dtype)


def scaled(spec: BlockSpec, **kw) -> BlockSpec:
    """A copy of `spec` with some fields replaced (small parity shapes)."""
    return dataclasses.replace(spec, **kw)


# ----------------------------------------------------------------------------- Spatial ResBlock group

@dataclasses.dataclass(frozen=True)
class ResSpec:
    """Shape of one Spatial ResBlock workload (GroupNorm, SiLU, 3x3 convolutions, identity skip)."""
    name: str
    dtype: str
    B: int
    C: int
    F: int
    H: int
    W: int
    temb_dim: int = 0        # 0: no timestep-embedding term
    C_out: int = 0           # 0: same as C (identity skip); else the 1x1 skip convolution maps C -> C_out
    gn_groups: int = 32
    gn_eps: float = 1e-6
    slice_len: int = 1       # frames per slice
    seed: int = 0

    @property
    def tokens(self) -> int:
        return self.B * self.F * self.H * self.W

    def flops(self) -> float:
        """Two 3x3 convolutions as dense contractions (2 * positions * 9 * C * C each, padding taps
        counted) plus the embedding projection; norms and SiLU are not counted."""
        Co = self.C_out or self.C
        skip = 2.0 * self.tokens * self.C * Co if Co != self.C else 0.0
        return 2.0 * self.tokens * 9 * (self.C * Co + Co * Co) + skip + 2.0 * self.B * self.temb_dim * Co


RES_CONFIGS: Dict[str, ResSpec] = {
    # SVD-XT-shaped first-level ResBlock: the feature of cfg4, one frame per slice
    "res4": ResSpec("res4", "bf16", 2, 320, 25, 72, 128, temb_dim=1280, slice_len=1, seed=7000),
    # deeper level, smaller map: C = 640 at 36 x 64, two frames per slice
    "res4b": ResSpec("res4b", "bf16", 2, 640, 25, 36, 64, temb_dim=1280, slice_len=2, seed=7100),
    # level transition: 320 -> 640 channels with the 1x1 skip, at the deeper level's map
    "res4c": ResSpec("res4c", "bf16", 2, 320, 25, 36, 64, temb_dim=1280, C_out=640, slice_len=2, seed=7300),
    # small case the oracle finishes in seconds; map sizes that are no multiple of any tile
    "res1": ResSpec("res1", "bf16", 2, 64, 3, 10, 12, temb_dim=32, slice_len=2, seed=7200),
}


def res_weight_shapes(spec: ResSpec) -> Dict[str, tuple]:
    C, Co = spec.C, spec.C_out or spec.C
    shapes = {"gn1_g": (C,), "gn1_b": (C,), "w_conv1": (Co, C, 3, 3), "b_conv1": (Co,),
              "gn2_g": (Co,), "gn2_b": (Co,), "w_conv2": (Co, Co, 3, 3), "b_conv2": (Co,)}
    if spec.temb_dim:
        shapes.update({"w_temb": (spec.temb_dim, Co), "b_temb": (Co,)})
    if Co != C:
        shapes.update({"w_skip": (Co, C), "b_skip": (Co,)})
    return shapes


def make_res_weights(spec: ResSpec, seed: Optional[int] = None, *, randomize_affine: bool = False,
                     kernel_std: float = 0.02) -> Dict[str, np.ndarray]:
    """Kernels and W_t ~ N(0, kernel_std^2); biases 0, gains 1, shifts 0 unless `randomize_affine`
    (gains ~ N(1, 0.1^2), shifts and biases ~ N(0, 0.1^2))."""
    seed = spec.seed if seed is None else seed
    out: Dict[str, np.ndarray] = {}
    for k, (name, shape) in enumerate(res_weight_shapes(spec).items()):
        s = seed + 2 + k
        if len(shape) >= 2:
            out[name] = _normal(s, shape, kernel_std, spec.dtype)
        elif name.endswith("_g"):
            out[name] = (round_to_storage(1.0 + _normal(s, shape, 0.1, "f32"), spec.dtype) if randomize_affine
                         else np.ones(shape, np.float32))
        else:
            out[name] = _normal(s, shape, 0.1, spec.dtype) if randomize_affine else np.zeros(shape, np.float32)
    return out


def make_temb(spec: ResSpec, seed: Optional[int] = None) -> Optional[np.ndarray]:
    if not spec.temb_dim:
        return None
    seed = spec.seed if seed is None else seed
    return _normal(seed + 1, (spec.B, spec.temb_dim), 1.0, spec.dtype)
