"""ctypes binding of include/si.h.  Same names as the C entry points.

Tensors are torch tensors on a HIP device (torch is used for device memory
and streams only); descriptors are built from their shapes and data pointers.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence, Tuple

SI_F32, SI_BF16 = 0, 1
SI_BLOCK_TEMPORAL, SI_BLOCK_SPATIAL = 0, 1
SI_AXIS_F, SI_AXIS_HW = 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))


def library_path() -> str:
    return os.path.join(_HERE, "libsi.so")


class SiError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: si_status {status} ({si_status_str(status)})")


class _Tensor5(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("dtype", C.c_int32),
                ("B", C.c_int64), ("C", C.c_int64), ("F", C.c_int64), ("H", C.c_int64), ("W", C.c_int64)]


class _Context(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("dtype", C.c_int32),
                ("B", C.c_int64), ("M", C.c_int64), ("Cc", C.c_int64)]


WEIGHT_FIELDS = ("gn_g", "gn_b", "w_in", "b_in", "ln1_g", "ln1_b", "wq", "wk", "wv", "wo", "bo",
                 "ln2_g", "ln2_b", "wq2", "wk2", "wv2", "wo2", "bo2",
                 "ln3_g", "ln3_b", "w1", "b1", "w2", "b2", "w_out", "b_out")


class _Weights(C.Structure):
    _fields_ = ([("kind", C.c_int32), ("heads", C.c_int32), ("dim_head", C.c_int32), ("gn_groups", C.c_int32),
                 ("gn_eps", C.c_float), ("ln_eps", C.c_float), ("add_sin_pe", C.c_int32)]
                + [(n, C.c_void_p) for n in WEIGHT_FIELDS])


RES_WEIGHT_FIELDS = ("gn1_g", "gn1_b", "w_conv1", "b_conv1", "w_temb", "b_temb", "gn2_g", "gn2_b", "w_conv2", "b_conv2")


class _ResWeights(C.Structure):
    _fields_ = ([("gn_groups", C.c_int32), ("gn_eps", C.c_float), ("temb_dim", C.c_int32)]
                + [(n, C.c_void_p) for n in RES_WEIGHT_FIELDS]
                + [("c_out", C.c_int32), ("w_skip", C.c_void_p), ("b_skip", C.c_void_p)])


class _RehashCache(C.Structure):
    _fields_ = [("x_key", C.c_void_p), ("y_key", C.c_void_p), ("valid", C.c_int32)]


_lib = None


def lib() -> C.CDLL:
    """Loads libsi.so (built in-tree by paper_2411_01171_amd.build); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    L = C.CDLL(path)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    L.si_workspace_bytes.restype = sz
    L.si_workspace_bytes.argtypes = [C.POINTER(_Tensor5), C.POINTER(_Weights), C.POINTER(_Context), i32, i64]
    L.si_live_activation_bytes.restype = sz
    L.si_live_activation_bytes.argtypes = L.si_workspace_bytes.argtypes
    L.si_windows_in_flight.restype = i32
    L.si_windows_in_flight.argtypes = L.si_workspace_bytes.argtypes
    L.si_block_forward.restype = i32
    L.si_block_forward.argtypes = [C.POINTER(_Tensor5), C.POINTER(_Weights), C.POINTER(_Context), C.POINTER(_Tensor5),
                                   i32, i64, vp, sz, vp]
    L.si_block_forward_ex.restype = i32
    L.si_block_forward_ex.argtypes = L.si_block_forward.argtypes[:8] + [C.c_uint32, vp]
    L.si_block_forward_rehash.restype = i32
    L.si_block_forward_rehash.argtypes = L.si_block_forward.argtypes[:8] + [
        C.POINTER(_RehashCache), C.c_float, vp, C.POINTER(C.c_double), C.POINTER(i32)]
    L.si_resblock_workspace_bytes.restype = sz
    L.si_resblock_workspace_bytes.argtypes = [C.POINTER(_Tensor5), C.POINTER(_ResWeights), i64]
    L.si_resblock_live_activation_bytes.restype = sz
    L.si_resblock_live_activation_bytes.argtypes = L.si_resblock_workspace_bytes.argtypes
    L.si_resblock_forward.restype = i32
    L.si_resblock_forward.argtypes = [C.POINTER(_Tensor5), C.POINTER(_ResWeights), vp, C.POINTER(_Tensor5), i64, vp, sz, vp]
    L.si_resample_workspace_bytes.restype = sz
    L.si_resample_workspace_bytes.argtypes = [C.POINTER(_Tensor5), i32, i64]
    L.si_resample_forward.restype = i32
    L.si_resample_forward.argtypes = [C.POINTER(_Tensor5), i32, vp, vp, C.POINTER(_Tensor5), i64, vp, sz, vp]
    L.si_rehash_scratch_bytes.restype = sz
    L.si_rehash_scratch_bytes.argtypes = [i64]
    L.si_rehash_check.restype = i32
    L.si_rehash_check.argtypes = [vp, vp, i64, i32, C.c_float, vp, vp, vp, vp]
    L.si_rehash_check_sync.restype = i32
    L.si_rehash_check_sync.argtypes = [vp, vp, i64, i32, C.c_float, vp, vp, vp,
                                       C.POINTER(C.c_double), C.POINTER(i32)]
    L.si_init_device.restype = i32
    L.si_init_device.argtypes = []
    L.si_rehash_check_static.restype = i32
    L.si_rehash_check_static.argtypes = [vp, vp, i64, i32, C.c_float, vp, vp, vp]
    L.si_key_step_search.restype = i32
    L.si_key_step_search.argtypes = [C.POINTER(C.c_float), i32, C.c_float, C.POINTER(i32)]
    L.si_stage_timing_enable.restype = None
    L.si_stage_timing_enable.argtypes = [i32]
    L.si_stage_timing_read.restype = i32
    L.si_stage_timing_read.argtypes = [C.POINTER(C.c_char_p), C.POINTER(C.c_double), C.POINTER(i64), i32]
    L.si_status_str.restype = C.c_char_p
    L.si_status_str.argtypes = [i32]
    L.si_abi_version.restype = i32
    L.si_abi_version.argtypes = []
    _lib = L
    return L


def si_status_str(status: int) -> str:
    return lib().si_status_str(int(status)).decode()


def si_abi_version() -> int:
    return int(lib().si_abi_version())


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return SI_F32
    if t.dtype == torch.bfloat16:
        return SI_BF16
    return -1


def _tensor5(t) -> _Tensor5:
    if t.dim() != 5 or not t.is_contiguous():
        raise ValueError("feature must be a contiguous [B,C,F,H,W] tensor")
    B, Cc, F, H, W = t.shape
    return _Tensor5(t.data_ptr(), _dtype_code(t), B, Cc, F, H, W)


def _context(t) -> Optional[_Context]:
    if t is None:
        return None
    if t.dim() != 3 or not t.is_contiguous():
        raise ValueError("context must be a contiguous [B,M,Cc] tensor")
    return _Context(t.data_ptr(), _dtype_code(t), *t.shape)


class BlockWeights:
    """Holds the device tensors of one block and the matching C struct.

    `tensors` maps the field names of si_block_weights to torch tensors (or
    None); the tensors are kept alive by this object."""

    def __init__(self, kind: int, heads: int, dim_head: int, gn_groups: int, tensors: Dict[str, object],
                 gn_eps: float = 1e-6, ln_eps: float = 1e-5, add_sin_pe: bool = False):
        self.tensors = dict(tensors)
        s = _Weights()
        s.kind, s.heads, s.dim_head, s.gn_groups = kind, heads, dim_head, gn_groups
        s.gn_eps, s.ln_eps, s.add_sin_pe = gn_eps, ln_eps, int(bool(add_sin_pe))
        for name in WEIGHT_FIELDS:
            t = self.tensors.get(name)
            if t is not None and not t.is_contiguous():
                raise ValueError(f"{name} must be contiguous")
            setattr(s, name, None if t is None else t.data_ptr())
        self.struct = s


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return getattr(stream, "cuda_stream", stream) or None


def _pctx(ctx):
    c = _context(ctx)
    return (C.byref(c) if c is not None else None), c


def si_workspace_bytes(x, weights: BlockWeights, ctx, axis: int, slice_len: int) -> int:
    xd = _tensor5(x)
    pc, _keep = _pctx(ctx)
    return int(lib().si_workspace_bytes(C.byref(xd), C.byref(weights.struct), pc, axis, slice_len))


def si_live_activation_bytes(x, weights: BlockWeights, ctx, axis: int, slice_len: int) -> int:
    xd = _tensor5(x)
    pc, _keep = _pctx(ctx)
    return int(lib().si_live_activation_bytes(C.byref(xd), C.byref(weights.struct), pc, axis, slice_len))


def si_windows_in_flight(x, weights: BlockWeights, ctx, axis: int, slice_len: int) -> int:
    xd = _tensor5(x)
    pc, _keep = _pctx(ctx)
    return int(lib().si_windows_in_flight(C.byref(xd), C.byref(weights.struct), pc, axis, slice_len))


SI_FWD_WEIGHTS_PACKED = 1


def si_block_forward(x, weights: BlockWeights, ctx, out, axis: int, slice_len: int, workspace, stream=None) -> None:
    """Enqueues the sliced block forward on `stream` (default: torch's current stream)."""
    xd, od = _tensor5(x), _tensor5(out)
    pc, _keep = _pctx(ctx)
    st = lib().si_block_forward(C.byref(xd), C.byref(weights.struct), pc, C.byref(od), axis, slice_len,
                                workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                _stream_ptr(stream))
    if st != 0:
        raise SiError(st, "si_block_forward")


def si_block_forward_ex(x, weights: BlockWeights, ctx, out, axis: int, slice_len: int, workspace, flags: int = 0,
                        stream=None) -> None:
    """si_block_forward with flags (SI_FWD_WEIGHTS_PACKED: the workspace still holds these weights re-laid-out)."""
    xd, od = _tensor5(x), _tensor5(out)
    pc, _keep = _pctx(ctx)
    st = lib().si_block_forward_ex(C.byref(xd), C.byref(weights.struct), pc, C.byref(od), axis, slice_len,
                                   workspace.data_ptr(), workspace.numel() * workspace.element_size(), flags,
                                   _stream_ptr(stream))
    if st != 0:
        raise SiError(st, "si_block_forward_ex")


class ResBlockWeights:
    """Device tensors of one Spatial ResBlock and the matching C struct (kept alive by this object)."""

    def __init__(self, gn_groups: int, tensors: Dict[str, object], gn_eps: float = 1e-6, temb_dim: int = 0, c_out: int = 0):
        self.tensors = dict(tensors)
        s = _ResWeights()
        s.gn_groups, s.gn_eps, s.temb_dim, s.c_out = gn_groups, gn_eps, temb_dim, c_out
        for name in RES_WEIGHT_FIELDS + ("w_skip", "b_skip"):
            t = self.tensors.get(name)
            if t is not None and not t.is_contiguous():
                raise ValueError(f"{name} must be contiguous")
            setattr(s, name, None if t is None else t.data_ptr())
        self.struct = s


def si_resblock_workspace_bytes(x, weights: ResBlockWeights, slice_len: int) -> int:
    xd = _tensor5(x)
    return int(lib().si_resblock_workspace_bytes(C.byref(xd), C.byref(weights.struct), slice_len))


def si_resblock_live_activation_bytes(x, weights: ResBlockWeights, slice_len: int) -> int:
    xd = _tensor5(x)
    return int(lib().si_resblock_live_activation_bytes(C.byref(xd), C.byref(weights.struct), slice_len))


def si_resblock_forward(x, weights: ResBlockWeights, temb, out, slice_len: int, workspace, stream=None) -> None:
    """Enqueues the sliced Spatial ResBlock forward (frame windows of `slice_len`) on `stream`."""
    xd, od = _tensor5(x), _tensor5(out)
    if temb is not None and not temb.is_contiguous():
        raise ValueError("temb must be contiguous")
    st = lib().si_resblock_forward(C.byref(xd), C.byref(weights.struct), None if temb is None else temb.data_ptr(),
                                   C.byref(od), slice_len, workspace.data_ptr(),
                                   workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    if st != 0:
        raise SiError(st, "si_resblock_forward")


SI_RESAMPLE_DOWN, SI_RESAMPLE_UP = 0, 1


def si_resample_workspace_bytes(x, kind: int, slice_len: int) -> int:
    xd = _tensor5(x)
    return int(lib().si_resample_workspace_bytes(C.byref(xd), kind, slice_len))


def si_resample_forward(x, kind: int, w_conv, b_conv, out, slice_len: int, workspace, stream=None) -> None:
    """Enqueues the sliced Spatial Down/UpSample (3x3 convolution, stride 2 / after nearest doubling)."""
    xd, od = _tensor5(x), _tensor5(out)
    if not w_conv.is_contiguous() or (b_conv is not None and not b_conv.is_contiguous()):
        raise ValueError("parameters must be contiguous")
    st = lib().si_resample_forward(C.byref(xd), kind, w_conv.data_ptr(), None if b_conv is None else b_conv.data_ptr(),
                                   C.byref(od), slice_len, workspace.data_ptr(),
                                   workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    if st != 0:
        raise SiError(st, "si_resample_forward")


class RehashCache:
    """Anchor buffers of si_block_forward_rehash for one block (device tensors shaped like the feature)."""

    def __init__(self, like):
        import torch
        self.x_key = torch.empty_like(like)
        self.y_key = torch.empty_like(like)
        self.struct = _RehashCache(self.x_key.data_ptr(), self.y_key.data_ptr(), 0)

    @property
    def valid(self) -> bool:
        return bool(self.struct.valid)

    def reset(self) -> None:
        self.struct.valid = 0


def si_block_forward_rehash(x, weights: BlockWeights, ctx, out, axis: int, slice_len: int, workspace,
                            cache: RehashCache, gamma: float, stream=None) -> Tuple[bool, float]:
    """Step Rehash around the block, decided on its input.  Returns (reused, cos); waits for the stream
    when the cache holds an anchor."""
    xd, od = _tensor5(x), _tensor5(out)
    pc, _keep = _pctx(ctx)
    cos, reused = C.c_double(), C.c_int32()
    st = lib().si_block_forward_rehash(C.byref(xd), C.byref(weights.struct), pc, C.byref(od), axis, slice_len,
                                       workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                       C.byref(cache.struct), gamma, _stream_ptr(stream),
                                       C.byref(cos), C.byref(reused))
    if st != 0:
        raise SiError(st, "si_block_forward_rehash")
    return bool(reused.value), cos.value


def si_rehash_scratch_bytes(n: int) -> int:
    return int(lib().si_rehash_scratch_bytes(n))


def si_rehash_check(feat_t, feat_prev, thresh: float, cos_dev, decision_dev, scratch, stream=None) -> None:
    """Enqueues the similarity test; results land in cos_dev (float64[1] or None) and decision_dev (int32[1])."""
    if feat_t.numel() != feat_prev.numel() or feat_t.dtype != feat_prev.dtype:
        raise ValueError("features must have the same size and dtype")
    if not (feat_t.is_contiguous() and feat_prev.is_contiguous()):
        raise ValueError("features must be contiguous")
    st = lib().si_rehash_check(feat_t.data_ptr(), feat_prev.data_ptr(), feat_t.numel(), _dtype_code(feat_t),
                               thresh, None if cos_dev is None else cos_dev.data_ptr(), decision_dev.data_ptr(),
                               scratch.data_ptr(), _stream_ptr(stream))
    if st != 0:
        raise SiError(st, "si_rehash_check")


def si_init_device() -> None:
    st = lib().si_init_device()
    if st != 0:
        raise SiError(st, "si_init_device")


def si_rehash_check_static(feat_t, feat_prev, thresh: float, cos_dev, decision_dev, stream=None) -> None:
    """si_rehash_check without a scratch argument: the partial sums live in the library's device array."""
    if feat_t.numel() != feat_prev.numel() or feat_t.dtype != feat_prev.dtype:
        raise ValueError("features must have the same size and dtype")
    if not (feat_t.is_contiguous() and feat_prev.is_contiguous()):
        raise ValueError("features must be contiguous")
    st = lib().si_rehash_check_static(feat_t.data_ptr(), feat_prev.data_ptr(), feat_t.numel(), _dtype_code(feat_t),
                                      thresh, None if cos_dev is None else cos_dev.data_ptr(), decision_dev.data_ptr(),
                                      _stream_ptr(stream))
    if st != 0:
        raise SiError(st, "si_rehash_check_static")


def si_rehash_check_sync(feat_t, feat_prev, thresh: float, scratch, result_dev, stream=None) -> Tuple[float, int]:
    if feat_t.numel() != feat_prev.numel() or feat_t.dtype != feat_prev.dtype:
        raise ValueError("features must have the same size and dtype")
    cos, dec = C.c_double(), C.c_int32()
    st = lib().si_rehash_check_sync(feat_t.data_ptr(), feat_prev.data_ptr(), feat_t.numel(), _dtype_code(feat_t),
                                    thresh, scratch.data_ptr(), result_dev.data_ptr(), _stream_ptr(stream),
                                    C.byref(cos), C.byref(dec))
    if st != 0:
        raise SiError(st, "si_rehash_check_sync")
    return cos.value, dec.value


def si_key_step_search(S: Sequence[Sequence[float]], gamma: float) -> List[int]:
    """Algorithm 1 on a K x K similarity map (host)."""
    K = len(S)
    flat = (C.c_float * (K * K))(*[float(v) for row in S for v in row])
    G = (C.c_int32 * max(K, 1))()
    n = lib().si_key_step_search(flat, K, gamma, G)
    if n < 0:
        raise SiError(7, "si_key_step_search")
    return [int(G[i]) for i in range(n)]


def si_stage_timing_enable(on: bool) -> None:
    lib().si_stage_timing_enable(int(bool(on)))


def si_stage_timing_read() -> Dict[str, Tuple[float, int]]:
    """{stage: (total milliseconds, launches)} since the last read."""
    cap = 64
    names = (C.c_char_p * cap)()
    ms = (C.c_double * cap)()
    cnt = (C.c_int64 * cap)()
    n = lib().si_stage_timing_read(names, ms, cnt, cap)
    if n < 0:
        raise SiError(8, "si_stage_timing_read")
    return {names[i].decode(): (ms[i], int(cnt[i])) for i in range(min(n, cap)) if cnt[i] > 0}
