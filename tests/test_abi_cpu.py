"""Host-side checks that need no GPU: the library loads, exports every symbol the header
declares, validates arguments before any GPU call, and runs Algorithm 1 on the host."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
import paper_2411_01171_amd as si
from paper_2411_01171_amd import binding as B
from test_oracle_rehash import _golden_cases, _rule_matrix

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "si.h")


def _declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(si_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert {"si_block_forward", "si_rehash_check", "si_workspace_bytes", "si_key_step_search"} <= set(names)
    lib = si.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert si.si_abi_version() >= 1
    assert si.si_status_str(0) == "ok" and "slice" in si.si_status_str(4)


def _descs(kind=B.SI_BLOCK_TEMPORAL, dtype=B.SI_BF16, Bn=2, Cn=64, F=4, H=8, W=8, heads=2, dh=32, groups=8, fake=0x10000):
    x = B._Tensor5(fake, dtype, Bn, Cn, F, H, W)
    out = B._Tensor5(fake + (1 << 30), dtype, Bn, Cn, F, H, W)
    w = B._Weights()
    w.kind, w.heads, w.dim_head, w.gn_groups, w.gn_eps, w.ln_eps, w.add_sin_pe = kind, heads, dh, groups, 1e-6, 1e-5, 0
    for name in B.WEIGHT_FIELDS:
        setattr(w, name, fake + (2 << 30))
    ctx = B._Context(fake + (3 << 30), dtype, Bn, 5, 16)
    return x, w, ctx, out


def _forward(x, w, ctx, out, axis, slice_len, ws=0x7000000000, ws_bytes=1 << 40):
    return si.lib().si_block_forward(C.byref(x), C.byref(w), C.byref(ctx) if ctx is not None else None, C.byref(out),
                                     axis, slice_len, ws, ws_bytes, None)


def _wsbytes(x, w, ctx, axis, slice_len):
    return si.lib().si_workspace_bytes(C.byref(x), C.byref(w), C.byref(ctx) if ctx is not None else None, axis, slice_len)


def test_argument_validation_returns_codes_without_touching_the_gpu():
    x, w, ctx, out = _descs()
    assert _wsbytes(x, w, None, B.SI_AXIS_HW, 16) > 0
    # slicing a temporal block along frames is not lossless -> refused; same for spatial along positions
    assert _forward(x, w, None, out, B.SI_AXIS_F, 1) == 4
    assert _wsbytes(x, w, None, B.SI_AXIS_F, 1) == 0
    xs, ws_, cs, os_ = _descs(kind=B.SI_BLOCK_SPATIAL)
    assert _forward(xs, ws_, cs, os_, B.SI_AXIS_HW, 16) == 4
    assert _forward(xs, ws_, None, os_, B.SI_AXIS_F, 1) == 1          # spatial block without context
    assert _forward(x, w, None, out, B.SI_AXIS_HW, 0) == 4           # slice_len < 1
    assert _forward(x, w, None, out, 7, 4) == 4                      # unknown axis
    bad = B._Tensor5(x.ptr, 5, 2, 64, 4, 8, 8)
    assert _forward(bad, w, None, out, B.SI_AXIS_HW, 4) == 3          # unknown dtype
    o32 = B._Tensor5(out.ptr, B.SI_F32, 2, 64, 4, 8, 8)
    assert _forward(x, w, None, o32, B.SI_AXIS_HW, 4) == 3            # dtype mismatch
    o2 = B._Tensor5(out.ptr, B.SI_BF16, 2, 64, 4, 8, 9)
    assert _forward(x, w, None, o2, B.SI_AXIS_HW, 4) == 2             # shape mismatch
    x3, w3, _, out3 = _descs(Cn=60)
    assert _forward(x3, w3, None, out3, B.SI_AXIS_HW, 4) == 2         # C not divisible by groups / 8
    x4, w4, _, out4 = _descs(dh=20)
    assert _forward(x4, w4, None, out4, B.SI_AXIS_HW, 4) == 2         # dim_head not a multiple of 8
    xn = B._Tensor5(None, B.SI_BF16, 2, 64, 4, 8, 8)
    assert _forward(xn, w, None, out, B.SI_AXIS_HW, 4) == 1           # NULL feature
    w5 = _descs()[1]; w5.w1 = None
    assert _forward(x, w5, None, out, B.SI_AXIS_HW, 4) == 1           # NULL required matrix
    xm = B._Tensor5(x.ptr + 2, B.SI_BF16, 2, 64, 4, 8, 8)
    assert _forward(xm, w, None, out, B.SI_AXIS_HW, 4) == 5           # misaligned
    assert _forward(x, w, None, out, B.SI_AXIS_HW, 4, ws_bytes=1024) == 6   # workspace too small
    alias = B._Tensor5(x.ptr + 4096, B.SI_BF16, 2, 64, 4, 8, 8)
    assert _forward(x, w, None, alias, B.SI_AXIS_HW, 4) == 7          # out overlaps x
    assert si.lib().si_block_forward(None, None, None, None, 3, 1, None, 0, None) == 1


def test_forward_rehash_validation():
    x, w, _, out = _descs()
    lib = si.lib()
    fake = 0x10000
    reused, cos = C.c_int32(-1), C.c_double()

    def call(cache, gamma=0.95, xd=x, reused_p=C.byref(reused)):
        return lib.si_block_forward_rehash(C.byref(xd), C.byref(w), None, C.byref(out), B.SI_AXIS_HW, 4,
                                           0x7000000000, 1 << 40, cache, gamma, None, C.byref(cos), reused_p)

    good = B._RehashCache(fake + (4 << 30), fake + (5 << 30), 0)
    assert call(None) == 1                                             # no cache
    assert call(C.byref(good), reused_p=None) == 1                     # no place for the decision
    assert call(C.byref(B._RehashCache(None, fake + (5 << 30), 0))) == 1
    assert call(C.byref(B._RehashCache(fake + (4 << 30) + 4, fake + (5 << 30), 0))) == 5
    assert call(C.byref(good), gamma=float("nan")) == 7
    assert call(C.byref(B._RehashCache(x.ptr, fake + (5 << 30), 0))) == 7              # anchor aliases x
    assert call(C.byref(B._RehashCache(fake + (4 << 30), out.ptr + 256, 0))) == 7      # anchor overlaps out partially
    assert call(C.byref(B._RehashCache(fake + (4 << 30), fake + (4 << 30) + 1024, 0))) == 7  # anchors overlap
    assert call(C.byref(B._RehashCache(0x7000000000 + 4096, fake + (5 << 30), 0))) == 7      # inside the workspace
    bad = B._Tensor5(x.ptr, 5, 2, 64, 4, 8, 8)
    assert call(C.byref(good), xd=bad) == 3                            # the forward's own checks come first
    assert reused.value == -1 and good.valid == 0                      # nothing was decided or enqueued


def test_resblock_validation_and_workspace():
    lib = si.lib()
    fake = 0x10000
    x = B._Tensor5(fake, B.SI_BF16, 2, 64, 8, 6, 6)
    out = B._Tensor5(fake + (1 << 30), B.SI_BF16, 2, 64, 8, 6, 6)
    w = B._ResWeights()
    w.gn_groups, w.gn_eps, w.temb_dim = 32, 1e-6, 16
    for name in B.RES_WEIGHT_FIELDS:
        setattr(w, name, fake + (2 << 30))

    def call(xd=x, od=out, wd=w, temb=fake + (3 << 30), slice_len=1, ws=0x7000000000, ws_bytes=1 << 40):
        return lib.si_resblock_forward(C.byref(xd), C.byref(wd), temb, C.byref(od), slice_len, ws, ws_bytes, None)

    assert lib.si_resblock_workspace_bytes(C.byref(x), C.byref(w), 1) > 0
    assert call(slice_len=0) == 4
    assert call(temb=None) == 1                                         # embedding width > 0 needs temb
    assert call(xd=B._Tensor5(fake, B.SI_F32, 2, 64, 8, 6, 6)) == 3     # bf16 features only
    assert call(xd=B._Tensor5(fake, B.SI_BF16, 2, 48, 8, 6, 6), od=B._Tensor5(out.ptr, B.SI_BF16, 2, 48, 8, 6, 6)) == 2
    assert call(od=B._Tensor5(out.ptr, B.SI_BF16, 2, 64, 8, 6, 7)) == 2
    assert call(od=B._Tensor5(x.ptr + 1024, B.SI_BF16, 2, 64, 8, 6, 6)) == 7
    assert call(xd=B._Tensor5(fake + 2, B.SI_BF16, 2, 64, 8, 6, 6)) == 5
    assert call(ws_bytes=4096) == 6
    w2 = B._ResWeights.from_buffer_copy(w); w2.w_conv2 = None
    assert call(wd=w2) == 1
    w3 = B._ResWeights.from_buffer_copy(w); w3.gn_groups = 5
    assert call(wd=w3) == 2
    w4 = B._ResWeights.from_buffer_copy(w); w4.c_out = 96                  # channel change
    o96 = B._Tensor5(out.ptr, B.SI_BF16, 2, 96, 8, 6, 6)
    assert call(wd=w4) == 2                                               # out must have c_out channels
    assert call(wd=w4, od=o96) == 1                                       # ... and the 1x1 skip kernel is required
    w4.w_skip = fake + (2 << 30)
    w5 = B._ResWeights.from_buffer_copy(w4); w5.c_out = 80
    assert call(wd=w5, od=B._Tensor5(out.ptr, B.SI_BF16, 2, 80, 8, 6, 6)) == 2   # c_out not a multiple of 32
    assert lib.si_resblock_workspace_bytes(C.byref(x), C.byref(w4), 1) > lib.si_resblock_workspace_bytes(C.byref(x), C.byref(w), 1)
    # live bytes follow the window: 8 frames in windows of 1 run two at a time and still stay within a quarter
    x = B._Tensor5(fake, B.SI_BF16, 2, 64, 8, 48, 48)     # large enough that the fixed few KB do not matter
    live1 = lib.si_resblock_live_activation_bytes(C.byref(x), C.byref(w), 1)
    live8 = lib.si_resblock_live_activation_bytes(C.byref(x), C.byref(w), 8)
    assert 0 < live1 < live8 and live1 / live8 < 0.27
    assert lib.si_resblock_live_activation_bytes(C.byref(x), C.byref(w), 100) == live8


def test_resample_validation():
    lib = si.lib()
    fake = 0x10000
    x = B._Tensor5(fake, B.SI_BF16, 2, 64, 4, 7, 10)
    down = B._Tensor5(fake + (1 << 30), B.SI_BF16, 2, 64, 4, 4, 5)
    up = B._Tensor5(fake + (1 << 30), B.SI_BF16, 2, 64, 4, 14, 20)

    def call(kind, od, xd=x, w=fake + (2 << 30), slice_len=1, ws_bytes=1 << 40):
        return lib.si_resample_forward(C.byref(xd), kind, w, None, C.byref(od), slice_len, 0x7000000000, ws_bytes, None)

    assert lib.si_resample_workspace_bytes(C.byref(x), B.SI_RESAMPLE_DOWN, 1) > 0
    assert lib.si_resample_workspace_bytes(C.byref(x), 5, 1) == 0
    assert call(B.SI_RESAMPLE_DOWN, up) == 2 and call(B.SI_RESAMPLE_UP, down) == 2      # output map must match the kind
    assert call(7, down) == 7
    assert call(B.SI_RESAMPLE_DOWN, down, w=None) == 1
    assert call(B.SI_RESAMPLE_DOWN, down, slice_len=0) == 4
    assert call(B.SI_RESAMPLE_UP, up, ws_bytes=1024) == 6
    assert call(B.SI_RESAMPLE_UP, up, xd=B._Tensor5(fake, B.SI_F32, 2, 64, 4, 7, 10)) == 3
    assert call(B.SI_RESAMPLE_UP, up, xd=B._Tensor5(fake, B.SI_BF16, 2, 48, 4, 7, 10)) == 2
    assert call(B.SI_RESAMPLE_DOWN, B._Tensor5(x.ptr + 256, B.SI_BF16, 2, 64, 4, 4, 5)) == 7   # out overlaps x


def test_forward_ex_flags():
    x, w, _, out = _descs()
    lib = si.lib()
    args = (C.byref(x), C.byref(w), None, C.byref(out), B.SI_AXIS_HW, 4, 0x7000000000, 1 << 40)
    assert lib.si_block_forward_ex(*args, 2, None) == 7                    # unknown flag bit
    assert lib.si_block_forward_ex(*args[:5], 0, *args[6:], B.SI_FWD_WEIGHTS_PACKED, None) == 4   # the forward's checks still apply


def test_workspace_scales_with_the_slice():
    x, w, _, _ = _descs(Cn=320, heads=8, dh=40, groups=32, F=16, H=64, W=64)
    lib = si.lib()
    full = lib.si_live_activation_bytes(C.byref(x), C.byref(w), None, B.SI_AXIS_HW, 4096)
    quarter = lib.si_live_activation_bytes(C.byref(x), C.byref(w), None, B.SI_AXIS_HW, 1024)
    # a quarter of the window intermediates plus the slice-independent GroupNorm statistics (8 KiB here)
    assert 0 < quarter < full and quarter / full < 0.2501
    assert lib.si_workspace_bytes(C.byref(x), C.byref(w), None, B.SI_AXIS_HW, 1024) > quarter
    # slice_len beyond the extent behaves as unsliced
    assert lib.si_live_activation_bytes(C.byref(x), C.byref(w), None, B.SI_AXIS_HW, 10**9) == full


def test_live_bytes_of_the_five_configurations():
    """Sliced / unsliced live activation bytes at each configuration's default slicing: the window
    intermediates in flight never exceed a quarter of the unsliced run's; the slice-independent items
    (GroupNorm statistics, context keys / values) come on top, which shows where the plan sits
    exactly at a quarter (4 slices one at a time, 8 slices two at a time)."""
    import si_workloads as wl
    lib = si.lib()
    bound = {"cfg1": 0.26, "cfg2": 0.2501, "cfg3": 0.19, "cfg4s": 0.121, "cfg4t": 0.2501, "cfg5s": 0.256, "cfg5t": 0.2501}
    for name, spec in wl.CONFIGS.items():
        spatial = spec.kind == wl.SPATIAL
        dt = B.SI_F32 if spec.dtype == "f32" else B.SI_BF16
        x, w, _, _ = _descs(kind=B.SI_BLOCK_SPATIAL if spatial else B.SI_BLOCK_TEMPORAL, dtype=dt, Bn=spec.B, Cn=spec.C, F=spec.F,
                            H=spec.H, W=spec.W, heads=spec.heads, dh=spec.dim_head, groups=spec.gn_groups)
        w.add_sin_pe = int(spec.add_sin_pe)
        ctx = B._Context(0x10000 + (3 << 30), dt, spec.B, spec.ctx_tokens, spec.ctx_dim) if spatial else None
        pc = C.byref(ctx) if ctx is not None else None
        axis = B.SI_AXIS_F if spatial else B.SI_AXIS_HW
        sliced = lib.si_live_activation_bytes(C.byref(x), C.byref(w), pc, axis, spec.slice_len)
        full = lib.si_live_activation_bytes(C.byref(x), C.byref(w), pc, axis, 10**9)
        assert 0 < sliced < full, name
        assert sliced / full <= bound[name], (name, sliced / full)


def test_rehash_check_validation():
    lib = si.lib()
    fake = 0x10000
    assert lib.si_rehash_check(fake, fake, 16, 7, 0.9, None, fake, fake, None) == 3
    assert lib.si_rehash_check(fake, fake, -1, B.SI_BF16, 0.9, None, fake, fake, None) == 2
    assert lib.si_rehash_check(fake, fake, 16, B.SI_BF16, float("nan"), None, fake, fake, None) == 7
    assert lib.si_rehash_check(fake, fake, 16, B.SI_BF16, 0.9, None, None, fake, None) == 1
    assert lib.si_rehash_check(fake + 2, fake, 16, B.SI_BF16, 0.9, None, fake, fake, None) == 5
    assert si.si_rehash_scratch_bytes(0) >= 24 and si.si_rehash_scratch_bytes(1 << 30) <= 2048 * 24


@pytest.mark.parametrize("name,K,gamma,rule,G", list(_golden_cases()))
def test_key_step_search_matches_hand_worked_cases_and_oracle(name, K, gamma, rule, G):
    S = _rule_matrix(rule, K)
    assert si.si_key_step_search(S.tolist(), gamma) == G
    assert si.si_key_step_search(S.tolist(), gamma) == oracle.key_step_search_ref(S.astype(np.float32), np.float32(gamma), K)


def test_key_step_search_random_maps_and_errors():
    rng = np.random.default_rng(0)
    for K in (1, 2, 5, 10, 25):
        for _ in range(20):
            S = rng.uniform(0.8, 1.0, (K, K)).astype(np.float32)
            np.fill_diagonal(S, 1.0)
            g = float(np.float32(rng.uniform(0.85, 0.99)))
            assert si.si_key_step_search(S.tolist(), g) == oracle.key_step_search_ref(S, g, K)
    with pytest.raises(si.SiError):
        si.si_key_step_search([[1.0]], 1.5)
    with pytest.raises(si.SiError):
        si.si_key_step_search([[0.2, 0.1], [0.1, 0.2]], 0.5)     # diagonal below the threshold


def test_packed_promise_is_refused_for_a_workspace_that_was_never_packed():
    """SI_FWD_WEIGHTS_PACKED on a workspace that no re-laying-out call of this process used: the host
    can see that the promise is broken and refuses before anything is enqueued."""
    x, w, _, out = _descs()
    st = si.lib().si_block_forward_ex(C.byref(x), C.byref(w), None, C.byref(out), B.SI_AXIS_HW, 4,
                                      0x7100000000, 1 << 40, B.SI_FWD_WEIGHTS_PACKED, None)
    assert st == 7
    st = si.lib().si_block_forward_ex(C.byref(x), C.byref(w), None, C.byref(out), B.SI_AXIS_HW, 4,
                                      0x7100000000, 1 << 40, 2, None)          # unknown flag bit
    assert st == 7


def _in_flight(x, w, ctx, axis, slice_len):
    return si.lib().si_windows_in_flight(C.byref(x), C.byref(w), C.byref(ctx) if ctx is not None else None, axis, slice_len)


def test_windows_in_flight_follow_the_slice_count():
    """One window at a time for a few large slices, two from 8 slices on, three from 12 on (Sec. 4.2.2)."""
    x, w, _, _ = _descs(H=8, W=12)                                   # 96 positions
    assert _in_flight(x, w, None, B.SI_AXIS_HW, 96) == 1
    assert _in_flight(x, w, None, B.SI_AXIS_HW, 24) == 1             # 4 slices
    assert _in_flight(x, w, None, B.SI_AXIS_HW, 12) == 2             # 8 slices
    assert _in_flight(x, w, None, B.SI_AXIS_HW, 8) == 3              # 12 slices
    assert _in_flight(x, w, None, B.SI_AXIS_F, 1) == 0               # invalid: temporal block along frames
