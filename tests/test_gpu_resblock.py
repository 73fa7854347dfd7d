"""si_resblock_forward (Spatial ResBlock operator group, sliced along frames) vs the float64 oracle:
element by element on small shapes that span several tiles with ragged tails, and on sampled frames
of the full-size workloads in the launch configuration the benchmark times."""
import numpy as np
import pytest

import oracle
import si_workloads as wl

pytestmark = pytest.mark.gpu

BF16_MAX_ABS, BF16_REL_L2 = 2e-2, 5e-3


def _check(name, got, ref, x):
    from gpu_helpers import errors
    if x.shape != ref.shape:        # channel change: no identity residual to take out, the whole output is "branch"
        x = np.zeros_like(ref)
    e = errors(got, ref, x)
    print(name, e)
    assert np.all(np.isfinite(got))
    assert e["max_abs"] <= BF16_MAX_ABS, e
    assert e["rel_l2"] <= BF16_REL_L2, e
    assert e["rel_l2_branch"] <= 2e-2, e


@pytest.mark.parametrize("kw,slice_len", [
    (dict(), 2),                                        # 3 frames in windows of 2: ragged last window
    (dict(), 1),
    (dict(), 3),                                        # unsliced
    (dict(C=96, H=7, W=9, temb_dim=0), 1),              # C not a multiple of 64, odd map, no embedding term
    (dict(C=128, F=9, H=16, W=8), 1),                   # nine windows: two in flight at a time
    (dict(C=64, F=2, H=33, W=5), 1),                    # narrow map: every row of pixels touches both side borders
    (dict(B=1, C=32, F=1, H=1, W=1, temb_dim=8), 1),    # a single pixel: only the centre tap is inside
    (dict(B=3, C=64, F=4, H=3, W=40), 3),
    (dict(C=96, F=2, H=8, W=8), 1),                     # 64 pixels: the intermediate stays in fragment order
    (dict(C=160, F=3, H=4, W=16, temb_dim=0), 2),
    (dict(C=64, C_out=96, F=3), 2),                     # channel change: 1x1 skip convolution, token-major intermediate
    (dict(C=96, C_out=32, F=2, H=8, W=8), 1),           # fewer output channels, fragment-order intermediate
    (dict(C=64, C_out=160, F=9, H=4, W=8, temb_dim=0), 1),
])
def test_small_shapes_elementwise(kw, slice_len):
    from gpu_helpers import run_resblock
    spec = wl.scaled(wl.RES_CONFIGS["res1"], **kw)
    x = wl.make_x(spec)
    w = wl.make_res_weights(spec, randomize_affine=True, kernel_std=0.03)   # 1.5 x the workloads' kernel scale
    temb = wl.make_temb(spec)
    got = run_resblock(spec, x, w, temb, slice_len)
    ref = oracle.resblock_forward_ref(x, w, spec, temb)
    _check(f"res1 {kw} slice {slice_len}", got, ref, x)


def test_sliced_equals_unsliced_on_device():
    """Eq. 1 on the device: the same kernels on every window, so any slicing gives the same bits."""
    from gpu_helpers import run_resblock
    spec = wl.scaled(wl.RES_CONFIGS["res1"], F=9, C=64)
    x, w, temb = wl.make_x(spec), wl.make_res_weights(spec, randomize_affine=True), wl.make_temb(spec)
    full = run_resblock(spec, x, w, temb, 9)
    for sl in (1, 2, 4):
        assert np.array_equal(run_resblock(spec, x, w, temb, sl), full)


def test_large_mean_input():
    from gpu_helpers import run_resblock
    spec = wl.RES_CONFIGS["res1"]
    x = wl.make_x(spec, mean=30.0)
    w, temb = wl.make_res_weights(spec), wl.make_temb(spec)
    got = run_resblock(spec, x, w, temb)
    ref = oracle.resblock_forward_ref(x, w, spec, temb)
    d = got - ref
    # |out| ~ 30: the final bf16 rounding alone is up to 0.125; the branch is what is checked
    assert np.linalg.norm(d) / np.linalg.norm(ref) <= BF16_REL_L2
    assert np.max(np.abs(d)) <= 0.13


def _sampled_frames(spec, frames):
    from gpu_helpers import run_resblock
    x, w, temb = wl.make_x(spec), wl.make_res_weights(spec), wl.make_temb(spec)
    out = run_resblock(spec, x, w, temb)
    assert np.all(np.isfinite(out))
    got, ref, xs = [], [], []
    for f in frames:                                    # a frame's output depends on that frame only
        xf = x[:, :, f:f + 1]
        ref.append(oracle.resblock_forward_ref(xf, w, spec, temb))
        got.append(out[:, :, f:f + 1])
        xs.append(xf)
    return np.concatenate(got, 2), np.concatenate(ref, 2), np.concatenate(xs, 2)


def test_res4_svdxt_shape_sampled_frames():
    _check("res4", *_sampled_frames(wl.RES_CONFIGS["res4"], frames=[0, 24]))


def test_res4c_level_transition_sampled_frame():
    _check("res4c", *_sampled_frames(wl.RES_CONFIGS["res4c"], frames=[24]))     # 320 -> 640 channels, ragged last window


def test_res4b_deeper_level_sampled_frames():
    _check("res4b", *_sampled_frames(wl.RES_CONFIGS["res4b"], frames=[1, 24]))   # 24: the ragged last window


def test_live_bytes_bounded_by_one_slice():
    import paper_2411_01171_amd as si
    from gpu_helpers import device_res_weights, to_dev
    spec = wl.RES_CONFIGS["res4"]
    x = to_dev(np.zeros((spec.B, spec.C, spec.F, spec.H, spec.W), np.float32), "bf16")
    wd = device_res_weights(spec, wl.make_res_weights(spec))
    sliced = si.si_resblock_live_activation_bytes(x, wd, spec.slice_len)
    unsliced = si.si_resblock_live_activation_bytes(x, wd, spec.F)
    assert 0 < sliced <= unsliced / 4
