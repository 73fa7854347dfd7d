"""Full-size configurations in the launch configuration the benchmark times,
checked against the oracle on sampled outputs.

A temporal block's output at position p depends on x[:, :, :, p] and on the
GroupNorm statistics of the whole frame only; a spatial block's output frame
(b, f) depends on x[b, :, f] only.  The oracle therefore evaluates sampled
positions (with GroupNorm taken over the full tensor) or sampled frames one by
one; samples straddle slice and tile boundaries and include the last element.
"""
import numpy as np
import pytest

import oracle
import si_workloads as wl

pytestmark = pytest.mark.gpu

BF16_MAX_ABS, BF16_REL_L2 = 2e-2, 5e-3


def _sample_positions(P, slice_len, n_random, seed):
    rng = np.random.default_rng(seed)
    fixed = {0, 1, 31, 32, 63, 64, 127, 128, P - 1, P - 2}
    for s in range(slice_len, P, slice_len):
        fixed.update({s - 1, s})
    fixed = {p for p in fixed if 0 <= p < P}
    if len(fixed) > 40:
        fixed = set(sorted(fixed)[:20] + sorted(fixed)[-20:])
    fixed.update(int(p) for p in rng.integers(0, P, n_random))
    return np.array(sorted(fixed))


def _temporal_sampled(spec, n_random=24):
    from gpu_helpers import run_block
    x, w = wl.make_x(spec), wl.make_weights(spec)
    out = run_block(spec, x, w, None)
    assert np.all(np.isfinite(out))
    B, C, F, H, W = x.shape
    P = H * W
    sel = _sample_positions(P, spec.slice_len, n_random, spec.seed)
    xhat = oracle.group_norm_ref(x, spec.gn_groups, spec.gn_eps, w["gn_g"], w["gn_b"]).reshape(B, C, F, 1, P)
    xs = x.reshape(B, C, F, 1, P)[..., sel]
    ref = oracle.block_forward_ref(xs, w, spec, None, xhat=xhat[..., sel])
    got = out.reshape(B, C, F, 1, P)[..., sel]
    return got, ref, xs, out


def _spatial_sampled(spec, frames):
    from gpu_helpers import run_block
    x, w, ctx = wl.make_x(spec), wl.make_weights(spec), wl.make_context(spec)
    out = run_block(spec, x, w, ctx)
    assert np.all(np.isfinite(out))
    got, ref, xs = [], [], []
    for f in frames:
        xf = x[:, :, f:f + 1]
        ref.append(oracle.block_forward_ref(xf, w, spec, ctx))
        got.append(out[:, :, f:f + 1])
        xs.append(xf)
    return np.concatenate(got, 2), np.concatenate(ref, 2), np.concatenate(xs, 2), out


def _assert_bf16(name, got, ref, xs, out):
    from gpu_helpers import errors
    e = errors(got, ref, xs)
    e["max_out_full"] = float(np.max(np.abs(out)))
    i = np.unravel_index(np.argmax(np.abs(ref)), ref.shape)
    e["err_at_argmax"] = float(abs(got[i] - ref[i]))
    print(name, e)
    assert e["max_abs"] <= BF16_MAX_ABS, e
    assert e["rel_l2"] <= BF16_REL_L2, e
    assert e["rel_l2_branch"] <= 2e-2, e


def test_cfg2_animatediff_temporal():
    _assert_bf16("cfg2", *_temporal_sampled(wl.CONFIGS["cfg2"]))


def test_cfg3_spatial():
    _assert_bf16("cfg3", *_spatial_sampled(wl.CONFIGS["cfg3"], frames=[0, 7, 15]))


@pytest.mark.parametrize("slice_len", [2, 5, 16])
def test_cfg3_spatial_other_slice_lengths(slice_len):
    """The staged path picks its GEMM tiles from the window's tokens and the windows in flight:
    2 frames per slice (two windows in flight, 64-column tiles), 5 (ragged last window of one frame)
    and the unsliced run (256-token row tiles) take other kernels than the default one-frame slices."""
    spec = wl.scaled(wl.CONFIGS["cfg3"], slice_len=slice_len)
    _assert_bf16(f"cfg3/slice{slice_len}", *_spatial_sampled(spec, frames=[0, 9, 15]))


def test_cfg4_svdxt_spatial():
    _assert_bf16("cfg4s", *_spatial_sampled(wl.CONFIGS["cfg4s"], frames=[24]))


def test_cfg4_svdxt_temporal():
    _assert_bf16("cfg4t", *_temporal_sampled(wl.CONFIGS["cfg4t"]))


def test_cfg5_spatial():
    _assert_bf16("cfg5s", *_spatial_sampled(wl.CONFIGS["cfg5s"], frames=[0, 3, 4, 15]))


def test_cfg5_temporal():
    _assert_bf16("cfg5t", *_temporal_sampled(wl.CONFIGS["cfg5t"]))


@pytest.mark.parametrize("slice_len", [1, 16])
def test_cfg5_spatial_other_slice_lengths(slice_len):
    """One frame per slice (16 windows of 512 tokens, three in flight) and the unsliced run."""
    spec = wl.scaled(wl.CONFIGS["cfg5s"], slice_len=slice_len)
    _assert_bf16(f"cfg5s/slice{slice_len}", *_spatial_sampled(spec, frames=[0, 8, 15]))


@pytest.mark.parametrize("slice_len", [24, 256])
def test_cfg5_temporal_other_slice_lengths(slice_len):
    """24 positions per slice (11 windows, the last one of 16 positions, two in flight) and unsliced."""
    spec = wl.scaled(wl.CONFIGS["cfg5t"], slice_len=slice_len)
    _assert_bf16(f"cfg5t/slice{slice_len}", *_temporal_sampled(spec))
