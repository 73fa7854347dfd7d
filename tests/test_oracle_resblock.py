"""Pins for the Spatial ResBlock oracle: the convolution against brute force, a library routine and
closed-form kernels; SiLU identities; the block against an independent composition of library
operators; exact slicing invariance along frames (Eq. 1)."""
import math

import numpy as np
import pytest

import oracle
import si_workloads as wl


def _brute_conv(a, w, b):
    N, C, H, W = a.shape
    O = w.shape[0]
    out = np.zeros((N, O, H, W))
    for n in range(N):
        for o in range(O):
            for y in range(H):
                for x in range(W):
                    s = b[o]
                    for c in range(C):
                        for i in range(3):
                            for j in range(3):
                                yy, xx = y + i - 1, x + j - 1
                                if 0 <= yy < H and 0 <= xx < W:
                                    s += w[o, c, i, j] * a[n, c, yy, xx]
                    out[n, o, y, x] = s
    return out


def test_conv_matches_brute_force():
    rng = np.random.default_rng(0)
    a = rng.standard_normal((2, 3, 5, 4)); w = rng.standard_normal((4, 3, 3, 3)); b = rng.standard_normal(4)
    assert np.allclose(oracle.conv3x3_ref(a, w, b), _brute_conv(a, w, b), atol=1e-13)


def test_conv_matches_library_correlation():
    from scipy.signal import correlate2d
    rng = np.random.default_rng(1)
    a = rng.standard_normal((1, 2, 7, 9)); w = rng.standard_normal((3, 2, 3, 3))
    got = oracle.conv3x3_ref(a, w)
    for o in range(3):
        want = sum(correlate2d(a[0, c], w[o, c], mode="same", boundary="fill", fillvalue=0.0) for c in range(2))
        assert np.allclose(got[0, o], want, atol=1e-13)


def test_conv_closed_form_kernels():
    rng = np.random.default_rng(2)
    a = rng.standard_normal((2, 4, 6, 5))
    eye = np.zeros((4, 4, 3, 3))
    eye[np.arange(4), np.arange(4), 1, 1] = 1.0                       # centre tap, identity channel map
    assert np.array_equal(oracle.conv3x3_ref(a, eye), a)
    for i in range(3):
        for j in range(3):                                            # a single tap reads the pixel at (y+i-1, x+j-1)
            k = np.zeros((4, 4, 3, 3)); k[np.arange(4), np.arange(4), i, j] = 1.0
            want = np.zeros_like(a)
            for y in range(6):
                for x in range(5):
                    yy, xx = y + i - 1, x + j - 1
                    if 0 <= yy < 6 and 0 <= xx < 5:
                        want[:, :, y, x] = a[:, :, yy, xx]
            assert np.array_equal(oracle.conv3x3_ref(a, k), want), (i, j)
    ones = np.ones((1, 1, 4, 4)); box = np.ones((1, 1, 3, 3))         # box filter counts the neighbours inside the image
    cnt = oracle.conv3x3_ref(ones, box)[0, 0]
    assert cnt[0, 0] == 4 and cnt[0, 1] == 6 and cnt[1, 1] == 9 and cnt[3, 3] == 4
    # channel mixing is a matrix product at every pixel
    mix = np.zeros((3, 4, 3, 3)); M = rng.standard_normal((3, 4)); mix[:, :, 1, 1] = M
    assert np.allclose(oracle.conv3x3_ref(a, mix), np.einsum("oc,nchw->nohw", M, a), atol=1e-14)
    # linear in input and kernel; bias is added once per output channel
    w1, w2 = rng.standard_normal((2, 3, 4, 3, 3)); b = rng.standard_normal(3)
    assert np.allclose(oracle.conv3x3_ref(a, w1 + 2 * w2, b),
                       oracle.conv3x3_ref(a, w1) + 2 * oracle.conv3x3_ref(a, w2) + b.reshape(1, 3, 1, 1), atol=1e-12)


def test_silu_identities():
    v = np.linspace(-20, 20, 401)
    s = oracle.silu_ref(v)
    assert oracle.silu_ref(0.0) == 0.0
    assert np.allclose(s - oracle.silu_ref(-v), v, atol=1e-13)        # silu(v) - silu(-v) = v
    assert np.allclose(s, v * 0.5 * (1 + np.tanh(v / 2)), atol=1e-13)  # sigmoid(v) = (1 + tanh(v/2)) / 2
    assert oracle.silu_ref(40.0) == pytest.approx(40.0, abs=1e-12) and abs(oracle.silu_ref(-40.0)) < 1e-12
    assert oracle.silu_ref(1.0) == pytest.approx(1 / (1 + math.exp(-1.0)), abs=1e-15)
    i = np.argmin(s)                                                  # minimum -0.27846 at v = -1.27846
    assert v[i] == pytest.approx(-1.278, abs=0.06) and s[i] == pytest.approx(-0.27846, abs=1e-3)


def _spec(**kw):
    return wl.scaled(wl.RES_CONFIGS["res1"], **kw)


def test_block_matches_library_composition():
    """Same block from torch's CPU operators in float64 (group_norm, silu, conv2d, linear)."""
    import torch
    import torch.nn.functional as Fn
    spec = _spec()
    x = wl.make_x(spec).astype(np.float64)
    w = {k: v.astype(np.float64) for k, v in wl.make_res_weights(spec, randomize_affine=True).items()}
    temb = wl.make_temb(spec).astype(np.float64)
    got = oracle.resblock_forward_ref(x, w, spec, temb)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a))
    B, C, Fr, H, W = x.shape
    xf = t(x).permute(0, 2, 1, 3, 4).reshape(B * Fr, C, H, W)
    h = Fn.conv2d(Fn.silu(Fn.group_norm(xf, spec.gn_groups, t(w["gn1_g"]), t(w["gn1_b"]), spec.gn_eps)),
                  t(w["w_conv1"]), t(w["b_conv1"]), padding=1)
    e = Fn.linear(Fn.silu(t(temb)), t(w["w_temb"]).T, t(w["b_temb"]))           # [B, C]
    h = h + e.repeat_interleave(Fr, dim=0)[:, :, None, None]
    h = Fn.conv2d(Fn.silu(Fn.group_norm(h, spec.gn_groups, t(w["gn2_g"]), t(w["gn2_b"]), spec.gn_eps)),
                  t(w["w_conv2"]), t(w["b_conv2"]), padding=1)
    want = (xf + h).reshape(B, Fr, C, H, W).permute(0, 2, 1, 3, 4).numpy()
    assert np.allclose(got, want, atol=1e-11)
    # the embedding term matters and is per batch entry
    assert not np.allclose(got, oracle.resblock_forward_ref(x, w, spec, None), atol=1e-3)


def test_block_special_cases():
    spec = _spec(temb_dim=0)
    x = wl.make_x(spec).astype(np.float64)
    w = wl.make_res_weights(spec, randomize_affine=True)
    w0 = dict(w); w0["w_conv2"] = np.zeros_like(w["w_conv2"]); w0["b_conv2"] = np.zeros_like(w["b_conv2"])
    assert np.array_equal(oracle.resblock_forward_ref(x, w0, spec), x)           # dead branch: identity skip only
    wb = dict(w0); wb["b_conv2"] = np.arange(spec.C, dtype=np.float64)
    d = oracle.resblock_forward_ref(x, wb, spec) - x
    assert np.allclose(d, np.arange(spec.C).reshape(1, -1, 1, 1, 1), atol=1e-12)  # bias once per output channel
    # GroupNorm makes the branch invariant to a positive rescale and a shift of the input
    y1 = oracle.resblock_forward_ref(x, w, spec) - x
    x2 = 3.0 * x + 5.0
    y2 = oracle.resblock_forward_ref(x2, w, spec) - x2
    assert np.allclose(y1, y2, atol=1e-6)


@pytest.mark.parametrize("slice_len", [1, 2, 3, 5])
def test_slicing_along_frames_is_exact(slice_len):
    spec = _spec()
    x = wl.make_x(spec)
    w = wl.make_res_weights(spec, randomize_affine=True)
    temb = wl.make_temb(spec)
    full = oracle.resblock_forward_ref(x, w, spec, temb)
    sliced = oracle.sliced_resblock_forward_ref(x, w, spec, temb, slice_len)
    assert np.allclose(sliced, full, atol=1e-12) and not np.isnan(sliced).any()


def test_frames_are_independent_and_flop_count():
    spec = _spec(F=2)
    x = wl.make_x(spec)
    w = wl.make_res_weights(spec)
    full = oracle.resblock_forward_ref(x, w, spec, wl.make_temb(spec))
    x2 = x.copy(); x2[:, :, 1] += 1.0 + x2[:, :, 1] ** 2              # disturb frame 1 only
    again = oracle.resblock_forward_ref(x2, w, spec, wl.make_temb(spec))
    assert np.array_equal(full[:, :, 0], again[:, :, 0]) and not np.allclose(full[:, :, 1], again[:, :, 1])
    r4 = wl.RES_CONFIGS["res4"]
    assert r4.flops() == pytest.approx(2 * 2 * 2 * 25 * 9216 * 9 * 320 * 320 + 2 * 2 * 1280 * 320)


def test_resample_matches_library_operators():
    import torch
    import torch.nn.functional as Fn
    rng = np.random.default_rng(5)
    for (H, W) in [(6, 8), (7, 5), (1, 1), (2, 3)]:
        x = rng.standard_normal((2, 3, 2, H, W)); w = rng.standard_normal((4, 3, 3, 3)); b = rng.standard_normal(4)
        xf = torch.from_numpy(x).permute(0, 2, 1, 3, 4).reshape(4, 3, H, W)
        down = Fn.conv2d(xf, torch.from_numpy(w), torch.from_numpy(b), stride=2, padding=1)
        got = oracle.downsample_ref(x, w, b)
        assert got.shape == (2, 4, 2, (H + 1) // 2, (W + 1) // 2)
        assert np.allclose(got, down.reshape(2, 2, 4, *down.shape[2:]).permute(0, 2, 1, 3, 4).numpy(), atol=1e-12)
        up = Fn.conv2d(Fn.interpolate(xf, scale_factor=2, mode="nearest"), torch.from_numpy(w), torch.from_numpy(b), padding=1)
        got = oracle.upsample_ref(x, w, b)
        assert got.shape == (2, 4, 2, 2 * H, 2 * W)
        assert np.allclose(got, up.reshape(2, 2, 4, 2 * H, 2 * W).permute(0, 2, 1, 3, 4).numpy(), atol=1e-12)


def test_resample_closed_forms_and_slicing():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((1, 2, 3, 4, 6))
    eye = np.zeros((2, 2, 3, 3)); eye[np.arange(2), np.arange(2), 1, 1] = 1.0
    assert np.array_equal(oracle.downsample_ref(x, eye), x[:, :, :, ::2, ::2])             # centre tap: even pixels
    up = oracle.upsample_ref(x, eye)
    assert np.array_equal(up[:, :, :, 1::2, 0::2], x) and np.array_equal(up[:, :, :, 0::2, 1::2], x)   # each pixel four times
    right = np.zeros((2, 2, 3, 3)); right[np.arange(2), np.arange(2), 1, 2] = 1.0           # tap (0, +1)
    d = oracle.downsample_ref(x, right)
    assert np.array_equal(d, x[:, :, :, ::2, 1::2])                                         # reads pixel (2y, 2x+1)
    u = oracle.upsample_ref(x, right)
    assert np.array_equal(u[:, :, :, :, :-1], np.repeat(np.repeat(x, 2, 3), 2, 4)[:, :, :, :, 1:]) and not u[:, :, :, :, -1].any()
    box = np.ones((1, 2, 3, 3)); ones = np.ones((1, 2, 1, 4, 4))
    assert oracle.downsample_ref(ones, box)[0, 0, 0].tolist() == [[8.0, 12.0], [12.0, 18.0]]   # neighbours inside, 2 channels
    assert oracle.upsample_ref(ones, box)[0, 0, 0, 0, 0] == 8.0 and oracle.upsample_ref(ones, box)[0, 0, 0, 3, 3] == 18.0
    w = rng.standard_normal((3, 2, 3, 3)); b = rng.standard_normal(3)
    for kind, fn in (("down", oracle.downsample_ref), ("up", oracle.upsample_ref)):
        for sl in (1, 2, 3):
            assert np.array_equal(oracle.sliced_resample_ref(x, w, b, kind, sl), fn(x, w, b))


def test_block_with_channel_change_and_1x1_skip():
    import torch
    import torch.nn.functional as Fn
    spec = _spec(C_out=96)
    x = wl.make_x(spec).astype(np.float64)
    w = {k: v.astype(np.float64) for k, v in wl.make_res_weights(spec, randomize_affine=True).items()}
    assert w["w_conv1"].shape == (96, 64, 3, 3) and w["w_conv2"].shape == (96, 96, 3, 3) and w["w_skip"].shape == (96, 64)
    temb = wl.make_temb(spec).astype(np.float64)
    got = oracle.resblock_forward_ref(x, w, spec, temb)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a))
    B, C, Fr, H, W = x.shape
    xf = t(x).permute(0, 2, 1, 3, 4).reshape(B * Fr, C, H, W)
    h = Fn.conv2d(Fn.silu(Fn.group_norm(xf, spec.gn_groups, t(w["gn1_g"]), t(w["gn1_b"]), spec.gn_eps)),
                  t(w["w_conv1"]), t(w["b_conv1"]), padding=1)
    h = h + Fn.linear(Fn.silu(t(temb)), t(w["w_temb"]).T, t(w["b_temb"])).repeat_interleave(Fr, dim=0)[:, :, None, None]
    h = Fn.conv2d(Fn.silu(Fn.group_norm(h, spec.gn_groups, t(w["gn2_g"]), t(w["gn2_b"]), spec.gn_eps)),
                  t(w["w_conv2"]), t(w["b_conv2"]), padding=1)
    skip = Fn.conv2d(xf, t(w["w_skip"])[:, :, None, None], t(w["b_skip"]))
    want = (skip + h).reshape(B, Fr, 96, H, W).permute(0, 2, 1, 3, 4).numpy()
    assert got.shape == (B, 96, Fr, H, W) and np.allclose(got, want, atol=1e-11)
    # an identity 1x1 skip is the identity skip
    s2 = _spec()
    w2 = wl.make_res_weights(s2)
    a = oracle.resblock_forward_ref(x, w2, s2, None)
    w3 = dict(w2); w3["w_skip"] = np.eye(64); w3["b_skip"] = np.zeros(64)
    assert np.allclose(a, oracle.resblock_forward_ref(x, w3, s2, None), atol=1e-13)
    # slicing stays exact with the channel change
    full = oracle.resblock_forward_ref(x, w, spec, temb)
    assert np.allclose(oracle.sliced_resblock_forward_ref(x, w, spec, temb, 2), full, atol=1e-12)
