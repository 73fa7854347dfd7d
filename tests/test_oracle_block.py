"""Pins for the block oracle: closed forms, invariants, scalar brute force.

None of these re-type the oracle's own formulas with the same library calls:
the brute force is a scalar pure-Python evaluation with explicit indices, the
rest are identities that hold for the mathematical definition.
"""
import math

import numpy as np
import pytest

import oracle
import si_workloads as wl
from helpers import random_block, rel_l2, tiny_spec


# ----------------------------------------------------------------- scalar brute force
def _bf_layer_norm(row, g, b, eps):
    n = len(row)
    mu = sum(row) / n
    var = sum((v - mu) ** 2 for v in row) / n
    return [(row[i] - mu) / math.sqrt(var + eps) * g[i] + b[i] for i in range(n)]


def _bf_matvec(row, Wm, bias=None):
    n_in, n_out = len(Wm), len(Wm[0])
    assert len(row) == n_in
    out = []
    for o in range(n_out):
        s = 0.0 if bias is None else bias[o]
        for i in range(n_in):
            s += row[i] * Wm[i][o]
        out.append(s)
    return out


def _bf_attention(qs, ks, vs, heads):
    D = len(qs[0])
    d = D // heads
    outs = [[0.0] * D for _ in qs]
    for hd in range(heads):
        lo = hd * d
        for iq, q in enumerate(qs):
            sc = [sum(q[lo + c] * k[lo + c] for c in range(d)) / math.sqrt(d) for k in ks]
            m = max(sc)
            e = [math.exp(s - m) for s in sc]
            z = sum(e)
            for c in range(d):
                outs[iq][lo + c] = sum(e[j] / z * vs[j][lo + c] for j in range(len(ks)))
    return outs


def brute_force_block(x, w, spec, ctx):
    """Scalar evaluation of the block definition with explicit indices."""
    x = x.astype(np.float64)
    B, C, F, H, W = x.shape
    P = H * W
    G = spec.gn_groups
    n = C // G
    wl_ = {k: v.astype(np.float64).tolist() for k, v in w.items()}
    # GroupNorm per (b, f, g)
    xh = np.zeros_like(x)
    for b in range(B):
        for f in range(F):
            for g in range(G):
                vals = [x[b, c, f, i, j] for c in range(g * n, (g + 1) * n)
                        for i in range(H) for j in range(W)]
                mu = sum(vals) / len(vals)
                var = sum((v - mu) ** 2 for v in vals) / len(vals)
                for c in range(g * n, (g + 1) * n):
                    for i in range(H):
                        for j in range(W):
                            xh[b, c, f, i, j] = ((x[b, c, f, i, j] - mu) / math.sqrt(var + spec.gn_eps)
                                                 * wl_["gn_g"][c] + wl_["gn_b"][c])
    D = spec.D
    out = np.zeros_like(x)
    if spec.kind == wl.TEMPORAL:
        seqs = [[(b, f, p) for f in range(F)] for b in range(B) for p in range(P)]
    else:
        seqs = [[(b, f, p) for p in range(P)] for b in range(B) for f in range(F)]
    for seq in seqs:
        hs = []
        for (b, f, p) in seq:
            tok = [xh[b, c, f, p // W, p % W] for c in range(C)]
            hs.append(_bf_matvec(tok, wl_["w_in"], wl_["b_in"]))
        a = [_bf_layer_norm(h, wl_["ln1_g"], wl_["ln1_b"], spec.ln_eps) for h in hs]
        if spec.kind == wl.TEMPORAL and spec.add_sin_pe:
            for r, (b, f, p) in enumerate(seq):
                for i in range(D):
                    ang = f / (10000.0 ** ((i - i % 2) / D))
                    a[r][i] += math.sin(ang) if i % 2 == 0 else math.cos(ang)
        q = [_bf_matvec(r, wl_["wq"]) for r in a]
        k = [_bf_matvec(r, wl_["wk"]) for r in a]
        v = [_bf_matvec(r, wl_["wv"]) for r in a]
        o = _bf_attention(q, k, v, spec.heads)
        for r in range(len(seq)):
            upd = _bf_matvec(o[r], wl_["wo"], wl_["bo"])
            hs[r] = [hs[r][i] + upd[i] for i in range(D)]
        if spec.kind == wl.SPATIAL:
            b0 = seq[0][0]
            cb = ctx[b0].astype(np.float64).tolist()
            a = [_bf_layer_norm(h, wl_["ln2_g"], wl_["ln2_b"], spec.ln_eps) for h in hs]
            q = [_bf_matvec(r, wl_["wq2"]) for r in a]
            k = [_bf_matvec(r, wl_["wk2"]) for r in cb]
            v = [_bf_matvec(r, wl_["wv2"]) for r in cb]
            o = _bf_attention(q, k, v, spec.heads)
            for r in range(len(seq)):
                upd = _bf_matvec(o[r], wl_["wo2"], wl_["bo2"])
                hs[r] = [hs[r][i] + upd[i] for i in range(D)]
        a = [_bf_layer_norm(h, wl_["ln3_g"], wl_["ln3_b"], spec.ln_eps) for h in hs]
        for r, (b, f, p) in enumerate(seq):
            u = _bf_matvec(a[r], wl_["w1"], wl_["b1"])
            inner = len(u) // 2
            g = [u[i] * (0.5 * u[inner + i] * (1.0 + math.erf(u[inner + i] / math.sqrt(2.0))))
                 for i in range(inner)]
            upd = _bf_matvec(g, wl_["w2"], wl_["b2"])
            hrow = [hs[r][i] + upd[i] for i in range(D)]
            y = _bf_matvec(hrow, wl_["w_out"], wl_["b_out"])
            for c in range(C):
                out[b, c, f, p // W, p % W] = x[b, c, f, p // W, p % W] + y[c]
    return out


@pytest.mark.parametrize("kind,pe", [(wl.TEMPORAL, False), (wl.TEMPORAL, True), (wl.SPATIAL, False)])
def test_block_matches_scalar_brute_force(kind, pe):
    # C != D so that a transposed w_in / w_out cannot pass
    spec = tiny_spec(kind, B=2, C=6, F=3, H=2, W=3, heads=2, dim_head=4, groups=3, pe=pe)
    x, w, ctx = random_block(spec)
    ref = oracle.block_forward_ref(x, w, spec, ctx)
    bf = brute_force_block(x, w, spec, ctx)
    assert np.max(np.abs(ref - bf)) < 1e-11


def test_cfg1_matches_einsum_formulation():
    """Config-1 shape, evaluated with a differently organised float64 path
    (einsum over explicit index labels on the 5-D tensor, no token reshape)."""
    spec = wl.CONFIGS["cfg1"]
    x = wl.make_x(spec)
    w = wl.make_weights(spec, randomize_affine=True)
    ref = oracle.block_forward_ref(x, w, spec)
    W = {k: v.astype(np.float64) for k, v in w.items()}
    x64 = x.astype(np.float64)
    B, C, F, H, Wd = x64.shape
    n = C // spec.gn_groups
    xh = np.empty_like(x64)
    for g in range(spec.gn_groups):
        blk = x64[:, g * n:(g + 1) * n]
        mu = np.einsum("bcfhw->bf", blk) / (n * H * Wd)
        ce = blk - mu[:, None, :, None, None]
        var = np.einsum("bcfhw,bcfhw->bf", ce, ce) / (n * H * Wd)
        xh[:, g * n:(g + 1) * n] = ce / np.sqrt(var + spec.gn_eps)[:, None, :, None, None]
    xh = xh * W["gn_g"][None, :, None, None, None] + W["gn_b"][None, :, None, None, None]

    def ln(t, g, b):  # channel axis is 1 here
        mu = np.einsum("bcfhw->bfhw", t)[:, None] / t.shape[1]
        ce = t - mu
        var = np.einsum("bcfhw,bcfhw->bfhw", ce, ce)[:, None] / t.shape[1]
        return ce / np.sqrt(var + spec.ln_eps) * g[None, :, None, None, None] + b[None, :, None, None, None]

    def lin(t, Wm, b=None):
        y = np.einsum("bcfhw,cd->bdfhw", t, Wm)
        return y if b is None else y + b[None, :, None, None, None]

    h = lin(xh, W["w_in"], W["b_in"])
    a = ln(h, W["ln1_g"], W["ln1_b"])
    q, k, v = lin(a, W["wq"]), lin(a, W["wk"]), lin(a, W["wv"])
    d = spec.dim_head
    o = np.empty_like(q)
    for hd in range(spec.heads):
        cs = slice(hd * d, (hd + 1) * d)
        s = np.einsum("bcfhw,bcghw->bhwfg", q[:, cs], k[:, cs]) / math.sqrt(d)
        s = np.exp(s - s.max(-1, keepdims=True))
        s /= s.sum(-1, keepdims=True)
        o[:, cs] = np.einsum("bhwfg,bcghw->bcfhw", s, v[:, cs])
    h = h + lin(o, W["wo"], W["bo"])
    a = ln(h, W["ln3_g"], W["ln3_b"])
    u = lin(a, W["w1"], W["b1"])
    inner = u.shape[1] // 2
    from scipy.stats import norm
    gate = u[:, inner:] * norm.cdf(u[:, inner:])      # GELU(u) = u * Phi(u)
    h = h + lin(u[:, :inner] * gate, W["w2"], W["b2"])
    out = x64 + lin(h, W["w_out"], W["b_out"])
    assert rel_l2(ref, out) < 1e-13


# ----------------------------------------------------------------- operator identities
def test_group_norm_properties():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((2, 8, 3, 4, 5)) * 3.0 + 1.5
    ones, zeros = np.ones(8), np.zeros(8)
    eps = 1e-6
    y = oracle.group_norm_ref(x, 4, eps, ones, zeros)
    yg = y.reshape(2, 4, 2, 3, 4, 5)
    xg = x.reshape(2, 4, 2, 3, 4, 5)
    assert np.allclose(yg.mean(axis=(2, 4, 5)), 0.0, atol=1e-12)
    var = xg.var(axis=(2, 4, 5))
    assert np.allclose(yg.var(axis=(2, 4, 5)), var / (var + eps), rtol=1e-12)
    # per-frame statistics: changing frame 1 must not change frames 0 and 2
    x2 = x.copy()
    x2[:, :, 1] += rng.standard_normal((2, 8, 4, 5))
    y2 = oracle.group_norm_ref(x2, 4, eps, ones, zeros)
    assert np.array_equal(y2[:, :, 0], y[:, :, 0]) and np.array_equal(y2[:, :, 2], y[:, :, 2])
    assert not np.allclose(y2[:, :, 1], y[:, :, 1])
    # shift invariance, constant input -> beta, affine
    assert np.allclose(oracle.group_norm_ref(x + 7.0, 4, eps, ones, zeros), y, atol=1e-9)
    beta = np.arange(8.0)
    assert np.allclose(oracle.group_norm_ref(np.full_like(x, 2.5), 4, eps, ones * 3, beta),
                       beta.reshape(1, 8, 1, 1, 1))
    gam = rng.standard_normal(8)
    assert np.allclose(oracle.group_norm_ref(x, 4, eps, gam, beta),
                       y * gam.reshape(1, 8, 1, 1, 1) + beta.reshape(1, 8, 1, 1, 1))


def test_layer_norm_properties():
    rng = np.random.default_rng(1)
    h = rng.standard_normal((5, 7, 16)) * 2 + 3
    y = oracle.layer_norm_ref(h, np.ones(16), np.zeros(16), 1e-5)
    assert np.allclose(y.mean(-1), 0, atol=1e-12)
    assert np.allclose(y.var(-1), h.var(-1) / (h.var(-1) + 1e-5))
    assert np.allclose(oracle.layer_norm_ref(h + 11.0, np.ones(16), np.zeros(16), 1e-5), y, atol=1e-9)
    # scale invariance up to eps
    y10 = oracle.layer_norm_ref(h * 10, np.ones(16), np.zeros(16), 0.0)
    y1 = oracle.layer_norm_ref(h, np.ones(16), np.zeros(16), 0.0)
    assert np.allclose(y10, y1)


def test_sinusoidal_pe_values():
    pe = oracle.sinusoidal_pe_ref(9, 12)
    assert np.allclose(pe[0, 0::2], 0.0) and np.allclose(pe[0, 1::2], 1.0)
    assert np.allclose(pe[:, 0::2] ** 2 + pe[:, 1::2] ** 2, 1.0)
    assert pe[1, 0] == pytest.approx(math.sin(1.0)) and pe[1, 1] == pytest.approx(math.cos(1.0))
    assert pe[5, 6] == pytest.approx(math.sin(5.0 / 10000.0 ** 0.5))
    assert pe[5, 7] == pytest.approx(math.cos(5.0 / 10000.0 ** 0.5))
    assert pe[3, 10] == pytest.approx(math.sin(3.0 / 10000.0 ** (10.0 / 12.0)))


def test_gelu_known_values():
    # GELU(u) = u * Phi(u); Phi(1) = 0.841344746068543, Phi(2) = 0.977249868051821
    assert oracle.gelu_erf_ref(0.0) == 0.0
    assert oracle.gelu_erf_ref(1.0) == pytest.approx(0.841344746068543, abs=1e-14)
    assert oracle.gelu_erf_ref(-1.0) == pytest.approx(-0.158655253931457, abs=1e-14)
    assert oracle.gelu_erf_ref(2.0) == pytest.approx(2 * 0.977249868051821, abs=1e-13)
    assert oracle.gelu_erf_ref(40.0) == pytest.approx(40.0)
    assert abs(oracle.gelu_erf_ref(-40.0)) < 1e-300
    u = np.linspace(-3, 3, 13)
    assert np.allclose(oracle.gelu_erf_ref(u), [0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in u])


def test_attention_closed_forms():
    rng = np.random.default_rng(2)
    q = rng.standard_normal((3, 5, 8))
    k = rng.standard_normal((3, 7, 8))
    v = rng.standard_normal((3, 7, 8))
    # uniform keys -> mean of values
    o = oracle.attention_ref(q, np.zeros_like(k), v, heads=2)
    assert np.allclose(o, np.broadcast_to(v.mean(1, keepdims=True), o.shape))
    # a single key -> its value for every query
    o = oracle.attention_ref(q, k[:, :1], v[:, :1], heads=2)
    assert np.allclose(o, np.broadcast_to(v[:, :1], o.shape))
    # dominant key per head -> value of the arg-max key, head by head
    kk = rng.standard_normal((1, 6, 8))
    qq = 200.0 * kk[:, [4, 1, 1]]
    o = oracle.attention_ref(qq, kk, v[:1, :6], heads=2)
    for hd in range(2):
        cs = slice(hd * 4, hd * 4 + 4)
        best = np.argmax(qq[0, :, cs] @ kk[0, :, cs].T, axis=1)
        assert np.allclose(o[0, :, cs], v[0, best, cs], atol=1e-9)
    # permuting keys together with values changes nothing; scale is 1/sqrt(d)
    perm = rng.permutation(7)
    assert np.allclose(oracle.attention_ref(q, k[:, perm], v[:, perm], 2), oracle.attention_ref(q, k, v, 2))
    s = q[0, :, :8] @ k[0].T / math.sqrt(8)
    p = np.exp(s) / np.exp(s).sum(1, keepdims=True)
    assert np.allclose(oracle.attention_ref(q[:1], k[:1], v[:1], 1)[0], p @ v[0])
    assert np.allclose(oracle.softmax_rows_ref(s).sum(-1), 1.0)


# ----------------------------------------------------------------- block-level identities
def test_zero_matrices_give_x_plus_bias():
    spec = tiny_spec(wl.SPATIAL, C=8, heads=2, dim_head=4)
    x, w, ctx = random_block(spec)
    for name, arr in w.items():
        if arr.ndim == 2:
            w[name] = np.zeros_like(arr)
    out = oracle.block_forward_ref(x, w, spec, ctx)
    assert np.allclose(out, x.astype(np.float64) + w["b_out"].reshape(1, -1, 1, 1, 1).astype(np.float64))


def test_zero_gate_ffn_contributes_only_b2():
    spec = tiny_spec(wl.TEMPORAL)
    x, w, _ = random_block(spec)
    D = spec.D
    w0 = dict(w)
    w0["w1"] = w["w1"].copy(); w0["w1"][:, 4 * D:] = 0      # gate pre-activation = b1 gate half
    w0["b1"] = w["b1"].copy(); w0["b1"][4 * D:] = 0         # gate = GELU(0) = 0
    a = oracle.block_forward_ref(x, w0, spec)
    w1 = dict(w0)
    w1["w2"] = np.zeros_like(w["w2"])                        # FFN = b2 only
    b = oracle.block_forward_ref(x, w1, spec)
    assert np.allclose(a, b, atol=1e-13)


def test_uniform_keys_block_is_mean_of_values():
    """W_k = 0: self-attention output = mean over the sequence of v."""
    spec = tiny_spec(wl.TEMPORAL, F=4, pe=True)
    x, w, _ = random_block(spec)
    w["wk"] = np.zeros_like(w["wk"])
    ref = oracle.block_forward_ref(x, w, spec)
    # same block, but with the attention replaced by its closed form
    W = {k: v.astype(np.float64) for k, v in w.items()}
    xh = oracle.group_norm_ref(x, spec.gn_groups, spec.gn_eps, w["gn_g"], w["gn_b"])
    t = oracle.tokens_from_feature_ref(xh, spec.kind)
    h = t @ W["w_in"] + W["b_in"]
    a = oracle.layer_norm_ref(h, W["ln1_g"], W["ln1_b"], spec.ln_eps) + oracle.sinusoidal_pe_ref(4, spec.D)[None]
    vmean = (a @ W["wv"]).mean(axis=1, keepdims=True)
    h = h + np.broadcast_to(vmean, h.shape) @ W["wo"] + W["bo"]
    a = oracle.layer_norm_ref(h, W["ln3_g"], W["ln3_b"], spec.ln_eps)
    u = a @ W["w1"] + W["b1"]
    g = u[..., :4 * spec.D] * oracle.gelu_erf_ref(u[..., 4 * spec.D:])
    h = h + g @ W["w2"] + W["b2"]
    out = x + oracle.feature_from_tokens_ref(h @ W["w_out"] + W["b_out"], spec.kind, x.shape)
    assert np.allclose(ref, out, atol=1e-12)


def test_single_context_token_cross_attention_closed_form():
    """M = 1: cross-attention adds ctx W_v2 W_o2 + b_o2 to every token, whatever q is."""
    spec = tiny_spec(wl.SPATIAL, M=1, Cc=6)
    x, w, ctx = random_block(spec)
    ref = oracle.block_forward_ref(x, w, spec, ctx)
    w2 = dict(w)
    w2["wq2"] = w["wq2"] * 5.0 + 1.0               # q must not matter
    assert np.allclose(oracle.block_forward_ref(x, w2, spec, ctx), ref, atol=1e-12)
    # replace cross-attention by the closed form through a bias-only path
    W = {k: v.astype(np.float64) for k, v in w.items()}
    add = ctx.astype(np.float64)[:, 0] @ W["wv2"] @ W["wo2"] + W["bo2"]      # [B, D]
    outs = []
    for b in range(spec.B):
        wb = dict(w)
        wb["wv2"] = np.zeros_like(w["wv2"])
        wb["bo2"] = add[b]
        outs.append(oracle.block_forward_ref(x[b:b + 1], wb, spec, ctx[b:b + 1]))
    assert np.allclose(np.concatenate(outs), ref, atol=1e-12)


# ----------------------------------------------------------------- slicing (Sec. 4.1, Eq. 1)
def test_slice_windows_ceil_rule():
    assert list(oracle.slice_windows_ref(10, 4)) == [(0, 4), (4, 8), (8, 10)]
    assert list(oracle.slice_windows_ref(8, 4)) == [(0, 4), (4, 8)]
    assert list(oracle.slice_windows_ref(3, 7)) == [(0, 3)]
    # k sub-features of ceil(n/k): n=50 (B*T), k=4 -> 13,13,13,11
    n, k = 50, 4
    ln = -(-n // k)
    assert [b - a for a, b in oracle.slice_windows_ref(n, ln)] == [13, 13, 13, 11]


@pytest.mark.parametrize("slice_len", [1, 2, 4, 5, 6, 100])
def test_temporal_position_slicing_is_lossless(slice_len):
    spec = tiny_spec(wl.TEMPORAL, H=2, W=3, pe=True)
    x, w, _ = random_block(spec)
    ref = oracle.block_forward_ref(x, w, spec)
    out = oracle.sliced_block_forward_ref(x, w, spec, None, "HW", slice_len)
    assert np.max(np.abs(out - ref)) < 1e-12


@pytest.mark.parametrize("slice_len", [1, 2, 3, 5])
def test_spatial_frame_slicing_is_lossless(slice_len):
    spec = tiny_spec(wl.SPATIAL, F=5)
    x, w, ctx = random_block(spec)
    ref = oracle.block_forward_ref(x, w, spec, ctx)
    for local in (False, True):      # per-frame statistics: slice-local stats are exact too
        out = oracle.sliced_block_forward_ref(x, w, spec, ctx, "F", slice_len, local_stats=local)
        assert np.max(np.abs(out - ref)) < 1e-12


def test_lossy_slicings_do_change_the_result():
    """Slicing a temporal block along frames, or taking GroupNorm statistics
    from a position slice, is not lossless -- guards the invariance tests."""
    spec = tiny_spec(wl.TEMPORAL, F=4, H=2, W=3)
    x, w, _ = random_block(spec)
    ref = oracle.block_forward_ref(x, w, spec)
    a = oracle.sliced_block_forward_ref(x, w, spec, None, "F", 2)
    assert np.max(np.abs(a - ref)) > 1e-3
    b = oracle.sliced_block_forward_ref(x, w, spec, None, "HW", 2, local_stats=True)
    assert np.max(np.abs(b - ref)) > 1e-3


def test_permutation_equivariance():
    rng = np.random.default_rng(5)
    # temporal block: permuting positions permutes the output
    spec = tiny_spec(wl.TEMPORAL, H=2, W=3, pe=True)
    x, w, _ = random_block(spec)
    ref = oracle.block_forward_ref(x, w, spec)
    perm = rng.permutation(6)
    xp = x.reshape(1, 8, 3, 6)[..., perm].reshape(x.shape)
    outp = oracle.block_forward_ref(xp, w, spec)
    assert np.allclose(outp.reshape(1, 8, 3, 6), ref.reshape(1, 8, 3, 6)[..., perm], atol=1e-12)
    # ... but permuting frames does not (frame embedding + it is the sequence axis of nothing else)
    spec_s = tiny_spec(wl.SPATIAL, F=4)
    x, w, ctx = random_block(spec_s)
    ref = oracle.block_forward_ref(x, w, spec_s, ctx)
    fperm = np.array([2, 0, 3, 1])
    assert np.allclose(oracle.block_forward_ref(x[:, :, fperm], w, spec_s, ctx), ref[:, :, fperm], atol=1e-12)
    # spatial block: permuting positions inside a frame permutes the output (no positional term)
    pperm = rng.permutation(4)
    xp = x.reshape(1, 8, 4, 4)[..., pperm].reshape(x.shape)
    outp = oracle.block_forward_ref(xp, w, spec_s, ctx)
    assert np.allclose(outp.reshape(1, 8, 4, 4), ref.reshape(1, 8, 4, 4)[..., pperm], atol=1e-12)


def test_frame_embedding_matters_only_when_enabled():
    spec = tiny_spec(wl.TEMPORAL, F=4, pe=False)
    x, w, _ = random_block(spec)
    a = oracle.block_forward_ref(x, w, spec)
    b = oracle.block_forward_ref(x, w, tiny_spec(wl.TEMPORAL, F=4, pe=True))
    assert np.max(np.abs(a - b)) > 1e-3
    # without the embedding a temporal block is equivariant to frame permutations
    fperm = np.array([3, 1, 0, 2])
    assert np.allclose(oracle.block_forward_ref(x[:, :, fperm], w, spec), a[:, :, fperm], atol=1e-12)


def test_batch_entries_are_independent_and_use_their_own_context():
    spec = tiny_spec(wl.SPATIAL, B=2)
    x, w, ctx = random_block(spec)
    ref = oracle.block_forward_ref(x, w, spec, ctx)
    for b in range(2):
        one = oracle.block_forward_ref(x[b:b + 1], w, spec, ctx[b:b + 1])
        assert np.allclose(one[0], ref[b], atol=1e-12)
    swapped = oracle.block_forward_ref(x, w, spec, ctx[::-1])
    assert np.max(np.abs(swapped - ref)) > 1e-4
