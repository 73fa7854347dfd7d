"""si_block_forward_rehash: the one-pass Step Rehash walk on the GPU vs the oracle's walk.

Decisions and cosines are checked against the float64 oracle on the identical stored inputs
(bit-exact decisions); a recomputed step must equal si_block_forward bit for bit, a reused step
must hand back the anchor's output bit for bit.  The block outputs themselves are covered by the
parity tests of the forward."""
import math

import numpy as np
import pytest

import oracle
import si_workloads as wl

pytestmark = pytest.mark.gpu


def _walk(spec, xs_np, gamma, ctx_np=None):
    import torch
    import paper_2411_01171_amd as si
    from gpu_helpers import AXIS, device_weights, to_dev

    wd = device_weights(spec, wl.make_weights(spec))
    ctx = None if ctx_np is None else to_dev(ctx_np, spec.dtype)
    xs = [to_dev(x, spec.dtype) for x in xs_np]
    axis = AXIS[spec.slice_axis]
    ws = torch.empty(si.si_workspace_bytes(xs[0], wd, ctx, axis, spec.slice_len), dtype=torch.uint8, device="cuda")
    cache = si.RehashCache(xs[0])
    assert not cache.valid
    plain = torch.empty_like(xs[0])
    got = []
    for x in xs:
        out = torch.full_like(x, float("nan"))
        reused, cos = si.si_block_forward_rehash(x, wd, ctx, out, axis, spec.slice_len, ws, cache, gamma)
        torch.cuda.synchronize()
        if not reused:                      # a computed step is the plain forward, bit for bit, and re-anchors
            si.si_block_forward(x, wd, ctx, plain, axis, spec.slice_len, ws)
            torch.cuda.synchronize()
            assert torch.equal(out, plain)
            assert torch.equal(cache.x_key, x) and torch.equal(cache.y_key, out)
        got.append((reused, cos, out))
        assert cache.valid
    return got


def test_result_in_the_anchor_buffer_copies_nothing_back():
    """out == cache.y_key: same decisions and the same bits as the copying mode, the result read from the anchor buffer."""
    import torch
    import paper_2411_01171_amd as si
    from gpu_helpers import AXIS, device_weights, to_dev
    spec = wl.scaled(wl.CONFIGS["cfg2"], H=8, W=8, slice_len=24)
    rng = np.random.default_rng(31)
    xs_np = [wl.make_x(spec)]
    for s in (0.05, 0.4, 0.0, 0.05):
        xs_np.append(wl.round_to_storage(xs_np[-1] + np.float32(s) * rng.standard_normal(xs_np[-1].shape, dtype=np.float32), "bf16"))
    wd = device_weights(spec, wl.make_weights(spec))
    xs = [to_dev(x, "bf16") for x in xs_np]
    axis = AXIS[spec.slice_axis]
    ws = torch.empty(si.si_workspace_bytes(xs[0], wd, None, axis, spec.slice_len), dtype=torch.uint8, device="cuda")
    ref = _walk(spec, xs_np, 0.95)
    cache = si.RehashCache(xs[0])
    for x, (reused_ref, cos_ref, out_ref) in zip(xs, ref):
        reused, cos = si.si_block_forward_rehash(x, wd, None, cache.y_key, axis, spec.slice_len, ws, cache, 0.95)
        torch.cuda.synchronize()
        assert reused == reused_ref and (cos == cos_ref or (math.isnan(cos) and math.isnan(cos_ref)))
        assert torch.equal(cache.y_key, out_ref)
    assert [r for r, _, _ in ref] == [False, True, False, True, True]


def _check_against_oracle(xs_np, got, gamma):
    ref = list(oracle.rehash_causal_ref(xs_np, lambda x: x, gamma))      # identity "block": only the walk matters
    anchor = None
    for (t, _, recomputed, c_ref), (reused, cos, out) in zip(ref, got):
        assert reused == (not recomputed), t
        if math.isnan(c_ref):
            assert math.isnan(cos)
        else:
            assert cos == pytest.approx(c_ref, abs=1e-12)
        if recomputed:
            anchor = out
        else:
            import torch
            assert torch.equal(out, anchor)                              # handed back bit for bit
    return [t for t, _, r, _ in ref if r]


@pytest.mark.parametrize("dtype,shape", [("bf16", dict(C=64, F=8, H=12, W=12)), ("f32", dict(C=64, F=8, H=8, W=8)),
                                         ("bf16", dict(C=64, F=4, H=5, W=7))])
def test_temporal_walk_matches_oracle(dtype, shape):
    base = wl.CONFIGS["cfg1"]
    spec = wl.scaled(base, dtype=dtype, B=2, heads=2, dim_head=32, slice_len=16, **shape)
    rng = np.random.default_rng(21)
    xs = [wl.make_x(spec)]
    for t, s in enumerate([0.05, 0.1, 0.3, 0.02, 0.0, 0.5, 0.1], start=1):
        noise = rng.standard_normal(xs[-1].shape, dtype=np.float32)
        xs.append(wl.round_to_storage(xs[-1] + np.float32(s) * noise, dtype))
    for gamma in (0.95, 0.99, -1.0, 1.0):
        rec = _check_against_oracle(xs, _walk(spec, xs, gamma), gamma)
        assert rec[0] == 0
        if gamma == -1.0:
            assert rec == [0]
        if gamma == 1.0:                                                 # only the exact repeat (sigma = 0) passes a tie
            assert 5 not in rec and len(rec) == len(xs) - 1


def test_spatial_walk_with_context_matches_oracle():
    base = wl.CONFIGS["cfg3"]
    spec = wl.scaled(base, C=64, F=3, H=8, W=8, heads=1, dim_head=64, ctx_tokens=5, ctx_dim=16, B=2)
    xs = [wl.make_x(spec)]
    rng = np.random.default_rng(22)
    for s in (0.1, 0.1, 0.4, 0.05):
        xs.append(wl.round_to_storage(xs[-1] + np.float32(s) * rng.standard_normal(xs[-1].shape, dtype=np.float32), "bf16"))
    gamma = 0.97
    rec = _check_against_oracle(xs, _walk(spec, xs, gamma, wl.make_context(spec)), gamma)
    assert 0 in rec and len(rec) < len(xs)


def test_cfg5_stack_one_pass():
    """cfg5: 4 spatial+temporal pairs over the 10-step trajectory, every block under its own anchor.
    Checked: each block's decisions equal the oracle's walk over that block's actual input sequence;
    reported: computed vs reused block evaluations and the time next to the full trajectory."""
    import time
    import torch
    import paper_2411_01171_amd as si
    from gpu_helpers import AXIS, device_weights, to_dev

    K, NP, gamma = wl.CFG5_STEPS, wl.CFG5_PAIRS, wl.CFG5_GAMMA
    sp, tp = wl.CONFIGS["cfg5s"], wl.CONFIGS["cfg5t"]
    ctx = to_dev(wl.make_context(sp), "bf16")
    blocks = []
    for p in range(NP):
        blocks.append((sp, device_weights(sp, wl.make_weights(sp, seed=sp.seed + 100 * p)), ctx))
        blocks.append((tp, device_weights(tp, wl.make_weights(tp, seed=tp.seed + 100 * p)), None))
    x_np = wl.make_x(sp)
    xs = [to_dev(x_np, "bf16")]
    for t in range(1, K):
        x_np = wl.cfg5_step_input(x_np, t)
        xs.append(to_dev(x_np, "bf16"))
    wss = [torch.empty(si.si_workspace_bytes(xs[0], w, c, AXIS[s.slice_axis], s.slice_len), dtype=torch.uint8, device="cuda")
           for s, w, c in blocks]
    bufs = [torch.empty_like(xs[0]) for _ in range(2)]

    def trajectory(use_rehash, record=None):
        caches = [si.RehashCache(xs[0]) for _ in blocks]
        reused_n = 0
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(K):
            cur = xs[t]
            for i, (s, w, c) in enumerate(blocks):
                dst = bufs[i % 2]
                if record is not None:
                    record[i].append(cur.float().cpu().numpy())
                if use_rehash:
                    r, _ = si.si_block_forward_rehash(cur, w, c, dst, AXIS[s.slice_axis], s.slice_len, wss[i], caches[i], gamma)
                    reused_n += int(r)
                    if record is not None:
                        record[i].append(bool(r))
                else:
                    si.si_block_forward(cur, w, c, dst, AXIS[s.slice_axis], s.slice_len, wss[i])
                cur = dst
        torch.cuda.synchronize()
        return time.perf_counter() - t0, reused_n

    trajectory(False)                                   # warm-up
    t_full, _ = trajectory(False)
    t_rehash, reused_n = trajectory(True)
    record = [[] for _ in blocks]
    _, reused_again = trajectory(True, record)
    assert reused_again == reused_n                     # deterministic
    for i in range(len(blocks)):
        inputs, flags = record[i][0::2], record[i][1::2]
        want = [not r for _, _, r, _ in oracle.rehash_causal_ref(inputs, lambda x: x, gamma)]
        assert flags == want, (i, flags, want)
    total = K * len(blocks)
    assert 0 < reused_n < total
    first = [not f for f in record[0][1::2]]
    assert [t for t, c in enumerate(first) if c][:2] == [0, 4]      # the schedule's prediction for the first block
    print(f"cfg5 one-pass rehash: {total - reused_n} of {total} block evaluations computed, {reused_n} handed back; "
          f"full trajectory {t_full * 1e3:.1f} ms, with rehash {t_rehash * 1e3:.1f} ms")
