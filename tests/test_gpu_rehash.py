"""si_rehash_check vs the float64 oracle: cosine value and bit-exact decisions."""
import math

import numpy as np
import pytest

import oracle
import si_workloads as wl

pytestmark = pytest.mark.gpu


def _gpu_check(a, b, dtype, gamma):
    import torch
    import paper_2411_01171_amd as si
    from gpu_helpers import to_dev
    ad, bd = to_dev(a, dtype), to_dev(b, dtype)
    scratch = torch.empty(max(si.si_rehash_scratch_bytes(ad.numel()), 16), dtype=torch.uint8, device="cuda")
    cos = torch.full((1,), -7.0, dtype=torch.float64, device="cuda")
    dec = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    si.si_rehash_check(ad, bd, gamma, cos, dec, scratch)
    torch.cuda.synchronize()
    res = torch.empty(16, dtype=torch.uint8, device="cuda")
    c2, d2 = si.si_rehash_check_sync(ad, bd, gamma, scratch, res)
    assert (c2 == cos.item() or (math.isnan(c2) and math.isnan(cos.item()))) and d2 == dec.item()
    return cos.item(), dec.item()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n", [0, 1, 7, 8, 9, 1023, 4096, 100_003, 3_000_001])
def test_cosine_matches_oracle(dtype, n):
    rng = np.random.default_rng(n + 1)
    a = wl.round_to_storage(rng.standard_normal(n, dtype=np.float32), dtype)
    b = wl.round_to_storage(a + 0.3 * rng.standard_normal(n, dtype=np.float32), dtype)
    ref = oracle.cosine_ref(a, b)
    for gamma in (0.5, 0.95, 0.99, -1.0, 1.0):
        cos, dec = _gpu_check(a, b, dtype, gamma)
        assert cos == pytest.approx(ref, abs=1e-12)
        assert dec == oracle.rehash_decision_ref(a, b, gamma)


def test_closed_forms_and_degenerate_cases():
    rng = np.random.default_rng(0)
    a = wl.round_to_storage(rng.standard_normal(5000, dtype=np.float32), "bf16")
    assert _gpu_check(a, a, "bf16", 1.0) == (1.0, 1)              # tie: cos == gamma -> reuse
    c, d = _gpu_check(a, -a, "bf16", -1.0)
    assert c == -1.0 and d == 1
    c, d = _gpu_check(a, 2 * a, "bf16", 0.999)
    assert c == pytest.approx(1.0, abs=1e-15) and d == 1
    e0 = np.zeros(64, np.float32); e0[3] = 2
    e1 = np.zeros(64, np.float32); e1[40] = -5
    assert _gpu_check(e0, e1, "f32", 0.0) == (0.0, 1)
    z = np.zeros(64, np.float32)
    assert _gpu_check(z, z, "f32", 0.95) == (1.0, 1)
    assert _gpu_check(z, e0, "f32", 0.95) == (0.0, 0)
    bad = e0.copy(); bad[5] = np.inf
    c, d = _gpu_check(bad, e0, "f32", -1.0)
    assert math.isnan(c) and d == 0
    bad[5] = np.nan
    c, d = _gpu_check(bad, e0, "f32", -1.0)
    assert math.isnan(c) and d == 0
    assert _gpu_check(np.array([1, 0], np.float32), np.array([3, 4], np.float32), "f32", 0.6)[0] == pytest.approx(0.6, abs=1e-15)


def test_threshold_adjacent_decisions_bf16():
    """Drifted features around the 0.95 threshold: decisions must equal the oracle's."""
    rng = np.random.default_rng(11)
    n = 1 << 20
    x0 = wl.round_to_storage(rng.standard_normal(n, dtype=np.float32), "bf16")
    for s in np.linspace(0.30, 0.36, 13):        # cos ~ 1/sqrt(1+s^2): 0.958 .. 0.941
        xk = wl.round_to_storage(x0 + np.float32(s) * rng.standard_normal(n, dtype=np.float32), "bf16")
        cos, dec = _gpu_check(xk, x0, "bf16", 0.95)
        assert dec == oracle.rehash_decision_ref(xk, x0, 0.95)
        assert cos == pytest.approx(oracle.cosine_ref(xk, x0), abs=1e-12)
