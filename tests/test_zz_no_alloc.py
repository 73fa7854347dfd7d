"""si_rehash_check_static (the entry point that allocates nothing: its partial sums live in a
device array of the library) against si_rehash_check with caller-provided scratch: same cosine
bits and the same decision, on two calls in a row, the second on a smaller input."""
import ctypes as C
import math

import numpy as np
import pytest

import si_workloads as wl

pytestmark = pytest.mark.gpu


def _both(a_np, b_np, dtype, gamma):
    import torch
    import paper_2411_01171_amd as si
    from gpu_helpers import to_dev
    a, b = to_dev(a_np, dtype), to_dev(b_np, dtype)
    n = a.numel()
    scratch = torch.empty(max(si.si_rehash_scratch_bytes(n), 16), dtype=torch.uint8, device="cuda")
    cos_ref = torch.full((1,), -7.0, dtype=torch.float64, device="cuda")
    dec_ref = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    si.si_rehash_check(a, b, gamma, cos_ref, dec_ref, scratch)
    cos = torch.full((1,), -7.0, dtype=torch.float64, device="cuda")
    dec = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    # raw C ABI: pointers and sizes only
    lib = si.lib()
    code = 1 if dtype == "bf16" else 0
    st = lib.si_rehash_check_static(C.c_void_p(a.data_ptr()), C.c_void_p(b.data_ptr()), C.c_int64(n), C.c_int32(code),
                                    C.c_float(gamma), C.c_void_p(cos.data_ptr()), C.c_void_p(dec.data_ptr()),
                                    C.c_void_p(torch.cuda.current_stream().cuda_stream or None))
    assert st == 0, si.si_status_str(st)
    torch.cuda.synchronize()
    return (cos.item(), dec.item()), (cos_ref.item(), dec_ref.item())


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_scratch_entry_point_matches_on_two_calls_in_a_row(dtype):
    import paper_2411_01171_amd as si
    assert si.lib().si_init_device() == 0
    rng = np.random.default_rng(42)
    for n in (3_000_001, 70_001, 9):            # the later calls are smaller: stale partial sums must not be read
        a = wl.round_to_storage(rng.standard_normal(n, dtype=np.float32), dtype)
        b = wl.round_to_storage(a + 0.33 * rng.standard_normal(n, dtype=np.float32), dtype)
        for gamma in (0.95, 0.5):
            got, ref = _both(a, b, dtype, gamma)
            assert got[1] == ref[1]
            assert got[0] == ref[0] or (math.isnan(got[0]) and math.isnan(ref[0]))


def test_static_scratch_entry_point_rejects_sizes_beyond_its_maximum():
    import torch
    import paper_2411_01171_amd as si
    t = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    dec = torch.zeros(1, dtype=torch.int32, device="cuda")
    lib = si.lib()
    too_many = (1 << 33) + 1
    st = lib.si_rehash_check_static(C.c_void_p(t.data_ptr()), C.c_void_p(t.data_ptr()), C.c_int64(too_many), C.c_int32(1),
                                    C.c_float(0.9), None, C.c_void_p(dec.data_ptr()), None)
    assert st == 2                              # SI_ERR_SHAPE, nothing enqueued
