"""The scan entry point that allocates nothing (tfm_op_scan_noalloc: partial results in a static device array) against
tfm_op_scan with a caller-owned scratch buffer: same kernels, so flag and sum of squares must agree bit for bit - on two
calls in a row, the second with a smaller input (the array keeps the first call's partial results), and on the argument
checks.  Collected last: a failure here must not hide the other GPU tests."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _pair(x):
    import torch
    import paper_1904_01038_amd as T
    a = torch.full((2,), -1.0, dtype=torch.float32, device="cuda")
    b = torch.full((2,), -2.0, dtype=torch.float32, device="cuda")
    T.ops.scan(x, a)
    T.ops.scan_noalloc(x, b)
    torch.cuda.synchronize()
    return a.cpu().numpy(), b.cpu().numpy()


@pytest.mark.parametrize("prec", ["fp16", "fp32", "bf16"])
def test_two_calls_in_a_row_second_smaller(prec):
    import torch
    dt = {"fp16": torch.float16, "fp32": torch.float32, "bf16": torch.bfloat16}[prec]
    rng = np.random.default_rng(17)
    big = torch.tensor(rng.normal(size=(1 << 22) + 2048), dtype=torch.float32).to(dt).cuda()   # every block of the grid has work
    small = torch.tensor(rng.normal(size=4096), dtype=torch.float32).to(dt).cuda()              # two blocks
    ref_big, got_big = _pair(big)
    assert np.array_equal(ref_big, got_big) and ref_big[0] == 0.0 and ref_big[1] > 0.0
    ref_small, got_small = _pair(small)
    assert np.array_equal(ref_small, got_small) and ref_small[0] == 0.0
    want = float((small.double() ** 2).sum())
    assert abs(got_small[1] - want) <= 1e-5 * want
    # a non-finite value in the smaller input, then the clean one again
    bad = small.clone()
    bad[4095] = float("inf")
    ref_bad, got_bad = _pair(bad)
    assert got_bad[0] == ref_bad[0] == 1.0
    ref_again, got_again = _pair(small)
    assert np.array_equal(ref_again, got_again) and np.array_equal(got_again, got_small)
    # no elements at all (a valid pointer, n = 0): flag 0, sum 0 from both
    import paper_1904_01038_amd as T
    L = T.lib()
    r0 = torch.full((2,), -1.0, dtype=torch.float32, device="cuda")
    r1 = torch.full((2,), -2.0, dtype=torch.float32, device="cuda")
    scratch = torch.empty(64, dtype=torch.uint8, device="cuda")
    p = lambda t: C.c_void_p(t.data_ptr())
    code = {"fp16": T.FP16, "fp32": T.FP32, "bf16": T.BF16}[prec]
    assert L.tfm_op_scan(code, p(small), 0, p(r0), p(scratch), None) == 0
    assert L.tfm_op_scan_noalloc(code, p(small), 0, p(r1), None) == 0
    torch.cuda.synchronize()
    assert r0.cpu().tolist() == [0.0, 0.0] and r1.cpu().tolist() == [0.0, 0.0]


def test_argument_checks():
    import torch
    import paper_1904_01038_amd as T
    L = T.lib()
    x = torch.zeros(64, dtype=torch.float16, device="cuda")
    r = torch.zeros(2, dtype=torch.float32, device="cuda")
    px, pr = C.c_void_p(x.data_ptr()), C.c_void_p(r.data_ptr())
    assert L.tfm_op_scan_noalloc(T.FP16, px, 64, pr, None) == 0
    assert L.tfm_op_scan_noalloc(T.FP16, px, 63, pr, None) == -1            # not a multiple of 8
    assert L.tfm_op_scan_noalloc(T.FP16, None, 64, pr, None) == -1
    assert L.tfm_op_scan_noalloc(7, px, 64, pr, None) == -1
    too_many = (1 << 31) + 8                                                # beyond the stated maximum: refused, nothing runs
    assert L.tfm_op_scan_noalloc(T.FP16, px, too_many, pr, None) == -1
    assert b"TFM_SCAN_NOALLOC_MAX_N" in L.tfm_last_error(None)
    torch.cuda.synchronize()
