"""Kernel-level GPU parity through the tfm_op_* entry points against float64 numpy definitions."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _t(a, dtype):
    import torch
    return torch.tensor(a, dtype=torch.float32).to(dtype).cuda()


def _dtypes():
    import torch
    return {"fp32": torch.float32, "fp16": torch.float16, "bf16": torch.bfloat16}


GEMM_SHAPES = [  # M, N, K: several tiles plus ragged tails in every dimension
    (200, 136, 72), (128, 128, 64), (333, 264, 200), (1, 8, 8), (130, 8, 264), (257, 384, 1032),
]


@pytest.mark.parametrize("prec", ["fp32", "fp16", "bf16"])
@pytest.mark.parametrize("form", [0, 1, 2])
@pytest.mark.parametrize("shape", GEMM_SHAPES)
def test_gemm_forms_and_epilogues(prec, form, shape):
    import torch
    import paper_1904_01038_amd as T
    M, N, K = shape
    if form == 2 and M % 8:
        M = (M + 7) // 8 * 8
    dt = _dtypes()[prec]
    rng = np.random.default_rng(M * 7 + N * 3 + K + form)
    # small integers: products and sums are exact in every precision, so the comparison is bit-exact
    A = rng.integers(-3, 4, (M, K)).astype(np.float64)
    B = rng.integers(-3, 4, (K, N)).astype(np.float64)
    bias = rng.integers(-4, 5, N).astype(np.float64)
    res = rng.integers(-8, 9, (M, N)).astype(np.float64)
    mask = rng.integers(-1, 2, (M, N)).astype(np.float64)
    ref0 = A @ B
    tA = _t(A if form != 2 else A.T.copy(), dt)
    tB = _t(B if form != 0 else B.T.copy(), dt)
    for variant in ("plain", "bias_relu", "mask", "residual", "padded_ld"):
        ldc = N + 16 if variant == "padded_ld" else N
        out = torch.zeros(M, ldc, dtype=dt, device="cuda")
        kw = {}
        ref = ref0
        if variant == "bias_relu":
            kw = dict(bias=_t(bias, dt), relu=True)
            ref = np.maximum(ref0 + bias, 0)
        elif variant == "mask":
            kw = dict(mask=_t(mask, dt))
            ref = ref0 * (mask > 0)
        elif variant == "residual":
            kw = dict(residual=_t(res, dt), bias=_t(bias, dt))
            ref = ref0 + bias + res
        T.ops.gemm(form, tA, tB, out, M, N, K, ldc=ldc, **kw)
        got = out[:, :N].float().cpu().numpy().astype(np.float64)
        assert np.abs(ref).max() < 2048          # exactly representable in fp16 / bf16 range used here
        if prec == "bf16":
            ref = _t(ref, dt).float().cpu().numpy().astype(np.float64)   # output rounding to 8 bits of mantissa
        assert np.array_equal(got, ref), (variant, np.abs(got - ref).max())
        if variant == "padded_ld":
            assert not out[:, N:].any()


@pytest.mark.parametrize("prec", ["fp16", "bf16"])
def test_gemm_random_values_close_to_float64(prec):
    import torch
    import paper_1904_01038_amd as T
    dt = _dtypes()[prec]
    rng = np.random.default_rng(5)
    M, N, K = 520, 392, 776
    A = rng.normal(size=(M, K))
    B = rng.normal(size=(K, N))
    tA, tBt, tB, tAt = _t(A, dt), _t(B.T.copy(), dt), _t(B, dt), _t(A.T.copy(), dt)
    Ar, Br = tA.double().cpu().numpy(), tB.double().cpu().numpy()
    ref = Ar @ Br
    for form, (a, b) in enumerate([(tA, tBt), (tA, tB), (tAt, tB)]):
        out = torch.empty(M, N, dtype=dt, device="cuda")
        T.ops.gemm(form, a, b, out, M, N, K)
        got = out.double().cpu().numpy()
        tol = (2 ** -10 if prec == "fp16" else 2 ** -7) * np.abs(ref) + 1e-3
        assert np.all(np.abs(got - ref) <= tol), form
