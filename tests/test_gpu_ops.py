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
    # large outputs with short contractions: the 192x256 tiling (221 tiles, ragged in both directions) and the 256x256 tiling
    # (221 tiles where 192x256 would need a second round)
    (3200, 3080, 72), (3264, 4104, 40),
    # many rows, a narrow output, a long contraction: the 64x128 tiling (ragged in every direction)
    (1100, 520, 1032),
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
@pytest.mark.parametrize("shape", [(256, 128, 1100), (1024, 1024, 3041), (136, 264, 4000), (384, 128, 1024)])
def test_gemm_split_k_weight_gradient_is_exact_and_reproducible(prec, shape):
    import torch
    import paper_1904_01038_amd as T
    M, N, K = shape
    dt = _dtypes()[prec]
    rng = np.random.default_rng(K)
    A = rng.integers(-2, 3, (K, M)).astype(np.float64)         # "TN": A is [K, M]
    B = rng.integers(-2, 3, (K, N)).astype(np.float64)
    ref = A.T @ B
    assert np.abs(ref).max() < 2048
    tA, tB = _t(A, dt), _t(B, dt)
    ws = torch.empty(8 * 128 * 128 * 128, dtype=torch.float32, device="cuda")
    outs = []
    for _ in range(2):
        out = torch.zeros(M, N, dtype=dt, device="cuda")
        T.ops.gemm(2, tA, tB, out, M, N, K, workspace=ws)
        outs.append(out.float().cpu().numpy().astype(np.float64))
    want = _t(ref, dt).float().cpu().numpy().astype(np.float64)
    assert np.array_equal(outs[0], want)
    assert np.array_equal(outs[0], outs[1])
    small = torch.empty(16, dtype=torch.float32, device="cuda")   # a workspace that is too small falls back to one slice
    out = torch.zeros(M, N, dtype=dt, device="cuda")
    T.ops.gemm(2, tA, tB, out, M, N, K, workspace=small)
    assert np.array_equal(out.float().cpu().numpy().astype(np.float64), want)


@pytest.mark.parametrize("prec", ["fp32", "fp16", "bf16"])
@pytest.mark.parametrize("shape", [(200, 136, 72), (333, 264, 200), (257, 4096, 64)])
def test_gemm_result_dropout_and_scaled_mask_are_exact(prec, shape):
    """The two epilogue steps of the feed-forward layer with dropout on its hidden activations: relu(A B^T + b) with
    inverted dropout (p = 1/2: kept values double, exact on small integers; keep bits from the oracle's generator), and
    the masked product multiplied by the dropout scale."""
    import torch
    import paper_1904_01038_amd as T
    from oracle.transformer import dropout_keep, dropout_key, site_id
    M, N, K = shape
    dt = _dtypes()[prec]
    rng = np.random.default_rng(M + N)
    A = rng.integers(-3, 4, (M, K)).astype(np.float64)
    B = rng.integers(-3, 4, (N, K)).astype(np.float64)
    bias = rng.integers(-4, 5, N).astype(np.float64)
    key = int(dropout_key(3, 9, site_id(0, 1, 5)))
    keep = dropout_keep(key, 0, M, N, 0.5)
    assert 0.4 < keep.mean() < 0.6
    ref = np.where(keep, np.maximum(A @ B.T + bias, 0.0) * 2.0, 0.0)
    assert np.abs(ref).max() < 2048
    out = torch.full((M, N), 7.0, dtype=dt, device="cuda")
    T.ops.gemm(0, _t(A, dt), _t(B, dt), out, M, N, K, bias=_t(bias, dt), relu=True, drop_key=key, drop_p=0.5)
    got = out.float().cpu().numpy().astype(np.float64)
    want = _t(ref, dt).float().cpu().numpy().astype(np.float64)
    assert np.array_equal(got, want), np.abs(got - want).max()
    # masked input gradient: (dY W) * [h > 0] * 2
    W = rng.integers(-2, 3, (K, N)).astype(np.float64)      # "NN": B is [K, N]
    mask = np.where(keep, np.maximum(A @ B.T + bias, 0.0), 0.0)
    ref2 = np.where(mask > 0, (A @ W) * 2.0, 0.0)
    assert np.abs(ref2).max() < 2048
    out2 = torch.full((M, N), 7.0, dtype=dt, device="cuda")
    T.ops.gemm(1, _t(A, dt), _t(W, dt), out2, M, N, K, mask=_t(mask, dt), mask_scale=2.0)
    got2 = out2.float().cpu().numpy().astype(np.float64)
    want2 = _t(ref2, dt).float().cpu().numpy().astype(np.float64)
    assert np.array_equal(got2, want2), np.abs(got2 - want2).max()


@pytest.mark.parametrize("prec", ["fp16", "bf16"])
@pytest.mark.parametrize("tile", ["small", "large"])
def test_grouped_weight_gradients_with_bias_sums_are_exact(prec, tile):
    """Several A^T B products of different shapes plus the column sums of A in one launch, against the float64 definitions.
    Small integers make every product and sum exact.  "large" has enough tiles for the 256x256 configuration."""
    import torch
    import paper_1904_01038_amd as T
    dt = _dtypes()[prec]
    rng = np.random.default_rng(11)
    if tile == "small":
        shapes = [(136, 264, 300, True), (8, 8, 8, True), (384, 128, 1032, False), (200, 72, 77, True), (128, 512, 64, True)]
    else:   # M, N, K, with column sums
        shapes = [(1024, 1024, 520, True), (3072, 1024, 300, True), (1024, 4096, 264, False), (520, 264, 1000, True), (4096, 1024, 136, True)]
    jobs, refs = [], []
    for M, N, K, with_sum in shapes:
        A = rng.integers(-2, 3, (K, M)).astype(np.float64)
        B = rng.integers(-2, 3, (K, N)).astype(np.float64)
        ld = M + 24                                                 # a strided view, as the fused QKV gradient is
        tA = torch.zeros(K, ld, dtype=dt, device="cuda")
        tA[:, :M] = _t(A, dt)
        out = torch.full((M, N), 7.0, dtype=dt, device="cuda")
        cs = torch.full((M,), 7.0, dtype=dt, device="cuda") if with_sum else None
        jobs.append((tA[:, :M], _t(B, dt), out, cs))
        refs.append((A.T @ B, A.sum(axis=0)))
        assert np.abs(refs[-1][0]).max() < 2048 and np.abs(refs[-1][1]).max() < 256
    for _ in range(2):                                              # twice: the same bits
        T.ops.wgrad_grouped(jobs)
        for (tA, tB, out, cs), (rc, rs) in zip(jobs, refs):
            got = out.float().cpu().numpy().astype(np.float64)
            want = _t(rc, dt).float().cpu().numpy().astype(np.float64)
            assert np.array_equal(got, want), np.abs(got - want).max()
            if cs is not None:
                assert np.array_equal(cs.float().cpu().numpy().astype(np.float64), rs)
    with pytest.raises(T.TfmError):                                 # a width that is not a multiple of 8 is refused, nothing runs
        bad = torch.zeros(16, 12, dtype=dt, device="cuda")
        T.ops.wgrad_grouped([(bad, bad, torch.zeros(12, 12, dtype=dt, device="cuda"), None)])


@pytest.mark.parametrize("prec", ["fp16", "bf16"])
@pytest.mark.parametrize("shape,bias,relu", [((280, 1024, 1024), True, False), ((192, 1024, 4096), True, True), ((72, 512, 640), False, False),
                                             ((320, 3072, 1024), True, False)])
def test_gemm_few_rows_split_k_with_bias_and_relu_is_exact(prec, shape, bias, relu):
    """X W^T with few rows (a decoding step): 64x64 tiles, K split over blocks, bias and ReLU applied by the reduction."""
    import torch
    import paper_1904_01038_amd as T
    M, N, K = shape
    dt = _dtypes()[prec]
    rng = np.random.default_rng(M + K)
    A = rng.integers(-2, 3, (M, K)).astype(np.float64)
    B = rng.integers(-2, 3, (N, K)).astype(np.float64)
    bv = rng.integers(-3, 4, N).astype(np.float64)
    ref = A @ B.T + (bv if bias else 0.0)
    if relu:
        ref = np.maximum(ref, 0.0)
    assert np.abs(ref).max() < 2048 or prec == "bf16"
    want = _t(ref, dt).float().cpu().numpy().astype(np.float64)
    tA, tB, tb = _t(A, dt), _t(B, dt), _t(bv, dt)
    ws = torch.empty(8 * 320 * 3072, dtype=torch.float32, device="cuda")
    outs = []
    for w in (ws, None, ws):
        out = torch.zeros(M, N, dtype=dt, device="cuda")
        T.ops.gemm(0, tA, tB, out, M, N, K, bias=tb if bias else None, relu=relu, workspace=w)
        outs.append(out.float().cpu().numpy().astype(np.float64))
    if prec == "fp16":
        assert np.array_equal(outs[0], want)
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])    # split or not, run to run: the same bits


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


ATTN_CASES = [  # (query lengths, key lengths or None for self-attention, causal)
    ([5, 1, 33, 64], None, False),
    ([5, 1, 33, 64, 65, 100], None, True),
    ([7, 45, 80, 130], [9, 31, 97, 150], False),
    ([200, 3], None, True),
    # every sentence within one 64-row chunk: the backward kernel that forms dQ, dK and dV in one block
    ([5, 64, 33, 1], None, True),
    ([7, 45, 64, 1], [9, 64, 31, 64], False),
    # two chunks on one side or both
    ([7, 45, 80, 128], [9, 31, 97, 66], False),
    ([10, 60, 64], [70, 128, 1], False),
    ([70, 128, 3], [10, 64, 64], False),
    ([128, 127, 66, 2], None, True),
    # many short sentences (several per 64-row tile when a group table is passed)
    ([10, 12, 11, 30, 2, 1, 64, 5, 5, 5, 5, 40, 20, 3, 1, 1, 62], None, True),
    ([10, 12, 11, 30, 2, 1, 64, 5, 5, 5, 5, 40, 20, 3, 1, 1, 62], None, False),
    ([10, 12, 3, 30, 20, 7, 9, 9, 33], [12, 9, 40, 1, 33, 16, 8, 8, 31], False),
    ([1] * 40 + [3, 2] * 9, None, True),                 # more than 16 sentences would fit a tile: groups are cut at 16
]


def sentence_groups(lq, lk):
    """Runs of at most 16 consecutive sentences whose query rows and key rows each number at most 64 (greedy, as the library's
    ingest): one entry {first sentence, first query row, first key row, 0} per group and a closing entry."""
    out, first, sq, sk, rq, rk = [[0, 0, 0, 0]], 0, 0, 0, 0, 0
    for b in range(len(lq)):
        if b > first and (sq + lq[b] > 64 or sk + lk[b] > 64 or b - first >= 16):
            out.append([b, rq, rk, 0])
            first, sq, sk = b, 0, 0
        sq, sk, rq, rk = sq + lq[b], sk + lk[b], rq + lq[b], rk + lk[b]
    out.append([len(lq), rq, rk, 0])
    return out


@pytest.mark.parametrize("packed", [False, True])
@pytest.mark.parametrize("p_drop", [0.0, 0.25])
@pytest.mark.parametrize("prec,dh", [("fp32", 16), ("fp32", 64), ("fp16", 64), ("bf16", 64), ("fp16", 32)])
@pytest.mark.parametrize("case", ATTN_CASES)
def test_attention_forward_backward(prec, dh, case, p_drop, packed):
    """p_drop > 0: dropout on the attention weights; both sides derive the keep bits from the same key, query row, head and
    key index, each with its own implementation of the generator.  packed: the call also gets a table of sentence groups
    (several short sentences per 64-row tile); the results must not depend on it."""
    import torch
    import paper_1904_01038_amd as T
    from oracle.transformer import attention_fwd, attention_bwd, attention_keep, dropout_key, site_id
    lq, lk, causal = case
    dkey = int(dropout_key(17, 4, site_id(1, 2, 3)))
    lk = lq if lk is None else lk
    if packed and (max(lq) > 64 or max(lk) > 64 or dh != 64 or prec == "fp32"):
        pytest.skip("the group table only matters to the one-chunk matrix-core kernels")
    H = 3
    d = H * dh
    dt = _dtypes()[prec]
    rng = np.random.default_rng(len(lq) * 100 + dh)
    Tq, Tk = sum(lq), sum(lk)
    # q, k, v live in one [T, 3d] buffer like the fused projection output when the lengths agree
    q = _t(rng.normal(size=(Tq, d)), dt)
    k = _t(rng.normal(size=(Tk, d)), dt)
    v = _t(rng.normal(size=(Tk, d)), dt)
    do = _t(rng.normal(size=(Tq, d)), dt)
    q_off = torch.tensor(np.concatenate([[0], np.cumsum(lq)]), dtype=torch.int32).cuda()
    k_off = torch.tensor(np.concatenate([[0], np.cumsum(lk)]), dtype=torch.int32).cuda()
    o = torch.zeros(Tq, d, dtype=dt, device="cuda")
    lse = torch.zeros(H, Tq, dtype=torch.float32, device="cuda")
    groups = torch.tensor(sentence_groups(lq, lk), dtype=torch.int32).cuda() if packed else None
    T.ops.attention_fwd(q, k, v, o, lse, q_off, k_off, H, dh, max(lq), max(lk), causal, dkey, p_drop, groups)
    dq, dk, dv = (torch.zeros_like(x) for x in (q, k, v))
    T.ops.attention_bwd(q, k, v, o, do, lse, dq, dk, dv, q_off, k_off, H, dh, max(lq), max(lk), Tk, causal, dkey, p_drop, groups)
    qd, kd, vd, dod = (x.double().cpu().numpy() for x in (q, k, v, do))
    # With dropout the kept weights, and with them the outputs and their rounding, grow by 1 / (1 - p_drop); and where a
    # sentence has a single key, dS = P (dP - dO.O) vanishes only in exact arithmetic: the backward pass forms dO.O from the
    # rounded output, and dK sums that residue over all queries (reference exactly 0, so the bound is absolute).
    tol = {"fp32": 2e-5, "fp16": 4e-3, "bf16": 3e-2}[prec] * (1.0 if p_drop == 0 else 2.0 / (1.0 - p_drop))
    for b in range(len(lq)):
        qs, ks = slice(int(q_off[b]), int(q_off[b + 1])), slice(int(k_off[b]), int(k_off[b + 1]))
        keep = None
        if p_drop > 0:
            keep = [attention_keep(dkey, int(q_off[b]), lq[b], H, h, lk[b], p_drop) for h in range(H)]
        ctx, cache = attention_fwd(qd[qs], kd[ks], vd[ks], H, causal, keep, p_drop)
        rq, rk, rv = attention_bwd(dod[qs], cache)
        for name, got, ref in [("o", o[qs], ctx), ("dq", dq[qs], rq), ("dk", dk[ks], rk), ("dv", dv[ks], rv)]:
            got = got.double().cpu().numpy()
            scale = max(1.0, float(np.abs(ref).max()))
            assert np.abs(got - ref).max() <= tol * scale, (b, name, np.abs(got - ref).max(), scale)
        # log-sum-exp of the scaled scores
        for h in range(H):
            s = qd[qs, h * dh:(h + 1) * dh] @ kd[ks, h * dh:(h + 1) * dh].T / np.sqrt(dh)
            if causal:
                s = np.where(np.arange(s.shape[1])[None, :] <= np.arange(s.shape[0])[:, None], s, -np.inf)
            ref = np.log(np.exp(s - s.max(1, keepdims=True)).sum(1)) + s.max(1)
            assert np.abs(lse[h, qs].cpu().numpy() - ref).max() <= max(tol, 1e-4) * 4


@pytest.mark.parametrize("gprec", ["fp32", "fp16", "bf16"])
@pytest.mark.parametrize("wd", [0.0, 0.05])
@pytest.mark.parametrize("n", [8, 4096, 13288])          # less than one lane group, exactly one block, a ragged last block
def test_adam_kernel_against_the_library_optimiser(gprec, wd, n):
    """Three steps of the Adam kernel (gradient in fp32/fp16/bf16, unscaled by grad_mult, optional L2 weight decay) against
    torch.optim.Adam on the CPU in float64 fed with the same (rounded) gradients; the half copy equals the rounded master;
    nothing beyond the n elements is touched."""
    import torch
    import paper_1904_01038_amd as T
    lr, b1, b2, eps, mult = 3e-3, 0.9, 0.98, 1e-8, 1.0 / 64.0
    rng = np.random.default_rng(5)
    w0 = rng.normal(size=n)
    gdt = _dtypes()[gprec]
    pad = 4096                                               # guard elements behind every buffer
    wbuf = torch.full((n + pad,), 7.0, dtype=torch.float32, device="cuda")
    mbuf = torch.full((n + pad,), 7.0, dtype=torch.float32, device="cuda")
    vbuf = torch.full((n + pad,), 7.0, dtype=torch.float32, device="cuda")
    hbuf = torch.full((n + pad,), 7.0, dtype=torch.float16, device="cuda")
    w, m, v, half = wbuf[:n], mbuf[:n], vbuf[:n], hbuf[:n]
    w.copy_(torch.tensor(w0, dtype=torch.float32))
    m.zero_()
    v.zero_()
    half.zero_()
    ref = torch.tensor(w.cpu().numpy().astype(np.float64), requires_grad=True)
    opt = torch.optim.Adam([ref], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    for t in range(1, 4):
        g = _t(rng.normal(size=n) * 64.0, gdt)
        T.ops.adam(w, m, v, g, half, lr, b1, b2, eps, mult, 1.0 - b1 ** t, 1.0 - b2 ** t, weight_decay=wd)
        ref.grad = g.double().cpu() * mult
        opt.step()
        got = w.double().cpu().numpy()
        assert np.abs(got - ref.detach().numpy()).max() <= 2e-6 * t, (t, np.abs(got - ref.detach().numpy()).max())
        assert torch.equal(half, w.half())
    for buf in (wbuf, mbuf, vbuf, hbuf):
        assert bool((buf[n:] == 7.0).all())
