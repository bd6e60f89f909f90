"""Kernel-level GPU parity of the memory-bound kernels through the tfm_op_* entry points: residual + dropout + LayerNorm
forward and backward (every row/width path), the fused loss, and the inf/nan scan, against the oracle's float64 functions."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = {"fp32": 2e-5, "fp16": 2e-3, "bf16": 1.6e-2}


def _dt(prec):
    import torch
    return {"fp32": torch.float32, "fp16": torch.float16, "bf16": torch.bfloat16}[prec]


def _t(a, dt):
    import torch
    return torch.tensor(np.asarray(a), dtype=torch.float32).to(dt).cuda()


def _np(t):
    return t.double().cpu().numpy()


# rows x width: one row, a ragged handful, more rows than the row-per-wavefront kernel takes; widths that are / are not
# multiples of 512 (the row kernels need 512 | d), up to three 512-column chunks
LN_SHAPES = [(1, 64), (37, 512), (300, 1024), (130, 1536), (45, 136), (5000, 512), (4200, 1024), (70, 2048)]


@pytest.mark.parametrize("prec", ["fp32", "fp16", "bf16"])
@pytest.mark.parametrize("shape", LN_SHAPES)
@pytest.mark.parametrize("p", [0.0, 0.2])
def test_residual_layernorm_forward_and_backward(prec, shape, p):
    import torch
    import paper_1904_01038_amd as T
    from oracle.transformer import layer_norm_fwd, layer_norm_bwd, dropout_keep, dropout_key, site_id
    rows, d = shape
    dt = _dt(prec)
    rng = np.random.default_rng(rows + d)
    key = int(dropout_key(2, 5, site_id(1, 3, 2)))
    x, y, dn, add = (_t(rng.normal(size=(rows, d)), dt) for _ in range(4))
    gamma, beta = _t(1.0 + 0.2 * rng.normal(size=d), dt), _t(0.1 * rng.normal(size=d), dt)
    s_out, n_out = torch.zeros_like(x), torch.zeros_like(x)
    mean = torch.zeros(rows, dtype=torch.float32, device="cuda")
    rstd = torch.zeros(rows, dtype=torch.float32, device="cuda")
    T.ops.residual_layernorm_fwd(x, y, gamma, beta, s_out, n_out, mean, rstd, key, p)
    keep = dropout_keep(key, 0, rows, d, p) if p > 0 else np.ones((rows, d), bool)
    s_ref = _np(x) + np.where(keep, _np(y) / (1.0 - p), 0.0)
    n_ref, cache = layer_norm_fwd(s_ref, _np(gamma), _np(beta))
    tol = TOL[prec]
    assert np.abs(_np(s_out) - s_ref).max() <= tol * max(1.0, np.abs(s_ref).max())
    assert np.abs(_np(n_out) - n_ref).max() <= 2 * tol * max(1.0, np.abs(n_ref).max())
    assert np.abs(_np(mean) - s_ref.mean(1)).max() <= tol
    assert np.abs(_np(rstd) * np.sqrt(s_ref.var(1) + 1e-5) - 1.0).max() <= 2 * tol
    # backward from the kernel's own saved sum and statistics (what the step does)
    ds, ds_drop = torch.zeros_like(x), torch.zeros_like(x)
    dg, db, dbias = (torch.zeros(d, dtype=dt, device="cuda") for _ in range(3))
    T.ops.layernorm_bwd(dn, add, s_out, mean, rstd, gamma, ds, ds_drop, dg, db, dbias, key, p)
    _, cache = layer_norm_fwd(_np(s_out), _np(gamma), _np(beta))
    dx_ref, dg_ref, db_ref = layer_norm_bwd(_np(dn), cache)
    ds_ref = dx_ref + _np(add)
    assert np.abs(_np(ds) - ds_ref).max() <= 2 * tol * max(1.0, np.abs(ds_ref).max())
    drop_ref = np.where(keep, ds_ref / (1.0 - p), 0.0)
    if p > 0:
        assert np.abs(_np(ds_drop) - drop_ref).max() <= 3 * tol * max(1.0, np.abs(drop_ref).max())
    # column sums over `rows` terms: fp32 accumulation, results rounded to the compute dtype
    ctol = tol * np.sqrt(rows) * 3
    assert np.abs(_np(dg) - dg_ref).max() <= ctol * max(1.0, np.abs(dg_ref).max() / np.sqrt(rows))
    assert np.abs(_np(db) - db_ref).max() <= ctol * max(1.0, np.abs(db_ref).max() / np.sqrt(rows))
    assert np.abs(_np(dbias) - drop_ref.sum(0)).max() <= ctol * max(1.0, np.abs(drop_ref.sum(0)).max() / np.sqrt(rows))


@pytest.mark.parametrize("prec", ["fp32", "fp16", "bf16"])
@pytest.mark.parametrize("shape", [(5, 13), (33, 1000), (257, 32768), (3, 40000), (64, 4104)])
@pytest.mark.parametrize("eps", [0.0, 0.1])
def test_fused_loss_forward_and_backward(prec, shape, eps):
    import torch
    import paper_1904_01038_amd as T
    from oracle.transformer import label_smoothed_nll
    rows, V = shape
    dt = _dt(prec)
    rng = np.random.default_rng(V)
    z = _t(3.0 * rng.normal(size=(rows, V)), dt)
    y = rng.integers(0, V, rows)
    zr = _np(z)
    loss_ref, nll_ref, dz_ref = label_smoothed_nll(zr, y, eps)
    labels = torch.tensor(y, dtype=torch.int32).cuda()
    loss_rows = torch.zeros(rows, dtype=torch.float32, device="cuda")
    nll_rows = torch.zeros(rows, dtype=torch.float32, device="cuda")
    scale = 64.0
    T.ops.loss(z, labels, loss_rows, nll_rows, eps, scale)
    assert np.abs(_np(loss_rows) - loss_ref).max() <= 1e-5 * max(1.0, np.abs(loss_ref).max())
    assert np.abs(_np(nll_rows) - nll_ref).max() <= 1e-5 * max(1.0, np.abs(nll_ref).max())
    got = _np(z)
    tol = TOL[prec]
    assert np.abs(got - scale * dz_ref).max() <= tol * scale
    # the gradient of a row sums to zero (up to the rounding of its V entries)
    assert np.abs(got.sum(1)).max() <= tol * scale * np.sqrt(V) * 0.05 + 1e-3


@pytest.mark.parametrize("prec", ["fp32", "fp16", "bf16"])
@pytest.mark.parametrize("n", [8, 1000, 1 << 20, (1 << 22) + 264])
def test_scan_flag_and_sum_of_squares(prec, n):
    import torch
    import paper_1904_01038_amd as T
    dt = _dt(prec)
    rng = np.random.default_rng(n)
    x = _t(rng.normal(size=n), dt)
    res = torch.zeros(2, dtype=torch.float32, device="cuda")
    T.ops.scan(x, res)
    flag, ss = res.cpu().numpy()
    ref = float((_np(x) ** 2).sum())
    assert flag == 0.0 and abs(ss - ref) <= 1e-5 * ref
    for bad, pos in ((float("inf"), 0), (float("-inf"), n - 1), (float("nan"), n // 2)):
        xb = x.clone()
        xb[pos] = bad
        T.ops.scan(xb, res)
        assert res.cpu().numpy()[0] == 1.0, (bad, pos)
    # twice the same bits (fixed-order partial sums)
    T.ops.scan(x, res)
    assert res.cpu().numpy()[1] == ss


def test_measured_ceilings_are_plausible():
    """The two probes behind bench.py's `measured_ceilings`: below the published peaks, above half of them."""
    import paper_1904_01038_amd as T
    for dt in (T.FP16, T.BF16):
        tf = T.ops.probe_mfma(dt)
        assert 1000.0 < tf <= 2500.0 * 1.02, tf
    gbs = T.ops.probe_copy(1 << 28)
    assert 2000.0 < gbs <= 8000.0 * 1.02, gbs
    # operand fetch: an L2-resident region comes in faster than one served through the fabric, and no faster than 64 bytes
    # per clock and compute unit (2.4 GHz)
    l2_cu, l2_all = T.ops.probe_fetch(64 << 10)
    fab_cu, fab_all = T.ops.probe_fetch(512 << 10)
    assert 40.0 < l2_cu <= 64 * 2.4 * 1.02 and fab_cu < l2_cu and fab_all > 2000.0, (l2_cu, fab_cu, fab_all)
