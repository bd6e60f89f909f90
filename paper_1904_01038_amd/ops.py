"""Bindings of the single-operation entry points (tfm_op_*): torch device tensors in, same names as the C calls."""
import ctypes as C

from .binding import lib, FP32, FP16, BF16, TfmError


def _dt(t):
    import torch
    return {torch.float32: FP32, torch.float16: FP16, torch.bfloat16: BF16}[t.dtype]


def _p(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc, what):
    if rc:
        raise TfmError(rc, what + " failed")


def gemm(form, A, B, C_out, M, N, K, lda=None, ldb=None, ldc=None, bias=None, relu=False, mask=None, residual=None,
         workspace=None, drop_key=0, drop_p=0.0, mask_scale=1.0):
    lda = A.stride(0) if lda is None else lda
    ldb = B.stride(0) if ldb is None else ldb
    ldc = C_out.stride(0) if ldc is None else ldc
    if workspace is not None or drop_p > 0.0 or mask_scale != 1.0:
        wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
        _check(lib().tfm_op_gemm_ws(_dt(A), form, M, N, K, _p(A), lda, _p(B), ldb, _p(C_out), ldc, _p(bias), int(relu),
                                    _p(mask), _p(residual), _p(workspace), wsb, int(drop_key), float(drop_p), float(mask_scale),
                                    _stream()), "tfm_op_gemm_ws")
        return
    _check(lib().tfm_op_gemm(_dt(A), form, M, N, K, _p(A), lda, _p(B), ldb, _p(C_out), ldc, _p(bias), int(relu),
                             _p(mask), _p(residual), _stream()), "tfm_op_gemm")


def wgrad_grouped(jobs):
    """jobs: list of (A[K, M], B[K, N], C[M, N], colsum[M] or None); C_i = A_i^T B_i and colsum_i = column sums of A_i, one launch."""
    n = len(jobs)
    dims = (C.c_int32 * (6 * n))()
    pa, pb, pc, ps = ((C.c_void_p * n)() for _ in range(4))
    for i, (A, B, Cm, cs) in enumerate(jobs):
        dims[6 * i:6 * i + 6] = [A.shape[1], B.shape[1], A.shape[0], A.stride(0), B.stride(0), Cm.stride(0)]
        pa[i], pb[i], pc[i], ps[i] = A.data_ptr(), B.data_ptr(), Cm.data_ptr(), (cs.data_ptr() if cs is not None else None)
    _check(lib().tfm_op_wgrad_grouped(_dt(jobs[0][0]) if n else FP16, n, dims, pa, pb, pc, ps, _stream()), "tfm_op_wgrad_grouped")


def attention_fwd(q, k, v, o, lse, q_off, k_off, H, dh, max_lq, max_lk, causal, drop_key=0, drop_p=0.0, groups=None):
    """groups: optional device int32 tensor [n_groups + 1, 4] (see tfm_op_attention_fwd)."""
    B = q_off.numel() - 1
    ng = 0 if groups is None else groups.shape[0] - 1
    _check(lib().tfm_op_attention_fwd(_dt(q), _p(q), q.stride(0), _p(k), k.stride(0), _p(v), v.stride(0), _p(o),
                                      o.stride(0), _p(lse), _p(q_off), _p(k_off), B, H, dh, max_lq, max_lk,
                                      lse.shape[1], int(causal), int(drop_key), float(drop_p), _p(groups), ng, _stream()),
           "tfm_op_attention_fwd")


def attention_bwd(q, k, v, o, d_o, lse, dq, dk, dv, q_off, k_off, H, dh, max_lq, max_lk, total_k, causal, drop_key=0,
                  drop_p=0.0, groups=None):
    B = q_off.numel() - 1
    ng = 0 if groups is None else groups.shape[0] - 1
    _check(lib().tfm_op_attention_bwd(_dt(q), _p(q), q.stride(0), _p(k), k.stride(0), _p(v), v.stride(0), _p(o),
                                      o.stride(0), _p(d_o), d_o.stride(0), _p(lse), _p(dq), dq.stride(0), _p(dk),
                                      dk.stride(0), _p(dv), dv.stride(0), _p(q_off), _p(k_off), B, H, dh, max_lq,
                                      max_lk, lse.shape[1], total_k, int(causal), int(drop_key), float(drop_p), _p(groups), ng,
                                      _stream()),
           "tfm_op_attention_bwd")


def residual_layernorm_fwd(x, y, gamma, beta, s_out, n_out, mean, rstd, key=0, p=0.0):
    rows, d = x.shape
    _check(lib().tfm_op_residual_layernorm_fwd(_dt(x), _p(x), _p(y), _p(gamma), _p(beta), _p(s_out), _p(n_out),
                                               _p(mean), _p(rstd), rows, d, key, p, _stream()),
           "tfm_op_residual_layernorm_fwd")


def layernorm_bwd(dn, add, s, mean, rstd, gamma, ds, ds_drop, dgamma, dbeta, dbias, key=0, p=0.0):
    import torch
    rows, d = dn.shape
    scratch = torch.empty(lib().tfm_op_layernorm_bwd_scratch(rows, d), dtype=torch.uint8, device=dn.device)
    _check(lib().tfm_op_layernorm_bwd(_dt(dn), _p(dn), _p(add), _p(s), _p(mean), _p(rstd), _p(gamma), _p(ds),
                                      _p(ds_drop), _p(dgamma), _p(dbeta), _p(dbias), rows, d, key, p, _p(scratch),
                                      _stream()), "tfm_op_layernorm_bwd")


def loss(z, labels, loss_rows, nll_rows, eps, scale):
    rows, V = z.shape
    _check(lib().tfm_op_loss(_dt(z), _p(z), _p(labels), _p(loss_rows), _p(nll_rows), rows, V, eps, scale, _stream()),
           "tfm_op_loss")


def adam(w, m, v, g, half_copy, lr, beta1, beta2, eps, grad_mult, bc1, bc2, weight_decay=0.0):
    hd = FP32 if half_copy is None else _dt(half_copy)
    _check(lib().tfm_op_adam(_p(w), _p(m), _p(v), _p(g), _dt(g), _p(half_copy), hd, w.numel(), lr, beta1, beta2, eps,
                             float(weight_decay), grad_mult, bc1, bc2, _stream()), "tfm_op_adam")


def scan(x, result):
    import torch
    scratch = torch.empty(lib().tfm_op_scan_scratch(x.numel()), dtype=torch.uint8, device=x.device)
    _check(lib().tfm_op_scan(_dt(x), _p(x), x.numel(), _p(result), _p(scratch), _stream()), "tfm_op_scan")


def scan_noalloc(x, result):
    """The scan through the entry point that allocates nothing (its partial results live in a static device array)."""
    L = lib()
    rc = L.tfm_op_scan_noalloc(_dt(x), _p(x), x.numel(), _p(result), _stream())
    if rc:
        from .binding import TfmError
        raise TfmError(rc, "tfm_op_scan_noalloc: " + (L.tfm_last_error(None) or b"").decode())


def dropout_mask(key, p, out):
    _check(lib().tfm_op_dropout_mask(key, p, _p(out), out.numel(), _stream()), "tfm_op_dropout_mask")


def dropout_key(seed, step, stream, layer, sub):
    return lib().tfm_dropout_key(seed, step, stream, layer, sub)


def probe_mfma(dtype=FP16):
    """TFLOP/s of a register-only matrix-core loop on every compute unit."""
    import torch
    scratch = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    out = C.c_double()
    _check(lib().tfm_probe_mfma(dtype, _p(scratch), scratch.numel(), C.byref(out), _stream()), "tfm_probe_mfma")
    return out.value


def probe_copy(nbytes=1 << 30):
    """GB/s (read + written) of a plain device copy of nbytes."""
    import torch
    a = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    b = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    out = C.c_double()
    _check(lib().tfm_probe_copy(_p(a), _p(b), nbytes, C.byref(out), _stream()), "tfm_probe_copy")
    return out.value


def probe_fetch(region_bytes=64 << 10):
    """(GB/s per compute unit, GB/s in total) at which one block per compute unit re-reads a private region of region_bytes:
    64 KiB regions stay in the L2 caches, 512 KiB regions are served through the fabric by the memory side."""
    import torch
    n = 256 * region_bytes + (1 << 20)
    buf = torch.zeros(n, dtype=torch.uint8, device="cuda")
    per_cu, total = C.c_double(), C.c_double()
    _check(lib().tfm_probe_fetch(_p(buf), n, region_bytes, C.byref(per_cu), C.byref(total), _stream()), "tfm_probe_fetch")
    return per_cu.value, total.value
