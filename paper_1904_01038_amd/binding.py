"""ctypes binding of the C boundary declared in include/tfm.h.

Argument marshalling only: every step of the path runs in the library's HIP kernels.  PyTorch supplies the
device workspace and the stream.  There is no fallback: if libtfm.so is missing or does not load, importing
the library handle raises.
"""
import ctypes as C
import os

import numpy as np

FP32, FP16, BF16 = 0, 1, 2
PROF_CLASSES = ["gemm", "attention", "norm", "loss", "embed", "optim"]
_HERE = os.path.dirname(os.path.abspath(__file__))


def lib_path():
    return os.path.join(_HERE, "libtfm.so")


class TfmError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("tfm error %d: %s" % (code, msg))
        self.code = code


class TfmConfig(C.Structure):
    _fields_ = [("enc_layers", C.c_int32), ("dec_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("pad_id", C.c_int32), ("eos_id", C.c_int32),
                ("max_sentences", C.c_int32), ("max_len", C.c_int32), ("max_tokens", C.c_int32),
                ("precision", C.c_int32), ("pre_norm", C.c_int32), ("dropout", C.c_float),
                ("attn_dropout", C.c_float), ("relu_dropout", C.c_float), ("label_smoothing", C.c_float), ("adam_beta1", C.c_float), ("adam_beta2", C.c_float),
                ("adam_eps", C.c_float), ("weight_decay", C.c_float), ("clip_norm", C.c_float), ("init_loss_scale", C.c_float),
                ("scale_window", C.c_int32), ("min_loss_scale", C.c_float), ("seed", C.c_uint64),
                ("n_cutoffs", C.c_int32), ("cutoffs", C.c_int32 * 3), ("adaptive_factor", C.c_int32)]


class StepOut(C.Structure):
    _fields_ = [("loss_sum", C.c_double), ("nll_sum", C.c_double), ("ntokens", C.c_int64), ("overflow", C.c_int32),
                ("loss_scale", C.c_float)]


class UpdateOut(C.Structure):
    _fields_ = [("skipped", C.c_int32), ("loss_scale_after", C.c_float), ("clean_steps", C.c_int32),
                ("num_updates", C.c_int64), ("grad_norm", C.c_float), ("ntokens_total", C.c_int64)]


class ProfEntry(C.Structure):
    _fields_ = [("launches", C.c_int64), ("ms", C.c_double), ("flops", C.c_double), ("bytes", C.c_double)]


_lib = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise FileNotFoundError(path + " is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        # PyTorch owns the device memory and the stream, so its HIP runtime must be the one this library binds to:
        # import it first, otherwise the loader would pull in a second copy of the runtime.
        import torch  # noqa: F401
        L = C.CDLL(path)
        vp, i32, i64, f32, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_uint64
        L.tfm_workspace_bytes.argtypes = [C.POINTER(TfmConfig), C.POINTER(C.c_size_t)]
        L.tfm_create.argtypes = [C.POINTER(TfmConfig), vp, C.c_size_t, vp, C.POINTER(vp)]
        L.tfm_destroy.argtypes = [vp]
        L.tfm_destroy.restype = None
        L.tfm_last_error.argtypes = [vp]
        L.tfm_last_error.restype = C.c_char_p
        L.tfm_num_params.argtypes = [vp, C.POINTER(i32)]
        L.tfm_param_info.argtypes = [vp, i32, C.c_char_p, C.POINTER(i64)]
        for f in (L.tfm_set_param, L.tfm_get_param, L.tfm_get_grad):
            f.argtypes = [vp, i32, vp, i64]
        L.tfm_get_adam.argtypes = [vp, i32, i32, vp, i64]
        L.tfm_set_adam.argtypes = [vp, i32, i32, vp, i64]
        L.tfm_get_scaler.argtypes = [vp, C.POINTER(f32), C.POINTER(i32), C.POINTER(i64)]
        L.tfm_set_scaler.argtypes = [vp, f32, i32, i64]
        L.tfm_train_step.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, C.POINTER(StepOut)]
        L.tfm_apply_update.argtypes = [vp, f32, C.POINTER(UpdateOut)]
        L.tfm_debug_set_loss_multiplier.argtypes = [vp, f32]
        L.tfm_set_overlap.argtypes = [vp, i32]
        L.tfm_profile_enable.argtypes = [vp, i32]
        L.tfm_decoder_workspace_bytes.argtypes = [vp, i32, i32, i32, i32, C.POINTER(C.c_size_t)]
        L.tfm_decoder_create.argtypes = [vp, vp, C.c_size_t, i32, i32, i32, i32, C.POINTER(vp)]
        L.tfm_decoder_destroy.argtypes = [vp]
        L.tfm_decoder_destroy.restype = None
        L.tfm_decoder_begin.argtypes = [vp, vp, vp, i32, i32, i32]
        L.tfm_decoder_step.argtypes = [vp, vp, vp, vp, vp]
        L.tfm_decoder_get_logprobs.argtypes = [vp, vp, i64]
        L.tfm_lr_inverse_sqrt.argtypes = [i64, i64, C.c_double, C.c_double]
        L.tfm_lr_inverse_sqrt.restype = C.c_double
        L.tfm_lr_cosine_restarts.argtypes = [i64, i64, C.c_double, C.c_double, C.c_double, C.c_double, C.c_double, C.c_double]
        L.tfm_lr_cosine_restarts.restype = C.c_double
        L.tfm_batch_by_length.argtypes = [vp, vp, i64, i32, i32, i32, vp, vp, C.POINTER(i64)]
        L.tfm_shuffle_batches.argtypes = [i64, u64, u64, vp]
        L.tfm_profile_read.argtypes = [vp, C.POINTER(ProfEntry), i32]
        L.tfm_op_gemm.argtypes = [i32, i32, i32, i32, i32, vp, i32, vp, i32, vp, i32, vp, i32, vp, vp, vp]
        L.tfm_op_gemm_ws.argtypes = [i32, i32, i32, i32, i32, vp, i32, vp, i32, vp, i32, vp, i32, vp, vp, vp, C.c_size_t, u64, f32,
                                     f32, vp]
        L.tfm_probe_mfma.argtypes = [i32, vp, C.c_size_t, C.POINTER(C.c_double), vp]
        L.tfm_probe_copy.argtypes = [vp, vp, C.c_size_t, C.POINTER(C.c_double), vp]
        L.tfm_probe_fetch.argtypes = [vp, C.c_size_t, C.c_size_t, C.POINTER(C.c_double), C.POINTER(C.c_double), vp]
        L.tfm_op_wgrad_grouped.argtypes = [i32, i32, vp, vp, vp, vp, vp, vp]
        L.tfm_op_attention_fwd.argtypes = [i32, vp, i32, vp, i32, vp, i32, vp, i32, vp, vp, vp, i32, i32, i32, i32, i32,
                                           i32, i32, u64, f32, vp, i32, vp]
        L.tfm_op_attention_bwd.argtypes = [i32, vp, i32, vp, i32, vp, i32, vp, i32, vp, i32, vp, vp, i32, vp, i32, vp,
                                           i32, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, u64, f32, vp, i32, vp]
        L.tfm_op_residual_layernorm_fwd.argtypes = [i32, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, u64, f32, vp]
        L.tfm_op_layernorm_bwd_scratch.argtypes = [i32, i32]
        L.tfm_op_layernorm_bwd_scratch.restype = C.c_size_t
        L.tfm_op_layernorm_bwd.argtypes = [i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, u64, f32, vp, vp]
        L.tfm_op_loss.argtypes = [i32, vp, vp, vp, vp, i32, i32, f32, f32, vp]
        L.tfm_op_adam.argtypes = [vp, vp, vp, vp, i32, vp, i32, i64, f32, f32, f32, f32, f32, f32, f32, f32, vp]
        L.tfm_op_scan_scratch.argtypes = [i64]
        L.tfm_op_scan_scratch.restype = C.c_size_t
        L.tfm_op_scan.argtypes = [i32, vp, i64, vp, vp, vp]
        L.tfm_op_scan_noalloc.argtypes = [i32, vp, i64, vp, vp]
        L.tfm_op_dropout_mask.argtypes = [u64, f32, vp, i64, vp]
        L.tfm_dropout_key.argtypes = [u64, u64, i32, i32, i32]
        L.tfm_dropout_key.restype = u64
        _lib = L
    return _lib


def make_config(shape, *, precision, max_sentences, max_len, max_tokens, dropout=0.0, label_smoothing=0.1,
                adam_beta1=0.9, adam_beta2=0.98, adam_eps=1e-8, clip_norm=0.0, init_loss_scale=128.0,
                scale_window=2000, min_loss_scale=2.0 ** -14, seed=0, attn_dropout=0.0, relu_dropout=0.0, weight_decay=0.0):
    """shape: any object with enc_layers, dec_layers, d_model, n_heads, d_ffn, vocab, pad_id, eos_id, pre_norm."""
    cut = tuple(getattr(shape, "cutoffs", ()))
    return TfmConfig(shape.enc_layers, shape.dec_layers, shape.d_model, shape.n_heads, shape.d_ffn, shape.vocab,
                     shape.pad_id, shape.eos_id, max_sentences, max_len, max_tokens, precision, shape.pre_norm,
                     dropout, attn_dropout, relu_dropout, label_smoothing, adam_beta1, adam_beta2, adam_eps, weight_decay, clip_norm, init_loss_scale,
                     scale_window, min_loss_scale, seed, len(cut), (C.c_int32 * 3)(*(list(cut) + [0] * (3 - len(cut)))),
                     getattr(shape, "factor", 4))


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class Tfm:
    """One training context on the current CUDA/HIP device.  The workspace is a torch uint8 tensor."""

    def __init__(self, cfg: TfmConfig, stream=None):
        import torch
        self._L = lib()
        self.cfg = cfg
        n = C.c_size_t()
        rc = self._L.tfm_workspace_bytes(C.byref(cfg), C.byref(n))
        if rc:
            raise TfmError(rc, self._L.tfm_last_error(None).decode())
        self.workspace_bytes = n.value
        self.workspace = torch.empty(n.value + 256, dtype=torch.uint8, device="cuda")
        base = self.workspace.data_ptr()
        aligned = (base + 255) // 256 * 256
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        h = C.c_void_p()
        rc = self._L.tfm_create(C.byref(cfg), C.c_void_p(aligned), n.value, C.c_void_p(self.stream.cuda_stream), C.byref(h))
        if rc:
            raise TfmError(rc, self._L.tfm_last_error(None).decode())
        self._h = h
        k = C.c_int32()
        self._check(self._L.tfm_num_params(h, C.byref(k)))
        self.param_names, self.param_shapes = [], []
        for i in range(k.value):
            name = C.create_string_buffer(64)
            shp = (C.c_int64 * 2)()
            self._check(self._L.tfm_param_info(h, i, name, shp))
            self.param_names.append(name.value.decode())
            self.param_shapes.append((shp[0], shp[1]) if shp[1] else (shp[0],))
        self.index = {n_: i for i, n_ in enumerate(self.param_names)}

    def _check(self, rc):
        if rc:
            raise TfmError(rc, self._L.tfm_last_error(self._h).decode())

    def close(self):
        for dec in getattr(self, "_decoders", []):
            dec.close()                      # a decoder uses the context's stream until it is destroyed
        self._decoders = []
        if getattr(self, "_h", None):
            self._L.tfm_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- parameters and state
    def set_params(self, params):
        for name, a in params.items():
            a = np.ascontiguousarray(a, dtype=np.float32)
            self._check(self._L.tfm_set_param(self._h, self.index[name], _ptr(a), a.size))

    def _get_all(self, fn, *extra):
        out = {}
        for i, (name, shp) in enumerate(zip(self.param_names, self.param_shapes)):
            a = np.empty(shp, dtype=np.float32)
            self._check(fn(self._h, i, *extra, _ptr(a), a.size))
            out[name] = a
        return out

    def get_params(self):
        return self._get_all(self._L.tfm_get_param)

    def get_grads(self):
        return self._get_all(self._L.tfm_get_grad)

    def get_adam(self, which):
        return self._get_all(self._L.tfm_get_adam, which)

    def get_scaler(self):
        s, c, n = C.c_float(), C.c_int32(), C.c_int64()
        self._check(self._L.tfm_get_scaler(self._h, C.byref(s), C.byref(c), C.byref(n)))
        return dict(loss_scale=s.value, clean_steps=c.value, num_updates=n.value)

    def set_scaler(self, loss_scale, clean_steps, num_updates):
        self._check(self._L.tfm_set_scaler(self._h, loss_scale, clean_steps, num_updates))

    # ---- the path
    def train_step(self, src, tgt, src_lens, tgt_lens, sync=True):
        src, tgt, src_lens, tgt_lens = _i32(src), _i32(tgt), _i32(src_lens), _i32(tgt_lens)
        B, Lt = tgt.shape
        Ls = 0 if src is None else src.shape[1]
        out = StepOut() if sync else None
        self._check(self._L.tfm_train_step(self._h, _ptr(src), _ptr(tgt), _ptr(src_lens), _ptr(tgt_lens), B, Ls, Lt,
                                           C.byref(out) if sync else None))
        if not sync:
            return None
        return dict(loss_sum=out.loss_sum, nll_sum=out.nll_sum, ntokens=out.ntokens, overflow=out.overflow,
                    loss_scale=out.loss_scale)

    def apply_update(self, lr, sync=True):
        out = UpdateOut() if sync else None
        self._check(self._L.tfm_apply_update(self._h, lr, C.byref(out) if sync else None))
        if not sync:
            return None
        return dict(skipped=out.skipped, loss_scale_after=out.loss_scale_after, clean_steps=out.clean_steps,
                    num_updates=out.num_updates, grad_norm=out.grad_norm, ntokens_total=out.ntokens_total)

    def set_overlap(self, on):
        self._check(self._L.tfm_set_overlap(self._h, 1 if on else 0))

    def debug_set_loss_multiplier(self, mult):
        self._check(self._L.tfm_debug_set_loss_multiplier(self._h, mult))

    def profile_enable(self, on):
        self._check(self._L.tfm_profile_enable(self._h, 1 if on else 0))

    def profile_read(self, reset=True):
        arr = (ProfEntry * len(PROF_CLASSES))()
        self._check(self._L.tfm_profile_read(self._h, arr, 1 if reset else 0))
        return {n: dict(launches=arr[i].launches, ms=arr[i].ms, flops=arr[i].flops, bytes=arr[i].bytes)
                for i, n in enumerate(PROF_CLASSES)}


class Decoder:
    """Incremental decoding on top of a training context's parameters (argument marshalling only)."""

    def __init__(self, ctx: "Tfm", max_rows, max_steps, max_src_tokens, topk):
        import torch
        self._L, self.ctx, self.topk = lib(), ctx, topk
        n = C.c_size_t()
        rc = self._L.tfm_decoder_workspace_bytes(ctx._h, max_rows, max_steps, max_src_tokens, topk, C.byref(n))
        if rc:
            raise TfmError(rc, "tfm_decoder_workspace_bytes: invalid sizes")
        self.workspace = torch.empty(n.value + 256, dtype=torch.uint8, device="cuda")
        aligned = (self.workspace.data_ptr() + 255) // 256 * 256
        h = C.c_void_p()
        ctx._check(self._L.tfm_decoder_create(ctx._h, C.c_void_p(aligned), n.value, max_rows, max_steps, max_src_tokens,
                                              topk, C.byref(h)))
        self._h = h
        self.rows = 0
        if not hasattr(ctx, "_decoders"):
            ctx._decoders = []
        ctx._decoders.append(self)

    def begin(self, src, src_lens, beam, n_sentences=None):
        src, src_lens = _i32(src), _i32(src_lens)
        B = len(src_lens) if src_lens is not None else n_sentences
        Ls = 0 if src is None else src.shape[1]
        self.ctx._check(self._L.tfm_decoder_begin(self._h, _ptr(src), _ptr(src_lens), B, Ls, beam))
        self.rows = B * beam

    def step(self, prev, parent=None):
        prev, parent = _i32(prev), _i32(parent)
        assert len(prev) == self.rows and (parent is None or len(parent) == self.rows)
        lp = np.empty((self.rows, self.topk), dtype=np.float32)
        ids = np.empty((self.rows, self.topk), dtype=np.int32)
        self.ctx._check(self._L.tfm_decoder_step(self._h, _ptr(prev), _ptr(parent), _ptr(lp), _ptr(ids)))
        return lp, ids

    def logprobs(self):
        V = self.ctx.cfg.vocab
        out = np.empty((self.rows, V), dtype=np.float32)
        self.ctx._check(self._L.tfm_decoder_get_logprobs(self._h, _ptr(out), out.size))
        return out

    def close(self):
        if self._h:
            self._L.tfm_decoder_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def lr_inverse_sqrt(t, warmup, peak_lr, init_lr=0.0):
    return lib().tfm_lr_inverse_sqrt(int(t), int(warmup), float(peak_lr), float(init_lr))


def lr_cosine_restarts(t, warmup, max_lr, min_lr, period, t_mult=1.0, shrink=1.0, init_lr=0.0):
    return lib().tfm_lr_cosine_restarts(int(t), int(warmup), float(max_lr), float(min_lr), float(period), float(t_mult),
                                        float(shrink), float(init_lr))


def batch_by_length(src_lens, tgt_lens, max_tokens, max_sentences, multiple=1):
    """List of int64 index arrays, one per batch."""
    tl = _i32(tgt_lens)
    sl = _i32(src_lens)
    n = len(tl)
    order = np.empty(n, dtype=np.int64)
    begin = np.empty(n + 1, dtype=np.int64)
    nb = C.c_int64()
    rc = lib().tfm_batch_by_length(_ptr(sl), _ptr(tl), n, max_tokens, max_sentences, multiple, _ptr(order), _ptr(begin),
                                   C.byref(nb))
    if rc:
        raise TfmError(rc, "tfm_batch_by_length: invalid argument")
    return [order[begin[b]:begin[b + 1]] for b in range(nb.value)]


def shuffle_batches(n_batches, seed, epoch):
    perm = np.empty(n_batches, dtype=np.int64)
    rc = lib().tfm_shuffle_batches(n_batches, seed, epoch, _ptr(perm))
    if rc:
        raise TfmError(rc, "tfm_shuffle_batches: invalid argument")
    return perm
