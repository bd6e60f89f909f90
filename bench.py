"""Benchmark of the training step on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload big|base|lm16|big_accum|tiny|decode|gemm_shapes]

A "step" is one update window of the named workload: k sub-batches through tfm_train_step (forward, scaled loss,
backward, inf/nan scan) followed by tfm_apply_update (scaler + fp32 Adam).  Prints ONE JSON line:
metric = target tokens/s, with `roofline` for the dominant kernel class (measured live with HIP events on the
library's stream in a separate profiled pass) and `cpu_baseline` (the CPU oracle on a bounded sample).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_PEAK_TFLOPS = 2500.0      # MI355X dense fp16/bf16
FP32_PEAK_TFLOPS = 157.3
HBM_PEAK_GBS = 8000.0

WORKLOAD_RUN = {
    # name: (precision, dropout, update frequency k, init scale)
    "tiny": ("fp32", 0.0, 1, 1.0),
    "base": ("bf16", 0.1, 1, 1.0),
    "big": ("fp16", 0.1, 1, 128.0),
    "big_accum": ("fp16", 0.1, 16, 128.0),
    "lm16": ("fp16", 0.1, 4, 128.0),
    "lm16a": ("fp16", 0.1, 4, 128.0),
    "lm24": ("fp16", 0.1, 4, 128.0),
}


def cpu_baseline(workload, shape, batches, sample_tokens):
    """The oracle as it stands (numpy float64), timed on a bounded sample of the same workload."""
    import numpy as np
    from oracle.transformer import OracleTransformer, TrainConfig
    from synth import init_params
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    b = batches[0]
    n, tok = 0, 0
    while n < len(b.tgt_lens) and tok < sample_tokens:
        tok += int(b.tgt_lens[n])
        n += 1
    if shape.enc_layers == 0:
        n, cut = 1, min(int(b.tgt_lens[0]), sample_tokens)
        tgt, tl, src, sl = b.tgt[:1, :cut], np.array([cut], np.int32), None, None
    else:
        tgt, tl, src, sl = b.tgt[:n], b.tgt_lens[:n], b.src[:n], b.src_lens[:n]
    oracle = OracleTransformer(shape, init_params(shape, 0), TrainConfig(init_loss_scale=1.0, label_smoothing=0.0 if shape.cutoffs else 0.1))
    t0 = time.time()
    r = oracle.train_step(src, tgt, sl, tl)
    oracle.apply_update(1e-4)
    dt = time.time() - t0
    return {"value": r["ntokens"] / dt, "unit": "target tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d sentences / %d target tokens of the first %s batch, one train step + Adam update, "
                      "numpy float64, %.1f s" % (n, r["ntokens"], workload, dt)}


def run_decode(args):
    """Beam-search translation with incremental decoding (Implementation, Inference; the paper's Table 1 setting: big
    Transformer, beam 4, fp16).  A "step" is one token-capped batch of source sentences translated to the length cap."""
    import numpy as np
    import torch
    import paper_1904_01038_amd as T
    from tests.beam_search import beam_search
    from synth import PRESETS, init_params, count_params
    from synth.batches import zipf_ids

    torch.cuda.set_device(0)
    shape = PRESETS["big"]
    beam, extra = 4, 10
    rng = np.random.Generator(np.random.PCG64(6))
    n_pool = 3003                                         # size of the test set the paper's table uses; lengths only
    lens = rng.integers(10, 81, n_pool).astype(np.int32)
    sents = [np.append(zipf_ids(rng, int(n) - 1, shape.vocab), shape.eos_id).astype(np.int32) for n in lens]
    groups = T.batch_by_length(None, lens, args.decode_max_tokens, 1024, 8)
    order = rng.permutation(len(groups))
    max_b = max(len(g) for g in groups)
    max_len = int(lens.max()) + extra
    cfg = T.make_config(shape, precision=T.FP16, max_sentences=max_b, max_len=max_len,
                        max_tokens=(args.decode_max_tokens + 63) // 64 * 64, dropout=0.1)
    ctx = T.Tfm(cfg)
    ctx.set_params(init_params(shape, 0))
    dec = T.Decoder(ctx, max_b * beam, max_len, args.decode_max_tokens, 2 * beam)

    def translate(g):
        idx = groups[g]
        sl = lens[idx]
        src = np.full((len(idx), int(sl.max())), shape.pad_id, np.int32)
        for i, j in enumerate(idx):
            src[i, :sl[i]] = sents[j]
        dec.begin(src, sl, beam)
        out = beam_search(dec.step, len(idx), beam, int(sl.max()) + extra, shape.eos_id)
        return len(idx), sum(len(h[0][1]) for h in out), int(sl.max()) + extra

    for i in range(args.warmup):
        translate(order[i % len(order)])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    n_sent = n_tok = n_steps = 0
    for i in range(args.steps):
        a, b, c_ = translate(order[(args.warmup + i) % len(order)])
        n_sent, n_tok, n_steps = n_sent + a, n_tok + b, n_steps + c_
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    ctx.profile_enable(True)
    for i in range(min(args.profile_steps, 2)):
        translate(order[i % len(order)])
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    total_ms = sum(p["ms"] for p in prof.values())
    classes = {k: {"launches": p["launches"], "ms": p["ms"], "share": p["ms"] / total_ms,
                   "gbs": p["bytes"] / (p["ms"] * 1e-3) / 1e9 if p["ms"] > 0 else 0.0}
               for k, p in prof.items() if p["launches"]}
    dom = max(("gemm", "attention"), key=lambda k: prof[k]["ms"])
    g = prof[dom]
    achieved = g["bytes"] / (g["ms"] * 1e-3) / 1e9
    roofline = {"kernel": "%s class of the decoding step" % dom, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                "algorithmic_bytes_per_launch": g["bytes"] / g["launches"], "avg_launch_ms": g["ms"] / g["launches"],
                "classes": classes, "gpu_ms_share_of_wall": None}
    out = {"metric": "sentences/sec, beam search with incremental decoding on 1 MI355X", "value": n_sent / dt,
           "unit": "sentences/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "fp16", "data": "synthetic",
           "config": {"workload": "decode", "beam": beam,
                      "batch_cap_padded_tokens": args.decode_max_tokens, "sentences": n_sent, "decode_steps": n_steps,
                      "tokens_out_per_s": n_tok / dt,
                      "length_cap": "source length + %d (random weights never prefer eos: every hypothesis runs to the cap)" % extra},
           "roofline": roofline}
    if not args.no_cpu_baseline:
        from oracle.decoding import DecodingOracle, top_k
        oracle = DecodingOracle(shape, init_params(shape, 0))
        idx = groups[order[0]][:2]
        t1 = time.time()
        mems = [oracle.encode(sents[j]) for j in idx]
        hist = [[shape.eos_id] for _ in idx]
        n_cpu_steps = 4
        for _ in range(n_cpu_steps):                      # greedy, one row per sentence
            for r in range(len(idx)):
                hist[r].append(top_k(oracle.next_logprobs(mems[r], hist[r]), 1)[0][1])
        dtc = time.time() - t1
        try:
            from threadpoolctl import threadpool_info
            cores = max([p_.get("num_threads", 1) for p_ in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count()
        full = float(np.mean(lens[idx])) + extra
        out["cpu_baseline"] = {"value": len(idx) / (dtc * full / n_cpu_steps) , "unit": "sentences/s", "cores": int(cores),
                               "kind": "oracle",
                               "sample": "2 sentences, greedy (1 row each), encoder + %d decoding steps with the whole prefix "
                                         "recomputed per step, numpy float64, %.1f s; scaled linearly to the %d-step cap "
                                         "(an underestimate of the oracle's cost, which grows with the prefix)" % (n_cpu_steps, dtc, int(full))}
    print(json.dumps(out))


def run_gemm_shapes(args):
    """Context for the GEMM figures, not a step: every projection shape of the big Transformer at 3264 rows through
    tfm_op_gemm, stand-alone and cache-warm, beside the vendor library (torch.matmul) on the same operands."""
    import torch
    import paper_1904_01038_amd as T
    torch.cuda.set_device(0)
    rows, d, F, V, L = 3264, 1024, 4096, 32768, 6
    shapes = [  # form (0: X W^T, 1: dY W, 2: dY^T X), M, N, K, label
        (0, rows, 3 * d, d, "qkv fwd"), (0, rows, d, d, "out fwd"), (0, rows, F, d, "ffn1 fwd"), (0, rows, d, F, "ffn2 fwd"),
        (0, rows, L * 2 * d, d, "cross k/v of all layers fwd"), (0, rows, V, d, "vocabulary fwd"),
        (1, rows, d, 3 * d, "qkv dgrad"), (1, rows, d, d, "out dgrad"), (1, rows, F, d, "ffn2 dgrad"), (1, rows, d, F, "ffn1 dgrad"),
        (1, rows, d, L * 2 * d, "cross k/v of all layers dgrad"), (1, rows, d, V, "vocabulary dgrad"),
        (2, 3 * d, d, rows, "qkv wgrad"), (2, d, d, rows, "out wgrad"), (2, F, d, rows, "ffn1 wgrad"), (2, d, F, rows, "ffn2 wgrad"),
        (2, V, d, rows, "vocabulary wgrad"),
    ]
    dt = torch.float16
    torch.manual_seed(0)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(f, n):
        for _ in range(3):
            f()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(n):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    table = []
    for form, M, N, K, label in shapes:
        A = torch.randn((K, M) if form == 2 else (M, K), device="cuda", dtype=dt)
        B = torch.randn((N, K) if form == 0 else (K, N), device="cuda", dtype=dt)
        C = torch.empty(M, N, device="cuda", dtype=dt)
        ours = timed(lambda: T.ops.gemm(form, A, B, C, M, N, K), args.steps)
        lib = timed((lambda: torch.matmul(A, B.t())) if form == 0 else (lambda: torch.matmul(A, B)) if form == 1
                    else (lambda: torch.matmul(A.t(), B)), args.steps)
        fl = 2.0 * M * N * K
        table.append({"shape": label, "form": form, "M": M, "N": N, "K": K, "us": ours * 1e3, "tflops": fl / ours / 1e9,
                      "library_us": lib * 1e3, "library_tflops": fl / lib / 1e9})
    tot = sum(r["us"] for r in table)
    print(json.dumps({"metric": "stand-alone GEMM rate per projection shape (context, not a training step)",
                      "value": sum(2.0 * r["M"] * r["N"] * r["K"] for r in table) / (tot * 1e-6) / 1e12, "unit": "TFLOP/s",
                      "n_gpus": 1, "steps": args.steps, "warmup": 3, "higher_is_better": True, "dtype": "fp16", "data": "synthetic",
                      "config": {"workload": "gemm_shapes", "rows": rows}, "shapes": table}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=12)
    ap.add_argument("--workload", default="big", choices=list(WORKLOAD_RUN) + ["decode", "gemm_shapes"])
    ap.add_argument("--decode-max-tokens", type=int, default=3584, help="padded source tokens per decoding batch")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=1100)
    ap.add_argument("--profile-steps", type=int, default=3)
    ap.add_argument("--no-overlap", action="store_true", help="enqueue weight-gradient work on the main stream too")
    ap.add_argument("--attn-dropout", type=float, default=0.0, help="dropout on the attention weights (the named workloads use 0)")
    ap.add_argument("--relu-dropout", type=float, default=0.0, help="dropout on the feed-forward hidden activations (default 0)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_1904_01038_amd as T
    from synth import PRESETS, WORKLOADS, init_params, make_batches, count_params

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.workload == "decode":
        return run_decode(args)
    if args.workload == "gemm_shapes":
        return run_gemm_shapes(args)
    torch.cuda.set_device(0)
    w = WORKLOADS[args.workload]
    shape = PRESETS[w["model"]]
    prec_name, dropout, k, scale = WORKLOAD_RUN[args.workload]
    prec = {"fp32": T.FP32, "fp16": T.FP16, "bf16": T.BF16}[prec_name]
    n_pool = 16
    batches = make_batches(args.workload, n_pool)
    max_len = max(max(b.tgt.shape[1], 0 if b.src is None else b.src.shape[1]) for b in batches)
    max_tok = max(max(b.ntokens, 0 if b.src is None else int(b.src_lens.sum())) for b in batches)
    max_sent = max(len(b.tgt_lens) for b in batches)
    cfg = T.make_config(shape, precision=prec, max_sentences=max_sent, max_len=max_len, max_tokens=(max_tok + 63) // 64 * 64,
                        dropout=dropout, init_loss_scale=scale, seed=0, label_smoothing=0.0 if shape.cutoffs else 0.1,
                        attn_dropout=args.attn_dropout, relu_dropout=args.relu_dropout)
    ctx = T.Tfm(cfg)
    ctx.set_params(init_params(shape, 0))
    ctx.set_overlap(not args.no_overlap)
    lr = 1e-4

    def window(i, sync=False):
        tok = 0
        for j in range(k):
            b = batches[(i * k + j) % n_pool]
            ctx.train_step(b.src, b.tgt, b.src_lens, b.tgt_lens, sync=False)
            tok += b.ntokens
        u = ctx.apply_update(lr, sync=sync)
        return tok, u

    # Warm-up windows report their update synchronously, so the windows whose update was skipped (dynamic loss scaling:
    # the scale starts at 128 and halves on every overflow) are known by index; the timed windows do not synchronise,
    # their skips follow from the update counter.
    skipped_warmup = []
    for i in range(args.warmup):
        _, u = window(i, sync=True)
        if u["skipped"]:
            skipped_warmup.append(i)
    st0 = ctx.get_scaler()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    tokens = 0
    for i in range(args.steps):
        tokens += window(args.warmup + i)[0]
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    st = ctx.get_scaler()
    skipped_timed = args.steps - (st["num_updates"] - st0["num_updates"])

    # Profiled passes: HIP events around every launch, on the stream it is launched on.  The first pass puts all work
    # on one stream, so every kernel is timed with the GPU to itself: `roofline` is that pass.  The second keeps the
    # side stream of the timed region; its brackets overlap, so its per-kernel durations are longer and do not add up
    # to the step time (`overlapped`).
    def profiled(overlap):
        ctx.set_overlap(overlap)
        ctx.profile_enable(True)
        for i in range(args.profile_steps):
            window(args.warmup + args.steps + i)
        prof = ctx.profile_read()
        ctx.profile_enable(False)
        ctx.set_overlap(not args.no_overlap)
        total_ms = sum(p["ms"] for p in prof.values())
        classes = {}
        for name, p in prof.items():
            if p["launches"] == 0:
                continue
            e = {"launches_per_step": p["launches"] / args.profile_steps, "ms_per_step": p["ms"] / args.profile_steps,
                 "share": p["ms"] / total_ms}
            if p["flops"] > 0:
                e["tflops"] = p["flops"] / (p["ms"] * 1e-3) / 1e12
            if p["bytes"] > 0:
                e["gbs"] = p["bytes"] / (p["ms"] * 1e-3) / 1e9
            classes[name] = e
        return prof, classes

    prof, classes = profiled(False)
    overlapped = None
    if not args.no_overlap:
        p2, c2 = profiled(True)
        overlapped = {"gemm_tflops": c2["gemm"].get("tflops"), "ms_per_step": {k_: v["ms_per_step"] for k_, v in c2.items()}}
    g = prof["gemm"]
    achieved = g["flops"] / (g["ms"] * 1e-3) / 1e12 if g["ms"] > 0 else 0.0
    # HBM-side bytes per GEMM launch from the committed rocprofv3 counter runs of this workload (null if none)
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "train_step_%s_%s_hbm_traffic.json" % (args.workload, prec_name))
    if os.path.exists(tpath):
        t = json.load(open(tpath))["gemm"]
        traffic = (t["fetch_kib_raw"] * t["read_factor"] + t["write_kib_raw"] * t["write_factor"]) * 1024.0 / t["launches"]
    peak = FP32_PEAK_TFLOPS if prec == T.FP32 else MFMA_PEAK_TFLOPS
    roofline = {"kernel": "gemm (all projection, vocabulary and gradient GEMMs)", "bound": "mfma" if prec != T.FP32 else "alu",
                "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak, "traffic": traffic,
                "algorithmic_bytes_per_launch": g["bytes"] / max(g["launches"], 1),
                "avg_launch_ms": g["ms"] / max(g["launches"], 1), "launches_per_step": g["launches"] / args.profile_steps,
                "timed_with": "all launches on one stream (each kernel alone on the GPU)",
                "classes": classes, "overlapped": overlapped}
    # Step level: algorithmic matrix flops (GEMM + attention classes) of one step over the timed region's wall time per
    # step, against the same peak; and the sum of all kernels' stand-alone durations beside that wall time.
    ms_step = dt / args.steps * 1e3
    mfma_flops_step = (prof["gemm"]["flops"] + prof["attention"]["flops"]) / args.profile_steps
    kernel_ms = sum(p["ms"] for p in prof.values()) / args.profile_steps
    roofline["step_level"] = {"matrix_flops_per_step": mfma_flops_step, "tflops": mfma_flops_step / (ms_step * 1e-3) / 1e12,
                              "frac": mfma_flops_step / (ms_step * 1e-3) / 1e12 / peak,
                              "kernel_ms_per_step_single_stream": kernel_ms, "wall_ms_per_step": ms_step,
                              "wall_over_kernel": ms_step / kernel_ms if kernel_ms > 0 else None}
    # what this device sustains on the two resources, beside the published peaks (a register-only matrix-core loop; a plain
    # 1 GiB copy, bytes read plus written)
    ctx.close()
    del ctx
    torch.cuda.empty_cache()
    if prec != T.FP32:
        l2_cu, l2_all = T.ops.probe_fetch(64 << 10)
        fab_cu, fab_all = T.ops.probe_fetch(512 << 10)
        roofline["measured_ceilings"] = {"mfma_only_loop_tflops": T.ops.probe_mfma(prec), "copy_kernel_gbs": T.ops.probe_copy(1 << 30),
                                         "operand_fetch_gbs_per_cu": {"from_l2": l2_cu, "through_fabric": fab_cu},
                                         "operand_fetch_gbs_total": {"from_l2": l2_all, "through_fabric": fab_all},
                                         "published": {"mfma_tflops": MFMA_PEAK_TFLOPS, "hbm_gbs": HBM_PEAK_GBS}}

    out = {"metric": "target tokens/sec per training step on 1 MI355X", "value": tokens / dt, "unit": "tokens/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": prec_name, "data": "synthetic",
           "config": {"workload": args.workload, "update_freq": k, "dropout": dropout, "attn_dropout": args.attn_dropout, "relu_dropout": args.relu_dropout, "side_stream": not args.no_overlap, "tokens_per_step": tokens / args.steps,
                      "loss_scale_end": st["loss_scale"], "num_updates": st["num_updates"],
                      "skipped_warmup_windows": skipped_warmup, "skipped_timed_windows": skipped_timed},
           "roofline": roofline}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload, shape, batches, args.cpu_sample_tokens)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
