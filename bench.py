"""Benchmark of the training step on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload big|base|lm16|big_accum|tiny]

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
    oracle = OracleTransformer(shape, init_params(shape, 0), TrainConfig(init_loss_scale=1.0))
    t0 = time.time()
    r = oracle.train_step(src, tgt, sl, tl)
    oracle.apply_update(1e-4)
    dt = time.time() - t0
    return {"value": r["ntokens"] / dt, "unit": "target tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d sentences / %d target tokens of the first %s batch, one train step + Adam update, "
                      "numpy float64, %.1f s" % (n, r["ntokens"], workload, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=12)
    ap.add_argument("--workload", default="big", choices=list(WORKLOAD_RUN))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=384)
    ap.add_argument("--profile-steps", type=int, default=3)
    ap.add_argument("--no-overlap", action="store_true", help="enqueue weight-gradient work on the main stream too")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_1904_01038_amd as T
    from synth import PRESETS, WORKLOADS, init_params, make_batches, count_params

    assert torch.cuda.is_available(), "bench.py needs a GPU"
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
                        dropout=dropout, init_loss_scale=scale, seed=0)
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
        ctx.apply_update(lr, sync=sync)
        return tok

    for i in range(args.warmup):
        window(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    tokens = 0
    for i in range(args.steps):
        tokens += window(args.warmup + i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    st = ctx.get_scaler()

    # Profiled passes: HIP events around every launch, on the stream it is launched on.  The first pass puts all work
    # on one stream, so every kernel is timed with the GPU to itself: `roofline` is that pass.  The second keeps the
    # side stream of the timed region; its brackets overlap, so its per-kernel durations are longer and do not add up
    # to the step time (`overlapped`).
    def profiled(overlap):
        ctx.set_overlap(overlap)
        ctx.profile_enable(True)
        for i in range(args.profile_steps):
            window(i)
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

    out = {"metric": "target tokens/sec per training step on 1 MI355X", "value": tokens / dt, "unit": "tokens/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": prec_name, "data": "synthetic",
           "config": {"workload": args.workload, "model": w["model"], "params": count_params(shape),
                      "update_freq": k, "dropout": dropout, "side_stream": not args.no_overlap, "tokens_per_step": tokens / args.steps,
                      "loss_scale_end": st["loss_scale"], "num_updates": st["num_updates"]},
           "roofline": roofline}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload, shape, batches, args.cpu_sample_tokens)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
