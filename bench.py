#!/usr/bin/env python3
"""Benchmark of the batched MLP cross-validation evaluator on one MI355X.

A "step" is one full evaluation call (fold lists, training of every
(suggestion, fold) model for all epochs, validation scoring, fold means) on a
synthetic workload already resident in HBM.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}  # MI355X dense MFMA peaks


def cpu_baseline(cfg, seconds_hint=20.0):
    """The oracle as it stands, timed on this machine's cores on a bounded sample."""
    import numpy as np
    from oracle import mlp_cv_oracle as O
    from paper_2012_04201_amd import inputs
    cores = len(os.sched_getaffinity(0))
    K = cfg["n_folds"]
    hps = cfg["hparams"]
    total_flops, _ = inputs.workload_flops(cfg)
    per_model_epoch = total_flops / sum(h["epochs"] * K for h in hps)
    # aim at ~seconds_hint of work at ~4 GFLOP/s per core (what the scalar fp64 loops reach)
    budget = seconds_hint * cores * 4e9
    n_sugg = max(1, min(len(hps), -(-cores // K)))
    epochs = int(max(1, min(hps[0]["epochs"], budget / (per_model_epoch * n_sugg * K))))
    sample = [dict(h, epochs=epochs) for h in hps[:n_sugg]]
    t0 = time.perf_counter()
    O.cv_eval(cfg["X"], cfg["y"], cfg["n_classes"], cfg["fold_idx"], K, sample, dtype=cfg["dtype"], n_threads=cores)
    dt = time.perf_counter() - t0
    return {"value": n_sugg * K * epochs / dt, "unit": "model-epochs/s", "cores": min(cores, n_sugg * K),
            "kind": "oracle",
            "sample": "first %d suggestions x %d folds x %d epoch(s) of the same workload, %.1f s" % (n_sugg, K, epochs, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cfg4", choices=["cfg0", "cfg1", "cfg2", "cfg3", "cfg4"])
    ap.add_argument("--suggestions", type=int, default=0, help="debug: evaluate only the first B suggestions")
    ap.add_argument("--epochs", type=int, default=0, help="debug: override the epoch count")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this evaluator runs on one GPU (items are independent; a multi-GPU run would only "
                 "split the work list); use --gpus 1")

    import torch
    from paper_2012_04201_amd import binding, inputs

    idx = int(args.workload[3])
    cfg = inputs.make_config(idx, B=args.suggestions or None, epochs=args.epochs or None)
    reduced = bool(args.suggestions or args.epochs)
    flops, model_epochs = inputs.workload_flops(cfg)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    X, y, ft = binding.to_device(cfg, dev)
    K, c, dt = cfg["n_folds"], cfg["n_classes"], cfg["dtype"]
    hps = cfg["hparams"]
    hp_arr = binding.make_hparams(hps)
    ws = binding.alloc_workspace(binding.bbo_mlp_workspace_bytes(len(cfg["y"]), X.shape[1], c, K, hps, dt, hp_arr), dev)
    stream = torch.cuda.current_stream()

    def step():
        return binding.bbo_mlp_cv_eval(X, y, c, ft, K, hps, dt, workspace=ws, stream=stream, hp_arr=hp_arr)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # events are recorded on the stream the kernels are launched on
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for a, b in ev:
        a.record(stream)
        scores, status = step()
        b.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_ms = [a.elapsed_time(b) for a, b in ev]
    avg_kernel_s = sum(kern_ms) / len(kern_ms) / 1e3
    ms_per_step = wall / args.steps * 1e3
    n_bad = int(status.sum().item())

    dname = "bf16" if dt else "f32"
    tflops = flops / (wall / args.steps) / 1e12
    achieved = flops / avg_kernel_s / 1e12
    out = {
        "metric": "MLP models x epochs/sec for batched CV eval",
        "value": model_epochs / (wall / args.steps),
        "unit": "model-epochs/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dname, "data": "synthetic",
        "config": {"workload": cfg["name"], "mlps": len(hps) * K, "suggestions": len(hps), "folds": K,
                   "rows": int(len(cfg["y"])), "features": int(X.shape[1]), "classes": c,
                   "epochs": hps[0]["epochs"], "reduced": reduced},
        "tflops": tflops, "pct_mfma_peak": 100.0 * tflops / PEAK_TFLOPS[dname],
        "nonfinite_suggestions": n_bad,
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_TFLOPS[dname], "unit": "TFLOP/s",
                     "frac": achieved / PEAK_TFLOPS[dname], "traffic": None,
                     "kernel": "k_train", "kernel_ms": avg_kernel_s * 1e3},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
