#!/usr/bin/env python3
"""Benchmark of the batched MLP cross-validation evaluator on one MI355X.

A "step" is one full evaluation call (fold lists, training of every
(suggestion, fold) model for all epochs, validation scoring, fold means) on a
synthetic workload already resident in HBM.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4]
    python bench.py --workload cfg3 --linear   # the same suggestions without hidden layers
    python bench.py --copy-probe BYTES     # plain device copy, to calibrate HBM counters
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}  # MI355X dense MFMA peaks
PEAK_VALU_TFLOPS = 157.3  # fp32 vector: 256 CUs x 128 lanes x 2 flop (multiply-add) x 2.4 GHz
PEAK_HBM_GBS = 8000.0
# the sources each workload's training kernel is built from (the host code in bbo_mlp.hip does not count)
KERNEL_SOURCES = {"k_train_tiled": ["common.h", "train_tiled_bf16.h"], "k_train_small": ["common.h", "train_small_f32.h"],
                  "k_train_linear": ["common.h", "train_linear_f32.h"], "k_train": ["common.h", "bbo_mlp.hip"],
                  "k_train_mid": ["common.h", "train_mid_f32.h"]}
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")


def kernel_source_hash(kernel):
    """Hash of the code of one training kernel's sources: comments and white space do not count, so that a
    reworded comment does not void the counter record."""
    import re
    h = hashlib.sha256()
    for name in KERNEL_SOURCES[kernel]:
        with open(os.path.join(ROOT, "paper_2012_04201_amd", "csrc", name), "r") as fh:
            text = fh.read()
        text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)
        text = re.sub(r"//[^\n]*", " ", text)
        h.update(" ".join(text.split()).encode())
    return h.hexdigest()[:16]


def measured_traffic(workload, kernel):
    """HBM bytes per launch from the committed rocprofv3 counter runs; None when
    there is no record for this workload or the kernel's sources changed since."""
    if not os.path.exists(TRAFFIC_FILE):
        return None
    rec = {}
    for line in open(TRAFFIC_FILE):
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = line.split("=", 1)
            rec[k.strip()] = v.strip()
    if rec.get(workload + ".source_hash") != kernel_source_hash(kernel):
        return None
    try:
        return float(rec[workload + ".bytes_per_launch"])
    except (KeyError, ValueError):
        return None


def algorithmic_bytes(cfg):
    """HBM bytes one launch must move when the optimizer state does not fit on chip:
    every step reads and writes the fp32 weights and both moments (24 B per
    parameter; 16 B for SGD) and reads the minibatch's input rows; validation reads
    its rows once."""
    import numpy as np
    fold = cfg["fold_idx"]
    K = cfg["n_folds"]
    d = cfg["X"].shape[1]
    xb = 2 if cfg["dtype"] else 4
    c_out = cfg["n_classes"] if cfg["n_classes"] >= 2 else 1
    total = 0.0
    for f in range(K):
        n_va = int((fold == f).sum())
        n_tr = int((fold >= 0).sum()) - n_va
        for h in cfg["hparams"]:
            dims = [d] + list(h["hidden"]) + [c_out]
            P = sum(dims[l] * dims[l + 1] + dims[l + 1] for l in range(len(dims) - 1))
            bs = h["batch_size"] if 0 < h["batch_size"] <= n_tr else n_tr
            steps = -(-n_tr // bs) if n_tr else 0
            per_param = 24 if h.get("solver", "adam") == "adam" else 16
            total += h["epochs"] * (steps * per_param * P + n_tr * d * xb) + n_va * d * xb
    return total


def cpu_baseline(cfg, seconds_hint=20.0):
    """The oracle as it stands, timed on this machine's cores on a bounded sample."""
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
    if epochs == hps[0]["epochs"]:  # cheap models at their full epoch count: more suggestions instead
        n_sugg = int(max(n_sugg, min(len(hps), budget / (per_model_epoch * K * epochs))))
    sample = [dict(h, epochs=epochs) for h in hps[:n_sugg]]
    t0 = time.perf_counter()
    O.cv_eval(cfg["X"], cfg["y"], cfg["n_classes"], cfg["fold_idx"], K, sample, dtype=cfg["dtype"], n_threads=cores)
    dt = time.perf_counter() - t0
    return {"value": n_sugg * K * epochs / dt, "unit": "model-epochs/s", "cores": min(cores, n_sugg * K),
            "kind": "oracle",
            "sample": "first %d suggestions x %d folds x %d epoch(s) of the same workload, %.1f s" % (n_sugg, K, epochs, dt)}


def run_workload(idx, steps, warmup, suggestions=0, epochs=0, linear=False):
    import torch
    from paper_2012_04201_amd import binding, inputs
    cfg = inputs.make_config(idx, B=suggestions or None, epochs=epochs or None)
    if linear:  # the same suggestions without their hidden layers: linear / logistic regression
        cfg = dict(cfg, name=cfg["name"] + "_linear", hparams=[dict(h, hidden=[]) for h in cfg["hparams"]])
    flops, model_epochs = inputs.workload_flops(cfg)
    dev = torch.device("cuda:0")
    X, y, ft = binding.to_device(cfg, dev)
    K, c, dt = cfg["n_folds"], cfg["n_classes"], cfg["dtype"]
    hps = cfg["hparams"]
    hp_arr = binding.make_hparams(hps)
    ws = binding.alloc_workspace(binding.bbo_mlp_workspace_bytes(len(cfg["y"]), X.shape[1], c, K, hps, dt, hp_arr), dev)
    stream = torch.cuda.current_stream()

    def step():
        return binding.bbo_mlp_cv_eval(X, y, c, ft, K, hps, dt, workspace=ws, stream=stream, hp_arr=hp_arr)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    # Events are recorded on the stream the kernels are launched on.  One call launches the fold-list
    # kernel, the training kernel and the fold-mean kernel; the first and last take tens of microseconds
    # (see profiles/), so the bracket is the training kernel's duration to better than 0.1 %.
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for a, b in ev:
        a.record(stream)
        scores, status = step()
        b.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_s = sum(a.elapsed_time(b) for a, b in ev) / len(ev) / 1e3
    per_step = wall / steps
    dname = "bf16" if dt else "f32"
    kernel = "k_train_tiled" if dt else ("k_train_linear" if linear else ("k_train_small" if idx in (0, 2, 3) else "k_train_mid"))
    tflops = flops / per_step / 1e12
    abytes = algorithmic_bytes(cfg)
    traffic = measured_traffic(cfg["name"], kernel)
    mfma = {"bound": "mfma", "achieved": flops / kern_s / 1e12, "peak": PEAK_TFLOPS[dname], "unit": "TFLOP/s",
            "frac": flops / kern_s / 1e12 / PEAK_TFLOPS[dname], "traffic": traffic, "kernel": kernel,
            "kernel_ms": kern_s * 1e3}
    if linear:  # no matrix instructions in this kernel: vector multiply-adds fed from LDS
        mfma = {"bound": "alu", "achieved": flops / kern_s / 1e12, "peak": PEAK_VALU_TFLOPS, "unit": "TFLOP/s",
                "frac": flops / kern_s / 1e12 / PEAK_VALU_TFLOPS, "traffic": traffic, "kernel": kernel,
                "kernel_ms": kern_s * 1e3}
    hbm = {"bound": "hbm", "achieved": abytes / kern_s / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
           "frac": abytes / kern_s / 1e9 / PEAK_HBM_GBS, "traffic": traffic, "kernel": kernel,
           "kernel_ms": kern_s * 1e3, "algorithmic_bytes": abytes}
    res = {
        "value": model_epochs / per_step, "ms_per_step": per_step * 1e3, "dtype": dname,
        "config": {"workload": cfg["name"], "mlps": len(hps) * K, "suggestions": len(hps), "folds": K,
                   "rows": int(len(cfg["y"])), "features": int(X.shape[1]), "classes": c,
                   "epochs": hps[0]["epochs"], "reduced": bool(suggestions or epochs)},
        "tflops": tflops, "pct_mfma_peak": 100.0 * tflops / PEAK_TFLOPS[dname],
        "nonfinite_suggestions": int(status.sum().item()),
    }
    return cfg, res, mfma, hbm


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cfg4", choices=["cfg0", "cfg1", "cfg2", "cfg3", "cfg4"])
    ap.add_argument("--suggestions", type=int, default=0, help="debug: evaluate only the first B suggestions")
    ap.add_argument("--epochs", type=int, default=0, help="debug: override the epoch count")
    ap.add_argument("--linear", action="store_true",
                    help="drop the hidden layers of the workload's suggestions (fp32 workloads cfg0..cfg3)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true", help="skip the extra cfg3 measurements")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="BYTES",
                    help="only run a plain device-to-device copy of BYTES (HBM counter calibration)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this evaluator runs on one GPU (items are independent; a multi-GPU run would only "
                 "split the work list); use --gpus 1")

    import torch
    torch.cuda.set_device(0)
    if args.copy_probe:
        a = torch.empty(args.copy_probe, dtype=torch.uint8, device="cuda:0")
        b = torch.ones(args.copy_probe, dtype=torch.uint8, device="cuda:0")
        torch.cuda.synchronize()
        for _ in range(3):
            a.copy_(b)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes": args.copy_probe, "copies": 3}))
        return

    idx = int(args.workload[3])
    if args.linear and idx == 4:
        sys.exit("bench.py: --linear goes with the fp32 workloads cfg0..cfg3")
    cfg, res, mfma, hbm = run_workload(idx, args.steps, args.warmup, args.suggestions, args.epochs, args.linear)
    # The metric is throughput against the dense MFMA peak of the arithmetic type, so that is `roofline`.
    # For cfg4 the optimizer state streams from HBM every step; `roofline_hbm` shows the same kernel
    # against the HBM peak (algorithmic state + input bytes), with the counter-measured traffic beside it.
    out = {
        "metric": "MLP models x epochs/sec for batched CV eval",
        "value": res["value"], "unit": "model-epochs/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": res["dtype"], "data": "synthetic", "config": res["config"],
        "tflops": res["tflops"], "pct_mfma_peak": res["pct_mfma_peak"],
        "nonfinite_suggestions": res["nonfinite_suggestions"],
        "roofline": mfma,
    }
    if idx == 4:
        out["roofline_hbm"] = hbm
    if idx == 4 and not args.no_secondary and not (args.suggestions or args.epochs):
        _, r3, m3, _ = run_workload(3, 3, 1)
        out["secondary"] = {"config": r3["config"], "value": r3["value"], "unit": "model-epochs/s",
                            "ms_per_step": r3["ms_per_step"], "dtype": r3["dtype"], "tflops": r3["tflops"],
                            "roofline": m3}
        _, rl, ml, _ = run_workload(3, 3, 1, linear=True)
        out["secondary_linear"] = {"config": rl["config"], "value": rl["value"], "unit": "model-epochs/s",
                                   "ms_per_step": rl["ms_per_step"], "dtype": rl["dtype"], "tflops": rl["tflops"],
                                   "roofline": ml}
    if idx == 4 and not args.no_secondary and not (args.suggestions or args.epochs):
        # the three 40-model configurations (latency-bound parity workloads), full size, 1 warm-up + 5 calls each
        out["parity_workloads"] = {}
        for i in (0, 1, 2):
            _, r, m, _ = run_workload(i, 5, 1)
            out["parity_workloads"][r["config"]["workload"]] = {
                "ms_per_step": r["ms_per_step"], "value": r["value"], "unit": "model-epochs/s", "dtype": r["dtype"],
                "mlps": r["config"]["mlps"], "epochs": r["config"]["epochs"], "tflops": r["tflops"], "kernel": m["kernel"]}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
