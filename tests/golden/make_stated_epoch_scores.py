#!/usr/bin/env python3
"""Writes tests/golden/stated_epoch_scores.json: the ORACLE's final cross-validation scores of the benchmark
configurations at their stated sizes and epoch counts, for the suggestions the GPU tests compare.

Calls only the CPU oracle (oracle/) and the seeded input generators.  Nothing here comes from the GPU
library.  The scores themselves have no published value (the paper prints none for single models): the
file holds the oracle's own results so that the GPU machine need not spend its minutes recomputing them.

Per suggestion it records the per-fold scores, the status flag, and the run's sensitivity ("noise"): the
largest change of a fold's first score when the same run is repeated (a) without any fp32 rounding of the
state, (b, c) with the learning rate moved by one fp32 ulp up / down, (d) with fp32 running sums in the
contractions (the level at which a single-precision accumulator differs).

    python tests/golden/make_stated_epoch_scores.py [--threads N] [--only cfg4]
"""
import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import mlp_cv_oracle as O  # noqa: E402
from paper_2012_04201_amd import inputs  # noqa: E402

OUT = os.path.join(HERE, "stated_epoch_scores.json")

# configuration index -> which suggestions of the full-size configuration are recorded
PICKS = {
    0: list(range(8)),
    1: list(range(8)),
    2: list(range(8)),
    3: [0, 1, 255, 256, 777, 1024, 1500, 2047, 100, 333, 512, 640, 900, 1111, 1300, 1400, 1601, 1700, 1800, 1900,
        1999, 2000, 2020, 2040],
    4: [0, 205, 410, 819, 1024, 1230, 1435, 1639],
}


def inputs_digest(cfg, picks):
    """Fingerprint of everything the recorded scores depend on: data, folds and the picked suggestions."""
    h = hashlib.sha256()
    h.update(np.ascontiguousarray(cfg["X"]).tobytes())
    h.update(np.ascontiguousarray(cfg["y"]).tobytes())
    h.update(np.ascontiguousarray(cfg["fold_idx"], dtype=np.int32).tobytes())
    h.update(json.dumps([cfg["hparams"][i] for i in picks], sort_keys=True).encode())
    return h.hexdigest()[:24]


def probes(hps):
    yield "fp64_state", hps, 1
    for name, toward in (("lr_up", np.float32(1e9)), ("lr_down", np.float32(0))):
        yield name, [dict(h, lr=float(np.nextafter(np.float32(h["lr"]), toward))) for h in hps], 0
    yield "fp32_sums", hps, 2


def record(idx, threads):
    cfg = inputs.make_config(idx)
    picks = PICKS[idx]
    hps = [cfg["hparams"][i] for i in picks]
    K, c, dt = cfg["n_folds"], cfg["n_classes"], cfg["dtype"]
    run = lambda h, prec: O.cv_eval(cfg["X"], cfg["y"], c, cfg["fold_idx"], K, h, dtype=dt, prec=prec, n_threads=threads)
    t0 = time.time()
    rs, rst, rpf = run(hps, 0)
    print("%s: base run %.0f s" % (cfg["name"], time.time() - t0), flush=True)
    noise = np.zeros(len(hps))
    per_probe = {}
    for name, h, prec in probes(hps):
        t0 = time.time()
        q = run(h, prec)[2]
        dev = np.array([np.abs(rpf[b, :, 0] - q[b, :, 0]).max() if np.all(np.isfinite(q[b])) and np.all(np.isfinite(rpf[b]))
                        else np.inf for b in range(len(hps))])
        per_probe[name] = [float(x) if np.isfinite(x) else None for x in dev]
        noise = np.maximum(noise, dev)
        print("%s: probe %s %.0f s" % (cfg["name"], name, time.time() - t0), flush=True)
    return {
        "name": cfg["name"], "picks": picks, "digest": inputs_digest(cfg, picks),
        "epochs": hps[0]["epochs"], "rows": int(len(cfg["y"])),
        "status": [int(x) for x in rst],
        "scores": [[float(v) if np.isfinite(v) else None for v in row] for row in rs],
        "per_fold": [[[float(v) if np.isfinite(v) else None for v in f] for f in b] for b in rpf],
        "noise": [float(x) if np.isfinite(x) else None for x in noise],
        "noise_by_probe": per_probe,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--threads", type=int, default=len(os.sched_getaffinity(0)))
    ap.add_argument("--only", default="", help="comma-separated configuration names to (re)compute, e.g. cfg4,cfg1")
    args = ap.parse_args()
    data = json.load(open(OUT)) if os.path.exists(OUT) else {}
    todo = [int(s[3]) for s in args.only.split(",") if s] or sorted(PICKS)
    for idx in todo:
        data["cfg%d" % idx] = record(idx, args.threads)
        with open(OUT, "w") as fh:
            json.dump(data, fh, indent=1, sort_keys=True)
            fh.write("\n")
    print("wrote", OUT)


if __name__ == "__main__":
    main()
