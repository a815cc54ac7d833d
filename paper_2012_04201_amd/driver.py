"""Suggest-evaluate-observe loop over many independent studies (Algorithm 1).

Every study owns an optimizer.  In each of N_STEP iterations every optimizer
suggests N_BATCH hyper-parameter settings; the suggestions of ALL studies go to
the evaluator in ONE call (on the GPU that is one launch that trains
studies x N_BATCH x folds models), and each study's scores are passed back to
its optimizer.  `Ensemble` is the paper's two-optimizer heuristic (Algorithm 1,
right): each member contributes half of the batch and both observe every score.

The optimizers built in here (uniform random search and a shrinking-step local
search) are stand-ins with the suggest/observe interface the paper's third-party
optimizers have; any object with `suggest(n) -> [point]` and
`observe(points, scores)` over the unit cube can be plugged in.

    python -m paper_2012_04201_amd.driver --workload cfg3 --studies 256 --steps 16 --batch 8
"""
import argparse
import json
import time

import numpy as np


class Space:
    """Box of MLP hyper-parameters, addressed through the unit cube.

    Each axis is ("name", "int" | "log", lo, hi); hidden widths are the axes
    "h0", "h1", ...  `decode` turns a point of [0, 1)^D into the dict the
    evaluator takes; everything not on an axis comes from `fixed`."""

    def __init__(self, axes, fixed):
        self.axes = list(axes)
        self.fixed = dict(fixed)

    @property
    def dim(self):
        return len(self.axes)

    def decode(self, u, seed):
        u = np.clip(np.asarray(u, dtype=np.float64), 0.0, np.nextafter(1.0, 0.0))
        hp = dict(self.fixed)
        hidden = {}
        for x, (name, kind, lo, hi) in zip(u, self.axes):
            if kind == "int":
                v = int(lo + np.floor(x * (hi - lo + 1)))
            elif kind == "log":
                v = float(np.exp(np.log(lo) + x * (np.log(hi) - np.log(lo))))
            else:
                raise ValueError(kind)
            if name[0] == "h" and name[1:].isdigit():
                hidden[int(name[1:])] = v
            else:
                hp[name] = v
        if hidden:
            hp["hidden"] = [hidden[i] for i in sorted(hidden)]
        hp["seed"] = int(seed)
        return hp


def workload_space(idx, epochs=None):
    """The search boxes of the five synthetic workloads (the same ranges their fixed suggestion lists are drawn from)."""
    adam = {"solver": "adam", "beta1": 0.9, "beta2": 0.999, "eps": 1e-8, "batch_size": 0}
    if idx == 0:
        return Space([("h0", "int", 8, 32), ("lr", "log", 1e-4, 1e-1), ("alpha", "log", 1e-5, 1e-1)],
                     dict(adam, epochs=epochs or 20))
    if idx == 1:
        return Space([("h0", "int", 50, 200), ("lr", "log", 1e-5, 1e-1), ("alpha", "log", 1e-5, 1e1),
                      ("batch_size", "int", 16, 256)], dict(adam, epochs=epochs or 200))
    if idx == 2:
        return Space([("h0", "int", 50, 200), ("lr", "log", 1e-5, 1e-1), ("alpha", "log", 1e-5, 1e1),
                      ("batch_size", "int", 16, 128), ("momentum", "log", 0.5, 0.99)],
                     {"solver": "sgd", "nesterov": True, "epochs": epochs or 200})
    if idx == 3:
        return Space([("h0", "int", 50, 200), ("lr", "log", 1e-5, 1e-1), ("alpha", "log", 1e-5, 1e1),
                      ("batch_size", "int", 16, 256)], dict(adam, epochs=epochs or 100))
    if idx == 4:
        return Space([("h0", "int", 128, 256), ("h1", "int", 128, 256), ("lr", "log", 1e-4, 1e-2),
                      ("alpha", "log", 1e-5, 1e-1)], dict(adam, batch_size=256, epochs=epochs or 50))
    raise ValueError(idx)


class RandomSearch:
    """Uniform draws from the unit cube; observations are only recorded."""

    def __init__(self, dim, seed):
        self.dim = dim
        self.rng = np.random.default_rng(seed)
        self.points, self.scores = [], []

    def suggest(self, n):
        return [self.rng.random(self.dim) for _ in range(n)]

    def observe(self, points, scores):
        self.points += [np.asarray(p, dtype=np.float64) for p in points]
        self.scores += [float(s) for s in scores]


class LocalSearch(RandomSearch):
    """Gaussian steps around the best point seen so far (by anyone: it observes whatever it is shown), with
    a step size that shrinks as observations accumulate; uniform draws until something finite is known."""

    def __init__(self, dim, seed, sigma0=0.25, shrink=0.97):
        super().__init__(dim, seed)
        self.sigma0, self.shrink = sigma0, shrink

    def suggest(self, n):
        finite = [i for i, s in enumerate(self.scores) if np.isfinite(s)]
        if not finite:
            return super().suggest(n)
        best = self.points[min(finite, key=lambda i: self.scores[i])]
        sigma = self.sigma0 * self.shrink ** len(self.scores)
        return [np.clip(best + sigma * self.rng.standard_normal(self.dim), 0.0, np.nextafter(1.0, 0.0))
                for _ in range(n)]


class Ensemble:
    """Two optimizers share a study (Algorithm 1, right): each suggests half of the batch, and every score
    is passed to both, so each learns from the other's suggestions."""

    def __init__(self, opt_1, opt_2):
        self.opt_1, self.opt_2 = opt_1, opt_2

    def suggest(self, n):
        n1 = n // 2
        return list(self.opt_1.suggest(n1)) + list(self.opt_2.suggest(n - n1))

    def observe(self, points, scores):
        self.opt_1.observe(points, scores)
        self.opt_2.observe(points, scores)


def run_studies(evaluate, space, optimizers, n_step, n_batch, seed=0):
    """Algorithm 1 (left) for len(optimizers) studies at once.

    evaluate(list of hyper-parameter dicts) -> array of scores (lower is better; non-finite = failed run).
    Returns dict(best_score[study], best_hparams[study], history[step][study] = best so far,
    seconds = {"suggest", "evaluate", "observe"})."""
    S = len(optimizers)
    seeds = np.random.default_rng(seed)
    best_score = np.full(S, np.inf)
    best_hp = [None] * S
    history = []
    sec = {"suggest": 0.0, "evaluate": 0.0, "observe": 0.0}
    for _ in range(n_step):
        t0 = time.perf_counter()
        points = [opt.suggest(n_batch) for opt in optimizers]
        hps = [space.decode(p, seeds.integers(0, 2 ** 63)) for study in points for p in study]
        t1 = time.perf_counter()
        scores = np.asarray(evaluate(hps), dtype=np.float64).reshape(S, n_batch)
        t2 = time.perf_counter()
        for s, opt in enumerate(optimizers):
            sc = np.where(np.isfinite(scores[s]), scores[s], np.inf)
            opt.observe(points[s], sc)
            j = int(np.argmin(sc))
            if sc[j] < best_score[s]:
                best_score[s] = sc[j]
                best_hp[s] = hps[s * n_batch + j]
        history.append(best_score.copy())
        t3 = time.perf_counter()
        sec["suggest"] += t1 - t0
        sec["evaluate"] += t2 - t1
        sec["observe"] += t3 - t2
    return {"best_score": best_score, "best_hparams": best_hp, "history": history, "seconds": sec}


def gpu_evaluator(cfg, device="cuda:0"):
    """evaluate() backed by the HIP library: the cross-validation score (first metric) of every suggestion,
    inputs resident on the device, one library call per iteration."""
    import torch
    from . import binding
    X, y, ft = binding.to_device(cfg, torch.device(device))
    K, c, dt = cfg["n_folds"], cfg["n_classes"], cfg["dtype"]

    def evaluate(hps):
        scores, status = binding.bbo_mlp_cv_eval(X, y, c, ft, K, hps, dt)
        return scores[:, 0].cpu().numpy()

    return evaluate


def main():
    from . import inputs
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="cfg3", choices=["cfg0", "cfg1", "cfg2", "cfg3", "cfg4"])
    ap.add_argument("--studies", type=int, default=256)
    ap.add_argument("--steps", type=int, default=16)
    ap.add_argument("--batch", type=int, default=8)
    ap.add_argument("--epochs", type=int, default=0)
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    idx = int(args.workload[3])
    cfg = inputs.make_config(idx, B=1)
    space = workload_space(idx, args.epochs or None)
    kinds = ["random", "local", "ensemble"]
    opts = []
    for s in range(args.studies):
        k = kinds[s % 3]
        a, b = RandomSearch(space.dim, 2 * s + 1 + args.seed), LocalSearch(space.dim, 2 * s + 2 + args.seed)
        opts.append(a if k == "random" else b if k == "local" else Ensemble(a, b))
    res = run_studies(gpu_evaluator(cfg), space, opts, args.steps, args.batch, args.seed)
    by_kind = {k: float(np.mean([res["best_score"][s] for s in range(args.studies) if kinds[s % 3] == k and
                                 np.isfinite(res["best_score"][s])] or [np.nan])) for k in kinds}
    print(json.dumps({"workload": cfg["name"], "studies": args.studies, "steps": args.steps, "batch": args.batch,
                      "models_trained": args.studies * args.steps * args.batch * cfg["n_folds"],
                      "seconds": res["seconds"], "mean_best_cv_score": by_kind}))


if __name__ == "__main__":
    main()
