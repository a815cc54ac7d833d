"""The suggest-evaluate-observe loop (Algorithm 1): protocol checks with a stub evaluator on the CPU, and one
small end-to-end run through the HIP library whose winners are re-scored by the oracle."""
import numpy as np
import pytest

from paper_2012_04201_amd import driver, inputs


class Recorder:
    """Optimizer that suggests labelled points and records what it is shown."""

    def __init__(self, tag):
        self.tag, self.calls, self.seen = tag, [], []

    def suggest(self, n):
        self.calls.append(n)
        return [np.full(3, (self.tag + 0.01 * i + 0.1 * len(self.calls)) % 1.0) for i in range(n)]

    def observe(self, points, scores):
        self.seen.append((len(points), list(np.round(scores, 6))))


def bowl(hps):
    """A smooth stand-in for the model-evaluation call: lowest near lr = 1e-2, alpha = 1e-3, width 20."""
    return np.array([(np.log10(h["lr"]) + 2) ** 2 + 0.3 * (np.log10(h["alpha"]) + 3) ** 2 + 1e-3 * (h["hidden"][0] - 20) ** 2
                     for h in hps])


def test_space_decodes_the_unit_cube_into_the_box():
    sp = driver.workload_space(2)
    lo = sp.decode(np.zeros(sp.dim), 1)
    hi = sp.decode(np.full(sp.dim, 1.0), 2)
    assert lo["hidden"] == [50] and hi["hidden"] == [200]
    assert abs(lo["lr"] - 1e-5) < 1e-12 and abs(hi["lr"] - 1e-1) < 1e-6
    assert lo["batch_size"] == 16 and hi["batch_size"] == 128
    assert lo["solver"] == "sgd" and lo["nesterov"] is True and lo["seed"] == 1 and hi["seed"] == 2
    assert len(driver.workload_space(4).decode(np.full(4, 0.5), 0)["hidden"]) == 2


def test_ensemble_takes_half_from_each_member_and_shows_both_every_score():
    a, b = Recorder(0.2), Recorder(0.7)
    ens = driver.Ensemble(a, b)
    pts = ens.suggest(7)
    assert a.calls == [3] and b.calls == [4] and len(pts) == 7
    ens.observe(pts, np.arange(7.0))
    assert a.seen == b.seen == [(7, [0, 1, 2, 3, 4, 5, 6])]


def test_all_studies_share_one_evaluation_call_and_get_their_own_scores_back():
    sp = driver.workload_space(0, epochs=3)
    calls = []

    def ev(hps):
        calls.append(len(hps))
        return bowl(hps)

    mk = lambda: [driver.RandomSearch(sp.dim, 1), driver.LocalSearch(sp.dim, 2),
                  driver.Ensemble(driver.RandomSearch(sp.dim, 3), driver.LocalSearch(sp.dim, 4))]
    res = driver.run_studies(ev, sp, mk(), n_step=5, n_batch=6, seed=9)
    assert calls == [18] * 5
    # every study ends where it would have ended alone (scores are routed to their own optimizer)
    for s in range(3):
        alone = driver.run_studies(bowl, sp, [mk()[s]], n_step=5, n_batch=6, seed=9)
        hp_a, hp_b = dict(alone["best_hparams"][0]), dict(res["best_hparams"][s])
        hp_a.pop("seed"), hp_b.pop("seed")  # per-model seeds are drawn per call position
        assert hp_a == hp_b and alone["best_score"][0] == res["best_score"][s]
    # same seeds, same run; the best-so-far never gets worse
    again = driver.run_studies(bowl, sp, mk(), n_step=5, n_batch=6, seed=9)
    assert np.array_equal(again["best_score"], res["best_score"])
    h = np.array(res["history"])
    assert np.all(np.diff(h, axis=0) <= 0)
    assert set(res["seconds"]) == {"suggest", "evaluate", "observe"}


def test_local_search_uses_what_the_ensemble_partner_found():
    sp = driver.workload_space(0)
    loc = driver.LocalSearch(sp.dim, 5, sigma0=0.05)
    target = np.array([0.5, 0.66, 0.5])
    loc.observe([target, np.zeros(3)], [0.1, 9.0])
    pts = np.array(loc.suggest(64))
    assert np.abs(pts - target).max() < 0.3 and np.abs(pts.mean(0) - target).max() < 0.05


def test_failed_runs_count_as_worst():
    sp = driver.workload_space(0)

    def ev(hps):
        s = bowl(hps)
        s[::2] = np.nan
        return s

    res = driver.run_studies(ev, sp, [driver.RandomSearch(sp.dim, 1)], n_step=2, n_batch=4, seed=0)
    assert np.isfinite(res["best_score"][0])


@pytest.mark.gpu
def test_end_to_end_on_the_gpu_matches_the_oracle(oracle):
    cfg = inputs.make_config(0, B=1)
    sp = driver.workload_space(0, epochs=6)
    opts = [driver.RandomSearch(sp.dim, 1), driver.LocalSearch(sp.dim, 2),
            driver.Ensemble(driver.RandomSearch(sp.dim, 3), driver.LocalSearch(sp.dim, 4))]
    res = driver.run_studies(driver.gpu_evaluator(cfg), sp, opts, n_step=3, n_batch=4, seed=1)
    assert np.all(np.isfinite(res["best_score"]))
    ref, st, _ = oracle.cv_eval(cfg["X"], cfg["y"], 3, cfg["fold_idx"], 5, res["best_hparams"])
    assert np.all(st == 0) and np.abs(ref[:, 0] - res["best_score"]).max() < 1e-3
