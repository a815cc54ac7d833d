"""The recorded oracle scores (tests/golden/stated_epoch_scores.json) belong to the inputs and to the oracle as
they are now: the fingerprints match, the record covers the suggestions its script names, and the cheap
configurations are reproduced bit for bit by running the oracle again (CPU only)."""
import importlib.util
import json
import os

import numpy as np
import pytest

from paper_2012_04201_amd import inputs

HERE = os.path.dirname(os.path.abspath(__file__))


def script():
    spec = importlib.util.spec_from_file_location("make_stated_epoch_scores",
                                                  os.path.join(HERE, "golden", "make_stated_epoch_scores.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


@pytest.mark.parametrize("idx", [0, 1, 2, 3, 4])
def test_record_belongs_to_the_inputs(idx):
    mod = script()
    rec = json.load(open(os.path.join(HERE, "golden", "stated_epoch_scores.json")))["cfg%d" % idx]
    cfg = inputs.make_config(idx)
    assert rec["picks"] == mod.PICKS[idx]
    assert rec["digest"] == mod.inputs_digest(cfg, rec["picks"])
    assert rec["rows"] == len(cfg["y"]) and rec["epochs"] == cfg["hparams"][0]["epochs"]
    n = len(rec["picks"])
    assert len(rec["scores"]) == len(rec["status"]) == len(rec["noise"]) == len(rec["per_fold"]) == n
    assert sorted(rec["noise_by_probe"]) == ["fp32_sums", "fp64_state", "lr_down", "lr_up"]


@pytest.mark.parametrize("idx,sample", [(0, None), (3, [0, 1, 2])])
def test_record_is_what_the_oracle_computes_now(oracle, idx, sample):
    rec = json.load(open(os.path.join(HERE, "golden", "stated_epoch_scores.json")))["cfg%d" % idx]
    cfg = inputs.make_config(idx)
    at = list(range(len(rec["picks"]))) if sample is None else sample
    hps = [cfg["hparams"][rec["picks"][i]] for i in at]
    rs, rst, rpf = oracle.cv_eval(cfg["X"], cfg["y"], cfg["n_classes"], cfg["fold_idx"], cfg["n_folds"], hps, dtype=cfg["dtype"])
    want = np.array([[np.nan if v is None else v for v in rec["scores"][i]] for i in at])
    assert np.array_equal(rs.astype(np.float64), want, equal_nan=True)
    assert rst.tolist() == [rec["status"][i] for i in at]
    wpf = np.array([[[np.nan if v is None else v for v in f] for f in rec["per_fold"][i]] for i in at])
    assert np.array_equal(rpf, wpf, equal_nan=True)
