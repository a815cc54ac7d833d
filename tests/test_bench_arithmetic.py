"""The benchmark's own arithmetic, without a GPU: algorithmic FLOPs and bytes of the workloads written out by hand for
small cases and compared with the figures the workloads are specified with; the kernel-source fingerprint that
gates the recorded counter traffic; the refusal of more than one GPU."""
import os
import subprocess
import sys

import numpy as np

import bench
from paper_2012_04201_amd import inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_flops_per_sample_is_two_passes_for_the_first_layer_and_three_for_the_others():
    # forward + weight gradient for every layer, data gradient for every layer but the first
    assert inputs.flops_per_sample(30, [100], 2) == 2 * (2 * 30 * 100) + 3 * (2 * 100 * 2)
    assert inputs.flops_per_sample(128, [256, 128], 10) == 2 * (2 * 128 * 256) + 3 * (2 * 256 * 128) + 3 * (2 * 128 * 10)
    assert inputs.flops_per_sample(30, [], 2) == 2 * (2 * 30 * 2)


def test_workload_totals_match_the_stated_sizes():
    cfg = inputs.make_config(3)
    total, model_epochs = inputs.workload_flops(cfg)
    assert model_epochs == 2048 * 5 * 100
    assert 7.0e12 < total < 8.4e12          # 7.7 TFLOP for 10,240 models of 50..200 hidden units
    cfg = inputs.make_config(4)
    total, model_epochs = inputs.workload_flops(cfg)
    assert model_epochs == 1640 * 5 * 50
    assert 2.0e15 < total < 2.35e15         # 2.17 PFLOP for 8,200 two-hidden-layer models
    # bytes: 24 B per parameter-step (three fp32 arrays read and written) + the input rows of every epoch
    b = bench.algorithmic_bytes(cfg)
    P = np.mean([128 * h["hidden"][0] + h["hidden"][0] + h["hidden"][0] * h["hidden"][1] + h["hidden"][1] + h["hidden"][1] * 10 + 10
                 for h in cfg["hparams"]])
    steps = -(-16000 // 256)
    want = 8200 * (50 * (steps * 24 * P + 16000 * 128 * 2) + 4000 * 128 * 2)
    assert abs(b - want) / want < 1e-9
    assert 40 < total / b < 60              # ~53 FLOP per byte: far left of the bf16 ridge of 312


def test_algorithmic_bytes_of_a_hand_sized_case():
    cfg = {"X": np.zeros((10, 3), dtype=np.float32), "fold_idx": np.array([0, 1] * 5, dtype=np.int32), "n_folds": 2, "dtype": 0,
           "n_classes": 0, "hparams": [{"hidden": [4], "batch_size": 2, "epochs": 3, "solver": "sgd"}]}
    P = 3 * 4 + 4 + 4 + 1
    per_fold = 3 * (3 * 16 * P + 5 * 3 * 4) + 5 * 3 * 4   # 5 training rows -> 3 steps; SGD: weights and one moment
    assert bench.algorithmic_bytes(cfg) == 2 * per_fold


def test_kernel_fingerprint_ignores_comments_only(tmp_path, monkeypatch):
    src = os.path.join(ROOT, "paper_2012_04201_amd", "csrc")
    work = tmp_path / "paper_2012_04201_amd" / "csrc"
    work.mkdir(parents=True)
    for name in ("common.h", "train_small_f32.h"):
        (work / name).write_text(open(os.path.join(src, name)).read())
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    h0 = bench.kernel_source_hash("k_train_small")
    p = work / "train_small_f32.h"
    text = p.read_text()
    p.write_text("// a new remark\n" + text.replace("namespace {", "namespace {  /* another */\n\n", 1))
    assert bench.kernel_source_hash("k_train_small") == h0
    p.write_text(text.replace("SM_RC = 64", "SM_RC = 32", 1))
    assert bench.kernel_source_hash("k_train_small") != h0


def test_more_than_one_gpu_is_refused_before_anything_runs():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)
