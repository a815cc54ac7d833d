"""The allocation-free entry point (static workspace inside the library) against the entry point that takes
a caller's workspace: same kernels, so the scores must be bit-identical.  Two calls in a row on the one
static array, the second with a smaller input, so that leftovers of the first call would show."""
import numpy as np
import pytest
import torch

from paper_2012_04201_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bb():
    from paper_2012_04201_amd import binding
    binding.lib()
    return binding


def both_ways(bb, cfg):
    X, y, ft = bb.to_device(cfg)
    K, c, dt, hps = cfg["n_folds"], cfg["n_classes"], cfg["dtype"], cfg["hparams"]
    B = len(hps)
    want_s, want_st, want_pf = bb.bbo_mlp_cv_eval(X, y, c, ft, K, hps, dt, want_per_fold=True)
    torch.cuda.synchronize()
    # outputs allocated by the caller, ahead of the call
    scores = torch.full((B, 2), -7.0, dtype=torch.float32, device=X.device)
    status = torch.full((B,), -7, dtype=torch.int32, device=X.device)
    pf = torch.full((B, K, 2), -7.0, dtype=torch.float32, device=X.device)
    torch.cuda.synchronize()
    # torch's count of device allocations made so far: the call must not add to it (the library itself has no
    # way to allocate through torch; this guards the binding)
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    bb.bbo_mlp_cv_eval_static(X, y, c, ft, K, hps, dt, scores=scores, status=status, per_fold=pf)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
    assert torch.equal(scores, want_s) and torch.equal(status, want_st) and torch.equal(pf, want_pf)
    assert np.all(np.isfinite(scores.cpu().numpy()[status.cpu().numpy() == 0]))
    return scores


def test_static_workspace_entry_matches_twice_the_second_call_smaller(bb, oracle):
    # first call: the regression workload (SGD, 40 models with a hidden layer: LDS-resident kernel with its
    # per-workgroup slots in the workspace) plus models without a hidden layer (wavefront-per-model kernel)
    big = inputs.make_config(2, epochs=6)
    big["hparams"] = big["hparams"] + [dict(h, hidden=[]) for h in big["hparams"][:3]]
    both_ways(bb, big)
    # second call, smaller in every respect: fewer rows, fewer and narrower models, other kernel shapes
    small = inputs.make_config(0, B=3, epochs=5)
    s = both_ways(bb, small)
    # and the result is the right one, not merely the same one
    rs, rst, _ = oracle.cv_eval(small["X"], small["y"], small["n_classes"], small["fold_idx"], small["n_folds"],
                                small["hparams"])
    assert np.abs(s.cpu().numpy()[:, 0] - rs[:, 0]).max() < 1e-3
    # a bf16 call (LDS-tiled kernel, 2 MB slot per workgroup) fits the static array too when it is small
    tiny4 = inputs.make_config(4, B=1, epochs=1, n=600)
    both_ways(bb, tiny4)


def test_static_workspace_entry_refuses_what_does_not_fit(bb):
    cfg = inputs.make_config(4, B=64, epochs=1, n=600)  # 256 workgroup slots of ~2 MB
    X, y, ft = bb.to_device(cfg)
    with pytest.raises(bb.BboError) as e:
        bb.bbo_mlp_cv_eval_static(X, y, cfg["n_classes"], ft, cfg["n_folds"], cfg["hparams"], cfg["dtype"])
    assert e.value.code == bb.WORKSPACE_TOO_SMALL and "allocation-free" in str(e.value)
    # the library still works afterwards
    ok = inputs.make_config(0, B=2, epochs=2)
    both_ways(bb, ok)
