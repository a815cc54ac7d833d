"""Pins for the CPU oracle: each checks it against something other than itself
(published vectors, closed forms, library autograd/optimizers, invariants,
brute force), so that a dropped term, a wrong sign or index, or a transposed
operand in the oracle fails at least one of them."""
import os

import numpy as np
import pytest
import torch

from paper_2012_04201_amd import inputs

GOLD = os.path.join(os.path.dirname(__file__), "golden")
G = 0x9E3779B97F4A7C15
M64 = 2**64 - 1


def tiny_problem(seed, n=40, d=4, n_classes=3):
    rng = np.random.default_rng(seed)
    X = rng.normal(size=(n, d)).astype(np.float32)
    if n_classes >= 1:  # 1: labels 0/1 for the single-logit binary head
        y = rng.integers(0, max(n_classes, 2), size=n).astype(np.int32)
    else:
        y = (X[:, 0] - 0.5 * X[:, 1] + 0.1 * rng.normal(size=n)).astype(np.float32)
    return X, y


def unpack(theta, dims):
    """Packed parameters -> [(W[in,out], b[out])] following the oracle's layout."""
    out, off = [], 0
    for l in range(len(dims) - 1):
        fi, fo = dims[l], dims[l + 1]
        W = theta[off:off + fi * fo].reshape(fi, fo)
        off += fi * fo
        b = theta[off:off + fo]
        off += fo
        out.append((W, b))
    assert off == theta.shape[0]
    return out


def torch_loss(theta_t, dims, Xb, yb, n_classes, alpha):
    """Library definition of the training objective (float64, autograd-able)."""
    off, a = 0, Xb
    pen = 0.0
    L = len(dims) - 1
    for l in range(L):
        fi, fo = dims[l], dims[l + 1]
        W = theta_t[off:off + fi * fo].reshape(fi, fo)
        off += fi * fo
        b = theta_t[off:off + fo]
        off += fo
        a = a @ W + b
        if l + 1 < L:
            a = torch.relu(a)
        pen = pen + (W * W).sum()
    m = Xb.shape[0]
    if n_classes >= 2:
        data = torch.nn.functional.cross_entropy(a, yb, reduction="mean")
    elif n_classes == 1:
        data = torch.nn.functional.binary_cross_entropy_with_logits(a[:, 0], yb.to(torch.float64), reduction="mean")
    else:
        data = 0.5 * torch.nn.functional.mse_loss(a[:, 0], yb, reduction="mean")
    return data + 0.5 * alpha * pen / m


# ------------------------------------------------------------ RNG pins ----

def test_mix64_published_vectors(oracle):
    want = [int(l, 16) for l in open(os.path.join(GOLD, "splitmix64_kat.txt")) if l.startswith("0x")]
    got = [oracle.mix64((k * G) & M64) for k in (1, 2, 3)]
    assert got == want
    # combine(h, v) is the SplitMix64 stream started at h read at position v
    assert [oracle.combine(0, v) for v in range(3)] == want


@pytest.mark.parametrize("n", list(range(1, 130)) + [255, 256, 257, 405, 455, 1023, 1024, 1025, 1438, 2048, 4097,
                                                      16000, 20000])
def test_permutation_is_bijection(oracle, n):
    p = oracle.permutation(12345, 2, 7, n)
    assert p.min() == 0 and p.max() == n - 1
    assert np.array_equal(np.sort(p), np.arange(n))


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 15, 16, 17, 63, 64, 65, 255, 256, 257, 1023, 1024, 1025, 4096, 4097])
def test_permutation_network_width_at_powers_of_two(oracle, n):
    """The network works on the smallest even number of bits (at least 2) that holds n - 1: at a power of two
    no position is walked twice, one past it the width grows.  Checked against the network in plain integers."""
    kep = py_fold(py_fold(py_fold(py_fold(77, 0x4D4C50), 3), 1), 6)
    ps = range(n) if n <= 300 else list(range(0, n, 37)) + [n - 1]
    assert [oracle.perm_index(77, 3, 6, n, p) for p in ps] == [py_perm(kep, n, p) for p in ps]


def test_permutation_depends_on_key_and_mixes(oracle):
    n = 1000
    a = oracle.permutation(1, 0, 0, n)
    assert not np.array_equal(a, oracle.permutation(1, 0, 1, n))  # epoch
    assert not np.array_equal(a, oracle.permutation(1, 1, 0, n))  # fold
    assert not np.array_equal(a, oracle.permutation(2, 0, 0, n))  # seed
    # no structure a sorted or shifted order would leave: displacement statistics of a random permutation
    disp = np.abs(a - np.arange(n)).mean()
    assert 0.25 * n < disp < 0.42 * n  # E|i - pi(i)| = n/3
    assert (a == np.arange(n)).sum() < 8  # fixed points ~ Poisson(1)


def test_fold_lists_partition_rows(oracle):
    rng = np.random.default_rng(0)
    fold = rng.integers(-1, 5, size=501).astype(np.int32)
    for f in range(5):
        tr, va = oracle.fold_lists(fold, f)
        assert np.array_equal(va, np.nonzero(fold == f)[0])
        assert np.array_equal(tr, np.nonzero((fold >= 0) & (fold != f))[0])
    # the hold-out split (f = -1): rows of every fold train, rows of none are scored
    tr, va = oracle.fold_lists(fold, -1)
    assert np.array_equal(tr, np.nonzero(fold >= 0)[0]) and np.array_equal(va, np.nonzero(fold < 0)[0])


def test_minibatches_cover_train_rows_once_per_epoch(oracle):
    fold = inputs.make_folds(103, 5, 9)
    hp = {"hidden": [3], "batch_size": 16, "seed": 77, "epochs": 2}
    fold[[5, 50, 77]] = -1
    for f in (0, 3, -1):
        tr, _ = oracle.fold_lists(fold, f)
        for ep in (0, 1):
            steps = -(-len(tr) // 16)
            got = [oracle.minibatch_rows(fold, hp, f, ep, s) for s in range(steps)]
            assert all(len(g) == 16 for g in got[:-1]) and len(got[-1]) == len(tr) - 16 * (steps - 1)
            assert np.array_equal(np.sort(np.concatenate(got)), tr)
            perm = oracle.permutation(77, f, ep, len(tr))
            assert np.array_equal(np.concatenate(got), tr[perm])
    # batch_size 0 or larger than the fold => one full batch
    for bs in (0, 1000):
        hp2 = dict(hp, batch_size=bs)
        tr, _ = oracle.fold_lists(fold, 1)
        assert len(oracle.minibatch_rows(fold, hp2, 1, 0, 0)) == len(tr)


def test_init_tensors_draw_from_streams_of_their_own(oracle):
    """Divided by its layer's bound every tensor is a sequence of centred 24-bit draws; no tensor repeats the
    draws of another one (a shared or shifted key would), and none is correlated with another."""
    hp = {"hidden": [40, 40, 40], "seed": 9}
    d, c = 40, 40
    dims = [d, 40, 40, 40, c]
    th = oracle.init_params(d, c, hp, 0)
    assert th.shape[0] == oracle.param_count(d, c, hp) == sum(fi * fo + fo for fi, fo in zip(dims[:-1], dims[1:]))
    draws = []
    for (W, b), fi, fo in zip(unpack(th, dims), dims[:-1], dims[1:]):
        bound = float(np.float32(np.sqrt(6.0 / (fi + fo))))
        draws += [W.ravel() / bound, b / bound]
    for i, a in enumerate(draws):
        k = np.round(a * 2**23)
        assert np.abs(a * 2**23 - k).max() < 1.0  # a 24-bit draw times a bound, rounded once to fp32
        for b in draws[i + 1:]:
            m = min(a.size, b.size)
            assert np.abs(a[:m] - b[:m]).max() > 0.5          # not the same draws
            assert abs(np.corrcoef(a[:m], b[:m])[0, 1]) < 5 / np.sqrt(m)


def test_shapes_at_the_limits_are_taken(oracle):
    """Four hidden layers and a hidden layer of one unit are legal; five layers or a width of zero are not."""
    assert oracle.param_count(4, 3, {"hidden": [3, 1, 2, 4]}) == 4 * 3 + 3 + 3 * 1 + 1 + 1 * 2 + 2 + 2 * 4 + 4 + 4 * 3 + 3
    assert oracle.param_count(4, 0, {"hidden": [1]}) == 4 + 1 + 1 + 1
    import ctypes as C
    hp = oracle.make_hparams([{"hidden": [3]}])
    hp[0].n_hidden = 5
    assert oracle.lib().oracle_param_count(C.c_int32(4), C.c_int32(3), hp) < 0
    hp[0].n_hidden, hp[0].hidden[0] = 1, 0
    assert oracle.lib().oracle_param_count(C.c_int32(4), C.c_int32(3), hp) < 0


def test_init_glorot_bounds_and_moments(oracle):
    hp = {"hidden": [200, 150], "seed": 42}
    d, c = 64, 10
    th = oracle.init_params(d, c, hp, 1)
    dims = [d, 200, 150, c]
    for (W, b), fi, fo in zip(unpack(th, dims), dims[:-1], dims[1:]):
        bound = float(np.float32(np.sqrt(6.0 / (fi + fo))))
        for t in (W, b):
            assert np.all(np.abs(t) <= bound)
            assert np.array_equal(t, t.astype(np.float32).astype(np.float64))  # fp32 values
        assert abs(W.mean()) < 4 * bound / np.sqrt(3 * W.size)
        assert abs(W.var() / (bound**2 / 3) - 1) < 0.05
    # different fold / seed / layer streams are different
    assert not np.array_equal(th, oracle.init_params(d, c, hp, 2))
    assert not np.array_equal(th, oracle.init_params(d, c, dict(hp, seed=43), 1))
    # the draw is the top 24 bits of the element hash, centred: check one element by hand
    km = oracle.combine(oracle.combine(42, 0x4D4C50), 1)
    kt = oracle.combine(km, 16 + 2 * 0 + 0)
    k24 = oracle.combine(kt, 5) >> 40
    bound = np.float32(np.sqrt(6.0 / (64 + 200)))
    assert th[5] == float(np.float32(float(bound) * ((k24 - 2**23) / 2**23)))


def test_bf16_rounding_matches_library(oracle):
    rng = np.random.default_rng(1)
    bits = np.concatenate([
        rng.integers(0, 2**32, size=200000, dtype=np.uint64).astype(np.uint32),
        # ties, just-above/below ties, for many upper halves
        (np.arange(0, 2**16, 7, dtype=np.uint32) << 16) | 0x8000,
        (np.arange(0, 2**16, 7, dtype=np.uint32) << 16) | 0x8001,
        (np.arange(0, 2**16, 7, dtype=np.uint32) << 16) | 0x7FFF,
        np.array([0, 0x80000000, 0x7F800000, 0xFF800000, 0x00000001, 0x00008000, 0x7F7FFFFF], dtype=np.uint32),
    ])
    f = bits.view(np.float32)
    want = torch.from_numpy(f.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got_gen = inputs.to_bf16_bits(f)
    lib = oracle.lib().oracle_bf16_bits
    import ctypes as C
    sel = np.concatenate([np.arange(0, 200000, 37), np.arange(200000, bits.shape[0])])
    nan = np.isnan(f)
    for i in sel:
        g = lib(C.c_float(f[i]))
        if nan[i]:
            assert (g & 0x7F80) == 0x7F80 and (g & 0x7F) != 0
        else:
            assert g == want[i], hex(int(bits[i]))
    assert np.array_equal(got_gen[~nan], want[~nan])


# ----------------------------------------------- forward/backward pins ----

CASES = [
    # (n_classes, hidden, alpha)
    (3, [5], 0.3),
    (2, [4], 0.0),
    (3, [], 0.7),
    (0, [5], 0.2),
    (0, [], 0.0),
    (4, [5, 3], 0.5),
    (0, [4, 4, 3], 0.1),
    (1, [5], 0.3),      # single-logit binary head
    (1, [], 0.0),
    (1, [4, 3], 0.6),
    (3, [3, 1, 2, 4], 0.2),   # the maximum depth, with a hidden layer one unit wide
]


@pytest.mark.parametrize("n_classes,hidden,alpha", CASES)
def test_gradient_matches_autograd_and_finite_differences(oracle, n_classes, hidden, alpha):
    X, y = tiny_problem(3, n=23, d=4, n_classes=n_classes)
    hp = {"hidden": hidden, "alpha": alpha, "seed": 5}
    dims = [4] + hidden + [n_classes if n_classes >= 2 else 1]
    rng = np.random.default_rng(8)
    theta = oracle.init_params(4, n_classes, hp, 0) + 0.3 * rng.normal(size=oracle.param_count(4, n_classes, hp))
    rows = np.array([3, 17, 5, 8, 21, 0, 11], dtype=np.int32)
    loss, grad = oracle.loss_grad(X, y, n_classes, rows, hp, theta, prec=1)

    # library autograd on the textbook objective
    tt = torch.tensor(theta, dtype=torch.float64, requires_grad=True)
    Xb = torch.tensor(X[rows], dtype=torch.float64)
    yb = torch.tensor(y[rows].astype(np.int64)) if n_classes >= 1 else torch.tensor(y[rows], dtype=torch.float64)
    tl = torch_loss(tt, dims, Xb, yb, n_classes, float(np.float32(alpha)))
    tl.backward()
    assert abs(loss - tl.item()) < 1e-12 * max(1, abs(loss))
    np.testing.assert_allclose(grad, tt.grad.numpy(), rtol=1e-10, atol=1e-13)

    # central finite differences of the oracle's own loss
    eps = 1e-6
    fd = np.zeros_like(theta)
    for i in range(theta.shape[0]):
        tp, tm = theta.copy(), theta.copy()
        tp[i] += eps
        tm[i] -= eps
        fd[i] = (oracle.loss_grad(X, y, n_classes, rows, hp, tp, prec=1)[0]
                 - oracle.loss_grad(X, y, n_classes, rows, hp, tm, prec=1)[0]) / (2 * eps)
    assert np.linalg.norm(fd - grad) / np.linalg.norm(grad) < 1e-6


def test_softmax_gradient_invariants_and_binary_equals_logistic(oracle):
    X, y = tiny_problem(4, n=30, d=4, n_classes=2)
    hp = {"hidden": [6], "alpha": 0.0, "seed": 1}
    theta = oracle.init_params(4, 2, hp, 0)
    rows = np.arange(12, dtype=np.int32)
    loss, grad = oracle.loss_grad(X, y, 2, rows, hp, theta, prec=1)
    (W1, b1), (W2, b2) = unpack(theta, [4, 6, 2])
    gb2 = unpack(grad, [4, 6, 2])[1][1]
    assert abs(gb2.sum()) < 1e-14  # softmax deltas sum to zero over classes
    # two-class softmax == logistic regression on the logit difference
    a1 = np.maximum(X[rows].astype(np.float64) @ W1 + b1, 0)
    z = a1 @ W2 + b2
    s = (2 * y[rows] - 1) * (z[:, 1] - z[:, 0])
    assert abs(loss - np.mean(np.log1p(np.exp(-s)))) < 1e-13


def test_single_logit_head_is_the_two_class_softmax_with_a_fixed_zero_logit(oracle):
    """One output z with labels 0/1 is the two-class softmax model whose class-0 logit is pinned to 0: same
    loss, same gradient on the shared parameters, same accuracy; and the loss does not overflow for large |z|."""
    X, y = tiny_problem(9, n=34, d=4, n_classes=1)
    hp = {"hidden": [6], "alpha": 0.2, "seed": 3}
    rng = np.random.default_rng(2)
    th1 = oracle.init_params(4, 1, hp, 0) + 0.4 * rng.normal(size=oracle.param_count(4, 1, hp))
    rows = np.arange(5, 27, dtype=np.int32)
    l1, g1 = oracle.loss_grad(X, y, 1, rows, hp, th1, prec=1)
    (W1, b1), (W2, b2) = unpack(th1, [4, 6, 1])
    # the softmax twin: output weights (0, w), output biases (0, b); the zero column adds nothing to the penalty
    th2 = np.concatenate([W1.ravel(), b1, np.stack([np.zeros(6), W2[:, 0]], axis=1).ravel(), [0.0, b2[0]]])
    l2, g2 = oracle.loss_grad(X, y, 2, rows, hp, th2, prec=1)
    assert abs(l1 - l2) < 1e-13
    (gW1, gb1), (gW2, gb2) = unpack(g1, [4, 6, 1])
    (hW1, hb1), (hW2, hb2) = unpack(g2, [4, 6, 2])
    np.testing.assert_allclose(gW1, hW1, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(gb1, hb1, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(gW2[:, 0], hW2[:, 1], rtol=1e-11, atol=1e-14)
    assert abs(gb2[0] - hb2[1]) < 1e-13
    # by hand: mean of log(1 + e^z) - y z, plus the penalty
    a1 = np.maximum(X[rows].astype(np.float64) @ W1 + b1, 0)
    z = (a1 @ W2 + b2)[:, 0]
    want = np.mean(np.logaddexp(0.0, z) - y[rows] * z) + 0.5 * float(np.float32(0.2)) * ((W1 ** 2).sum() + (W2 ** 2).sum()) / len(rows)
    assert abs(l1 - want) < 1e-13
    # scores of a trained model: nll and accuracy recomputed by hand from the final parameters
    fold = (np.arange(34) % 5).astype(np.int32)
    hp2 = dict(hp, epochs=3, lr=0.01, batch_size=8, solver="adam")
    out = oracle.train_one(X, y, 1, fold, hp2, 2, prec=1)
    (W1, b1), (W2, b2) = unpack(out["theta"], [4, 6, 1])
    held = np.where(fold == 2)[0]
    z = (np.maximum(X[held].astype(np.float64) @ W1 + b1, 0) @ W2 + b2)[:, 0]
    assert abs(out["scores"][0] - np.mean(np.logaddexp(0.0, z) - y[held] * z)) < 1e-12
    assert abs(out["scores"][1] - np.mean((z > 0).astype(np.int32) == y[held])) < 1e-12
    # huge logits: finite loss, saturated gradient
    big = th1.copy()
    big[-1] = 800.0  # output bias
    lb, gb = oracle.loss_grad(X, y, 1, rows, dict(hp, alpha=0.0), big, prec=1)
    assert np.isfinite(lb) and np.isfinite(gb).all()
    assert abs(unpack(gb, [4, 6, 1])[1][1][0] - np.mean(1.0 - y[rows])) < 1e-9


def test_fp32_mode_tracks_fp64_mode(oracle):
    X, y = tiny_problem(5, n=64, d=4, n_classes=3)
    hp = {"hidden": [16], "alpha": 0.01, "seed": 3}
    theta = oracle.init_params(4, 3, hp, 0)
    rows = np.arange(40, dtype=np.int32)
    l64, g64 = oracle.loss_grad(X, y, 3, rows, hp, theta, prec=1)
    l32, g32 = oracle.loss_grad(X, y, 3, rows, hp, theta, prec=0)
    assert abs(l64 - l32) < 1e-6
    assert np.linalg.norm(g64 - g32) / np.linalg.norm(g64) < 1e-6
    assert np.array_equal(g32, g32.astype(np.float32).astype(np.float64))


def test_fp32_running_sum_probe_is_the_same_computation_up_to_single_precision(oracle):
    """prec=2 (the sensitivity probe: fp32 running sums in the contractions) differs from the definition
    by single-precision summation error only, and does differ."""
    X, y = tiny_problem(6, n=200, d=8, n_classes=3)
    hp = {"hidden": [32, 16], "alpha": 0.01, "seed": 4}
    theta = oracle.init_params(8, 3, hp, 0)
    rows = np.arange(150, dtype=np.int32)
    l0, g0 = oracle.loss_grad(X, y, 3, rows, hp, theta, prec=0)
    l2, g2 = oracle.loss_grad(X, y, 3, rows, hp, theta, prec=2)
    rel = np.linalg.norm(g0 - g2) / np.linalg.norm(g0)
    assert 0 < rel < 2e-6 and abs(l0 - l2) < 1e-6


def test_bf16_mode_rounds_operands_only(oracle):
    """bf16 configuration == the fp32 computation run on bf16-rounded operands
    (checked for a linear model, where the only operands are X and W)."""
    rng = np.random.default_rng(2)
    Xf = rng.normal(size=(20, 8)).astype(np.float32)
    Xb = inputs.to_bf16_bits(Xf).reshape(20, 8)
    y = rng.integers(0, 3, size=20).astype(np.int32)
    hp = {"hidden": [], "alpha": 0.5, "seed": 9}
    theta = oracle.init_params(8, 3, hp, 0)
    rows = np.arange(20, dtype=np.int32)
    lb, gb = oracle.loss_grad(Xb, y, 3, rows, hp, theta, dtype=1, prec=0)
    # reference: torch float64 on rounded X and rounded W (penalty on the unrounded W)
    Xr = inputs.bf16_bits_to_f32(Xb).reshape(20, 8).astype(np.float64)
    W = theta[:24].reshape(8, 3)
    b = theta[24:]
    Wr = inputs.bf16_bits_to_f32(inputs.to_bf16_bits(W.astype(np.float32))).reshape(8, 3).astype(np.float64)
    z = torch.tensor(Xr @ Wr + b)
    data = torch.nn.functional.cross_entropy(z, torch.tensor(y.astype(np.int64))).item()
    want = data + 0.5 * float(np.float32(0.5)) * (W * W).sum() / 20
    assert abs(lb - want) < 2e-6
    # deltas are rounded to bf16 before the weight-gradient product
    p = torch.softmax(z, dim=1).numpy()
    p[np.arange(20), y] -= 1
    dl = inputs.bf16_bits_to_f32(inputs.to_bf16_bits((p / 20).astype(np.float32))).reshape(20, 3).astype(np.float64)
    gW = Xr.T @ dl + float(np.float32(0.5)) / 20 * W
    np.testing.assert_allclose(gb[:24].reshape(8, 3), gW, rtol=2e-6, atol=1e-8)
    np.testing.assert_allclose(gb[24:], dl.sum(axis=0), rtol=2e-6, atol=1e-8)


# ------------------------------------------------------ optimizer pins ----

def test_adam_first_step_closed_form(oracle):
    rng = np.random.default_rng(3)
    g = rng.normal(size=50) * 10.0 ** rng.integers(-3, 2, size=50)
    theta = rng.normal(size=50)
    hp = {"solver": "adam", "lr": 0.01, "beta1": 0.9, "beta2": 0.999, "eps": 1e-8}
    th = theta.copy()
    m, v = np.zeros(50), np.zeros(50)
    t = oracle.opt_step(hp, th, g, m, v, 0, prec=1)
    assert t == 1
    b2, eps, lr = float(np.float32(0.999)), float(np.float32(1e-8)), float(np.float32(0.01))
    want = theta - lr * g / (np.abs(g) + eps / np.sqrt(1 - b2))
    np.testing.assert_allclose(th, want, rtol=1e-9, atol=1e-15)
    big = np.abs(g) > 1e-2  # |g| >> eps: the first Adam step is lr * sign(g)
    np.testing.assert_allclose(th[big], (theta - lr * np.sign(g))[big], atol=1e-6)


def test_single_sgd_steps_closed_form(oracle):
    """The single-step entry point with the momentum solver: u = mu u - lr g, then theta + u, or with Nesterov's
    look-ahead theta + mu u - lr g."""
    rng = np.random.default_rng(3)
    theta0, g, u0 = rng.normal(size=9), rng.normal(size=9), rng.normal(size=9)
    lr, mu = float(np.float32(0.07)), float(np.float32(0.6))
    for nesterov in (False, True):
        theta, u, v = theta0.copy(), u0.copy(), np.zeros(9)
        oracle.opt_step({"hidden": [], "solver": "sgd", "nesterov": nesterov, "lr": 0.07, "momentum": 0.6, "alpha": 0.3}, theta, g, u, v, 0,
                        prec=1)
        un = mu * u0 - lr * g
        np.testing.assert_allclose(u, un, rtol=1e-14)
        np.testing.assert_allclose(theta, theta0 + (mu * un - lr * g if nesterov else un), rtol=1e-14)


@pytest.mark.parametrize("solver,nesterov,f", [("adam", False, 2), ("sgd", False, 2), ("sgd", True, 2), ("adam", False, -1)])
def test_training_trajectory_matches_library_optimizer(oracle, solver, nesterov, f):
    """A few epochs of minibatch training in fp64 mode equal the same loop
    written with library autograd + library optimizer, fed the oracle's own
    minibatch rows and initial weights.  (Adam: eps is set tiny, where the two
    published placements of eps coincide.)"""
    n_classes = 3 if solver == "adam" else 0
    X, y = tiny_problem(6, n=50, d=4, n_classes=n_classes)
    fold = inputs.make_folds(50, 5, 1)
    if f < 0:  # hold-out model: 40 rows in folds, 10 in none
        fold[fold == 4] = -1
    hp = {"hidden": [7], "solver": solver, "nesterov": nesterov, "lr": 0.02, "alpha": 0.05, "momentum": 0.8,
          "batch_size": 16, "epochs": 3, "eps": 1e-30, "seed": 11}
    dims = [4, 7, n_classes if n_classes >= 2 else 1]
    res = oracle.train_one(X, y, n_classes, fold, hp, f, prec=1, step_begin=0, step_end=9)
    tt = torch.tensor(oracle.init_params(4, n_classes, hp, f), dtype=torch.float64, requires_grad=True)
    lr, mu = float(np.float32(0.02)), float(np.float32(0.8))
    if solver == "adam":
        opt = torch.optim.Adam([tt], lr=lr, betas=(float(np.float32(0.9)), float(np.float32(0.999))), eps=1e-30)
    else:
        opt = torch.optim.SGD([tt], lr=lr, momentum=mu, nesterov=nesterov)
    k = 0
    for ep in range(3):
        for s in range(3):  # 40 train rows / 16 -> 3 steps, last one of 8 rows
            rows = oracle.minibatch_rows(fold, hp, f, ep, s)
            assert len(rows) == (16 if s < 2 else 8)
            Xb = torch.tensor(X[rows], dtype=torch.float64)
            yb = torch.tensor(y[rows].astype(np.int64)) if n_classes >= 1 else torch.tensor(y[rows], dtype=torch.float64)
            opt.zero_grad()
            loss = torch_loss(tt, dims, Xb, yb, n_classes, float(np.float32(0.05)))
            loss.backward()
            assert abs(loss.item() - res["loss"][k]) < 1e-10
            np.testing.assert_allclose(res["grad"][k], tt.grad.numpy(), rtol=1e-8, atol=1e-12)
            opt.step()
            np.testing.assert_allclose(res["theta_after"][k], tt.detach().numpy(), rtol=1e-8, atol=1e-12)
            # the recorded optimizer state is the library's: both Adam moments, or the velocity
            # (the library keeps buf = mu buf + g and steps by -lr buf: the velocity is -lr buf at a constant rate)
            st = opt.state[tt]
            if solver == "adam":
                np.testing.assert_allclose(res["m_after"][k], st["exp_avg"].numpy(), rtol=1e-8, atol=1e-14)
                np.testing.assert_allclose(res["v_after"][k], st["exp_avg_sq"].numpy(), rtol=1e-8, atol=1e-16)
            else:
                np.testing.assert_allclose(res["m_after"][k], -lr * st["momentum_buffer"].numpy(), rtol=1e-8, atol=1e-14)
            k += 1
    np.testing.assert_allclose(res["theta"], tt.detach().numpy(), rtol=1e-8, atol=1e-12)
    # a later window of steps records the same steps, and a run told to stop after its window hands back the
    # parameters of the window's last step
    win = oracle.train_one(X, y, n_classes, fold, hp, f, prec=1, step_begin=4, step_end=7, stop_after=True)
    for key in ("loss", "grad", "theta_after", "m_after", "v_after"):
        assert np.array_equal(win[key], res[key][4:7]), key
    assert np.array_equal(win["theta"], res["theta_after"][6])
    assert not np.array_equal(win["theta"], res["theta"])


def test_linear_mse_converges_to_least_squares_and_ridge(oracle):
    rng = np.random.default_rng(4)
    n, d = 60, 3
    X = rng.normal(size=(n, d)).astype(np.float32)
    y = (X @ np.array([1.0, -2.0, 0.5]) + 0.7 + 0.1 * rng.normal(size=n)).astype(np.float32)
    fold = np.full(n, 1, dtype=np.int32)
    fold[:12] = 0  # fold 0 held out; train on the other 48 rows, full batch
    tr = np.arange(12, n)
    Xd, yd = X[tr].astype(np.float64), y[tr].astype(np.float64)
    for alpha in (0.0, 3.0):
        hp = {"hidden": [], "solver": "sgd", "momentum": 0.0, "lr": 0.3, "alpha": alpha, "batch_size": 0,
              "epochs": 400, "seed": 2}
        res = oracle.train_one(X, y, 0, fold, hp, 0, prec=1)
        w, b = res["theta"][:d], res["theta"][d]
        Xc, yc = Xd - Xd.mean(0), yd - yd.mean()
        w_ref = np.linalg.solve(Xc.T @ Xc + alpha * np.eye(d), Xc.T @ yc)  # intercept unpenalised
        b_ref = yd.mean() - Xd.mean(0) @ w_ref
        np.testing.assert_allclose(w, w_ref, rtol=1e-8, atol=1e-10)
        assert abs(b - b_ref) < 1e-9
        if alpha == 0.0:
            w_ls = np.linalg.lstsq(np.c_[Xd, np.ones(len(tr))], yd, rcond=None)[0]
            np.testing.assert_allclose(np.r_[w, b], w_ls, rtol=1e-8, atol=1e-10)
        # the reported score is the plain mean squared error on the held rows
        pred = X[:12].astype(np.float64) @ w + b
        assert abs(res["scores"][0] - np.mean((pred - y[:12]) ** 2)) < 1e-12
        assert abs(res["scores"][1] - np.mean(np.abs(pred - y[:12]))) < 1e-12  # and the mean absolute error


def test_full_batch_gradient_descent_loss_is_monotone(oracle):
    X, y = tiny_problem(7, n=80, d=4, n_classes=3)
    fold = inputs.make_folds(80, 5, 3)
    hp = {"hidden": [10], "solver": "sgd", "momentum": 0.0, "lr": 0.05, "alpha": 0.1, "batch_size": 0, "epochs": 60,
          "seed": 6}
    res = oracle.train_one(X, y, 3, fold, hp, 0, prec=0, step_begin=0, step_end=60)
    assert np.all(np.diff(res["loss"]) <= 1e-7)
    assert res["loss"][-1] < res["loss"][0] - 0.05


def test_zero_learning_rate_or_zero_epochs_keeps_init(oracle):
    X, y = tiny_problem(8, n=40, d=4, n_classes=3)
    fold = inputs.make_folds(40, 5, 3)
    base = {"hidden": [6], "solver": "sgd", "momentum": 0.0, "alpha": 0.0, "batch_size": 8, "seed": 4}
    init = oracle.init_params(4, 3, base, 1)
    r0 = oracle.train_one(X, y, 3, fold, dict(base, lr=0.0, epochs=3), 1)
    r1 = oracle.train_one(X, y, 3, fold, dict(base, lr=0.1, epochs=0), 1)
    assert np.array_equal(r0["theta"], init) and np.array_equal(r1["theta"], init)
    assert np.array_equal(r0["scores"], r1["scores"])
    # score of the init, by the library definition
    (W1, b1), (W2, b2) = unpack(init, [4, 6, 3])
    _, va = oracle.fold_lists(fold, 1)
    z = np.maximum(X[va].astype(np.float64) @ W1 + b1, 0) @ W2 + b2
    nll = torch.nn.functional.cross_entropy(torch.tensor(z), torch.tensor(y[va].astype(np.int64))).item()
    assert abs(r0["scores"][0] - nll) < 1e-6
    assert abs(r0["scores"][1] - np.mean(z.argmax(1) == y[va])) < 1e-7


# ------------------------------------------------ whole-call properties ----

def test_cv_score_is_unweighted_mean_of_folds_and_batch_invariant(oracle):
    cfg = inputs.make_config(0, epochs=5)
    hps = cfg["hparams"]
    s, st, pf = oracle.cv_eval(cfg["X"], cfg["y"], 3, cfg["fold_idx"], 5, hps)
    np.testing.assert_allclose(s, pf.mean(axis=1), rtol=1e-6)
    assert np.all(st == 0)
    # each suggestion's score does not depend on what else is in the batch, nor on its position
    order = [5, 2, 2, 7]
    s2, _, _ = oracle.cv_eval(cfg["X"], cfg["y"], 3, cfg["fold_idx"], 5, [hps[i] for i in order])
    assert np.array_equal(s2, s[order])
    # per-fold value equals the single-model entry point
    one = oracle.train_one(cfg["X"], cfg["y"], 3, cfg["fold_idx"], hps[3], 4)
    assert np.array_equal(one["scores"], pf[3, 4])


@pytest.mark.parametrize("n_classes", [0, 1, 2, 3])
def test_scores_are_the_library_metrics_of_the_returned_model(oracle, n_classes):
    """Both reported scores, recomputed with library routines from the parameters the run hands back, on the
    held fold: mean negative log-likelihood and accuracy (argmax, or the sign of the one logit), or mean
    squared and mean absolute error."""
    X, y = tiny_problem(21, n=90, d=5, n_classes=n_classes)
    fold = inputs.make_folds(90, 5, 2)
    hp = {"hidden": [6], "solver": "adam", "lr": 0.02, "alpha": 0.01, "batch_size": 16, "epochs": 6, "seed": 3}
    f = 3
    res = oracle.train_one(X, y, n_classes, fold, hp, f, prec=1)
    c_out = n_classes if n_classes >= 2 else 1
    (W1, b1), (W2, b2) = unpack(res["theta"], [5, 6, c_out])
    va = np.flatnonzero(fold == f)
    z = torch.tensor(np.maximum(X[va].astype(np.float64) @ W1 + b1, 0.0) @ W2 + b2)
    if n_classes >= 2:
        yt = torch.tensor(y[va].astype(np.int64))
        want = [torch.nn.functional.cross_entropy(z, yt).item(), (z.argmax(1) == yt).double().mean().item()]
        assert 0.0 < want[1] < 1.0  # neither score is trivial here
    elif n_classes == 1:
        yt = torch.tensor(y[va].astype(np.float64))
        want = [torch.nn.functional.binary_cross_entropy_with_logits(z[:, 0], yt).item(),
                ((z[:, 0] > 0).double() == yt).double().mean().item()]
        assert 0.0 < want[1] < 1.0
    else:
        yt = torch.tensor(y[va].astype(np.float64))
        want = [torch.nn.functional.mse_loss(z[:, 0], yt).item(), torch.nn.functional.l1_loss(z[:, 0], yt).item()]
    np.testing.assert_allclose(res["scores"], want, rtol=1e-12, atol=1e-14)


def test_smallest_problems_are_taken(oracle):
    """One feature, one fold, no suggestions: legal.  With a single fold every row is held out, nothing is
    trained on, and the score is that of the initial weights."""
    X, y = tiny_problem(2, n=30, d=2, n_classes=0)
    X = np.ascontiguousarray(X[:, :1])
    fold = inputs.make_folds(30, 3, 0)
    hp = {"hidden": [4], "solver": "sgd", "lr": 0.01, "batch_size": 8, "epochs": 4, "seed": 1}
    s, st, pf = oracle.cv_eval(X, y, 0, fold, 3, [hp])
    assert np.all(np.isfinite(s)) and st[0] == 0
    s0, st0, pf0 = oracle.cv_eval(X, y, 0, fold, 3, [])
    assert s0.shape[0] == 0
    one = np.zeros(30, dtype=np.int32)
    s1, st1, _ = oracle.cv_eval(X, y, 0, one, 1, [hp])
    s2, _, _ = oracle.cv_eval(X, y, 0, one, 1, [dict(hp, epochs=0)])
    assert st1[0] == 0 and np.isfinite(s1[0, 0]) and np.array_equal(s1, s2)
    h1, hst = oracle.holdout_eval(X, y, 0, np.where(np.arange(30) < 20, 0, -1).astype(np.int32), [hp])
    assert np.all(np.isfinite(h1)) and hst[0] == 0
    assert oracle.holdout_eval(X, y, 0, fold, [])[0].shape[0] == 0
    # no rows at all: every fold is empty, which is a score that does not exist, not an error
    sn, stn, _ = oracle.cv_eval(X[:0], y[:0], 0, fold[:0], 3, [hp])
    assert stn[0] == 1 and np.all(np.isnan(sn[0]))


def test_stratified_folds_are_balanced():
    cfg = inputs.make_config(0)
    for f in range(5):
        cnt = np.bincount(cfg["y"][cfg["fold_idx"] == f], minlength=3)
        assert cnt.max() - cnt.min() <= 1 and cnt.sum() == 30


def test_hidden_unit_permutation_symmetry(oracle):
    X, y = tiny_problem(9, n=30, d=4, n_classes=3)
    hp = {"hidden": [6], "alpha": 0.2, "seed": 3}
    theta = oracle.init_params(4, 3, hp, 0)
    (W1, b1), (W2, b2) = unpack(theta, [4, 6, 3])
    perm = np.array([4, 0, 5, 2, 1, 3])
    theta_p = np.concatenate([W1[:, perm].ravel(), b1[perm], W2[perm, :].ravel(), b2])
    rows = np.arange(30, dtype=np.int32)
    l0, g0 = oracle.loss_grad(X, y, 3, rows, hp, theta, prec=1)
    l1, g1 = oracle.loss_grad(X, y, 3, rows, hp, theta_p, prec=1)
    assert abs(l0 - l1) < 1e-13
    (gW1, gb1), (gW2, gb2) = unpack(g0, [4, 6, 3])
    want = np.concatenate([gW1[:, perm].ravel(), gb1[perm], gW2[perm, :].ravel(), gb2])
    np.testing.assert_allclose(g1, want, rtol=1e-12, atol=1e-15)


def test_divergent_run_sets_status_not_error(oracle):
    X, y = tiny_problem(10, n=40, d=4, n_classes=0)
    fold = inputs.make_folds(40, 5, 3)
    bad = {"hidden": [8], "solver": "sgd", "momentum": 0.99, "nesterov": True, "lr": 50.0, "batch_size": 8,
           "epochs": 60, "seed": 1}
    good = dict(bad, lr=0.01, momentum=0.5)
    s, st, _ = oracle.cv_eval(X, y, 0, fold, 5, [bad, good])
    assert st[0] == 1 and not np.isfinite(s[0, 0])
    assert st[1] == 0 and np.isfinite(s[1, 0])


def test_holdout_score_is_the_held_rows_loss_of_the_model_trained_on_all_folds(oracle):
    """Generalization score (Section 6.2): one model per suggestion, trained on every row that
    belongs to a fold, scored on the rows that belong to none; checked against the held rows'
    loss / accuracy recomputed with the library from the final weights."""
    for n_classes in (3, 0):
        X, y = tiny_problem(21, n=90, d=5, n_classes=n_classes)
        fold = inputs.make_folds(90, 4, 5)
        fold[::4] = -1
        hps = [{"hidden": [6], "lr": 0.01, "alpha": 0.01, "batch_size": 20, "epochs": 4, "seed": 5},
               {"hidden": [4, 3], "solver": "sgd", "lr": 0.02, "momentum": 0.5, "batch_size": 0, "epochs": 6, "seed": 6}]
        s, st = oracle.holdout_eval(X, y, n_classes, fold, hps, prec=1)
        assert np.all(st == 0)
        held = np.nonzero(fold < 0)[0]
        for b, hp in enumerate(hps):
            one = oracle.train_one(X, y, n_classes, fold, hp, -1, prec=1)
            assert np.allclose(one["scores"], s[b], rtol=1e-6)
            dims = [5] + hp["hidden"] + [n_classes if n_classes >= 2 else 1]
            tt = torch.tensor(one["theta"], dtype=torch.float64)
            Xh = torch.tensor(X[held], dtype=torch.float64)
            if n_classes >= 2:
                yh = torch.tensor(y[held].astype(np.int64))
                loss = torch_loss(tt, dims, Xh, yh, n_classes, 0.0).item()
            else:
                yh = torch.tensor(y[held], dtype=torch.float64)
                loss = 2.0 * torch_loss(tt, dims, Xh, yh, n_classes, 0.0).item()  # reported mse has no 1/2
                # the second regression metric (Section 2 lists mse and mae): mean |prediction - target|
                a = Xh
                for l, (W, bb_) in enumerate(unpack(tt, dims)):
                    a = a @ W + bb_
                    if l + 2 < len(dims):
                        a = torch.relu(a)
                assert abs((a[:, 0] - yh).abs().mean().item() - s[b, 1]) < 1e-6
            assert abs(loss - s[b, 0]) < 1e-6 * max(1.0, abs(loss))
        # the hold-out model shares no stream with the cross-validation models of the suggestion
        assert not np.array_equal(oracle.init_params(5, n_classes, hps[0], -1), oracle.init_params(5, n_classes, hps[0], 0))
    # no held rows: non-finite score, status 1
    s, st = oracle.holdout_eval(X, y, 0, np.zeros(90, dtype=np.int32), hps[:1])
    assert st[0] == 1 and not np.isfinite(s[0, 0])


def test_inverse_scaling_rate_matches_a_hand_written_sgd_loop(oracle):
    """SGD with the inverse-scaling schedule: the rate of epoch e is lr / (1 + e * n_train)^power_t;
    checked against the same loop written with library autograd and an explicit momentum update."""
    X, y = tiny_problem(8, n=50, d=4, n_classes=0)
    fold = inputs.make_folds(50, 5, 1)
    f, p_t = 1, 0.5
    hp = {"hidden": [5], "solver": "sgd", "nesterov": False, "lr": 0.05, "alpha": 0.0, "momentum": 0.6, "batch_size": 20,
          "epochs": 3, "seed": 4, "power_t": p_t}
    res = oracle.train_one(X, y, 0, fold, hp, f, prec=1, step_begin=0, step_end=6)
    tt = torch.tensor(oracle.init_params(4, 0, hp, f), dtype=torch.float64, requires_grad=True)
    vel = torch.zeros_like(tt)
    lr0, mu = float(np.float32(0.05)), float(np.float32(0.6))
    n_tr, k = 40, 0
    for ep in range(3):
        lr_e = lr0 / (1.0 + ep * n_tr) ** float(np.float32(p_t))
        for s in range(2):
            rows = oracle.minibatch_rows(fold, hp, f, ep, s)
            loss = torch_loss(tt, [4, 5, 1], torch.tensor(X[rows], dtype=torch.float64),
                              torch.tensor(y[rows], dtype=torch.float64), 0, 0.0)
            (g,) = torch.autograd.grad(loss, tt)
            vel = mu * vel - lr_e * g
            tt = (tt + vel).detach().requires_grad_(True)
            np.testing.assert_allclose(res["theta_after"][k], tt.detach().numpy(), rtol=1e-9, atol=1e-12)
            k += 1
    # Adam ignores the schedule
    a0 = oracle.train_one(X, y, 0, fold, dict(hp, solver="adam", power_t=0.0), f, prec=1)["theta"]
    a1 = oracle.train_one(X, y, 0, fold, dict(hp, solver="adam", power_t=0.5), f, prec=1)["theta"]
    assert np.array_equal(a0, a1)


def test_plateau_stop_ends_training_at_the_epoch_the_rule_gives(oracle):
    """With n_iter_no_change = k, training ends after the first epoch that closes a run of more than k epochs
    whose mean data loss failed to beat the best so far by tol; the epoch losses are recomputed here from
    the recorded per-step losses (alpha = 0, so the step loss is the data loss)."""
    X, y = tiny_problem(9, n=60, d=4, n_classes=3)
    fold = inputs.make_folds(60, 5, 2)
    f = 0
    base = {"hidden": [6], "solver": "adam", "lr": 0.05, "alpha": 0.0, "batch_size": 16, "epochs": 60, "seed": 12}
    free = oracle.train_one(X, y, 3, fold, base, f, step_begin=0, step_end=60 * 3)
    sizes = np.array([16, 16, 16])  # 48 training rows
    ep_loss = (free["loss"].reshape(60, 3) * sizes).sum(1) / 48.0
    for tol, k in [(1e-3, 2), (5e-2, 1), (0.0, 3)]:
        best, stalled, stop_at = np.float32(np.inf), 0, 60
        for e in range(60):
            le = np.float32(ep_loss[e])
            stalled = stalled + 1 if le > np.float32(best - np.float32(tol)) else 0
            best = min(best, le)
            if stalled > k:
                stop_at = e + 1
                break
        hp = dict(base, tol=tol, n_iter_no_change=k)
        got = oracle.train_one(X, y, 3, fold, hp, f, step_begin=0, step_end=60 * 3)
        done = int(np.isfinite(got["loss"]).sum()) // 3
        assert done == stop_at, (tol, k, done, stop_at)
        # the stopped model is the free run's model at that epoch
        np.testing.assert_array_equal(got["theta"], free["theta_after"][3 * stop_at - 1])
    # n_iter_no_change = 0 switches the rule off whatever tol is
    off = oracle.train_one(X, y, 3, fold, dict(base, tol=10.0), f)
    np.testing.assert_array_equal(off["theta"], free["theta"])


# ------------------------------------------ validation-fraction early stopping ----

def py_mix64(z):
    z &= M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def py_fold(h, v):
    return py_mix64((h + (v + 1) * G) & M64)


def py_perm(key, n, p):
    """The keyed bijection of [0, n) written out in plain integers: 4-round balanced Feistel network on an
    even number of bits, cycle-walked into range."""
    if n <= 1:
        return 0
    bits = max(2, (n - 1).bit_length())
    bits += bits & 1
    hb = bits // 2
    mask = (1 << hb) - 1
    x = p
    while True:
        L, R = x >> hb, x & mask
        for r in range(4):
            L, R = R, L ^ (py_fold(key, (r << 32) | R) & mask)
        x = (L << hb) | R
        if x < n:
            return x


def test_early_stop_split_is_a_keyed_cut_of_the_training_list(oracle):
    """The rows set aside are the tail of a keyed shuffle of the fold's training list, n_hold = floor(fraction x
    n_train) clamped to [1, n_train - 1]; every epoch's minibatches cover exactly the remaining rows once.
    The shuffle is recomputed here in plain Python integers from the SplitMix64 mixer."""
    fold = inputs.make_folds(103, 5, 4)
    for frac, bs, seed, f in [(0.1, 16, 5, 0), (0.25, 0, 77, 3), (0.001, 7, 9, 1), (0.9999, 5, 3, 2), (0.5, 200, 1, 4)]:
        hp = {"hidden": [3], "batch_size": bs, "seed": seed, "n_iter_no_change": 2, "validation_fraction": frac}
        tr, _ = oracle.fold_lists(fold, f)
        n_tr = len(tr)
        n_hold = min(max(int(np.floor(float(np.float32(frac)) * n_tr)), 1), n_tr - 1)
        n_fit = n_tr - n_hold
        kmodel = py_fold(py_fold(seed, 0x4D4C50), f)
        ksplit = py_fold(kmodel, 2)
        held = [tr[py_perm(ksplit, n_tr, n_fit + i)] for i in range(n_hold)]
        assert oracle.early_stop_rows(fold, hp, f).tolist() == held
        fit = sorted(set(tr.tolist()) - set(held))
        assert len(fit) == n_fit
        eb = bs if 0 < bs <= n_fit else n_fit
        for epoch in (0, 3):
            kep = py_fold(py_fold(kmodel, 1), epoch)
            seen = []
            for s in range(-(-n_fit // eb)):
                rows = oracle.minibatch_rows(fold, hp, f, epoch, s).tolist()
                want = [tr[py_perm(ksplit, n_tr, py_perm(kep, n_fit, p))] for p in range(s * eb, min((s + 1) * eb, n_fit))]
                assert rows == want
                seen += rows
            assert sorted(seen) == fit
    # the cut keeps at least one row on either side
    two = np.array([0, 1, 1, 0, 1], dtype=np.int32)  # fold 0 leaves three rows, fold 1 two
    for frac, f, want in [(0.01, 0, 1), (0.99, 0, 2), (1.0, 0, 2), (1.34, 0, 2), (7.5, 0, 2), (0.5, 1, 1), (0.01, 1, 1),
                          (3.0, 1, 1)]:
        hp = {"hidden": [3], "seed": 5, "n_iter_no_change": 1, "validation_fraction": frac}
        assert len(oracle.early_stop_rows(two, hp, f)) == want, (frac, f)
    one = np.array([0, 1, 1, 1], dtype=np.int32)      # fold 1 leaves one training row: nothing to set aside
    assert len(oracle.early_stop_rows(one, dict(hp, validation_fraction=0.5), 1)) == 0
    # switched off (no patience, or no fraction): nothing is set aside, the order is the plain one
    for off in ({"n_iter_no_change": 0, "validation_fraction": 0.3}, {"n_iter_no_change": 3, "validation_fraction": 0.0}):
        hp = dict({"hidden": [3], "batch_size": 16, "seed": 5}, **off)
        assert len(oracle.early_stop_rows(fold, hp, 0)) == 0
        assert oracle.minibatch_rows(fold, hp, 0, 1, 2).tolist() == oracle.minibatch_rows(fold, {"hidden": [3], "batch_size": 16, "seed": 5}, 0, 1, 2).tolist()


@pytest.mark.parametrize("n_classes", [3, 0])
def test_early_stop_on_held_rows_matches_a_hand_written_loop(oracle, n_classes):
    """Validation-fraction early stopping against the same training written with library autograd: plain SGD
    on the rows that are not set aside, the held rows' loss (cross-entropy / plain mean squared error)
    after every epoch, the stall rule in single precision; stop epoch, final parameters and score."""
    X, y = tiny_problem(21 + n_classes, n=90, d=5, n_classes=n_classes)
    fold = inputs.make_folds(90, 5, 6)
    f, E, frac = 2, 40, 0.2
    dims = [5, 7, n_classes if n_classes else 1]
    # (the regression case also runs the inverse-scaling rate, which counts the rows that are fitted on)
    p_t = 0.0 if n_classes else 0.25
    base = {"hidden": [7], "solver": "sgd", "nesterov": False, "momentum": 0.0, "lr": 0.08, "alpha": 0.01,
            "batch_size": 16, "epochs": E, "seed": 14, "validation_fraction": frac, "power_t": p_t}
    tr, va = oracle.fold_lists(fold, f)
    n_tr = len(tr)
    n_hold = int(np.floor(float(np.float32(frac)) * n_tr))
    n_fit = n_tr - n_hold
    kmodel = py_fold(py_fold(14, 0x4D4C50), f)
    ksplit = py_fold(kmodel, 2)
    held = np.array([tr[py_perm(ksplit, n_tr, n_fit + i)] for i in range(n_hold)])
    Xt = torch.tensor(X, dtype=torch.float64)
    yt = torch.tensor(y.astype(np.int64) if n_classes else y.astype(np.float64))
    lr, alpha = float(np.float32(0.08)), float(np.float32(0.01))

    def held_loss(tt):
        return float(torch_loss(tt, dims, Xt[held], yt[held], n_classes, 0.0)) * (1.0 if n_classes else 2.0)

    stops, late = [], []
    for tol, k in [(1e-3, 2), (2e-2, 1), (0.0, 4)]:
        tt = torch.tensor(oracle.init_params(5, n_classes, base, f), dtype=torch.float64, requires_grad=True)
        best, stalled, stop_at, tt_best, best_epoch = np.float32(np.inf), 0, E, None, -1
        for e in range(E):
            kep = py_fold(py_fold(kmodel, 1), e)
            lr_e = lr / (1.0 + e * n_fit) ** float(np.float32(p_t))
            for s in range(-(-n_fit // 16)):
                rows = [tr[py_perm(ksplit, n_tr, py_perm(kep, n_fit, p))] for p in range(s * 16, min((s + 1) * 16, n_fit))]
                loss = torch_loss(tt, dims, Xt[rows], yt[rows], n_classes, alpha)
                (g,) = torch.autograd.grad(loss, tt)
                tt = (tt - lr_e * g).detach().requires_grad_(True)
            le = np.float32(held_loss(tt.detach()))
            stalled = stalled + 1 if le > np.float32(best - np.float32(tol)) else 0
            if le < best:  # the best iterate on the held rows is the model that is handed back
                best, tt_best, best_epoch = le, tt.detach().clone(), e
            if stalled > k:
                stop_at = e + 1
                break
        hp = dict(base, tol=tol, n_iter_no_change=k)
        spe = -(-n_fit // 16)
        got = oracle.train_one(X, y, n_classes, fold, hp, f, prec=1, step_begin=0, step_end=E * spe)
        assert int(np.isfinite(got["loss"]).sum()) == stop_at * spe, (tol, k, stop_at)
        np.testing.assert_allclose(got["theta"], tt_best.numpy(), rtol=1e-9, atol=1e-12)
        # ... which is the recorded state after that epoch's last step, not the last one when the rule let training run on
        np.testing.assert_allclose(got["theta"], got["theta_after"][(best_epoch + 1) * spe - 1], rtol=0, atol=0)
        late.append(best_epoch + 1 < stop_at)
        tt = tt_best
        want = float(torch_loss(tt.detach(), dims, Xt[va], yt[va], n_classes, 0.0)) * (1.0 if n_classes else 2.0)
        assert abs(got["scores"][0] - want) < 1e-10
        stops.append(stop_at)
    assert min(stops) < E, stops  # the rule does end some run early
    assert any(late) or p_t > 0, late  # and (at a constant rate) some run's best epoch is not its last one
    # the same rule on the training loss (no fraction) stops elsewhere: the held rows really are what is watched
    other = oracle.train_one(X, y, n_classes, fold, dict(base, tol=2e-2, n_iter_no_change=1, validation_fraction=0.0), f,
                             prec=1, step_begin=0, step_end=E * 5)
    assert int(np.isfinite(other["loss"]).sum()) != stops[1] * spe or not np.array_equal(other["theta"], got["theta"])
