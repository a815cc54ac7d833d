"""Seeded synthetic inputs for the batched MLP cross-validation evaluator.

Only input generation lives here: data matrices shaped like the small tabular
datasets the paper's benchmark uses (Section 2, Table 1: iris-, digits-,
boston- and breast-cancer-sized sets; Section 5: added sets of 10,000 rows),
fold assignments, and hyper-parameter suggestions drawn the way a random-search
optimizer would draw them.  None of the evaluator's arithmetic is here; both
the GPU library and the CPU oracle are fed from these generators.

Hyper-parameter suggestions are plain dicts:
  hidden (list of widths), solver ("adam"|"sgd"), nesterov, batch_size
  (0 = full batch), epochs, lr, alpha, momentum, beta1, beta2, eps, seed.
"""
import numpy as np

N_FOLDS = 5


def to_bf16_bits(x):
    """float32 array -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def standardize(X):
    X = np.asarray(X, dtype=np.float64)
    sd = X.std(axis=0)
    sd[sd == 0] = 1.0
    return ((X - X.mean(axis=0)) / sd).astype(np.float32)


def make_folds(n, n_folds, seed, y=None):
    """Fold id per row from a seeded permutation; stratified by class if y is given."""
    rng = np.random.default_rng(seed)
    order = rng.permutation(n)
    fold = np.zeros(n, dtype=np.int32)
    if y is None:
        fold[order] = np.arange(n) % n_folds
    else:
        seen = {}
        for r in order:
            c = int(y[r])
            fold[r] = seen.get(c, 0) % n_folds
            seen[c] = seen.get(c, 0) + 1
    return fold


def _logu(rng, lo, hi):
    return float(np.exp(rng.uniform(np.log(lo), np.log(hi))))


def _seed64(rng):
    return int(rng.integers(0, 2**63 - 1))


# ---------------------------------------------------------------- data ----

def data_clusters(seed, n=150, d=4, n_classes=3):
    """Gaussian clusters, balanced classes, standardized (iris-shaped)."""
    rng = np.random.default_rng(seed)
    means = rng.normal(0.0, 2.0, size=(n_classes, d))
    y = (np.arange(n) % n_classes).astype(np.int32)
    X = means[y] + rng.normal(0.0, 1.0, size=(n, d))
    return standardize(X), y


def data_digits(seed, n=1797, d=64, n_classes=10):
    """Per-class templates of pixel probabilities; pixel = Binomial(16,p)/16."""
    rng = np.random.default_rng(seed)
    templ = rng.beta(0.6, 0.9, size=(n_classes, d))
    y = (np.arange(n) % n_classes).astype(np.int32)
    rng.shuffle(y)
    X = rng.binomial(16, templ[y]).astype(np.float32) / np.float32(16.0)
    return X.astype(np.float32), y


def data_regression(seed, n=506, d=13):
    """Log-normal and Gaussian columns; y = w.x + 0.5 sin(x0) + noise."""
    rng = np.random.default_rng(seed)
    cols = []
    for j in range(d):
        if j % 2 == 0:
            cols.append(rng.lognormal(0.0, 0.75, size=n))
        else:
            cols.append(rng.normal(0.0, 1.0, size=n))
    X = standardize(np.stack(cols, axis=1))
    w = rng.normal(0.0, 1.0, size=d)
    y = X.astype(np.float64) @ w + 0.5 * np.sin(X[:, 0].astype(np.float64)) + rng.normal(0.0, 0.3, size=n)
    return X, y.astype(np.float32)


def data_binary(seed, n=569, d=30):
    """Correlated Gaussian features (mean off-diagonal correlation 0.6), logistic labels."""
    rng = np.random.default_rng(seed)
    load = np.sqrt(rng.uniform(0.45, 0.75, size=d))
    common = rng.normal(size=(n, 1))
    X = common * load + rng.normal(size=(n, d)) * np.sqrt(1.0 - load**2)
    X = standardize(X)
    w = rng.normal(0.0, 1.0, size=d)
    logit = X.astype(np.float64) @ w + rng.normal(0.0, 0.5)
    y = (rng.uniform(size=n) < 1.0 / (1.0 + np.exp(-logit))).astype(np.int32)
    return X, y


def data_mixture(seed, n=20000, d=128, n_classes=10):
    """Gaussian mixture, label = component, standardized, rounded to bfloat16."""
    rng = np.random.default_rng(seed)
    means = rng.normal(0.0, 0.35, size=(n_classes, d))
    y = rng.integers(0, n_classes, size=n).astype(np.int32)
    X = standardize(means[y] + rng.normal(0.0, 1.0, size=(n, d)))
    return to_bf16_bits(X).reshape(n, d), y


# ------------------------------------------------------------- hparams ----

def suggest(rng, *, n_hidden, width, solver, epochs, batch=None, lr=(1e-5, 1e-1), alpha=(1e-5, 1e1),
            momentum=None, nesterov=False):
    h = {
        "hidden": [int(rng.integers(width[0], width[1] + 1)) for _ in range(n_hidden)],
        "solver": solver,
        "nesterov": nesterov,
        "alpha": _logu(rng, *alpha),
        "batch_size": 0 if batch is None else int(rng.integers(batch[0], batch[1] + 1)),
        "lr": _logu(rng, *lr),
        "momentum": 0.9 if momentum is None else _logu(rng, *momentum),
        "beta1": 0.9, "beta2": 0.999, "eps": 1e-8,
        "epochs": epochs,
        "seed": _seed64(rng),
    }
    return h


CONFIG_NAMES = ["cfg0_tiny_cls", "cfg1_digits_cls", "cfg2_regression", "cfg3_many_studies", "cfg4_scaleup_bf16"]


def make_config(i, B=None, epochs=None, n=None):
    """The five benchmark configurations (index 0..4).

    Returns dict(name, X, y, n_classes, dtype, fold_idx, n_folds, hparams).
    B / epochs / n shrink the configuration for tests; the defaults are the
    full sizes.
    """
    rng = np.random.default_rng(2000 + i)
    dseed, fseed = 1000 + i, 3000 + i
    if i == 0:
        X, y = data_clusters(dseed, n=n or 150)
        ncls, dtype = 3, 0
        fold = make_folds(len(y), N_FOLDS, fseed, y=y)
        hps = [suggest(rng, n_hidden=1, width=(8, 32), solver="adam", epochs=epochs or 20,
                       lr=(1e-4, 1e-1), alpha=(1e-5, 1e-1)) for _ in range(B or 8)]
    elif i == 1:
        X, y = data_digits(dseed, n=n or 1797)
        ncls, dtype = 10, 0
        fold = make_folds(len(y), N_FOLDS, fseed)
        hps = [suggest(rng, n_hidden=1, width=(50, 200), solver="adam", epochs=epochs or 200,
                       batch=(16, 256)) for _ in range(B or 8)]
    elif i == 2:
        X, y = data_regression(dseed, n=n or 506)
        ncls, dtype = 0, 0
        fold = make_folds(len(y), N_FOLDS, fseed)
        hps = [suggest(rng, n_hidden=1, width=(50, 200), solver="sgd", nesterov=True, epochs=epochs or 200,
                       batch=(16, 128), momentum=(0.5, 0.99)) for _ in range(B or 8)]
    elif i == 3:
        X, y = data_binary(dseed, n=n or 569)
        ncls, dtype = 2, 0
        fold = make_folds(len(y), N_FOLDS, fseed)
        hps = [suggest(rng, n_hidden=1, width=(50, 200), solver="adam", epochs=epochs or 100,
                       batch=(16, 256)) for _ in range(B or 2048)]
    elif i == 4:
        X, y = data_mixture(dseed, n=n or 20000)
        ncls, dtype = 10, 1
        fold = make_folds(len(y), N_FOLDS, fseed)
        hps = [suggest(rng, n_hidden=2, width=(128, 256), solver="adam", epochs=epochs or 50,
                       batch=(256, 256), lr=(1e-4, 1e-2), alpha=(1e-5, 1e-1)) for _ in range(B or 1640)]
    else:
        raise ValueError("config index 0..4")
    return {"name": CONFIG_NAMES[i], "X": X, "y": y, "n_classes": ncls, "dtype": dtype, "fold_idx": fold,
            "n_folds": N_FOLDS, "hparams": hps}


def flops_per_sample(d, hidden, c_out):
    """Algorithmic training FLOPs per sample: 2*in*out per GEMM, two GEMMs for
    the first layer (forward, weight gradient), three for later layers."""
    dims = [d] + list(hidden) + [c_out]
    f = 0
    for l in range(len(dims) - 1):
        f += 2 * dims[l] * dims[l + 1] * (2 if l == 0 else 3)
    return f


def workload_flops(cfg):
    """Total algorithmic FLOPs (training + one validation forward) and model-epochs."""
    fold = cfg["fold_idx"]
    K = cfg["n_folds"]
    d = cfg["X"].shape[1]
    c_out = cfg["n_classes"] if cfg["n_classes"] >= 2 else 1
    total, model_epochs = 0.0, 0
    for f in range(K):
        n_va = int((fold == f).sum())
        n_tr = int((fold >= 0).sum()) - n_va
        for h in cfg["hparams"]:
            dims = [d] + list(h["hidden"]) + [c_out]
            fwd = sum(2 * dims[l] * dims[l + 1] for l in range(len(dims) - 1))
            total += float(flops_per_sample(d, h["hidden"], c_out)) * n_tr * h["epochs"] + float(fwd) * n_va
            model_epochs += h["epochs"]
    return total, model_epochs
