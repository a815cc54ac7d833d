"""ctypes access to the CPU oracle (oracle/mlp_cv_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the reported
CPU-baseline leg of the benchmark.  Nothing here touches the GPU library.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mlp_cv_oracle.c")
_LIB = os.path.join(_HERE, "libmlp_cv_oracle.so")

MAX_HIDDEN = 4
ADAM, SGD = 0, 1


class HParams(C.Structure):
    _fields_ = [
        ("n_hidden", C.c_int32),
        ("hidden", C.c_int32 * MAX_HIDDEN),
        ("solver", C.c_int32),
        ("nesterov", C.c_int32),
        ("batch_size", C.c_int32),
        ("epochs", C.c_int32),
        ("lr", C.c_float),
        ("alpha", C.c_float),
        ("momentum", C.c_float),
        ("beta1", C.c_float),
        ("beta2", C.c_float),
        ("eps", C.c_float),
        ("power_t", C.c_float),
        ("seed", C.c_uint64),
        ("tol", C.c_float),
        ("n_iter_no_change", C.c_int32),
        ("validation_fraction", C.c_float),
        ("reserved", C.c_int32),
    ]


def build(force=False):
    """Compile the oracle with gcc (no fast-math, no contraction)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    tmp = _LIB + ".%d.tmp" % os.getpid()
    cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-fno-fast-math", "-Wall", "-o", tmp, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, _LIB)  # a process that has the old library mapped keeps it
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.oracle_mix64.restype = C.c_uint64
        L.oracle_mix64.argtypes = [C.c_uint64]
        L.oracle_combine.restype = C.c_uint64
        L.oracle_combine.argtypes = [C.c_uint64, C.c_uint64]
        L.oracle_perm_index.restype = C.c_int64
        L.oracle_perm_index.argtypes = [C.c_uint64, C.c_int32, C.c_int32, C.c_int64, C.c_int64]
        L.oracle_bf16_bits.restype = C.c_uint16
        L.oracle_bf16_bits.argtypes = [C.c_float]
        L.oracle_param_count.restype = C.c_int64
        L.oracle_minibatch_rows.restype = C.c_int64
        L.oracle_early_stop_rows.restype = C.c_int64
        _lib = L
    return _lib


def make_hparams(dicts):
    """List of dicts (see the inputs module) -> ctypes array of HParams."""
    arr = (HParams * max(len(dicts), 1))()
    for h, dct in zip(arr, dicts):
        hidden = list(dct.get("hidden", []))
        h.n_hidden = len(hidden)
        for i, w in enumerate(hidden):
            h.hidden[i] = int(w)
        h.solver = SGD if dct.get("solver", "adam") == "sgd" else ADAM
        h.nesterov = int(bool(dct.get("nesterov", False)))
        h.batch_size = int(dct.get("batch_size", 0))
        h.epochs = int(dct.get("epochs", 1))
        h.lr = float(dct.get("lr", 1e-3))
        h.alpha = float(dct.get("alpha", 0.0))
        h.momentum = float(dct.get("momentum", 0.9))
        h.beta1 = float(dct.get("beta1", 0.9))
        h.beta2 = float(dct.get("beta2", 0.999))
        h.eps = float(dct.get("eps", 1e-8))
        h.seed = int(dct.get("seed", 0))
        h.power_t = float(dct.get("power_t", 0.0))
        h.tol = float(dct.get("tol", 0.0))
        h.n_iter_no_change = int(dct.get("n_iter_no_change", 0))
        h.validation_fraction = float(dct.get("validation_fraction", 0.0))
    return arr


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _xy(X, y, n_classes, dtype):
    X = np.ascontiguousarray(X, dtype=np.uint16 if dtype else np.float32)
    y = np.ascontiguousarray(y, dtype=np.int32 if n_classes >= 1 else np.float32)  # 1: single-logit binary head
    return X, y


def mix64(x):
    return int(lib().oracle_mix64(C.c_uint64(x & (2**64 - 1))))


def combine(h, v):
    return int(lib().oracle_combine(C.c_uint64(h & (2**64 - 1)), C.c_uint64(v & (2**64 - 1))))


def perm_index(seed, fold, epoch, n, p):
    return int(lib().oracle_perm_index(seed, fold, epoch, n, p))


def permutation(seed, fold, epoch, n):
    f = lib().oracle_perm_index
    return np.array([f(seed, fold, epoch, n, p) for p in range(n)], dtype=np.int64)


def bf16_bits(x):
    return int(lib().oracle_bf16_bits(C.c_float(x)))


def param_count(d, n_classes, hp):
    return int(lib().oracle_param_count(C.c_int32(d), C.c_int32(n_classes), C.byref(make_hparams([hp])[0])))


def init_params(d, n_classes, hp, fold):
    h = make_hparams([hp])
    P = param_count(d, n_classes, hp)
    out = np.zeros(P, dtype=np.float64)
    rc = lib().oracle_init_params(C.c_int32(d), C.c_int32(n_classes), C.byref(h[0]), C.c_int32(fold), _p(out))
    assert rc == 0
    return out


def fold_lists(fold_idx, f):
    fold_idx = np.ascontiguousarray(fold_idx, dtype=np.int32)
    n = fold_idx.shape[0]
    tr = np.zeros(max(n, 1), dtype=np.int32)
    va = np.zeros(max(n, 1), dtype=np.int32)
    ntr, nva = C.c_int64(0), C.c_int64(0)
    lib().oracle_fold_lists(_p(fold_idx), C.c_int64(n), C.c_int32(f), _p(tr), _p(va), C.byref(ntr), C.byref(nva))
    return tr[: ntr.value].copy(), va[: nva.value].copy()


def minibatch_rows(fold_idx, hp, f, epoch, step):
    fold_idx = np.ascontiguousarray(fold_idx, dtype=np.int32)
    n = fold_idx.shape[0]
    h = make_hparams([hp])
    out = np.zeros(max(n, 1), dtype=np.int32)
    cnt = lib().oracle_minibatch_rows(_p(fold_idx), C.c_int64(n), C.byref(h[0]), C.c_int32(f), C.c_int32(epoch),
                                      C.c_int64(step), _p(out))
    return out[:cnt].copy()


def early_stop_rows(fold_idx, hp, f):
    """The rows fold f's model sets aside for early stopping (empty when the rule is off)."""
    fold_idx = np.ascontiguousarray(fold_idx, dtype=np.int32)
    n = fold_idx.shape[0]
    h = make_hparams([hp])
    out = np.zeros(max(n, 1), dtype=np.int32)
    cnt = lib().oracle_early_stop_rows(_p(fold_idx), C.c_int64(n), C.byref(h[0]), C.c_int32(f), _p(out))
    return out[:cnt].copy()


def loss_grad(X, y, n_classes, rows, hp, theta, dtype=0, prec=0):
    X, y = _xy(X, y, n_classes, dtype)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    theta = np.ascontiguousarray(theta, dtype=np.float64)
    h = make_hparams([hp])
    grad = np.zeros_like(theta)
    loss = C.c_double(0)
    rc = lib().oracle_loss_grad(_p(X), _p(y), C.c_int64(X.shape[0]), C.c_int32(X.shape[1]), C.c_int32(n_classes),
                                _p(rows), C.c_int64(rows.shape[0]), C.byref(h[0]), _p(theta), C.c_int32(dtype),
                                C.c_int32(prec), C.byref(loss), _p(grad))
    assert rc == 0
    return loss.value, grad


def opt_step(hp, theta, g, m, v, t, prec=0):
    """One optimizer step in place on float64 arrays; returns the new t."""
    h = make_hparams([hp])
    tt = C.c_int64(t)
    lib().oracle_opt_step(C.byref(h[0]), C.c_int64(theta.shape[0]), _p(theta), _p(g), _p(m), _p(v), C.byref(tt),
                          C.c_int32(prec))
    return tt.value


def train_one(X, y, n_classes, fold_idx, hp, fold, dtype=0, prec=0, step_begin=0, step_end=0, stop_after=False):
    """Train one (suggestion, fold) model.

    Returns dict(theta, scores, loss[T], grad[T,P], theta_after[T,P],
    m_after[T,P], v_after[T,P]) with T = step_end - step_begin recorded steps
    (m = first moment or SGD velocity, v = second moment).
    """
    X, y = _xy(X, y, n_classes, dtype)
    fold_idx = np.ascontiguousarray(fold_idx, dtype=np.int32)
    h = make_hparams([hp])
    P = param_count(X.shape[1], n_classes, hp)
    T = max(step_end - step_begin, 0)
    trace = np.full((T, 1 + 4 * P), np.nan, dtype=np.float64) if T else None
    theta = np.zeros(P, dtype=np.float64)
    sc = np.zeros(2, dtype=np.float64)
    rc = lib().oracle_train_one(_p(X), _p(y), C.c_int64(X.shape[0]), C.c_int32(X.shape[1]), C.c_int32(n_classes),
                                _p(fold_idx), C.byref(h[0]), C.c_int32(fold), C.c_int32(dtype), C.c_int32(prec),
                                C.c_int64(step_begin), C.c_int64(step_end), C.c_int32(int(stop_after)),
                                _p(trace) if T else None, _p(theta), _p(sc))
    assert rc == 0, rc
    out = {"theta": theta, "scores": sc}
    if T:
        out["loss"] = trace[:, 0].copy()
        out["grad"] = trace[:, 1:1 + P].copy()
        out["theta_after"] = trace[:, 1 + P:1 + 2 * P].copy()
        out["m_after"] = trace[:, 1 + 2 * P:1 + 3 * P].copy()
        out["v_after"] = trace[:, 1 + 3 * P:].copy()
    return out


def cv_eval(X, y, n_classes, fold_idx, n_folds, hps, dtype=0, prec=0, n_threads=None):
    """scores[B,2] float32, status[B] int32, per_fold[B,K,2] float64."""
    X, y = _xy(X, y, n_classes, dtype)
    fold_idx = np.ascontiguousarray(fold_idx, dtype=np.int32)
    B = len(hps)
    h = make_hparams(hps)
    scores = np.zeros((max(B, 1), 2), dtype=np.float32)
    status = np.zeros(max(B, 1), dtype=np.int32)
    pf = np.zeros((max(B, 1), n_folds, 2), dtype=np.float64)
    if n_threads is None:
        n_threads = len(os.sched_getaffinity(0))
    d = X.shape[1] if X.ndim == 2 else 1
    rc = lib().oracle_mlp_cv_eval(_p(X), _p(y), C.c_int64(X.shape[0]), C.c_int32(d), C.c_int32(n_classes),
                                  _p(fold_idx), C.c_int32(n_folds), h, C.c_int32(B), C.c_int32(dtype), C.c_int32(prec),
                                  _p(scores), _p(status), _p(pf), C.c_int32(n_threads))
    if rc != 0:
        raise ValueError("oracle_mlp_cv_eval: invalid argument (%d)" % rc)
    return scores[:B], status[:B], pf[:B]


def holdout_eval(X, y, n_classes, fold_idx, hps, dtype=0, prec=0, n_threads=None):
    """Hold-out (generalization) scores: train on the rows of all folds, score the rows of none.
    scores[B,2] float32, status[B] int32."""
    X, y = _xy(X, y, n_classes, dtype)
    fold_idx = np.ascontiguousarray(fold_idx, dtype=np.int32)
    B = len(hps)
    h = make_hparams(hps)
    scores = np.zeros((max(B, 1), 2), dtype=np.float32)
    status = np.zeros(max(B, 1), dtype=np.int32)
    if n_threads is None:
        n_threads = len(os.sched_getaffinity(0))
    d = X.shape[1] if X.ndim == 2 else 1
    rc = lib().oracle_mlp_holdout_eval(_p(X), _p(y), C.c_int64(X.shape[0]), C.c_int32(d), C.c_int32(n_classes),
                                       _p(fold_idx), h, C.c_int32(B), C.c_int32(dtype), C.c_int32(prec),
                                       _p(scores), _p(status), C.c_int32(n_threads))
    if rc != 0:
        raise ValueError("oracle_mlp_holdout_eval: invalid argument (%d)" % rc)
    return scores[:B], status[:B]
