"""Thin ctypes binding over libbbo_mlp.so (the C ABI of include/bbo_mlp.h).

Argument marshalling only: every step of the evaluation runs in the HIP
kernels.  PyTorch supplies device memory and the stream.  There is no CPU
fallback: a missing library is an ImportError at first use.
"""
import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbbo_mlp.so")

MAX_HIDDEN = 4
OK, INVALID_ARG, UNSUPPORTED, WORKSPACE_TOO_SMALL, DEVICE_ERROR = range(5)
ADAM, SGD = 0, 1
F32, BF16 = 0, 1

EXPORTS = ["bbo_mlp_workspace_bytes", "bbo_mlp_cv_eval", "bbo_mlp_cv_eval_static", "bbo_mlp_cv_eval_traced", "bbo_mlp_fold_lists",
           "bbo_mlp_holdout_eval", "bbo_mlp_holdout_lists", "bbo_mlp_minibatch_rows", "bbo_mlp_init_params", "bbo_mlp_param_count", "bbo_mlp_kernel_class",
           "bbo_mlp_last_error"]


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


class BboError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("bbo_mlp error %d: %s" % (code, msg))
        self.code = code


_lib = None


def lib():
    """Load the shared library (built by paper_2012_04201_amd/build.py)."""
    global _lib
    if _lib is None:
        path = os.environ.get("BBO_MLP_LIB", LIB_PATH)  # override: an alternative build of the same ABI
        if not os.path.exists(path):
            raise ImportError("libbbo_mlp.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(path)
        L.bbo_mlp_last_error.restype = C.c_char_p
        L.bbo_mlp_param_count.restype = C.c_int64
        _lib = L
    return _lib


def _check(rc):
    if rc != OK:
        raise BboError(rc, lib().bbo_mlp_last_error().decode())


def make_hparams(dicts):
    arr = (HParams * max(len(dicts), 1))()
    for h, dct in zip(arr, dicts):
        hidden = list(dct.get("hidden", []))
        h.n_hidden = len(hidden)
        for i, w in enumerate(hidden[:MAX_HIDDEN]):
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


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def _check_inputs(X, y, fold_idx, n_classes, dtype):
    """The library takes plain pointers: the tensors must be dense, on one device and of the types it reads."""
    if X.dim() != 2 or not X.is_contiguous():
        raise ValueError("X must be a contiguous [n, d] tensor")
    if X.dtype != (torch.bfloat16 if dtype == BF16 else torch.float32):
        raise ValueError("X must be %s for this dtype" % ("bfloat16" if dtype == BF16 else "float32"))
    if not y.is_contiguous() or y.shape[0] != X.shape[0] or (
            n_classes >= 0 and y.dtype != (torch.int32 if n_classes >= 1 else torch.float32)):
        raise ValueError("y must be a contiguous [n] tensor, int32 for classification, float32 for regression")
    if not fold_idx.is_contiguous() or fold_idx.shape[0] != X.shape[0] or fold_idx.dtype != torch.int32:
        raise ValueError("fold_idx must be a contiguous int32 [n] tensor")
    if not (X.device == y.device == fold_idx.device) or X.device.type != "cuda":
        raise ValueError("X, y and fold_idx must be on the same GPU")


def _new(stream, *args, **kw):
    """A tensor the kernels of `stream` will use: allocated under that stream, so that the caching allocator
    does not hand the block to other work while they run."""
    if stream is None:
        return torch.empty(*args, **kw)
    with torch.cuda.stream(stream):
        return torch.empty(*args, **kw)


def _stream(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def to_device(cfg, device="cuda:0"):
    """inputs.make_config() dict -> device tensors (X as float32 or bfloat16)."""
    X = cfg["X"]
    if cfg["dtype"] == BF16:
        Xt = torch.from_numpy(np.ascontiguousarray(X).view(np.int16)).to(device).view(torch.bfloat16)
    else:
        Xt = torch.from_numpy(np.ascontiguousarray(X, dtype=np.float32)).to(device)
    ydt = np.int32 if cfg["n_classes"] >= 1 else np.float32
    yt = torch.from_numpy(np.ascontiguousarray(cfg["y"], dtype=ydt)).to(device)
    ft = torch.from_numpy(np.ascontiguousarray(cfg["fold_idx"], dtype=np.int32)).to(device)
    return Xt, yt, ft


def bbo_mlp_param_count(d, n_classes, hp):
    h = make_hparams([hp])
    return int(lib().bbo_mlp_param_count(C.c_int32(d), C.c_int32(n_classes), h))


KERNEL_TILED, KERNEL_SMALL, KERNEL_LINEAR, KERNEL_GENERIC, KERNEL_MID = range(5)


def bbo_mlp_kernel_class(n, d, n_classes, hp, dtype=F32):
    h = make_hparams([hp])
    return int(lib().bbo_mlp_kernel_class(C.c_int64(n), C.c_int32(d), C.c_int32(n_classes), h, C.c_int32(dtype)))


def bbo_mlp_workspace_bytes(n, d, n_classes, n_folds, hps, dtype, hp_arr=None):
    h = hp_arr if hp_arr is not None else make_hparams(hps)
    out = C.c_size_t(0)
    _check(lib().bbo_mlp_workspace_bytes(C.c_int64(n), C.c_int32(d), C.c_int32(n_classes), C.c_int32(n_folds), h,
                                         C.c_int32(len(hps)), C.c_int32(dtype), C.byref(out)))
    return out.value


def alloc_workspace(nbytes, device):
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def bbo_mlp_cv_eval(X, y, n_classes, fold_idx, n_folds, hps, dtype=F32, workspace=None, stream=None,
                    want_per_fold=False, hp_arr=None, trace=None):
    """Evaluate a list of suggestions.  X, y, fold_idx: CUDA tensors.

    trace = (b, fold, step_begin, step_end[, state_in]) records those steps of
    one model; state_in (float32 [3P] CUDA tensor) resumes it at step_begin.
    Returns (scores[B,2], status[B]) and, if asked, per_fold[B,K,2] and the
    trace dict(loss[T], grad[T,P], theta_after[T,P]) — all device tensors.
    """
    _check_inputs(X, y, fold_idx, n_classes, dtype)
    dev = X.device
    n, d = (int(X.shape[0]), int(X.shape[1]))
    B = len(hps)
    h = hp_arr if hp_arr is not None else make_hparams(hps)
    if workspace is None:
        workspace = _new(stream, max(bbo_mlp_workspace_bytes(n, d, n_classes, n_folds, hps, dtype, h), 256),
                         dtype=torch.uint8, device=dev)
    scores = _new(stream, (max(B, 1), 2), dtype=torch.float32, device=dev)
    status = _new(stream, max(B, 1), dtype=torch.int32, device=dev)
    pf = _new(stream, (max(B, 1), n_folds, 2), dtype=torch.float32, device=dev) if want_per_fold else None
    common = [_ptr(X), _ptr(y), C.c_int64(n), C.c_int32(d), C.c_int32(n_classes), _ptr(fold_idx), C.c_int32(n_folds),
              h, C.c_int32(B), C.c_int32(dtype), _ptr(scores), _ptr(status), _ptr(pf), _ptr(workspace),
              C.c_size_t(workspace.numel()), _stream(stream)]
    out = [scores[:B], status[:B]]
    if trace is None:
        _check(lib().bbo_mlp_cv_eval(*common))
    else:
        tb, tf, s0, s1 = trace[:4]
        state_in = trace[4] if len(trace) > 4 else None
        P = bbo_mlp_param_count(d, n_classes, hps[tb]) if 0 <= tb < B else 0
        T = max(s1 - s0, 0)
        tr = torch.full((max(T, 1), 1 + 2 * P), float("nan"), dtype=torch.float32, device=dev)
        _check(lib().bbo_mlp_cv_eval_traced(*common, C.c_int32(tb), C.c_int32(tf), C.c_int64(s0), C.c_int64(s1),
                                            _ptr(tr), C.c_size_t(tr.numel()), _ptr(state_in)))
    if want_per_fold:
        out.append(pf[:B])
    if trace is not None:
        out.append({"loss": tr[:T, 0], "grad": tr[:T, 1:1 + P], "theta_after": tr[:T, 1 + P:]})
    return tuple(out)


def bbo_mlp_cv_eval_static(X, y, n_classes, fold_idx, n_folds, hps, dtype=F32, scores=None, status=None, per_fold=None,
                           stream=None, hp_arr=None):
    """bbo_mlp_cv_eval on the library's static workspace: allocates nothing when the caller passes the
    output tensors (scores float32 [B,2], status int32 [B], optionally per_fold float32 [B,K,2]).
    Returns (scores, status)."""
    _check_inputs(X, y, fold_idx, n_classes, dtype)
    B = len(hps)
    h = hp_arr if hp_arr is not None else make_hparams(hps)
    if scores is None:
        scores = _new(stream, (max(B, 1), 2), dtype=torch.float32, device=X.device)
    if status is None:
        status = _new(stream, max(B, 1), dtype=torch.int32, device=X.device)
    _check(lib().bbo_mlp_cv_eval_static(_ptr(X), _ptr(y), C.c_int64(int(X.shape[0])), C.c_int32(int(X.shape[1])),
                                        C.c_int32(n_classes), _ptr(fold_idx), C.c_int32(n_folds), h, C.c_int32(B),
                                        C.c_int32(dtype), _ptr(scores), _ptr(status), _ptr(per_fold), _stream(stream)))
    return scores[:B], status[:B]


def bbo_mlp_holdout_eval(X, y, n_classes, fold_idx, hps, dtype=F32, workspace=None, stream=None, hp_arr=None):
    """Hold-out scores of a list of suggestions: trained on the rows with fold_idx >= 0, scored on the
    rows with fold_idx < 0.  Returns (scores[B,2], status[B]) device tensors."""
    _check_inputs(X, y, fold_idx, n_classes, dtype)
    dev = X.device
    n, d = (int(X.shape[0]), int(X.shape[1]))
    B = len(hps)
    h = hp_arr if hp_arr is not None else make_hparams(hps)
    if workspace is None:
        workspace = _new(stream, max(bbo_mlp_workspace_bytes(n, d, n_classes, 1, hps, dtype, h), 256), dtype=torch.uint8,
                         device=dev)
    scores = _new(stream, (max(B, 1), 2), dtype=torch.float32, device=dev)
    status = _new(stream, max(B, 1), dtype=torch.int32, device=dev)
    _check(lib().bbo_mlp_holdout_eval(_ptr(X), _ptr(y), C.c_int64(n), C.c_int32(d), C.c_int32(n_classes),
                                      _ptr(fold_idx), h, C.c_int32(B), C.c_int32(dtype), _ptr(scores), _ptr(status),
                                      _ptr(workspace), C.c_size_t(workspace.numel()), _stream(stream)))
    return scores[:B], status[:B]


def bbo_mlp_holdout_lists(fold_idx, stream=None):
    """-> (train_idx[n], val_idx[n], counts[2]) int32 device tensors."""
    n = int(fold_idx.shape[0])
    dev = fold_idx.device
    tr = torch.full((max(n, 1),), -1, dtype=torch.int32, device=dev)
    va = torch.full((max(n, 1),), -1, dtype=torch.int32, device=dev)
    cnt = torch.zeros(2, dtype=torch.int32, device=dev)
    _check(lib().bbo_mlp_holdout_lists(_ptr(fold_idx), C.c_int64(n), _ptr(tr), _ptr(va), _ptr(cnt), _stream(stream)))
    return tr, va, cnt


def bbo_mlp_fold_lists(fold_idx, n_folds, stream=None):
    """-> (train_idx[K,n], val_idx[K,n], counts[K,2]) int32 device tensors."""
    n = int(fold_idx.shape[0])
    dev = fold_idx.device
    tr = torch.full((n_folds, max(n, 1)), -1, dtype=torch.int32, device=dev)
    va = torch.full((n_folds, max(n, 1)), -1, dtype=torch.int32, device=dev)
    cnt = torch.zeros((n_folds, 2), dtype=torch.int32, device=dev)
    _check(lib().bbo_mlp_fold_lists(_ptr(fold_idx), C.c_int64(n), C.c_int32(n_folds), _ptr(tr), _ptr(va), _ptr(cnt),
                                    _stream(stream)))
    return tr, va, cnt


def bbo_mlp_minibatch_rows(train_idx, counts, n, hp, fold, epoch, step, stream=None):
    """Rows of one minibatch; step = -1: the rows the model sets aside for early stopping."""
    dev = train_idx.device
    rows = torch.full((max(n, 1),), -1, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    h = make_hparams([hp])
    _check(lib().bbo_mlp_minibatch_rows(_ptr(train_idx), _ptr(counts), C.c_int64(n), h, C.c_int32(fold),
                                        C.c_int32(epoch), C.c_int64(step), _ptr(rows), _ptr(cnt), _stream(stream)))
    return rows[: int(cnt.item())]


def bbo_mlp_init_params(d, n_classes, hp, fold, device="cuda:0", stream=None):
    P = bbo_mlp_param_count(d, n_classes, hp)
    out = torch.empty(P, dtype=torch.float32, device=device)
    h = make_hparams([hp])
    _check(lib().bbo_mlp_init_params(C.c_int32(d), C.c_int32(n_classes), h, C.c_int32(fold), _ptr(out),
                                     _stream(stream)))
    return out
