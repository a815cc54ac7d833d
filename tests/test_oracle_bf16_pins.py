"""Pins for the oracle's bfloat16 configuration on models WITH hidden layers.

The bf16 configuration rounds GEMM operands to bfloat16 at fixed points (weight copy, hidden activations
after ReLU, output deltas, hidden deltas; the data gradient contracts with the rounded weights; the bias
gradient sums the rounded deltas; the penalty sees the unrounded weights).  The reference below recomputes
loss and every layer's gradient with library float64 tensors and explicit library bfloat16 casts at exactly
those points, and a second test shows that the pin has teeth: the oracle is rebuilt on the CPU with each
rounding point switched off in turn, and every such mutant must fail the comparison."""
import ctypes as C
import os
import re
import subprocess

import numpy as np
import pytest
import torch

from paper_2012_04201_amd import inputs

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "mlp_cv_oracle.c")


def bf(t):
    """float64 tensor -> nearest bfloat16 (through float32, as a float32 pipeline would), back in float64."""
    return t.to(torch.float32).to(torch.bfloat16).to(torch.float64)


def problem(seed, n, d, n_classes):
    rng = np.random.default_rng(seed)
    Xf = (rng.normal(size=(n, d)) * rng.uniform(0.3, 2.0, size=d)).astype(np.float32)
    Xb = inputs.to_bf16_bits(Xf).reshape(n, d)
    if n_classes >= 1:
        y = rng.integers(0, max(n_classes, 2), size=n).astype(np.int32)
    else:
        y = (Xf[:, 0] - 0.5 * Xf[:, 1] + 0.1 * rng.normal(size=n)).astype(np.float32)
    return Xb, y


def reference(Xb, y, n_classes, rows, dims, theta, alpha):
    """Loss and packed gradient of the bf16 configuration, library float64 + explicit bfloat16 casts."""
    m = len(rows)
    L = len(dims) - 1
    th = torch.tensor(theta, dtype=torch.float64)
    Ws, bs, off = [], [], 0
    for l in range(L):
        fi, fo = dims[l], dims[l + 1]
        Ws.append(th[off:off + fi * fo].reshape(fi, fo))
        off += fi * fo
        bs.append(th[off:off + fo])
        off += fo
    Wop = [bf(W) for W in Ws]  # the weight copy the products see
    a = [torch.tensor(inputs.bf16_bits_to_f32(Xb[rows]).reshape(m, dims[0]).astype(np.float64))]
    for l in range(L):
        z = a[l] @ Wop[l] + bs[l]  # the bias is not an operand: added unrounded
        a.append(bf(torch.relu(z)) if l + 1 < L else z)
    z = a[L]
    if n_classes >= 2:
        yt = torch.tensor(y[rows].astype(np.int64))
        data = torch.nn.functional.cross_entropy(z, yt, reduction="mean")
        g = torch.softmax(z, dim=1)
        g[torch.arange(m), yt] -= 1.0
    elif n_classes == 1:
        yt = torch.tensor(y[rows].astype(np.float64))
        data = torch.nn.functional.binary_cross_entropy_with_logits(z[:, 0], yt, reduction="mean")
        g = (torch.sigmoid(z[:, 0]) - yt)[:, None]
    else:
        yt = torch.tensor(y[rows].astype(np.float64))
        data = 0.5 * torch.mean((z[:, 0] - yt) ** 2)
        g = (z[:, 0] - yt)[:, None]
    delta = bf(g / m)  # output deltas are operands of two products
    pen = sum((W * W).sum() for W in Ws)  # the unrounded weights
    loss = data + 0.5 * alpha * pen / m
    grads = [None] * L
    for l in range(L - 1, -1, -1):
        gW = a[l].T @ delta + (alpha / m) * Ws[l]
        gb = delta.sum(dim=0)  # the rounded deltas
        grads[l] = torch.cat([gW.reshape(-1), gb])
        if l > 0:
            delta = bf(delta @ Wop[l].T) * (a[l] > 0).to(torch.float64)  # mask from the rounded activation
    return float(loss), torch.cat(grads).numpy()


CASES = [
    # n_classes, hidden, alpha
    (3, [12], 0.3),
    (3, [10, 7], 0.3),
    (1, [9, 6], 0.05),
    (0, [8, 11], 0.2),
    (4, [16, 16, 5], 0.0),
]


def oracle_loss_grad(lib, Xb, y, n_classes, rows, hidden, alpha, theta):
    """oracle_loss_grad of an oracle build given as a ctypes handle, float64 mode with the bf16 roundings on."""
    from oracle import mlp_cv_oracle as O
    h = O.make_hparams([{"hidden": hidden, "alpha": alpha}])
    X = np.ascontiguousarray(Xb, dtype=np.uint16)
    yy = np.ascontiguousarray(y, dtype=np.int32 if n_classes >= 1 else np.float32)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    theta = np.ascontiguousarray(theta, dtype=np.float64)
    grad = np.zeros_like(theta)
    loss = C.c_double(0)
    p = lambda a: a.ctypes.data_as(C.c_void_p)
    rc = lib.oracle_loss_grad(p(X), p(yy), C.c_int64(X.shape[0]), C.c_int32(X.shape[1]), C.c_int32(n_classes),
                              p(rows), C.c_int64(rows.shape[0]), C.byref(h[0]), p(theta), C.c_int32(1), C.c_int32(1),
                              C.byref(loss), p(grad))
    assert rc == 0
    return loss.value, grad


def worst_mismatch(lib, oracle):
    """Largest relative deviation of loss / any layer's gradient from the reference over all cases."""
    worst = 0.0
    for ci, (n_classes, hidden, alpha) in enumerate(CASES):
        d = 16
        Xb, y = problem(100 + ci, 48, d, n_classes)
        dims = [d] + hidden + [n_classes if n_classes >= 2 else 1]
        hp = {"hidden": hidden, "alpha": alpha, "seed": 77 + ci}
        theta = oracle.init_params(d, n_classes, hp, 0)
        # a trained-looking state: bigger weights, so that deltas and activations spread over many binades
        theta = theta * np.random.default_rng(5 + ci).uniform(0.5, 3.0, size=theta.shape)
        rows = np.random.default_rng(9 + ci).permutation(48)[:37].astype(np.int32)
        a32 = float(np.float32(alpha))
        want_l, want_g = reference(Xb, y, n_classes, rows, dims, theta, a32)
        got_l, got_g = oracle_loss_grad(lib, Xb, y, n_classes, rows, hidden, alpha, theta)
        worst = max(worst, abs(got_l - want_l) / max(abs(want_l), 1e-30))
        off = 0
        for l in range(len(dims) - 1):
            for cnt in (dims[l] * dims[l + 1], dims[l + 1]):
                w, g = want_g[off:off + cnt], got_g[off:off + cnt]
                worst = max(worst, float(np.linalg.norm(g - w) / max(np.linalg.norm(w), 1e-30)))
                off += cnt
    return worst


TOL = 1e-11  # float64 summation order only; one skipped bfloat16 rounding moves a tensor by ~1e-3


def test_bf16_rounding_points_with_hidden_layers(oracle):
    assert worst_mismatch(oracle.lib(), oracle) < TOL


# Each entry switches ONE rounding point of the oracle off (pattern -> replacement on the lines marked BF).
MUTANTS = {
    "weight copy": (r"s->wop\[i\] = opnd\(theta\[i\], dt\)", "s->wop[i] = theta[i]"),
    "hidden activations": (r"z = opnd\(z, dt\); /\* BF: hidden activations \*/", "/* off */"),
    "softmax output deltas": (r"dl\[j\] = opnd\(rnd\(g / \(double\)m, prec\), D->dtype\)", "dl[j] = rnd(g / (double)m, prec)"),
    "one-logit output delta": (r"double g = rnd\(p - yr, prec\);\s*dl\[0\] = opnd\(rnd\(g / \(double\)m, prec\), D->dtype\)",
                               "double g = rnd(p - yr, prec); dl[0] = rnd(g / (double)m, prec)"),
    "regression output delta": (r"dl\[0\] = opnd\(rnd\(e / \(double\)m, prec\), D->dtype\)", "dl[0] = rnd(e / (double)m, prec)"),
    "hidden deltas": (r"v = opnd\(rnd\(acc, prec\), dt\)", "v = rnd(acc, prec)"),
    "data gradient through the rounded weights": (r"dl\[r \* fo \+ j\] \* Wop\[", "dl[r * fo + j] * W["),
    "bias gradient over the deltas as the products see them": (r"acc = accum\(acc, dl\[r \* fo \+ j\], prec\);", "acc = accum(acc, dl[r * fo + j] * (1.0 + 1e-3), prec);"),
    "ReLU mask of the data gradient": (r"if \(s->a\[l\]\[r \* fi \+ k\] > 0\.0\)", "if (s->a[l][r * fi + k] > 0.05)"),
    "penalty on the unrounded weights": (r"pen \+= W\[i\] \* W\[i\];", "pen += opnd(W[i], dt) * opnd(W[i], dt);"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pin_fails_when_a_rounding_point_is_switched_off(oracle, name, tmp_path):
    pat, rep = MUTANTS[name]
    src = open(SRC).read()
    mutated, n_sub = re.subn(pat, rep, src)
    assert n_sub == 1, "the oracle source no longer has the line this mutant edits: " + name
    c_file, so_file = tmp_path / "mutant.c", tmp_path / "libmutant.so"
    c_file.write_text(mutated)
    subprocess.run(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-o", str(so_file),
                    str(c_file), "-lm"], check=True)
    lib = C.CDLL(str(so_file))
    assert worst_mismatch(lib, oracle) > 1e-6, "a mutant oracle passes the pin: " + name
