"""Pins for the oracle's minibatch gradients (Algorithm 1 step 3 with footnote [a]).

Two independent comparators: central finite differences of the oracle's own loss (catches any
backward mistake) and PyTorch-CPU fp64 autograd over library ops written in the test (catches
forward mistakes: a dropped bias, a transposed weight, a wrong stride or shortcut)."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from paper_1705_09056_amd import synth
from paper_1705_09056_amd.configs import CONFIGS

from conftest import rel_err


def finite_diff(kind, widths, x, inp, tgt, idx, h=1e-6):
    g = np.zeros(len(idx))
    for t, c in enumerate(idx):
        e = h * max(1.0, abs(x[c]))
        xp, xm = x.copy(), x.copy()
        xp[c] += e
        xm[c] -= e
        g[t] = (oracle.loss_grad(kind, widths, xp, inp, tgt, False)[0]
                - oracle.loss_grad(kind, widths, xm, inp, tgt, False)[0]) / (2 * e)
    return g


def test_model_dims_match_the_benchmark_definition():
    assert oracle.model_dim(oracle.LSQ, [64]) == 64
    assert oracle.model_dim(oracle.SOFTMAX, [3072, 10]) == 3072 * 10 + 10
    assert oracle.model_dim(oracle.MLP, [3072, 1024, 10]) == 3157002
    assert oracle.model_dim(oracle.MLP, [3072, 4096, 4096, 10]) == 29409290
    d = oracle.model_dim(oracle.RESNET20, [3, 32, 32, 16, 3, 10])
    assert d == 267696 + 650 + 19        # ~0.27M parameters
    for cfg in CONFIGS:                   # the generator's layout agrees
        assert synth.model_dim(cfg.model_kind, cfg.widths) == oracle.model_dim(cfg.model_kind, cfg.widths)


# ------------------------------------------------------------------ least squares
def test_lsq_gradient_closed_form_and_fd():
    rng = np.random.default_rng(1)
    B, Fd = 9, 6
    A = rng.standard_normal((B, Fd))
    y = rng.standard_normal(B)
    x = rng.standard_normal(Fd)
    loss, g = oracle.loss_grad(oracle.LSQ, [Fd], x, A, y)
    # normal-equation form via library routines
    assert loss == pytest.approx(0.5 / B * np.linalg.norm(A @ x - y) ** 2, rel=1e-13)
    np.testing.assert_allclose(g, (A.T @ A @ x - A.T @ y) / B, atol=1e-13)
    np.testing.assert_allclose(g, finite_diff(oracle.LSQ, [Fd], x, A, y, range(Fd)), rtol=1e-6, atol=1e-8)
    # the minimiser of the batch objective has zero gradient
    xs = np.linalg.lstsq(A, y, rcond=None)[0]
    assert np.abs(oracle.loss_grad(oracle.LSQ, [Fd], xs, A, y)[1]).max() < 1e-13


# ----------------------------------------------------------- softmax regression / MLP
def torch_mlp(widths, x, inp, lab):
    xs = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    a = torch.tensor(inp, dtype=torch.float64)
    off = 0
    L = len(widths) - 1
    for l in range(L):
        O, I = widths[l + 1], widths[l]
        W = xs[off:off + O * I].reshape(O, I)
        off += O * I
        b = xs[off:off + O]
        off += O
        a = F.linear(a, W, b)
        if l < L - 1:
            a = F.relu(a)
    loss = F.cross_entropy(a, torch.tensor(lab, dtype=torch.long))
    loss.backward()
    return float(loss.detach()), xs.grad.numpy()


@pytest.mark.parametrize("kind,widths", [(oracle.SOFTMAX, [7, 4]), (oracle.MLP, [5, 6, 3]), (oracle.MLP, [4, 3, 5, 2])])
def test_mlp_against_autograd_and_fd(kind, widths):
    rng = np.random.default_rng(sum(widths))
    B = 5
    d = oracle.model_dim(kind, widths)
    x = rng.standard_normal(d) * 0.7
    inp = rng.standard_normal((B, widths[0]))
    lab = rng.integers(0, widths[-1], B).astype(np.int32)
    loss, g = oracle.loss_grad(kind, widths, x, inp, lab)
    tl, tg = torch_mlp(widths, x, inp, lab)
    assert loss == pytest.approx(tl, rel=1e-12)
    np.testing.assert_allclose(g, tg, atol=1e-13)
    fd = finite_diff(kind, widths, x, inp, lab, range(d))
    assert rel_err(g, fd) < 1e-6
    # softmax rows sum to one => the gradient w.r.t. the last bias sums to zero
    assert abs(g[-widths[-1]:].sum()) < 1e-14


def test_cross_entropy_at_zero_weights_is_log_classes():
    rng = np.random.default_rng(0)
    widths = [12, 10]
    x = np.zeros(oracle.model_dim(oracle.SOFTMAX, widths))
    inp = rng.standard_normal((6, 12))
    lab = rng.integers(0, 10, 6).astype(np.int32)
    loss, g = oracle.loss_grad(oracle.SOFTMAX, widths, x, inp, lab)
    assert loss == pytest.approx(math.log(10.0), rel=1e-15)
    # at zero weights softmax = 1/10: dW[c] = mean_b (1/10 - [c == label_b]) a_b
    ref = np.zeros((10, 12))
    for b in range(6):
        p = np.full(10, 0.1)
        p[lab[b]] -= 1.0
        ref += np.outer(p, inp[b]) / 6
    np.testing.assert_allclose(g[:120].reshape(10, 12), ref, atol=1e-15)


def test_logits_are_stabilised():
    widths = [3, 4]
    x = np.zeros(oracle.model_dim(oracle.SOFTMAX, widths))
    x[-4:] = [800.0, -800.0, 0.0, 799.0]
    inp = np.zeros((2, 3))
    loss, g = oracle.loss_grad(oracle.SOFTMAX, widths, x, inp, np.array([0, 3], dtype=np.int32))
    assert np.isfinite(loss) and np.all(np.isfinite(g))
    assert loss == pytest.approx(0.5 * (math.log1p(math.exp(-1.0)) + 1.0 + math.log1p(math.exp(-1.0))), rel=1e-12)


# ------------------------------------------------------------------------- CNN
def torch_resnet(widths, x, inp, lab):
    cin, H, W, base, blocks, classes = widths
    xs = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    B = inp.shape[0]
    a = torch.tensor(inp, dtype=torch.float64).reshape(B, cin, H, W)
    off = 0

    def take(shape):
        nonlocal off
        n = int(np.prod(shape))
        t = xs[off:off + n].reshape(shape)
        off += n
        return t

    w = take((base, cin, 3, 3))
    b = take((1,))
    a = F.relu(F.conv2d(a, w, padding=1) + b)
    cprev = base
    for s in range(3):
        c = base << s
        for j in range(blocks):
            stride = 2 if (s > 0 and j == 0) else 1
            w1, b1 = take((c, cprev, 3, 3)), take((1,))
            w2, b2 = take((c, c, 3, 3)), take((1,))
            u = F.relu(F.conv2d(a, w1, stride=stride, padding=1) + b1)
            v = F.conv2d(u, w2, padding=1) + b2
            sc = a
            if stride == 2:
                sc = F.pad(a[:, :, ::2, ::2], (0, 0, 0, 0, 0, c - cprev))
            a = F.relu(v + sc)
            cprev = c
    pooled = a.mean(dim=(2, 3))
    wf, bf = take((classes, cprev)), take((classes,))
    loss = F.cross_entropy(F.linear(pooled, wf, bf), torch.tensor(lab, dtype=torch.long))
    loss.backward()
    assert off == x.size
    return float(loss.detach()), xs.grad.numpy()


@pytest.mark.parametrize("widths,B", [([2, 6, 6, 2, 1, 3], 2), ([3, 8, 8, 4, 3, 10], 3), ([3, 7, 5, 2, 2, 4], 2)])
def test_resnet_against_autograd(widths, B):
    rng = np.random.default_rng(sum(widths))
    d = oracle.model_dim(oracle.RESNET20, widths)
    x = rng.standard_normal(d) * 0.4
    inp = rng.standard_normal((B, widths[0] * widths[1] * widths[2]))
    lab = rng.integers(0, widths[-1], B).astype(np.int32)
    loss, g = oracle.loss_grad(oracle.RESNET20, widths, x, inp, lab)
    tl, tg = torch_resnet(widths, x, inp, lab)
    assert loss == pytest.approx(tl, rel=1e-12)
    assert rel_err(g, tg) < 1e-12
    assert abs(g[-widths[-1]:].sum()) < 1e-13


def test_resnet_finite_differences():
    widths = [2, 6, 6, 2, 1, 3]
    rng = np.random.default_rng(77)
    d = oracle.model_dim(oracle.RESNET20, widths)
    x = rng.standard_normal(d) * 0.5
    inp = rng.standard_normal((1, 72))
    lab = np.array([2], dtype=np.int32)
    _, g = oracle.loss_grad(oracle.RESNET20, widths, x, inp, lab)
    idx = rng.choice(d, size=60, replace=False)
    fd = finite_diff(oracle.RESNET20, widths, x, inp, lab, idx)
    assert rel_err(g[idx], fd) < 1e-6


def test_grad_all_equals_per_worker_calls():
    widths = [6, 5, 3]
    rng = np.random.default_rng(2)
    n, B = 4, 3
    d = oracle.model_dim(oracle.MLP, widths)
    X = rng.standard_normal((n, d))
    inp = rng.standard_normal((n, B, 6))
    lab = rng.integers(0, 3, (n, B)).astype(np.int32)
    G, loss = oracle.grad_all(oracle.MLP, widths, X, inp, lab)
    for i in range(n):
        li, gi = oracle.loss_grad(oracle.MLP, widths, X[i], inp[i], lab[i])
        assert loss[i] == li
        assert np.array_equal(G[i], gi)
