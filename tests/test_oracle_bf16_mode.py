"""Pins for the oracle's "bf16 operands" mode: every operand of a contraction (weights, stored
activations, back-propagated deltas) rounded to bf16, sums in fp64.  Comparator: PyTorch-CPU fp64
autograd in which the same roundings are inserted with torch's own bf16 cast (straight-through in
the forward direction, a rounding hook in the backward direction)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from paper_1705_09056_amd import synth

from conftest import rel_err


class Casts:
    """The roundings of the bf16 workloads as torch operations in arithmetic type `dtype`; with casts=False every
    one of them is the identity (plain autograd)."""

    def __init__(self, dtype=torch.float64, casts=True):
        self.dtype, self.casts = dtype, casts
        outer = self

        class RoundGrad(torch.autograd.Function):
            """Identity whose incoming gradient is rounded to bf16."""

            @staticmethod
            def forward(ctx, x):
                return x.clone()

            @staticmethod
            def backward(ctx, g):
                return outer.tq(g)

        self.round_grad = RoundGrad.apply

    def tq(self, x):
        return x.to(torch.bfloat16).to(self.dtype) if self.casts else x

    def rq(self, x):
        """Value rounded to bf16, gradient passed through unchanged."""
        return x + (self.tq(x) - x).detach()


def torch_mlp_bf16(widths, x, inp, lab, dtype=torch.float64, casts=True):
    c = Casts(dtype, casts)
    xs = torch.tensor(x, dtype=dtype, requires_grad=True)
    a = c.tq(torch.tensor(inp, dtype=dtype))
    off, L = 0, len(widths) - 1
    for l in range(L):
        O, I = widths[l + 1], widths[l]
        W = xs[off:off + O * I].reshape(O, I); off += O * I
        b = xs[off:off + O]; off += O
        z = c.round_grad(F.linear(a, c.rq(W), b))
        a = c.rq(F.relu(z)) if l < L - 1 else z
    loss = F.cross_entropy(a, torch.tensor(lab, dtype=torch.long))
    loss.backward()
    return float(loss.detach()), xs.grad.double().numpy()


@pytest.mark.parametrize("kind,widths", [(oracle.SOFTMAX, [9, 4]), (oracle.MLP, [12, 10, 5]), (oracle.MLP, [8, 7, 6, 3])])
def test_mlp_bf16_mode_against_autograd_with_casts(kind, widths):
    rng = np.random.default_rng(sum(widths) + 1)
    B = 6
    d = oracle.model_dim(kind, widths)
    x = (rng.standard_normal(d) * 0.6).astype(np.float32).astype(np.float64)
    inp = rng.standard_normal((B, widths[0]))
    lab = rng.integers(0, widths[-1], B).astype(np.int32)
    loss, g = oracle.loss_grad(kind, widths, x, inp, lab, bf16_operands=True)
    tl, tg = torch_mlp_bf16(widths, x, inp, lab)
    assert loss == pytest.approx(tl, rel=1e-12)
    assert rel_err(g, tg) < 1e-12
    # and the mode really rounds: it differs from the plain fp64 gradient at the bf16 level
    _, g_plain = oracle.loss_grad(kind, widths, x, inp, lab)
    assert 1e-5 < rel_err(g, g_plain) < 5e-2


def torch_resnet_bf16(widths, x, inp, lab, dtype=torch.float64, casts=True):
    q = Casts(dtype, casts)
    cin, H, W, base, blocks, classes = widths
    xs = torch.tensor(x, dtype=dtype, requires_grad=True)
    B = inp.shape[0]
    a = q.tq(torch.tensor(inp, dtype=dtype)).reshape(B, cin, H, W)
    off = 0

    def take(shape):
        nonlocal off
        n = int(np.prod(shape))
        t = xs[off:off + n].reshape(shape)
        off += n
        return t

    w, b = take((base, cin, 3, 3)), take((1,))
    a = q.rq(F.relu(q.round_grad(F.conv2d(a, q.rq(w), padding=1) + b)))
    cprev = base
    for s in range(3):
        c = base << s
        for j in range(blocks):
            stride = 2 if (s > 0 and j == 0) else 1
            w1, b1 = take((c, cprev, 3, 3)), take((1,))
            w2, b2 = take((c, c, 3, 3)), take((1,))
            u = q.rq(F.relu(q.round_grad(F.conv2d(a, q.rq(w1), stride=stride, padding=1) + b1)))
            sc = a if stride == 1 else F.pad(a[:, :, ::2, ::2], (0, 0, 0, 0, 0, c - cprev))
            a = q.rq(F.relu(q.round_grad(F.conv2d(u, q.rq(w2), padding=1) + b2 + sc)))
            cprev = c
    wf, bf = take((classes, cprev)), take((classes,))
    loss = F.cross_entropy(F.linear(a.mean(dim=(2, 3)), wf, bf), torch.tensor(lab, dtype=torch.long))
    loss.backward()
    return float(loss.detach()), xs.grad.double().numpy()


@pytest.mark.parametrize("widths,B", [([2, 6, 6, 2, 1, 3], 2), ([3, 8, 8, 4, 2, 10], 3)])
def test_resnet_bf16_mode_against_autograd_with_casts(widths, B):
    rng = np.random.default_rng(sum(widths) + 5)
    d = oracle.model_dim(oracle.RESNET20, widths)
    x = (rng.standard_normal(d) * 0.4).astype(np.float32).astype(np.float64)
    inp = rng.standard_normal((B, widths[0] * widths[1] * widths[2]))
    lab = rng.integers(0, widths[-1], B).astype(np.int32)
    loss, g = oracle.loss_grad(oracle.RESNET20, widths, x, inp, lab, bf16_operands=True)
    tl, tg = torch_resnet_bf16(widths, x, inp, lab)
    assert loss == pytest.approx(tl, rel=1e-12)
    assert rel_err(g, tg) < 1e-12


def test_rounding_is_nearest_even_like_the_input_generator():
    """The oracle's rounding, the generator's and torch's agree on ties and ordinary values: a
    1 x 1 'network' whose weight gradient is the rounded input."""
    vals = np.array([1.0, 1.00390625, 1.005859375, 1.01171875, 3.14159, -2.71828, 1e-20, 65504.0], dtype=np.float32)
    for v in vals:
        # softmax regression with one feature, two classes, zero weights: dW[c] = (1/2 - [c == 0]) * round(v)
        _, g = oracle.loss_grad(oracle.SOFTMAX, [1, 2], np.zeros(4), np.array([[v]], dtype=np.float64),
                                np.array([0], dtype=np.int32), bf16_operands=True)
        want = float(synth.round_to_bf16(np.array([v]))[0])
        assert want == float(torch.tensor([v]).to(torch.bfloat16).to(torch.float32)[0])
        # dz = (-1/2, 1/2) is exactly representable, so g[0] = -round(v)/2
        assert g[0] == -0.5 * want
