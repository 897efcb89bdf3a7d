"""Pins for the oracle's objectives and gradients (no GPU).

The paper never fixes F_i, so the gradient code is pinned to things outside the
oracle: central finite differences, torch.autograd in float64 (an independent
library routine), scipy's log-softmax, the least-squares closed form, and
torch's float32 -> bfloat16 conversion for the rounding helper.
"""
import numpy as np
import pytest
import torch
from scipy.special import log_softmax

from oracle.models import (lsq_loss_grad, mlp_loss_grad, mlp_unflatten, round_bf16)
from workloads import make_gmm_data, make_lsq_data, make_x0


def _fd_grad(f, x, eps=1e-6):
    g = np.zeros_like(x)
    for k in range(x.size):
        e = np.zeros_like(x)
        e[k] = eps
        g[k] = (f(x + e) - f(x - e)) / (2 * eps)
    return g


def test_lsq_gradient_finite_differences_and_closed_form():
    feats, targs = make_lsq_data(1, 32, 6, seed=5)
    a, y = feats[0][:9].astype(np.float64), targs[0][:9].astype(np.float64)
    x = np.linspace(-1, 1, 6)
    loss, g = lsq_loss_grad(x, a, y)
    # value: half the mean squared residual, written out row by row
    want = sum((a[j] @ x - y[j]) ** 2 for j in range(9)) / (2 * 9)
    assert loss == pytest.approx(want, rel=1e-13)
    fd = _fd_grad(lambda v: lsq_loss_grad(v, a, y)[0], x)
    assert np.allclose(g, fd, rtol=1e-7, atol=1e-9)
    # the gradient vanishes exactly at the normal-equation solution of the batch
    xs = np.linalg.lstsq(a, y, rcond=None)[0]
    assert np.abs(lsq_loss_grad(xs, a, y)[1]).max() < 1e-12


@pytest.mark.parametrize("activation", ["tanh", "relu"])
def test_mlp_gradient_finite_differences(activation):
    dims = (5, 4, 3, 3)
    feats, labels = make_gmm_data(1, 16, 5, 3, seed=9)
    a, c = feats[0][:7], labels[0][:7]
    x = make_x0("mlp", dims, activation, seed=4).astype(np.float64)
    x += 0.05 * np.random.default_rng(1).standard_normal(x.size)   # non-zero biases
    loss, g = mlp_loss_grad(x, dims, activation, a, c)
    fd = _fd_grad(lambda v: mlp_loss_grad(v, dims, activation, a, c)[0], x)
    assert np.allclose(g, fd, rtol=2e-6, atol=2e-8)


@pytest.mark.parametrize("activation", ["tanh", "relu"])
@pytest.mark.parametrize("dims", [(12, 9, 4), (10, 8, 6, 5), (7, 3)])
def test_mlp_loss_and_gradient_match_torch_autograd(activation, dims):
    feats, labels = make_gmm_data(1, 64, dims[0], dims[-1], seed=2)
    a, c = feats[0][:13], labels[0][:13]
    x = make_x0("mlp", dims, activation, seed=8).astype(np.float64)
    x += 0.1 * np.random.default_rng(3).standard_normal(x.size)
    loss, g = mlp_loss_grad(x, dims, activation, a, c)

    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    h = torch.tensor(a, dtype=torch.float64)
    off = 0
    for l in range(len(dims) - 1):
        w = xt[off:off + dims[l] * dims[l + 1]].reshape(dims[l], dims[l + 1])
        off += dims[l] * dims[l + 1]
        b = xt[off:off + dims[l + 1]]
        off += dims[l + 1]
        h = h @ w + b
        if l < len(dims) - 2:
            h = torch.tanh(h) if activation == "tanh" else torch.relu(h)
    lt = torch.nn.functional.cross_entropy(h, torch.tensor(c, dtype=torch.long))
    lt.backward()
    assert loss == pytest.approx(float(lt.detach()), rel=1e-12)
    assert np.allclose(g, xt.grad.numpy(), rtol=1e-10, atol=1e-13)


def test_mlp_loss_is_mean_negative_log_softmax():
    dims = (6, 5)
    feats, labels = make_gmm_data(1, 16, 6, 5, seed=3)
    a, c = feats[0][:8].astype(np.float64), labels[0][:8]
    x = np.random.default_rng(0).standard_normal(6 * 5 + 5)
    (w, b), = mlp_unflatten(x, dims)
    want = -log_softmax(a @ w + b, axis=1)[np.arange(8), c].mean()
    assert mlp_loss_grad(x, dims, "relu", a, c)[0] == pytest.approx(want, rel=1e-13)


def test_mlp_softmax_is_shift_invariant_and_stable_for_large_logits():
    dims = (3, 4)
    a = np.array([[1000.0, -1000.0, 500.0]])
    c = np.array([2])
    x = np.concatenate([np.eye(3, 4).ravel(), np.zeros(4)])
    loss, g = mlp_loss_grad(x, dims, "relu", a, c)
    assert np.isfinite(loss) and np.all(np.isfinite(g))
    # logits (1000, -1000, 500, 0): loss = 1000 - 500 up to exp(-500)
    assert loss == pytest.approx(500.0, rel=1e-12)


def test_mlp_bias_gradient_rows_sum_to_zero_and_relu_kink_convention():
    # softmax - onehot sums to zero across classes, so the last-layer bias gradient does too
    dims = (4, 3, 5)
    feats, labels = make_gmm_data(1, 16, 4, 5, seed=6)
    x = make_x0("mlp", dims, "relu", seed=1).astype(np.float64)
    _, g = mlp_loss_grad(x, dims, "relu", feats[0][:6], labels[0][:6])
    gb_last = mlp_unflatten(g, dims)[-1][1]
    assert abs(gb_last.sum()) < 1e-15
    # phi'(0) = 0 for ReLU: with all-zero first layer the hidden units sit exactly on the
    # kink, so nothing flows back into W_1
    x0 = x.copy()
    mlp_unflatten(x0, dims)[0][0][...] = 0.0
    _, g0 = mlp_loss_grad(x0, dims, "relu", feats[0][:6], labels[0][:6])
    assert np.all(mlp_unflatten(g0, dims)[0][0] == 0.0)


def test_round_bf16_matches_torch_conversion_including_ties():
    rng = np.random.default_rng(0)
    vals = np.concatenate([
        rng.standard_normal(4000).astype(np.float32) * np.float32(3.0),
        np.float32(2.0) ** rng.integers(-30, 30, 500).astype(np.float32),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, -1.00390625, 3.3895314e38,
                  1e-40, 65504.0], dtype=np.float32),
    ])
    want = torch.tensor(vals).to(torch.bfloat16).to(torch.float32).numpy()
    got = round_bf16(vals).astype(np.float32)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_bf16_mode_rounds_operands_only():
    # With inputs and weights already representable in bf16 and a single layer, the only
    # rounding left is delta: loss equals the unrounded loss exactly.
    dims = (4, 3)
    a = np.array([[1.0, 0.5, -2.0, 0.25], [0.0, 1.5, 1.0, -1.0]])
    c = np.array([0, 2])
    x = np.array([0.5, -1.0, 2.0, 1.0, 0.0, -0.5, 0.25, 4.0, 1.0, -2.0, 0.5, 1.0, 0.1, 0.2, 0.3])
    x[:12] = round_bf16(x[:12])
    l32, g32 = mlp_loss_grad(x, dims, "relu", a, c, bf16=False)
    l16, g16 = mlp_loss_grad(x, dims, "relu", a, c, bf16=True)
    assert l16 == l32
    assert np.abs(g16 - g32).max() <= 2.0 ** -7 * np.abs(g32).max()
    assert not np.array_equal(g16, g32)
    # and a weight that is not representable changes the loss
    x[0] = 0.5 + 2.0 ** -10
    assert mlp_loss_grad(x, dims, "relu", a, c, bf16=True)[0] != \
        mlp_loss_grad(x, dims, "relu", a, c, bf16=False)[0]
