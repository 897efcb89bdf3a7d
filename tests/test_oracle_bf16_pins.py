"""Pins for the oracle's bfloat16-operand mode on nets with hidden layers (no GPU).

The reading pinned here: the operands of every matrix product -- the gathered rows, the weights,
the hidden activations, the back-propagated deltas -- are rounded to bfloat16 (nearest, ties to
even); bias add, activation, its derivative, softmax and loss are not; the bias gradient sums
the rounded delta.  Two pins outside the oracle:
  * an emulation written out here with torch's float32 -> bfloat16 conversion (a library
    routine) around float64 products, on nets with one and two hidden layers;
  * a hand-sized net whose values are chosen so that every rounding point moves a known bit:
    the expected numbers below are worked out by hand in exact binary fractions.
"""
import math

import numpy as np
import pytest
import torch

from oracle.models import mlp_loss_grad, round_bf16
from workloads import make_gmm_data, make_x0


def _bf(t: torch.Tensor) -> torch.Tensor:
    return t.to(torch.float32).to(torch.bfloat16).to(torch.float64)


def _emulated(x, dims, activation, a, c):
    """Loss and gradient with every matrix-product operand passed through torch.bfloat16."""
    x = torch.tensor(x, dtype=torch.float64)
    ws, bs, off = [], [], 0
    for l in range(len(dims) - 1):
        ws.append(x[off:off + dims[l] * dims[l + 1]].reshape(dims[l], dims[l + 1]))
        off += dims[l] * dims[l + 1]
        bs.append(x[off:off + dims[l + 1]])
        off += dims[l + 1]
    nb = a.shape[0]
    hs = [_bf(torch.tensor(a, dtype=torch.float64))]
    for l in range(len(ws)):
        z = hs[-1] @ _bf(ws[l]) + bs[l]
        if l < len(ws) - 1:
            hs.append(_bf(torch.tanh(z) if activation == "tanh" else torch.relu(z)))
    logp = torch.log_softmax(z, dim=1)
    idx = torch.arange(nb)
    lab = torch.tensor(np.asarray(c), dtype=torch.long)
    loss = float(-logp[idx, lab].mean())
    p = torch.exp(logp)
    p[idx, lab] -= 1.0
    delta = _bf(p / nb)
    grads = [None] * len(ws)
    for l in range(len(ws) - 1, -1, -1):
        grads[l] = (hs[l].T @ delta, delta.sum(dim=0))
        if l > 0:
            dphi = (1.0 - hs[l] * hs[l]) if activation == "tanh" else (hs[l] > 0).to(torch.float64)
            delta = _bf((delta @ _bf(ws[l]).T) * dphi)
    flat = torch.cat([torch.cat([gw.reshape(-1), gb]) for gw, gb in grads])
    return loss, flat.numpy()


@pytest.mark.parametrize("activation", ["tanh", "relu"])
@pytest.mark.parametrize("dims", [(12, 9, 4), (10, 8, 6, 5), (33, 17, 20, 9, 3)])
def test_bf16_mode_matches_an_emulation_with_torch_bfloat16_casts(activation, dims):
    feats, labels = make_gmm_data(1, 64, dims[0], dims[-1], seed=12)
    a, c = feats[0][:11], labels[0][:11]
    x = make_x0("mlp", dims, activation, seed=5).astype(np.float64)
    x += 0.1 * np.random.default_rng(7).standard_normal(x.size)       # non-zero biases
    loss, g = mlp_loss_grad(x, dims, activation, a, c, bf16=True)
    want_loss, want_g = _emulated(x, dims, activation, a, c)
    assert loss == pytest.approx(want_loss, rel=1e-13)
    assert np.allclose(g, want_g, rtol=1e-12, atol=1e-16)
    # the rounding is not a no-op on this input
    loss64, g64 = mlp_loss_grad(x, dims, activation, a, c, bf16=False)
    assert abs(loss - loss64) > 1e-6 and np.abs(g - g64).max() > 1e-6


def test_every_rounding_point_moves_a_known_bit():
    # 1-1-2 ReLU net, two identical minibatch rows, label 0.  bfloat16 keeps 8 significant bits:
    # spacing 2^-7 in [1, 2), 2^-8 in [1/2, 1).
    #   input      a   = 1 + 2^-9                     -> bf16 1
    #   W_1            = 1 + 2^-9                     -> bf16 1
    #   b_1            = 2^-8 - 2^-12 (never rounded)
    #   z_1 = 1*1 + b_1 = 1 + 2^-8 - 2^-12, just below the tie 1 + 2^-8 -> h_1 = bf16(z_1) = 1.
    #     Any of: unrounded input, unrounded W_1, rounding before the bias add, an unrounded
    #     hidden activation puts h_1 off 1 and changes dW_2 = h_1^T delta_2.
    #   W_2 = [0, v],  v = 1 + 2^-7 + 2^-10             -> bf16 1 + 2^-7 = 129/128
    #   b_2 = [0, ln 2 - 129/128]  => logits [0, ln 2], softmax [1/3, 2/3], loss ln 3
    #   delta_2 rows = bf16([-2/3, 2/3] / 2):  2/3 = 0.101010101..b -> 0.10101011b = 171/256
    #   db_2 = column sums of the ROUNDED delta = [-171/256, 171/256]      (2/3 itself otherwise)
    #   back-propagated: (171/512) * (129/128) = 22059/65536 -> bf16 172/512 (round down);
    #     with an unrounded W_2 the product 171/512 * 1033/1024 lies above the midpoint
    #     172.5/512 and rounds UP to 173/512.
    #   dW_1 = sum over the two rows of a_q * delta_1 = 172/256,  db_1 = 172/256
    a = np.full((2, 1), 1.0 + 2.0 ** -9)
    c = np.array([0, 0])
    v = 1.0 + 2.0 ** -7 + 2.0 ** -10
    x = np.array([1.0 + 2.0 ** -9,                 # W_1
                  2.0 ** -8 - 2.0 ** -12,          # b_1
                  0.0, v,                          # W_2
                  0.0, math.log(2.0) - 129.0 / 128.0])   # b_2
    loss, g = mlp_loss_grad(x, (1, 1, 2), "relu", a, c, bf16=True)
    d = 171.0 / 256.0
    assert loss == pytest.approx(math.log(3.0), rel=1e-14)
    gw1, gb1, gw2, gb2 = g[0], g[1], g[2:4], g[4:6]
    assert np.array_equal(gb2, [-d, d])            # db from the rounded delta
    assert np.array_equal(gw2, [-d, d])            # h_1 rounded to exactly 1
    assert gb1 == 172.0 / 256.0                    # delta_1 rounded, with the rounded W_2
    assert gw1 == 172.0 / 256.0                    # the input rows are rounded too
    # the same net without the operand roundings gives none of these values
    loss64, g64 = mlp_loss_grad(x, (1, 1, 2), "relu", a, c, bf16=False)
    assert abs(loss64 - math.log(3.0)) > 1e-4
    assert g64[1] != 172.0 / 256.0 and g64[4] != -d


def test_round_bf16_keeps_nan_and_infinity():
    # a NaN whose payload would carry into the exponent under the rounding bias
    pats = np.array([0x7F800001, 0x7FFFFFFF, 0xFFFFFFFF, 0x7FC00000, 0x7F800000, 0xFF800000],
                    dtype=np.uint32).view(np.float32)
    got = round_bf16(pats)
    want = torch.tensor(pats).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.all(np.isnan(got[:4])) and np.all(np.isnan(want[:4]))
    assert got[4] == np.inf and got[5] == -np.inf
    # the largest finite floats round to infinity, as in torch's conversion
    big = np.array([3.4028235e38, -3.4028235e38], dtype=np.float32)
    assert np.array_equal(round_bf16(big).astype(np.float32),
                          torch.tensor(big).to(torch.bfloat16).to(torch.float32).numpy())


def _hand_case():
    a = np.full((2, 1), 1.0 + 2.0 ** -9)
    c = np.array([0, 0])
    v = 1.0 + 2.0 ** -7 + 2.0 ** -10
    x = np.array([1.0 + 2.0 ** -9, 2.0 ** -8 - 2.0 ** -12, 0.0, v, 0.0, math.log(2.0) - 129.0 / 128.0])
    return x, a, c


def _hand_case_holds():
    x, a, c = _hand_case()
    loss, g = mlp_loss_grad(x, (1, 1, 2), "relu", a, c, bf16=True)
    d = 171.0 / 256.0
    return (abs(loss - math.log(3.0)) <= 1e-13 and np.array_equal(g[4:6], [-d, d]) and
            np.array_equal(g[2:4], [-d, d]) and g[1] == 172.0 / 256.0 and g[0] == 172.0 / 256.0)


# the rounding points of a net with one hidden layer, in the order the computation reaches them
ROUNDING_POINTS = ["input rows", "W_1 (forward)", "hidden activation", "W_2 (forward)", "delta_2",
                   "W_2 (backward)", "back-propagated delta_1"]


@pytest.mark.parametrize("skip", range(len(ROUNDING_POINTS)), ids=ROUNDING_POINTS)
def test_hand_case_fails_when_one_rounding_is_forgotten(monkeypatch, skip):
    # the mistake is planted in the oracle, on the CPU: the skip-th rounding becomes the identity
    import oracle.models as om
    assert _hand_case_holds()
    calls = {"n": 0}
    real = om.round_bf16

    def forgetful(v):
        k = calls["n"]
        calls["n"] += 1
        return np.asarray(v, dtype=np.float64) if k == skip else real(v)

    monkeypatch.setattr(om, "round_bf16", forgetful)
    assert not _hand_case_holds(), ROUNDING_POINTS[skip]
    assert calls["n"] == len(ROUNDING_POINTS)
