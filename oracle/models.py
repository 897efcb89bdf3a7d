"""Stochastic objectives F_i(x; zeta) and their gradients for the oracle (test infrastructure).

The paper leaves F_i abstract (Section 1, eq. 1: f_i(x) = E_zeta F_i(x; zeta));
Algorithm 1 only needs G_i^t = grad F_i(x_i^{t-1}; zeta_i^t).  Two concrete
objectives are used, each a mean over the B rows of the minibatch zeta:

least squares
    F(x) = 1/(2B) sum_j (a_j . x - y_j)^2,      G = (1/B) A_b^T (A_b x - y_b)

MLP classifier (layer sizes d_0 .. d_L, hidden activation phi, last layer linear)
    h_0 = a,  h_l = phi(h_{l-1} W_l + b_l),  logits = h_{L-1} W_L + b_L
    F(x) = -(1/B) sum_j log softmax(logits_j)[c_j]
    delta_L = (softmax - onehot) / B
    dW_l = h_{l-1}^T delta_l,   db_l = column sums of delta_l
    delta_{l-1} = (delta_l W_l^T) * phi'(h_{l-1})        phi'(relu)(0) = 0

All arithmetic is float64.  With ``bf16=True`` the operands of every matrix
product (weights, activations h_l including the input rows, back-propagated
delta_l) are first rounded to bfloat16 (round to nearest, ties to even); bias
add, phi, phi', softmax, the loss, the gradients themselves and the update stay
unrounded.  The rounded delta_l is also what the bias gradient sums.

Flat parameter layout: [W_1 (d_0 x d_1, row-major), b_1, W_2, b_2, ...].
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np


def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round float values to the nearest bfloat16 (ties to even); returns float64.
    A NaN stays a NaN (the rounding bias must not carry its payload into the exponent)."""
    with np.errstate(invalid="ignore"):                       # signalling NaNs in the cast
        f = np.asarray(a, dtype=np.float64).astype(np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    rounded = (bits + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    out = rounded.astype(np.uint32).view(np.float32).astype(np.float64)
    out = np.where(np.isnan(f), np.nan, out)
    return out.reshape(np.shape(a))


def lsq_loss_grad(x: np.ndarray, a_b: np.ndarray, y_b: np.ndarray) -> Tuple[float, np.ndarray]:
    """Least-squares minibatch loss and gradient at x (float64)."""
    x = np.asarray(x, dtype=np.float64)
    a_b = np.asarray(a_b, dtype=np.float64)
    y_b = np.asarray(y_b, dtype=np.float64)
    nb = a_b.shape[0]
    r = a_b @ x - y_b
    loss = float(r @ r) / (2.0 * nb)
    grad = (a_b.T @ r) / nb
    return loss, grad


def mlp_unflatten(x: np.ndarray, dims: Sequence[int]) -> List[Tuple[np.ndarray, np.ndarray]]:
    """Split a flat parameter vector into [(W_l, b_l)] views."""
    out = []
    off = 0
    for l in range(len(dims) - 1):
        d_in, d_out = int(dims[l]), int(dims[l + 1])
        w = x[off:off + d_in * d_out].reshape(d_in, d_out)
        off += d_in * d_out
        b = x[off:off + d_out]
        off += d_out
        out.append((w, b))
    if off != x.shape[0]:
        raise ValueError("parameter vector length does not match dims")
    return out


def _phi(z: np.ndarray, activation: str) -> np.ndarray:
    if activation == "tanh":
        return np.tanh(z)
    if activation == "relu":
        return np.maximum(z, 0.0)
    raise ValueError(activation)


def _phi_prime_from_h(h: np.ndarray, activation: str) -> np.ndarray:
    if activation == "tanh":
        return 1.0 - h * h
    if activation == "relu":
        return (h > 0.0).astype(np.float64)
    raise ValueError(activation)


def mlp_loss_grad(x: np.ndarray, dims: Sequence[int], activation: str, a_b: np.ndarray,
                  c_b: np.ndarray, bf16: bool = False) -> Tuple[float, np.ndarray]:
    """Softmax cross-entropy minibatch loss of the MLP and its gradient w.r.t. the flat x."""
    x = np.asarray(x, dtype=np.float64)
    layers = mlp_unflatten(x, dims)
    n_layers = len(layers)
    nb = a_b.shape[0]
    q = round_bf16 if bf16 else (lambda v: v)

    # forward
    hs = [q(np.asarray(a_b, dtype=np.float64))]
    for l, (w, b) in enumerate(layers):
        z = hs[-1] @ q(w) + b
        if l < n_layers - 1:
            hs.append(q(_phi(z, activation)))
        else:
            logits = z
    zmax = logits.max(axis=1, keepdims=True)
    e = np.exp(logits - zmax)
    se = e.sum(axis=1, keepdims=True)
    logp = logits - zmax - np.log(se)
    rows = np.arange(nb)
    c_b = np.asarray(c_b, dtype=np.int64)
    loss = float(-logp[rows, c_b].sum() / nb)

    # backward
    p = e / se
    p[rows, c_b] -= 1.0
    delta = q(p / nb)
    grad = np.empty_like(x)
    gl = mlp_unflatten(grad, dims)
    for l in range(n_layers - 1, -1, -1):
        w, _ = layers[l]
        gw, gb = gl[l]
        gw[...] = hs[l].T @ delta
        gb[...] = delta.sum(axis=0)
        if l > 0:
            delta = q((delta @ q(w).T) * _phi_prime_from_h(hs[l], activation))
    return loss, grad


def loss_grad(model: str, x: np.ndarray, dims: Sequence[int], activation: str,
              a_b: np.ndarray, t_b: np.ndarray, bf16: bool = False) -> Tuple[float, np.ndarray]:
    """Dispatch on the objective."""
    if model == "lsq":
        return lsq_loss_grad(x, a_b, t_b)
    if model == "mlp":
        return mlp_loss_grad(x, dims, activation, a_b, t_b, bf16=bf16)
    raise ValueError(model)
