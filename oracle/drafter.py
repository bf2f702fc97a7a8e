"""CPU fp64 oracle of one step of the drafter's recurrent cell.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``): plain numpy in float64,
written from the paper's equations (Sec. 3.2.1, Eq. 1-8), sharing nothing with
the HIP path.

One step takes the token just predicted, the hidden state it was predicted from
and the running cell state, and returns the next hidden state and cell state:

    e   = E[t]                                              (Eq. 1)
    s^m = W^m h + alpha * e          m in {f, i, o, c}      (Eq. 2)
    g^m = sigmoid(s^m)               m in {f, i, o}         (Eq. 5)
    c   = f(s^c) * g^i                                      (Eq. 6)
    z'  = z * g^f + c                                       (Eq. 7)
    h'  = f(z') * g^o                                       (Eq. 8)

``f`` is layer normalisation over the d channels followed by GeLU.  Readings
taken where the paper is silent (each is listed in the design notes):
  * W^m is applied as a linear layer without bias, stored output-major,
    ``W[m]`` of shape (d, d_in), so ``s = W[m] @ h``;
  * the layer normalisation uses the biased variance with ``eps`` added under
    the square root and an affine pair (gamma, beta); the two uses of ``f``
    (on s^c and on z') have separate affine pairs;
  * GeLU is the exact form x * Phi(x), Phi the standard normal CDF;
  * alpha is the number Eq. 3-4 give, as printed.
In tree drafting several tokens can follow the same state: row r of the step
uses state row ``parent_row[r]`` and its own token.
"""
from __future__ import annotations

import math
from typing import Optional, Tuple

import numpy as np

GATES = ("f", "i", "o", "c")          # order of the four projections in W


def drafter_alpha(n: int, d: int) -> float:
    """Eq. 3-4: alpha_0 = 2^(-1/(2n)), alpha = 2 alpha_0 / ((1 - alpha_0^2) d);
    n = the greatest tree depth to be generated, d = the cell's width."""
    if n < 1 or d < 1:
        raise ValueError("n and d must be positive")
    alpha0 = 2.0 ** (-1.0 / (2.0 * n))
    return 2.0 * alpha0 / ((1.0 - alpha0 * alpha0) * d)


def _sigmoid(x: np.ndarray) -> np.ndarray:
    return 1.0 / (1.0 + np.exp(-x))


def _gelu(x: np.ndarray) -> np.ndarray:
    erf = np.vectorize(math.erf, otypes=[np.float64])
    return 0.5 * x * (1.0 + erf(x / math.sqrt(2.0)))


def _layer_norm(x: np.ndarray, gamma: Optional[np.ndarray], beta: Optional[np.ndarray], eps: float) -> np.ndarray:
    """Per row over the last axis: (x - mean) / sqrt(biased variance + eps) * gamma + beta."""
    mu = x.sum(axis=-1, keepdims=True) / x.shape[-1]
    xc = x - mu
    var = (xc * xc).sum(axis=-1, keepdims=True) / x.shape[-1]
    y = xc / np.sqrt(var + eps)
    if gamma is not None:
        y = y * gamma
    if beta is not None:
        y = y + beta
    return y


def _f(x, gamma, beta, eps):
    """The paper's f: layer normalisation, then the activation (GeLU)."""
    return _gelu(_layer_norm(x, gamma, beta, eps))


def drafter_cell(h: np.ndarray, z: np.ndarray, tokens: np.ndarray, parent_row: Optional[np.ndarray],
                 W: np.ndarray, E: np.ndarray, alpha: float,
                 gamma_c: Optional[np.ndarray] = None, beta_c: Optional[np.ndarray] = None,
                 gamma_z: Optional[np.ndarray] = None, beta_z: Optional[np.ndarray] = None,
                 eps: float = 1e-5) -> Tuple[np.ndarray, np.ndarray]:
    """One step of the cell for M rows.

    h (P, d_in), z (P, d): the P distinct states; tokens (M,): the token each row
    consumes; parent_row (M,) or None (identity, M == P): the state row each row
    continues; W (4, d, d_in) in the order f, i, o, c; E (vocab, d).
    Returns (h_new (M, d), z_new (M, d)) in float64.
    """
    h = np.asarray(h, dtype=np.float64)
    z = np.asarray(z, dtype=np.float64)
    W = np.asarray(W)
    E = np.asarray(E)
    tokens = np.asarray(tokens)
    P, d_in = h.shape
    d = z.shape[1]
    if W.shape != (4, d, d_in) or z.shape[0] != P or E.shape[1] != d:
        raise ValueError("shape mismatch")
    M = tokens.shape[0]
    if parent_row is None:
        if M != P:
            raise ValueError("identity parent_row needs M == P")
        parent_row = np.arange(M)
    parent_row = np.asarray(parent_row)
    if ((parent_row < 0) | (parent_row >= P)).any() or ((tokens < 0) | (tokens >= E.shape[0])).any():
        raise ValueError("index out of range")

    # W^m h for each of the P states (the product of Eq. 2 does not depend on the token)
    proj = {m: (W[k].astype(np.float64) @ h.T).T for k, m in enumerate(GATES)}
    h_new = np.empty((M, d), dtype=np.float64)
    z_new = np.empty((M, d), dtype=np.float64)
    for r in range(M):
        e = E[tokens[r]].astype(np.float64)                                   # Eq. 1
        s = {m: proj[m][parent_row[r]] + alpha * e for m in GATES}           # Eq. 2
        g = {m: _sigmoid(s[m]) for m in ("f", "i", "o")}                     # Eq. 5
        c = _f(s["c"], gamma_c, beta_c, eps) * g["i"]                        # Eq. 6
        z_new[r] = z[parent_row[r]] * g["f"] + c                             # Eq. 7
        h_new[r] = _f(z_new[r], gamma_z, beta_z, eps) * g["o"]               # Eq. 8
    return h_new, z_new


def _widen(bits: np.ndarray, dtype: int) -> np.ndarray:
    """Stored 16-bit patterns -> float32 values (exact).  dtype: 0 = bf16, 2 = fp16."""
    bits = np.asarray(bits)
    if dtype == 0:
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    if dtype == 2:
        return bits.view(np.float16).astype(np.float32)
    raise ValueError("dtype")


def drafter_cell_case(case, alpha: float, rows: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """The step on a seeded case (any object with the fields of the generator's
    ``DrafterCase``).  ``rows`` restricts the result to those rows of the step."""
    tokens = case.tokens
    parent_row = case.parent_row if case.parent_row is not None else np.arange(case.M)
    if rows is not None:
        tokens, parent_row = tokens[rows], parent_row[rows]
    used, inv = np.unique(parent_row, return_inverse=True)                # only the states these rows continue
    return drafter_cell(_widen(case.h[used], case.dtype), case.z[used], tokens, inv,
                        _widen(case.W, case.dtype), _widen(case.E, case.dtype), alpha,
                        case.gamma_c, case.beta_c, case.gamma_z, case.beta_z, case.eps)
