"""Pins of the drafter-cell oracle (``oracle/drafter.py``; Sec. 3.2.1, Eq. 1-8)
against closed forms, hand-worked cases, invariants of the equations and
independent library routines (torch's linear / layer_norm / gelu / sigmoid in
float64).  Each is chosen so that a plausible slip (a dropped term, swapped
gates, a transposed weight, a missing normalisation) fails it.  No GPU."""
import decimal
import math

import numpy as np
import pytest
import torch

from oracle import drafter as D
from paper_2510_07535_amd import workloads as W

PHI1 = 0.8413447460685429            # standard normal CDF at 1 (textbook table value 0.84134)


# --------------------------------------------------------------------------- alpha, Eq. 3-4
def test_alpha_closed_forms():
    # n = 1: alpha_0 = 2^(-1/2), alpha_0^2 = 1/2, alpha = 2 * 2^(-1/2) / (d / 2) = 2 sqrt(2) / d
    assert D.drafter_alpha(1, 8) == pytest.approx(2.0 * math.sqrt(2.0) / 8.0, rel=1e-15)
    # alpha scales as 1/d
    assert D.drafter_alpha(5, 300) * 300 == pytest.approx(D.drafter_alpha(5, 1), rel=1e-15)
    # alpha_0^(2n) = 1/2 whatever n: recover alpha_0 from alpha by solving the quadratic
    # alpha d (1 - x^2) = 2 x  for x in (0, 1)
    for n in (1, 2, 8, 13):
        a = D.drafter_alpha(n, 1)
        x = (-1.0 + math.sqrt(1.0 + a * a)) / a
        assert x ** (2 * n) == pytest.approx(0.5, rel=1e-12)


def test_alpha_high_precision_value():
    """n = 8 (the tree depth of Appendix A.1), d = 12288 (Sec. 4.1), in 50-digit decimal arithmetic."""
    decimal.getcontext().prec = 50
    a0 = (decimal.Decimal(2).ln() * decimal.Decimal(-1) / decimal.Decimal(16)).exp()
    want = 2 * a0 / ((1 - a0 * a0) * 12288)
    assert D.drafter_alpha(8, 12288) == pytest.approx(float(want), rel=1e-13)
    assert 1.8e-3 < float(want) < 2.0e-3


# --------------------------------------------------------------------------- hand-worked cell
def test_cell_two_channels_by_hand():
    """d = 2, d_in = 1, eps = 0, no affine: the normalisation of any two distinct numbers is
    (-1, +1) in their order, so f gives (GeLU(-1), GeLU(1)) = (-(1 - Phi(1)), Phi(1))."""
    h = np.array([[2.0]])
    z = np.array([[3.0, -5.0]])
    Wm = np.zeros((4, 2, 1))
    Wm[3, :, 0] = [0.5, 1.5]          # s^c = (1, 3): normalises to (-1, +1)
    # s^f = s^i = s^o = 0: every gate is 1/2
    E = np.zeros((1, 2))
    h1, z1 = D.drafter_cell(h, z, np.array([0]), None, Wm, E, alpha=1.0, eps=0.0)
    cand = np.array([-(1 - PHI1), PHI1]) * 0.5
    assert z1[0] == pytest.approx(np.array([1.5, -2.5]) + cand, abs=1e-15)
    # z' = (1.5 - 0.0793, -2.5 + 0.4207): first > second, so it normalises to (+1, -1)
    assert h1[0] == pytest.approx(np.array([PHI1, -(1 - PHI1)]) * 0.5, abs=1e-12)


def test_cell_embedding_term_and_alpha():
    """Same shape, the projection switched off: s^m = alpha * e for every gate."""
    h = np.zeros((1, 1))
    z = np.zeros((1, 2))
    Wm = np.zeros((4, 2, 1))
    E = np.array([[9.0, 9.0], [1.0, -1.0]])
    alpha = 0.25
    h1, z1 = D.drafter_cell(h, z, np.array([1]), None, Wm, E, alpha=alpha, eps=0.0)
    sg = 1 / (1 + math.exp(-0.25)), 1 / (1 + math.exp(0.25))          # sigmoid(+-0.25)
    # s^c = (0.25, -0.25) -> normalised (+1, -1); candidate = GeLU(.) * g^i; z' = candidate (z = 0)
    z_want = np.array([PHI1 * sg[0], -(1 - PHI1) * sg[1]])
    assert z1[0] == pytest.approx(z_want, abs=1e-15)
    assert h1[0] == pytest.approx(np.array([PHI1 * sg[0], -(1 - PHI1) * sg[1]]), abs=1e-12)
    # token 0 has equal channels: zero variance, eps > 0 keeps it finite and the candidate is GeLU(0) = 0
    h0, z0 = D.drafter_cell(h, z, np.array([0]), None, Wm, E, alpha=alpha, eps=1e-5)
    assert np.all(z0 == 0) and np.all(h0 == 0)


# --------------------------------------------------------------------------- against library routines
def _torch_cell(case, alpha):
    """The same equations through torch's own linear / layer_norm / gelu / sigmoid, float64."""
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64))
    h = t(W.widen(case.h, case.dtype))
    Wm = t(W.widen(case.W, case.dtype))
    E = t(W.widen(case.E, case.dtype))
    z = t(case.z)
    pr = torch.from_numpy(case.parent_row.astype(np.int64)) if case.parent_row is not None else torch.arange(case.M)
    e = torch.nn.functional.embedding(torch.from_numpy(case.tokens.astype(np.int64)), E)
    s = [torch.nn.functional.linear(h, Wm[m])[pr] + alpha * e for m in range(4)]
    f = lambda x, g, b: torch.nn.functional.gelu(
        torch.nn.functional.layer_norm(x, (case.d,), t(g), t(b), case.eps))
    cand = f(s[3], case.gamma_c, case.beta_c) * torch.sigmoid(s[1])
    z1 = z[pr] * torch.sigmoid(s[0]) + cand
    h1 = f(z1, case.gamma_z, case.beta_z) * torch.sigmoid(s[2])
    return h1.numpy(), z1.numpy()


@pytest.mark.parametrize("dtype,d_in,d,P,M,alpha", [(W.DT_BF16, 96, 48, 3, 7, 1.0), (W.DT_F16, 32, 80, 5, 5, 0.3),
                                                    (W.DT_BF16, 64, 64, 1, 4, None)])
def test_cell_matches_torch_library_ops(dtype, d_in, d, P, M, alpha):
    case = W.make_drafter_case("pin", 11, dtype=dtype, d_in=d_in, d=d, P=P, M=M)
    if alpha is None:
        alpha = D.drafter_alpha(8, d)
    h1, z1 = D.drafter_cell_case(case, alpha)
    h_t, z_t = _torch_cell(case, alpha)
    assert np.abs(z1 - z_t).max() < 1e-12
    assert np.abs(h1 - h_t).max() < 1e-12


# --------------------------------------------------------------------------- invariants of the equations
def _case(seed=5, **kw):
    args = dict(dtype=W.DT_BF16, d_in=64, d=32, P=4, M=6)
    args.update(kw)
    return W.make_drafter_case("inv", seed, **args)


def _run(case, alpha=1.0, **over):
    a = dict(h=W.widen(case.h, case.dtype), z=case.z.astype(np.float64), tokens=case.tokens,
             parent_row=case.parent_row, W=W.widen(case.W, case.dtype), E=W.widen(case.E, case.dtype),
             alpha=alpha, gamma_c=case.gamma_c, beta_c=case.beta_c, gamma_z=case.gamma_z, beta_z=case.beta_z,
             eps=case.eps)
    a.update(over)
    return D.drafter_cell(**a)


def test_candidate_is_scale_and_shift_invariant():
    """f normalises: with eps = 0, scaling W^c and the embedding's share of s^c by a positive
    constant leaves everything unchanged; so does adding a constant to every channel of s^c."""
    case = _case()
    Wm = W.widen(case.W, case.dtype)
    E = W.widen(case.E, case.dtype)
    base = _run(case, alpha=0.0, eps=0.0)
    W2 = Wm.copy()
    W2[3] *= 7.0
    scaled = _run(case, alpha=0.0, eps=0.0, W=W2)
    assert np.abs(scaled[0] - base[0]).max() < 1e-10 and np.abs(scaled[1] - base[1]).max() < 1e-10
    h_big = np.concatenate([W.widen(case.h, case.dtype), np.ones((case.P, 1))], axis=1)
    W_shift = np.concatenate([Wm, np.zeros((4, case.d, 1))], axis=2)
    W_shift[3, :, -1] = 5.0            # every channel of s^c moves by +5
    shifted = _run(case, alpha=0.0, eps=0.0, h=h_big, W=W_shift)
    assert np.abs(shifted[0] - base[0]).max() < 1e-10 and np.abs(shifted[1] - base[1]).max() < 1e-10
    W3 = Wm.copy()
    W3[1] *= 7.0                       # the input gate is NOT normalised: this must change the result
    assert np.abs(_run(case, alpha=0.0, eps=0.0, W=W3)[1] - base[1]).max() > 1e-3


@pytest.mark.filterwarnings("ignore:overflow")
def test_forget_gate_closed_and_open():
    case = _case()
    Wm = W.widen(case.W, case.dtype)
    h = W.widen(case.h, case.dtype)
    # close the forget gate: a huge negative pre-activation through one extra input channel
    h_big = np.concatenate([h, np.ones((case.P, 1))], axis=1)
    W_big = np.concatenate([Wm, np.zeros((4, case.d, 1))], axis=2)
    W_big[0, :, -1] = -1e3
    closed = _run(case, h=h_big, W=W_big)
    closed_other_z = _run(case, h=h_big, W=W_big, z=case.z.astype(np.float64) * 3 + 1)
    assert np.array_equal(closed[1], closed_other_z[1])               # z' no longer depends on z
    zero_state = _run(case, z=np.zeros_like(case.z, dtype=np.float64))
    assert np.abs(closed[1] - zero_state[1]).max() < 1e-12            # and equals the start-from-zero step
    # open it (+1e3): z' - z = candidate, the same candidate as before
    W_big[0, :, -1] = 1e3
    opened = _run(case, h=h_big, W=W_big)
    pr = case.parent_row
    assert np.abs((opened[1] - case.z.astype(np.float64)[pr]) - closed[1]).max() < 1e-12


@pytest.mark.filterwarnings("ignore:overflow")
def test_output_gate_bounds_and_gate_roles():
    """|h'| <= max|GeLU(LN(z'))| since 0 < g^o < 1; closing the output gate zeroes h' but not z';
    closing the input gate leaves z' = z * g^f exactly."""
    case = _case()
    Wm = W.widen(case.W, case.dtype)
    h = W.widen(case.h, case.dtype)
    h_big = np.concatenate([h, np.ones((case.P, 1))], axis=1)
    Wo = np.concatenate([Wm, np.zeros((4, case.d, 1))], axis=2)
    Wo[2, :, -1] = -1e3
    h1, z1 = _run(case, h=h_big, W=Wo)
    base = _run(case)
    assert np.abs(h1).max() < 1e-300 and np.abs(z1 - base[1]).max() < 1e-12
    Wi = np.concatenate([Wm, np.zeros((4, case.d, 1))], axis=2)
    Wi[1, :, -1] = -1e3
    _, z2 = _run(case, h=h_big, W=Wi, alpha=0.0)
    sf = h @ Wm[0].T                                                   # (P, d)
    want = case.z.astype(np.float64)[case.parent_row] / (1 + np.exp(-sf[case.parent_row]))
    assert np.abs(z2 - want).max() < 1e-12


def test_rows_sharing_a_state_equal_replicated_states():
    case = _case(P=3, M=8)
    a = _run(case)
    pr = case.parent_row
    b = _run(case, h=W.widen(case.h, case.dtype)[pr], z=case.z.astype(np.float64)[pr], parent_row=None)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    # rows with the same state and the same token are equal, a different token changes the row
    toks = case.tokens.copy()
    toks[:] = toks[0]
    c = _run(case, tokens=toks)
    same = [r for r in range(case.M) if pr[r] == pr[0]]
    for r in same:
        assert np.array_equal(c[0][r], c[0][0])


def test_weight_orientation_rectangular():
    """d_in != d: W[m] is (d, d_in); a transposed use cannot even be formed, and the product is the
    plain definition sum_k W[m][j][k] h[k] (checked on one gate by an explicit double loop)."""
    case = _case(d_in=32, d=16, P=2, M=2, identity=True)
    Wm = W.widen(case.W, case.dtype)
    h = W.widen(case.h, case.dtype)
    _, z1 = _run(case, alpha=0.0, z=np.ones((2, 16)), W=np.concatenate([Wm[:1], np.zeros_like(Wm[1:])]),
                 beta_c=None)
    # gates i, o and the candidate's projection are zero: s^c = 0 -> candidate GeLU(0)*0.5 = 0, so z' = g^f
    for r in range(2):
        for j in range(16):
            s = 0.0
            for k in range(32):
                s += Wm[0, j, k] * h[r, k]
            assert z1[r, j] == pytest.approx(1 / (1 + math.exp(-s)), abs=1e-13)
    with pytest.raises(ValueError):
        D.drafter_cell(h, np.ones((2, 16)), case.tokens, None, np.swapaxes(Wm, 1, 2), W.widen(case.E, case.dtype), 1.0)


def test_recurrence_two_steps_with_square_weights():
    """d_in = d: the cell can be applied to its own output (the paper reuses the weights at every
    depth); two chained steps equal the torch formulation chained the same way."""
    case = W.make_drafter_case("rec", 3, dtype=W.DT_F16, d_in=48, d=48, P=2, M=2, identity=True, zero_state=True)
    alpha = D.drafter_alpha(8, 48)
    h1, z1 = D.drafter_cell_case(case, alpha)
    Wm, E = W.widen(case.W, case.dtype), W.widen(case.E, case.dtype)
    tok2 = (case.tokens + 1) % case.vocab
    h2, z2 = D.drafter_cell(h1, z1, tok2, None, Wm, E, alpha, case.gamma_c, case.beta_c, case.gamma_z,
                            case.beta_z, case.eps)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64))
    ht, zt = t(W.widen(case.h, case.dtype)), t(case.z)
    for toks in (case.tokens, tok2):
        e = t(E)[torch.from_numpy(toks.astype(np.int64))]
        s = [ht @ t(Wm[m]).T + alpha * e for m in range(4)]
        ln = lambda x, g, b: torch.nn.functional.gelu(torch.nn.functional.layer_norm(x, (48,), t(g), t(b), case.eps))
        zt = zt * torch.sigmoid(s[0]) + ln(s[3], case.gamma_c, case.beta_c) * torch.sigmoid(s[1])
        ht = ln(zt, case.gamma_z, case.beta_z) * torch.sigmoid(s[2])
    assert np.abs(h2 - ht.numpy()).max() < 1e-12 and np.abs(z2 - zt.numpy()).max() < 1e-12


def test_rejects_bad_indices():
    case = _case()
    with pytest.raises(ValueError):
        _run(case, tokens=np.full(case.M, case.vocab))
    with pytest.raises(ValueError):
        _run(case, parent_row=np.full(case.M, case.P))
