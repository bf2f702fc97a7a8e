"""GPU parity of the drafter's recurrent cell (Sec. 3.2.1, Eq. 1-8) against
``oracle/drafter.py``.  Needs an MI355X (-m gpu); every call goes through the C ABI.

Tolerance.  The inputs of the cell are the same 16-bit values on both sides, the
products of the projection are exact in fp32 and its sums carry an fp32 rounding
error of about sqrt(d_in) * 2^-24 * |s| (1e-5 at d_in = 12288); the normalisation
divides by a standard deviation of order one and sigmoid / GeLU have slopes below
1.13, so z' and h' in fp32 agree with the fp64 oracle to a few 1e-5.  The bar is
max-abs 2e-4 on z' and on the fp32 h'; the 16-bit h' must be the fp32 h' rounded
to nearest even, bit for bit, hence within that bar plus half a unit in the last
place (at most 2^-8 relative for bf16, 2^-11 for fp16) of the oracle's value."""
import numpy as np
import pytest
import torch

from oracle import drafter as OD
from paper_2510_07535_amd import binding as B
from paper_2510_07535_amd import workloads as W
from paper_2510_07535_amd.runner import DrafterStep

pytestmark = pytest.mark.gpu
TOL = 2e-4


def _check(case, alpha, rows=None, tiled=True):
    step = DrafterStep(case, alpha, tiled=tiled)
    step.run()
    h32, h16, z1 = step.result()
    assert step.dev_status() == 0
    h_ref, z_ref = OD.drafter_cell_case(case, alpha, rows)
    if rows is not None:
        h32, h16, z1 = h32[rows], h16[rows], z1[rows]
    assert np.abs(z1 - z_ref).max() < TOL, np.abs(z1 - z_ref).max()
    assert np.abs(h32 - h_ref).max() < TOL, np.abs(h32 - h_ref).max()
    half_ulp = 2.0 ** -8 if case.dtype == W.DT_BF16 else 2.0 ** -11
    excess = float((np.abs(W.widen(h16, case.dtype) - h_ref) - half_ulp * np.abs(h_ref)).max())
    assert excess < TOL, excess
    # the 16-bit output is the fp32 output rounded to nearest even, exactly
    assert np.array_equal(h16, W.store(h32, case.dtype))
    return step


@pytest.mark.parametrize("dtype", [W.DT_BF16, W.DT_F16])
@pytest.mark.parametrize("d_in,d,P,M", [
    (32, 16, 1, 1),          # the smallest shape: one k-step, one weight tile per gate
    (96, 48, 3, 7),          # k-steps not a multiple of the unroll; 12 weight tiles = 3 workgroups
    (160, 80, 5, 5),         # 20 tiles; odd k-step count
    (640, 272, 17, 30),      # two state tiles; 68 tiles = 17 workgroups; k-steps spread unevenly over the wavefronts
    (1024, 1040, 40, 64),    # three state tiles, the row limit, more than one channel per thread
    (512, 2064, 64, 33),     # four state tiles, ragged last channel round
])
def test_cell_matches_oracle(dtype, d_in, d, P, M):
    case = W.make_drafter_case("t", 100 + d, dtype=dtype, d_in=d_in, d=d, P=P, M=M, vocab=50)
    _check(case, 1.0)                                    # alpha = 1: the embedding weighs as much as the projection
    _check(case, OD.drafter_alpha(8, d), tiled=False)    # the paper's alpha; weights as a plain [4d][d_in] matrix


def _tiled_by_definition(w_bits, d_in, d):
    """The tiled layout built from its definition in the header, granule by granule."""
    rows = w_bits.reshape(4 * d, d_in)
    groups = -(-4 * d // 64)
    out = np.zeros((groups * (d_in // 32) * 4 * 64, 8), dtype=np.uint16)
    for row in range(4 * d):
        for k in range(0, d_in, 8):
            g = ((row // 64 * (d_in // 32) + k // 32) * 4 + row % 64 // 16) * 64 + (k % 32 // 8) * 16 + row % 16
            out[g] = rows[row, k:k + 8]
    return out.reshape(-1)


@pytest.mark.parametrize("d_in,d", [(32, 16), (96, 48), (160, 272)])
def test_tiled_weights_are_the_documented_permutation(d_in, d):
    case = W.make_drafter_case("t", 5, d_in=d_in, d=d, P=1, M=1)
    step = DrafterStep(case, 1.0, tiled=True)
    torch.cuda.synchronize()
    got = step.w.cpu().numpy().view(np.uint16)
    want = _tiled_by_definition(case.W, d_in, d)
    assert got.size == want.size == B.owl_drafter_tiled_weight_bytes(step.desc) // 2
    assert np.array_equal(got, want)


def test_identity_rows_and_zero_start():
    case = W.make_drafter_case("t", 7, d_in=256, d=256, P=9, M=9, identity=True, zero_state=True)
    _check(case, 0.5)


def test_null_affine_and_single_outputs():
    case = W.make_drafter_case("t", 8, d_in=128, d=96, P=2, M=4)
    step = DrafterStep(case, 1.0)
    step.gamma_c = step.beta_c = step.gamma_z = step.beta_z = None
    step.run()
    h32, h16, z1 = step.result()
    bare = W.make_drafter_case("t", 8, d_in=128, d=96, P=2, M=4)
    bare.gamma_c = bare.gamma_z = np.ones(96, np.float32)
    bare.beta_c = bare.beta_z = np.zeros(96, np.float32)
    h_ref, z_ref = OD.drafter_cell_case(bare, 1.0)
    assert np.abs(z1 - z_ref).max() < TOL and np.abs(h32 - h_ref).max() < TOL
    # only one of the two h' outputs asked for
    step.h_out_f32 = None
    step.h_out.zero_()
    step.run()
    torch.cuda.synchronize()
    assert np.array_equal(step.h_out.cpu().numpy().view(np.uint16), h16)


def test_two_steps_recurrence():
    """d_in == d: the 16-bit h' and the fp32 z' of one step are the next step's state."""
    case = W.make_drafter_case("t", 9, dtype=W.DT_F16, d_in=384, d=384, P=4, M=4, identity=True, zero_state=True)
    alpha = OD.drafter_alpha(8, 384)
    s1 = _check(case, alpha)
    _, h16, z1 = s1.result()
    import dataclasses
    nxt = dataclasses.replace(case, h=h16.copy(), z=z1.copy(), tokens=(case.tokens + 3) % case.vocab)
    _check(nxt, alpha)


def test_phases_split():
    case = W.make_drafter_case("t", 10, d_in=224, d=112, P=6, M=11)
    whole = DrafterStep(case, 1.0)
    whole.run()
    want = whole.result()
    parts = DrafterStep(case, 1.0)
    parts.run(phases=B.OWL_DRAFTER_PROJ)
    parts.run(phases=B.OWL_DRAFTER_GATES)
    got = parts.result()
    for a, b in zip(want, got):
        assert np.array_equal(a, b)
    # the projection in the workspace is W^m h: sampled entries against the plain definition
    proj = parts.workspace.cpu().numpy().view(np.float32)[:case.P * 4 * case.d].reshape(case.P, 4, case.d)
    Wm, h = W.widen(case.W, case.dtype), W.widen(case.h, case.dtype)
    r = np.random.Generator(np.random.Philox(key=1))
    for _ in range(50):
        p, m, j = int(r.integers(case.P)), int(r.integers(4)), int(r.integers(case.d))
        assert abs(proj[p, m, j] - float(Wm[m, j] @ h[p])) < 1e-5


def test_bad_indices_are_flagged_and_contained():
    case = W.make_drafter_case("t", 11, d_in=64, d=32, P=3, M=5, vocab=20)
    good = DrafterStep(case, 1.0)
    good.run()
    ref = good.result()
    bad = W.make_drafter_case("t", 11, d_in=64, d=32, P=3, M=5, vocab=20)
    bad.tokens[1] = 20
    bad.parent_row[3] = -1
    step = DrafterStep(bad, 1.0)
    step.run()
    got = step.result()
    assert step.dev_status() == (B.OWL_DEV_BAD_TOKEN | B.OWL_DEV_BAD_ROW)
    for r in (0, 2, 4):                                   # the other rows are untouched by the bad ones
        assert np.array_equal(got[0][r], ref[0][r]) and np.array_equal(got[2][r], ref[2][r])
    assert np.isfinite(got[0]).all() and np.isfinite(got[2]).all()


def test_alpha_matches_oracle():
    for n, d in ((1, 8), (8, 12288), (5, 4096), (13, 300)):
        assert B.owl_drafter_alpha(n, d) == pytest.approx(np.float32(OD.drafter_alpha(n, d)), rel=1e-7)


def test_full_width_sampled_rows():
    """The paper's width (Sec. 4.1: d = 12288) with a square W, the ten rows of one tree level
    (Appendix A.1: top-k 10) continuing ten states: three rows checked against the oracle."""
    case = W.make_drafter_case("level", 21, d_in=12288, d=12288, P=10, M=10, vocab=512)
    _check(case, OD.drafter_alpha(8, 12288), rows=np.array([0, 4, 9]))
    _check(case, OD.drafter_alpha(8, 12288), rows=np.array([7]), tiled=False)
