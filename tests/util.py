"""Shared pieces of the GPU parity tests."""
import numpy as np

from paper_2510_07535_amd import workloads as W

# The bar for 16-bit inputs (bf16 / f16 storage, fp32 accumulate): max-abs 1e-2
# and mean-abs 1e-3 against the fp64 oracle.  fp32 inputs run fp32 MFMA and a
# hardware exp2; 2e-4 / 2e-5 is ~20x the observed error and far inside the bar.
TOL = {W.DT_BF16: (1e-2, 1e-3), W.DT_F16: (1e-2, 1e-3), W.DT_F32: (2e-4, 2e-5)}


def assert_close(got: np.ndarray, want: np.ndarray, dtype: int, what: str = ""):
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got.astype(np.float64) - want)
    mx, mean = float(err.max()), float(err.mean())
    tmax, tmean = TOL[dtype]
    assert mx <= tmax and mean <= tmean, f"{what}: max-abs {mx:.3e} (<= {tmax}), mean-abs {mean:.3e} (<= {tmean})"
    return mx, mean


def sample_rows(case, n, seed=0, always=()):
    """n distinct (b, i, h) triples, plus the listed ones."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    total = case.B * case.N * case.Hq
    pick = rng.choice(total, size=min(n, total), replace=False)
    rows = [(int(x // (case.N * case.Hq)), int((x // case.Hq) % case.N), int(x % case.Hq)) for x in pick]
    for r in always:
        if r not in rows:
            rows.append(r)
    return np.array(rows, dtype=np.int32)
