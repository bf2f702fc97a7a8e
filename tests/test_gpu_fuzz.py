"""Seeded random sweep of the verify attention against the oracle: shapes, layouts,
paging, batch sizes, tree shapes, split sizes and storage types drawn at random,
every output element compared.  Needs an MI355X (-m gpu); calls go through the C ABI."""
import numpy as np
import pytest

from paper_2510_07535_amd import binding as B
from paper_2510_07535_amd import workloads as W
from paper_2510_07535_amd.runner import VerifyStep
from util import assert_close

pytestmark = pytest.mark.gpu


def _draw(seed):
    r = np.random.Generator(np.random.Philox(key=10_000 + seed))
    dtype = [W.DT_BF16, W.DT_BF16, W.DT_F16, W.DT_F32][int(r.integers(4))]
    D = 64 if dtype == W.DT_F32 else int(r.choice([64, 128]))
    Hkv = int(r.choice([1, 2, 4, 8]))
    G = int(r.choice([1, 2, 4, 8]))
    N = int(r.choice([1, 2, 5, 13, 26, 40, 60, 64]))
    if dtype == W.DT_F32:
        N = min(N, 13)
        G = min(G, 4)
    B = int(r.choice([1, 1, 2, 3, 7]))
    top = int(r.choice([0, 17, 300, 1100, 2600]))
    ctx = [int(r.integers(0, top + 1)) for _ in range(B)]
    kind = int(r.integers(3))
    trees = []
    for _ in range(B):
        if kind == 0 or N == 1:
            trees.append(W.chain_tree(N))
        elif kind == 1:
            trees.append(W.random_tree(N, int(r.integers(2, 9)), r))
        else:
            trees.append(W.random_tree(N, None, r))
    paged = bool(r.integers(2)) or B > 1
    head_major = bool(r.integers(2))
    split = int(r.choice([0, 0, 64, 192, 448, 1024]))
    outliers = 0.05 if r.integers(4) == 0 else 0.0
    case = W.make_case(f"fuzz{seed}", 500 + seed, dtype=dtype, Hq=Hkv * G, Hkv=Hkv, D=D, ctx_lens=ctx, trees=trees,
                       paged=paged, head_major=head_major, outlier_frac=outliers,
                       spare_pages=int(r.integers(0, 4)))
    return case, split


@pytest.mark.parametrize("seed", range(48))
def test_random_shape_matches_oracle(oracle_mod, seed):
    case, split = _draw(seed)
    # the two formats of the split partials take turns; every third case goes through the entry point
    # without a workspace (the library's own scratch buffer), shared by all of them in this process
    flags = B.OWL_FLAG_FP32_PARTIALS if seed % 2 else 0
    step = VerifyStep(case, split_tokens=split, flags=flags)
    if seed % 3 == 0 and step.plan.workspace_bytes <= B.OWL_NOALLOC_SCRATCH_BYTES:
        B.owl_verify_attn_noalloc(step.desc, step.q, step.k, step.v, step.page_table, step.ctx_lens,
                                  step.tree_parent, step.out, step.status)
    else:
        step.run()
    got = step.result()
    assert step.dev_status() == 0
    want = oracle_mod.verify_attn_case(case)
    what = (f"seed {seed}: dtype {case.dtype} B {case.B} N {case.N} Hq {case.Hq} Hkv {case.Hkv} D {case.D} "
            f"ctx {case.ctx_lens.tolist()} split {split} plan {step.plan.as_dict()}")
    assert_close(got, want, case.dtype, what)


def _draw_batch(seed):
    """Medium-size batches for the split sizes the library chooses itself: mixed lengths (a quarter of the
    sequences nearly empty), an announced maximum at or above the real one, sometimes per-sequence draft counts."""
    r = np.random.Generator(np.random.Philox(key=77_000 + seed))
    dtype = [W.DT_BF16, W.DT_BF16, W.DT_F16][int(r.integers(3))]
    D = int(r.choice([64, 128, 128]))
    Hkv = int(r.choice([1, 2, 4, 8]))
    G = int(r.choice([1, 2, 4, 8]))
    N = int(r.choice([1, 3, 6, 13, 26, 40, 60, 64]))
    Bn = int(r.choice([1, 1, 2, 4, 9, 16, 33]))
    top = int(r.choice([500, 5000, 20000]))
    if Hkv * G * N > 1024 or Bn >= 9:
        top = min(top, 5000)
    ctx = [int(r.integers(0, top + 1)) if r.integers(4) else int(r.integers(0, 40)) for _ in range(Bn)]
    trees = [W.random_tree(N, int(r.integers(2, 9)), r) if N > 1 and r.integers(3) else W.chain_tree(N)
             for _ in range(Bn)]
    case = W.make_case(f"batch{seed}", 900 + seed, dtype=dtype, Hq=Hkv * G, Hkv=Hkv, D=D, ctx_lens=ctx, trees=trees,
                       paged=True, head_major=bool(r.integers(2)), spare_pages=int(r.integers(0, 3)))
    planned = int(max(ctx) * float(r.choice([1.0, 1.0, 1.7, 4.0]))) + int(r.integers(0, 3))
    counts = [int(r.integers(0, N + 1)) for _ in range(Bn)] if r.integers(3) == 0 else None
    return case, max(planned, max(ctx)), counts


@pytest.mark.parametrize("seed", range(24))
def test_random_batch_through_the_library_plan(oracle_mod, seed):
    import dataclasses
    import torch
    case, planned, counts = _draw_batch(seed)
    cols = max((planned + case.N + 15) // 16, case.page_table.shape[1])   # the table covers the announced length
    table = np.zeros((case.B, cols), dtype=np.int32)
    table[:, :case.page_table.shape[1]] = case.page_table
    wide = dataclasses.replace(case, page_table=table, max_pages_per_seq=cols)
    step = VerifyStep(wide, max_ctx_len=planned, flags=B.OWL_FLAG_FP32_PARTIALS if seed % 2 else 0)
    if counts is None:
        step.run()
        want = oracle_mod.verify_attn_case(case)
    else:
        nd = torch.tensor(counts, dtype=torch.int32, device=step.device)
        B.owl_verify_attn_ragged(step.desc, step.q, step.k, step.v, step.page_table, step.ctx_lens,
                                 step.tree_parent, nd, step.out, step.workspace, step.status)
        want = oracle_mod.verify_attn_ragged_case(case, counts)
    got = step.result()
    assert step.dev_status() == 0
    assert_close(got, want, case.dtype,
                 f"seed {seed}: dtype {case.dtype} B {case.B} N {case.N} Hq {case.Hq} Hkv {case.Hkv} D {case.D} "
                 f"ctx {case.ctx_lens.tolist()} announced {planned} counts {counts} plan {step.plan.as_dict()}")
