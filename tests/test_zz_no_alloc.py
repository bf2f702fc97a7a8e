"""The entry point without a workspace argument (the library's own fixed scratch buffer, for
callers that cannot allocate) against the ordinary entry point, through the C ABI.  Two calls
in a row share the buffer, the second with a smaller input: stale partials of the first call
must not leak into it.  Needs an MI355X (-m gpu)."""
import numpy as np
import pytest
import torch

from paper_2510_07535_amd import binding as B
from paper_2510_07535_amd import workloads as W
from paper_2510_07535_amd.runner import VerifyStep
from util import assert_close

pytestmark = pytest.mark.gpu


def _rng(k):
    return np.random.Generator(np.random.Philox(key=k))


def _both(case):
    """(ordinary entry point's output, no-workspace entry point's output) on the same device buffers."""
    step = VerifyStep(case)
    B.owl_verify_attn_init(step.desc)
    step.run()
    want = step.result().copy()
    assert step.dev_status() == 0
    step.out.fill_(float("nan"))
    B.owl_verify_attn_noalloc(step.desc, step.q, step.k, step.v, step.page_table, step.ctx_lens,
                              step.tree_parent, step.out, step.status)
    got = step.result().copy()
    assert step.dev_status() == 0
    return want, got


def test_noalloc_matches_the_workspace_entry_point_twice_in_a_row(oracle_mod):
    r = _rng(808)
    big = W.make_case("noalloc_big", 81, dtype=W.DT_BF16, Hq=32, Hkv=8, D=128, ctx_lens=[20000],
                      trees=[W.random_tree(60, 6, r)])
    small = W.make_case("noalloc_small", 82, dtype=W.DT_BF16, Hq=8, Hkv=2, D=128, ctx_lens=[700, 90],
                        trees=[W.random_tree(5, 3, r) for _ in range(2)])
    for case in (big, small):                             # same process, same buffer; the second is smaller
        want, got = _both(case)
        assert np.isfinite(got).all()
        assert np.array_equal(got, want), case.name       # same kernels, same order of operations
        assert_close(got, oracle_mod.verify_attn_case(case), case.dtype, case.name)


def test_noalloc_refuses_what_does_not_fit():
    case = W.make_case("noalloc_batch", 83, dtype=W.DT_BF16, Hq=32, Hkv=8, D=128, ctx_lens=[64] * 16,
                       trees=[W.chain_tree(26)] * 16)
    step = VerifyStep(case, max_ctx_len=65536)            # planned for 16 x 64K: partials beyond the fixed buffer
    assert step.plan.workspace_bytes > B.OWL_NOALLOC_SCRATCH_BYTES
    with pytest.raises(B.OwlError) as e:
        B.owl_verify_attn_noalloc(step.desc, step.q, step.k, step.v, step.page_table, step.ctx_lens,
                                  step.tree_parent, step.out, step.status)
    assert e.value.code == B.OWL_ERR_WORKSPACE
