"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.  Everything here needs an MI355X (-m gpu)."""
import numpy as np
import pytest
import torch

from paper_2510_07535_amd import binding as B
from paper_2510_07535_amd import workloads as W
from paper_2510_07535_amd.runner import VerifyStep, _to_dev
from util import assert_close, sample_rows
from tree_helpers import spec_tree

pytestmark = pytest.mark.gpu


def _rng(k):
    return np.random.Generator(np.random.Philox(key=k))


def _run(case, **kw):
    step = VerifyStep(case, **kw)
    step.run()
    out = step.result()
    assert step.dev_status() == 0
    return out, step


# ---------------------------------------------------------------------------
# small and ragged shapes, full element-by-element comparison
# ---------------------------------------------------------------------------
def _small_cases():
    r = _rng(1234)
    mk = W.make_case
    cs = [
        # several 64-key stages, ragged tail, chain (row tiles: 2)
        mk("bf16_chain6_L1000", 101, dtype=W.DT_BF16, Hq=32, Hkv=8, D=128, ctx_lens=[1000], trees=[W.chain_tree(6)]),
        # one row tile, n_draft = 1 (plain decode)
        mk("bf16_decode_L777", 102, dtype=W.DT_BF16, Hq=8, Hkv=2, D=128, ctx_lens=[777], trees=[W.chain_tree(1)]),
        # empty prefix: only the drafts are visible
        mk("bf16_L0_tree20", 103, dtype=W.DT_BF16, Hq=8, Hkv=2, D=128, ctx_lens=[0], trees=[W.random_tree(20, 5, r)]),
        # prefix shorter than a page / exactly a page; drafts straddle pages
        mk("bf16_L15_L16_L17", 104, dtype=W.DT_BF16, Hq=4, Hkv=2, D=128, ctx_lens=[15, 16, 17],
           trees=[W.random_tree(9, 4, r) for _ in range(3)]),
        # 3..4 row tiles -> 2x2 wave layout
        mk("bf16_tree14_G4", 105, dtype=W.DT_BF16, Hq=8, Hkv=2, D=128, ctx_lens=[2500], trees=[W.random_tree(14, 4, r)]),
        # 7 row tiles (the batched configuration's tile count), ragged batch
        mk("bf16_tree26_batch3", 106, dtype=W.DT_BF16, Hq=32, Hkv=8, D=128, ctx_lens=[3000, 129, 1999],
           trees=[W.random_tree(26, 5, r) for _ in range(3)]),
        # 15 row tiles (60-node tree, G=4)
        mk("bf16_tree60", 107, dtype=W.DT_BF16, Hq=8, Hkv=2, D=128, ctx_lens=[1500], trees=[W.random_tree(60, 6, r)]),
        # 20 row tiles (40 nodes, G=8) with outlier keys
        mk("bf16_hybrid40_G8", 108, dtype=W.DT_BF16, Hq=16, Hkv=2, D=128, ctx_lens=[2100],
           trees=[W.hybrid_tree(32, 8, r)], outlier_frac=0.05),
        # maximum draft count, G=8 -> 32 row tiles -> two row groups
        mk("bf16_chain64_G8", 109, dtype=W.DT_BF16, Hq=8, Hkv=1, D=128, ctx_lens=[700], trees=[W.chain_tree(64)]),
        # head_dim 64, token-major cache layout, G=1
        mk("bf16_D64_tokmajor", 110, dtype=W.DT_BF16, Hq=4, Hkv=4, D=64, ctx_lens=[900, 64],
           trees=[W.random_tree(12, 4, r) for _ in range(2)], head_major=False),
        mk("bf16_D64_tree40", 111, dtype=W.DT_BF16, Hq=16, Hkv=4, D=64, ctx_lens=[1300], trees=[W.random_tree(40, 8, r)]),
        # identity paging (page_table NULL)
        mk("bf16_identity_pages", 112, dtype=W.DT_BF16, Hq=8, Hkv=2, D=128, ctx_lens=[555], trees=[W.random_tree(7, 3, r)],
           paged=False),
        # forest: several roots
        mk("bf16_forest", 113, dtype=W.DT_BF16, Hq=4, Hkv=1, D=128, ctx_lens=[300],
           trees=[np.array([-1, -1, 0, 1, 1, -1, 5, 2], np.int32)]),
        # fp16 storage (the paper's inference type)
        mk("f16_tree30", 114, dtype=W.DT_F16, Hq=16, Hkv=4, D=128, ctx_lens=[1100], trees=[spec_tree(W.random_tree(15, 4, r))]),
        # fp16 (the paper's dtype) through the fast loop: long enough for many fast stages; with
        # outlier keys the fp16 P overflows its stale reference and the split is redone
        mk("f16_tree60_L5000", 117, dtype=W.DT_F16, Hq=8, Hkv=2, D=128, ctx_lens=[5000], trees=[W.random_tree(60, 6, r)]),
        mk("f16_outliers_L3000", 118, dtype=W.DT_F16, Hq=16, Hkv=2, D=128, ctx_lens=[3000, 900],
           trees=[W.hybrid_tree(32, 8, r) for _ in range(2)], outlier_frac=0.05),
        # fp32 storage, both head dims
        mk("f32_D64_tree10", 115, dtype=W.DT_F32, Hq=8, Hkv=2, D=64, ctx_lens=[700, 33], trees=[W.random_tree(10, 4, r) for _ in range(2)]),
        mk("f32_D128_chain5", 116, dtype=W.DT_F32, Hq=4, Hkv=2, D=128, ctx_lens=[390], trees=[W.chain_tree(5)]),
    ]
    return cs


@pytest.mark.parametrize("case", _small_cases(), ids=lambda c: c.name)
def test_small_shapes_match_oracle(oracle_mod, case):
    want = oracle_mod.verify_attn_case(case)
    for split in (0, 64, 192, 512):
        got, step = _run(case, split_tokens=split)
        assert_close(got, want, case.dtype, f"{case.name} split={split} plan={step.plan.as_dict()}")


# ---------------------------------------------------------------------------
# 16-bit output types
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("N,G", [(6, 4), (26, 4)])
def test_sixteen_bit_outputs_are_the_rounded_fp32_result(oracle_mod, N, G):
    """out_dtype = bf16 / f16: bit for bit the fp32 output rounded to nearest even, and within the
    fp32 bar widened by one unit in the last place of the output type against the rounded oracle."""
    r = _rng(640 + N)
    case = W.make_case("out16", 640 + N, dtype=W.DT_BF16, Hq=2 * G, Hkv=2, D=128, ctx_lens=[3000, 500],
                       trees=[W.random_tree(N, 5, r) for _ in range(2)])
    ref, _ = _run(case)
    want64 = oracle_mod.verify_attn_case(case)
    for od, dt in ((B.OWL_BF16, W.DT_BF16), (B.OWL_F16, W.DT_F16)):
        got, step = _run(case, out_dtype=od)
        assert got.dtype == np.uint16
        assert np.array_equal(got, W.store(ref, dt)), od
        want = W.widen(W.store(want64.astype(np.float32), dt), dt)           # the oracle rounded to the output type
        ulp = np.abs(want) * (2.0 ** -8 if dt == W.DT_BF16 else 2.0 ** -11) + 1e-7
        err = np.abs(W.widen(got, dt) - want)
        assert (err <= 1e-2 + ulp).all() and err.mean() <= 1e-3 + ulp.mean(), (od, err.max())


# ---------------------------------------------------------------------------
# the five named configurations
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("idx", range(5), ids=W.CONFIG_NAMES)
def test_configs_reduced_context_full_compare(oracle_mod, idx):
    """Same head shapes, trees and paging as the named configuration with the
    context cut to 1/16 (config 0 runs at its full 512 tokens), every output
    element compared."""
    case = W.make_config(idx, ctx_scale=1.0 if idx == 0 else 1.0 / 16)
    want = oracle_mod.verify_attn_case(case)
    got, step = _run(case)
    assert_close(got, want, case.dtype, f"{case.name} plan={step.plan.as_dict()}")


@pytest.mark.parametrize("idx", range(5), ids=W.CONFIG_NAMES)
def test_configs_full_size_all_rows(oracle_mod, idx):
    """Full context lengths, in the launch configuration the benchmark times
    (library-chosen splits); every output element against the oracle."""
    case = W.make_config(idx)
    got, step = _run(case)
    want = oracle_mod.verify_attn_case(case)
    assert_close(got, want, case.dtype, f"{case.name} plan={step.plan.as_dict()}")


@pytest.mark.parametrize("idx", [2, 3])
def test_configs_full_size_fp16(oracle_mod, idx):
    """The long-context configurations stored as fp16 (the paper's inference type), full size, every element."""
    case = W.make_config(idx, dtype=W.DT_F16)
    got, step = _run(case)
    want = oracle_mod.verify_attn_case(case)
    assert_close(got, want, case.dtype, f"{case.name} plan={step.plan.as_dict()}")


# ---------------------------------------------------------------------------
# evaluation-order invariance and exact properties on the GPU
# ---------------------------------------------------------------------------
def test_split_count_invariance(oracle_mod):
    """1 split vs many splits vs the planner's choice: all within tolerance of
    the oracle and of each other (catches combine races and stale partials)."""
    case = W.make_case("splitinv", 201, dtype=W.DT_BF16, Hq=32, Hkv=8, D=128, ctx_lens=[6000, 4097],
                       trees=[W.random_tree(26, 5, _rng(5)) for _ in range(2)])
    want = oracle_mod.verify_attn_case(case)
    outs = []
    for split in (16384, 4096, 1024, 128, 0):
        got, _ = _run(case, split_tokens=split)
        assert_close(got, want, case.dtype, f"split={split}")
        outs.append(got)
        raw, _ = _run(case, split_tokens=split, flags=B.OWL_FLAG_FP32_PARTIALS)      # partials as fp32 accumulators
        assert_close(raw, want, case.dtype, f"split={split}, fp32 partials")
        assert np.abs(raw - got).max() < 2e-3
    for o in outs[1:]:
        assert np.abs(o - outs[0]).max() < 5e-3


def test_non_ancestor_perturbation_is_invisible():
    """Overwriting K/V of draft j must leave every row whose path does not
    contain j bit-identical."""
    tree = W.random_tree(20, 5, _rng(7))
    base_case = W.make_case("perturb", 202, dtype=W.DT_BF16, Hq=8, Hkv=2, D=128, ctx_lens=[1000], trees=[tree])
    base, _ = _run(base_case)
    on_path = np.zeros((20, 20), bool)
    for i in range(20):
        j = i
        while j != -1:
            on_path[i, j] = True
            j = int(tree[j])
    for j in (0, 3, 11, 19):
        c2 = W.make_case("perturb", 202, dtype=W.DT_BF16, Hq=8, Hkv=2, D=128, ctx_lens=[1000], trees=[tree])
        pos = 1000 + j
        page = int(c2.page_table[0, pos // 16])
        c2.k_pool[page, :, pos % 16, :] = W.store(np.full((2, 128), 2.0, np.float32), W.DT_BF16)
        c2.v_pool[page, :, pos % 16, :] = W.store(np.full((2, 128), -9.0, np.float32), W.DT_BF16)
        got, _ = _run(c2)
        for i in range(20):
            if on_path[i, j]:
                assert np.abs(got[0, i] - base[0, i]).max() > 1e-4, (i, j)
            else:
                assert np.array_equal(got[0, i], base[0, i]), (i, j)


def test_page_permutation_is_invisible():
    kw = dict(dtype=W.DT_BF16, Hq=8, Hkv=2, D=128, ctx_lens=[3000, 700],
              trees=[W.random_tree(12, 4, _rng(8)) for _ in range(2)])
    a, _ = _run(W.make_case("perm", 203, paged=True, **kw))
    b, _ = _run(W.make_case("perm", 203, paged=False, **kw))
    c, _ = _run(W.make_case("perm", 203, paged=True, head_major=False, **kw))
    assert np.array_equal(a, b)
    assert np.array_equal(a, c)


def test_zero_query_integer_values_exact_mean():
    """q = 0, small-integer V, L + depth a power of two for the chain's last
    node: every weight is exactly 1, so the mean must be exact in fp32 -- any
    wrong, missing or doubled cache row shows up as a bit difference.  Exactness
    needs the partials in fp32 (OWL_FLAG_FP32_PARTIALS); the default partials,
    normalised and in fp16, must still be within 2^-11 of a row's largest value."""
    N, L = 4, 4096 - 4
    case = W.make_case("exact", 204, dtype=W.DT_BF16, Hq=4, Hkv=2, D=128, ctx_lens=[L], trees=[W.chain_tree(N)])
    case.q[...] = 0
    r = _rng(9)
    T = L + N
    vals = r.integers(-8, 9, size=(T, 2, 128)).astype(np.float32)
    for pos in range(T):
        page = int(case.page_table[0, pos // 16])
        case.v_pool[page, :, pos % 16, :] = W.store(vals[pos], W.DT_BF16)
    for split in (0, 128, 1024):
        want = vals.sum(axis=0, dtype=np.float64) / T            # last node sees all T rows
        got, _ = _run(case, split_tokens=split, flags=B.OWL_FLAG_FP32_PARTIALS)
        for h in range(4):
            assert np.array_equal(got[0, N - 1, h].astype(np.float64), want[h // 2]), split
        got, _ = _run(case, split_tokens=split)
        for h in range(4):
            assert np.abs(got[0, N - 1, h] - want[h // 2]).max() <= 2.0 ** -11 * np.abs(want[h // 2]).max() + 1e-6, split


def test_quad_max_lane_semantics():
    """The softmax's cross-lane maximum must cover exactly lanes l, l^16, l^32,
    l^48 (a wrong exchange would still give finite, nearly right outputs, so
    it is pinned here on its own)."""
    r = _rng(77)
    for _ in range(4):
        x = r.standard_normal(64).astype(np.float32)
        dx = torch.from_numpy(x).cuda()
        dy = torch.empty(64, dtype=torch.float32, device="cuda")
        B.owl_selftest_quad_max(dx, dy)
        torch.cuda.synchronize()
        want = x.reshape(4, 16).max(axis=0)
        assert np.array_equal(dy.cpu().numpy(), np.tile(want, 4))


# ---------------------------------------------------------------------------
# mask builder and paging: bit-exact
# ---------------------------------------------------------------------------
def test_tree_mask_bit_exact(oracle_mod):
    r = _rng(10)
    trees64 = [W.random_tree(64, md, r) for md in (None, 2, 8)] + [W.chain_tree(64), np.full(64, -1, np.int32)]
    trees6 = [spec_tree([-1, 0, 0]), W.chain_tree(6)]
    for trees in (trees64, trees6, [W.chain_tree(1)]):
        par = np.stack(trees).astype(np.int32)
        Bn, N = par.shape
        dpar = torch.from_numpy(par).cuda()
        anc = torch.zeros((Bn, N), dtype=torch.int64, device="cuda")
        dep = torch.zeros((Bn, N), dtype=torch.int32, device="cuda")
        st = torch.zeros(1, dtype=torch.int32, device="cuda")
        B.owl_build_tree_mask(dpar, anc, dep, st)
        torch.cuda.synchronize()
        assert int(st.item()) == 0
        for b in range(Bn):
            want_anc, want_dep = oracle_mod.tree_mask(par[b])
            assert np.array_equal(anc[b].cpu().numpy().view(np.uint64), want_anc)
            assert np.array_equal(dep[b].cpu().numpy(), want_dep)
            h_anc, h_dep = B.owl_build_tree_mask_host(par[b])
            assert np.array_equal(h_anc, want_anc) and np.array_equal(h_dep, want_dep)


def test_gather_bit_exact(oracle_mod):
    for head_major, dtype in ((True, W.DT_BF16), (False, W.DT_BF16), (True, W.DT_F32)):
        case = W.make_case("gather", 301, dtype=dtype, Hq=8, Hkv=4, D=128, ctx_lens=[1000, 37, 4000],
                           trees=[W.chain_tree(5)] * 3, head_major=head_major, spare_pages=7)
        step = VerifyStep(case)
        for b in range(case.B):
            T = int(case.ctx_lens[b]) + case.N
            for which, cache in (("k", step.k), ("v", step.v)):
                dst = torch.empty((T, case.Hkv, case.D), dtype=cache.dtype, device="cuda")
                B.owl_gather_kv(step.desc, cache, step.page_table, b, 0, T, dst, step.status)
                torch.cuda.synchronize()
                want = oracle_mod.gather_kv(case, which, b, 0, T)
                got = dst.cpu().numpy()
                assert np.array_equal(got.view(want.dtype), want)
        assert step.dev_status() == 0


def test_measurement_aids():
    """The streaming probes read what they claim to (their XOR folds agree with
    numpy) and the timeline hook records ordered timestamps for every workgroup."""
    r = _rng(78)
    host = r.integers(0, 2**31 - 1, size=(64 * 1024,), dtype=np.int64).astype(np.uint32)   # 256 KiB = 64 blocks
    dev = torch.from_numpy(host.view(np.int32)).cuda()
    want = int(np.bitwise_xor.reduce(host))
    sink = torch.zeros(64, dtype=torch.int32, device="cuda")
    B.owl_stream_read_probe(dev, sink, 8)
    torch.cuda.synchronize()
    assert int(np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32)[:8])) == want
    order = torch.from_numpy(r.permutation(64).astype(np.int32)).cuda()
    sink.zero_()
    B.owl_gather_read_probe(dev, order, sink, 5)
    torch.cuda.synchronize()
    assert int(np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32)[:5])) == want

    # the matrix-pipe probe: operands all 1.0 -> every accumulator is 32 per MFMA, 16 MFMAs deep per
    # iteration and lane: after 3 iterations sink = acc[i][0] + acc[i][3] summed over 16 accumulators
    ones = torch.ones(4096, dtype=torch.bfloat16, device="cuda")
    fs = torch.zeros(2 * 512, dtype=torch.float32, device="cuda")
    ghz = torch.zeros(2, dtype=torch.float32, device="cuda")
    B.owl_mfma_probe(ones, 3, fs, 2, clock_ghz=ghz)
    torch.cuda.synchronize()
    assert (fs.cpu().numpy() == 16 * 2 * 3 * 32.0).all()
    B.owl_mfma_probe(ones, 20000, fs, 2, clock_ghz=ghz)          # long enough for the 100 MHz counter to resolve
    torch.cuda.synchronize()
    assert ((ghz.cpu().numpy() > 0.3) & (ghz.cpu().numpy() < 3.0)).all()

    case = W.make_case("tl", 79, dtype=W.DT_BF16, Hq=32, Hkv=8, D=128, ctx_lens=[3000], trees=[W.random_tree(20, 4, r)])
    step = VerifyStep(case, split_tokens=512)
    step.run()
    ref = step.result().copy()
    nwg = step.plan.n_workgroups
    tl = torch.zeros(10 * nwg, dtype=torch.int64, device="cuda")
    B.owl_debug_set_timeline(tl)
    try:
        step.run()
        got = step.result()
    finally:
        B.owl_debug_set_timeline(None)
    assert np.array_equal(got, ref)                      # recording does not change the result
    t = tl.cpu().numpy().reshape(nwg, 10)
    ran = t[t[:, 0] > 0]
    # one workgroup per (kv head, split, row group): 48 streams do not fill the chip, so the 5 row tiles go to 2 groups
    assert step.plan.row_groups == 2 and len(ran) == 8 * ((3000 + 20 + 511) // 512) * step.plan.row_groups
    assert (np.diff(ran[:, :6], axis=1) >= 0).all()
    assert sorted(ran[:, 7]) == sorted(set(ran[:, 7]))
    assert (ran[:, 9] >= ran[:, 8]).all() and (ran[:, 8] > 0).all()   # shader cycles at both ends of the fast loop

    # the split-KV launch with events attached to its dispatch: same result, a plausible duration
    timer = B.KernelTimer()
    step.out.fill_(float("nan"))
    step.run_split_timed(timer)
    step.run(phases=B.PHASE_COMBINE)
    assert np.array_equal(step.result(), ref)
    assert 1e-3 < timer.elapsed_ms() < 50.0

    # the step probe: every wavefront reports its loop cycles, and the matrix pipe cannot be more than busy
    src = torch.randn(8192, device="cuda").to(torch.bfloat16)
    fs = torch.zeros(4 * 512, dtype=torch.float32, device="cuda")
    cyc = torch.zeros(4 * 8, dtype=torch.int64, device="cuda")
    for variant, _, tiles in B.STEP_PROBE_VARIANTS:
        cyc.zero_()
        B.owl_step_probe(variant, src, 200, fs, cyc, 4)
        torch.cuda.synchronize()
        per_step = cyc.cpu().numpy() / 200.0
        assert (per_step > tiles * 17 * 16 * 0.5).all() and (per_step < 50000).all(), (variant, per_step)
        assert np.isfinite(fs.cpu().numpy()).all()


# ---------------------------------------------------------------------------
# data errors on the device are flagged, never followed out of bounds
# ---------------------------------------------------------------------------
def test_device_side_errors_are_flagged():
    tree = W.random_tree(10, 4, _rng(11))
    def fresh():
        return W.make_case("bad", 401, dtype=W.DT_BF16, Hq=8, Hkv=2, D=128, ctx_lens=[500, 300], trees=[tree, tree])
    c = fresh()
    c.tree_parent[1, 4] = 7                      # child before parent
    s = VerifyStep(c); s.run()
    assert s.dev_status() & B.OWL_DEV_BAD_PARENT
    c = fresh()
    c.page_table[0, 3] = c.n_pool_pages + 5      # page outside the pool
    s = VerifyStep(c); s.run()
    assert s.dev_status() & B.OWL_DEV_BAD_PAGE
    c = fresh()
    s = VerifyStep(c, max_ctx_len=400)           # ctx_lens[0] = 500 > announced bound
    s.run()
    assert s.dev_status() & B.OWL_DEV_BAD_CTX_LEN
    # the sequence that was fine is still right next to a flagged one
    par = torch.from_numpy(np.array([[-1, 0, 5, 1]], np.int32)).cuda()
    anc = torch.zeros((1, 4), dtype=torch.int64, device="cuda")
    st = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.owl_build_tree_mask(par, anc, None, st)
    torch.cuda.synchronize()
    assert int(st.item()) & B.OWL_DEV_BAD_PARENT


# ---------------------------------------------------------------------------
# per-sequence draft counts
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,N,G,counts", [
    (W.DT_BF16, 26, 4, [26, 0, 9, 1, 17]),          # 7 row tiles, one sequence without drafts
    (W.DT_BF16, 60, 4, [60, 31, 2]),                # 15 row tiles (pipelined loop)
    (W.DT_BF16, 40, 8, [40, 13]),                   # 20 row tiles (three tiles per wave)
    (W.DT_BF16, 6, 4, [3, 6, 1, 5]),                # 2 row tiles (two key groups)
    (W.DT_F32, 10, 4, [4, 10]),
])
def test_ragged_draft_counts(oracle_mod, dtype, N, G, counts):
    r = _rng(900 + N)
    B_ = len(counts)
    ctx = [int(x) for x in r.integers(0, 3000, size=B_)]
    ctx[0] = 2500
    D = 64 if dtype == W.DT_F32 else 128
    case = W.make_case("ragged", 300 + N, dtype=dtype, Hq=2 * G, Hkv=2, D=D, ctx_lens=ctx,
                       trees=[W.random_tree(N, 6, r) for _ in range(B_)])
    want = oracle_mod.verify_attn_ragged_case(case, counts)
    for split in (0, 192):
        step = VerifyStep(case, split_tokens=split)
        nd = torch.tensor(counts, dtype=torch.int32, device=step.device)
        step.out.fill_(float("nan"))
        B.owl_verify_attn_ragged(step.desc, step.q, step.k, step.v, step.page_table, step.ctx_lens,
                                 step.tree_parent, nd, step.out, step.workspace, step.status)
        got = step.result()
        assert step.dev_status() == 0
        assert_close(got, want, case.dtype, f"ragged N={N} split={split}")
        for b, n in enumerate(counts):
            assert (got[b, n:] == 0).all()


@pytest.mark.parametrize("name,ctx,Hkv", [
    ("one long, many short", [9000] + [300] * 15, 8),            # under-filled launch: the long one is cut finer
    ("more sequences than lanes", None, 2),                      # 70 sequences: the second 64-chunk of the search
    ("equal lengths", [2000] * 12, 4),
    ("all empty prefixes", [0] * 5, 2),
])
def test_batch_split_follows_the_lengths(oracle_mod, name, ctx, Hkv):
    """A batch with a library-chosen split size: the kernels derive the split size from the
    actual lengths and number the (sequence, split) pairs densely; the result must not care,
    and the planned grid must hold every pair (an unserved pair would leave a row's partials
    unwritten and show as a mismatch)."""
    r = _rng(4242)
    if ctx is None:
        ctx = [int(x) for x in r.integers(0, 400, size=70)]
        ctx[3] = ctx[66] = 0
        ctx[69] = 1500
    n = 5
    case = W.make_case("batchsplit", 77, dtype=W.DT_BF16, Hq=4 * Hkv, Hkv=Hkv, D=128, ctx_lens=ctx,
                       trees=[W.random_tree(n, 3, r) for _ in ctx])
    want = oracle_mod.verify_attn_case(case)
    got, step = _run(case)
    assert_close(got, want, case.dtype, name)
    # the batch plan sits at the end of the workspace (split size, pair count, pairs before each sequence):
    # the size is a multiple of the 64-token stage, at most the planned one, and the pairs fit the launched grid
    plan_bytes = -(-(4 * (len(ctx) + 3)) // 256) * 256
    tail = step.workspace[-plan_bytes:].view(torch.int32).cpu().numpy()
    c_dev = int(tail[0])
    assert int(tail[1]) == sum(-(-(int(L) + n) // c_dev) for L in ctx) == int(tail[2 + len(ctx)])
    plan = step.plan
    assert c_dev % 64 == 0 and 64 <= c_dev <= plan.split_tokens
    pairs = sum(-(-(int(L) + n) // c_dev) for L in ctx)
    assert pairs * Hkv * plan.row_groups <= plan.n_workgroups
    assert all(-(-(int(L) + n) // c_dev) <= plan.max_splits for L in ctx)
    # announced longer than anything present: the plan (grid, partials) is for 65536, the lengths are not
    import dataclasses
    cols = (65536 + n + 15) // 16                        # the page table has to cover the planned length
    table = np.zeros((case.B, cols), dtype=np.int32)
    table[:, :case.page_table.shape[1]] = case.page_table
    wide = dataclasses.replace(case, page_table=table, max_pages_per_seq=cols)
    got2, step2 = _run(wide, max_ctx_len=65536)
    assert_close(got2, want, case.dtype, name + " (planned for 65536)")
    if len(ctx) <= 16:                                   # with per-sequence draft counts on top
        counts = [n if b % 3 else max(0, n - 2 - b % 2) for b in range(len(ctx))]
        counts[0] = 0 if len(ctx) > 1 else n
        want3 = oracle_mod.verify_attn_ragged_case(case, counts)
        nd = torch.tensor(counts, dtype=torch.int32, device=step.device)
        B.owl_verify_attn_ragged(step.desc, step.q, step.k, step.v, step.page_table, step.ctx_lens,
                                 step.tree_parent, nd, step.out, step.workspace, step.status)
        got3 = step.result()
        assert step.dev_status() == 0
        assert_close(got3, want3, case.dtype, name + " (ragged counts)")


@pytest.mark.parametrize("frac,gain,tag", [(0.05, 8.0, "frequent outliers: guarded reference"),
                                           (0.0007, 40.0, "rare late outliers: frozen reference, overflow, redo"),
                                           (0.02, 3.0, "mild tail: frozen reference holds")])
@pytest.mark.parametrize("N,G", [(6, 4), (60, 4), (40, 8)])     # 2 / 15 / 20 row tiles: all three fast loops
def test_fp16_score_range_paths(oracle_mod, frac, gain, tag, N, G):
    """fp16 probabilities overflow 2^16 above their reference.  The kernel probes the first stages of
    a split and takes a loop with a guarded (moving) reference if the scores already show a long
    tail; otherwise it freezes the reference and, should a later score overflow it after all,
    redoes the split with the exact loop.  All three routes must give the oracle's result."""
    r = _rng(77 + N)
    case = W.make_case("f16range", 910 + N, dtype=W.DT_F16, Hq=2 * G, Hkv=2, D=128, ctx_lens=[9000, 700],
                       trees=[W.random_tree(N, 6, r) for _ in range(2)], outlier_frac=frac, outlier_gain=gain)
    got, step = _run(case)
    assert_close(got, oracle_mod.verify_attn_case(case), case.dtype, f"{tag}, N={N} G={G}")


@pytest.mark.parametrize("N,G", [(6, 4), (60, 4), (40, 8)])     # 2 / 15 / 20 row tiles: all three fast loops
def test_bf16_reference_overflow_redo(oracle_mod, N, G):
    """bf16 storage keeps the softmax reference of a split frozen at the maxima of its first keys.
    A later score more than ~100 (log2 units) above it overflows 2^(x - m); the row sum shows it
    and the split is redone with the exact loop.  Here a few late prefix keys of every split are
    64 times longer than the rest (an exact change of exponent in bf16), which puts some row's
    score more than 104 above everything in the first 64 keys of that split -- checked below on
    the host, so that the redo is known to be on the path -- and the result must still be the
    oracle's."""
    r = _rng(5100 + N)
    L, C = 9000, 2048
    case = W.make_case("bf16_redo", 930 + N, dtype=W.DT_BF16, Hq=2 * G, Hkv=2, D=128, ctx_lens=[L],
                       trees=[W.random_tree(N, 6, r)])
    hot = [C + 700, 2 * C + 1500, 3 * C + 100, 4 * C + 300]        # one per split but the first; never in a split's first 64 keys
    for pos in hot:
        page = int(case.page_table[0, pos // 16])
        row = W.widen(case.k_pool[page, :, pos % 16, :], W.DT_BF16) * 64.0
        case.k_pool[page, :, pos % 16, :] = W.store(row.astype(np.float32), W.DT_BF16)
    # host check of the premise, from the stored values: x = scale * log2(e) * q.k in float64
    q = W.widen(case.q[0], W.DT_BF16)                                # [N, Hq, D]
    c = case.scale * 1.4426950408889634
    for pos in hot:
        first = np.arange(pos // C * C, pos // C * C + 64)
        pages = case.page_table[0, first // 16]
        k_first = W.widen(case.k_pool[pages, :, first % 16, :], W.DT_BF16)          # [64, Hkv, D]
        k_hot = W.widen(case.k_pool[int(case.page_table[0, pos // 16]), :, pos % 16, :], W.DT_BF16)
        over = -np.inf
        for h in range(case.Hq):
            x_first = c * np.einsum("nd,kd->nk", q[:, h], k_first[:, h // G])     # [N, 64]
            x_hot = c * q[:, h] @ k_hot[h // G]                                    # [N]
            over = max(over, float((x_hot - x_first.max(axis=1)).max()))
        assert over > 104.0, f"the case does not overflow the frozen reference of the split of key {pos}: {over:.1f}"
    want = oracle_mod.verify_attn_case(case)
    for split in (C, 0):                                  # the split size the premise was checked for, and the library's own
        got, step = _run(case, split_tokens=split)
        assert_close(got, want, case.dtype, f"N={N} G={G} split={split} plan={step.plan.as_dict()}")


def test_graph_capture_replays_match_eager(oracle_mod):
    """No entry point allocates, clears memory or synchronises, so a verify step can be captured
    in a HIP graph.  The graph is replayed several times with new queries and lengths in the
    same buffers, with eager work and synchronisations in between; every replay must equal the
    eager result on the same inputs."""
    r = _rng(606)
    ctx = [1500, 40, 700]
    case = W.make_case("graph", 61, dtype=W.DT_BF16, Hq=16, Hkv=4, D=128, ctx_lens=ctx,
                       trees=[W.random_tree(12, 4, r) for _ in ctx])
    step = VerifyStep(case)
    B.owl_verify_attn_init(step.desc)                     # one-time kernel attributes, outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step.run()
    torch.cuda.synchronize()
    q0 = step.q.clone()
    for rep in range(4):
        if rep:                                           # new inputs in place: scaled queries, shorter contexts
            step.q.copy_((q0.view(torch.bfloat16).float() * (1.0 + 0.25 * rep)).to(torch.bfloat16).view(torch.int16))
            step.ctx_lens.copy_(torch.tensor([1500 - 100 * rep, 40, 700 - 300 * (rep % 2)], dtype=torch.int32))
        torch.cuda.synchronize()
        step.out.fill_(float("nan"))
        graph.replay()
        got = step.result().copy()
        step.out.fill_(float("nan"))
        step.run()                                        # eager, same buffers
        want = step.result().copy()
        assert step.dev_status() == 0
        assert np.array_equal(got, want), f"replay {rep}"
    # and the first replay's inputs were the seeded case: against the oracle too
    step.q.copy_(q0)
    step.ctx_lens.copy_(torch.tensor(ctx, dtype=torch.int32))
    torch.cuda.synchronize()
    graph.replay()
    assert_close(step.result(), oracle_mod.verify_attn_case(case), case.dtype, "graph replay")


def test_ragged_flags_bad_counts():
    case = W.make_case("ragged_bad", 77, dtype=W.DT_BF16, Hq=8, Hkv=2, D=128, ctx_lens=[300, 200],
                       trees=[W.chain_tree(5) for _ in range(2)])
    step = VerifyStep(case)
    nd = torch.tensor([9, -1], dtype=torch.int32, device=step.device)
    B.owl_verify_attn_ragged(step.desc, step.q, step.k, step.v, step.page_table, step.ctx_lens,
                             step.tree_parent, nd, step.out, step.workspace, step.status)
    got = step.result()
    assert step.dev_status() & B.OWL_DEV_BAD_NDRAFT
    assert np.isfinite(got).all() and (got[1] == 0).all()            # 9 -> 5 nodes, -1 -> none


# ---------------------------------------------------------------------------
# a single sequence much shorter than the length the plan was made for
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("L,planned", [(0, 131072), (100, 131072), (3000, 131072), (40000, 65536), (5000, 5000), (4999, 5000)])
def test_context_shorter_than_planned(oracle_mod, L, planned):
    """The plan is sized by max_ctx_len; the kernels re-cut a shorter lone sequence into the
    same number of splits.  Same result either way."""
    case = W.make_case("short_ctx", 500 + L % 97, dtype=W.DT_BF16, Hq=8, Hkv=2, D=128, ctx_lens=[L],
                       trees=[W.random_tree(14, 4, _rng(L + 1))])
    want = oracle_mod.verify_attn_case(case)
    # the page table has to cover the planned length: pad its row (the extra entries are never read)
    import dataclasses
    cols = (planned + case.N + 15) // 16
    table = np.zeros((1, cols), dtype=np.int32)
    table[:, :case.page_table.shape[1]] = case.page_table
    wide = dataclasses.replace(case, page_table=table, max_pages_per_seq=cols)
    got, step = _run(wide, max_ctx_len=planned)
    assert_close(got, want, case.dtype, f"L={L} planned={planned} plan={step.plan.as_dict()}")
    exact, _ = _run(case)
    assert_close(got, exact.astype(np.float64), case.dtype, "planned-for-longer vs planned-exactly")


# ---------------------------------------------------------------------------
# the largest shapes the entry point takes
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("name,kw", [
    # 64 drafted nodes x 8 query heads per KV head = 512 rows = 32 row tiles: two row groups of 24 + 8 tiles
    ("n64_g8_tree", dict(dtype=W.DT_BF16, Hq=16, Hkv=2, D=128, ctx_lens=[20000], N=64, depth=8)),
    # the same with fp16 storage and head_dim 64
    ("n64_g8_f16_d64", dict(dtype=W.DT_F16, Hq=16, Hkv=2, D=64, ctx_lens=[9000, 1], N=64, depth=8)),
    # 16 query heads on ONE KV head (multi-query attention), 24 row tiles exactly: three tiles on every wave
    ("mqa_g16_n24", dict(dtype=W.DT_BF16, Hq=16, Hkv=1, D=128, ctx_lens=[15000], N=24, depth=6)),
    # no grouping at all (Hq = Hkv), the deepest chain the mask word holds
    ("mha_chain64", dict(dtype=W.DT_BF16, Hq=4, Hkv=4, D=128, ctx_lens=[5000, 33], N=64, depth=None)),
    # a forest of 64 roots: every node sees only itself among the drafts
    ("forest64", dict(dtype=W.DT_BF16, Hq=8, Hkv=2, D=128, ctx_lens=[3000], N=64, depth=0)),
])
def test_largest_shapes_every_element(oracle_mod, name, kw):
    r = _rng(sum(map(ord, name)))                      # a fixed seed per case
    N, depth = kw.pop("N"), kw.pop("depth")
    def tree():
        if depth is None:
            return W.chain_tree(N)
        if depth == 0:
            return np.full(N, -1, np.int32)
        return W.random_tree(N, depth, r)
    case = W.make_case(name, 7000 + N, trees=[tree() for _ in kw["ctx_lens"]], **kw)
    want = oracle_mod.verify_attn_case(case)
    for split in (0, 1024):
        got, step = _run(case, split_tokens=split)
        assert_close(got, want, case.dtype, f"{name} split={split} plan={step.plan.as_dict()}")


# ---------------------------------------------------------------------------
# one GPU's share of a model whose KV heads are spread over several GPUs
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("name,Hkv,G,N,L,groups,split,groups_at_split", [
    ("70b_over_8_gpus", 1, 8, 40, 24000, 5, 1472, 5),     # 20 row tiles on one KV head: five row groups of four tiles
    ("70b_over_4_gpus", 2, 8, 40, 24000, 5, 512, 3),      # two KV heads; with 47 splits: three groups of seven tiles
    ("70b_over_4_gpus_b", 2, 8, 40, 24000, 5, 256, 2),    # with 94 splits: two groups of ten (two tiles per wave)
    ("8b_over_8_gpus", 1, 4, 60, 12000, 4, 320, 4),       # 15 tiles: 4 + 4 + 4 + 3
    ("wide_on_one_head", 1, 8, 64, 6000, 8, 1472, 8),     # 32 tiles on one head of a short context: eight groups
])
def test_few_kv_heads_use_row_groups(oracle_mod, name, Hkv, G, N, L, groups, split, groups_at_split):
    """With one or two KV heads the splits alone cannot give every compute unit a workgroup: the rows
    are cut into row groups (workgroups that read the same split).  Every element against the oracle,
    with the library's own plan and with a forced split size that does not divide the context."""
    r = _rng(sum(map(ord, name)))
    case = W.make_case(name, 8100 + N, dtype=W.DT_BF16, Hq=Hkv * G, Hkv=Hkv, D=128, ctx_lens=[L],
                       trees=[W.random_tree(N, 8, r)], outlier_frac=0.05)
    want = oracle_mod.verify_attn_case(case)
    got, step = _run(case)
    assert step.plan.row_groups == groups, step.plan.as_dict()
    assert_close(got, want, case.dtype, f"{name} plan={step.plan.as_dict()}")
    got, step = _run(case, split_tokens=split)
    assert step.plan.row_groups == groups_at_split, step.plan.as_dict()
    assert_close(got, want, case.dtype, f"{name} split={split} plan={step.plan.as_dict()}")


# ---------------------------------------------------------------------------
# a context near the upper end: one million tokens, pools beyond 2^31 bytes
# ---------------------------------------------------------------------------
def test_million_token_context(oracle_mod):
    """64-bit addressing of the pool (beyond 2^31 bytes), 68 splits per KV head, page ids above 2^16."""
    L = 1_100_003
    case = W.make_case("ctx_1m", 4242, dtype=W.DT_BF16, Hq=16, Hkv=8, D=128, ctx_lens=[L],
                       trees=[W.random_tree(10, 4, _rng(3))])
    assert case.k_pool.nbytes > 2**31
    got, step = _run(case)
    rows = sample_rows(case, 10, seed=9, always=[(0, 0, 0), (0, case.N - 1, case.Hq - 1)])
    want = oracle_mod.verify_attn_case(case, rows=rows)
    sub = np.stack([got[b, i, h] for b, i, h in rows])
    assert_close(sub, want, case.dtype, f"plan={step.plan.as_dict()}")
    assert np.isfinite(got).all()
