"""GPU parity of the steps around the verify attention (Prepare, greedy
acceptance, KV commit) against ``oracle/steps.py``: all bit-exact.  Needs an
MI355X (-m gpu); every call goes through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import steps as S
from paper_2510_07535_amd import binding as B
from paper_2510_07535_amd import workloads as W
from paper_2510_07535_amd.runner import VerifyStep, _to_dev

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _rng(k):
    return np.random.Generator(np.random.Philox(key=k))


def _i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


# --------------------------------------------------------------------------- Prepare
@pytest.mark.parametrize("n,B_,seed", [(1, 1, 1), (3, 2, 2), (17, 5, 3), (30, 16, 4), (32, 3, 5)])
def test_prepare_matches_oracle(n, B_, seed):
    r = _rng(seed)
    parents = np.stack([W.random_tree(n, 8 if b % 2 else None, r) for b in range(B_)])
    if B_ > 1:
        parents[1] = W.chain_tree(n)
    ctx = r.integers(0, 131072, size=B_).astype(np.int32)
    p2_o, anc_o, dep_o, pos_o = S.prepare_spec_tree(parents, ctx)
    p2 = torch.full((B_, 2 * n), -7, dtype=torch.int32, device=DEV)
    anc = torch.zeros((B_, 2 * n), dtype=torch.int64, device=DEV)
    dep = torch.zeros((B_, 2 * n), dtype=torch.int32, device=DEV)
    pos = torch.zeros((B_, 2 * n), dtype=torch.int32, device=DEV)
    st = torch.zeros(1, dtype=torch.int32, device=DEV)
    B.owl_prepare_spec_tree(_i32(parents), _i32(ctx), p2, anc, dep, pos, st)
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    assert np.array_equal(p2.cpu().numpy(), p2_o)
    assert np.array_equal(anc.cpu().numpy().view(np.uint64), anc_o)
    assert np.array_equal(dep.cpu().numpy(), dep_o)
    assert np.array_equal(pos.cpu().numpy(), pos_o)


def test_prepare_output_feeds_the_verify_attention():
    """The 2n-token tree from Prepare is an ordinary tree_parent for owl_verify_attn:
    an extra token's output row equals that of an ordinary leaf child of its node."""
    import oracle
    r = _rng(77)
    n = 10
    tree = W.random_tree(n, 4, r)
    p2 = torch.zeros((1, 2 * n), dtype=torch.int32, device=DEV)
    anc = torch.zeros((1, 2 * n), dtype=torch.int64, device=DEV)
    B.owl_prepare_spec_tree(_i32(tree[None]), _i32([900]), p2, anc)
    torch.cuda.synchronize()
    tree2 = p2.cpu().numpy()[0]
    case = W.make_case("spec20", 5, dtype=W.DT_BF16, Hq=8, Hkv=2, D=128, ctx_lens=[900], trees=[tree2])
    step = VerifyStep(case)
    step.run()
    out = step.result()
    ref = oracle.verify_attn_case(case)
    assert np.abs(out - ref).max() < 1e-2 and np.abs(out - ref).mean() < 1e-3
    assert step.dev_status() == 0


def test_prepare_flags_bad_parent():
    parents = np.array([[-1, 0, 5, 1]], dtype=np.int32)               # node 2 points forward
    p2 = torch.zeros((1, 8), dtype=torch.int32, device=DEV)
    anc = torch.zeros((1, 8), dtype=torch.int64, device=DEV)
    st = torch.zeros(1, dtype=torch.int32, device=DEV)
    B.owl_prepare_spec_tree(_i32(parents), _i32([3]), p2, anc, None, None, st)
    torch.cuda.synchronize()
    assert int(st.item()) & B.OWL_DEV_BAD_PARENT
    assert p2.cpu().numpy()[0, 2] == -1                                # treated as a root, output stays a valid tree


# --------------------------------------------------------------------------- acceptance
def _accept_gpu(tok, parent, root, tgt, n_cand):
    B_, N = tok.shape
    acc = torch.full((B_, N), -9, dtype=torch.int32, device=DEV)
    na = torch.full((B_,), -9, dtype=torch.int32, device=DEV)
    bonus = torch.full((B_,), -9, dtype=torch.int32, device=DEV)
    last = torch.full((B_,), -9, dtype=torch.int32, device=DEV)
    st = torch.zeros(1, dtype=torch.int32, device=DEV)
    B.owl_accept_greedy(_i32(tok), _i32(parent), _i32(root), _i32(tgt), n_cand, acc, na, bonus, last, st)
    torch.cuda.synchronize()
    return acc.cpu().numpy(), na.cpu().numpy(), bonus.cpu().numpy(), last.cpu().numpy(), int(st.item())


@pytest.mark.parametrize("N,B_,vocab,seed", [(1, 1, 2, 1), (6, 4, 2, 2), (26, 16, 3, 3), (60, 7, 2, 4), (64, 5, 4, 5),
                                             (64, 3, 1, 6)])
def test_accept_matches_oracle(N, B_, vocab, seed):
    """Small vocabularies make agreements (and duplicate siblings, i.e. ties) frequent."""
    r = _rng(seed)
    parent = np.stack([W.chain_tree(N) if b == 0 else W.random_tree(N, 8, r) for b in range(B_)])
    tok = r.integers(0, vocab, size=(B_, N))
    tgt = r.integers(0, vocab, size=(B_, N))
    root = r.integers(0, vocab, size=B_)
    for n_cand in sorted({N, N // 2, 0}):
        want = S.accept_greedy(tok, parent, root, tgt, n_cand)
        got = _accept_gpu(tok, parent, root, tgt, n_cand)
        assert got[4] == 0
        for w, g in zip(want, got[:4]):
            assert np.array_equal(w, g), (n_cand, w, g)


def test_accept_on_a_prepared_tree():
    r = _rng(9)
    n = 30
    parent = np.stack([W.random_tree(n, 8, r) for _ in range(4)])
    p2, *_ = S.prepare_spec_tree(parent, np.zeros(4, np.int32))
    tok = r.integers(0, 2, size=(4, 2 * n))
    tgt = r.integers(0, 2, size=(4, 2 * n))
    root = r.integers(0, 2, size=4)
    want = S.accept_greedy(tok, p2, root, tgt, n)
    got = _accept_gpu(tok, p2, root, tgt, n)
    for w, g in zip(want, got[:4]):
        assert np.array_equal(w, g)
    assert (got[3] < n).all()                                          # an extra token is never accepted


# --------------------------------------------------------------------------- KV commit
def _commit_case(dtype, D, head_major, paged, seed):
    r = _rng(seed)
    N = 24
    ctx = [37, 1000, 0, 16]
    trees = [W.random_tree(N, 6, r) for _ in ctx]
    return W.make_case("commit", seed, dtype=dtype, Hq=8, Hkv=4, D=D, ctx_lens=ctx, trees=trees,
                       head_major=head_major, paged=paged)


def _random_paths(case, r):
    acc = np.full((case.B, case.N), -1, dtype=np.int32)
    na = np.zeros(case.B, dtype=np.int32)
    for b in range(case.B):
        leaf = int(r.integers(0, case.N))
        path = []
        j = leaf
        while j >= 0:
            path.append(j)
            j = int(case.tree_parent[b, j])
        path = path[::-1]
        if b == 2:
            path = []                                                 # nothing accepted for this sequence
        acc[b, :len(path)] = path
        na[b] = len(path)
    return acc, na


@pytest.mark.parametrize("dtype,D,head_major,paged", [(W.DT_BF16, 128, True, True), (W.DT_BF16, 64, False, True),
                                                      (W.DT_F32, 64, True, True), (W.DT_F16, 128, True, False)])
def test_commit_matches_oracle(dtype, D, head_major, paged):
    case = _commit_case(dtype, D, head_major, paged, 31)
    r = _rng(32)
    acc, na = _random_paths(case, r)
    step = VerifyStep(case)
    new_ctx = torch.zeros(case.B, dtype=torch.int32, device=DEV)
    B.owl_commit_kv(step.desc, step.k, step.v, step.page_table, step.ctx_lens, _i32(acc), _i32(na), new_ctx,
                    step.status)
    torch.cuda.synchronize()
    assert step.dev_status() == 0
    for name, pool, dev in (("k", case.k_pool, step.k), ("v", case.v_pool, step.v)):
        want, want_ctx = S.commit_kv(pool, case.page_table, case.ctx_lens, acc, na, case.stride_page,
                                     case.stride_head, case.stride_token, case.Hkv, case.D)
        got = dev.cpu().numpy().view(pool.dtype).reshape(pool.shape)
        assert np.array_equal(got.view(np.uint8), want.view(np.uint8)), name
        assert np.array_equal(new_ctx.cpu().numpy(), want_ctx)


def test_commit_then_verify_sees_the_committed_rows():
    """After the commit, a verify step over the longer context reads the moved rows:
    compare with the oracle run on the oracle-committed cache."""
    import dataclasses
    import oracle
    case = _commit_case(W.DT_BF16, 128, True, True, 41)
    acc, na = _random_paths(case, _rng(42))
    step = VerifyStep(case)
    new_ctx = torch.zeros(case.B, dtype=torch.int32, device=DEV)
    B.owl_commit_kv(step.desc, step.k, step.v, step.page_table, step.ctx_lens, _i32(acc), _i32(na), new_ctx)
    # the next step: a chain of 3 fresh nodes behind the grown context; their K/V rows are whatever
    # the cache holds at those positions, on both sides alike
    k2, ctx2 = S.commit_kv(case.k_pool, case.page_table, case.ctx_lens, acc, na, case.stride_page,
                           case.stride_head, case.stride_token, case.Hkv, case.D)
    v2, _ = S.commit_kv(case.v_pool, case.page_table, case.ctx_lens, acc, na, case.stride_page,
                        case.stride_head, case.stride_token, case.Hkv, case.D)
    n2 = 3
    nxt = dataclasses.replace(case, k_pool=k2, v_pool=v2, ctx_lens=ctx2, N=n2,
                              tree_parent=np.tile(W.chain_tree(n2), (case.B, 1)),
                              q=np.ascontiguousarray(case.q[:, :n2]))
    ref = oracle.verify_attn_case(nxt)
    step2 = VerifyStep(nxt, max_ctx_len=int(ctx2.max()))
    step2.k, step2.v = step.k, step.v                                  # the GPU-committed caches
    step2.ctx_lens = new_ctx
    step2.run()
    out = step2.result()
    assert step2.dev_status() == 0
    assert np.abs(out - ref).max() < 1e-2 and np.abs(out - ref).mean() < 1e-3


def test_commit_flags_bad_lists_and_moves_nothing():
    case = _commit_case(W.DT_BF16, 128, True, True, 51)
    step = VerifyStep(case)
    acc = np.full((case.B, case.N), -1, dtype=np.int32)
    na = np.array([2, 3, 1, 0], dtype=np.int32)
    acc[0, :2] = [3, 3]                                                # not strictly increasing
    acc[1, :3] = [0, 1, case.N]                                        # out of range
    acc[2, :1] = [5]                                                   # fine
    new_ctx = torch.zeros(case.B, dtype=torch.int32, device=DEV)
    B.owl_commit_kv(step.desc, step.k, step.v, step.page_table, step.ctx_lens, _i32(acc), _i32(na), new_ctx,
                    step.status)
    torch.cuda.synchronize()
    assert step.dev_status() & B.OWL_DEV_BAD_ACCEPT
    assert new_ctx.cpu().numpy().tolist() == [37, 1000, 1, 16]
    want, _ = S.commit_kv(case.k_pool, case.page_table, case.ctx_lens, acc, np.array([0, 0, 1, 0]), case.stride_page,
                          case.stride_head, case.stride_token, case.Hkv, case.D)
    got = step.k.cpu().numpy().view(case.k_pool.dtype).reshape(case.k_pool.shape)
    assert np.array_equal(got, want)


def test_commit_with_a_bad_page_moves_nothing_for_that_sequence():
    """A page-table entry outside the pool under a source or a destination row: the sequence is
    flagged and left alone (pools byte-identical, length unchanged); the other sequences commit."""
    case = _commit_case(W.DT_BF16, 128, True, True, 61)
    acc, na = _random_paths(case, _rng(62))
    assert na[0] > 0 and na[1] > 0
    for which in ("destination", "source"):
        table = case.page_table.copy()
        L0 = int(case.ctx_lens[0])
        pos = L0 if which == "destination" else L0 + int(acc[0, na[0] - 1])
        table[0, pos // 16] = -1
        step = VerifyStep(case)
        step.page_table = _i32(table)
        new_ctx = torch.zeros(case.B, dtype=torch.int32, device=DEV)
        B.owl_commit_kv(step.desc, step.k, step.v, step.page_table, step.ctx_lens, _i32(acc), _i32(na), new_ctx,
                        step.status)
        torch.cuda.synchronize()
        assert step.dev_status() & B.OWL_DEV_BAD_PAGE, which
        na_eff = na.copy()
        na_eff[0] = 0                                                  # what the flagged sequence is reduced to
        for name, pool, dev in (("k", case.k_pool, step.k), ("v", case.v_pool, step.v)):
            want, want_ctx = S.commit_kv(pool, case.page_table, case.ctx_lens, acc, na_eff, case.stride_page,
                                         case.stride_head, case.stride_token, case.Hkv, case.D)
            got = dev.cpu().numpy().view(pool.dtype).reshape(pool.shape)
            assert np.array_equal(got.view(np.uint8), want.view(np.uint8)), (which, name)
            assert np.array_equal(new_ctx.cpu().numpy(), want_ctx), which


# --------------------------------------------------------------------------- the steps in a loop
def test_decode_loop_stays_in_step_with_the_oracle():
    """Five rounds of Prepare -> verify attention -> acceptance -> KV commit with every array
    staying on the device between the calls (the tree, the accepted path, the new lengths and the
    compacted cache of one call are the next call's inputs), against the same loop on the oracle:
    integer state and cache bytes identical after every round, attention within the bf16 bound."""
    import dataclasses
    import oracle
    r = _rng(2024)
    n, rounds = 12, 5
    N = 2 * n
    start = np.array([37, 1000, 0, 16, 255], dtype=np.int32)
    room = rounds * n                                                  # a round accepts at most n nodes
    trees0 = [W.chain_tree(N) for _ in start]
    cap = W.make_case("loop", 88, dtype=W.DT_BF16, Hq=8, Hkv=4, D=128, ctx_lens=(start + room).tolist(),
                      trees=trees0, paged=True, head_major=True)
    case = dataclasses.replace(cap, ctx_lens=start.copy())
    step = VerifyStep(case, max_ctx_len=int(start.max()) + room)
    Bn = case.B
    p2 = torch.zeros((Bn, N), dtype=torch.int32, device=DEV)
    anc = torch.zeros((Bn, N), dtype=torch.int64, device=DEV)
    acc = torch.zeros((Bn, N), dtype=torch.int32, device=DEV)
    na = torch.zeros(Bn, dtype=torch.int32, device=DEV)
    bonus = torch.zeros(Bn, dtype=torch.int32, device=DEV)
    last = torch.zeros(Bn, dtype=torch.int32, device=DEV)
    ctx_dev = [step.ctx_lens, torch.zeros(Bn, dtype=torch.int32, device=DEV)]
    k_o, v_o, ctx_o = case.k_pool, case.v_pool, start.copy()
    strides = (case.stride_page, case.stride_head, case.stride_token, case.Hkv, case.D)
    grew = 0
    for it in range(rounds):
        parents = np.stack([W.chain_tree(n) if b == it % Bn else W.random_tree(n, 4, r) for b in range(Bn)])
        tok = r.integers(0, 2, size=(Bn, N))                           # two-word vocabulary: long accepted paths
        tgt = r.integers(0, 2, size=(Bn, N))
        root = r.integers(0, 2, size=Bn)
        # oracle round
        p2_o, *_ = S.prepare_spec_tree(parents, ctx_o)
        ref = oracle.verify_attn_case(dataclasses.replace(case, k_pool=k_o, v_pool=v_o, ctx_lens=ctx_o,
                                                          tree_parent=p2_o))
        acc_o, na_o, bonus_o, last_o = S.accept_greedy(tok, p2_o, root, tgt, n)
        k_o, ctx_n = S.commit_kv(k_o, case.page_table, ctx_o, acc_o, na_o, *strides)
        v_o, _ = S.commit_kv(v_o, case.page_table, ctx_o, acc_o, na_o, *strides)
        # device round: no host copies between the calls
        cur, nxt = ctx_dev[it % 2], ctx_dev[(it + 1) % 2]
        B.owl_prepare_spec_tree(_i32(parents), cur, p2, anc, None, None, step.status)
        step.ctx_lens, step.tree_parent = cur, p2
        step.run()
        B.owl_accept_greedy(_i32(tok), p2, _i32(root), _i32(tgt), n, acc, na, bonus, last, step.status)
        B.owl_commit_kv(step.desc, step.k, step.v, step.page_table, cur, acc, na, nxt, step.status)
        out = step.result()
        assert step.dev_status() == 0, it
        assert np.array_equal(p2.cpu().numpy(), p2_o), it
        assert np.abs(out - ref).max() < 1e-2 and np.abs(out - ref).mean() < 1e-3, (it, np.abs(out - ref).max())
        assert np.array_equal(acc.cpu().numpy(), acc_o) and np.array_equal(na.cpu().numpy(), na_o), it
        assert np.array_equal(bonus.cpu().numpy(), bonus_o) and np.array_equal(last.cpu().numpy(), last_o), it
        assert np.array_equal(nxt.cpu().numpy(), ctx_n), it
        for name, want, dev in (("k", k_o, step.k), ("v", v_o, step.v)):
            got = dev.cpu().numpy().view(want.dtype).reshape(want.shape)
            assert np.array_equal(got.view(np.uint8), want.view(np.uint8)), (it, name)
        grew += int((ctx_n - ctx_o).sum())
        ctx_o = ctx_n
    assert grew > rounds                                               # the loop did move rows
