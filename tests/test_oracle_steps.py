"""Pins of the oracle's integer / data-movement steps (``oracle/steps.py``) against
what the paper prints, closed forms, hand-worked cases and the already pinned C
oracle (``tree_mask``, ``gather_kv``).  No GPU."""
import dataclasses
import os

import numpy as np
import pytest

import oracle
from oracle import steps as S
from paper_2510_07535_amd import workloads as W
from tree_helpers import node_depths

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "spec_tree_example.txt")


def _golden():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    parent = np.array([int(x) for x in rows[0]], dtype=np.int32)
    anc = np.array([int(x, 2) for x in rows[1]], dtype=np.uint64)
    depth = np.array([int(x) for x in rows[2]], dtype=np.int32)
    return parent, anc, depth


# --------------------------------------------------------------------------- Prepare
def test_prepare_paper_example():
    """Sec. 3.2.2: tree t1 -> {t2, t2'}; the three extra tokens follow (t1), (t1,t2), (t1,t2')."""
    parent2, anc, depth = _golden()
    n = len(parent2) // 2
    p2, a, d, pos = S.prepare_spec_tree(parent2[None, :n], np.array([100]))
    assert np.array_equal(p2[0], parent2)
    assert np.array_equal(a[0], anc)
    assert np.array_equal(d[0], depth)
    # t1 is the first new token: position 100; t2, t2' and t1's extra token come second; the others third
    assert pos[0].tolist() == [100, 101, 101, 101, 102, 102]


def test_prepare_chain_closed_form():
    n, L = 7, 1234
    p2, a, d, pos = S.prepare_spec_tree(W.chain_tree(n)[None], np.array([L]))
    assert pos[0, :n].tolist() == list(range(L, L + n))
    assert pos[0, n:].tolist() == list(range(L + 1, L + n + 1))
    for i in range(n):
        assert int(a[0, i]) == (1 << (i + 1)) - 1                      # causal
        assert int(a[0, n + i]) == ((1 << (i + 1)) - 1) | (1 << (n + i))


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_prepare_agrees_with_pinned_mask_sweep(seed):
    """The doubled parent array, fed to the (separately pinned) C mask builder,
    must give the same masks and depths as the path walk; positions = L + depth - 1."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    n = 30
    parents = np.stack([W.random_tree(n, 8, rng), W.random_tree(n, None, rng)])
    ctx = np.array([4097, 77], dtype=np.int32)
    p2, a, d, pos = S.prepare_spec_tree(parents, ctx)
    for b in range(2):
        anc_c, depth_c = oracle.tree_mask(p2[b])
        assert np.array_equal(anc_c, a[b])
        assert np.array_equal(depth_c, d[b])
        assert np.array_equal(pos[b], ctx[b] + d[b] - 1)
        for k in range(n):                                             # an extra token sees its node's path + itself
            assert int(a[b, n + k]) == int(a[b, k]) | (1 << (n + k))
            assert int(a[b, n + k]) >> n == 1 << k                     # and no other extra token


def test_prepare_rejects_forward_parent():
    with pytest.raises(ValueError):
        S.prepare_spec_tree(np.array([[-1, 2, 0]]), np.array([5]))


# --------------------------------------------------------------------------- acceptance
def test_accept_chain_counts_leading_agreements():
    """Sequence verify: the accepted length is the number of leading drafted tokens the target reproduces."""
    N = 6
    tok = np.array([[11, 12, 13, 14, 15, 16]])
    parent = W.chain_tree(N)[None]
    # target: after ctx -> 11, after 11 -> 12, after 12 -> 13, after 13 -> 99 (disagrees with 14), ...
    tgt = np.array([[12, 13, 99, 15, 16, 17]])
    acc, na, bonus, last = S.accept_greedy(tok, parent, np.array([11]), tgt, N)
    assert na[0] == 3 and acc[0, :3].tolist() == [0, 1, 2] and (acc[0, 3:] == -1).all()
    assert bonus[0] == 99 and last[0] == 2
    # nothing agrees: no draft accepted, the bonus token is the target's own next token
    acc, na, bonus, last = S.accept_greedy(tok, parent, np.array([5]), tgt, N)
    assert na[0] == 0 and bonus[0] == 5 and last[0] == -1
    # everything agrees
    tgt_all = np.array([[12, 13, 14, 15, 16, 42]])
    acc, na, bonus, last = S.accept_greedy(tok, parent, np.array([11]), tgt_all, N)
    assert na[0] == 6 and bonus[0] == 42 and last[0] == 5


def test_accept_tree_hand_case():
    #        0(a)            tokens: a=1 b=2 c=3 d=4 e=5 f=6
    #       /    \
    #     1(b)   2(c)
    #     /      /  \
    #   3(d)   4(e) 5(f)
    parent = np.array([[-1, 0, 0, 1, 2, 2]])
    tok = np.array([[1, 2, 3, 4, 5, 6]])
    # target: ctx->1 ; after a -> 3 (so c, not b) ; after c -> 6 (f) ; after f -> 9 ; after b -> 4 (d would agree, but b did not)
    tgt = np.array([[3, 4, 6, 0, 0, 9]])
    acc, na, bonus, last = S.accept_greedy(tok, parent, np.array([1]), tgt, 6)
    assert acc[0, :3].tolist() == [0, 2, 5] and na[0] == 3 and bonus[0] == 9 and last[0] == 5
    # with the extra tokens of Prepare behind the tree: they are never candidates
    p2, *_ = S.prepare_spec_tree(parent, np.array([10]))
    tok2 = np.concatenate([tok, np.full((1, 6), 6)], axis=1)           # extra tokens carry a token id that would "agree"
    tgt2 = np.concatenate([tgt, np.full((1, 6), 7)], axis=1)
    acc, na, bonus, last = S.accept_greedy(tok2, p2, np.array([1]), tgt2, 6)
    assert acc[0, :3].tolist() == [0, 2, 5] and na[0] == 3 and last[0] == 5


def test_accept_tie_takes_smallest_end_node():
    parent = np.array([[-1, 0, 0]])
    tok = np.array([[1, 7, 7]])                                        # duplicate siblings
    tgt = np.array([[7, 3, 4]])
    acc, na, bonus, last = S.accept_greedy(tok, parent, np.array([1]), tgt, 3)
    assert acc[0, :2].tolist() == [0, 1] and bonus[0] == 3


@pytest.mark.parametrize("seed", [4, 5, 6, 7])
def test_accept_properties_random(seed):
    rng = np.random.Generator(np.random.Philox(key=seed))
    B, N = 5, 24
    parent = np.stack([W.random_tree(N, 6, rng) for _ in range(B)])
    tok = rng.integers(0, 4, size=(B, N))
    tgt = rng.integers(0, 4, size=(B, N))
    root = rng.integers(0, 4, size=B)
    acc, na, bonus, last = S.accept_greedy(tok, parent, root, tgt, N)
    depth = np.stack([node_depths(p) for p in parent])
    for b in range(B):
        agrees = np.zeros(N, bool)                                     # forward sweep, independent of the enumeration
        for i in range(N):
            p = parent[b, i]
            agrees[i] = tok[b, i] == (root[b] if p < 0 else tgt[b, p]) and (p < 0 or agrees[p])
        best = depth[b][agrees].max() if agrees.any() else 0
        assert na[b] == best
        path = acc[b, :na[b]]
        for x, y in zip(path[:-1], path[1:]):
            assert parent[b, y] == x
        if na[b]:
            assert parent[b, path[0]] == -1 and agrees[path].all()
            assert last[b] == min(i for i in range(N) if agrees[i] and depth[b, i] == best)
            assert bonus[b] == tgt[b, last[b]]


# --------------------------------------------------------------------------- KV commit
def _small_case():
    rng = np.random.Generator(np.random.Philox(key=9))
    trees = [W.random_tree(12, 5, rng), W.random_tree(12, 5, rng)]
    return W.make_case("commit", 21, dtype=W.DT_BF16, Hq=4, Hkv=2, D=64, ctx_lens=[37, 50], trees=trees)


def test_commit_moves_exactly_the_accepted_rows():
    case = _small_case()
    acc = np.full((2, case.N), -1, dtype=np.int32)
    acc[0, :3] = [0, 4, 9]
    acc[1, :1] = [2]
    na = np.array([3, 1], dtype=np.int32)
    for which in ("k", "v"):
        pool = case.k_pool if which == "k" else case.v_pool
        new_pool, new_ctx = S.commit_kv(pool, case.page_table, case.ctx_lens, acc, na, case.stride_page,
                                        case.stride_head, case.stride_token, case.Hkv, case.D)
        assert new_ctx.tolist() == [40, 51]
        after = dataclasses.replace(case, **{which + "_pool": new_pool})
        for b in range(2):
            L = int(case.ctx_lens[b])
            before_rows = oracle.gather_kv(case, which, b, 0, L + case.N)     # pinned gather, logical order
            after_rows = oracle.gather_kv(after, which, b, 0, L + case.N)
            assert np.array_equal(after_rows[:L], before_rows[:L])            # the context is untouched
            for i in range(na[b]):
                assert np.array_equal(after_rows[L + i], before_rows[L + acc[b, i]])
            untouched = [t for t in range(L + na[b], L + case.N)]
            assert np.array_equal(after_rows[untouched], before_rows[untouched])
        changed = np.flatnonzero(new_pool.reshape(-1) != np.asarray(pool).reshape(-1)).size
        assert changed <= int(na.sum()) * case.Hkv * case.D                  # nothing else in the pool moved


def test_commit_of_a_leading_chain_is_the_identity():
    case = _small_case()
    acc = np.tile(np.arange(case.N, dtype=np.int32), (2, 1))
    na = np.array([5, 12], dtype=np.int32)
    new_pool, new_ctx = S.commit_kv(case.k_pool, case.page_table, case.ctx_lens, acc, na, case.stride_page,
                                    case.stride_head, case.stride_token, case.Hkv, case.D)
    assert np.array_equal(new_pool, case.k_pool) and new_ctx.tolist() == [42, 62]


def test_commit_reads_before_it_writes():
    """Accepted path (1, 2): row 2 must land in slot 1 with its OLD content even though slot 1 ... and row 1 moves to slot 0."""
    case = _small_case()
    acc = np.full((2, case.N), -1, dtype=np.int32)
    acc[0, :2] = [1, 2]
    na = np.array([2, 0], dtype=np.int32)
    new_pool, _ = S.commit_kv(case.v_pool, case.page_table, case.ctx_lens, acc, na, case.stride_page,
                              case.stride_head, case.stride_token, case.Hkv, case.D)
    after = dataclasses.replace(case, v_pool=new_pool)
    L = int(case.ctx_lens[0])
    b4 = oracle.gather_kv(case, "v", 0, L, 3)
    af = oracle.gather_kv(after, "v", 0, L, 3)
    assert np.array_equal(af[0], b4[1]) and np.array_equal(af[1], b4[2]) and np.array_equal(af[2], b4[2])
