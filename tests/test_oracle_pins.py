"""Pins of the CPU oracle against things other than itself (CPU only).

Each test names the mistake it would catch.  The dense brute force below is
written independently of oracle/owl_oracle.c: it materialises logical K/V by
its own page walk, builds the visibility matrix by transitive closure of the
parent relation instead of walking root paths, and uses a two-pass softmax
over a dense masked score matrix.
"""
import os

import numpy as np
import pytest
import torch

from paper_2510_07535_amd import workloads as W
from tree_helpers import node_depths, spec_tree

HERE = os.path.dirname(os.path.abspath(__file__))


# ---------------------------------------------------------------------------
# independent brute force
# ---------------------------------------------------------------------------
def logical_kv(case, b):
    """[T, Hkv, D] float64 K and V of sequence b in logical order."""
    T = int(case.ctx_lens[b]) + case.N
    K = np.zeros((T, case.Hkv, case.D))
    V = np.zeros((T, case.Hkv, case.D))
    kf = W.widen(case.k_pool, case.dtype).reshape(-1)
    vf = W.widen(case.v_pool, case.dtype).reshape(-1)
    for pos in range(T):
        lp, slot = divmod(pos, 16)
        page = lp if case.page_table is None else int(case.page_table[b, lp])
        for g in range(case.Hkv):
            o = page * case.stride_page + g * case.stride_head + slot * case.stride_token
            K[pos, g] = kf[o:o + case.D]
            V[pos, g] = vf[o:o + case.D]
    return K, V


def closure_mask(parent):
    """visible[i, j] by reflexive-transitive closure of 'j is the parent of i'."""
    n = len(parent)
    A = np.eye(n, dtype=bool)
    for i, p in enumerate(parent):
        if p >= 0:
            A[i, p] = True
    while True:
        A2 = (A.astype(np.int64) @ A.astype(np.int64)) > 0
        if (A2 == A).all():
            return A
        A = A2


def brute_force(case):
    out = np.zeros((case.B, case.N, case.Hq, case.D))
    q = W.widen(case.q, case.dtype)
    G = case.Hq // case.Hkv
    for b in range(case.B):
        L = int(case.ctx_lens[b])
        K, V = logical_kv(case, b)
        vis = np.concatenate([np.ones((case.N, L), bool), closure_mask(case.tree_parent[b])], axis=1)
        for h in range(case.Hq):
            S = case.scale * (q[b, :, h, :] @ K[:, h // G, :].T)     # [N, T]
            S = np.where(vis, S, -np.inf)
            P = np.exp(S - S.max(axis=1, keepdims=True))
            P /= P.sum(axis=1, keepdims=True)
            out[b, :, h, :] = P @ V[:, h // G, :]
    return out


def small_cases():
    rng = np.random.Generator(np.random.Philox(key=99))
    cs = []
    cs.append(W.make_case("bf_a", 11, dtype=W.DT_BF16, Hq=4, Hkv=2, D=16, ctx_lens=[37],
                          trees=[W.random_tree(8, 4, rng)]))
    cs.append(W.make_case("bf_b", 12, dtype=W.DT_F32, Hq=6, Hkv=2, D=8, ctx_lens=[0, 5, 64],
                          trees=[W.random_tree(7, None, rng) for _ in range(3)], spare_pages=3))
    cs.append(W.make_case("bf_c", 13, dtype=W.DT_F16, Hq=3, Hkv=3, D=32, ctx_lens=[16, 31],
                          trees=[W.chain_tree(5), W.chain_tree(5)], head_major=False))
    cs.append(W.make_case("bf_d", 14, dtype=W.DT_BF16, Hq=8, Hkv=1, D=64, ctx_lens=[50],
                          trees=[np.array([-1, -1, 0, 1, 1, -1], np.int32)], paged=False))
    cs.append(W.make_case("bf_e", 15, dtype=W.DT_F32, Hq=2, Hkv=1, D=4, ctx_lens=[1],
                          trees=[spec_tree([-1, 0, 0])], scale=0.37))
    return cs


@pytest.mark.parametrize("case", small_cases(), ids=lambda c: c.name)
def test_brute_force_tiny(oracle_mod, case):
    """Catches: wrong GQA head mapping, wrong page/slot/stride arithmetic,
    transposed operands, dropped scale, mask off by one, forest handling."""
    got = oracle_mod.verify_attn_case(case)
    want = brute_force(case)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


# ---------------------------------------------------------------------------
# special cases that reduce to a library routine
# ---------------------------------------------------------------------------
def _sdpa(case, b, mask):
    q = torch.from_numpy(W.widen(case.q, case.dtype))[b].permute(1, 0, 2)       # [Hq, N, D]
    K, V = logical_kv(case, b)
    G = case.Hq // case.Hkv
    k = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(G, dim=0)        # [Hq, T, D]
    v = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(G, dim=0)
    o = torch.nn.functional.scaled_dot_product_attention(
        q[None], k[None], v[None], attn_mask=mask, scale=case.scale)
    return o[0].permute(1, 0, 2).numpy()                                          # [N, Hq, D]


def test_single_draft_is_decode_attention(oracle_mod):
    """n_draft = 1 is ordinary decode attention over L+1 keys, no mask."""
    case = W.make_case("dec", 21, dtype=W.DT_BF16, Hq=8, Hkv=2, D=64, ctx_lens=[333, 48],
                       trees=[W.chain_tree(1)] * 2)
    got = oracle_mod.verify_attn_case(case)
    for b in range(case.B):
        np.testing.assert_allclose(got[b], _sdpa(case, b, None), rtol=0, atol=1e-12)


def test_chain_is_causal_attention(oracle_mod):
    """A chain-shaped tree is causal attention of the last N positions
    (self included -- would fail with a strict-ancestor rule)."""
    N = 6
    case = W.make_case("chain", 22, dtype=W.DT_F32, Hq=4, Hkv=4, D=32, ctx_lens=[100, 7],
                       trees=[W.chain_tree(N)] * 2)
    got = oracle_mod.verify_attn_case(case)
    for b in range(case.B):
        L = int(case.ctx_lens[b])
        causal = torch.ones(N, L + N, dtype=torch.bool).tril(diagonal=L)
        np.testing.assert_allclose(got[b], _sdpa(case, b, causal), rtol=0, atol=1e-12)


# ---------------------------------------------------------------------------
# closed forms
# ---------------------------------------------------------------------------
def test_zero_query_gives_mean_of_visible_values(oracle_mod):
    """q = 0 makes every visible key weigh the same: the output is the plain
    mean of the visible V rows, and their number is L + depth(i)."""
    rng = np.random.Generator(np.random.Philox(key=5))
    tree = W.random_tree(9, 4, rng)
    case = W.make_case("q0", 31, dtype=W.DT_F32, Hq=4, Hkv=2, D=8, ctx_lens=[23], trees=[tree])
    case.q[...] = 0
    got = oracle_mod.verify_attn_case(case)
    _, V = logical_kv(case, 0)
    for i in range(case.N):
        path, j = [], i
        while j != -1:
            path.append(j)
            j = int(tree[j])
        assert len(path) == node_depths(tree)[i]
        idx = list(range(23)) + [23 + j for j in path]
        for h in range(case.Hq):
            np.testing.assert_allclose(got[0, i, h], V[idx, h // 2].mean(axis=0), atol=1e-13)


def test_constant_value_rows(oracle_mod):
    """If every V row equals c the output is c whatever the weights are."""
    case = W.make_case("vc", 32, dtype=W.DT_F32, Hq=2, Hkv=1, D=8, ctx_lens=[40],
                       trees=[W.chain_tree(3)], paged=False)
    c = np.arange(8, dtype=np.float32) - 3.5
    case.v_pool[...] = c
    got = oracle_mod.verify_attn_case(case)
    np.testing.assert_allclose(got, np.broadcast_to(c, got.shape), atol=1e-13)


def test_dominant_key_selects_its_value(oracle_mod):
    """One key with a score far above the rest: output -> that key's V row
    (would fail if K and V rows were paired wrongly)."""
    case = W.make_case("dom", 33, dtype=W.DT_F32, Hq=1, Hkv=1, D=4, ctx_lens=[30],
                       trees=[W.chain_tree(2)], paged=True, scale=1.0)
    case.q[...] = 0
    case.q[0, :, 0, 0] = 1.0
    K, V = logical_kv(case, 0)
    # make logical position 17 the dominant key
    lp, slot = divmod(17, 16)
    page = int(case.page_table[0, lp])
    case.k_pool[page, 0, slot, :] = np.array([200.0, 0, 0, 0], np.float32)
    got = oracle_mod.verify_attn_case(case)
    np.testing.assert_allclose(got[0, :, 0], np.broadcast_to(V[17, 0], (2, 4)), atol=1e-12)


# ---------------------------------------------------------------------------
# invariants
# ---------------------------------------------------------------------------
def _tree_case(seed=41, **kw):
    tree = np.array([-1, 0, 0, 1, 1, 2, 5, 3], np.int32)
    args = dict(dtype=W.DT_BF16, Hq=4, Hkv=2, D=16, ctx_lens=[45], trees=[tree])
    args.update(kw)
    return W.make_case("inv", seed, **args)


def _draft_slot(case, b, j):
    pos = int(case.ctx_lens[b]) + j
    return int(case.page_table[b, pos // 16]), pos % 16


def test_non_ancestor_perturbation_leaves_row_unchanged(oracle_mod):
    """Changing K/V of a draft that is not on node i's root path must not move
    row i at all; changing one that is on the path must."""
    case = _tree_case()
    base = oracle_mod.verify_attn_case(case)
    tree = case.tree_parent[0]
    anc = closure_mask(tree)
    for j in range(case.N):
        c2 = _tree_case()
        page, slot = _draft_slot(c2, 0, j)
        c2.k_pool[page, :, slot, :] = W.store(np.full((2, 16), 3.0, np.float32), W.DT_BF16)
        c2.v_pool[page, :, slot, :] = W.store(np.full((2, 16), -7.0, np.float32), W.DT_BF16)
        got = oracle_mod.verify_attn_case(c2)
        for i in range(case.N):
            if anc[i, j]:
                assert np.abs(got[0, i] - base[0, i]).max() > 1e-6, (i, j)
            else:
                assert np.array_equal(got[0, i], base[0, i]), (i, j)


def test_page_permutation_changes_nothing(oracle_mod):
    """Same logical cache under another physical page order: identical bits."""
    a = _tree_case(paged=True)
    b = _tree_case(paged=False)
    assert not np.array_equal(a.page_table, b.page_table)
    assert np.array_equal(oracle_mod.verify_attn_case(a), oracle_mod.verify_attn_case(b))
    c = _tree_case(paged=True, head_major=False)
    assert np.array_equal(oracle_mod.verify_attn_case(a), oracle_mod.verify_attn_case(c))


def test_gqa_equals_expanded_mha(oracle_mod):
    """Repeating each KV head G times and running with Hkv = Hq is the same."""
    a = _tree_case()
    out_a = oracle_mod.verify_attn_case(a)
    G = a.G
    kw = oracle_mod.case_kwargs(a)
    kw["k_cache"] = np.repeat(a.k_pool, G, axis=1)
    kw["v_cache"] = np.repeat(a.v_pool, G, axis=1)
    kw["Hkv"] = a.Hq
    kw["stride_page"] = a.stride_page * G
    out_b = oracle_mod.verify_attn(**kw)
    assert np.array_equal(out_a, out_b)


def test_relabelling_nodes_permutes_rows(oracle_mod):
    """Any other topological numbering of the same tree gives the same rows."""
    a = _tree_case()
    # new order: swap the two subtrees' numbering; old index of new node k
    order = np.array([0, 2, 1, 5, 6, 3, 4, 7])
    assert sorted(order) == list(range(8))
    inv = np.argsort(order)
    old_parent = a.tree_parent[0]
    new_parent = np.array([-1 if old_parent[o] < 0 else inv[old_parent[o]] for o in order], np.int32)
    assert all(new_parent[i] < i for i in range(8))
    b = _tree_case()
    b.tree_parent[0] = new_parent
    b.q[0] = a.q[0][order]
    L = int(a.ctx_lens[0])
    for new, old in enumerate(order):
        pn, sn = _draft_slot(b, 0, new)
        po, so = _draft_slot(a, 0, int(old))
        b.k_pool[pn, :, sn] = a.k_pool[po, :, so]
        b.v_pool[pn, :, sn] = a.v_pool[po, :, so]
    out_a = oracle_mod.verify_attn_case(a)
    out_b = oracle_mod.verify_attn_case(b)
    np.testing.assert_allclose(out_b[0], out_a[0][order], rtol=0, atol=1e-13)


def test_split_and_merge_is_order_invariant(oracle_mod):
    """The log-sum-exp combine of per-piece (m, l, acc) equals the one-piece
    result for any piece size, including pieces in which a row sees no key."""
    case = _tree_case(ctx_lens=[75])
    ref = oracle_mod.verify_attn_case(case)
    for chunk in (1, 7, 16, 32, 80, 1000):
        got = oracle_mod.verify_attn_case(case, chunk_tokens=chunk)
        np.testing.assert_allclose(got, ref, rtol=0, atol=1e-13)


def test_rows_subset_matches_full(oracle_mod):
    case = _tree_case()
    full = oracle_mod.verify_attn_case(case)
    rows = np.array([[0, 7, 3], [0, 0, 0], [0, 4, 2]], np.int32)
    sub = oracle_mod.verify_attn_case(case, rows=rows)
    for r, (b, i, h) in enumerate(rows):
        assert np.array_equal(sub[r], full[b, i, h])


# ---------------------------------------------------------------------------
# mask builder and paging on their own
# ---------------------------------------------------------------------------
def _golden():
    lines = [l for l in open(os.path.join(HERE, "golden", "spec_tree_example.txt")).read().splitlines()
             if l and not l.startswith("#")]
    parent = np.array([int(x) for x in lines[0].split()], np.int32)
    masks = np.array([int(x, 2) for x in lines[1].split()], np.uint64)
    depth = np.array([int(x) for x in lines[2].split()], np.int32)
    return parent, masks, depth


def test_tree_mask_matches_paper_example(oracle_mod):
    parent, masks, depth = _golden()
    assert np.array_equal(parent, spec_tree([-1, 0, 0]))
    anc, dep = oracle_mod.tree_mask(parent)
    assert np.array_equal(anc, masks)
    assert np.array_equal(dep, depth)


def test_tree_mask_matches_closure(oracle_mod):
    rng = np.random.Generator(np.random.Philox(key=6))
    for n, md in ((1, None), (2, None), (17, 3), (60, 6), (64, None), (64, 2)):
        parent = W.random_tree(n, md, rng)
        anc, dep = oracle_mod.tree_mask(parent)
        A = closure_mask(parent)
        want = np.array([sum(1 << j for j in range(n) if A[i, j]) for i in range(n)], np.uint64)
        assert np.array_equal(anc, want)
        assert np.array_equal(dep, A.sum(axis=1))
    anc, dep = oracle_mod.tree_mask(W.chain_tree(64))
    assert anc[63] == np.uint64(0xFFFFFFFFFFFFFFFF) and dep[63] == 64


def test_bad_trees_are_rejected(oracle_mod):
    for bad in ([0], [-1, 1], [-1, 2, 0], [-2], [-1, 0, 3]):
        with pytest.raises(oracle_mod.OracleError) as e:
            oracle_mod.tree_mask(np.array(bad, np.int32))
        assert e.value.code == -2
    with pytest.raises(oracle_mod.OracleError) as e:
        oracle_mod.tree_mask(W.chain_tree(65))
    assert e.value.code == -3
    case = _tree_case()
    case.tree_parent[0, 3] = 5
    with pytest.raises(oracle_mod.OracleError):
        oracle_mod.verify_attn_case(case)


def test_gather_follows_page_table(oracle_mod):
    case = W.make_case("g", 51, dtype=W.DT_BF16, Hq=2, Hkv=2, D=8, ctx_lens=[40, 9],
                       trees=[W.chain_tree(3)] * 2, spare_pages=2)
    for b in range(2):
        T = int(case.ctx_lens[b]) + 3
        got = oracle_mod.gather_kv(case, "k", b, 0, T)
        for pos in range(T):
            page = int(case.page_table[b, pos // 16])
            assert np.array_equal(got[pos], case.k_pool[page, :, pos % 16, :])
        part = oracle_mod.gather_kv(case, "v", b, 5, 4)
        full = oracle_mod.gather_kv(case, "v", b, 0, T)
        assert np.array_equal(part, full[5:9])


# ---------------------------------------------------------------------------
# the generators themselves (recipe checks, no arithmetic of the method)
# ---------------------------------------------------------------------------
def test_generators_follow_the_recipe():
    rng = np.random.Generator(np.random.Philox(key=7))
    t = W.random_tree(60, 6, rng)
    assert t[0] == -1 and all(0 <= t[i] < i for i in range(1, 60))
    assert node_depths(t).max() <= 6
    h = W.hybrid_tree(32, 8, rng)
    d = node_depths(h)
    assert len(h) == 40 and all(h[k] == k - 1 for k in range(33, 40))
    assert d[h[32]] == d[:32].max() and h[32] == int(np.argmax(d[:32]))
    assert np.array_equal(W.chain_tree(4), [-1, 0, 1, 2])
    x = np.array([1.0, 1.00390625, 1.01171875, -3.1415926, 1e-40], np.float32)
    bits = W.f32_to_bf16_bits(x)
    back = W.bf16_bits_to_f32(bits)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(back, ref)
    c = W.make_config(4, ctx_scale=1 / 256)
    assert c.B == 16 and c.N == 26 and c.Hq == 32 and c.Hkv == 8
    pages = c.page_table[c.page_table >= 0]
    assert len(np.unique(pages)) == len(pages)          # no page shared
    full = W.config_ctx_lens(4)
    assert full.min() >= 8192 and full.max() <= 65536 and len(full) == 16


# --------------------------------------------------------------------------- ragged draft counts
def _ragged_case():
    r = np.random.Generator(np.random.Philox(key=77))
    trees = [W.random_tree(12, 5, r) for _ in range(3)]
    return W.make_case("ragged", 55, dtype=W.DT_BF16, Hq=4, Hkv=2, D=32, ctx_lens=[40, 7, 19], trees=trees)


def test_ragged_with_full_counts_is_the_plain_step(oracle_mod):
    oracle = oracle_mod
    case = _ragged_case()
    full = oracle.verify_attn_case(case)
    assert np.array_equal(oracle.verify_attn_ragged_case(case, [case.N] * case.B), full)


def test_ragged_rows_and_cache_rows_of_absent_nodes_do_not_matter(oracle_mod):
    import dataclasses
    oracle = oracle_mod
    case = _ragged_case()
    nd = [5, 0, 12]
    out = oracle.verify_attn_ragged_case(case, nd)
    assert (out[0, 5:] == 0).all() and (out[1] == 0).all()
    assert np.isfinite(out).all() and np.abs(out[0, :5]).max() > 0
    # a node's output depends on its ancestors only, and those precede it: the present rows
    # equal the rows of the full step (pinned above by the non-ancestor invariance)
    full = oracle.verify_attn_case(case)
    assert np.array_equal(out[0, :5], full[0, :5]) and np.array_equal(out[2], full[2])
    # scrambling q, the parents and the cached K/V rows of the absent nodes changes nothing
    q2 = case.q.copy(); q2[0, 5:] = q2[0, 5:][::-1]; q2[1] = 0
    par2 = case.tree_parent.copy(); par2[0, 5:] = 0; par2[1] = -1
    k2 = case.k_pool.copy().reshape(-1); v2 = case.v_pool.copy().reshape(-1)
    for b, n in enumerate(nd):
        for j in range(n, case.N):
            t = int(case.ctx_lens[b]) + j
            pg = int(case.page_table[b, t // 16])
            for g in range(case.Hkv):
                off = pg * case.stride_page + g * case.stride_head + (t % 16) * case.stride_token
                k2[off:off + case.D] = k2[off:off + case.D][::-1]
                v2[off:off + case.D] = 0
    other = dataclasses.replace(case, q=q2, tree_parent=par2, k_pool=k2.reshape(case.k_pool.shape),
                                v_pool=v2.reshape(case.v_pool.shape))
    assert np.array_equal(oracle.verify_attn_ragged_case(other, nd), out)
