"""Seeded synthetic inputs for the verify-step attention path.

This module only *draws data*: random q/k/v values, draft trees, context
lengths and page permutations.  It contains none of the method's arithmetic
(no scores, no softmax, no masks) and imports neither the HIP binding nor the
CPU oracle, so both sides can be fed the very same buffers.

The paper measures on LongSpecBench (Sec. 3.1: 200 real conversations with
4K-64K-token inputs) with Llama-3.1-8B / Llama-3.3-70B targets and a 60-node
draft tree (Appendix A.1).  None of that data is reproduced here; the cases
below only take its *shapes*: the context-length range (extended to the 128K
limit named in Sec. 1), the public head shapes of the two target models, and
the tree sizes.  Values are N(0,1).

Conventions shared by every consumer of a ``Case``:
  * q          [B, N, Hq, D]      draft-token queries (already position-encoded)
  * k_pool     [pages, Hkv, 16, D] paged key cache, v_pool alike
  * page_table [B, max_pages]     physical page of logical page p; -1 = unused
  * ctx_lens   [B]                prefix length L_b, *excluding* the N drafts
  * tree_parent[B, N]             -1 = root, else index of an earlier node
  * draft node j of sequence b has its K/V row at logical position L_b + j
bf16 tensors are carried as uint16 bit patterns (numpy has no bf16).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional, Sequence

import numpy as np

PAGE = 16

DT_BF16 = 0
DT_F32 = 1
DT_F16 = 2


# ----------------------------------------------------------------------------
# storage helpers (format conversion only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16, returned as uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def store(x_f32: np.ndarray, dtype: int) -> np.ndarray:
    if dtype == DT_BF16:
        return f32_to_bf16_bits(x_f32)
    if dtype == DT_F16:
        return x_f32.astype(np.float16).view(np.uint16)
    return np.ascontiguousarray(x_f32, dtype=np.float32)


def widen(x: np.ndarray, dtype: int) -> np.ndarray:
    """Stored tensor -> float64 (exact)."""
    if dtype == DT_BF16:
        return bf16_bits_to_f32(x).astype(np.float64)
    if dtype == DT_F16:
        return x.view(np.float16).astype(np.float64)
    return x.astype(np.float64)


# ----------------------------------------------------------------------------
# draft-tree shapes
# ----------------------------------------------------------------------------
def chain_tree(n: int) -> np.ndarray:
    """Sequence (non-tree) verify: node i follows node i-1."""
    return np.arange(-1, n - 1, dtype=np.int32)


def _grow_tree(n: int, max_depth: Optional[int], rng: np.random.Generator):
    """(parent, level) of a random tree; ``level`` is the bookkeeping the draw itself
    needs (which earlier nodes may still take a child): 1 for the root, parent's + 1 below."""
    if max_depth is not None and max_depth < 2 and n > 1:
        raise ValueError("a tree of several nodes under one root needs max_depth >= 2")
    parent = np.full(n, -1, dtype=np.int32)
    depth = np.zeros(n, dtype=np.int32)
    depth[0] = 1
    for i in range(1, n):
        if max_depth is None:
            cand = np.arange(i)
        else:
            cand = np.nonzero(depth[:i] <= max_depth - 1)[0]
        p = int(cand[rng.integers(0, len(cand))])
        parent[i] = p
        depth[i] = depth[p] + 1
    return parent, depth


def random_tree(n: int, max_depth: Optional[int], rng: np.random.Generator) -> np.ndarray:
    """Node 0 is the root; every later node draws its parent uniformly from
    the earlier nodes whose depth is below ``max_depth`` (root depth = 1)."""
    return _grow_tree(n, max_depth, rng)[0]


def hybrid_tree(n_tree: int, n_chain: int, rng: np.random.Generator) -> np.ndarray:
    """A random tree with a chain hung off its deepest leaf (lowest index on
    ties); the chain nodes take the indices after the tree's."""
    t, d = _grow_tree(n_tree, None, rng)
    leaf = int(np.argmax(d))  # argmax returns the first maximal entry
    chain = np.arange(n_tree - 1, n_tree + n_chain - 1, dtype=np.int32)
    chain[0] = leaf
    return np.concatenate([t, chain]).astype(np.int32)


# ----------------------------------------------------------------------------
# the case container
# ----------------------------------------------------------------------------
@dataclasses.dataclass
class Case:
    name: str
    seed: int
    dtype: int
    B: int
    N: int
    Hq: int
    Hkv: int
    D: int
    scale: float                 # already rounded to float32
    q: np.ndarray
    k_pool: np.ndarray
    v_pool: np.ndarray
    page_table: Optional[np.ndarray]   # None => identity paging
    ctx_lens: np.ndarray
    tree_parent: np.ndarray
    max_pages_per_seq: int
    stride_page: int
    stride_head: int
    stride_token: int
    n_pool_pages: int

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def max_ctx_len(self) -> int:
        return int(self.ctx_lens.max()) if self.B else 0

    def kv_bytes(self) -> int:
        """K+V bytes of every visible-or-not cached row the step has to scan:
        sum_b (L_b + N) * Hkv * D * 2 tensors * element size."""
        esz = 4 if self.dtype == DT_F32 else 2
        return int((self.ctx_lens.astype(np.int64) + self.N).sum()) * self.Hkv * self.D * 2 * esz


def _normal(rng: np.random.Generator, shape) -> np.ndarray:
    return rng.standard_normal(size=shape, dtype=np.float32)


def make_case(
    name: str,
    seed: int,
    *,
    dtype: int,
    Hq: int,
    Hkv: int,
    D: int,
    ctx_lens: Sequence[int],
    trees: Sequence[np.ndarray],
    paged: bool = True,
    head_major: bool = True,
    outlier_frac: float = 0.0,
    outlier_gain: float = 8.0,
    spare_pages: int = 0,
    scale: Optional[float] = None,
) -> Case:
    """Build one verify step.  ``trees`` holds one parent array per sequence
    (all of the same length N).  With ``paged`` the logical pages of all
    sequences are scattered over one shared pool by a seeded permutation;
    otherwise sequence b owns a contiguous run of pages and page_table is
    None when B == 1.  ``head_major`` picks [page][Hkv][16][D] over
    [page][16][Hkv][D] (the latter is a plain [token][Hkv][D] array when the
    pages are in order)."""
    rng = np.random.Generator(np.random.Philox(key=seed))            # values
    prng = np.random.Generator(np.random.Philox(key=seed ^ 0x9A6E))  # page order only
    B = len(ctx_lens)
    N = len(trees[0])
    assert all(len(t) == N for t in trees) and len(trees) == B
    ctx = np.asarray(ctx_lens, dtype=np.int32)
    pages_per_seq = [(int(L) + N + PAGE - 1) // PAGE for L in ctx]
    max_pages = max(pages_per_seq) if B else 0
    total_pages = sum(pages_per_seq) + spare_pages

    if paged:
        perm = prng.permutation(total_pages).astype(np.int32)
    else:
        perm = np.arange(total_pages, dtype=np.int32)
    page_table = np.full((B, max(max_pages, 1)), -1, dtype=np.int32)
    o = 0
    for b in range(B):
        page_table[b, : pages_per_seq[b]] = perm[o : o + pages_per_seq[b]]
        o += pages_per_seq[b]

    sdtype = np.float32 if dtype == DT_F32 else np.uint16
    if head_major:
        pool_shape = (max(total_pages, 1), Hkv, PAGE, D)
        stride_page, stride_head, stride_token = Hkv * PAGE * D, PAGE * D, D
    else:
        pool_shape = (max(total_pages, 1), PAGE, Hkv, D)
        stride_page, stride_head, stride_token = PAGE * Hkv * D, D, Hkv * D
    # unused slots (page padding, spare pages) keep a recognisable filler so a
    # wrong gather shows up as a large error rather than as a near miss
    filler = store(np.full((1,), 977.0, np.float32), dtype)[0]
    k_pool = np.full(pool_shape, filler, dtype=sdtype)
    v_pool = np.full(pool_shape, filler, dtype=sdtype)

    q = store(_normal(rng, (B, N, Hq, D)), dtype)
    for b in range(B):
        T = int(ctx[b]) + N
        if T == 0:
            continue
        k = _normal(rng, (T, Hkv, D))
        v = _normal(rng, (T, Hkv, D))
        if outlier_frac > 0.0:
            hot = rng.random(int(ctx[b])) < outlier_frac   # prefix positions only
            k[: int(ctx[b])][hot] *= np.float32(outlier_gain)
        npg = pages_per_seq[b]
        pad = npg * PAGE - T
        for src, pool in ((k, k_pool), (v, v_pool)):
            s = store(src, dtype)
            if pad:
                s = np.concatenate([s, np.full((pad, Hkv, D), filler, dtype=sdtype)], axis=0)
            s = s.reshape(npg, PAGE, Hkv, D)
            if head_major:
                s = s.transpose(0, 2, 1, 3)
            pool[page_table[b, :npg]] = s
        del k, v

    if scale is None:
        scale = 1.0 / math.sqrt(D)
    scale = float(np.float32(scale))
    pt: Optional[np.ndarray] = page_table
    if not paged and B == 1:
        pt = None
    return Case(
        name=name, seed=seed, dtype=dtype, B=B, N=N, Hq=Hq, Hkv=Hkv, D=D, scale=scale,
        q=q, k_pool=k_pool, v_pool=v_pool, page_table=pt, ctx_lens=ctx,
        tree_parent=np.stack([np.asarray(t, np.int32) for t in trees]).astype(np.int32),
        max_pages_per_seq=page_table.shape[1],
        stride_page=stride_page, stride_head=stride_head, stride_token=stride_token,
        n_pool_pages=pool_shape[0],
    )


# ----------------------------------------------------------------------------
# the five named configurations
# ----------------------------------------------------------------------------
CONFIG_NAMES = ("tiny_chain4_f32", "8b_chain6_32k", "8b_tree60_64k", "70b_hybrid40_128k", "8b_batch16_tree26")


def config_ctx_lens(idx: int, seed: Optional[int] = None) -> np.ndarray:
    """Context lengths of configuration ``idx`` (0-based) without building it."""
    seed = idx + 1 if seed is None else seed
    if idx == 0:
        return np.array([512], np.int32)
    if idx == 1:
        return np.array([32768], np.int32)
    if idx == 2:
        return np.array([65536], np.int32)
    if idx == 3:
        return np.array([131072], np.int32)
    if idx == 4:
        r = np.random.Generator(np.random.Philox(key=seed ^ 0x5EED))
        return r.integers(8192, 65536, size=16, endpoint=True).astype(np.int32)
    raise ValueError(idx)


def make_config(idx: int, seed: Optional[int] = None, ctx_scale: float = 1.0, dtype: Optional[int] = None,
                kv_shards: int = 1) -> Case:
    """Configuration ``idx`` (0-based, in the order of the benchmark list).
    ``ctx_scale`` < 1 shrinks every context length by that factor (kept for
    CPU-sized parity runs of the same structure); 1.0 is the named size.
    ``dtype`` replaces the storage type of configurations 1..4 (bf16 as listed;
    DT_F16 is the type the paper's runs used).  ``kv_shards`` > 1 gives one GPU's
    share of the configuration when its KV heads (and their query heads) are
    spread over that many GPUs: the same lengths and trees on 1/kv_shards of the heads."""
    seed = idx + 1 if seed is None else seed
    if kv_shards > 1:
        base = make_config(idx, seed, ctx_scale, dtype)
        if idx == 0 or base.Hkv % kv_shards:
            raise ValueError("kv_shards must divide the KV heads of configurations 1..4")
        return make_case(f"{base.name}_heads1of{kv_shards}", seed, dtype=base.dtype, Hq=base.Hq // kv_shards,
                         Hkv=base.Hkv // kv_shards, D=base.D, ctx_lens=base.ctx_lens,
                         trees=list(base.tree_parent), outlier_frac=0.05 if idx == 3 else 0.0)
    if dtype is not None and idx > 0:
        base = make_config(idx, seed, ctx_scale)
        if dtype == base.dtype:
            return base
        return make_case(base.name + {DT_F16: "_f16", DT_F32: "_f32", DT_BF16: ""}[dtype], seed, dtype=dtype,
                         Hq=base.Hq, Hkv=base.Hkv, D=base.D, ctx_lens=base.ctx_lens,
                         trees=list(base.tree_parent), outlier_frac=0.05 if idx == 3 else 0.0)
    trng = np.random.Generator(np.random.Philox(key=seed ^ 0x7EE))
    ctx = np.maximum(1, (config_ctx_lens(idx, seed).astype(np.float64) * ctx_scale).astype(np.int64))
    name = CONFIG_NAMES[idx] + ("" if ctx_scale == 1.0 else f"@{ctx_scale:g}")
    if idx == 0:
        return make_case(name, seed, dtype=DT_F32, Hq=4, Hkv=1, D=64, ctx_lens=ctx,
                         trees=[chain_tree(4)], paged=False, head_major=False)
    if idx == 1:
        return make_case(name, seed, dtype=DT_BF16, Hq=32, Hkv=8, D=128, ctx_lens=ctx,
                         trees=[chain_tree(6)])
    if idx == 2:
        return make_case(name, seed, dtype=DT_BF16, Hq=32, Hkv=8, D=128, ctx_lens=ctx,
                         trees=[random_tree(60, 6, trng)])
    if idx == 3:
        return make_case(name, seed, dtype=DT_BF16, Hq=64, Hkv=8, D=128, ctx_lens=ctx,
                         trees=[hybrid_tree(32, 8, trng)], outlier_frac=0.05)
    if idx == 4:
        return make_case(name, seed, dtype=DT_BF16, Hq=32, Hkv=8, D=128, ctx_lens=ctx,
                         trees=[random_tree(26, 5, trng) for _ in range(len(ctx))])
    raise ValueError(idx)


# ----------------------------------------------------------------------------
# inputs of the drafter's recurrent cell (Sec. 3.2.1): random weights of the
# paper's width (Sec. 4.1: d = 12288), random states and tokens.  Data only.
# ----------------------------------------------------------------------------
@dataclasses.dataclass
class DrafterCase:
    name: str
    seed: int
    dtype: int                   # storage type of h, W, E (DT_BF16 or DT_F16)
    d_in: int
    d: int
    P: int                       # distinct parent states
    M: int                       # rows of the step (children)
    vocab: int
    h: np.ndarray                # [P, d_in]   dtype bits
    z: np.ndarray                # [P, d]      float32
    W: np.ndarray                # [4, d, d_in] dtype bits, gates in the order f, i, o, c
    E: np.ndarray                # [vocab, d]  dtype bits
    tokens: np.ndarray           # [M] int32
    parent_row: Optional[np.ndarray]   # [M] int32 or None (identity)
    gamma_c: np.ndarray          # [d] float32, affine pair of the normalisation of the candidate
    beta_c: np.ndarray
    gamma_z: np.ndarray          # [d] float32, affine pair of the normalisation of the cell state
    beta_z: np.ndarray
    eps: float

    def weight_bytes(self) -> int:
        return 4 * self.d * self.d_in * 2


def make_drafter_case(name: str, seed: int, *, dtype: int = DT_BF16, d_in: int, d: int, P: int, M: int,
                      vocab: int = 1000, identity: bool = False, zero_state: bool = False,
                      eps: float = 1e-5) -> DrafterCase:
    """W ~ N(0, 1/d_in) so that the projections are O(1); h, E ~ N(0, 1);
    z ~ N(0, 1) (zeros with ``zero_state``: the paper starts the cell state at
    zero); the affine pairs are 1 + 0.1 N(0,1) and 0.1 N(0,1).  ``identity``
    leaves parent_row out (row r continues state r; needs M == P)."""
    if dtype not in (DT_BF16, DT_F16):
        raise ValueError("the cell's storage type is bf16 or fp16")
    rng = np.random.Generator(np.random.Philox(key=seed ^ 0xD4AF))
    W = np.empty((4, d, d_in), dtype=np.uint16)
    for m in range(4):                                       # gate by gate: bounds the fp32 transient
        W[m] = store(_normal(rng, (d, d_in)) * np.float32(1.0 / math.sqrt(d_in)), dtype)
    h = store(_normal(rng, (P, d_in)), dtype)
    z = np.zeros((P, d), np.float32) if zero_state else _normal(rng, (P, d))
    E = store(_normal(rng, (vocab, d)), dtype)
    tokens = rng.integers(0, vocab, size=M).astype(np.int32)
    if identity:
        if M != P:
            raise ValueError("identity needs M == P")
        parent_row = None
    else:
        parent_row = rng.integers(0, P, size=M).astype(np.int32)
    aff = [(_normal(rng, (d,)) * np.float32(0.1)) for _ in range(4)]
    return DrafterCase(name=name, seed=seed, dtype=dtype, d_in=d_in, d=d, P=P, M=M, vocab=vocab, h=h, z=z, W=W,
                       E=E, tokens=tokens, parent_row=parent_row, gamma_c=aff[0] + np.float32(1.0), beta_c=aff[1],
                       gamma_z=aff[2] + np.float32(1.0), beta_z=aff[3], eps=eps)
