"""CPU oracle of the integer / data-movement steps around the verify attention.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``): plain Python loops and
numpy, written from the paper's description of the decode step, sharing
nothing with the HIP path.

* ``prepare_spec_tree``  -- Sec. 3.2.2 "Decode Stage" / Algorithm 1 ``Prepare``:
  one extra token per tree node, placed after that node's root path; the mask
  and the position ids are what place it there.
* ``accept_greedy``      -- Sec. 1 / Sec. 2: the target model verifies the drafted
  tokens in one pass and keeps the longest drafted path that agrees with its own
  (greedy) choices, which leaves its output unchanged.
* ``commit_kv``          -- Algorithm 1, ``l <- l;d`` and ``N <- N + |d|``: the
  accepted tokens become part of the context, so their K/V rows move from their
  tree slots to the next context positions.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

PAGE = 16


def _root_path(parent: Sequence[int], i: int) -> List[int]:
    """Nodes from the root down to i, by walking the parent links."""
    path = []
    while i >= 0:
        path.append(i)
        i = int(parent[i])
    return path[::-1]


def prepare_spec_tree(parent: np.ndarray, ctx_lens: np.ndarray):
    """parent: (B, n) drafter tree (parent[i] in {-1} u [0, i)).  Returns for the
    2n-token verify input (tree nodes first, then the extra token of node k at
    index n + k):
      parent2 (B, 2n) int32, anc (B, 2n) uint64 (bit j = token j visible),
      depth (B, 2n) int32 (root = 1), pos (B, 2n) int32 (position id).
    The extra token of node k follows the path root..k, so it sees exactly that
    path and itself, and sits one position behind node k; a token's position id
    is the context length plus the number of tokens in front of it on its path.
    """
    parent = np.asarray(parent, dtype=np.int64)
    B, n = parent.shape
    parent2 = np.empty((B, 2 * n), dtype=np.int32)
    anc = np.zeros((B, 2 * n), dtype=np.uint64)
    depth = np.zeros((B, 2 * n), dtype=np.int32)
    pos = np.zeros((B, 2 * n), dtype=np.int32)
    for b in range(B):
        for i in range(n):
            if not (-1 <= parent[b, i] < i):
                raise ValueError("parents must precede their children")
        for i in range(n):
            path = _root_path(parent[b], i)
            parent2[b, i] = parent[b, i]
            anc[b, i] = np.uint64(sum(1 << j for j in path))
            depth[b, i] = len(path)
            pos[b, i] = int(ctx_lens[b]) + len(path) - 1
            # the extra token after that path
            k = n + i
            parent2[b, k] = i
            anc[b, k] = np.uint64(sum(1 << j for j in path) | (1 << k))
            depth[b, k] = len(path) + 1
            pos[b, k] = int(ctx_lens[b]) + len(path)
    return parent2, anc, depth, pos


def accept_greedy(tokens: np.ndarray, parent: np.ndarray, target_root: np.ndarray, target_next: np.ndarray,
                  n_cand: int):
    """tokens (B, N): drafted token of each node; parent (B, N); target_root (B,):
    the target model's own next token after the context; target_next (B, N): its
    own next token after node i given i's root path (row i of the verify pass).
    Only the first n_cand nodes carry drafted tokens (the rest are the extra
    tokens of ``prepare_spec_tree``).

    A node agrees if its token is what the target chose at its parent (at the
    context end for a root); a path is accepted if all its nodes agree.  Returns
      accepted (B, N) int32: the nodes of the longest accepted path from the root
                             down, padded with -1 (ties: the path ending in the
                             smallest node index),
      n_accept (B,) int32, bonus (B,) int32: the target's next token after the
      accepted path, last (B,) int32: last accepted node or -1.
    Written as an enumeration of all root paths, not as a sweep.
    """
    tokens = np.asarray(tokens)
    parent = np.asarray(parent)
    B, N = tokens.shape
    accepted = np.full((B, N), -1, dtype=np.int32)
    n_accept = np.zeros(B, dtype=np.int32)
    bonus = np.zeros(B, dtype=np.int32)
    last = np.full(B, -1, dtype=np.int32)
    for b in range(B):
        best: List[int] = []
        for i in range(n_cand):
            path = _root_path(parent[b], i)
            if any(j >= n_cand for j in path):
                continue
            ok = True
            for j in path:
                pj = int(parent[b, j])
                want = int(target_root[b]) if pj < 0 else int(target_next[b, pj])
                if int(tokens[b, j]) != want:
                    ok = False
                    break
            if ok and len(path) > len(best):          # strict: the smallest end node wins ties
                best = path
        n_accept[b] = len(best)
        accepted[b, :len(best)] = best
        if best:
            last[b] = best[-1]
            bonus[b] = int(target_next[b, best[-1]])
        else:
            bonus[b] = int(target_root[b])
    return accepted, n_accept, bonus, last


def commit_kv(pool: np.ndarray, page_table, ctx_lens: np.ndarray, accepted: np.ndarray, n_accept: np.ndarray,
              stride_page: int, stride_head: int, stride_token: int, n_heads: int, head_dim: int):
    """Moves, for every sequence b and KV head, the rows of the accepted nodes
    from logical positions L_b + accepted[b, i] to L_b + i (i < n_accept[b]) in a
    copy of the flat element pool, and returns (new_pool, new_ctx_lens).  Logical
    position t of sequence b lives in page page_table[b, t // 16] (identity when
    page_table is None and B == 1), slot t % 16.
    All source rows are read before any row is written.
    """
    flat = np.array(pool, copy=True).reshape(-1)
    src = np.asarray(pool).reshape(-1)
    B = len(ctx_lens)

    def row(b: int, t: int, g: int) -> slice:
        pg = t // PAGE if page_table is None else int(page_table[b, t // PAGE])
        off = pg * stride_page + g * stride_head + (t % PAGE) * stride_token
        return slice(off, off + head_dim)

    for b in range(B):
        L = int(ctx_lens[b])
        for g in range(n_heads):
            for i in range(int(n_accept[b])):
                flat[row(b, L + i, g)] = src[row(b, L + int(accepted[b, i]), g)]
    new_ctx = (np.asarray(ctx_lens, dtype=np.int64) + np.asarray(n_accept, dtype=np.int64)).astype(np.int32)
    return flat.reshape(np.asarray(pool).shape), new_ctx
