// Device-side helpers used by more than one kernel.
#pragma once

#include "owl_internal.h"

namespace owl {

__device__ __forceinline__ void flag_status(uint32_t *st, uint32_t bit)
{
    if (st) atomicOr(st, bit);
}

// Prefix length of sequence b, forced into [0, max_ctx_len].
__device__ __forceinline__ int load_ctx_len(const int32_t *ctx_lens, int b, int max_ctx_len,
                                            uint32_t *st)
{
    int L = ctx_lens[b];
    if (L < 0 || L > max_ctx_len) {
        flag_status(st, OWL_DEV_BAD_CTX_LEN);
        L = L < 0 ? 0 : max_ctx_len;
    }
    return L;
}

// Number of drafted tokens of sequence b: N unless a per-sequence array is given,
// whose entries are forced into [0, N].
__device__ __forceinline__ int load_n_draft(const int32_t *n_draft_seq, int b, int N, uint32_t *st)
{
    if (!n_draft_seq) return N;
    int n = n_draft_seq[b];
    if (n < 0 || n > N) {
        flag_status(st, OWL_DEV_BAD_NDRAFT);
        n = n < 0 ? 0 : N;
    }
    return n;
}

// Tokens per split for a sequence of T cached rows.  The host plans for the
// longest context it was told about; a lone, shorter sequence is cut into the
// same number of (shorter) splits instead of leaving most of the chip idle.
// Never above p.C, never below the planner's minimum, a multiple of the stage.
__device__ __forceinline__ int split_tokens_for(const KParams &p, int T)
{
    if (!p.adapt) return p.C;
    int C = (T + p.max_splits - 1) / p.max_splits;
    C = (C + kSplitQuantum - 1) / kSplitQuantum * kSplitQuantum;
    C = max(C, p.c_min);
    return min(C, p.C);
}

// Physical page of logical page lp of sequence b; an id outside the pool (or a
// logical page beyond the table) is replaced by page 0 and flagged.
__device__ __forceinline__ int load_page(const int32_t *page_table, int b, int max_pages,
                                         int64_t n_pool_pages, int lp, uint32_t *st)
{
    int pg;
    if (page_table) {
        if (lp >= max_pages) {
            flag_status(st, OWL_DEV_BAD_PAGE);
            return 0;
        }
        pg = page_table[(int64_t)b * max_pages + lp];
    } else {
        pg = lp;
    }
    if (pg < 0 || pg >= n_pool_pages) {
        flag_status(st, OWL_DEV_BAD_PAGE);
        pg = 0;
    }
    return pg;
}

// Ancestor-or-self set of node i (Sec. 3.2.2: a token placed after a tree path
// sees that path).  `parent` is a copy of the sequence's parent array in LDS or
// registers-backed memory; a parent that is not in {-1} u [0, j) ends the walk
// as if it were a root and is flagged.  The walk visits strictly decreasing
// indices, so it ends after at most i + 1 steps.
__device__ __forceinline__ uint64_t ancestor_set(const int32_t *parent, int i, int *depth_out,
                                                 uint32_t *st)
{
    uint64_t set = 0;
    int depth = 0;
    int jn = i;
    while (jn >= 0) {
        set |= (uint64_t)1 << jn;
        ++depth;
        int pj = parent[jn];
        if (pj < -1 || pj >= jn) {
            flag_status(st, OWL_DEV_BAD_PARENT);
            pj = -1;
        }
        jn = pj;
    }
    if (depth_out) *depth_out = depth;
    return set;
}

}  // namespace owl
