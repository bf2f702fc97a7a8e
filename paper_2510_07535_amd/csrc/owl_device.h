// Device-side helpers used by more than one kernel.
#pragma once

#include "owl_internal.h"

namespace owl {

__device__ __forceinline__ void flag_status(uint32_t *st, uint32_t bit)
{
    if (st) atomicOr(st, bit);
}

// Four consecutive output channels, starting at element index `e` of the output array, in the
// output type: fp32 as it is, 16-bit types rounded to nearest even from the fp32 value.
__device__ __forceinline__ void store_out4(void *out, int64_t e, float4 v, int out_dtype)
{
    typedef float o_f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 o_bf16x2 __attribute__((ext_vector_type(2)));
    typedef _Float16 o_f16x2 __attribute__((ext_vector_type(2)));
    if (out_dtype == OWL_F32) {
        *reinterpret_cast<float4 *>(static_cast<float *>(out) + e) = v;
        return;
    }
    const o_f32x2 lo = {v.x, v.y}, hi = {v.z, v.w};
    uint2 w;
    if (out_dtype == OWL_BF16) {
        w.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, o_bf16x2));
        w.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, o_bf16x2));
    } else {
        w.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, o_f16x2));
        w.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, o_f16x2));
    }
    *reinterpret_cast<uint2 *>(static_cast<uint16_t *>(out) + e) = w;
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
    if (p.adapt != 1) return p.C;
    int C = (T + p.max_splits - 1) / p.max_splits;
    C = (C + kSplitQuantum - 1) / kSplitQuantum * kSplitQuantum;
    C = max(C, p.c_min);
    return min(C, p.C);
}

// Cached rows of sequence b that the pass has to scan: 0 for a sequence without drafts.
__device__ __forceinline__ int seq_tokens(const KParams &p, int b)
{
    int L = p.ctx_lens[b];
    L = L < 0 ? 0 : (L > p.max_ctx_len ? p.max_ctx_len : L);        // flagged where the sequence is processed
    int n = p.n_draft_seq ? p.n_draft_seq[b] : p.N;
    n = n < 0 ? 0 : (n > p.N ? p.N : n);
    return n == 0 ? 0 : L + n;
}

// Sum / maximum over lanes [0, n) of a wavefront, as scalars (n uniform, <= 64).
__device__ __forceinline__ int lanes_sum(int v, int n)
{
    int s = 0;
    for (int l = 0; l < n; ++l) s += __builtin_amdgcn_readlane(v, l);
    return s;
}
__device__ __forceinline__ int lanes_max(int v, int n)
{
    int m = 0;
    for (int l = 0; l < n; ++l) m = max(m, __builtin_amdgcn_readlane(v, l));
    return m;
}

// Split size for a batch (adapt == 2).  The host plans for B sequences of the
// longest admissible length; a real batch is ragged, and with one workgroup per
// compute unit at a time a launch of, say, 1.4 rounds leaves most of the chip
// idle for its last round.  Every wavefront derives, from the actual lengths,
// about the smallest split size (a multiple of the stage, within the planner's
// bounds and the launched grid) whose workgroup count still fits the whole
// number of rounds that the planned size needs: the rounds come out full and as
// short as they can be.  All lanes of the calling wavefront, and every wavefront
// of the launch, get the same value: it depends only on p and the two length
// arrays, and the combine reads the value the split-KV pass stored.
//
// The search runs across lanes: lane l prices one candidate size against all
// sequences (their lengths travel as scalars), a ballot picks the first
// candidate that fits, a second pass refines between it and its neighbour.
// Workgroup counts of candidates are formed in float: a count that is off by
// one moves the choice by a stage, never the validity of the result.
__device__ __forceinline__ int batch_split_tokens(const KParams &p)
{
    const int lane = threadIdx.x & 63;
    const int streams = p.Hkv * p.row_groups;        // workgroups per split
    // sequence lengths: sequence b < 64 sits in lane b; further ones are re-read (uniform loads)
    const int t_lane = lane < p.B ? seq_tokens(p, lane) : 0;
    const int n_lane = min(p.B, 64);
    auto tokens_of = [&](int b) { return b < 64 ? __builtin_amdgcn_readlane(t_lane, b) : seq_tokens(p, b); };

    int max_t = lanes_max(t_lane, n_lane);
    for (int b = 64; b < p.B; ++b) max_t = max(max_t, seq_tokens(p, b));

    const int hi = p.C / kSplitQuantum;
    int lo = ((max_t + p.max_splits - 1) / p.max_splits + kSplitQuantum - 1) / kSplitQuantum;   // the grid has max_splits
    lo = min(max(max(lo, p.c_min / kSplitQuantum), 1), hi);

    // whole rounds the planned size needs (exact)
    int at_hi = lanes_sum((t_lane + p.C - 1) / p.C, n_lane);
    for (int b = 64; b < p.B; ++b) at_hi += (seq_tokens(p, b) + p.C - 1) / p.C;
    const int rounds = (at_hi * streams + p.n_cu - 1) / p.n_cu;
    const float budget = (float)(rounds * p.n_cu) / (float)streams + 0.5f;      // splits that fit

    // first candidate q0 + lane * step (capped at hi) whose split count fits; -1 if none does
    auto first_fit = [&](int q0, int step) {
        const int q = min(q0 + lane * step, hi);
        const float rc = 1.0f / (float)(q * kSplitQuantum);
        float n = 0.f;
        for (int b = 0; b < p.B; ++b) n += ceilf((float)tokens_of(b) * rc);
        const unsigned long long ok = __ballot(n <= budget);
        return ok ? (int)__ffsll((long long)ok) - 1 : -1;
    };
    if (hi == lo) return hi * kSplitQuantum;
    const int step = (hi - lo + 62) / 63;            // lane 63 reaches hi; <= 5 for the largest split the planner allows
    const int l1 = first_fit(lo, step);
    if (l1 < 0) return hi * kSplitQuantum;
    int q = lo + l1 * step;
    if (l1 > 0 && step > 1) {                        // refine between the last misfit and the first fit
        const int q1 = lo + (l1 - 1) * step + 1;
        const int l2 = first_fit(q1, 1);
        if (l2 >= 0) q = q1 + l2;
    }
    const int C = min(q, hi) * kSplitQuantum;
    // the launched grid has room for what the bounds above allow; should the float counts ever
    // have let more through, the planned size (which always fits) is used instead
    int total = lanes_sum((t_lane + C - 1) / C, n_lane);
    for (int b = 64; b < p.B; ++b) total += (seq_tokens(p, b) + C - 1) / C;
    return total <= p.item_slots ? C : p.C;
}

// Layout of the batch plan that batch_plan_kernel leaves in the workspace (int32): [0] the split
// size C derived from the lengths, [1] the number of (sequence, split) pairs, [2 + b] the pairs
// of the sequences before b (b = 0 .. B).
constexpr int kPlanHeader = 2;

// The (sequence, split) pair that work item `id` of a batch stands for when the items of all
// sequences are numbered densely, sequence by sequence: workgroups that have something to do then
// come first in launch order and the surplus of the grid (sized for the worst case) trails behind,
// instead of being dispatched in between and holding up the ones behind them.  Reads the plan; one
// round trip for up to 64 sequences.  Wave-uniform; false if id is beyond the last item.
__device__ __forceinline__ bool batch_item(const KParams &p, int id, int *b_out, int *c_out)
{
    const int lane = threadIdx.x & 63;
    const int32_t *prefix = p.dev_c + kPlanHeader;
    for (int b0 = 0; b0 < p.B; b0 += 64) {
        const bool live = b0 + lane < p.B;
        const int lo = live ? prefix[b0 + lane] : 0x7fffffff;
        const int up = live ? prefix[b0 + lane + 1] : 0x7fffffff;
        const unsigned long long hit = __ballot(live && id >= lo && id < up);
        if (hit) {
            const int l = (int)__ffsll((long long)hit) - 1;
            *b_out = b0 + l;
            *c_out = id - __builtin_amdgcn_readlane(lo, l);
            return true;
        }
    }
    return false;
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

// max over the four lanes {l, l^16, l^32, l^48}.  permlane32_swap(a, b) trades
// a's upper 32 lanes against b's lower 32; permlane16_swap trades a's odd
// 16-lane rows against b's even rows; fed with two copies of x, the two
// results together hold x and its partner for every lane.
__device__ __forceinline__ float quad_column_max(float v)
{
    const uint32_t x = __builtin_bit_cast(uint32_t, v);
    auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    const float a = fmaxf(__builtin_bit_cast(float, (uint32_t)r[0]), __builtin_bit_cast(float, (uint32_t)r[1]));
    const uint32_t y = __builtin_bit_cast(uint32_t, a);
    auto r2 = __builtin_amdgcn_permlane16_swap(y, y, false, false);
    return fmaxf(__builtin_bit_cast(float, (uint32_t)r2[0]), __builtin_bit_cast(float, (uint32_t)r2[1]));
}

}  // namespace owl
