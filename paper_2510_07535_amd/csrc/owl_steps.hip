// The integer / data-movement steps on either side of the verify attention
// (Algorithm 1 of the paper): Prepare (Sec. 3.2.2, one extra token per tree
// node, mask and position ids), the greedy choice of the accepted path
// (Sec. 1 / Sec. 2: the target keeps the longest drafted path that agrees with
// its own next tokens), and the commit of that path's K/V rows into the
// context (Algorithm 1: l <- l;d, N <- N + |d|).  All results are exact.
#include "owl_device.h"

namespace owl {

// ---------------------------------------------------------------------------
// Prepare: one workgroup per sequence, thread i < 2n owns token i of the verify
// input.  Tokens 0..n-1 are the tree nodes, token n+k is the extra token of node
// k: its parent is k, so the ordinary root-path walk gives its mask and depth.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(64) prepare_kernel(const int32_t *parent, const int32_t *ctx_lens, int n,
                                                     int32_t *parent2, uint64_t *anc, int32_t *depth,
                                                     int32_t *pos, uint32_t *status)
{
    __shared__ int32_t s_parent[64];
    const int b = blockIdx.x, i = threadIdx.x, n2 = 2 * n;
    if (i < n) s_parent[i] = parent[(int64_t)b * n + i];
    else if (i < n2) s_parent[i] = i - n;
    __syncthreads();
    if (i < n2) {
        int d;
        const uint64_t a = ancestor_set(s_parent, i, &d, status);
        int p = s_parent[i];
        if (p < -1 || p >= i) p = -1;                      // flagged by the walk; keep the output a valid tree
        const int64_t o = (int64_t)b * n2 + i;
        parent2[o] = p;
        anc[o] = a;
        if (depth) depth[o] = d;
        if (pos) pos[o] = ctx_lens[b] + d - 1;
    }
}

hipError_t launch_prepare(const int32_t *parent, const int32_t *ctx_lens, int B, int n, int32_t *parent2,
                          uint64_t *anc, int32_t *depth, int32_t *pos, uint32_t *status, hipStream_t s)
{
    hipLaunchKernelGGL(prepare_kernel, dim3(B), dim3(64), 0, s, parent, ctx_lens, n, parent2, anc, depth, pos,
                       status);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Acceptance: one wavefront per sequence, lane i owns node i.  A node "agrees"
// if its token is the target's next token at its parent (at the context end for
// a root); it is reachable if it and all its ancestors agree.  Parents precede
// children, so reachability spreads one tree level per round of a ballot loop
// that ends when a round adds nothing (at most depth rounds).  The answer is the
// reachable node of greatest depth, smallest index on ties; its root path is
// written from the root down.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(64) accept_kernel(const int32_t *tokens, const int32_t *parent,
                                                    const int32_t *target_root, const int32_t *target_next,
                                                    int N, int n_cand, int32_t *accepted, int32_t *n_accept,
                                                    int32_t *bonus, int32_t *last, uint32_t *status)
{
    __shared__ int32_t s_parent[64];
    const int b = blockIdx.x, i = threadIdx.x;
    const int64_t row = (int64_t)b * N;
    int p = -1;
    bool agrees = false;
    if (i < N) {
        p = parent[row + i];
        if (p < -1 || p >= i) {
            flag_status(status, OWL_DEV_BAD_PARENT);
            p = -1;
        }
        s_parent[i] = p;
        if (i < n_cand && p < n_cand) {
            const int want = p < 0 ? target_root[b] : target_next[row + p];
            agrees = tokens[row + i] == want;
        }
    }
    __syncthreads();
    uint64_t reach = 0;
    int depth = 0;                                          // depth of lane's node once reached
    for (int round = 1; round <= N; ++round) {              // uniform: `reach` is the same in every lane
        const bool now = agrees && !((reach >> i) & 1) && (p < 0 ? round == 1 : ((reach >> p) & 1));
        const uint64_t add = __builtin_amdgcn_ballot_w64(now);
        if (now) depth = round;
        if (add == 0) break;
        reach |= add;
    }
    // deepest reachable node, smallest index on ties: key = depth * 64 + (63 - i)
    int key = ((reach >> i) & 1) ? depth * 64 + (63 - i) : -1;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) key = max(key, __shfl_xor(key, off));
    const int best = key < 0 ? -1 : 63 - (key & 63);
    const int na = key < 0 ? 0 : key >> 6;
    if (i < N) accepted[row + i] = -1;
    __syncthreads();
    if (i == 0) {
        n_accept[b] = na;
        last[b] = best;
        bonus[b] = best < 0 ? target_root[b] : target_next[row + best];
        int jn = best;
        for (int k = na - 1; k >= 0 && jn >= 0; --k) {       // walks strictly decreasing indices
            accepted[row + k] = jn;
            jn = s_parent[jn];
        }
    }
}

hipError_t launch_accept(const int32_t *tokens, const int32_t *parent, const int32_t *target_root,
                         const int32_t *target_next, int B, int N, int n_cand, int32_t *accepted,
                         int32_t *n_accept, int32_t *bonus, int32_t *last, uint32_t *status, hipStream_t s)
{
    hipLaunchKernelGGL(accept_kernel, dim3(B), dim3(64), 0, s, tokens, parent, target_root, target_next, N,
                       n_cand, accepted, n_accept, bonus, last, status);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// KV commit: one workgroup per (KV head, sequence, tensor).  Row i of the
// accepted path moves from logical position L + accepted[i] to L + i.  A source
// slot can be another row's destination (accepted = (1, 2): slot 1 is read by
// row 0 and written by row 1), so every thread loads all its 16-byte pieces
// first, the workgroup meets at a barrier, and only then anything is stored.
// accepted[] must be strictly increasing (a root path in a tree whose parents
// precede their children is); anything else is flagged and nothing is moved.
// The same holds for pages: every source and destination page of the sequence
// is looked up before anything is loaded, and one entry outside the pool (or a
// position beyond the table) means OWL_DEV_BAD_PAGE, no row of that sequence
// moves, and its new length equals the old one.  A kernel that writes must not
// replace a bad page by some other page.
// ---------------------------------------------------------------------------
constexpr int kCommitThreads = 256;
constexpr int kCommitMaxPieces = 8;                         // 64 rows x 32 pieces / 256 threads

__global__ void __launch_bounds__(kCommitThreads) commit_kernel(
    unsigned char *k_cache, unsigned char *v_cache, const int32_t *page_table, const int32_t *ctx_lens,
    const int32_t *accepted, const int32_t *n_accept, int N, int max_pages, int max_ctx_len,
    int64_t n_pool_pages, int row_bytes, int es, int64_t stride_page, int64_t stride_head,
    int64_t stride_token, int32_t *new_ctx_lens, uint32_t *status)
{
    __shared__ int32_t s_src[64];
    __shared__ int64_t s_src_page[64], s_dst_page[64];
    __shared__ int s_bad, s_bad_page;
    const int g = blockIdx.x, b = blockIdx.y;
    unsigned char *cache = blockIdx.z ? v_cache : k_cache;
    const int tid = threadIdx.x;
    const int L = load_ctx_len(ctx_lens, b, max_ctx_len, status);
    int na = n_accept[b];
    if (tid == 0) s_bad = s_bad_page = 0;
    __syncthreads();
    if (na < 0 || na > N) {
        if (tid == 0) flag_status(status, OWL_DEV_BAD_ACCEPT);
        na = 0;
    }
    if (tid < na) {
        const int a = accepted[(int64_t)b * N + tid];
        const int prev = tid > 0 ? accepted[(int64_t)b * N + tid - 1] : -1;
        if (a < 0 || a >= N || a <= prev) s_bad = 1;
        s_src[tid] = a;
        // physical pages of the row's source and destination, unchecked ids; -1 = not in the table
        auto page_of = [&](int pos) -> int64_t {
            const int lp = pos / kPage;
            if (!page_table) return lp;
            return lp < max_pages ? (int64_t)page_table[(int64_t)b * max_pages + lp] : -1;
        };
        const int64_t sp = (a >= 0 && a < N) ? page_of(L + a) : 0, dp = page_of(L + tid);
        if (sp < 0 || sp >= n_pool_pages || dp < 0 || dp >= n_pool_pages) s_bad_page = 1;
        s_src_page[tid] = sp;
        s_dst_page[tid] = dp;
    }
    __syncthreads();
    if (s_bad) {                                            // uniform over the workgroup
        if (tid == 0) flag_status(status, OWL_DEV_BAD_ACCEPT);
        na = 0;
    } else if (s_bad_page) {
        if (tid == 0) flag_status(status, OWL_DEV_BAD_PAGE);
        na = 0;
    }
    if (g == 0 && blockIdx.z == 0 && tid == 0 && new_ctx_lens) new_ctx_lens[b] = L + na;

    const int ppr = row_bytes / 16;
    const int total = na * ppr;
    uint4 held[kCommitMaxPieces];
#pragma unroll
    for (int r = 0; r < kCommitMaxPieces; ++r) {
        const int id = tid + r * kCommitThreads;
        if (id < total) {
            const int i = id / ppr, piece = id % ppr;
            const int pos = L + s_src[i];
            const int64_t off = (s_src_page[i] * stride_page + g * stride_head + (pos % kPage) * stride_token) * es;
            held[r] = *reinterpret_cast<const uint4 *>(cache + off + piece * 16);
        }
    }
    __syncthreads();                                        // all reads done before the first write
#pragma unroll
    for (int r = 0; r < kCommitMaxPieces; ++r) {
        const int id = tid + r * kCommitThreads;
        if (id < total) {
            const int i = id / ppr, piece = id % ppr;
            if (s_src[i] != i) {                            // a row already in place is left alone
                const int pos = L + i;
                const int64_t off = (s_dst_page[i] * stride_page + g * stride_head + (pos % kPage) * stride_token) * es;
                *reinterpret_cast<uint4 *>(cache + off + piece * 16) = held[r];
            }
        }
    }
}

hipError_t launch_commit(const owl_verify_desc &d, void *k_cache, void *v_cache, const int32_t *page_table,
                         const int32_t *ctx_lens, const int32_t *accepted, const int32_t *n_accept,
                         int32_t *new_ctx_lens, uint32_t *status, hipStream_t s)
{
    const int es = d.qkv_dtype == OWL_F32 ? 4 : 2;
    const int row_bytes = d.head_dim * es;
    static_assert(64 * 32 <= kCommitThreads * kCommitMaxPieces, "64 rows of up to 512 bytes fit the held pieces");
    hipLaunchKernelGGL(commit_kernel, dim3(d.n_kv_heads, d.batch, 2), dim3(kCommitThreads), 0, s,
                       static_cast<unsigned char *>(k_cache), static_cast<unsigned char *>(v_cache), page_table,
                       ctx_lens, accepted, n_accept, d.n_draft, d.max_pages_per_seq, d.max_ctx_len,
                       d.n_pool_pages, row_bytes, es, d.kv_stride_page, d.kv_stride_head, d.kv_stride_token,
                       new_ctx_lens, status);
    return hipGetLastError();
}

}  // namespace owl
