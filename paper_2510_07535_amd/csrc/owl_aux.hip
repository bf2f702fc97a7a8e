// Log-sum-exp combine of the split partials, the tree-mask builder and the
// page-gather test hook.
#include "owl_device.h"

namespace owl {

// ---------------------------------------------------------------------------
// Combine.  A partial of split s is the triple (m_s, l_s, O_s) with
// O_s = sum_k 2^(x_k - m_s) v_k and l_s = sum_k 2^(x_k - m_s) over the split's
// visible keys (x = score * log2 e; m_s is the reference the split happened to
// use, not necessarily its max).  With M = max_s m_s:
//     out = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s.
// For fp32 inputs the partials are the raw accumulator fragments, float4
// [slot][u][lane] = channels 16*u + 4*quad .. +3 of row lane%16.  For 16-bit
// inputs (HALF) a row of a partial is stored normalised, O_s / (l_s s_s) with s_s
// its largest magnitude, as fp16: uint4 [slot][u/2][lane] holds the lane's four
// channels of tiles u and u + 1; the weight of split s is then 2^(m_s - M) l_s s_s.
//
// One workgroup per (sequence, KV head, 16-row tile, pair of channel tiles);
// its WAVES wavefronts (4, or 8 when there are more than 32 splits; 16 gained nothing) take every
// WAVES-th split, reduce their share against their own running maximum, and are
// merged through LDS with the same formula.
// ---------------------------------------------------------------------------
typedef _Float16 c_f16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float2 unpack_half2(uint32_t w)
{
    const c_f16x2 h = __builtin_bit_cast(c_f16x2, w);
    return make_float2((float)h[0], (float)h[1]);
}

template <int D, bool HALF, int WAVES>
__global__ void __launch_bounds__(64 * WAVES) combine_kernel(const KParams p)
{
    constexpr int NT = D / 16, UPW = 2;              // channel tiles per workgroup
    constexpr int NUG = NT / UPW;
    const int tg = blockIdx.x / NUG, u0 = (blockIdx.x % NUG) * UPW;
    const int g = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int j = lane & 15, qd = lane >> 4;

    const int L = load_ctx_len(p.ctx_lens, b, p.max_ctx_len, nullptr);
    const int Nb = load_n_draft(p.n_draft_seq, b, p.N, nullptr);
    int C = split_tokens_for(p, L + Nb);
    if (p.adapt == 2) {                                           // what the split-KV pass derived for this batch;
        C = *p.dev_c;                                             // forced into range should that pass not have run
        C = min(max(C / kSplitQuantum, 1) * kSplitQuantum, p.C);
    }
    int ns = Nb == 0 ? 0 : (L + Nb + C - 1) / C;                  // a sequence without drafts wrote no partials
    ns = min(ns, p.max_splits);
    const size_t slot0 = (((size_t)b * p.Hkv + g) * p.max_splits) * p.RT + tg;

    float mw = -INFINITY, lw = 0.f;
    float4 acc[UPW];
#pragma unroll
    for (int u = 0; u < UPW; ++u) acc[u] = make_float4(0.f, 0.f, 0.f, 0.f);
    // The merge is a chain (each split rescales the running sums), the loads are not: the
    // partials of kInFlight splits are requested together, so that a wavefront pays the
    // memory latency once per batch rather than once per split (up to 32 splits: once).
    constexpr int kInFlight = 8;
    for (int s0 = w; s0 < ns; s0 += WAVES * kInFlight) {
        float ms[kInFlight], ls[kInFlight], os[kInFlight];
        float4 x[kInFlight][UPW];
#pragma unroll
        for (int k = 0; k < kInFlight; ++k) {
            const int s = min(s0 + WAVES * k, ns - 1);       // past the end: re-read the last split, not merged
            const size_t slot = slot0 + (size_t)s * p.RT;
            ms[k] = p.part_ml[slot * kPartMl + j];
            ls[k] = p.part_ml[slot * kPartMl + 16 + j];
            if constexpr (HALF) {
                static_assert(UPW == 2, "one 16-byte piece per lane holds a pair of channel tiles");
                os[k] = ls[k] * p.part_ml[slot * kPartMl + 32 + j];   // the stored rows are O / (l s)
                const uint4 h = static_cast<const uint4 *>(p.part_o)[slot * (size_t)(NT / 2 * 64) + (u0 / 2) * 64 + lane];
                const float2 a0 = unpack_half2(h.x), a1 = unpack_half2(h.y), b0 = unpack_half2(h.z), b1 = unpack_half2(h.w);
                x[k][0] = make_float4(a0.x, a0.y, a1.x, a1.y);
                x[k][1] = make_float4(b0.x, b0.y, b1.x, b1.y);
            } else {
                const float4 *po = static_cast<const float4 *>(p.part_o) + slot * (size_t)(NT * 64) + lane;
#pragma unroll
                for (int u = 0; u < UPW; ++u) x[k][u] = po[(u0 + u) * 64];
            }
        }
#pragma unroll
        for (int k = 0; k < kInFlight; ++k) {
            if (s0 + WAVES * k < ns) {                       // uniform over the wavefront
                const float mn = fmaxf(mw, ms[k]);
                const float a = __builtin_amdgcn_exp2f(mw - mn);     // 0 on the first round (mw = -inf)
                const float c = __builtin_amdgcn_exp2f(ms[k] - mn);
                mw = mn;
                lw = lw * a + ls[k] * c;
                const float co = HALF ? c * os[k] : c;       // weight of the stored O fragment
#pragma unroll
                for (int u = 0; u < UPW; ++u) {
                    acc[u].x = acc[u].x * a + x[k][u].x * co; acc[u].y = acc[u].y * a + x[k][u].y * co;
                    acc[u].z = acc[u].z * a + x[k][u].z * co; acc[u].w = acc[u].w * a + x[k][u].w * co;
                }
            }
        }
    }
    __shared__ float4 s_acc[WAVES][UPW][64];
    __shared__ float s_m[WAVES][64], s_l[WAVES][64];
#pragma unroll
    for (int u = 0; u < UPW; ++u) s_acc[w][u][lane] = acc[u];
    s_m[w][lane] = mw;
    s_l[w][lane] = lw;
    __syncthreads();
    if (w != 0) return;
    float M = s_m[0][lane];
#pragma unroll
    for (int k = 1; k < WAVES; ++k) M = fmaxf(M, s_m[k][lane]);
    float lsum = 0.f;
    float4 tot[UPW];
#pragma unroll
    for (int u = 0; u < UPW; ++u) tot[u] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int k = 0; k < WAVES; ++k) {
        const float wk = s_m[k][lane] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(s_m[k][lane] - M);
        lsum += wk * s_l[k][lane];
#pragma unroll
        for (int u = 0; u < UPW; ++u) {
            const float4 x = s_acc[k][u][lane];
            tot[u].x += wk * x.x; tot[u].y += wk * x.y; tot[u].z += wk * x.z; tot[u].w += wk * x.w;
        }
    }
    const int row = tg * kRowTile + j;
    if (row >= p.R) return;
    const int i = row / p.G, hh = row % p.G;
    const float inv = i < Nb ? 1.0f / lsum : 0.f;                   // rows of absent nodes come out as zeros
    const int64_t o = (((int64_t)b * p.N + i) * p.Hq + g * p.G + hh) * D + 4 * qd;
#pragma unroll
    for (int u = 0; u < UPW; ++u)
        store_out4(p.out, o + 16 * (u0 + u),
                   i < Nb ? make_float4(tot[u].x * inv, tot[u].y * inv, tot[u].z * inv, tot[u].w * inv)
                          : make_float4(0.f, 0.f, 0.f, 0.f),
                   p.out_dtype);
}

template <int WAVES>
static void launch_combine_waves(const KParams &p, int D, bool half_partials, dim3 grid, hipStream_t s)
{
    const dim3 block(64 * WAVES);
    if (D == 128 && half_partials) hipLaunchKernelGGL((combine_kernel<128, true, WAVES>), grid, block, 0, s, p);
    else if (D == 128) hipLaunchKernelGGL((combine_kernel<128, false, WAVES>), grid, block, 0, s, p);
    else if (half_partials) hipLaunchKernelGGL((combine_kernel<64, true, WAVES>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((combine_kernel<64, false, WAVES>), grid, block, 0, s, p);
}

hipError_t launch_combine(const KParams &p, int D, bool half_partials, hipStream_t s)
{
    dim3 grid(p.RT * (D / 32), p.Hkv, p.B);
    // a wavefront merges its splits as a chain, 8 loads in flight: beyond 32 splits more wavefronts share them
    if (p.max_splits > 32) launch_combine_waves<8>(p, D, half_partials, grid, s);
    else launch_combine_waves<4>(p, D, half_partials, grid, s);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Tree mask: one wavefront per sequence, lane i walks node i's root path.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(64) tree_mask_kernel(const int32_t *parent, int N, uint64_t *anc,
                                                       int32_t *depth, uint32_t *status)
{
    __shared__ int32_t s_parent[64];
    const int b = blockIdx.x, i = threadIdx.x;
    if (i < N) s_parent[i] = parent[(int64_t)b * N + i];
    __syncthreads();
    if (i < N) {
        int d;
        anc[(int64_t)b * N + i] = ancestor_set(s_parent, i, &d, status);
        if (depth) depth[(int64_t)b * N + i] = d;
    }
}

hipError_t launch_tree_mask(const int32_t *parent, int B, int N, uint64_t *anc, int32_t *depth,
                            uint32_t *status, hipStream_t s)
{
    hipLaunchKernelGGL(tree_mask_kernel, dim3(B), dim3(64), 0, s, parent, N, anc, depth, status);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Gather: dst[t][g][:] = cache row of logical position first + t, 16 bytes per
// thread.  Same page walk as the split-KV pass.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) gather_kernel(const unsigned char *cache,
                                                     const int32_t *page_table, int seq,
                                                     int max_pages, int64_t n_pool_pages, int Hkv,
                                                     int row_bytes, int es, int64_t stride_page,
                                                     int64_t stride_head, int64_t stride_token,
                                                     int64_t first, int64_t n, unsigned char *dst,
                                                     uint32_t *status)
{
    const int ppr = row_bytes / 16;
    const int64_t total = n * Hkv * ppr;
    for (int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x; id < total;
         id += (int64_t)gridDim.x * 256) {
        const int piece = (int)(id % ppr);
        const int g = (int)((id / ppr) % Hkv);
        const int64_t t = id / ((int64_t)ppr * Hkv);
        const int64_t pos = first + t;
        const int64_t pg = load_page(page_table, seq, max_pages, n_pool_pages, (int)(pos / kPage), status);
        const int64_t off = (pg * stride_page + g * stride_head + (pos % kPage) * stride_token) * es;
        *reinterpret_cast<uint4 *>(dst + (t * Hkv + g) * row_bytes + piece * 16) =
            *reinterpret_cast<const uint4 *>(cache + off + piece * 16);
    }
}

hipError_t launch_gather(const owl_verify_desc &d, const void *cache, const int32_t *page_table,
                         int seq, int64_t first, int64_t n, void *dst, uint32_t *status,
                         hipStream_t s)
{
    if (n == 0) return hipSuccess;
    const int es = d.qkv_dtype == OWL_F32 ? 4 : 2;
    const int row_bytes = d.head_dim * es;
    const int64_t total = n * d.n_kv_heads * (row_bytes / 16);
    int blocks = (int)((total + 255) / 256);
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(gather_kernel, dim3(blocks), dim3(256), 0, s,
                       static_cast<const unsigned char *>(cache), page_table, seq,
                       d.max_pages_per_seq, d.n_pool_pages, d.n_kv_heads, row_bytes, es,
                       d.kv_stride_page, d.kv_stride_head, d.kv_stride_token, first, n,
                       static_cast<unsigned char *>(dst), status);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Batch plan (batches with a library-chosen split size): one wavefront derives the
// split size from the actual lengths (batch_split_tokens) and numbers the
// (sequence, split) pairs densely; the split-KV pass and the combine read the
// result instead of deriving it once per workgroup (which cost every workgroup of
// the batched benchmark shape 4 us).
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(64) batch_plan_kernel(const KParams p)
{
    const int lane = threadIdx.x;
    const int C = batch_split_tokens(p);
    int32_t *prefix = p.dev_c + kPlanHeader;
    int base = 0;
    for (int b0 = 0; b0 < p.B; b0 += 64) {
        const bool live = b0 + lane < p.B;
        const int n = live ? (seq_tokens(p, b0 + lane) + C - 1) / C : 0;
        int scan = n;                                 // inclusive scan over the lanes
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(scan, off);
            if (lane >= off) scan += up;
        }
        if (live) prefix[b0 + lane] = base + scan - n;
        base += __builtin_amdgcn_readlane(scan, 63);
    }
    if (lane == 0) {
        prefix[p.B] = base;
        p.dev_c[0] = C;
        p.dev_c[1] = base;
    }
}

hipError_t launch_batch_plan(const KParams &p, hipStream_t s)
{
    hipLaunchKernelGGL(batch_plan_kernel, dim3(1), dim3(64), 0, s, p);
    return hipGetLastError();
}

// Makes the runtime resolve the combine kernels now, so that their first launch may happen
// inside a stream capture.
hipError_t load_aux_kernels()
{
    hipFuncAttributes a;
    hipError_t e = hipSuccess;
    const void *fns[] = {
        reinterpret_cast<const void *>(&combine_kernel<128, true, 4>), reinterpret_cast<const void *>(&combine_kernel<128, false, 4>),
        reinterpret_cast<const void *>(&combine_kernel<64, true, 4>), reinterpret_cast<const void *>(&combine_kernel<64, false, 4>),
        reinterpret_cast<const void *>(&combine_kernel<128, true, 8>), reinterpret_cast<const void *>(&combine_kernel<128, false, 8>),
        reinterpret_cast<const void *>(&combine_kernel<64, true, 8>), reinterpret_cast<const void *>(&combine_kernel<64, false, 8>),
    };
    for (const void *f : fns)
        if (e == hipSuccess) e = hipFuncGetAttributes(&a, f);
    if (e == hipSuccess) e = hipFuncGetAttributes(&a, reinterpret_cast<const void *>(&batch_plan_kernel));
    return e;
}

}  // namespace owl
