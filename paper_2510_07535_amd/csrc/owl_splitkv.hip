// Split-KV pass of the verify-step attention for gfx950 (MI355X).
//
// One workgroup (4 wavefronts) owns one (sequence, KV head, KV split, row
// group).  It streams its split of the paged K/V cache through LDS exactly once
// and holds, in MFMA accumulators, the un-normalised outputs of ALL query rows
// that share this KV head: rows = (draft node i, query head within the group),
// R = (Hq/Hkv) * N of them, cut into 16-row tiles.  That packing is what makes
// the cost of verifying N drafted tokens "hidden" behind the scan of the
// context (Sec. 1 / Sec. 2 of the paper): the cache is read once whatever N is.
//
// Tile algebra (all MFMA tiles are 16x16, wave64):
//   S^T[key][row] = K[key][:] . Q[row][:]        A = K fragment, B = Q fragment
//   O^T[d][row]  += V^T[d][key] * P^T[key][row]  A = V^T fragment, B = P fragment
// With keys along M, a lane owns ONE query row (column lane%16) and the keys of
// a tile sit in its registers, so the softmax needs only a 4-lane exchange, and
// the fp32 S^T accumulators turn into the bf16 P^T operand in place.  The order
// of the contraction index is free as long as both operands agree, which is
// used twice: K/Q take channels 32*kk + 8*quad + e, and V^T is fed with output
// channel d = NT*m + t for row m of channel tile t, so a lane fetches NT
// contiguous channels of a key with one LDS read and transposes 16-bit halves
// in registers.  The row sum l rides along as one more channel tile whose V^T
// operand is all ones, so it is summed from the very P values (after rounding
// to bf16) that weigh V.
//
// Visibility (Sec. 3.2.2, Decode Stage): every row sees the whole prefix; among
// the drafts, row (i, .) sees node j iff j is on i's root path, i included.
// Only 32-key steps that reach past the prefix take the masked path.
#include <type_traits>

#include "owl_device.h"

namespace owl {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

constexpr float kMInit = -1.0e30f;   // "no key seen yet"; finite so that m - m is 0
constexpr float kTau = 8.0f;         // rescale only when a row's max moved by > 2^8

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <typename T>
__device__ __forceinline__ f32x4 mfma16(const uint4 &a, const uint4 &b, const f32x4 &c)
{
    if constexpr (std::is_same<T, __bf16>::value)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a),
                                                      __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

template <typename T>
__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    f32x2 v = {lo, hi};
    if constexpr (std::is_same<T, __bf16>::value)
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    else
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
}

template <typename T>
__device__ __forceinline__ uint32_t ones2()
{
    return std::is_same<T, __bf16>::value ? 0x3F803F80u : 0x3C003C00u;
}

// Geometry of one instantiation.
template <typename T, int D, int TPW, int WR, int WK>
struct Geo {
    static constexpr bool kF32 = std::is_same<T, float>::value;
    static constexpr int ES = sizeof(T);
    static constexpr int KSTEPS = WK == 4 ? 4 : 2;      // 32-key steps per LDS stage
    static constexpr int SK = 32 * KSTEPS;              // keys per stage
    static constexpr int ROWB = D * ES;                 // bytes of one key row
    static constexpr int PPR = ROWB / 16;               // 16-byte pieces per row
    static constexpr int LPT = SK * PPR / 256;          // pieces per thread per tensor
    static constexpr int NT = D / 16;                   // channel tiles of O^T
    static constexpr int STAGE = SK * ROWB;             // bytes per tensor per stage
    static constexpr int QREGS = kF32 ? D / 4 : D / 32; // Q fragment slots per tile
    static constexpr size_t LDS = 4 * (size_t)STAGE + kMaxPagesPerSplit * 4 + 64 * 8 + 64 * 4;
    static_assert(WR * WK == 4, "four wavefronts per workgroup");
    static_assert(SK * PPR % 256 == 0, "stage must divide over the workgroup");
    static_assert((WK - 1) * WR * TPW * (4 * (NT + 1) + 1) * 256 <= 4 * STAGE,
                  "cross-wave merge buffer must fit in the stage buffers");
};

template <typename T, int D, int TPW, int WR, int WK>
__global__ void __launch_bounds__(256, (TPW <= 2 && !std::is_same<T, float>::value) ? 2 : 1)
splitkv_kernel(const KParams p)
{
    using GEO = Geo<T, D, TPW, WR, WK>;
    constexpr bool kF32 = GEO::kF32;
    constexpr int ES = GEO::ES, KSTEPS = GEO::KSTEPS, SK = GEO::SK, ROWB = GEO::ROWB;
    constexpr int PPR = GEO::PPR, LPT = GEO::LPT, NT = GEO::NT, STAGE = GEO::STAGE;
    constexpr int QREGS = GEO::QREGS;
    constexpr int SWZ = (PPR - 1) & 15;

    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char *Ks = smem;
    unsigned char *Vs = smem + 2 * STAGE;
    int32_t *s_pages = reinterpret_cast<int32_t *>(smem + 4 * STAGE);
    uint64_t *s_anc = reinterpret_cast<uint64_t *>(s_pages + kMaxPagesPerSplit);
    int32_t *s_parent = reinterpret_cast<int32_t *>(s_anc + 64);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave % WR, wk = wave / WR;
    const int j = lane & 15, qd = lane >> 4;

    const int c = blockIdx.x;
    const int g = blockIdx.y / p.row_groups, rg = blockIdx.y % p.row_groups;
    const int b = blockIdx.z;

    const int L = load_ctx_len(p.ctx_lens, b, p.max_ctx_len, p.dev_status);
    const int Ttot = L + p.N;
    const int pos0 = c * p.C;
    if (pos0 >= Ttot) return;                       // this split does not exist for b
    const int pos1 = min(pos0 + p.C, Ttot);
    const int nstages = (pos1 - pos0 + SK - 1) / SK;

    // ---- page list of this split, and the tree mask if drafts are in reach ----
    {
        const int npg = (pos1 - pos0 + kPage - 1) / kPage;
        for (int idx = tid; idx < npg; idx += 256)
            s_pages[idx] = load_page(p.page_table, b, p.max_pages, p.n_pool_pages,
                                     pos0 / kPage + idx, p.dev_status);
    }
    const bool has_drafts = pos1 > L;               // uniform over the workgroup
    if (has_drafts) {
        if (tid < p.N) s_parent[tid] = p.parent[(int64_t)b * p.N + tid];
        __syncthreads();
        if (tid < p.N) s_anc[tid] = ancestor_set(s_parent, tid, nullptr, p.dev_status);
    }
    __syncthreads();

    // ---- this wave's query rows ----
    uint4 qf[TPW][kF32 ? 1 : QREGS];
    float qs[TPW][kF32 ? QREGS : 1];
    int irow[TPW];
    bool tile_ok[TPW];
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
        const int tg = (rg * WR + wr) * TPW + t;
        tile_ok[t] = tg < p.RT;
        const int row = tg * kRowTile + j;
        const bool ok = tile_ok[t] && row < p.R;
        const int i = ok ? row / p.G : 0;
        const int hh = ok ? row % p.G : 0;
        irow[t] = ok ? i : -1;
        const unsigned char *qp = static_cast<const unsigned char *>(p.q) +
            ((((int64_t)b * p.N + i) * p.Hq + g * p.G + hh) * D) * ES;
        if constexpr (kF32) {
#pragma unroll
            for (int kk = 0; kk < QREGS; ++kk)
                qs[t][kk] = ok ? reinterpret_cast<const float *>(qp)[4 * kk + qd] : 0.f;
        } else {
#pragma unroll
            for (int kk = 0; kk < QREGS; ++kk)
                qf[t][kk] = ok ? *reinterpret_cast<const uint4 *>(qp + (32 * kk + 8 * qd) * ES)
                               : make_uint4(0, 0, 0, 0);
        }
    }

    f32x4 O[TPW][NT + 1];
    float m[TPW];
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
        m[t] = kMInit;
#pragma unroll
        for (int u = 0; u <= NT; ++u) O[t][u] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // ---- stage loads: global -> registers -> LDS ----
    const unsigned char *kbase = static_cast<const unsigned char *>(p.k);
    const unsigned char *vbase = static_cast<const unsigned char *>(p.v);
    uint4 kreg[LPT], vreg[LPT];

    auto load_stage = [&](int s) {
        const int sbase = pos0 + s * SK;
#pragma unroll
        for (int it = 0; it < LPT; ++it) {
            const int id = it * 256 + tid;
            const int key = id / PPR, piece = id % PPR;
            const int pos = sbase + key;
            if (pos < pos1) {
                const int64_t pg = s_pages[(pos - pos0) >> 4];
                const int64_t off = (pg * p.stride_page + (int64_t)g * p.stride_head +
                                     (int64_t)(pos & (kPage - 1)) * p.stride_token) * ES + piece * 16;
                kreg[it] = *reinterpret_cast<const uint4 *>(kbase + off);
                vreg[it] = *reinterpret_cast<const uint4 *>(vbase + off);
            } else {
                kreg[it] = make_uint4(0, 0, 0, 0);   // keys past the end: finite, masked later
                vreg[it] = make_uint4(0, 0, 0, 0);
            }
        }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int it = 0; it < LPT; ++it) {
            const int id = it * 256 + tid;
            const int key = id / PPR, piece = id % PPR;
            *reinterpret_cast<uint4 *>(Ks + buf * STAGE + key * ROWB + ((piece ^ (key & SWZ)) << 4)) = kreg[it];
            *reinterpret_cast<uint4 *>(Vs + buf * STAGE + key * ROWB + (piece << 4)) = vreg[it];
        }
    };

    // ---- softmax of one row tile over one 32-key step ----
    auto softmax_step = [&](f32x4 &s0, f32x4 &s1, int t, int step_pos, bool masked) {
        if (masked) {
            uint64_t anc = ~(uint64_t)0;
            if (has_drafts && irow[t] >= 0) anc = s_anc[irow[t]];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int pa = step_pos + 4 * qd + r, pb = pa + 16;
                const bool va = pa < L || (pa < Ttot && ((anc >> (pa - L)) & 1));
                const bool vb = pb < L || (pb < Ttot && ((anc >> (pb - L)) & 1));
                s0[r] = va ? s0[r] : -INFINITY;
                s1[r] = vb ? s1[r] : -INFINITY;
            }
        }
        float tm = fmaxf(fmaxf(fmaxf(s0[0], s0[1]), fmaxf(s0[2], s0[3])),
                         fmaxf(fmaxf(s1[0], s1[1]), fmaxf(s1[2], s1[3])));
        tm = fmaxf(tm, __shfl_xor(tm, 16));
        tm = fmaxf(tm, __shfl_xor(tm, 32));
        const float sc = tm * p.c_log2;
        if (__builtin_amdgcn_ballot_w64(sc > m[t] + kTau) != 0) {   // uniform over the wave
            const float mn = fmaxf(m[t], sc);
            const float alpha = fast_exp2(m[t] - mn);
            m[t] = mn;
#pragma unroll
            for (int u = 0; u <= NT; ++u) O[t][u] *= alpha;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            s0[r] = fast_exp2(__builtin_fmaf(s0[r], p.c_log2, -m[t]));
            s1[r] = fast_exp2(__builtin_fmaf(s1[r], p.c_log2, -m[t]));
        }
    };

    // ---- one 32-key step of a stage held in LDS buffer `buf` ----
    auto compute_step = [&](int buf, int ks, int step_pos) {
        const unsigned char *Kb = Ks + buf * STAGE + ks * 32 * ROWB;
        const unsigned char *Vb = Vs + buf * STAGE + ks * 32 * ROWB;
        const bool masked = step_pos + 32 > L;       // reaches drafts or the ragged end
        if constexpr (kF32) {
            // fp32 path: 16x16x4 MFMA, one channel per quad and step
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                float kf[QREGS];
                const int key = kt * 16 + j;
#pragma unroll
                for (int kk = 0; kk < QREGS; ++kk)
                    kf[kk] = *reinterpret_cast<const float *>(
                        Kb + key * ROWB + ((kk ^ (key & SWZ)) << 4) + qd * 4);
                float vraw[4][NT];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int vkey = kt * 16 + 4 * qd + r;
#pragma unroll
                    for (int u = 0; u < NT / 4; ++u) {
                        const float4 x = *reinterpret_cast<const float4 *>(
                            Vb + vkey * ROWB + (j * NT + 4 * u) * 4);
                        vraw[r][4 * u] = x.x; vraw[r][4 * u + 1] = x.y;
                        vraw[r][4 * u + 2] = x.z; vraw[r][4 * u + 3] = x.w;
                    }
                }
#pragma unroll
                for (int t = 0; t < TPW; ++t) {
                    if (!tile_ok[t]) continue;
                    f32x4 s0 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kk = 0; kk < QREGS; ++kk)
                        s0 = __builtin_amdgcn_mfma_f32_16x16x4f32(kf[kk], qs[t][kk], s0, 0, 0, 0);
                    // the second half-tile of the step is handled by the kt loop:
                    // feed a fully masked dummy so the softmax sees 16 keys only
                    f32x4 s1 = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
                    softmax_step(s0, s1, t, step_pos + kt * 16, masked);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
#pragma unroll
                        for (int u = 0; u < NT; ++u)
                            O[t][u] = __builtin_amdgcn_mfma_f32_16x16x4f32(vraw[r][u], s0[r], O[t][u], 0, 0, 0);
                        O[t][NT] = __builtin_amdgcn_mfma_f32_16x16x4f32(1.0f, s0[r], O[t][NT], 0, 0, 0);
                    }
                }
            }
        } else {
            // K fragments: 2 key tiles x D/32 contraction steps
            uint4 kf[2][QREGS];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                const int key = kt * 16 + j;
#pragma unroll
                for (int kk = 0; kk < QREGS; ++kk)
                    kf[kt][kk] = *reinterpret_cast<const uint4 *>(
                        Kb + key * ROWB + (((4 * kk + qd) ^ (key & SWZ)) << 4));
            }
            // V: NT contiguous channels of 8 keys per lane, then a 16-bit transpose
            uint32_t vraw[8][NT / 2];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int vkey = (e < 4) ? 4 * qd + e : 16 + 4 * qd + (e - 4);
                const unsigned char *src = Vb + vkey * ROWB + j * NT * 2;
                if constexpr (NT == 8) {
                    const uint4 x = *reinterpret_cast<const uint4 *>(src);
                    vraw[e][0] = x.x; vraw[e][1] = x.y; vraw[e][2] = x.z; vraw[e][3] = x.w;
                } else {
                    const uint2 x = *reinterpret_cast<const uint2 *>(src);
                    vraw[e][0] = x.x; vraw[e][1] = x.y;
                }
            }
            uint4 vf[NT];
#pragma unroll
            for (int u = 0; u < NT; ++u) {
                const uint32_t sel = (u & 1) ? 0x07060302u : 0x05040100u;
                vf[u].x = __builtin_amdgcn_perm(vraw[1][u / 2], vraw[0][u / 2], sel);
                vf[u].y = __builtin_amdgcn_perm(vraw[3][u / 2], vraw[2][u / 2], sel);
                vf[u].z = __builtin_amdgcn_perm(vraw[5][u / 2], vraw[4][u / 2], sel);
                vf[u].w = __builtin_amdgcn_perm(vraw[7][u / 2], vraw[6][u / 2], sel);
            }
            const uint4 ones = make_uint4(ones2<T>(), ones2<T>(), ones2<T>(), ones2<T>());
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                if (!tile_ok[t]) continue;
                f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < QREGS; ++kk) {
                    s0 = mfma16<T>(kf[0][kk], qf[t][kk], s0);
                    s1 = mfma16<T>(kf[1][kk], qf[t][kk], s1);
                }
                softmax_step(s0, s1, t, step_pos, masked);
                uint4 pf;
                pf.x = pack2<T>(s0[0], s0[1]);
                pf.y = pack2<T>(s0[2], s0[3]);
                pf.z = pack2<T>(s1[0], s1[1]);
                pf.w = pack2<T>(s1[2], s1[3]);
#pragma unroll
                for (int u = 0; u < NT; ++u) O[t][u] = mfma16<T>(vf[u], pf, O[t][u]);
                O[t][NT] = mfma16<T>(ones, pf, O[t][NT]);
            }
        }
    };

    // ---- main loop: double-buffered stages ----
    load_stage(0);
    store_stage(0);
    __syncthreads();
    for (int s = 0; s < nstages; ++s) {
        const int buf = s & 1;
        const bool more = s + 1 < nstages;
        if (more) load_stage(s + 1);
        const int sbase = pos0 + s * SK;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            if (ks % WK != wk) continue;
            if (sbase + ks * 32 >= pos1) continue;   // uniform: nothing left in this step
            compute_step(buf, ks, sbase + ks * 32);
        }
        if (more) store_stage(buf ^ 1);
        __syncthreads();
    }

    // ---- merge the key groups of a row group through LDS (reuses the stages) ----
    if constexpr (WK > 1) {
        float *mb = reinterpret_cast<float *>(smem);
        constexpr int PER_TILE = 4 * (NT + 1) + 1;
        if (wk > 0) {
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                float *dst = mb + ((size_t)(((wk - 1) * WR + wr) * TPW + t) * PER_TILE) * 64 + lane;
#pragma unroll
                for (int u = 0; u <= NT; ++u)
#pragma unroll
                    for (int r = 0; r < 4; ++r) dst[(u * 4 + r) * 64] = O[t][u][r];
                dst[4 * (NT + 1) * 64] = m[t];
            }
        }
        __syncthreads();
        if (wk == 0) {
            for (int w2 = 1; w2 < WK; ++w2) {
#pragma unroll
                for (int t = 0; t < TPW; ++t) {
                    const float *src = mb + ((size_t)(((w2 - 1) * WR + wr) * TPW + t) * PER_TILE) * 64 + lane;
                    const float m2 = src[4 * (NT + 1) * 64];
                    const float mn = fmaxf(m[t], m2);
                    const float a1 = fast_exp2(m[t] - mn), a2 = fast_exp2(m2 - mn);
                    m[t] = mn;
#pragma unroll
                    for (int u = 0; u <= NT; ++u)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            O[t][u][r] = O[t][u][r] * a1 + src[(u * 4 + r) * 64] * a2;
                }
            }
        }
    }

    // ---- write this split's partial: accumulator fragments as they are ----
    if (wk == 0) {
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            const int tg = (rg * WR + wr) * TPW + t;
            if (tg >= p.RT) continue;
            const size_t slot = (((size_t)b * p.Hkv + g) * p.max_splits + c) * p.RT + tg;
            float4 *po = reinterpret_cast<float4 *>(p.part_o) + slot * (size_t)(NT * 64) + lane;
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int u = 0; u < NT / 4; ++u)
                    po[(r * (NT / 4) + u) * 64] = make_float4(O[t][4 * u][r], O[t][4 * u + 1][r],
                                                              O[t][4 * u + 2][r], O[t][4 * u + 3][r]);
            if (qd == 0) {
                p.part_ml[slot * 32 + j] = m[t];
                p.part_ml[slot * 32 + 16 + j] = O[t][NT][0];
            }
        }
    }
}

// ---------------------------------------------------------------------------
// instantiations
// ---------------------------------------------------------------------------
template <typename T, int D, int TPW, int WR, int WK>
static void launch_variant(const KParams &p, dim3 grid, hipStream_t s)
{
    using GEO = Geo<T, D, TPW, WR, WK>;
    hipLaunchKernelGGL((splitkv_kernel<T, D, TPW, WR, WK>), grid, dim3(256), GEO::LDS, s, p);
}

#define OWL_VARIANT(DT, T, D, TPW, WR, WK)                                              \
    Variant { DT, D, TPW, WR, WK, Geo<T, D, TPW, WR, WK>::LDS,                         \
              &launch_variant<T, D, TPW, WR, WK>,                                       \
              reinterpret_cast<const void *>(&splitkv_kernel<T, D, TPW, WR, WK>) }

#define OWL_VARIANTS_16BIT(DT, T, D)                                                    \
    OWL_VARIANT(DT, T, D, 1, 1, 4), OWL_VARIANT(DT, T, D, 2, 1, 4),                     \
    OWL_VARIANT(DT, T, D, 2, 2, 2), OWL_VARIANT(DT, T, D, 2, 4, 1),                     \
    OWL_VARIANT(DT, T, D, 3, 4, 1), OWL_VARIANT(DT, T, D, 4, 4, 1),                     \
    OWL_VARIANT(DT, T, D, 5, 4, 1)

static const Variant kVariants[] = {
    OWL_VARIANTS_16BIT(OWL_BF16, __bf16, 128),
    OWL_VARIANTS_16BIT(OWL_BF16, __bf16, 64),
    OWL_VARIANTS_16BIT(OWL_F16, _Float16, 128),
    OWL_VARIANTS_16BIT(OWL_F16, _Float16, 64),
    OWL_VARIANT(OWL_F32, float, 64, 1, 4, 1),
    OWL_VARIANT(OWL_F32, float, 128, 1, 4, 1),
};

const Variant *find_variant(int dtype, int D, int tpw, int wr, int wk)
{
    for (const Variant &v : kVariants)
        if (v.dtype == dtype && v.D == D && v.tpw == tpw && v.wr == wr && v.wk == wk) return &v;
    return nullptr;
}

int variant_index(const Variant *v) { return v ? static_cast<int>(v - kVariants) : -1; }

}  // namespace owl
