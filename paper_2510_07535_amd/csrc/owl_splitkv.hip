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
// Data movement: K/V go from HBM straight into LDS with 128-bit
// global_load_lds (no VGPR staging), one 16-token page per wavefront and
// stage, 64 tokens per stage, in a ring of up to 4 stages that is kept full
// ahead of the compute; readiness is tracked with vmcnt and one barrier per
// stage.
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

// 16 bytes per lane from global memory straight into LDS: lane l's data lands
// at lds_addr + 16*l.  lds_addr must be uniform over the wavefront.
__device__ __forceinline__ void dma16(const void *gptr, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n"
                 :
                 : "s"(lds_addr), "v"(gptr)
                 : "memory", "m0");
}

// Wait until at most N of this wavefront's vector-memory loads are in flight.
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
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

// Geometry of one instantiation.
template <typename T, int D, int TPW, int WR, int WK>
struct Geo {
    static constexpr bool kF32 = std::is_same<T, float>::value;
    static constexpr int ES = sizeof(T);
    static constexpr int KSTEPS = 2;                    // 32-key steps per stage
    static constexpr int SK = 32 * KSTEPS;              // keys per stage: one page per wave
    static constexpr int ROWB = D * ES;                 // bytes of one key row
    static constexpr int PPR = ROWB / 16;               // 16-byte pieces per row
    static constexpr int RPI = 1024 / ROWB;             // key rows per DMA instruction
    static constexpr int IPP = kPage / RPI;             // DMA instructions per page and tensor
    static constexpr int LPS = 2 * IPP;                 // DMA instructions per wave and stage
    static constexpr int NT = D / 16;                   // channel tiles of O^T
    static constexpr int STAGE = SK * ROWB;             // bytes per tensor per stage
    static constexpr int NS = (8 * STAGE <= 131072) ? 4 : ((6 * STAGE <= 131072) ? 3 : 2);
    static constexpr int QREGS = kF32 ? D / 4 : D / 32; // Q fragment slots per tile
    static constexpr size_t LDS = (size_t)NS * 2 * STAGE + kMaxPagesPerSplit * 4 + 64 * 8 + 64 * 4;
    static_assert(WR * WK == 4 && (WK == 1 || WK == 2), "four wavefronts per workgroup");
    static_assert(NS * LPS < 64, "loads in flight must fit vmcnt");
    static_assert((WK - 1) * WR * TPW * (4 * (NT + 1) + 1) * 256 <= NS * 2 * STAGE,
                  "cross-wave merge buffer must fit in the stage ring");
};

template <typename T, int D, int TPW, int WR, int WK>
__global__ void __launch_bounds__(256) splitkv_kernel(const KParams p)
{
    using GEO = Geo<T, D, TPW, WR, WK>;
    constexpr bool kF32 = GEO::kF32;
    constexpr int ES = GEO::ES, KSTEPS = GEO::KSTEPS, SK = GEO::SK, ROWB = GEO::ROWB;
    constexpr int PPR = GEO::PPR, NT = GEO::NT, STAGE = GEO::STAGE, NS = GEO::NS;
    constexpr int RPI = GEO::RPI, IPP = GEO::IPP, LPS = GEO::LPS;
    constexpr int QREGS = GEO::QREGS;
    constexpr int SWZ = (PPR - 1) & 15;

    extern __shared__ __align__(16) unsigned char smem[];
    int32_t *s_pages = reinterpret_cast<int32_t *>(smem + NS * 2 * STAGE);
    uint64_t *s_anc = reinterpret_cast<uint64_t *>(s_pages + kMaxPagesPerSplit);
    int32_t *s_parent = reinterpret_cast<int32_t *>(s_anc + 64);
    const uint32_t lds0 =
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;

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

    // ---- stage issue: wave w brings page 4*s + w of the split into the ring ----
    // Lane l of DMA instruction `it` carries piece l % PPR of slot it*RPI + l / PPR.
    // K rows are stored with their 16-byte pieces XOR-permuted by the slot number
    // (the permutation is applied to the global address, the LDS side of the
    // transfer is always lane-linear), V rows as they are.  Slots past the end
    // of the split (ragged last stage only) re-read the last valid row: finite
    // data whose scores are masked out later.
    const unsigned char *kbase = static_cast<const unsigned char *>(p.k);
    const unsigned char *vbase = static_cast<const unsigned char *>(p.v);
    const int last_pgx = (pos1 - 1 - pos0) >> 4, last_slot = (pos1 - 1) & (kPage - 1);
    const int ld_piece = lane % PPR, ld_row = lane / PPR;
    const int64_t head_off = (int64_t)g * p.stride_head * ES;
    const int64_t tok_bytes = p.stride_token * ES;

    auto issue_stage = [&](int s) {
        const int buf = s % NS;
        const int pgx_raw = s * (SK / kPage) + wave;
        const int pgx = min(pgx_raw, last_pgx);
        const int slot_max = pgx_raw >= last_pgx ? last_slot : kPage - 1;
        const int64_t base = (int64_t)s_pages[pgx] * p.stride_page * ES + head_off;
        const uint32_t lds_k = lds0 + buf * 2 * STAGE + wave * kPage * ROWB;
#pragma unroll
        for (int it = 0; it < IPP; ++it) {
            const int row = it * RPI + ld_row;
            const int64_t off = base + min(row, slot_max) * tok_bytes;
            const uint32_t dst = __builtin_amdgcn_readfirstlane(lds_k + it * RPI * ROWB);
            dma16(kbase + off + ((ld_piece ^ (row & SWZ)) << 4), dst);
            dma16(vbase + off + (ld_piece << 4), dst + STAGE);
        }
    };

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

    // ---- fragment loads of one 32-key step (16-bit types) ----
    // K: 2 key tiles x D/32 contraction steps.  V: NT contiguous channels of 8
    // keys per lane, then a 16-bit transpose in registers.
    auto load_kv_frags = [&](const unsigned char *Kb, const unsigned char *Vb, uint4 (&kf)[2][QREGS],
                             uint4 (&vf)[NT]) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            const int key = kt * 16 + j;
#pragma unroll
            for (int kk = 0; kk < QREGS; ++kk)
                kf[kt][kk] = *reinterpret_cast<const uint4 *>(
                    Kb + key * ROWB + (((4 * kk + qd) ^ (key & SWZ)) << 4));
        }
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
#pragma unroll
        for (int u = 0; u < NT; ++u) {
            const uint32_t sel = (u & 1) ? 0x07060302u : 0x05040100u;
            vf[u].x = __builtin_amdgcn_perm(vraw[1][u / 2], vraw[0][u / 2], sel);
            vf[u].y = __builtin_amdgcn_perm(vraw[3][u / 2], vraw[2][u / 2], sel);
            vf[u].z = __builtin_amdgcn_perm(vraw[5][u / 2], vraw[4][u / 2], sel);
            vf[u].w = __builtin_amdgcn_perm(vraw[7][u / 2], vraw[6][u / 2], sel);
        }
    };

    // ---- fast step: no mask, fixed reference m, accumulators touched by MFMA only ----
    // p = 2^(x - m) is exact in relative terms whatever m is; with m frozen at
    // the first step's row maximum, p overflows only if a later score exceeds
    // it by more than ~100 (log2 units), which the row sum exposes afterwards.
    auto fast_step = [&](int buf, int ks) {
        if constexpr (!kF32) {
            const unsigned char *Kb = smem + buf * 2 * STAGE + ks * 32 * ROWB;
            uint4 kf[2][QREGS], vf[NT];
            load_kv_frags(Kb, Kb + STAGE, kf, vf);
            const uint4 ones = make_uint4(ones2<T>(), ones2<T>(), ones2<T>(), ones2<T>());
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < QREGS; ++kk) {
                    s0 = mfma16<T>(kf[0][kk], qf[t][kk], s0);
                    s1 = mfma16<T>(kf[1][kk], qf[t][kk], s1);
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    s0[r] = fast_exp2(__builtin_fmaf(s0[r], p.c_log2, -m[t]));
                    s1[r] = fast_exp2(__builtin_fmaf(s1[r], p.c_log2, -m[t]));
                }
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

    // ---- reference m of every row tile from one unmasked step (before the fast loop) ----
    auto init_reference = [&](int buf, int ks) {
        if constexpr (!kF32) {
            const unsigned char *Kb = smem + buf * 2 * STAGE + ks * 32 * ROWB;
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kt = 0; kt < 2; ++kt) {
                    const int key = kt * 16 + j;
#pragma unroll
                    for (int kk = 0; kk < QREGS; ++kk) {
                        const uint4 kfr = *reinterpret_cast<const uint4 *>(
                            Kb + key * ROWB + (((4 * kk + qd) ^ (key & SWZ)) << 4));
                        if (kt == 0) s0 = mfma16<T>(kfr, qf[t][kk], s0);
                        else s1 = mfma16<T>(kfr, qf[t][kk], s1);
                    }
                }
                float tm = fmaxf(fmaxf(fmaxf(s0[0], s0[1]), fmaxf(s0[2], s0[3])),
                                 fmaxf(fmaxf(s1[0], s1[1]), fmaxf(s1[2], s1[3])));
                m[t] = quad_column_max(tm) * p.c_log2;
            }
        }
    };

    // ---- careful softmax of one row tile over one 32-key step: mask + exact online rescale ----
    auto softmax_step = [&](f32x4 &s0, f32x4 &s1, int t, int step_pos) {
        if (step_pos + 32 > L) {                     // reaches drafts or the ragged end (uniform)
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
        tm = quad_column_max(tm);
        const float sc = tm * p.c_log2;
        if (__builtin_amdgcn_ballot_w64(sc > m[t]) != 0) {          // uniform over the wave
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

    // ---- careful step: any step, any type ----
    auto careful_step = [&](int buf, int ks, int step_pos) {
        const unsigned char *Kb = smem + buf * 2 * STAGE + ks * 32 * ROWB;
        const unsigned char *Vb = Kb + STAGE;
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
                    // the other 16 keys of the step come with the next kt: give
                    // the softmax a fully masked second half
                    f32x4 s1 = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
                    softmax_step(s0, s1, t, step_pos + kt * 16);
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
            uint4 kf[2][QREGS], vf[NT];
            load_kv_frags(Kb, Vb, kf, vf);
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
                softmax_step(s0, s1, t, step_pos);
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

    // ---- stage loop skeleton: keep NS-1 stages in flight ahead of the one computed ----
    int issued = 0;
    auto wait_stage = [&](int s) {
        // stage s has landed once at most (younger stages) * LPS loads remain
        const int ahead = issued - (s + 1);
        if (NS > 3 && ahead >= 3) wait_vmcnt<(NS > 3 ? 3 : 0) * LPS>();
        else if (NS > 2 && ahead == 2) wait_vmcnt<(NS > 2 ? 2 : 0) * LPS>();
        else if (NS > 1 && ahead == 1) wait_vmcnt<LPS>();
        else wait_vmcnt<0>();
    };
    auto run_stages = [&](int s_begin, int s_end, auto fast_tag) {
        for (int s = s_begin; s < s_end; ++s) {
            wait_stage(s);
            __syncthreads();     // everyone's part of stage s is in; stage s-1 is fully consumed
            if (issued < nstages && issued <= s + NS - 1) {
                issue_stage(issued);                // refills the slot stage s-1 occupied
                ++issued;
            }
            const int sbase = pos0 + s * SK;
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                if (ks % WK != wk) continue;
                if constexpr (decltype(fast_tag)::value) {
                    fast_step(s % NS, ks);
                } else {
                    if (sbase + ks * 32 >= pos1) continue;   // uniform: nothing left in this step
                    careful_step(s % NS, ks, sbase + ks * 32);
                }
            }
        }
    };

    // ---- software-pipelined fast loop (two or more row tiles per wave) ----
    // The wave walks its 32-key steps tile by tile; slot (step j, tile t) holds
    // three mutually independent pieces so that the matrix pipe and the vector
    // ALU can run side by side inside ONE wavefront:
    //     MFMA : O[prev tile] += V^T P(prev)      and   S(next tile) = K Q^T
    //     VALU : P(this tile) = 2^(S - m), packed to bf16
    //     LDS  : K fragments / raw V rows of the NEXT step
    // "next" wraps into the following step (whose K fragments sit in the other
    // half of a double buffer), so the pipeline never drains inside the loop.
    // The barrier that admits stage s+1 is taken at the start of the last step
    // this wave has in stage s; by then all of the wave's LDS reads of stage s
    // have completed, so stage s+NS is issued into that slot right away.
    auto run_fast_pipelined = [&](int n_fast) {
        if constexpr (!kF32 && TPW >= 2) {
            const int J = (WK == 2) ? n_fast : 2 * n_fast;       // this wave's steps
            auto step_base = [&](int jj) -> const unsigned char * {
                const int sj = (WK == 2) ? jj : (jj >> 1);
                const int ks = (WK == 2) ? wk : (jj & 1);
                return smem + (sj % NS) * 2 * STAGE + ks * 32 * ROWB;
            };
            auto load_k = [&](const unsigned char *Kb, uint4 (&kf)[2][QREGS]) {
#pragma unroll
                for (int kt = 0; kt < 2; ++kt) {
                    const int key = kt * 16 + j;
#pragma unroll
                    for (int kk = 0; kk < QREGS; ++kk)
                        kf[kt][kk] = *reinterpret_cast<const uint4 *>(
                            Kb + key * ROWB + (((4 * kk + qd) ^ (key & SWZ)) << 4));
                }
            };
            auto load_vraw = [&](const unsigned char *Vb, uint32_t (&vraw)[8][NT / 2]) {
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
            };
            auto make_vf = [&](const uint32_t (&vraw)[8][NT / 2], uint4 (&vf)[NT]) {
#pragma unroll
                for (int u = 0; u < NT; ++u) {
                    const uint32_t sel = (u & 1) ? 0x07060302u : 0x05040100u;
                    vf[u].x = __builtin_amdgcn_perm(vraw[1][u / 2], vraw[0][u / 2], sel);
                    vf[u].y = __builtin_amdgcn_perm(vraw[3][u / 2], vraw[2][u / 2], sel);
                    vf[u].z = __builtin_amdgcn_perm(vraw[5][u / 2], vraw[4][u / 2], sel);
                    vf[u].w = __builtin_amdgcn_perm(vraw[7][u / 2], vraw[6][u / 2], sel);
                }
            };
            auto scores = [&](const uint4 (&kf)[2][QREGS], int t, f32x4 &s0, f32x4 &s1) {
                s0 = f32x4{0.f, 0.f, 0.f, 0.f};
                s1 = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < QREGS; ++kk) {
                    s0 = mfma16<T>(kf[0][kk], qf[t][kk], s0);
                    s1 = mfma16<T>(kf[1][kk], qf[t][kk], s1);
                }
            };
            const uint4 ones = make_uint4(ones2<T>(), ones2<T>(), ones2<T>(), ones2<T>());

            uint4 kfA[2][QREGS], kfB[2][QREGS], vf[NT];
            uint32_t vraw[8][NT / 2];
            f32x4 sn0, sn1;
            uint4 pprev = make_uint4(0, 0, 0, 0);

            // prologue: one more stage in flight than the plain loop keeps, the
            // first step's fragments, the frozen reference, S of the first slot
            if (issued < nstages) {
                issue_stage(issued);
                ++issued;
            }
            wait_stage(0);
            __syncthreads();
            load_k(step_base(0), kfA);
            load_vraw(step_base(0) + STAGE, vraw);
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                scores(kfA, t, sn0, sn1);
                const float tm = fmaxf(fmaxf(fmaxf(sn0[0], sn0[1]), fmaxf(sn0[2], sn0[3])),
                                       fmaxf(fmaxf(sn1[0], sn1[1]), fmaxf(sn1[2], sn1[3])));
                m[t] = quad_column_max(tm) * p.c_log2;
            }
            scores(kfA, 0, sn0, sn1);
            make_vf(vraw, vf);       // placeholder operand for the first (all-zero P) slot

            auto do_step = [&](int jj, uint4 (&kf_cur)[2][QREGS], uint4 (&kf_nxt)[2][QREGS]) {
                const int jn = min(jj + 1, J - 1);
                const int s_cur = (WK == 2) ? jj : (jj >> 1), s_nxt = (WK == 2) ? jn : (jn >> 1);
                if (s_nxt != s_cur) {                            // uniform over the workgroup
                    __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0): my LDS reads are done
                    wait_stage(s_nxt);
                    __syncthreads();
                    if (issued < nstages) {
                        issue_stage(issued);                     // into the slot of stage s_cur
                        ++issued;
                    }
                }
                const unsigned char *Kn = step_base(jn);
#pragma unroll
                for (int t = 0; t < TPW; ++t) {
                    const f32x4 c0 = sn0, c1 = sn1;
                    constexpr int kNone = 0;
                    (void)kNone;
                    const int tp = (t + TPW - 1) % TPW;
                    // MFMA: PV of the previous slot
#pragma unroll
                    for (int u = 0; u < NT; ++u) O[tp][u] = mfma16<T>(vf[u], pprev, O[tp][u]);
                    O[tp][NT] = mfma16<T>(ones, pprev, O[tp][NT]);
                    if (t == 0) make_vf(vraw, vf);               // this step's V^T fragments
                    // MFMA: scores of the next slot
                    if (t + 1 < TPW) scores(kf_cur, t + 1, sn0, sn1);
                    else scores(kf_nxt, 0, sn0, sn1);
                    // VALU: probabilities of this slot
                    float e0[4], e1[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        e0[r] = fast_exp2(__builtin_fmaf(c0[r], p.c_log2, -m[t]));
                        e1[r] = fast_exp2(__builtin_fmaf(c1[r], p.c_log2, -m[t]));
                    }
                    pprev.x = pack2<T>(e0[0], e0[1]);
                    pprev.y = pack2<T>(e0[2], e0[3]);
                    pprev.z = pack2<T>(e1[0], e1[1]);
                    pprev.w = pack2<T>(e1[2], e1[3]);
                    // LDS: fragments of the next step
                    if (t == 0) {
                        load_k(Kn, kf_nxt);
                        load_vraw(Kn + STAGE, vraw);
                    }
                }
            };
            for (int jj = 0; jj < J; jj += 2) {
                do_step(jj, kfA, kfB);
                if (jj + 1 < J) do_step(jj + 1, kfB, kfA);
            }
            // drain: PV of the very last slot
#pragma unroll
            for (int u = 0; u < NT; ++u) O[TPW - 1][u] = mfma16<T>(vf[u], pprev, O[TPW - 1][u]);
            O[TPW - 1][NT] = mfma16<T>(ones, pprev, O[TPW - 1][NT]);
        }
    };

    // The Q fragments must have arrived before the first DMA is issued: from
    // here on vmcnt counts DMA stages only.
    wait_vmcnt<0>();

    // Pass 0: stages that lie wholly inside the prefix run the fast step with a
    // frozen reference; the rest (drafts, ragged end) run the careful step.
    // Pass 1 happens only if a row sum of pass 0 is not a modest finite number:
    // the whole split is redone with the careful step.  bf16 only: an fp16 P
    // cannot hold 2^(x - m) for a stale m, fp32 is the small correctness shape.
    constexpr bool kHasFast = std::is_same<T, __bf16>::value;
    for (int pass = 0; pass < 2; ++pass) {
        issued = 0;
        for (; issued < NS - 1 && issued < nstages; ++issued) issue_stage(issued);
        int n_fast = 0;
        if (kHasFast && pass == 0) n_fast = max(0, min(nstages, (L - pos0) / SK));
        if (n_fast > 0) {
            if constexpr (TPW >= 2) {
                run_fast_pipelined(n_fast);
            } else {
                wait_stage(0);
                __syncthreads();
                init_reference(0, wk);
                run_stages(0, n_fast, std::true_type{});
            }
        }
        run_stages(n_fast, nstages, std::false_type{});
        if (!kHasFast || pass == 1) break;
        bool bad = false;
#pragma unroll
        for (int t = 0; t < TPW; ++t) bad |= !(O[t][NT][0] < 1.0e30f);
        if (!__syncthreads_or(bad ? 1 : 0)) break;
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            m[t] = kMInit;
#pragma unroll
            for (int u = 0; u <= NT; ++u) O[t][u] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }

    // ---- merge the key groups of a row group through LDS (reuses the ring) ----
    if constexpr (WK > 1) {
        __syncthreads();
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
// A one-wavefront check of quad_column_max's lane semantics (test hook).
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(64) quad_max_kernel(const float *in, float *out)
{
    out[threadIdx.x] = quad_column_max(in[threadIdx.x]);
}

hipError_t launch_quad_max(const float *in, float *out, hipStream_t s)
{
    hipLaunchKernelGGL(quad_max_kernel, dim3(1), dim3(64), 0, s, in, out);
    return hipGetLastError();
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
    OWL_VARIANT(DT, T, D, 1, 2, 2), OWL_VARIANT(DT, T, D, 2, 2, 2),                     \
    OWL_VARIANT(DT, T, D, 2, 4, 1), OWL_VARIANT(DT, T, D, 3, 4, 1),                     \
    OWL_VARIANT(DT, T, D, 4, 4, 1), OWL_VARIANT(DT, T, D, 5, 4, 1)

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
