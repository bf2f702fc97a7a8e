// Split-KV pass of the verify-step attention for gfx950 (MI355X).
//
// One workgroup (8 wavefronts, two per SIMD) owns one (sequence, KV head, KV
// split, row group).  It streams its split of the paged K/V cache through LDS
// exactly once and holds, in MFMA accumulators, the un-normalised outputs of
// ALL query rows that share this KV head: rows = (draft node i, query head
// within the group), R = (Hq/Hkv) * N of them, cut into 16-row tiles that are
// dealt out to the wavefronts.  That packing is what makes the cost of
// verifying N drafted tokens "hidden" behind the scan of the context (Sec. 1 /
// Sec. 2 of the paper): the cache is read once whatever N is.
//
// Data movement: K/V go from HBM straight into LDS with 128-bit
// global_load_lds (no VGPR staging), one 16-token page of one tensor per
// wavefront and stage, 64 tokens per stage, in a ring of up to 4 stages (K
// stages in the lower half of the ring, V stages behind them) that is kept
// full ahead of the compute; readiness is tracked with vmcnt and one barrier
// per stage.
//
// Three loops share the ring: the pipelined fast loop (unmasked steps, up to
// two tiles per wave: matrix, vector and LDS work of neighbouring steps woven
// into one instruction stream), the plain fast loop (three tiles per wave, and
// the layout with two key groups: scores -> softmax -> V^T P per step, the two
// waves of a SIMD overlapping each other), and the careful loop (masked or
// ragged steps, exact online softmax; also the fallback when a frozen softmax
// reference overflowed).
//
// Tile algebra (all MFMA tiles are 16x16, wave64):
//   S^T[key][row] = K[key][:] . Q[row][:]        A = K fragment, B = Q fragment
//   O^T[d][row]  += V^T[d][key] * P^T[key][row]  A = V^T fragment, B = P fragment
// With keys along M, a lane owns ONE query row (column lane%16) and the keys of
// a tile sit in its registers, so the fp32 S^T accumulators turn into the bf16
// P^T operand in place.  K/Q take channels 32*kk + 8*quad + e (the order of the
// contraction index is free as long as both operands agree).  V^T fragments
// come from ds_read_b64_tr_b16, the transposing LDS read: in a block of 16
// lanes, lane i receives element i%4 of the 8 bytes addressed by lanes
// 4e + i/4 (e = 0..3); with lane 4e+c pointing at channels 4c..4c+3 of key e,
// lane i ends up with channel i of four keys.  The row sum l rides along as
// one more channel tile whose V^T operand is all ones, so it is summed from the
// very P values (after rounding to bf16) that weigh V.
//
// Visibility (Sec. 3.2.2, Decode Stage): every row sees the whole prefix; among
// the drafts, row (i, .) sees node j iff j is on i's root path, i included.
// Only 32-key steps that reach past the prefix take the masked ("careful") path.
#include <hip/hip_ext.h>

#include <type_traits>

#include "owl_device.h"

namespace owl {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 512;        // 8 wavefronts
constexpr int kWaves = kThreads / 64;
constexpr float kMInit = -1.0e30f;   // "no key seen yet"; finite so that m - m is 0

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
// at lds_addr + 16*l.  lds_addr must be uniform over the wavefront.  K and V are
// read exactly once, so the transfer is marked non-temporal (`nt`): the lines are
// not kept in L2 or the memory-side cache, which leaves those to the queries, the
// page lists and the partials, and makes the 32K chain step 10 % shorter (the
// 128K tree step 2.5 %); the scope bits of the instruction make no difference.
#define OWL_DMA_POLICY " nt"
__device__ __forceinline__ void dma16(const void *gptr, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" OWL_DMA_POLICY "\n"
                 :
                 : "s"(lds_addr), "v"(gptr)
                 : "memory", "m0");
}

// The same with a wave-uniform 64-bit base and a 32-bit per-lane byte offset.
__device__ __forceinline__ void dma16s(uint64_t sbase, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" OWL_DMA_POLICY "\n"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(sbase)
                 : "memory", "m0");
}

// Wait until at most N of this wavefront's vector-memory loads are in flight.
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// Transposing 64-bit LDS read (see the file comment for the lane mapping).
__device__ __forceinline__ uint2 lds_read_tr16(const unsigned char *p)
{
    const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (s16x4 __attribute__((address_space(3))) *)(p));
    return __builtin_bit_cast(uint2, v);
}

// f(integral_constant<int, B>) ... f(integral_constant<int, E-1>), unrolled at compile time.
template <int B, int E, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

// Geometry of one instantiation.
template <typename T, int D, int TPW, int WR, int WK>
struct Geo {
    static constexpr bool kF32 = std::is_same<T, float>::value;
    static constexpr int ES = sizeof(T);
    static constexpr int KSTEPS = 2;                    // 32-key steps per stage
    static constexpr int SK = 32 * KSTEPS;              // keys per stage: 4 pages x 2 tensors = 8 waves
    static constexpr int ROWB = D * ES;                 // bytes of one key row
    static constexpr int PPR = ROWB / 16;               // 16-byte pieces per row
    static constexpr int RPI = 1024 / ROWB;             // key rows per DMA instruction
    static constexpr int LPS = kPage / RPI;             // DMA instructions per wave and stage
    static constexpr int NT = D / 16;                   // channel tiles of O^T
    static constexpr int STAGE = SK * ROWB;             // bytes per tensor per stage
    static constexpr int NS = (8 * STAGE <= 131072) ? 4 : ((6 * STAGE <= 131072) ? 3 : 2);
    static constexpr int VREG = NS * STAGE;             // LDS ring: K stages at [0, VREG), V stages behind them
    static constexpr int QREGS = kF32 ? D / 4 : D / 32; // Q fragment slots per tile
    static constexpr int KSWZ = (PPR - 1) & 15;         // K rows: piece ^= key & KSWZ
    static constexpr int VSWM = PPR >= 16 ? 7 : PPR / 2 - 1;   // V rows: piece ^= (key & VSWM) << 1
    static constexpr size_t LDS = (size_t)NS * 2 * STAGE + kMaxPagesPerSplit * 4 + 64 * 8 + 64 * 4;
    static_assert(WR * WK == kWaves && (WK == 1 || WK == 2), "eight wavefronts per workgroup");
    static_assert(NS * LPS < 64, "loads in flight must fit vmcnt");
    static_assert((WK - 1) * WR * TPW * (4 * (NT + 1) + 1) * 256 <= NS * 2 * STAGE,
                  "cross-wave merge buffer must fit in the stage ring");
};

template <typename T, int D, int TPW, int WR, int WK, bool TL>
__global__ void __launch_bounds__(kThreads) splitkv_kernel(const KParams p)
{
    using GEO = Geo<T, D, TPW, WR, WK>;
    constexpr bool kF32 = GEO::kF32;
    constexpr int ES = GEO::ES, KSTEPS = GEO::KSTEPS, SK = GEO::SK, ROWB = GEO::ROWB;
    constexpr int PPR = GEO::PPR, NT = GEO::NT, STAGE = GEO::STAGE, NS = GEO::NS;
    constexpr int RPI = GEO::RPI, LPS = GEO::LPS, QREGS = GEO::QREGS;
    constexpr int KSWZ = GEO::KSWZ, VSWM = GEO::VSWM, VREG = GEO::VREG;
    constexpr int KQ = kF32 ? 1 : QREGS;             // K/Q fragment slots of the 16-bit paths

    extern __shared__ __align__(16) unsigned char smem[];
    int32_t *s_pages = reinterpret_cast<int32_t *>(smem + NS * 2 * STAGE);
    uint64_t *s_anc = reinterpret_cast<uint64_t *>(s_pages + kMaxPagesPerSplit);
    int32_t *s_parent = reinterpret_cast<int32_t *>(s_anc + 64);
    const uint32_t lds0 =
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave % WR, wk = wave / WR;
    const int j = lane & 15, qd = lane >> 4;

    // Workgroups go to the chip's eight XCDs round-robin in launch order, whether or not
    // they have work.  KV heads (all with the same amount of work) vary fastest, so that
    // splits that do not exist for a short sequence do not leave whole XCDs idle.
    // n numbers the workgroups in launch order; a "stream" is one (KV head, split, sequence).
    // Row groups (workgroups that take different row tiles of the same stream, each reading its
    // K/V) are laid out so that the groups of a stream follow each other on ONE XCD: stream u sits
    // on XCD u mod 8, its groups in consecutive slots of that XCD, and all but the first find the
    // split in that XCD's L2.  With a single row group this is the plain order (n = u).
    // (the host keeps the workgroup count of a launch below 2^31)
    uint32_t n = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    int rg = 0;
    if (p.row_groups > 1) {                          // the host pads the stream count to a multiple of 8
        const uint32_t slot = n >> 3;
        rg = (int)(slot % (uint32_t)p.row_groups);
        n = ((slot / (uint32_t)p.row_groups) << 3) | (n & 7);
    }
    const int g = (int)(n % (uint32_t)p.Hkv);
    const uint32_t item = n / (uint32_t)p.Hkv;       // (split, sequence), split fastest
    int c = (int)(item % gridDim.y);
    int b = (int)(item / gridDim.y);
    if (p.adapt != 2 && b >= p.B) return;            // cannot happen with the grids the host launches

    // timeline of this workgroup (profiling instantiations only; the production kernels
    // carry neither the pointer nor a branch)
    long long *tl = nullptr;
    if constexpr (TL) {
        const long long flat = blockIdx.x + (long long)gridDim.x * (blockIdx.y + (long long)gridDim.y * blockIdx.z);
        tl = p.timeline + 10 * flat;
        if (tid == 0) {
            tl[0] = wall_clock64();
            tl[1] = tl[2] = tl[3] = tl[4] = tl[5] = tl[8] = tl[9] = 0;
            // XCC_ID register (bits 3:0) above the shader-engine / CU id: one value per compute unit
            tl[6] = ((long long)(__builtin_amdgcn_s_getreg((3 << 11) | 20) & 15) << 16) | __smid();
            tl[7] = flat;
        }
    }
    auto stamp = [&](int k) {
        if constexpr (TL) {
            if (tid == 0) {
                tl[k] = wall_clock64();
                if (k == 2) tl[8] = clock64();        // shader cycles at both ends of the fast loop:
                if (k == 3) tl[9] = clock64();        // their rate is the clock the chip really ran at
            }
        }
    };

    // ---- everything that does not depend on the context length is requested
    // first, so that all of the kernel's set-up reads are in flight together:
    // raw page-table entries of this split's window, the parent array, Q ----
    int C = p.C;                                      // revised below once the context length is known
    if (p.adapt == 2) {                               // a batch: the split size follows all its lengths
        C = p.dev_c[0];                               // derived by the plan kernel that precedes this launch
        C = min(max(C / kSplitQuantum, 1) * kSplitQuantum, p.C);
        // (y, z) is only a number here: the items that exist are the first ones in launch order
        if (item >= (uint32_t)p.item_slots || !batch_item(p, (int)item, &b, &c)) return;
    }
    int pos0 = c * C;
    // drafted tokens of this sequence (a batch may mix tree sizes): rows of nodes >= Nb are
    // idle, their K/V rows are not part of the sequence, and the combine writes zeros for them
    const int Nb = load_n_draft(p.n_draft_seq, b, p.N, p.dev_status);
    if (Nb == 0) return;
    // The context length is requested before everything else: vector loads complete in
    // order, so asked for after the query fragments it would only arrive behind them
    // (2.4 us later with 15-20 row tiles), and the whole prologue hangs on it.
    const int L = load_ctx_len(p.ctx_lens, b, p.max_ctx_len, p.dev_status);
    int raw_page[kMaxPagesPerSplit / kThreads];
    auto request_pages = [&]() {
        const int win_pages = C / kPage;             // pages a full split spans (<= kMaxPagesPerSplit)
#pragma unroll
        for (int r = 0; r < kMaxPagesPerSplit / kThreads; ++r) {
            const int idx = tid + r * kThreads, lp = pos0 / kPage + idx;
            raw_page[r] = -1;
            if (idx < win_pages) {
                if (!p.page_table) raw_page[r] = lp;
                else if (lp < p.max_pages) raw_page[r] = p.page_table[(int64_t)b * p.max_pages + lp];
            }
        }
    };
    request_pages();
    if (tid < p.N) s_parent[tid] = p.parent[(int64_t)b * p.N + tid];
    // ---- this wave's query rows: tiles wr, wr + WR, ... of the row group ----
    uint4 qf[TPW][KQ];
    float qs[TPW][kF32 ? QREGS : 1];
    int irow[TPW];
    int my_nt = 0;
    // Requested only after the first K/V stage (below): the query fragments of all workgroups of
    // a KV head are the same few L2 lines, they take ~2 us to come in with 15-20 row tiles, and
    // vector loads complete in order, so the first stage's DMA would queue up behind them.
    auto load_queries = [&]() {
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
        const int tg = rg * p.group_tiles + t * WR + wr;
        const bool tile_ok = t * WR + wr < p.group_tiles && tg < p.RT;
        my_nt += tile_ok ? 1 : 0;
        const int row = tg * kRowTile + j;
        const bool ok = tile_ok && row < p.R && row / p.G < Nb;
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
    my_nt = __builtin_amdgcn_readfirstlane(my_nt);
    };

    const int Ttot = L + Nb;
    if (p.adapt == 1 && split_tokens_for(p, Ttot) != C) {   // uniform: a context shorter than planned for
        C = split_tokens_for(p, Ttot);
        pos0 = c * C;
        request_pages();                            // the window moved: one more round trip
    }
    if (pos0 >= Ttot) return;                       // this split does not exist for b
    const int pos1 = min(pos0 + C, Ttot);
    const int nstages = (pos1 - pos0 + SK - 1) / SK;

    // ---- page list of this split (validated now that its extent is known),
    // and the tree mask if drafts are in reach ----
    {
        const int npg = (pos1 - pos0 + kPage - 1) / kPage;
#pragma unroll
        for (int r = 0; r < kMaxPagesPerSplit / kThreads; ++r) {
            const int idx = tid + r * kThreads;
            if (idx < npg) {
                int pg = raw_page[r];
                if (pg < 0 || pg >= p.n_pool_pages) {    // also: logical page beyond the table
                    flag_status(p.dev_status, OWL_DEV_BAD_PAGE);
                    pg = 0;
                }
                s_pages[idx] = pg;
            }
        }
    }
    const bool has_drafts = pos1 > L;               // uniform over the workgroup
    __syncthreads();
    if (has_drafts) {
        if (tid < Nb) s_anc[tid] = ancestor_set(s_parent, tid, nullptr, p.dev_status);
        __syncthreads();
    }
    stamp(1);

    // ---- stage issue ----
    // Wave w brings one 16-token page of one tensor per stage: tensor w/4 (K, V),
    // page 4*s + w%4 of the split.  Lane l of DMA instruction `it` carries piece
    // l % PPR of slot it*RPI + l / PPR.  The 16-byte pieces of a row are stored
    // XOR-permuted by the slot number (K: piece ^ slot, V: piece ^ 2*(slot%8)) so
    // that the fragment reads below are bank-conflict free; the permutation is
    // applied to the global address, the LDS side of the transfer is always
    // lane-linear.  Slots past the end of the split (ragged last stage only)
    // re-read the last valid row: finite data whose scores are masked out later.
    const int ld_tensor = wave >> 2, ld_page = wave & 3;
    const unsigned char *ld_base = static_cast<const unsigned char *>(ld_tensor ? p.v : p.k);
    const int last_pgx = (pos1 - 1 - pos0) >> 4, last_slot = (pos1 - 1) & (kPage - 1);
    const int ld_piece = lane % PPR, ld_row = lane / PPR;
    const int64_t head_off = (int64_t)g * p.stride_head * ES;
    const int64_t tok_bytes = p.stride_token * ES;

    // A whole page (every stage but the split's last page) needs no clamping:
    // the lane's byte offsets inside the page are fixed, only the page base
    // (wave-uniform, kept in scalar registers) changes from stage to stage.
    constexpr bool kKeepLdOff = TPW <= 2;            // three tiles per wave: no registers to spare, recompute
    auto ld_off_of = [&](int it) -> uint32_t {
        const int row = it * RPI + ld_row;
        const int swz = ld_tensor ? ((row & VSWM) << 1) : (row & KSWZ);
        return (uint32_t)(row * tok_bytes) + (uint32_t)((ld_piece ^ swz) << 4);
    };
    uint32_t ld_off[LPS];
#pragma unroll
    for (int it = 0; it < LPS; ++it) ld_off[it] = kKeepLdOff ? ld_off_of(it) : 0u;
    const bool ld_off_ok = tok_bytes * kPage < ((int64_t)1 << 31);
    const uint32_t ld_lds = lds0 + ld_tensor * VREG + ld_page * kPage * ROWB;

    // page id of this wave's page of stage s (to be handed to issue_stage; reading it
    // ahead of the stage barrier takes the LDS round trip off the issue path)
    auto stage_page = [&](int s) -> int { return s_pages[min(s * (SK / kPage) + ld_page, last_pgx)]; };
    auto issue_stage_pg = [&](int s, int pg_lane) {
        const int buf = s % NS;
        const int pgx_raw = s * (SK / kPage) + ld_page;
        const uint32_t lds_dst = ld_lds + buf * STAGE;
        if (pgx_raw < last_pgx && ld_off_ok) {           // uniform over the wave
            const int64_t pg = __builtin_amdgcn_readfirstlane(pg_lane);
            const uint64_t sb = (uint64_t)(uintptr_t)ld_base + (uint64_t)(pg * p.stride_page * ES + head_off);
            const uint64_t sbase = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(sb >> 32)) << 32) |
                                   (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)sb);
#pragma unroll
            for (int it = 0; it < LPS; ++it)
                dma16s(sbase, kKeepLdOff ? ld_off[it] : ld_off_of(it),
                       __builtin_amdgcn_readfirstlane(lds_dst + it * RPI * ROWB));
            return;
        }
        const int slot_max = pgx_raw >= last_pgx ? last_slot : kPage - 1;
        const int64_t base = (int64_t)pg_lane * p.stride_page * ES + head_off;
#pragma unroll
        for (int it = 0; it < LPS; ++it) {
            const int row = it * RPI + ld_row;
            const int64_t off = base + min(row, slot_max) * tok_bytes;
            const int swz = ld_tensor ? ((row & VSWM) << 1) : (row & KSWZ);
            dma16(ld_base + off + ((ld_piece ^ swz) << 4),
                  __builtin_amdgcn_readfirstlane(lds_dst + it * RPI * ROWB));
        }
    };
    auto issue_stage = [&](int s) { issue_stage_pg(s, stage_page(s)); };

    f32x4 O[TPW][NT + 1];
    float m[TPW];
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
        m[t] = kMInit;
#pragma unroll
        for (int u = 0; u <= NT; ++u) O[t][u] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // ---- lane-constant parts of the fragment addresses (16-bit types) ----
    // K fragment (kt, kk): 16 bytes at key kt*16 + j, piece (4*kk + quad) ^ (j & KSWZ).
    // V^T fragment (u, h): transposing read; lane 4e + c of block `quad` points at
    // key 16*h + 4*quad + e, channels 16*u + 4*c .. +3.
    const int v_e = j >> 2, v_c = j & 3;
    const int v_key0 = 4 * qd + v_e;
    const int v_swz = (v_key0 & VSWM) << 1;
    const int v_lane_off = v_key0 * ROWB + (v_c & 1) * 8;

    // ---- K fragments of one 32-key step ----
    auto load_k_frags = [&](const unsigned char *Kb, uint4 (&kf)[2][KQ]) {
        if constexpr (!kF32) {
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                const int key = kt * 16 + j;
#pragma unroll
                for (int kk = 0; kk < KQ; ++kk)
                    kf[kt][kk] = *reinterpret_cast<const uint4 *>(
                        Kb + key * ROWB + (((4 * kk + qd) ^ (key & KSWZ)) << 4));
            }
        }
    };
    // ---- V^T fragment of channel tile u for the 32 keys of a step ----
    auto load_v_frag = [&](const unsigned char *Vb, int u) -> uint4 {
        const unsigned char *a = Vb + v_lane_off + ((((2 * u) ^ v_swz) | (v_c >> 1)) << 4);
        const uint2 lo = lds_read_tr16(a);
        const uint2 hi = lds_read_tr16(a + 16 * ROWB);
        return make_uint4(lo.x, lo.y, hi.x, hi.y);
    };

    // ---- fast step: no mask, fixed reference m, accumulators touched by MFMA only ----
    // fp16 storage: a workgroup whose first step shows a wide spread of scores takes the plain loop
    // with a guarded reference (see fast_sx) instead of the frozen one; the choice only affects
    // speed (a frozen reference that overflows is caught by the row sums and the split redone)
    constexpr bool kGuard = std::is_same<T, _Float16>::value;
    bool use_guard = false;
    // p = 2^(x - m) is exact in relative terms whatever m is; with m frozen at
    // the first step's row maximum, p overflows only if a later score exceeds
    // it by more than ~100 (log2 units), which the row sum exposes afterwards.
    // A step is cut in two: scores + softmax -> P (fast_sx), and O += V^T P with
    // the V^T fragments already in registers (fast_pv), so that the stage loop
    // can put a barrier between them.
    auto fast_sx = [&](const unsigned char *Kb, const unsigned char *Vb, uint4 (&pf)[TPW], uint4 (&vf)[NT],
                       auto ntag, auto gtag) {
        constexpr int NA = decltype(ntag)::value;    // tiles this wave really owns
        constexpr bool kGuarded = decltype(gtag)::value;
        if constexpr (!kF32 && NA > 0) {
            // The score -> softmax -> P chain is the latency-critical part of a step; O += V^T P
            // is throughput work without dependents.  Raising this wave's priority for the
            // first and dropping it for the second lets the other wave of the SIMD fill the
            // gaps of the chain with its PV MFMAs (13 % fewer cycles in the three-tile loop).
            __builtin_amdgcn_s_setprio(1);
            uint4 kf[2][KQ];
            load_k_frags(Kb, kf);
#pragma unroll
            for (int t = 0; t < NA; ++t) {
                f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < KQ; ++kk) {
                    s0 = mfma16<T>(kf[0][kk], qf[t][kk], s0);
                    s1 = mfma16<T>(kf[1][kk], qf[t][kk], s1);
                }
                if constexpr (kGuarded) {
                    // fp16 holds 2^(x - m) only up to 2^16.  The reference stays frozen as long as no
                    // score of the step comes within 2^5 of that; a row that does moves its reference
                    // 4 above the offender and rescales its accumulators (rare; uniform branch).
                    const float tm = fmaxf(fmaxf(fmaxf(s0[0], s0[1]), fmaxf(s0[2], s0[3])),
                                           fmaxf(fmaxf(s1[0], s1[1]), fmaxf(s1[2], s1[3])));
                    // detection needs no cross-lane step: any lane's own keys can raise the alarm
                    if (__builtin_amdgcn_ballot_w64(__builtin_fmaf(tm, p.c_log2, -m[t]) > 11.0f) != 0) {
                        const float sc = quad_column_max(tm) * p.c_log2;
                        const float mn = sc > m[t] + 11.0f ? sc + 4.0f : m[t];
                        const float alpha = fast_exp2(m[t] - mn);
                        m[t] = mn;
#pragma unroll
                        for (int u = 0; u <= NT; ++u) O[t][u] *= alpha;
                    }
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    s0[r] = fast_exp2(__builtin_fmaf(s0[r], p.c_log2, -m[t]));
                    s1[r] = fast_exp2(__builtin_fmaf(s1[r], p.c_log2, -m[t]));
                }
                pf[t].x = pack2<T>(s0[0], s0[1]);
                pf[t].y = pack2<T>(s0[2], s0[3]);
                pf[t].z = pack2<T>(s1[0], s1[1]);
                pf[t].w = pack2<T>(s1[2], s1[3]);
            }
#pragma unroll
            for (int u = 0; u < NT; ++u) vf[u] = load_v_frag(Vb, u);
        }
    };
    auto fast_pv = [&](const uint4 (&pf)[TPW], const uint4 (&vf)[NT], auto ntag) {
        constexpr int NA = decltype(ntag)::value;
        if constexpr (!kF32 && NA > 0) {
            __builtin_amdgcn_s_setprio(0);
            const uint4 ones = make_uint4(ones2<T>(), ones2<T>(), ones2<T>(), ones2<T>());
#pragma unroll
            for (int u = 0; u < NT; ++u) {
#pragma unroll
                for (int t = 0; t < NA; ++t) O[t][u] = mfma16<T>(vf[u], pf[t], O[t][u]);
            }
#pragma unroll
            for (int t = 0; t < NA; ++t) O[t][NT] = mfma16<T>(ones, pf[t], O[t][NT]);
        }
    };

    // ---- pipelined fast loop (WK == 1, up to two tiles per wave) ----
    // Iteration i runs three mutually independent instruction streams over
    // 32-key steps: the matrix stream does O += V^T P of step i-1 and the
    // scores of step i+1, the vector stream turns the scores of step i into P
    // (fma, exp2, pack), and the LDS stream fetches each K / V^T fragment PF
    // MFMA groups before its use (one group = one fragment's MFMAs for all tiles
    // of the wave).  The streams are woven together group by group, with a
    // scheduling fence after every group so that the order written here is the
    // order issued: a wave can issue only one instruction every few cycles, so
    // what keeps the matrix pipe busy is a short, evenly mixed stream per wave.
    // Ring offsets are compile-time (the stage loop is unrolled over the ring)
    // and travel in the LDS instructions' offset fields: no address arithmetic
    // is left in the loop.
    constexpr bool kPipe = !kF32 && WK == 1 && TPW <= 2;      // three tiles: not enough registers
    constexpr int PF = 3;                                      // fragment prefetch distance (groups, <= NT)
    uint32_t k_off[KQ], v_off[NT];
    if constexpr (kPipe) {
#pragma unroll
        for (int kk = 0; kk < KQ; ++kk) k_off[kk] = j * ROWB + (((4 * kk + qd) ^ (j & KSWZ)) << 4);
#pragma unroll
        for (int u = 0; u < NT; ++u) v_off[u] = VREG + v_lane_off + ((((2 * u) ^ v_swz) | (v_c >> 1)) << 4);
    }
    // V^T fragment of channel tile u / K fragment (kt, kk) at ring offset `off` (bytes, compile-time)
    auto pipe_v = [&](auto off, auto uu) -> uint4 {
        constexpr uint32_t C = decltype(off)::value;
        const unsigned char *a = smem + v_off[decltype(uu)::value];
        const uint2 lo = lds_read_tr16(a + C);
        const uint2 hi = lds_read_tr16(a + (C + 16 * ROWB));
        return make_uint4(lo.x, lo.y, hi.x, hi.y);
    };
    auto pipe_k = [&](auto off, auto ktt, auto kkk) -> uint4 {
        constexpr uint32_t C = decltype(off)::value + decltype(ktt)::value * 16 * ROWB;
        return *reinterpret_cast<const uint4 *>(smem + k_off[decltype(kkk)::value] + C);
    };
    // vprev / knext / vnext: ring offsets of V of step i-1, K of step i+1, V of step i
    auto pipe_iter = [&](f32x4 (&Sc)[TPW][2], f32x4 (&Sn)[TPW][2], const uint4 (&Pp)[TPW], uint4 (&Pc)[TPW],
                         uint4 (&vpre)[PF], auto vprev, auto knext, auto vnext, auto haspv, auto ntag) {
        constexpr int NA = decltype(ntag)::value;
        constexpr bool kPV = decltype(haspv)::value;
        if constexpr (kPipe && NA > 0) {
            constexpr int G = NT + 1 + 2 * KQ;           // MFMA groups: PV tiles, row sum, score fragments
            constexpr int NV = NA * 8;                   // scores per lane
            const uint4 ones = make_uint4(ones2<T>(), ones2<T>(), ones2<T>(), ones2<T>());
            const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
            uint4 fr[G];
            if constexpr (kPV) static_for<0, PF>([&](auto uu) { fr[decltype(uu)::value] = vpre[decltype(uu)::value]; });
            static_for<0, G>([&](auto nn) {
                constexpr int n = decltype(nn)::value;
                // first half of an iteration (PV groups + the bulk of the exponentials) above the
                // other wave of the SIMD, second half below it: 2-3 % fewer cycles than equal priority
                if constexpr (n == 0) __builtin_amdgcn_s_setprio(1);
                if constexpr (n == NT + 1) __builtin_amdgcn_s_setprio(0);
                // LDS stream
                constexpr int pn = n + PF;
                if constexpr (pn < NT) {
                    if constexpr (kPV) fr[pn] = pipe_v(vprev, std::integral_constant<int, pn>{});
                } else if constexpr (pn > NT && pn < G) {
                    fr[pn] = pipe_k(knext, std::integral_constant<int, (pn - NT - 1) & 1>{},
                                    std::integral_constant<int, ((pn - NT - 1) >> 1)>{});
                } else if constexpr (pn >= G) {
                    vpre[pn - G] = pipe_v(vnext, std::integral_constant<int, pn - G>{});
                }
                if constexpr (!kPV && n == 0) {          // the first PF score fragments, not prefetched by anyone
                    static_for<NT + 1, (NT + 1 + PF < G ? NT + 1 + PF : G)>([&](auto gg) {
                        constexpr int g2 = decltype(gg)::value;
                        fr[g2] = pipe_k(knext, std::integral_constant<int, (g2 - NT - 1) & 1>{},
                                        std::integral_constant<int, ((g2 - NT - 1) >> 1)>{});
                    });
                }
                // matrix stream
                static_for<0, NA>([&](auto tt) {
                    constexpr int t = decltype(tt)::value;
                    if constexpr (n < NT) {
                        if constexpr (kPV) O[t][n] = mfma16<T>(fr[n], Pp[t], O[t][n]);
                    } else if constexpr (n == NT) {
                        if constexpr (kPV) O[t][NT] = mfma16<T>(ones, Pp[t], O[t][NT]);
                    } else {
                        constexpr int kt = (n - NT - 1) & 1, kk = (n - NT - 1) >> 1;
                        if constexpr (kk == 0) Sn[t][kt] = mfma16<T>(fr[n], qf[t][kk], zero);
                        else Sn[t][kt] = mfma16<T>(fr[n], qf[t][kk], Sn[t][kt]);
                    }
                });
                // vector stream: scores [done1, done2) in this group, packs of the scores of the group before
                constexpr int done0 = n >= 2 ? ((n - 1) * NV / (G - 1) < NV ? (n - 1) * NV / (G - 1) : NV) : 0;
                constexpr int done1 = n >= 1 ? (n * NV / (G - 1) < NV ? n * NV / (G - 1) : NV) : 0;
                constexpr int done2 = (n + 1) * NV / (G - 1) < NV ? (n + 1) * NV / (G - 1) : NV;
                static_for<done1, done2>([&](auto ii) {
                    constexpr int idx = decltype(ii)::value;
                    constexpr int t = idx >> 3, kt = (idx >> 2) & 1, r = idx & 3;
                    float e = fast_exp2(__builtin_fmaf(Sc[t][kt][r], p.c_log2, -m[t]));
                    asm volatile("" : "+v"(e));          // pins the computation of the value to this group
                    Sc[t][kt][r] = e;
                });
                static_for<done0 / 2, done1 / 2>([&](auto cc) {
                    constexpr int cidx = decltype(cc)::value;
                    constexpr int t = cidx >> 2, kt = (cidx >> 1) & 1, h = cidx & 1;
                    uint32_t w = pack2<T>(Sc[t][kt][2 * h], Sc[t][kt][2 * h + 1]);
                    asm volatile("" : "+v"(w));
                    if constexpr (kt == 0 && h == 0) Pc[t].x = w;
                    else if constexpr (kt == 0) Pc[t].y = w;
                    else if constexpr (h == 0) Pc[t].z = w;
                    else Pc[t].w = w;
                });
                __builtin_amdgcn_sched_barrier(0);
            });
        }
    };

    // ---- reference m of every row tile from one unmasked step (before the fast loop) ----
    auto init_reference = [&](int buf, int ks, f32x4 (&keep)[TPW][2]) {
        if constexpr (!kF32) {
            const unsigned char *Kb = smem + buf * STAGE + ks * 32 * ROWB;
            uint4 kf[2][KQ];
            load_k_frags(Kb, kf);
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < KQ; ++kk) {
                    s0 = mfma16<T>(kf[0][kk], qf[t][kk], s0);
                    s1 = mfma16<T>(kf[1][kk], qf[t][kk], s1);
                }
                keep[t][0] = s0;
                keep[t][1] = s1;
                const float tm = fmaxf(fmaxf(fmaxf(s0[0], s0[1]), fmaxf(s0[2], s0[3])),
                                       fmaxf(fmaxf(s1[0], s1[1]), fmaxf(s1[2], s1[3])));
                // fp16 holds 2^(x - m) only up to 2^16: its reference sits a little above the
                // first step's maximum, which trades low-end resolution for head room
                m[t] = quad_column_max(tm) * p.c_log2 + (std::is_same<T, _Float16>::value ? 4.0f : 0.0f);
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
        const unsigned char *Kb = smem + buf * STAGE + ks * 32 * ROWB;
        const unsigned char *Vb = Kb + VREG;
        if constexpr (kF32) {
            // fp32 path: 16x16x4 MFMA, one channel (QK) / one key (PV) per quad and step
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                float kf[QREGS];
                const int key = kt * 16 + j;
#pragma unroll
                for (int kk = 0; kk < QREGS; ++kk)
                    kf[kk] = *reinterpret_cast<const float *>(
                        Kb + key * ROWB + ((kk ^ (key & KSWZ)) << 4) + qd * 4);
                float vraw[4][NT];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int vkey = kt * 16 + 4 * qd + r;
                    const int vs = (vkey & VSWM) << 1;
#pragma unroll
                    for (int u = 0; u < NT; ++u)
                        vraw[r][u] = *reinterpret_cast<const float *>(
                            Vb + vkey * ROWB + (((4 * u + (j >> 2)) ^ vs) << 4) + (j & 3) * 4);
                }
#pragma unroll
                for (int t = 0; t < TPW; ++t) {
                    if (t >= my_nt) continue;
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
            uint4 kf[2][KQ];
            load_k_frags(Kb, kf);
            uint4 pf[TPW];
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                pf[t] = make_uint4(0, 0, 0, 0);
                if (t >= my_nt) continue;
                f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < KQ; ++kk) {
                    s0 = mfma16<T>(kf[0][kk], qf[t][kk], s0);
                    s1 = mfma16<T>(kf[1][kk], qf[t][kk], s1);
                }
                softmax_step(s0, s1, t, step_pos);
                pf[t].x = pack2<T>(s0[0], s0[1]);
                pf[t].y = pack2<T>(s0[2], s0[3]);
                pf[t].z = pack2<T>(s1[0], s1[1]);
                pf[t].w = pack2<T>(s1[2], s1[3]);
            }
            const uint4 ones = make_uint4(ones2<T>(), ones2<T>(), ones2<T>(), ones2<T>());
#pragma unroll
            for (int u = 0; u < NT; ++u) {
                const uint4 vf = load_v_frag(Vb, u);
#pragma unroll
                for (int t = 0; t < TPW; ++t) O[t][u] = mfma16<T>(vf, pf[t], O[t][u]);
            }
#pragma unroll
            for (int t = 0; t < TPW; ++t) O[t][NT] = mfma16<T>(ones, pf[t], O[t][NT]);
        }
    };

    // ---- stage loop skeleton: keep NS-1 stages in flight ahead of the one computed ----
    int issued = 0;
    auto wait_stage = [&](int s) {
        // stage s has landed once at most (younger stages) * LPS loads remain
        const int ahead = issued - (s + 1);
        if (NS > 3 && ahead >= 2) wait_vmcnt<(NS > 3 ? 2 : 0) * LPS>();
        else if (NS > 2 && ahead == 1) wait_vmcnt<(NS > 2 ? 1 : 0) * LPS>();
        else wait_vmcnt<0>();
    };
    // careful stages [s_begin, s_end)
    auto run_careful = [&](int s_begin, int s_end) {
        for (int s = s_begin; s < s_end; ++s) {
            wait_stage(s);
            __syncthreads();     // everyone's part of stage s is in; stage s-1 is fully consumed
            if (issued < nstages) {
                issue_stage(issued);                // refills the slot stage s-1 occupied
                ++issued;
            }
            const int sbase = pos0 + s * SK;
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                if (ks % WK != wk) continue;
                if (sbase + ks * 32 >= pos1) continue;       // uniform: nothing left in this step
                careful_step(s % NS, ks, sbase + ks * 32);
            }
        }
    };
    // fast stages [0, n_fast); the caller has admitted stage 0.
    // The two waves of a SIMD (w and w + 4) would run in lockstep if both took
    // the per-stage barrier at the same place in their instruction stream, and
    // their MFMA phases and their exp/convert phases would collide.  So waves
    // 4..7 take it one PV block later than waves 0..3: they carry the last PV of
    // a stage (its P and V^T fragments are in registers by then, so the stage's
    // ring slot is free all the same) across the barrier.  After every barrier
    // the two waves of a SIMD are then half a step apart, and one's matrix work
    // overlaps the other's vector work.
    auto run_fast_n = [&](int n_fast, auto ntag, auto gtag) {
        if constexpr (!kF32) {
            const bool late = wave >= kWaves / 2;
            auto kptr = [&](int s, int ks) -> const unsigned char * {
                return smem + (s % NS) * STAGE + ks * 32 * ROWB;
            };
            auto admit = [&](int s) {
                wait_stage(s);
                __syncthreads();     // stage s is in; all LDS reads of stage s-1 have completed
                if (issued < nstages) {
                    issue_stage(issued);
                    ++issued;
                }
            };
            uint4 pf[TPW], vf[NT];
            for (int s = 0; s < n_fast; ++s) {
                if constexpr (WK == 1) {
                    if (s > 0) {
                        if (!late) fast_pv(pf, vf, ntag);       // early waves finish stage s-1 first
                        admit(s);
                        if (late) fast_pv(pf, vf, ntag);        // late waves carry it over
                    }
                    fast_sx(kptr(s, 0), kptr(s, 0) + VREG, pf, vf, ntag, gtag);
                    fast_pv(pf, vf, ntag);
                    fast_sx(kptr(s, 1), kptr(s, 1) + VREG, pf, vf, ntag, gtag);
                } else {
                    if (s > 0) {
                        if (!late) fast_pv(pf, vf, ntag);
                        admit(s);
                        if (late) fast_pv(pf, vf, ntag);
                    }
                    fast_sx(kptr(s, wk), kptr(s, wk) + VREG, pf, vf, ntag, gtag);
                }
            }
            fast_pv(pf, vf, ntag);
        }
    };
    // Pipelined fast stages [0, n_fast); the caller has admitted stage 0 and Sa
    // holds the scores of step 0.  V of a step is read one iteration after its
    // K, so a ring slot is refilled one stage later than in the plain loop: at
    // the barrier in front of step 2s+1 every wave is done with stage s-1.
    auto run_pipe_n = [&](int n_fast, f32x4 (&Sa)[TPW][2], auto ntag) {
        if constexpr (kPipe) {
            constexpr int NA = decltype(ntag)::value;
            using yes = std::true_type;
            using no = std::false_type;
            f32x4 Sb[TPW][2];
            uint4 Pa[TPW], Pb[TPW], vpre[PF];
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                Pa[t] = Pb[t] = make_uint4(0, 0, 0, 0);
                Sb[t][0] = Sb[t][1] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int u = 0; u < PF; ++u) vpre[u] = make_uint4(0, 0, 0, 0);
            // step 0: P of step 0, scores of step 1; no V^T P yet
            pipe_iter(Sa, Sb, Pb, Pa, vpre, std::integral_constant<uint32_t, 0>{},
                      std::integral_constant<uint32_t, 32 * ROWB>{}, std::integral_constant<uint32_t, 0>{}, no{}, ntag);
            for (int s4 = 0; s4 < n_fast; s4 += NS) {
                static_for<0, NS>([&](auto bb) {
                    constexpr uint32_t B = decltype(bb)::value, B1 = (B + 1) % NS;
                    constexpr uint32_t cur0 = B * STAGE, cur1 = B * STAGE + 32 * ROWB;
                    constexpr uint32_t nxt0 = B1 * STAGE, nxt1 = B1 * STAGE + 32 * ROWB;
                    const int s = s4 + (int)B;
                    if (s < n_fast) {                                   // uniform
                        // stage s+1 in; every wave is done with stage s-1: refill its slot
                        const int pg = stage_page(issued);
                        wait_stage(s + 1);
                        __syncthreads();
                        if (issued < nstages && issued <= s + NS - 1) {
                            issue_stage_pg(issued, pg);
                            ++issued;
                        }
                        // step 2s+1: its P; O += V^T P of step 2s; scores of step 2s+2
                        pipe_iter(Sb, Sa, Pa, Pb, vpre, std::integral_constant<uint32_t, cur0>{},
                                  std::integral_constant<uint32_t, nxt0>{}, std::integral_constant<uint32_t, cur1>{},
                                  yes{}, ntag);
                        // step 2s+2: its P; O += V^T P of step 2s+1; scores of step 2s+3.  After the
                        // last fast stage only the V^T P part counts: the P and the scores it
                        // produces belong to steps the careful loop redoes, and are dropped.
                        pipe_iter(Sa, Sb, Pb, Pa, vpre, std::integral_constant<uint32_t, cur1>{},
                                  std::integral_constant<uint32_t, nxt1>{}, std::integral_constant<uint32_t, nxt0>{},
                                  yes{}, ntag);
                    }
                });
            }
        }
    };
    // fp16 only: which fast loop?  The scores of the stages already requested (up to 192 keys)
    // are formed once more, without the softmax; if some lane's keys span more than 2^14 (ten
    // standard deviations of the scores of unit-variance inputs: no false alarm in 10^5 lanes) the
    // scores have a long tail, a later one is likely to pass the head room above the first
    // step's maximum, and the workgroup takes the guarded loop.  A wrong guess costs time only.
    auto probe_spread = [&](int n_fast) {
        if constexpr (kGuard) {
            float lo[TPW], hi[TPW];
#pragma unroll
            for (int t = 0; t < TPW; ++t) lo[t] = INFINITY, hi[t] = -INFINITY;
            // stage `issued - 1` may still be in flight; a short split is probed less
            const int n_probe = min(min(n_fast, issued - 1), max(1, n_fast / 16));
            for (int sb = 0; sb < n_probe; ++sb) {
                if (sb > 0) {
                    wait_stage(sb);
                    __syncthreads();
                }
#pragma unroll
                for (int ks = 0; ks < KSTEPS; ++ks) {
                    uint4 kf[2][KQ];
                    load_k_frags(smem + sb * STAGE + ks * 32 * ROWB, kf);
#pragma unroll
                    for (int t = 0; t < TPW; ++t) {
                        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int kk = 0; kk < KQ; ++kk) {
                            s0 = mfma16<T>(kf[0][kk], qf[t][kk], s0);
                            s1 = mfma16<T>(kf[1][kk], qf[t][kk], s1);
                        }
                        hi[t] = fmaxf(hi[t], fmaxf(fmaxf(fmaxf(s0[0], s0[1]), fmaxf(s0[2], s0[3])),
                                                   fmaxf(fmaxf(s1[0], s1[1]), fmaxf(s1[2], s1[3]))));
                        lo[t] = fminf(lo[t], fminf(fminf(fminf(s0[0], s0[1]), fminf(s0[2], s0[3])),
                                                   fminf(fminf(s1[0], s1[1]), fminf(s1[2], s1[3]))));
                    }
                }
            }
            bool wide = false;
#pragma unroll
            for (int t = 0; t < TPW; ++t) wide |= (hi[t] - lo[t]) * p.c_log2 > 14.0f;
            use_guard = __syncthreads_or(wide ? 1 : 0) != 0;
        }
    };
    // the fast loop is compiled once per possible tile count of a wave, so that
    // its body has no per-tile branches
    auto run_fast_tag = [&](int n_fast, f32x4 (&Sa)[TPW][2], auto ntag) {
        if constexpr (kGuard) {
            if (use_guard) {                          // uniform over the workgroup
                run_fast_n(n_fast, ntag, std::true_type{});
                return;
            }
        }
        if constexpr (kPipe) run_pipe_n(n_fast, Sa, ntag);
        else run_fast_n(n_fast, ntag, std::false_type{});
    };
    auto run_fast = [&](int n_fast, f32x4 (&Sa)[TPW][2]) {
        if (my_nt == TPW) run_fast_tag(n_fast, Sa, std::integral_constant<int, TPW>{});
        else if (TPW > 1 && my_nt == TPW - 1)
            run_fast_tag(n_fast, Sa, std::integral_constant<int, (TPW > 1 ? TPW - 1 : 0)>{});
        else if (TPW > 2 && my_nt == TPW - 2)
            run_fast_tag(n_fast, Sa, std::integral_constant<int, (TPW > 2 ? TPW - 2 : 0)>{});
        else run_fast_tag(n_fast, Sa, std::integral_constant<int, 0>{});
    };
    static_assert(TPW <= 3, "run_fast dispatches on at most three tile counts");

    // The set-up loads are drained here, so that vmcnt counts the K/V stages from now on; the
    // query fragments, requested between stage 0 and stage 1, complete in order with them (a
    // wait that leaves only younger stages outstanding covers stage 0 and the queries alike).
    wait_vmcnt<0>();

    // Pass 0: stages that lie wholly inside the prefix run the fast step with a
    // frozen reference; the rest (drafts, ragged end) run the careful step.
    // Pass 1 happens only if a row sum of pass 0 is not a modest finite number:
    // the whole split is redone with the careful step.  bf16 shares fp32's
    // exponent range, so that happens only for scores ~100 above the reference;
    // an fp16 P overflows 12 above it (and the redo is then the price).  fp32 is
    // the small correctness shape and has no fast loop.
    constexpr bool kHasFast = !kF32;
    issue_stage(0);                                   // nstages >= 1: the split exists
    load_queries();
    for (int pass = 0; pass < 2; ++pass) {
        issued = pass == 0 ? 1 : 0;                   // the redo pass starts over
        for (; issued < NS - 1 && issued < nstages; ++issued) issue_stage(issued);
        int n_fast = 0;
        if (kHasFast && pass == 0) n_fast = max(0, min(nstages, (L - pos0) / SK));
        if (n_fast > 0) {
            wait_stage(0);
            __syncthreads();
            stamp(2);
            if (issued < nstages) {                 // the slot beyond the prologue's stages is free
                issue_stage(issued);
                ++issued;
            }
            f32x4 Sa[TPW][2];
            init_reference(0, wk, Sa);
            probe_spread(n_fast);
            run_fast(n_fast, Sa);
        } else {
            stamp(2);
        }
        stamp(3);
        run_careful(n_fast, nstages);
        stamp(4);
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

    // ---- write this split's partial ----
    // fp32 partials (fp32 inputs, or on request): the accumulator fragments as they are, float4 [slot][u][lane] =
    // channels 16*u + 4*quad .. +3 of row lane%16.  Otherwise: each row normalised by its row sum and by its largest magnitude s, as fp16,
    // uint4 [slot][u/2][lane] = the four halves of channel tile u (even) and of u + 1; (m, l, s) beside it.
    if (wk == 0) {
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            const int tg = rg * p.group_tiles + t * WR + wr;
            if (t * WR + wr >= p.group_tiles || tg >= p.RT) continue;
            const size_t slot = (((size_t)b * p.Hkv + g) * p.max_splits + c) * p.RT + tg;
            const float l = O[t][NT][0];
            if (kF32 || !p.half_partials) {                          // uniform over the launch
                float4 *po = static_cast<float4 *>(p.part_o) + slot * (size_t)(NT * 64) + lane;
#pragma unroll
                for (int u = 0; u < NT; ++u)
                    po[u * 64] = make_float4(O[t][u][0], O[t][u][1], O[t][u][2], O[t][u][3]);
                if (qd == 0) {
                    p.part_ml[slot * kPartMl + j] = m[t];
                    p.part_ml[slot * kPartMl + 16 + j] = l;
                    p.part_ml[slot * kPartMl + 32 + j] = 1.0f;
                }
            } else {
                const float inv_l = l > 0.f ? 1.0f / l : 0.f;          // a row that saw no key: all zeros
                float big = 0.f;
#pragma unroll
                for (int u = 0; u < NT; ++u)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        O[t][u][r] *= inv_l;
                        big = fmaxf(big, fabsf(O[t][u][r]));
                    }
                big = quad_column_max(big);                             // over the four lanes that hold this row
                const float inv_s = big > 0.f ? 1.0f / big : 0.f;
                uint4 *po = static_cast<uint4 *>(p.part_o) + slot * (size_t)(NT / 2 * 64) + lane;
#pragma unroll
                for (int u = 0; u < NT; u += 2)
                    po[(u / 2) * 64] = make_uint4(pack2<_Float16>(O[t][u][0] * inv_s, O[t][u][1] * inv_s),
                                                   pack2<_Float16>(O[t][u][2] * inv_s, O[t][u][3] * inv_s),
                                                   pack2<_Float16>(O[t][u + 1][0] * inv_s, O[t][u + 1][1] * inv_s),
                                                   pack2<_Float16>(O[t][u + 1][2] * inv_s, O[t][u + 1][3] * inv_s));
                if (qd == 0) {
                    p.part_ml[slot * kPartMl + j] = m[t];
                    p.part_ml[slot * kPartMl + 16 + j] = l;
                    p.part_ml[slot * kPartMl + 32 + j] = big;
                }
            }
        }
    }
    if constexpr (TL) {
        __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0): the partial stores have left
        stamp(5);
    }
}

// ---------------------------------------------------------------------------
// instantiations
// ---------------------------------------------------------------------------
template <typename T, int D, int TPW, int WR, int WK, bool TL>
static void launch_variant(const KParams &p, dim3 grid, hipStream_t s, hipEvent_t start, hipEvent_t stop)
{
    using GEO = Geo<T, D, TPW, WR, WK>;
    if (start || stop)
        hipExtLaunchKernelGGL((splitkv_kernel<T, D, TPW, WR, WK, TL>), grid, dim3(kThreads), GEO::LDS, s, start, stop, 0, p);
    else
        hipLaunchKernelGGL((splitkv_kernel<T, D, TPW, WR, WK, TL>), grid, dim3(kThreads), GEO::LDS, s, p);
}

#define OWL_VARIANT(DT, T, D, TPW, WR, WK, TL)                                          \
    Variant { DT, D, TPW, WR, WK, TL, Geo<T, D, TPW, WR, WK>::LDS,                     \
              &launch_variant<T, D, TPW, WR, WK, TL>,                                   \
              reinterpret_cast<const void *>(&splitkv_kernel<T, D, TPW, WR, WK, TL>) }

#define OWL_VARIANTS_16BIT(DT, T, D, TL)                                                \
    OWL_VARIANT(DT, T, D, 1, 4, 2, TL), OWL_VARIANT(DT, T, D, 1, 8, 1, TL),             \
    OWL_VARIANT(DT, T, D, 2, 8, 1, TL), OWL_VARIANT(DT, T, D, 3, 8, 1, TL)

static const Variant kVariants[] = {
    OWL_VARIANTS_16BIT(OWL_BF16, __bf16, 128, false),
    OWL_VARIANTS_16BIT(OWL_BF16, __bf16, 64, false),
    OWL_VARIANTS_16BIT(OWL_F16, _Float16, 128, false),
    OWL_VARIANTS_16BIT(OWL_F16, _Float16, 64, false),
    OWL_VARIANT(OWL_F32, float, 64, 1, 8, 1, false),
    OWL_VARIANT(OWL_F32, float, 128, 1, 8, 1, false),
    // copies with the per-workgroup timeline hook: the benchmark's type and head size only
    OWL_VARIANTS_16BIT(OWL_BF16, __bf16, 128, true),
};

const Variant *find_variant(int dtype, int D, int tpw, int wr, int wk, bool timeline)
{
    for (const Variant &v : kVariants)
        if (v.dtype == dtype && v.D == D && v.tpw == tpw && v.wr == wr && v.wk == wk && v.timeline == timeline)
            return &v;
    return nullptr;
}

int variant_index(const Variant *v) { return v ? static_cast<int>(v - kVariants) : -1; }

}  // namespace owl
