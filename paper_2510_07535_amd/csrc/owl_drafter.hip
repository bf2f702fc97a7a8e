// One step of the drafter's recurrent cell (Sec. 3.2.1, Eq. 1-8 of the paper):
//     e   = E[t]                                   s^m = W^m h + alpha e,  m in {f, i, o, c}
//     g^m = sigmoid(s^m), m in {f, i, o}           c   = f(s^c) g^i
//     z'  = z g^f + c                              h'  = f(z') g^o
// with f = layer normalisation over the d channels followed by GeLU.
//
// The projection W^m h reads every weight exactly once (4 d d_in
// elements, 1.2 GB for the paper's d = 12288 with a square W) against at most
// 64 state rows: a streaming read of HBM with a thin contraction on the side,
// done with MFMA only because 64 rows x 4 d x d_in multiply-adds per step are
// beyond the vector ALUs at that rate.  Weights go from global memory straight
// into the MFMA operand registers: no element is used twice, so there is
// nothing to stage in LDS.  The gates then need whole-row statistics twice (of
// s^c and of z'): three small launches, see below.
#include "owl_device.h"

namespace owl {

typedef float d_f32x4 __attribute__((ext_vector_type(4)));
typedef int d_i32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 d_bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 d_f16x8 __attribute__((ext_vector_type(8)));

template <bool kF16>
__device__ __forceinline__ d_f32x4 mfma16(d_i32x4 a, d_i32x4 b, d_f32x4 c)
{
    if constexpr (kF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(d_f16x8, a),
                                                      __builtin_bit_cast(d_f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(d_bf16x8, a),
                                                       __builtin_bit_cast(d_bf16x8, b), c, 0, 0, 0);
}

// ---------------------------------------------------------------------------
// Projection.  The four W^m, each [d][d_in] (one output channel's weights
// contiguous), are one matrix of 4d rows.  A workgroup of four wavefronts owns
// 64 consecutive rows (four 16-row MFMA tiles); every wavefront works on all
// four tiles, so that a fragment of h is loaded once per four weight fragments,
// and the wavefronts split the contraction dimension: wavefront w takes the
// k-blocks w, w + 4, ... of 128 elements.  In MFMA terms A = h (rows = states),
// B = W^T (columns = weight rows): lane l supplies the 8 consecutive k values of
// group l / 16 for state row / weight row l % 16, 16 bytes straight from memory.
// The four partial sums meet in LDS and are added in a fixed order.
//     s [P][4d] fp32, s[p][m * d + j] = (W^m h_p)[j]
//
// Two weight layouts.  OWL_W_ROWS is the matrix as it stands: a load instruction
// then touches 16 rows with 64 bytes each and the chip holds ~50 000 row streams
// open at once, which DRAM serves at 4.6-4.9 TB/s.  OWL_W_TILED stores the same
// numbers in the order the kernel consumes them,
//     granule(row, k) = ((row / 64 * KS + k / 32) * 4 + row % 64 / 16) * 64 + (k % 32 / 8) * 16 + row % 16
// in units of 16 bytes (8 elements), KS = d_in / 32, rows padded with zeros to a
// multiple of 64: one load instruction reads 1 KB contiguous, a workgroup reads
// one contiguous run of 64 d_in elements from end to end, and the same kernel
// reaches 5.6-5.9 TB/s, what a plain streaming read gets on this chip.
// ---------------------------------------------------------------------------
constexpr int kProjWaves = 4;
constexpr int kProjTiles = 4;     // 16-row weight tiles per workgroup (fixed by the tiled layout)
constexpr int kProjUnroll = 4;    // k-steps of 32 per wavefront and round
static_assert(kProjTiles <= kProjWaves, "wavefront w adds up and stores weight tile w");

template <bool kF16, int PT, bool kTiled>
__global__ void __launch_bounds__(kProjWaves * 64) drafter_proj_kernel(const uint16_t *__restrict__ h,
                                                                       const uint16_t *__restrict__ w,
                                                                       float *__restrict__ s, int P, int d_in,
                                                                       int n_rows)
{
    __shared__ d_f32x4 red[kProjWaves][kProjTiles][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, kg = lane >> 4;
    const int n_tiles = n_rows / 16;
    const int tile0 = blockIdx.x * kProjTiles;
    const int k_steps = d_in / 32;

    // wp[nb] + ks * w_step is this lane's 16 bytes of k-step ks of weight tile nb.
    const uint16_t *wp[kProjTiles];
    int64_t w_step;
    if constexpr (kTiled) {
        w_step = kProjTiles * 512;
#pragma unroll
        for (int nb = 0; nb < kProjTiles; ++nb)
            wp[nb] = w + ((int64_t)blockIdx.x * k_steps * kProjTiles + nb) * 512 + lane * 8;
    } else {
        w_step = 32;
#pragma unroll
        for (int nb = 0; nb < kProjTiles; ++nb) {
            // A tile past the end re-reads the last tile (in bounds); its sums are not stored.
            const int t = min(tile0 + nb, n_tiles - 1);
            wp[nb] = w + (int64_t)(t * 16 + n) * d_in + kg * 8;
        }
    }
    // State rows past P read row P - 1 (in bounds) and are not stored either.
    const uint16_t *hp[PT];
#pragma unroll
    for (int pt = 0; pt < PT; ++pt) hp[pt] = h + (int64_t)min(pt * 16 + n, P - 1) * d_in + kg * 8;

    d_f32x4 acc[PT][kProjTiles];
#pragma unroll
    for (int pt = 0; pt < PT; ++pt)
#pragma unroll
        for (int nb = 0; nb < kProjTiles; ++nb) acc[pt][nb] = d_f32x4{0.f, 0.f, 0.f, 0.f};

    // With more than 16 state rows the h fragments weigh as much as the weights in the L1/L2
    // traffic, and every workgroup of the chip asks for the same lines of h at the same time if
    // all sweep k in the same order: each starts at a round of its own instead.
    const int rounds = (k_steps + kProjWaves * kProjUnroll - 1) / (kProjWaves * kProjUnroll);
    const int first = PT > 1 ? (int)((blockIdx.x * 7u) % (unsigned)rounds) : 0;
    for (int it = 0; it < rounds; ++it) {
        const int rr = it + first < rounds ? it + first : it + first - rounds;
        const int ks0 = (rr * kProjWaves + wave) * kProjUnroll;
        d_i32x4 b[kProjUnroll][kProjTiles], a[kProjUnroll][PT];
#pragma unroll
        for (int u = 0; u < kProjUnroll; ++u) {
            const bool live = ks0 + u < k_steps;            // uniform over the wavefront
            const int ks = live ? ks0 + u : 0;
#pragma unroll
            for (int nb = 0; nb < kProjTiles; ++nb) {
                // every weight is used once: a non-temporal load, which leaves the caches to h (re-read by
                // every workgroup) and is worth 11 % on this chip (square step: 206 -> 183 us)
                b[u][nb] = __builtin_nontemporal_load(reinterpret_cast<const d_i32x4 *>(wp[nb] + ks * w_step));
                if (!live) b[u][nb] = d_i32x4{0, 0, 0, 0};
            }
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) a[u][pt] = *reinterpret_cast<const d_i32x4 *>(hp[pt] + ks * 32);
        }
#pragma unroll
        for (int u = 0; u < kProjUnroll; ++u)
#pragma unroll
            for (int pt = 0; pt < PT; ++pt)
#pragma unroll
                for (int nb = 0; nb < kProjTiles; ++nb) acc[pt][nb] = mfma16<kF16>(a[u][pt], b[u][nb], acc[pt][nb]);
    }

    // Accumulator layout: lane l holds, for weight row l % 16, the state rows 4 (l / 16) + i.
    const int t_mine = tile0 + wave;
#pragma unroll
    for (int pt = 0; pt < PT; ++pt) {
        if (pt) __syncthreads();
#pragma unroll
        for (int nb = 0; nb < kProjTiles; ++nb) red[wave][nb][lane] = acc[pt][nb];
        __syncthreads();
        if (wave < kProjTiles && t_mine < n_tiles) {
            d_f32x4 v = red[0][wave][lane];
#pragma unroll
            for (int ww = 1; ww < kProjWaves; ++ww) v += red[ww][wave][lane];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int p = pt * 16 + kg * 4 + i;
                if (p < P) s[(int64_t)p * n_rows + t_mine * 16 + n] = v[i];
            }
        }
    }
}

static int proj_groups(int d) { return (4 * d / 16 + kProjTiles - 1) / kProjTiles; }

template <bool kF16, int PT>
static hipError_t launch_proj_pt(const void *h, const void *w, bool tiled, float *s, int P, int d_in, int d,
                                 hipStream_t st)
{
    const int n_rows = 4 * d;
    const dim3 grid(proj_groups(d)), block(kProjWaves * 64);
    const uint16_t *hh = static_cast<const uint16_t *>(h), *ww = static_cast<const uint16_t *>(w);
    if (tiled)
        hipLaunchKernelGGL((drafter_proj_kernel<kF16, PT, true>), grid, block, 0, st, hh, ww, s, P, d_in, n_rows);
    else
        hipLaunchKernelGGL((drafter_proj_kernel<kF16, PT, false>), grid, block, 0, st, hh, ww, s, P, d_in, n_rows);
    return hipGetLastError();
}

template <bool kF16>
static hipError_t launch_proj_dt(const void *h, const void *w, bool tiled, float *s, int P, int d_in, int d,
                                 hipStream_t st)
{
    switch ((P + 15) / 16) {
    case 1: return launch_proj_pt<kF16, 1>(h, w, tiled, s, P, d_in, d, st);
    case 2: return launch_proj_pt<kF16, 2>(h, w, tiled, s, P, d_in, d, st);
    case 3: return launch_proj_pt<kF16, 3>(h, w, tiled, s, P, d_in, d, st);
    default: return launch_proj_pt<kF16, 4>(h, w, tiled, s, P, d_in, d, st);
    }
}

hipError_t launch_drafter_proj(int dtype, const void *h, const void *w, bool tiled, float *s, int P, int d_in,
                               int d, hipStream_t st)
{
    return dtype == OWL_F16 ? launch_proj_dt<true>(h, w, tiled, s, P, d_in, d, st)
                            : launch_proj_dt<false>(h, w, tiled, s, P, d_in, d, st);
}

// Bytes of the tiled copy of the weights: whole groups of 64 rows.
size_t drafter_tiled_bytes(int d_in, int d) { return (size_t)proj_groups(d) * (d_in / 32) * kProjTiles * 1024; }

// One thread per 16-byte granule of the tiled layout: find the (row, k) it holds
// and copy it from the row layout, zeros for the padding rows.
__global__ void __launch_bounds__(256) drafter_tile_weights_kernel(const uint4 *__restrict__ w_rows,
                                                                   uint4 *__restrict__ w_tiled, int d_in,
                                                                   int n_rows, int64_t n_granules)
{
    const int64_t gi = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gi >= n_granules) return;
    const int k_steps = d_in / 32;
    const int lane = (int)(gi & 63);
    const int nb = (int)((gi >> 6) % kProjTiles);
    const int64_t rest = (gi >> 6) / kProjTiles;
    const int ks = (int)(rest % k_steps);
    const int64_t g = rest / k_steps;
    const int64_t row = g * (kProjTiles * 16) + nb * 16 + (lane & 15);
    const int k = ks * 32 + (lane >> 4) * 8;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (row < n_rows) v = w_rows[(row * d_in + k) / 8];
    w_tiled[gi] = v;
}

hipError_t launch_drafter_tile_weights(const void *w_rows, void *w_tiled, int d_in, int d, hipStream_t st)
{
    const int64_t n_granules = (int64_t)(drafter_tiled_bytes(d_in, d) / 16);
    const int64_t blocks = (n_granules + 255) / 256;
    hipLaunchKernelGGL(drafter_tile_weights_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                       static_cast<const uint4 *>(w_rows), static_cast<uint4 *>(w_tiled), d_in, 4 * d, n_granules);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Gates and state update.  f needs the mean and variance of a whole row twice
// (of s^c, then of z'), and the transcendental work of one row (three sigmoids
// and two GeLUs per channel) keeps a single compute unit busy for ~20 us, so a
// row is spread over workgroups of 256 threads x 4 channels and the two row
// statistics travel through memory between three small launches:
//   1. per chunk of 1024 channels: count, mean and centred sum of squares of s^c
//   2. merge those; z' = z g^f + f(s^c) g^i; the same partials of z'
//   3. merge those; h' = f(z') g^o
// Partials are (mean, M2) pairs merged with the pairwise update
//     M2 = sum_c M2_c + n_c (mean_c - mean)^2 ,
// which keeps the variance as accurate as a two-pass sum.
// ---------------------------------------------------------------------------
constexpr int kGateThreads = 256;
constexpr int kGateChunk = kGateThreads * 4;               // channels per workgroup
constexpr int kGateMaxChunks = 16;                         // d <= 16384

__device__ __forceinline__ float block_sum(float v, float *scratch)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();                                        // scratch may still be read from the last call
    if (lane == 0) scratch[wave] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < kGateThreads / 64; ++i) t += scratch[i];   // same order in every thread
    return t;
}

__device__ __forceinline__ float sigmoid_f(float x) { return 1.0f / (1.0f + expf(-x)); }
__device__ __forceinline__ float gelu_f(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }

template <bool kF16> __device__ __forceinline__ float widen16(uint16_t b)
{
    if constexpr (kF16) return (float)__builtin_bit_cast(_Float16, b);
    else return __builtin_bit_cast(float, (uint32_t)b << 16);
}

template <bool kF16> __device__ __forceinline__ uint16_t narrow16(float x)
{
    if constexpr (kF16) {
        return __builtin_bit_cast(uint16_t, (_Float16)x);   // round to nearest even in hardware
    } else {
        uint32_t u = __builtin_bit_cast(uint32_t, x);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);   // NaN stays NaN
        u += 0x7fffu + ((u >> 16) & 1u);                    // round to nearest even
        return (uint16_t)(u >> 16);
    }
}

// alpha * (four consecutive channels of a 16-bit embedding row)
template <bool kF16> __device__ __forceinline__ float4 scaled_emb4(const uint16_t *p, float alpha)
{
    const uint2 raw = *reinterpret_cast<const uint2 *>(p);
    return make_float4(alpha * widen16<kF16>((uint16_t)(raw.x & 0xffffu)), alpha * widen16<kF16>((uint16_t)(raw.x >> 16)),
                       alpha * widen16<kF16>((uint16_t)(raw.y & 0xffffu)), alpha * widen16<kF16>((uint16_t)(raw.y >> 16)));
}

__device__ __forceinline__ float4 ld4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ __forceinline__ float4 ld4_or(const float *p, int j, float fill)
{
    return p ? ld4(p + j) : make_float4(fill, fill, fill, fill);
}
__device__ __forceinline__ float4 add4(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }

struct GateArgs {
    const float *s, *z;
    const int32_t *tokens, *parent_row;
    const uint16_t *emb;
    const float *gamma_c, *beta_c, *gamma_z, *beta_z;
    uint16_t *h_out;
    float *h_out_f32, *z_out;
    float *part_c, *part_z;       // [M][kGateMaxChunks][2]: mean and centred sum of squares per chunk
    int P, d, vocab;
    float alpha, eps;
    uint32_t *status;
};

// What every gate kernel needs first: the row's state, its token's embedding
// row and the embedding weight (0 for a token outside the table).
struct GateRow {
    const float *sp, *zp;
    const uint16_t *ep;
    float alpha;
};

__device__ __forceinline__ GateRow gate_row(const GateArgs &a, int r, bool flag)
{
    int p = a.parent_row ? a.parent_row[r] : r;
    if (p < 0 || p >= a.P) {
        if (flag && threadIdx.x == 0) flag_status(a.status, OWL_DEV_BAD_ROW);
        p = 0;
    }
    int tok = a.tokens[r];
    float alpha = a.alpha;
    if (tok < 0 || tok >= a.vocab) {
        if (flag && threadIdx.x == 0) flag_status(a.status, OWL_DEV_BAD_TOKEN);
        tok = 0;
        alpha = 0.f;
    }
    return GateRow{a.s + (int64_t)p * 4 * a.d, a.z + (int64_t)p * a.d, a.emb + (int64_t)tok * a.d, alpha};
}

// Mean and centred sum of squares of the live channels of this workgroup's chunk.
__device__ __forceinline__ void chunk_stats(float4 v, bool live, int n_live, float *scratch, float *out2)
{
    const float sum = block_sum(live ? (v.x + v.y) + (v.z + v.w) : 0.f, scratch);
    const float mean = sum / (float)n_live;
    float sq = 0.f;
    if (live) {
        v.x -= mean, v.y -= mean, v.z -= mean, v.w -= mean;
        sq = (v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w);
    }
    const float m2 = block_sum(sq, scratch);
    if (threadIdx.x == 0) out2[0] = mean, out2[1] = m2;
}

// Mean and 1 / sqrt(variance + eps) of a row from its chunks' partials.
__device__ __forceinline__ void merge_stats(const float *part, int d, float eps, float *mean_out, float *rstd_out)
{
    const int n_chunks = (d + kGateChunk - 1) / kGateChunk;
    float mean = 0.f;
    for (int c = 0; c < n_chunks; ++c) mean += part[2 * c] * (float)min(kGateChunk, d - c * kGateChunk);
    mean /= (float)d;
    float m2 = 0.f;
    for (int c = 0; c < n_chunks; ++c) {
        const float dm = part[2 * c] - mean;
        m2 += part[2 * c + 1] + (float)min(kGateChunk, d - c * kGateChunk) * dm * dm;
    }
    *mean_out = mean;
    *rstd_out = 1.0f / sqrtf(m2 / (float)d + eps);
}

template <bool kF16>
__global__ void __launch_bounds__(kGateThreads) drafter_stats_kernel(GateArgs a)
{
    __shared__ float scratch[kGateThreads / 64];
    const int c = blockIdx.x, r = blockIdx.y, j = c * kGateChunk + threadIdx.x * 4;
    const GateRow g = gate_row(a, r, c == 0);
    const bool live = j < a.d;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (live) v = add4(ld4(g.sp + 3 * a.d + j), scaled_emb4<kF16>(g.ep + j, g.alpha));
    chunk_stats(v, live, min(kGateChunk, a.d - c * kGateChunk), scratch, a.part_c + ((int64_t)r * kGateMaxChunks + c) * 2);
}

template <bool kF16>
__global__ void __launch_bounds__(kGateThreads) drafter_state_kernel(GateArgs a)
{
    __shared__ float scratch[kGateThreads / 64];
    const int c = blockIdx.x, r = blockIdx.y, j = c * kGateChunk + threadIdx.x * 4;
    const GateRow g = gate_row(a, r, false);
    float mean, rstd;
    merge_stats(a.part_c + (int64_t)r * kGateMaxChunks * 2, a.d, a.eps, &mean, &rstd);
    const bool live = j < a.d;
    float4 zn = make_float4(0.f, 0.f, 0.f, 0.f);
    if (live) {
        const float4 e = scaled_emb4<kF16>(g.ep + j, g.alpha);
        const float4 sf = add4(ld4(g.sp + j), e), si = add4(ld4(g.sp + a.d + j), e), sc = add4(ld4(g.sp + 3 * a.d + j), e);
        const float4 zo = ld4(g.zp + j), ga = ld4_or(a.gamma_c, j, 1.f), be = ld4_or(a.beta_c, j, 0.f);
        zn.x = zo.x * sigmoid_f(sf.x) + gelu_f((sc.x - mean) * rstd * ga.x + be.x) * sigmoid_f(si.x);
        zn.y = zo.y * sigmoid_f(sf.y) + gelu_f((sc.y - mean) * rstd * ga.y + be.y) * sigmoid_f(si.y);
        zn.z = zo.z * sigmoid_f(sf.z) + gelu_f((sc.z - mean) * rstd * ga.z + be.z) * sigmoid_f(si.z);
        zn.w = zo.w * sigmoid_f(sf.w) + gelu_f((sc.w - mean) * rstd * ga.w + be.w) * sigmoid_f(si.w);
        *reinterpret_cast<float4 *>(a.z_out + (int64_t)r * a.d + j) = zn;
    }
    chunk_stats(zn, live, min(kGateChunk, a.d - c * kGateChunk), scratch, a.part_z + ((int64_t)r * kGateMaxChunks + c) * 2);
}

template <bool kF16>
__global__ void __launch_bounds__(kGateThreads) drafter_hidden_kernel(GateArgs a)
{
    const int c = blockIdx.x, r = blockIdx.y, j = c * kGateChunk + threadIdx.x * 4;
    const GateRow g = gate_row(a, r, false);
    float mean, rstd;
    merge_stats(a.part_z + (int64_t)r * kGateMaxChunks * 2, a.d, a.eps, &mean, &rstd);
    if (j >= a.d) return;
    const float4 so = add4(ld4(g.sp + 2 * a.d + j), scaled_emb4<kF16>(g.ep + j, g.alpha));
    const float4 zn = ld4(a.z_out + (int64_t)r * a.d + j), ga = ld4_or(a.gamma_z, j, 1.f), be = ld4_or(a.beta_z, j, 0.f);
    float4 hn;
    hn.x = gelu_f((zn.x - mean) * rstd * ga.x + be.x) * sigmoid_f(so.x);
    hn.y = gelu_f((zn.y - mean) * rstd * ga.y + be.y) * sigmoid_f(so.y);
    hn.z = gelu_f((zn.z - mean) * rstd * ga.z + be.z) * sigmoid_f(so.z);
    hn.w = gelu_f((zn.w - mean) * rstd * ga.w + be.w) * sigmoid_f(so.w);
    if (a.h_out) {
        uint2 pk;
        pk.x = (uint32_t)narrow16<kF16>(hn.x) | ((uint32_t)narrow16<kF16>(hn.y) << 16);
        pk.y = (uint32_t)narrow16<kF16>(hn.z) | ((uint32_t)narrow16<kF16>(hn.w) << 16);
        *reinterpret_cast<uint2 *>(a.h_out + (int64_t)r * a.d + j) = pk;
    }
    if (a.h_out_f32) *reinterpret_cast<float4 *>(a.h_out_f32 + (int64_t)r * a.d + j) = hn;
}

size_t drafter_gate_scratch_floats(int M) { return (size_t)2 * M * kGateMaxChunks * 2; }

template <bool kF16> static hipError_t launch_gates_dt(const GateArgs &a, int M, hipStream_t st)
{
    const dim3 grid((a.d + kGateChunk - 1) / kGateChunk, M), block(kGateThreads);
    hipLaunchKernelGGL(drafter_stats_kernel<kF16>, grid, block, 0, st, a);
    hipLaunchKernelGGL(drafter_state_kernel<kF16>, grid, block, 0, st, a);
    hipLaunchKernelGGL(drafter_hidden_kernel<kF16>, grid, block, 0, st, a);
    return hipGetLastError();
}

hipError_t launch_drafter_gates(int dtype, const float *s, const float *z, const int32_t *tokens,
                                const int32_t *parent_row, const void *emb, const float *gamma_c,
                                const float *beta_c, const float *gamma_z, const float *beta_z, void *h_out,
                                float *h_out_f32, float *z_out, float *gate_scratch, int P, int M, int d, int vocab,
                                float alpha, float eps, uint32_t *status, hipStream_t st)
{
    GateArgs a;
    a.s = s, a.z = z, a.tokens = tokens, a.parent_row = parent_row, a.emb = static_cast<const uint16_t *>(emb);
    a.gamma_c = gamma_c, a.beta_c = beta_c, a.gamma_z = gamma_z, a.beta_z = beta_z;
    a.h_out = static_cast<uint16_t *>(h_out), a.h_out_f32 = h_out_f32, a.z_out = z_out;
    a.part_c = gate_scratch, a.part_z = gate_scratch + (size_t)M * kGateMaxChunks * 2;
    a.P = P, a.d = d, a.vocab = vocab, a.alpha = alpha, a.eps = eps, a.status = status;
    return dtype == OWL_F16 ? launch_gates_dt<true>(a, M, st) : launch_gates_dt<false>(a, M, st);
}

}  // namespace owl
