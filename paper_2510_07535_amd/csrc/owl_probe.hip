// Measurement and self-test aids of the verify-attention library: kernels that
// measure what the chip can do (streaming reads, the matrix pipe), a one-wave
// check of a cross-lane step, and the switch of the per-workgroup timeline
// hook.  Declared in owl_probe.h; nothing here is on the product path.
#include <mutex>

#include "owl_device.h"
#include "owl_probe.h"

namespace owl {

// ---------------------------------------------------------------------------
// Streaming-read probe.  Every workgroup owns one contiguous piece of the
// buffer and walks it front to back; a thread keeps 16 independent 16-byte
// non-temporal loads in flight (64 KiB per workgroup and round), the way the
// library's own streaming kernels do.  What it reaches is the practical ceiling of a plain
// HBM read on this chip.
// ---------------------------------------------------------------------------
constexpr int kStreamUnroll = 16;

// Non-temporal: the data is read once and need not stay in any cache.  On this chip that is worth
// 12 % (6.2 -> 6.9 TB/s) to a streaming read.
__device__ __forceinline__ uint4 load_stream(const uint4 *p)
{
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return make_uint4(v[0], v[1], v[2], v[3]);
}

__global__ void __launch_bounds__(256) stream_read_kernel(const uint4 *__restrict__ src, size_t n_vec,
                                                          uint32_t *sink)
{
    uint32_t acc = 0;
    // piece of this workgroup: whole rounds of kStreamUnroll * 256 vectors, the remainder goes to the last one
    const size_t round = (size_t)kStreamUnroll * 256;
    const size_t rounds_total = n_vec / round;
    const size_t per_wg = (rounds_total + gridDim.x - 1) / gridDim.x;
    const size_t r0 = min(per_wg * blockIdx.x, rounds_total), r1 = min(r0 + per_wg, rounds_total);
    for (size_t r = r0; r < r1; ++r) {
        const uint4 *base = src + r * round + threadIdx.x;
        uint4 v[kStreamUnroll];
#pragma unroll
        for (int k = 0; k < kStreamUnroll; ++k) v[k] = load_stream(base + k * 256);
#pragma unroll
        for (int k = 0; k < kStreamUnroll; ++k) acc ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
    }
    if (blockIdx.x == gridDim.x - 1)
        for (size_t i = rounds_total * round + threadIdx.x; i < n_vec; i += 256) {
            const uint4 a = src[i];
            acc ^= a.x ^ a.y ^ a.z ^ a.w;
        }
    for (int off = 32; off > 0; off >>= 1) acc ^= __shfl_xor(acc, off);
    __shared__ uint32_t s_acc[4];
    if ((threadIdx.x & 63) == 0) s_acc[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = s_acc[0] ^ s_acc[1] ^ s_acc[2] ^ s_acc[3];
}

// The buffer is visited in 4 KiB blocks in the order given by `perm` (one block
// = 256 threads x 16 bytes), eight blocks in flight per workgroup: the access
// pattern of a head-major paged cache whose pages were handed out in random
// order.
__global__ void __launch_bounds__(256) gather_read_kernel(const uint4 *src, const int32_t *perm,
                                                          int n_blocks, uint32_t *sink)
{
    uint32_t acc = 0;
    int blk = blockIdx.x;
    const int stride = gridDim.x;
    for (; blk + 7 * stride < n_blocks; blk += 8 * stride) {
        uint4 v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = src[(size_t)perm[blk + i * stride] * 256 + threadIdx.x];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc ^= v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
    }
    for (; blk < n_blocks; blk += stride) {
        const uint4 a = src[(size_t)perm[blk] * 256 + threadIdx.x];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    for (int off = 32; off > 0; off >>= 1) acc ^= __shfl_xor(acc, off);
    __shared__ uint32_t s_acc[4];
    if ((threadIdx.x & 63) == 0) s_acc[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = s_acc[0] ^ s_acc[1] ^ s_acc[2] ^ s_acc[3];
}

// ---------------------------------------------------------------------------
// Matrix-pipe probe: 8 wavefronts per workgroup, each issuing nothing but
// 16x16x32 bf16 MFMAs on operands taken once from `src` (so their bit patterns
// are the caller's: the sustained rate of this chip depends on them).  16
// independent accumulators per lane; sums are scaled down now and then to stay
// finite.  2 * 16*16*32 flop per MFMA, 16 MFMAs per lane and iteration.
// ---------------------------------------------------------------------------
typedef float probe_f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));

__global__ void __launch_bounds__(512) mfma_probe_kernel(const uint4 *src, int n_vec, int iters, float *sink,
                                                         float *clock_ghz)
{
    uint4 a[8], b[2];
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = src[(threadIdx.x * 8 + i) % n_vec];
#pragma unroll
    for (int i = 0; i < 2; ++i) b[i] = src[(threadIdx.x * 2 + i + 77) % n_vec];
    probe_f32x4 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = probe_f32x4{0.f, 0.f, 0.f, 0.f};
    // shader cycles over constant-rate (100 MHz) ticks = the clock this workgroup really ran at
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
            acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(probe_bf16x8, a[i & 7]),
                                                             __builtin_bit_cast(probe_bf16x8, b[i >> 3]), acc[i], 0, 0, 0);
        if ((it & 63) == 63) {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] *= 1.0e-3f;
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[i][0] + acc[i][3];
    sink[blockIdx.x * 512 + threadIdx.x] = s;
    const long long c1 = clock64(), w1 = wall_clock64();
    if (clock_ghz && threadIdx.x == 0) clock_ghz[blockIdx.x] = w1 > w0 ? (float)(c1 - c0) / ((float)(w1 - w0) * 10.0f) : 0.f;
}

// ---------------------------------------------------------------------------
// Step probe: the instruction mix of one 32-key step of the split-KV fast loop
// (K fragments from LDS, QK MFMAs, exp2 softmax, pack, V fragments from LDS, PV
// and row-sum MFMAs) on register- and LDS-resident data, without the HBM side:
// what the matrix pipe can be kept busy at by two wavefronts per SIMD holding
// TA and TB row tiles, with and without a workgroup barrier every 64 keys, with
// the V fragments fetched by 128-bit or by 64-bit LDS reads.  Plain step
// structure, scheduled by the compiler.  Every wavefront reports the shader
// cycles of its loop.
// ---------------------------------------------------------------------------
__device__ __forceinline__ probe_f32x4 probe_mfma(uint4 a, uint4 b, probe_f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(probe_bf16x8, a),
                                                   __builtin_bit_cast(probe_bf16x8, b), c, 0, 0, 0);
}

__device__ __forceinline__ uint32_t probe_pack2(float a, float b)
{
    typedef float p_f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 p_bf16x2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(p_f32x2{a, b}, p_bf16x2));
}

template <int T, bool BAR, bool V64>
__device__ __forceinline__ void step_probe_wave(const unsigned char *lds, int iters, const uint4 *qsrc, float *out,
                                                long long *cyc)
{
    const int lane = threadIdx.x & 63;
    uint4 qf[T][4];
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
        for (int k = 0; k < 4; ++k) qf[t][k] = qsrc[(lane + 64 * (t * 4 + k)) & 1023];
    probe_f32x4 O[T][9];
    float m[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        m[t] = 3.0f + t;
#pragma unroll
        for (int u = 0; u < 9; ++u) O[t][u] = probe_f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const uint4 ones = make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u);
    const long long c0 = clock64();
    for (int it = 0; it < iters; ++it) {
        const unsigned char *Kb = lds + (it & 1) * 8192 + lane * 16;
        uint4 kf[2][4];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) kf[kt][kk] = *reinterpret_cast<const uint4 *>(Kb + (kt * 4 + kk) * 1024);
        uint4 pf[T];
#pragma unroll
        for (int t = 0; t < T; ++t) {
            probe_f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                s0 = probe_mfma(kf[0][kk], qf[t][kk], s0);
                s1 = probe_mfma(kf[1][kk], qf[t][kk], s1);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                s0[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s0[r], 0.127f, -m[t]));
                s1[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s1[r], 0.127f, -m[t]));
            }
            pf[t] = make_uint4(probe_pack2(s0[0], s0[1]), probe_pack2(s0[2], s0[3]), probe_pack2(s1[0], s1[1]),
                               probe_pack2(s1[2], s1[3]));
        }
        uint4 vf[8];
        if constexpr (V64) {
            const unsigned char *Vh = lds + 16384 + (it & 1) * 8192 + lane * 8;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const uint2 lo = *reinterpret_cast<const uint2 *>(Vh + u * 1024);
                const uint2 hi = *reinterpret_cast<const uint2 *>(Vh + u * 1024 + 512);
                vf[u] = make_uint4(lo.x, lo.y, hi.x, hi.y);
            }
        } else {
            const unsigned char *Vb = lds + 16384 + (it & 1) * 8192 + lane * 16;
#pragma unroll
            for (int u = 0; u < 8; ++u) vf[u] = *reinterpret_cast<const uint4 *>(Vb + u * 1024);
        }
        if constexpr (BAR)
            if (it & 1) __syncthreads();              // every wavefront of the workgroup runs the same number of steps
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int t = 0; t < T; ++t) O[t][u] = probe_mfma(vf[u], pf[t], O[t][u]);
#pragma unroll
        for (int t = 0; t < T; ++t) O[t][8] = probe_mfma(ones, pf[t], O[t][8]);
    }
    const long long c1 = clock64();
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
        for (int u = 0; u < 9; ++u) s += O[t][u][0] + O[t][u][3];
    out[blockIdx.x * 512 + threadIdx.x] = s;
    if (lane == 0) cyc[blockIdx.x * 8 + (threadIdx.x >> 6)] = c1 - c0;
}

template <bool BAR, bool V64, int TA, int TB>
__global__ void __launch_bounds__(512) step_probe_kernel(const uint4 *src, int iters, float *out, long long *cyc)
{
    __shared__ unsigned char lds[32768];
    for (int i = threadIdx.x; i < 2048; i += 512) reinterpret_cast<uint4 *>(lds)[i] = src[i & 1023];
    __syncthreads();
    if (threadIdx.x < 256) step_probe_wave<TA, BAR, V64>(lds, iters, src, out, cyc);
    else step_probe_wave<TB, BAR, V64>(lds, iters, src, out, cyc);
}

// One wavefront: out[l] = max over the lanes {l, l^16, l^32, l^48} of in[.].
__global__ void __launch_bounds__(64) quad_max_kernel(const float *in, float *out)
{
    out[threadIdx.x] = quad_column_max(in[threadIdx.x]);
}

// ---------------------------------------------------------------------------
// The timeline hook's switch: a pointer and a capacity, read by the verify
// entry points at launch time.
// ---------------------------------------------------------------------------
static std::mutex g_tl_mutex;
static TimelineHook g_tl_hook = {nullptr, 0};

TimelineHook timeline_hook()
{
    std::lock_guard<std::mutex> lock(g_tl_mutex);    // pointer and capacity always belong together
    return g_tl_hook;
}

void set_timeline_hook(long long *buffer, long long capacity)
{
    std::lock_guard<std::mutex> lock(g_tl_mutex);
    g_tl_hook.buffer = buffer;
    g_tl_hook.capacity = buffer ? capacity : 0;
}

}  // namespace owl

using namespace owl;

namespace {
bool misaligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) % 16) != 0; }
}  // namespace

extern "C" {

owl_status owl_stream_read_probe(const void *src, size_t bytes, uint32_t *sink, int32_t n_workgroups, void *stream)
{
    if (!src || !sink || n_workgroups < 1 || bytes % 16 != 0 || misaligned16(src)) return OWL_ERR_INVALID_ARG;
    hipLaunchKernelGGL(stream_read_kernel, dim3(n_workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(src), bytes / 16, sink);
    return hipGetLastError() == hipSuccess ? OWL_OK : OWL_ERR_HIP;
}

owl_status owl_gather_read_probe(const void *src, const int32_t *block_order, int32_t n_blocks, uint32_t *sink,
                                 int32_t n_workgroups, void *stream)
{
    if (!src || !block_order || !sink || n_blocks < 1 || n_workgroups < 1 || misaligned16(src))
        return OWL_ERR_INVALID_ARG;
    hipLaunchKernelGGL(gather_read_kernel, dim3(n_workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(src), block_order, n_blocks, sink);
    return hipGetLastError() == hipSuccess ? OWL_OK : OWL_ERR_HIP;
}

owl_status owl_mfma_probe(const void *src, size_t bytes, int32_t iters, float *sink, float *clock_ghz,
                          int32_t n_workgroups, void *stream)
{
    if (!src || !sink || n_workgroups < 1 || iters < 1 || bytes < 16 || bytes % 16 != 0 ||
        bytes / 16 > 0x7fffffff || misaligned16(src))
        return OWL_ERR_INVALID_ARG;
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(n_workgroups), dim3(512), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(src), (int)(bytes / 16), iters, sink, clock_ghz);
    return hipGetLastError() == hipSuccess ? OWL_OK : OWL_ERR_HIP;
}

owl_status owl_selftest_quad_max(const float *in64, float *out64, void *stream)
{
    if (!in64 || !out64) return OWL_ERR_INVALID_ARG;
    hipLaunchKernelGGL(quad_max_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), in64, out64);
    return hipGetLastError() == hipSuccess ? OWL_OK : OWL_ERR_HIP;
}

owl_status owl_step_probe(int32_t variant, const void *src, int32_t iters, float *sink, long long *cycles,
                          int32_t n_workgroups, void *stream)
{
    if (!src || !sink || !cycles || iters < 2 || iters % 2 != 0 || n_workgroups < 1 || misaligned16(src))
        return OWL_ERR_INVALID_ARG;
    const dim3 grid(n_workgroups), block(512);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint4 *s4 = static_cast<const uint4 *>(src);
    switch (variant) {
    case OWL_STEP_PROBE_3_2: hipLaunchKernelGGL((step_probe_kernel<false, false, 3, 2>), grid, block, 0, st, s4, iters, sink, cycles); break;
    case OWL_STEP_PROBE_3_2_BARRIER: hipLaunchKernelGGL((step_probe_kernel<true, false, 3, 2>), grid, block, 0, st, s4, iters, sink, cycles); break;
    case OWL_STEP_PROBE_3_2_V64: hipLaunchKernelGGL((step_probe_kernel<false, true, 3, 2>), grid, block, 0, st, s4, iters, sink, cycles); break;
    case OWL_STEP_PROBE_3_2_BARRIER_V64: hipLaunchKernelGGL((step_probe_kernel<true, true, 3, 2>), grid, block, 0, st, s4, iters, sink, cycles); break;
    case OWL_STEP_PROBE_2_2: hipLaunchKernelGGL((step_probe_kernel<false, false, 2, 2>), grid, block, 0, st, s4, iters, sink, cycles); break;
    case OWL_STEP_PROBE_2_2_BARRIER_V64: hipLaunchKernelGGL((step_probe_kernel<true, true, 2, 2>), grid, block, 0, st, s4, iters, sink, cycles); break;
    default: return OWL_ERR_INVALID_ARG;
    }
    return hipGetLastError() == hipSuccess ? OWL_OK : OWL_ERR_HIP;
}

owl_status owl_debug_set_timeline(long long *buffer, int64_t n_workgroups)
{
    if (buffer && n_workgroups < 1) return OWL_ERR_INVALID_ARG;
    set_timeline_hook(buffer, buffer ? (long long)n_workgroups : 0);
    return OWL_OK;
}

}  // extern "C"
