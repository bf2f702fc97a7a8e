// Internal declarations shared by the host layer and the kernel translation
// units of the verify-attention library.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "owl.h"

namespace owl {

constexpr int kPage = 16;                 // tokens per cache page
constexpr int kRowTile = 16;              // query rows per MFMA tile
constexpr int kMaxSplitTokens = 16384;    // bounds the per-workgroup page list in LDS
constexpr int kMaxPagesPerSplit = kMaxSplitTokens / kPage;
constexpr int kSplitQuantum = 64;         // split_tokens is a multiple of every stage size

// Format of a split's partial, per 16-row tile ("slot").
//   fp32 inputs, and 16-bit inputs with OWL_FLAG_FP32_PARTIALS:
//                  O fragments as they stand, float4 [slot][channel tile][lane]; (m, l) in part_ml.
//   16-bit inputs: the NORMALISED output O / l of each row (a convex combination of V rows, so bounded by
//                  them), divided by s = its largest magnitude over the row's channels, as fp16:
//                  uint4 [slot][pair of channel tiles][lane] = 2 x 4 halves; (m, l, s) in part_ml.  Half the
//                  bytes to write and to read back; a value is stored to 2^-12 of its row's largest
//                  component whatever the magnitude of V, far below the bf16 rounding of P.
constexpr int kPartMl = 48;               // floats of part_ml per slot: m[16], l[16], s[16]

// Everything a kernel needs, passed by value.
struct KParams {
    const void *q, *k, *v;
    const int32_t *page_table, *ctx_lens, *parent;
    const int32_t *n_draft_seq;   // optional [B]: drafted tokens of each sequence (<= N), else null = N everywhere
    void *part_o;         // split partials: accumulator fragments (see kPartMl below)
    int32_t half_partials;// 1: normalised fp16 partials (16-bit inputs, the default), 0: raw fp32 fragments
    float *part_ml;       // split partials: per row reference m, row sum l and, for 16-bit partials, scale s
    void *out;            // [B][N][Hq][D] in out_dtype
    int32_t out_dtype;    // OWL_F32, OWL_BF16 or OWL_F16
    uint32_t *dev_status;
    int32_t B, N, Hq, Hkv, G, R;
    int32_t max_pages, max_ctx_len;
    int32_t C;            // tokens per split (an upper bound when `adapt` is set)
    int32_t adapt;        // library-chosen splits follow the actual lengths: 1 = the one sequence's, 2 = the batch's
    int32_t n_cu;         // compute units: the workgroup slots of one round
    int32_t item_slots;   // adapt == 2: (sequence, split) pairs the launched grid has room for
    int32_t *dev_c;       // adapt == 2: the batch plan (split size, pair count, pairs before each sequence)
    int32_t c_min;        // smallest split size the planner allows
    int32_t max_splits;
    int32_t RT;           // row tiles covering R
    int32_t row_groups;
    int32_t group_tiles;  // row tiles per row group (the last group may hold fewer)
    int64_t stride_page, stride_head, stride_token, n_pool_pages;
    float c_log2;         // scale * log2(e): scores live in the exp2 domain
    long long *timeline;  // instantiations with the timeline hook only: 10 slots per workgroup (profiling aid)
};

// One instantiated split-KV kernel.  `timeline` marks the copies that carry the
// per-workgroup timeline hook (profiling builds of the bf16 / D = 128 kernels);
// the production copies have no trace of it.
struct Variant {
    int dtype, D, tpw, wr, wk;
    bool timeline;
    size_t lds_bytes;
    // start / stop: optional events attached to the kernel's own dispatch (its begin and end), else null
    void (*launch)(const KParams &, dim3 grid, hipStream_t, hipEvent_t start, hipEvent_t stop);
    const void *func;     // for hipFuncSetAttribute
};

const Variant *find_variant(int dtype, int D, int tpw, int wr, int wk, bool timeline = false);
int variant_index(const Variant *v);

// Profiling hook state (set through the probe interface; read by the verify entry points).
struct TimelineHook {
    long long *buffer;    // device memory, 10 int64 per workgroup, or null
    long long capacity;   // workgroups the buffer has room for
};
TimelineHook timeline_hook();
void set_timeline_hook(long long *buffer, long long capacity);
hipError_t load_aux_kernels();
hipError_t launch_batch_plan(const KParams &p, hipStream_t s);

hipError_t launch_combine(const KParams &p, int D, bool half_partials, hipStream_t s);
hipError_t launch_prepare(const int32_t *parent, const int32_t *ctx_lens, int B, int n, int32_t *parent2,
                          uint64_t *anc, int32_t *depth, int32_t *pos, uint32_t *status, hipStream_t s);
hipError_t launch_accept(const int32_t *tokens, const int32_t *parent, const int32_t *target_root,
                         const int32_t *target_next, int B, int N, int n_cand, int32_t *accepted,
                         int32_t *n_accept, int32_t *bonus, int32_t *last, uint32_t *status, hipStream_t s);
hipError_t launch_commit(const owl_verify_desc &d, void *k_cache, void *v_cache, const int32_t *page_table,
                         const int32_t *ctx_lens, const int32_t *accepted, const int32_t *n_accept,
                         int32_t *new_ctx_lens, uint32_t *status, hipStream_t s);
hipError_t launch_drafter_proj(int dtype, const void *h, const void *w, bool tiled, float *s, int P, int d_in,
                               int d, hipStream_t st);
size_t drafter_tiled_bytes(int d_in, int d);
hipError_t launch_drafter_tile_weights(const void *w_rows, void *w_tiled, int d_in, int d, hipStream_t st);
hipError_t launch_drafter_gates(int dtype, const float *s, const float *z, const int32_t *tokens,
                                const int32_t *parent_row, const void *emb, const float *gamma_c,
                                const float *beta_c, const float *gamma_z, const float *beta_z, void *h_out,
                                float *h_out_f32, float *z_out, float *gate_scratch, int P, int M, int d, int vocab,
                                float alpha, float eps, uint32_t *status, hipStream_t st);
size_t drafter_gate_scratch_floats(int M);
hipError_t launch_tree_mask(const int32_t *parent, int B, int N, uint64_t *anc, int32_t *depth,
                            uint32_t *status, hipStream_t s);
hipError_t launch_gather(const owl_verify_desc &d, const void *cache, const int32_t *page_table,
                         int seq, int64_t first, int64_t n, void *dst, uint32_t *status,
                         hipStream_t s);

}  // namespace owl
