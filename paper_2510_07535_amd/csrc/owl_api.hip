// Host side of the C ABI: argument checks, the split plan, kernel launches.
#include <math.h>
#include <string.h>

#include <atomic>
#include <mutex>

#include "owl_internal.h"
#include "owl_probe.h"

using namespace owl;

namespace {

int elem_size(int dtype) { return dtype == OWL_F32 ? 4 : 2; }

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Compute units of the current device; 256 (an MI355X) when no device answers,
// so that planning stays usable for host-only checks.
int device_cus()
{
    static std::atomic<int> cached[16];            // zero-initialised; callers may be on any thread
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return 256;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

owl_status check_desc(const owl_verify_desc *d)
{
    if (!d) return OWL_ERR_INVALID_ARG;
    if (d->batch < 1 || d->n_draft < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1) return OWL_ERR_INVALID_ARG;
    if (d->n_draft > 64) return OWL_ERR_TOO_MANY_DRAFT;
    if (d->n_q_heads % d->n_kv_heads) return OWL_ERR_INVALID_ARG;
    if (d->qkv_dtype != OWL_BF16 && d->qkv_dtype != OWL_F32 && d->qkv_dtype != OWL_F16) return OWL_ERR_UNSUPPORTED;
    if (d->head_dim != 64 && d->head_dim != 128) return OWL_ERR_UNSUPPORTED;
    if (d->page_size != kPage) return OWL_ERR_UNSUPPORTED;
    if (d->max_ctx_len < 0 || d->max_ctx_len > (1 << 30)) return OWL_ERR_INVALID_ARG;
    if (d->max_pages_per_seq < 0 || d->n_pool_pages < 1) return OWL_ERR_INVALID_ARG;
    if (d->split_tokens < 0) return OWL_ERR_INVALID_ARG;
    if (d->out_dtype != OWL_F32 && d->out_dtype != OWL_BF16 && d->out_dtype != OWL_F16) return OWL_ERR_UNSUPPORTED;
    if ((d->flags & ~(int32_t)OWL_FLAG_FP32_PARTIALS) != 0 || d->reserved_ != 0) return OWL_ERR_INVALID_ARG;
    if (!(d->scale > 0.0f) || !isfinite(d->scale)) return OWL_ERR_INVALID_ARG;
    const int es = elem_size(d->qkv_dtype);
    const int64_t st[3] = {d->kv_stride_page, d->kv_stride_head, d->kv_stride_token};
    for (int64_t s : st)
        if (s < 0 || (s * es) % 16 != 0) return OWL_ERR_INVALID_ARG;
    if (d->kv_stride_token < d->head_dim) return OWL_ERR_INVALID_ARG;
    if ((int64_t)d->n_q_heads / d->n_kv_heads * d->n_draft > 64 * 64) return OWL_ERR_UNSUPPORTED;
    return OWL_OK;
}

struct FullPlan {
    owl_plan pub;
    const Variant *variant;
    size_t part_o_bytes, part_ml_bytes, plan_bytes;
    bool half_partials;       // normalised fp16 partials (16-bit inputs unless the caller asks for fp32 ones)
    int32_t adapt, c_min, group_tiles;
    int64_t item_slots;       // adapt == 2: (sequence, split) pairs the grid has room for
    dim3 grid;                // of the split-KV pass
};

owl_status make_plan(const owl_verify_desc *d, FullPlan *fp)
{
    owl_status st = check_desc(d);
    if (st != OWL_OK) return st;
    const int G = d->n_q_heads / d->n_kv_heads;
    const int R = G * d->n_draft;
    const int RT = (R + kRowTile - 1) / kRowTile;
    const int64_t T = (int64_t)d->max_ctx_len + d->n_draft;
    // shortest split the planner uses: the fp16 partials of a split (R rows) stay below an eighth of the K/V it reads
    int64_t cmin = align_up((size_t)(4 * R), kSplitQuantum);
    if (cmin < 256) cmin = 256;
    // Eight wavefronts per workgroup: WR of them split the row tiles, WK the
    // 32-key steps of a stage; a wave holds up to three tiles in accumulators.
    // A workgroup takes up to 4 (WK = 2) or 8, 16, 24 (WK = 1) row tiles; more
    // tiles than that go to further row groups, workgroups that read the same
    // split.  Few KV streams (one or two KV heads of a tensor-parallel shard, one
    // sequence) cannot fill the chip by splits alone without the partials
    // outgrowing the K/V they summarise: then the rows are cut into more, smaller
    // groups instead, each re-reading the split from its XCD's L2.
    int tpw, wr, wk, rgs, group_tiles;
    if (d->qkv_dtype == OWL_F32) {
        tpw = 1; wr = 8; wk = 1; rgs = (RT + 7) / 8;
        group_tiles = (RT + rgs - 1) / rgs;
    } else {
        static const int caps[4] = {24, 16, 8, 4};
        int li = RT <= 4 ? 3 : (RT <= 8 ? 2 : (RT <= 16 ? 1 : 0));
        const int64_t splits_at_most = d->split_tokens > 0
            ? (T + (int64_t)align_up((size_t)d->split_tokens, kSplitQuantum) - 1) / (int64_t)align_up((size_t)d->split_tokens, kSplitQuantum)
            : (T + cmin - 1) / cmin;
        const int64_t streams = (int64_t)d->batch * d->n_kv_heads * (splits_at_most < 1 ? 1 : splits_at_most);
        // (three quarters of the compute units will do: larger groups do more per K/V byte they read)
        while (li < 3 && 4 * streams * ((RT + caps[li] - 1) / caps[li]) < 3 * (int64_t)device_cus()) ++li;
        rgs = (RT + caps[li] - 1) / caps[li];
        group_tiles = (RT + rgs - 1) / rgs;
        rgs = (RT + group_tiles - 1) / group_tiles;
        if (caps[li] == 4) { tpw = 1; wr = 4; wk = 2; }
        else { wr = 8; wk = 1; tpw = (group_tiles + 7) / 8; }
    }
    const Variant *v = find_variant(d->qkv_dtype, d->head_dim, tpw, wr, wk);
    if (!v) return OWL_ERR_UNSUPPORTED;
    fp->group_tiles = group_tiles;
    int64_t C;
    if (d->split_tokens > 0) {
        C = align_up((size_t)d->split_tokens, kSplitQuantum);
    } else {
        // Enough workgroups to occupy every compute unit (several rounds when
        // many independent KV streams exist, which evens out ragged batches),
        // but splits long enough that the partials they write stay a small
        // fraction of the K/V bytes they read (ratio ~ R / 2C with fp16 partials).
        const int64_t streams = (int64_t)d->batch * d->n_kv_heads * rgs;
        const int rounds = streams >= 64 ? 4 : 1;
        const int64_t want = (int64_t)device_cus() * rounds;      // one workgroup per CU at a time
        // A single round must not spill a few workgroups into a second one.  With row groups the
        // kernel keeps the groups of a (KV head, split) on one XCD, streams dealt round-robin over
        // the eight XCDs: what has to fit is an XCD's share of the streams times the groups.
        int64_t S = (want + streams - 1) / streams;
        if (rounds == 1) {
            S = want / streams;
            if (rgs > 1) {
                const int64_t per_xcd = device_cus() / 8 / rgs;              // streams an XCD can hold at once
                const int64_t heads = (int64_t)d->batch * d->n_kv_heads;
                if (per_xcd >= 1 && 8 * per_xcd / heads >= 1) S = 8 * per_xcd / heads;
            }
        }
        if (S < 1) S = 1;
        C = align_up((size_t)((T + S - 1) / S), kSplitQuantum);
        if (C < cmin) C = cmin;
    }
    if (C > kMaxSplitTokens) C = kMaxSplitTokens;
    if (C < kSplitQuantum) C = kSplitQuantum;
    int64_t max_splits = (T + C - 1) / C;
    // One sequence and a library-chosen split size: the kernels cut a context
    // shorter than max_ctx_len into the same number of splits (never below the
    // minimum used above), so the launch still fills the chip.
    // A batch with a library-chosen size: the kernels shrink the split so that the real
    // (ragged) lengths fill whole rounds of workgroups (batch_split_tokens).  Going from
    // k-and-a-bit rounds to k + 1 full ones never needs less than half the planned size,
    // so the grid and the partials are sized for splits of C / 2.
    fp->adapt = d->split_tokens != 0 ? 0 : (d->batch == 1 ? 1 : 2);
    fp->c_min = (int32_t)(cmin < C ? cmin : C);
    fp->item_slots = (int64_t)d->batch * max_splits;
    if (fp->adapt == 2) {
        // The device never asks for more pairs than the planned size gives at full length,
        // rounded up to whole rounds, plus one per sequence for rounding: that many slots,
        // numbered densely, are launched; a single sequence may use up to twice its share.
        const int64_t streams = (int64_t)d->n_kv_heads * rgs;
        fp->item_slots = (int64_t)d->batch * max_splits + (device_cus() + streams - 1) / streams + d->batch;
        int64_t c_floor = align_up((size_t)(C / 2), kSplitQuantum);
        if (c_floor < fp->c_min) c_floor = fp->c_min;
        max_splits = (T + c_floor - 1) / c_floor;
        if (fp->item_slots > (int64_t)d->batch * max_splits) fp->item_slots = (int64_t)d->batch * max_splits;
    }

    const size_t slots = (size_t)d->batch * d->n_kv_heads * (size_t)max_splits * RT;
    fp->half_partials = d->qkv_dtype != OWL_F32 && !(d->flags & OWL_FLAG_FP32_PARTIALS);
    fp->part_o_bytes = align_up(slots * (size_t)d->head_dim * kRowTile * (fp->half_partials ? 2 : 4), 256);
    fp->part_ml_bytes = align_up(slots * kPartMl * sizeof(float), 256);
    fp->variant = v;
    owl_plan &pl = fp->pub;
    pl.reserved_ = 0;
    pl.split_tokens = (int32_t)C;
    pl.max_splits = (int32_t)max_splits;
    pl.rows_per_kv = R;
    pl.row_tiles = RT;
    pl.row_groups = rgs;
    pl.tiles_per_wave = tpw;
    pl.kernel_variant = variant_index(v);
    // KV heads vary fastest (see the kernel's block-index comment); for a batch with a library-chosen
    // split size (y, z) merely number its (sequence, split) pairs densely
    // With row groups the kernel deals the workgroups out in units of eight (KV head, split, sequence)
    // streams: the grid is padded so that their number is a multiple of 8 (the surplus exits at once).
    int64_t grid_y = max_splits;
    if (rgs > 1)
        while (((int64_t)d->n_kv_heads * grid_y * d->batch) % 8 != 0) ++grid_y;
    fp->grid = dim3(d->n_kv_heads * rgs, (unsigned)grid_y, d->batch);
    if (fp->adapt == 2) {
        int64_t per_z = fp->item_slots < 32768 ? fp->item_slots : 32768;
        if (rgs > 1) per_z = (per_z + 7) / 8 * 8;
        fp->grid = dim3(d->n_kv_heads * rgs, (unsigned)per_z, (unsigned)((fp->item_slots + per_z - 1) / per_z));
    }
    if ((int64_t)fp->grid.x * fp->grid.y * fp->grid.z >= ((int64_t)1 << 31)) return OWL_ERR_UNSUPPORTED;   // the kernel numbers them in 32 bits
    pl.n_workgroups = (int32_t)((int64_t)fp->grid.x * fp->grid.y * fp->grid.z);
    fp->plan_bytes = align_up(((size_t)d->batch + 3) * sizeof(int32_t), 256);     // the batch plan
    pl.workspace_bytes = fp->part_o_bytes + fp->part_ml_bytes + fp->plan_bytes;
    return OWL_OK;
}

// Kernels that need more than the default dynamic LDS must say so once per
// device before their first launch.
owl_status ensure_lds_attr(const Variant *v)
{
    static std::mutex mu;
    static bool done[16][64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return OWL_ERR_HIP;
    const int vi = variant_index(v);
    if (dev < 0 || dev >= 16 || vi < 0 || vi >= 64) return OWL_ERR_HIP;
    std::lock_guard<std::mutex> lock(mu);
    if (!done[dev][vi]) {
        if (hipFuncSetAttribute(v->func, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)v->lds_bytes) != hipSuccess)
            return OWL_ERR_HIP;
        done[dev][vi] = true;
    }
    return OWL_OK;
}

// Device memory of owl_verify_attn_noalloc: the split partials live here instead of in a
// caller's workspace.  One copy per GPU that loads the library, held until the process ends.
// In host code the array's name is only a handle: its device address comes from
// hipGetSymbolAddress, once per device (scratch_address), and only that address is ever
// handed to a kernel.
static __device__ __align__(256) unsigned char scratch[OWL_NOALLOC_SCRATCH_BYTES];

owl_status scratch_address(void **out)
{
    static std::mutex mu;
    static void *addr[16] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return OWL_ERR_HIP;
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return OWL_ERR_HIP;
        addr[dev] = ptr;
    }
    *out = addr[dev];
    return OWL_OK;
}

bool misaligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) != 0; }

}  // namespace

extern "C" {

owl_status owl_verify_attn_plan(const owl_verify_desc *desc, owl_plan *plan)
{
    if (!plan) return OWL_ERR_INVALID_ARG;
    FullPlan fp;
    owl_status st = make_plan(desc, &fp);
    if (st != OWL_OK) return st;
    *plan = fp.pub;
    return OWL_OK;
}

owl_status owl_verify_attn_workspace_size(const owl_verify_desc *desc, size_t *bytes)
{
    if (!bytes) return OWL_ERR_INVALID_ARG;
    FullPlan fp;
    owl_status st = make_plan(desc, &fp);
    if (st != OWL_OK) return st;
    *bytes = fp.pub.workspace_bytes;
    return OWL_OK;
}

owl_status owl_verify_attn(const owl_verify_desc *desc, const void *q, const void *k_cache,
                           const void *v_cache, const int32_t *page_table,
                           const int32_t *ctx_lens, const int32_t *tree_parent, void *out,
                           void *workspace, size_t workspace_bytes, uint32_t *dev_status,
                           void *stream)
{
    return owl_verify_attn_phases(desc, q, k_cache, v_cache, page_table, ctx_lens, tree_parent, out,
                                  workspace, workspace_bytes, dev_status, stream, OWL_PHASE_ALL);
}

static owl_status verify_impl(const owl_verify_desc *desc, const void *q, const void *k_cache,
                              const void *v_cache, const int32_t *page_table, const int32_t *ctx_lens,
                              const int32_t *tree_parent, const int32_t *n_draft_seq, void *out,
                              void *workspace, size_t workspace_bytes, uint32_t *dev_status, void *stream,
                              int32_t phases, hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);

owl_status owl_verify_attn_phases(const owl_verify_desc *desc, const void *q, const void *k_cache,
                                  const void *v_cache, const int32_t *page_table,
                                  const int32_t *ctx_lens, const int32_t *tree_parent, void *out,
                                  void *workspace, size_t workspace_bytes, uint32_t *dev_status,
                                  void *stream, int32_t phases)
{
    return verify_impl(desc, q, k_cache, v_cache, page_table, ctx_lens, tree_parent, nullptr, out, workspace,
                       workspace_bytes, dev_status, stream, phases);
}

owl_status owl_verify_attn_ragged(const owl_verify_desc *desc, const void *q, const void *k_cache,
                                  const void *v_cache, const int32_t *page_table,
                                  const int32_t *ctx_lens, const int32_t *tree_parent,
                                  const int32_t *n_draft_seq, void *out, void *workspace,
                                  size_t workspace_bytes, uint32_t *dev_status, void *stream)
{
    if (!n_draft_seq) return OWL_ERR_INVALID_ARG;
    return verify_impl(desc, q, k_cache, v_cache, page_table, ctx_lens, tree_parent, n_draft_seq, out,
                       workspace, workspace_bytes, dev_status, stream, OWL_PHASE_ALL);
}

static owl_status verify_impl(const owl_verify_desc *desc, const void *q, const void *k_cache,
                              const void *v_cache, const int32_t *page_table, const int32_t *ctx_lens,
                              const int32_t *tree_parent, const int32_t *n_draft_seq, void *out,
                              void *workspace, size_t workspace_bytes, uint32_t *dev_status, void *stream,
                              int32_t phases, hipEvent_t ev_start, hipEvent_t ev_stop)
{
    if (phases < 1 || phases > OWL_PHASE_ALL) return OWL_ERR_INVALID_ARG;
    FullPlan fp;
    owl_status st = make_plan(desc, &fp);
    if (st != OWL_OK) return st;
    if (!q || !k_cache || !v_cache || !ctx_lens || !tree_parent || !out) return OWL_ERR_INVALID_ARG;
    if (misaligned(q, 16) || misaligned(k_cache, 16) || misaligned(v_cache, 16) || misaligned(out, 16))
        return OWL_ERR_INVALID_ARG;
    if (page_table &&
        (int64_t)desc->max_pages_per_seq * kPage < (int64_t)desc->max_ctx_len + desc->n_draft)
        return OWL_ERR_INVALID_ARG;
    if (!workspace || workspace_bytes < fp.pub.workspace_bytes) return OWL_ERR_WORKSPACE;
    if (misaligned(workspace, 256)) return OWL_ERR_INVALID_ARG;

    // the profiling copy of the kernel, if the timeline hook is on and has room for this grid
    const Variant *variant = fp.variant;
    const TimelineHook hook = timeline_hook();
    if (hook.buffer && fp.pub.n_workgroups <= hook.capacity) {
        const Variant *tv = find_variant(variant->dtype, variant->D, variant->tpw, variant->wr, variant->wk, true);
        if (tv) variant = tv;
    }
    st = ensure_lds_attr(variant);
    if (st != OWL_OK) return st;

    // workspace: partial O | partial (m, l, s) | batch plan
    char *ws = static_cast<char *>(workspace);
    KParams p;
    memset(&p, 0, sizeof p);
    p.q = q; p.k = k_cache; p.v = v_cache;
    p.page_table = page_table; p.ctx_lens = ctx_lens; p.parent = tree_parent;
    p.n_draft_seq = n_draft_seq;
    p.part_o = ws;
    p.half_partials = fp.half_partials ? 1 : 0;
    p.part_ml = reinterpret_cast<float *>(ws + fp.part_o_bytes);
    p.dev_c = reinterpret_cast<int32_t *>(ws + fp.part_o_bytes + fp.part_ml_bytes);
    p.out = out;
    p.out_dtype = desc->out_dtype;
    p.dev_status = dev_status;
    p.B = desc->batch; p.N = desc->n_draft; p.Hq = desc->n_q_heads; p.Hkv = desc->n_kv_heads;
    p.G = p.Hq / p.Hkv; p.R = fp.pub.rows_per_kv;
    p.max_pages = desc->max_pages_per_seq; p.max_ctx_len = desc->max_ctx_len;
    p.C = fp.pub.split_tokens; p.max_splits = fp.pub.max_splits;
    p.adapt = fp.adapt; p.c_min = fp.c_min;
    p.n_cu = device_cus();
    p.RT = fp.pub.row_tiles; p.row_groups = fp.pub.row_groups; p.group_tiles = fp.group_tiles;
    p.stride_page = desc->kv_stride_page; p.stride_head = desc->kv_stride_head;
    p.stride_token = desc->kv_stride_token; p.n_pool_pages = desc->n_pool_pages;
    p.c_log2 = desc->scale * 1.4426950408889634f;
    p.timeline = variant->timeline ? hook.buffer : nullptr;

    hipStream_t s = static_cast<hipStream_t>(stream);
    p.item_slots = (int32_t)fp.item_slots;
    const dim3 grid = fp.grid;
    if (phases & OWL_PHASE_SPLIT) {
        if (p.adapt == 2 && launch_batch_plan(p, s) != hipSuccess) return OWL_ERR_HIP;
        variant->launch(p, grid, s, ev_start, ev_stop);
        if (hipGetLastError() != hipSuccess) return OWL_ERR_HIP;
    }
    if (phases & OWL_PHASE_COMBINE)
        if (launch_combine(p, desc->head_dim, fp.half_partials, s) != hipSuccess) return OWL_ERR_HIP;
    return OWL_OK;
}

// ---- measurement aids that need the verify path itself (declared in owl_probe.h) ----
owl_status owl_verify_attn_split_timed(const owl_verify_desc *desc, const void *q, const void *k_cache,
                                       const void *v_cache, const int32_t *page_table, const int32_t *ctx_lens,
                                       const int32_t *tree_parent, void *out, void *workspace, size_t workspace_bytes,
                                       uint32_t *dev_status, void *stream, void *start_event, void *stop_event)
{
    if (!start_event || !stop_event) return OWL_ERR_INVALID_ARG;
    return verify_impl(desc, q, k_cache, v_cache, page_table, ctx_lens, tree_parent, nullptr, out, workspace,
                       workspace_bytes, dev_status, stream, OWL_PHASE_SPLIT, static_cast<hipEvent_t>(start_event),
                       static_cast<hipEvent_t>(stop_event));
}

owl_status owl_probe_event_create(void **event)
{
    if (!event) return OWL_ERR_INVALID_ARG;
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return OWL_ERR_HIP;
    *event = e;
    return OWL_OK;
}

owl_status owl_probe_event_destroy(void *event)
{
    if (!event) return OWL_ERR_INVALID_ARG;
    return hipEventDestroy(static_cast<hipEvent_t>(event)) == hipSuccess ? OWL_OK : OWL_ERR_HIP;
}

owl_status owl_probe_event_elapsed_ms(void *start_event, void *stop_event, float *ms_host)
{
    if (!start_event || !stop_event || !ms_host) return OWL_ERR_INVALID_ARG;
    if (hipEventSynchronize(static_cast<hipEvent_t>(stop_event)) != hipSuccess) return OWL_ERR_HIP;
    return hipEventElapsedTime(ms_host, static_cast<hipEvent_t>(start_event), static_cast<hipEvent_t>(stop_event)) == hipSuccess
               ? OWL_OK : OWL_ERR_HIP;
}

owl_status owl_verify_attn_init(const owl_verify_desc *desc)
{
    FullPlan fp;
    owl_status st = make_plan(desc, &fp);
    if (st != OWL_OK) return st;
    st = ensure_lds_attr(fp.variant);
    if (st != OWL_OK) return st;
    if (load_aux_kernels() != hipSuccess) return OWL_ERR_HIP;
    void *ptr = nullptr;
    return scratch_address(&ptr);
}

owl_status owl_verify_attn_noalloc(const owl_verify_desc *desc, const void *q, const void *k_cache,
                                   const void *v_cache, const int32_t *page_table, const int32_t *ctx_lens,
                                   const int32_t *tree_parent, void *out, uint32_t *dev_status, void *stream)
{
    FullPlan fp;
    owl_status st = make_plan(desc, &fp);
    if (st != OWL_OK) return st;
    if (fp.pub.workspace_bytes > (size_t)OWL_NOALLOC_SCRATCH_BYTES) return OWL_ERR_WORKSPACE;
    void *ptr = nullptr;
    st = scratch_address(&ptr);
    if (st != OWL_OK) return st;
    return verify_impl(desc, q, k_cache, v_cache, page_table, ctx_lens, tree_parent, nullptr, out, ptr,
                       (size_t)OWL_NOALLOC_SCRATCH_BYTES, dev_status, stream, OWL_PHASE_ALL);
}

owl_status owl_build_tree_mask(const int32_t *tree_parent, int32_t batch, int32_t n_draft,
                               uint64_t *anc_mask, int32_t *depth, uint32_t *dev_status,
                               void *stream)
{
    if (!tree_parent || !anc_mask || batch < 1 || n_draft < 1) return OWL_ERR_INVALID_ARG;
    if (n_draft > 64) return OWL_ERR_TOO_MANY_DRAFT;
    if (launch_tree_mask(tree_parent, batch, n_draft, anc_mask, depth, dev_status,
                         static_cast<hipStream_t>(stream)) != hipSuccess)
        return OWL_ERR_HIP;
    return OWL_OK;
}

owl_status owl_prepare_spec_tree(const int32_t *tree_parent, const int32_t *ctx_lens, int32_t batch,
                                 int32_t n_nodes, int32_t *tree_parent2, uint64_t *anc_mask,
                                 int32_t *depth, int32_t *pos_ids, uint32_t *dev_status, void *stream)
{
    if (!tree_parent || !ctx_lens || !tree_parent2 || !anc_mask || batch < 1 || n_nodes < 1)
        return OWL_ERR_INVALID_ARG;
    if (n_nodes > 32) return OWL_ERR_TOO_MANY_DRAFT;
    if (launch_prepare(tree_parent, ctx_lens, batch, n_nodes, tree_parent2, anc_mask, depth, pos_ids,
                       dev_status, static_cast<hipStream_t>(stream)) != hipSuccess)
        return OWL_ERR_HIP;
    return OWL_OK;
}

owl_status owl_accept_greedy(const int32_t *tokens, const int32_t *tree_parent, const int32_t *target_root,
                             const int32_t *target_next, int32_t batch, int32_t n_draft, int32_t n_cand,
                             int32_t *accepted, int32_t *n_accept, int32_t *bonus, int32_t *last,
                             uint32_t *dev_status, void *stream)
{
    if (!tokens || !tree_parent || !target_root || !target_next || !accepted || !n_accept || !bonus || !last)
        return OWL_ERR_INVALID_ARG;
    if (batch < 1 || n_draft < 1 || n_cand < 0 || n_cand > n_draft) return OWL_ERR_INVALID_ARG;
    if (n_draft > 64) return OWL_ERR_TOO_MANY_DRAFT;
    if (launch_accept(tokens, tree_parent, target_root, target_next, batch, n_draft, n_cand, accepted,
                      n_accept, bonus, last, dev_status, static_cast<hipStream_t>(stream)) != hipSuccess)
        return OWL_ERR_HIP;
    return OWL_OK;
}

owl_status owl_commit_kv(const owl_verify_desc *desc, void *k_cache, void *v_cache, const int32_t *page_table,
                         const int32_t *ctx_lens, const int32_t *accepted, const int32_t *n_accept,
                         int32_t *new_ctx_lens, uint32_t *dev_status, void *stream)
{
    owl_status st = check_desc(desc);
    if (st != OWL_OK) return st;
    if (!k_cache || !v_cache || !ctx_lens || !accepted || !n_accept) return OWL_ERR_INVALID_ARG;
    if (new_ctx_lens == ctx_lens) return OWL_ERR_INVALID_ARG;
    if (misaligned(k_cache, 16) || misaligned(v_cache, 16)) return OWL_ERR_INVALID_ARG;
    if (page_table &&
        (int64_t)desc->max_pages_per_seq * kPage < (int64_t)desc->max_ctx_len + desc->n_draft)
        return OWL_ERR_INVALID_ARG;
    if (launch_commit(*desc, k_cache, v_cache, page_table, ctx_lens, accepted, n_accept, new_ctx_lens,
                      dev_status, static_cast<hipStream_t>(stream)) != hipSuccess)
        return OWL_ERR_HIP;
    return OWL_OK;
}

static owl_status check_drafter(const owl_drafter_desc *d)
{
    if (!d) return OWL_ERR_INVALID_ARG;
    if (d->d_in < 1 || d->d < 1 || d->n_states < 1 || d->n_rows < 1 || d->vocab < 1) return OWL_ERR_INVALID_ARG;
    if (!(d->eps >= 0.f) || d->alpha != d->alpha) return OWL_ERR_INVALID_ARG;
    if (d->n_states > 64 || d->n_rows > 64) return OWL_ERR_TOO_MANY_DRAFT;
    if (d->dtype != OWL_BF16 && d->dtype != OWL_F16) return OWL_ERR_UNSUPPORTED;
    if (d->d_in % 32 != 0 || d->d % 16 != 0 || d->d > 16384 || d->d_in > (1 << 20)) return OWL_ERR_UNSUPPORTED;
    if (d->w_layout != OWL_W_ROWS && d->w_layout != OWL_W_TILED) return OWL_ERR_UNSUPPORTED;
    return OWL_OK;
}

owl_status owl_drafter_tiled_weight_bytes(const owl_drafter_desc *desc, size_t *bytes)
{
    owl_status st = check_drafter(desc);
    if (st != OWL_OK) return st;
    if (!bytes) return OWL_ERR_INVALID_ARG;
    *bytes = drafter_tiled_bytes(desc->d_in, desc->d);
    return OWL_OK;
}

owl_status owl_drafter_tile_weights(const owl_drafter_desc *desc, const void *w_rows, void *w_tiled, void *stream)
{
    owl_status st = check_drafter(desc);
    if (st != OWL_OK) return st;
    if (!w_rows || !w_tiled || misaligned(w_rows, 16) || misaligned(w_tiled, 16)) return OWL_ERR_INVALID_ARG;
    if (launch_drafter_tile_weights(w_rows, w_tiled, desc->d_in, desc->d, static_cast<hipStream_t>(stream)) !=
        hipSuccess)
        return OWL_ERR_HIP;
    return OWL_OK;
}

owl_status owl_drafter_cell_workspace_size(const owl_drafter_desc *desc, size_t *bytes)
{
    owl_status st = check_drafter(desc);
    if (st != OWL_OK) return st;
    if (!bytes) return OWL_ERR_INVALID_ARG;
    // the projections [P][4d], then the chunk statistics of the two normalisations
    *bytes = ((size_t)desc->n_states * 4 * desc->d + drafter_gate_scratch_floats(desc->n_rows)) * sizeof(float);
    return OWL_OK;
}

owl_status owl_drafter_cell_phases(const owl_drafter_desc *desc, const void *h, const float *z,
                                   const int32_t *tokens, const int32_t *parent_row, const void *w,
                                   const void *emb, const float *gamma_c, const float *beta_c,
                                   const float *gamma_z, const float *beta_z, void *h_out, float *h_out_f32,
                                   float *z_out, void *workspace, size_t workspace_bytes, uint32_t *dev_status,
                                   void *stream, int32_t phases)
{
    owl_status st = check_drafter(desc);
    if (st != OWL_OK) return st;
    if (!h || !z || !tokens || !w || !emb || !z_out) return OWL_ERR_INVALID_ARG;
    if (phases < 1 || phases > OWL_DRAFTER_ALL) return OWL_ERR_INVALID_ARG;
    if (!parent_row && desc->n_rows != desc->n_states) return OWL_ERR_INVALID_ARG;
    for (const void *ptr : {h, (const void *)z, w, emb, (const void *)gamma_c, (const void *)beta_c,
                            (const void *)gamma_z, (const void *)beta_z, (const void *)h_out,
                            (const void *)h_out_f32, (const void *)z_out, (const void *)workspace})
        if (misaligned(ptr, 16)) return OWL_ERR_INVALID_ARG;      // a null pointer counts as aligned
    size_t need = 0;
    owl_drafter_cell_workspace_size(desc, &need);
    if (!workspace || workspace_bytes < need) return OWL_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *proj = static_cast<float *>(workspace);
    if (phases & OWL_DRAFTER_PROJ)
        if (launch_drafter_proj(desc->dtype, h, w, desc->w_layout == OWL_W_TILED, proj, desc->n_states, desc->d_in,
                                desc->d, s) != hipSuccess)
            return OWL_ERR_HIP;
    if (phases & OWL_DRAFTER_GATES)
        if (launch_drafter_gates(desc->dtype, proj, z, tokens, parent_row, emb, gamma_c, beta_c, gamma_z, beta_z,
                                 h_out, h_out_f32, z_out, proj + (size_t)desc->n_states * 4 * desc->d, desc->n_states,
                                 desc->n_rows, desc->d, desc->vocab,
                                 desc->alpha, desc->eps, dev_status, s) != hipSuccess)
            return OWL_ERR_HIP;
    return OWL_OK;
}

owl_status owl_drafter_cell(const owl_drafter_desc *desc, const void *h, const float *z, const int32_t *tokens,
                            const int32_t *parent_row, const void *w, const void *emb, const float *gamma_c,
                            const float *beta_c, const float *gamma_z, const float *beta_z, void *h_out,
                            float *h_out_f32, float *z_out, void *workspace, size_t workspace_bytes,
                            uint32_t *dev_status, void *stream)
{
    return owl_drafter_cell_phases(desc, h, z, tokens, parent_row, w, emb, gamma_c, beta_c, gamma_z, beta_z, h_out,
                                   h_out_f32, z_out, workspace, workspace_bytes, dev_status, stream,
                                   OWL_DRAFTER_ALL);
}

owl_status owl_drafter_alpha(int32_t max_depth, int32_t d, float *alpha_host)
{
    if (max_depth < 1 || d < 1 || !alpha_host) return OWL_ERR_INVALID_ARG;
    const double a0 = exp2(-1.0 / (2.0 * (double)max_depth));
    *alpha_host = (float)(2.0 * a0 / ((1.0 - a0 * a0) * (double)d));
    return OWL_OK;
}

owl_status owl_build_tree_mask_host(const int32_t *parent, int32_t n_draft, uint64_t *anc,
                                    int32_t *depth)
{
    if (!parent || !anc || n_draft < 1) return OWL_ERR_INVALID_ARG;
    if (n_draft > 64) return OWL_ERR_TOO_MANY_DRAFT;
    for (int i = 0; i < n_draft; ++i)
        if (parent[i] < -1 || parent[i] >= i) return OWL_ERR_BAD_TREE;
    // parents come first, so one forward sweep suffices
    for (int i = 0; i < n_draft; ++i) {
        const int pi = parent[i];
        anc[i] = ((uint64_t)1 << i) | (pi >= 0 ? anc[pi] : 0);
        if (depth) depth[i] = 1 + (pi >= 0 ? depth[pi] : 0);
    }
    return OWL_OK;
}

owl_status owl_gather_kv(const owl_verify_desc *desc, const void *cache, const int32_t *page_table,
                         int32_t seq, int64_t first_pos, int64_t n_tokens, void *dst,
                         uint32_t *dev_status, void *stream)
{
    owl_status st = check_desc(desc);
    if (st != OWL_OK) return st;
    if (!cache || !dst || seq < 0 || seq >= desc->batch || first_pos < 0 || n_tokens < 0)
        return OWL_ERR_INVALID_ARG;
    if (misaligned(cache, 16) || misaligned(dst, 16)) return OWL_ERR_INVALID_ARG;
    if (launch_gather(*desc, cache, page_table, seq, first_pos, n_tokens, dst, dev_status,
                      static_cast<hipStream_t>(stream)) != hipSuccess)
        return OWL_ERR_HIP;
    return OWL_OK;
}

const char *owl_status_str(owl_status s)
{
    switch (s) {
    case OWL_OK: return "ok";
    case OWL_ERR_INVALID_ARG: return "invalid argument";
    case OWL_ERR_BAD_TREE: return "tree_parent is not a forest in parent-first order";
    case OWL_ERR_TOO_MANY_DRAFT: return "n_draft exceeds 64";
    case OWL_ERR_UNSUPPORTED: return "unsupported head_dim, page_size, dtype or shape";
    case OWL_ERR_WORKSPACE: return "workspace missing or too small";
    case OWL_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

const char *owl_version(void) { return "0.2"; }

}  // extern "C"
