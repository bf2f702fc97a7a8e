/*
 * owl_probe.h -- measurement and self-test aids that ship in the same shared
 * library as the verify-step attention (owl.h) but are no part of its product
 * interface: kernels that measure what the chip sustains (a streaming read, a
 * gather read, the matrix pipe), a one-wavefront check of a cross-lane step of
 * the in-kernel softmax, and the switch of a per-workgroup timeline.  Used by
 * the benchmark and the tests.  Conventions as in owl.h: device pointers, the
 * caller owns every buffer, nothing allocates or synchronises.
 */
#ifndef OWL_PROBE_H_
#define OWL_PROBE_H_

#include "owl.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * A plain streaming read of `bytes` bytes (multiple of 16, 16-byte aligned) with
 * 128-bit loads by `n_workgroups` workgroups of 256 threads: every workgroup
 * walks one contiguous piece of the buffer with sixteen loads in flight per
 * thread and XOR-folds what it read into sink[workgroup] (uint32, device).  Its
 * achieved GB/s is what a streaming kernel can hope for on this chip, reported
 * next to the nominal HBM peak.
 */
owl_status owl_stream_read_probe(const void *src, size_t bytes, uint32_t *sink,
                                 int32_t n_workgroups, void *stream);

/*
 * The sustained rate of the matrix pipe.  n_workgroups
 * workgroups of 8 wavefronts issue `iters` x 16 bf16 16x16x32 MFMAs per lane on
 * operands read once from src (`bytes` bytes, a multiple of 16, 16-byte aligned,
 * interpreted as bf16 values; their bit patterns matter: under its power limit
 * this chip sustains a lower rate on random values than on constants).  Flop =
 * n_workgroups * 8 * iters * 16 * 16384.  sink: n_workgroups * 512 floats, device.
 * clock_ghz: optional, n_workgroups floats, device: the shader clock every
 * workgroup ran at over its loop (shader cycles per constant-rate 100 MHz tick),
 * which shows the throttling directly.
 */
owl_status owl_mfma_probe(const void *src, size_t bytes, int32_t iters, float *sink, float *clock_ghz,
                          int32_t n_workgroups, void *stream);

/*
 * Like owl_stream_read_probe, but the buffer is read in
 * 4 KiB blocks in the order block_order[0 .. n_blocks-1] (device int32, every
 * entry in [0, buffer bytes / 4096)).  With a random order this is the access
 * pattern of a head-major cache with 16-token pages of 128 bf16 channels
 * handed out at random, and its GB/s is the ceiling for that layout.
 */
owl_status owl_gather_read_probe(const void *src, const int32_t *block_order, int32_t n_blocks,
                                 uint32_t *sink, int32_t n_workgroups, void *stream);

/*
 * The instruction mix of one 32-key step of the split-KV fast loop (K fragments
 * from LDS, QK^T MFMAs, exp2 softmax, conversion, V fragments from LDS, PV and
 * row-sum MFMAs: 17 MFMAs of 16x16x32 per 16-row tile) on LDS- and
 * register-resident data, no HBM traffic: n_workgroups workgroups of 8 wavefronts
 * run `iters` (even, >= 2) steps; wavefronts 0..3 hold TA row tiles, 4..7 TB
 * (one of each per SIMD).  The variants differ in what the real loop adds:
 *     OWL_STEP_PROBE_3_2              3 + 2 tiles, nothing else
 *     OWL_STEP_PROBE_3_2_BARRIER      + a workgroup barrier every 64 keys
 *     OWL_STEP_PROBE_3_2_V64          + V fragments by 64-bit LDS reads
 *     OWL_STEP_PROBE_3_2_BARRIER_V64  + both (the real three-tile loop's structure)
 *     OWL_STEP_PROBE_2_2 / _2_2_BARRIER_V64   the same with 2 + 2 tiles
 * src: 16 KiB of bf16 operand values (device, 16-byte aligned); sink:
 * n_workgroups * 512 floats; cycles: n_workgroups * 8 int64, the shader cycles of
 * each wavefront's loop.  With T = TA + TB tiles per SIMD the matrix pipe needs
 * T * 17 * 16 cycles per step, so its busy fraction is that over cycles / iters.
 */
#define OWL_STEP_PROBE_3_2 0
#define OWL_STEP_PROBE_3_2_BARRIER 1
#define OWL_STEP_PROBE_3_2_V64 2
#define OWL_STEP_PROBE_3_2_BARRIER_V64 3
#define OWL_STEP_PROBE_2_2 4
#define OWL_STEP_PROBE_2_2_BARRIER_V64 5
owl_status owl_step_probe(int32_t variant, const void *src, int32_t iters, float *sink, long long *cycles,
                          int32_t n_workgroups, void *stream);

/*
 * Self-test of the cross-lane step of the in-kernel softmax: one wavefront
 * reads in64[64] and writes, for every lane l, the maximum over the lanes
 * {l, l^16, l^32, l^48} (the four lanes that hold the keys of one query row in
 * a 16x16 MFMA accumulator tile) to out64[64].  Device pointers.
 */
owl_status owl_selftest_quad_max(const float *in64, float *out64, void *stream);

/*
 * The split-KV pass of the verify step, i.e. OWL_PHASE_SPLIT of
 * owl_verify_attn_phases with the same arguments, with two HIP events attached to the kernel's own dispatch:
 * start_event is stamped when the kernel begins, stop_event when its last
 * workgroup has ended, so their difference is the duration of the kernel alone
 * (what a kernel trace reports), without the few microseconds that a pair of
 * hipEventRecord calls around a launch adds.  The events come from
 * owl_probe_event_create (plain hipEvent_t behind a void*); read them with
 * owl_probe_event_elapsed_ms, which waits for stop_event on the host.
 */
owl_status owl_verify_attn_split_timed(const owl_verify_desc *desc, const void *q, const void *k_cache,
                                       const void *v_cache, const int32_t *page_table, const int32_t *ctx_lens,
                                       const int32_t *tree_parent, void *out, void *workspace, size_t workspace_bytes,
                                       uint32_t *dev_status, void *stream, void *start_event, void *stop_event);
owl_status owl_probe_event_create(void **event);
owl_status owl_probe_event_destroy(void *event);
owl_status owl_probe_event_elapsed_ms(void *start_event, void *stop_event, float *ms_host);

/*
 * Per-workgroup timeline of the split-KV pass.  With a device buffer of
 * 10 * n_workgroups int64, later owl_verify_attn calls whose split-KV grid has
 * at most n_workgroups workgroups (owl_plan.n_workgroups) and whose shape has a
 * profiling copy of the kernel (bf16, head_dim 128) run that copy; every
 * workgroup records the GPU's constant-rate (100 MHz) wall clock at: [0] entry,
 * [1] page list and tree mask ready, [2] first stage in LDS, [3] end of the fast
 * loop, [4] end of the careful loop, [5] partials written; [6] = (XCC id << 16) |
 * CU id, [7] = its flat workgroup index; [8], [9] = the shader cycle counter at
 * [2] and [3], so that ([9] - [8]) / ([3] - [2]) / 10 is the shader clock in GHz
 * the workgroup really ran its main loop at.  Calls that do not qualify (larger
 * grid, other type) run the ordinary kernel and record nothing.  buffer = NULL
 * switches recording off (the default); the ordinary kernels contain no trace of
 * the hook.  One switch per process; set it from the measuring thread.
 */
owl_status owl_debug_set_timeline(long long *buffer, int64_t n_workgroups);

#ifdef __cplusplus
}
#endif
#endif /* OWL_PROBE_H_ */
