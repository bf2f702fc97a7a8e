/*
 * owl.h -- C ABI of the MI355X (gfx950) verify-step attention library.
 *
 * The operation is the attention sub-step of the target model's verification
 * forward pass in tree / sequence speculative decoding: N drafted tokens (a
 * chain, or a token tree) of each sequence attend over that sequence's long
 * prefix KV cache plus the drafted tokens on their own root path.
 *
 * Where the paper defines it:
 *   - Sec. 1 / Sec. 2: the target model verifies all drafted tokens in one
 *     parallel pass whose cost, in the memory-bound regime, is the scan of the
 *     cached context.
 *   - Sec. 3.2.2 "Decode Stage" and Algorithm 1 (Prepare / OurTreeVerify): a
 *     token placed after a tree path sees exactly that path; the paper gets
 *     there by adjusting the attention mask.  The example there fixes the rule:
 *     ancestor-or-self visibility among the drafts, full visibility of the
 *     prefix.
 *   - Sec. 3.2.3 / Algorithm 1 (NonTreeVerify): sequence verification is the
 *     chain-shaped tree.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers unless the name ends in _host.
 *   - The caller owns every buffer, the workspace included.  No entry point
 *     allocates or frees device memory, and none synchronises: work is
 *     enqueued on `stream` (a hipStream_t passed as void*, NULL = the default
 *     stream) and the call returns.
 *   - Errors the host can see (null pointers, unsupported shapes, a workspace
 *     that is too small) give a negative owl_status before anything is
 *     launched.  Errors that live in device-resident arrays (a parent index
 *     out of order, a page id outside the pool, a context longer than
 *     announced) cannot be seen without a synchronisation; the kernels never
 *     follow such a value out of bounds, they neutralise it (a bad parent
 *     counts as a root, a bad page reads page 0, a bad length is clamped) and
 *     OR a bit into *dev_status if that pointer is not NULL.  `out` of the
 *     affected sequence is then unspecified.
 */
#ifndef OWL_H_
#define OWL_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum owl_status {
    OWL_OK = 0,
    OWL_ERR_INVALID_ARG = -1,    /* null pointer, non-positive size, Hq % Hkv != 0 ...  */
    OWL_ERR_BAD_TREE = -2,       /* parent[i] outside {-1} u [0, i)   (host variant)    */
    OWL_ERR_TOO_MANY_DRAFT = -3, /* n_draft > 64: one 64-bit word holds a node's mask   */
    OWL_ERR_UNSUPPORTED = -4,    /* head_dim, page_size or dtype this build lacks       */
    OWL_ERR_WORKSPACE = -5,      /* workspace_bytes below owl_verify_attn_workspace_size */
    OWL_ERR_HIP = -6             /* a HIP runtime call failed (launch, attribute query) */
} owl_status;

typedef enum owl_dtype {
    OWL_BF16 = 0,   /* bf16 storage, bf16 MFMA, fp32 accumulate and softmax */
    OWL_F32 = 1,    /* fp32 storage and arithmetic (small correctness shape) */
    OWL_F16 = 2     /* fp16 storage (the paper's inference type, App. A.1), fp16 MFMA */
} owl_dtype;

/* bits OR-ed into *dev_status */
#define OWL_DEV_BAD_PARENT 1u   /* some parent[i] not in {-1} u [0, i)            */
#define OWL_DEV_BAD_PAGE 2u     /* a needed page id not in [0, n_pool_pages)      */
#define OWL_DEV_BAD_CTX_LEN 4u  /* some ctx_lens[b] not in [0, max_ctx_len]       */
#define OWL_DEV_BAD_ACCEPT 8u   /* accepted[] not a strictly increasing list in [0, n_draft) */
#define OWL_DEV_BAD_NDRAFT 16u  /* some n_draft_seq[b] not in [0, n_draft]        */
#define OWL_DEV_BAD_TOKEN 32u   /* drafter cell: some tokens[r] not in [0, vocab)  */
#define OWL_DEV_BAD_ROW 64u     /* drafter cell: some parent_row[r] not in [0, n_states) */

/*
 * Shape of one verify step.  Strides are in ELEMENTS of qkv_dtype.
 * The element (page p, kv head g, slot s, channel d) of a cache lives at
 *     p * kv_stride_page + g * kv_stride_head + s * kv_stride_token + d ,
 * channels contiguous.  [page][Hkv][16][D] ("head-major": each (page, head) is
 * one contiguous 16*D run, the layout the kernels stream best) and
 * [page][16][Hkv][D] (a plain [token][Hkv][D] array when pages are in order)
 * are both expressible.  Byte offsets of the strides must be multiples of 16.
 */
typedef struct owl_verify_desc {
    int32_t batch;              /* B >= 1 sequences                                      */
    int32_t n_draft;            /* N in [1, 64] drafted tokens per sequence              */
    int32_t n_q_heads;          /* Hq                                                    */
    int32_t n_kv_heads;         /* Hkv, divides Hq; query head h reads kv head h/(Hq/Hkv) */
    int32_t head_dim;           /* D: 64 or 128                                          */
    int32_t page_size;          /* tokens per page: 16                                   */
    int32_t max_pages_per_seq;  /* row length of page_table                              */
    int32_t max_ctx_len;        /* upper bound of ctx_lens[]; sizes the split plan       */
    int32_t qkv_dtype;          /* owl_dtype of q, k_cache, v_cache                      */
    int32_t split_tokens;       /* 0 = let the library choose; else tokens per KV split  */
                                /* (rounded up to a multiple of 64) -- testing / tuning   */
    float scale;                /* multiplies q.k before the softmax, e.g. 1/sqrt(D)     */
    int32_t out_dtype;          /* owl_dtype of `out`: OWL_F32, or OWL_BF16 / OWL_F16 =  */
                                /* the fp32 result rounded to nearest even on the way out */
    int64_t kv_stride_page, kv_stride_head, kv_stride_token;
    int64_t n_pool_pages;       /* pages in k_cache / v_cache (bounds for page ids)      */
    int32_t flags;              /* bit set of OWL_FLAG_*, 0 = none                       */
    int32_t reserved_;          /* set to 0                                              */
} owl_verify_desc;

/*
 * OWL_FLAG_FP32_PARTIALS (16-bit qkv_dtype only; fp32 inputs always behave so):
 * the split-KV pass hands its per-split results to the combine as raw fp32
 * accumulators.  By default it hands them over normalised and in fp16 (each row
 * divided by its row sum and by its largest magnitude, which is kept in fp32):
 * half the bytes to write and read back, for a rounding of 2^-12 of a row's
 * largest component, far below what the 16-bit softmax weights cost already.
 * With the flag the whole path adds in fp32 only, so that results that are
 * exactly representable (e.g. the mean of small integers over a power-of-two
 * number of rows) come out exact; the workspace is larger.
 */
#define OWL_FLAG_FP32_PARTIALS 1

/* What the library decided for a descriptor; informational (bench, tests). */
typedef struct owl_plan {
    int32_t split_tokens;    /* tokens of the logical sequence (prefix + drafts) per split */
                             /* for a context of max_ctx_len.  With a library-chosen size   */
                             /* the kernels follow the real lengths: one shorter sequence   */
                             /* is cut into max_splits shorter splits, a ragged batch into  */
                             /* the shortest splits that still fill whole rounds of one     */
                             /* workgroup per compute unit (never below the planner's       */
                             /* minimum, never above this value)                            */
    int32_t max_splits;      /* most splits one sequence can be cut into (sizes the partials) */
    int32_t rows_per_kv;     /* R = (Hq/Hkv) * N query rows packed against one KV stream   */
    int32_t row_tiles;       /* 16-row MFMA tiles covering R                               */
    int32_t row_groups;      /* workgroups sharing one KV split, each owning some tiles    */
    int32_t tiles_per_wave;  /* row tiles held in one wavefront's accumulators             */
    int32_t kernel_variant;  /* internal id of the instantiated split-KV kernel            */
    int32_t n_workgroups;    /* grid size of the split-KV pass                             */
    int32_t reserved_;       /* 0                                                          */
    size_t workspace_bytes;
} owl_plan;

/* Fill *plan for `desc` on the current device.  Host only, no launch. */
owl_status owl_verify_attn_plan(const owl_verify_desc *desc, owl_plan *plan);

/* Bytes of device scratch owl_verify_attn needs for `desc` (split partials). */
owl_status owl_verify_attn_workspace_size(const owl_verify_desc *desc, size_t *bytes);

/*
 * The verify-step attention (Sec. 3.2.2 Decode Stage; Algorithm 1,
 * OurTreeVerify / NonTreeVerify).  For every sequence b, draft node i and
 * query head h, with g = h / (Hq/Hkv) and L = ctx_lens[b]:
 *     keys    = logical positions 0..L-1  and  L + j for every j on the root
 *               path of i (i itself included)
 *     out[b,i,h,:] = softmax_over_keys(scale * q[b,i,h,:] . K[key,g,:]) @ V[key,g,:]
 * Logical position p of sequence b is slot p % 16 of physical page
 * page_table[b][p / 16]; the drafts' own K/V rows must already be in the
 * cache at positions L .. L+N-1, so page_table must cover L + N positions.
 *
 *   q            [B][N][Hq][D]  qkv_dtype, contiguous
 *   k_cache, v_cache             paged pools, see owl_verify_desc
 *   page_table   [B][max_pages_per_seq] int32, or NULL = identity (page p of
 *                every sequence is physical page p; only sensible for B == 1)
 *   ctx_lens     [B] int32, prefix lengths, drafts not counted, 0 allowed
 *   tree_parent  [B][N] int32, -1 = root, else an index < i
 *   out          [B][N][Hq][D] in desc->out_dtype, contiguous, fully overwritten
 *   workspace    >= owl_verify_attn_workspace_size() bytes, 256-byte aligned;
 *                contents need no initialisation and are garbage afterwards
 *   dev_status   optional uint32 on the device, OR-ed with OWL_DEV_* bits;
 *                the caller zeroes and reads it
 * Calls that share a workspace must be ordered on one stream.
 */
owl_status owl_verify_attn(const owl_verify_desc *desc, const void *q, const void *k_cache,
                           const void *v_cache, const int32_t *page_table,
                           const int32_t *ctx_lens, const int32_t *tree_parent, void *out,
                           void *workspace, size_t workspace_bytes, uint32_t *dev_status,
                           void *stream);

/*
 * One-time set-up for `desc` on the current device, host only: the kernel that
 * serves `desc` needs more LDS than the default and is told so once per device
 * (hipFuncSetAttribute), and the device address of the library's own scratch
 * memory (owl_verify_attn_noalloc) is looked up.  Every entry point does this
 * by itself on first use; a caller who wants the FIRST call for a shape to be
 * legal inside a stream capture (where such calls are not allowed) calls this
 * beforehand, outside the capture.  Launches nothing.
 */
owl_status owl_verify_attn_init(const owl_verify_desc *desc);

/*
 * owl_verify_attn for callers that cannot allocate device memory and have no
 * workspace to hand over: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels and the same
 * result as owl_verify_attn, minus the workspace: the split partials go to a
 * fixed buffer of OWL_NOALLOC_SCRATCH_BYTES inside the library's own device
 * image (one per GPU that loads the library, held until the process ends).
 *   - A `desc` whose owl_verify_attn_workspace_size exceeds
 *     OWL_NOALLOC_SCRATCH_BYTES is refused with OWL_ERR_WORKSPACE before
 *     anything is launched (the single-sequence shapes up to 128K context with
 *     320 rows per KV head fit; a large batch does not).
 *   - Calls no hipMalloc / hipFree or any other allocating routine.  The first
 *     call on a device looks up the buffer's address (owl_verify_attn_init
 *     does the same ahead of time).
 *   - All calls on one GPU share the one buffer: calls that may overlap in
 *     time (different streams, different threads) race and give garbage; order
 *     them on one stream.  The buffer keeps the previous call's contents;
 *     nothing in it needs to start at zero.
 */
#define OWL_NOALLOC_SCRATCH_BYTES (48u << 20)
owl_status owl_verify_attn_noalloc(const owl_verify_desc *desc, const void *q, const void *k_cache,
                                   const void *v_cache, const int32_t *page_table,
                                   const int32_t *ctx_lens, const int32_t *tree_parent, void *out,
                                   uint32_t *dev_status, void *stream);

/*
 * The same step, one phase at a time, for measurement: `phases` is a bit set of
 * OWL_PHASE_SPLIT (the split-KV pass that scans the cache and leaves partials
 * in the workspace) and OWL_PHASE_COMBINE (the log-sum-exp merge that turns
 * the partials into `out`).  OWL_PHASE_ALL is owl_verify_attn.  Running the
 * combine without a preceding split pass on the same workspace reads garbage
 * partials (finite or not) but stays in bounds.
 */
#define OWL_PHASE_SPLIT 1
#define OWL_PHASE_COMBINE 2
#define OWL_PHASE_ALL 3
owl_status owl_verify_attn_phases(const owl_verify_desc *desc, const void *q, const void *k_cache,
                                  const void *v_cache, const int32_t *page_table,
                                  const int32_t *ctx_lens, const int32_t *tree_parent, void *out,
                                  void *workspace, size_t workspace_bytes, uint32_t *dev_status,
                                  void *stream, int32_t phases);

/*
 * owl_verify_attn for a batch whose sequences carry different numbers of drafted
 * tokens (a verify step may mix sequence and tree drafts of different sizes,
 * Algorithm 1).  n_draft_seq [B] int32 device: sequence b has the nodes
 * 0 .. n_draft_seq[b]-1 of row b of q / tree_parent and draft K/V rows only at
 * ctx_lens[b] .. ctx_lens[b] + n_draft_seq[b] - 1; entries of tree_parent, q
 * and the cache beyond that are not interpreted.  Output rows of absent nodes
 * are written as zeros.  Entries outside [0, n_draft] are forced into the range
 * and flagged (OWL_DEV_BAD_NDRAFT).  Everything else as owl_verify_attn.
 */
owl_status owl_verify_attn_ragged(const owl_verify_desc *desc, const void *q, const void *k_cache,
                                  const void *v_cache, const int32_t *page_table,
                                  const int32_t *ctx_lens, const int32_t *tree_parent,
                                  const int32_t *n_draft_seq, void *out, void *workspace,
                                  size_t workspace_bytes, uint32_t *dev_status, void *stream);

/*
 * The attention mask of a drafted tree in packed form (Sec. 3.2.2, where the
 * mask and the position ids are adjusted to the tree; Algorithm 1, Prepare): for every
 * sequence b and node i,
 *     anc_mask[b][i]  bit j set  <=>  node j is on the path from i to its root,
 *                                     i itself included
 *     depth[b][i]     number of nodes on that path (root = 1); the position id
 *                     of node i is then ctx_lens[b] + depth - 1.  May be NULL.
 * tree_parent [B][N] int32 device; anc_mask [B][N] uint64 device; depth [B][N]
 * int32 device.  This is the same routine owl_verify_attn runs internally.
 */
owl_status owl_build_tree_mask(const int32_t *tree_parent, int32_t batch, int32_t n_draft,
                               uint64_t *anc_mask, int32_t *depth, uint32_t *dev_status,
                               void *stream);

/*
 * Prepare (Algorithm 1; Sec. 3.2.2, "Decode Stage"): the verify input of a
 * drafted tree of n nodes is the n nodes followed by one extra token per node,
 * the extra token of node k (index n + k) being placed after k's root path, so
 * that it sees exactly that path and itself.  For every sequence b and token
 * i < 2n this writes
 *     tree_parent2[b][i]  parent array of the 2n-token tree (parent of n + k is k),
 *                         ready to be handed to owl_verify_attn with n_draft = 2n
 *     anc_mask[b][i]      as owl_build_tree_mask
 *     depth[b][i]         tokens on i's root path, root = 1 (may be NULL)
 *     pos_ids[b][i]       ctx_lens[b] + depth - 1, the position id (may be NULL)
 * tree_parent [B][n], ctx_lens [B] int32 device; outputs [B][2n] device.
 * n <= 32 (OWL_ERR_TOO_MANY_DRAFT beyond).  A parent outside {-1} u [0, i) is
 * treated as a root and flagged (OWL_DEV_BAD_PARENT).
 */
owl_status owl_prepare_spec_tree(const int32_t *tree_parent, const int32_t *ctx_lens, int32_t batch,
                                 int32_t n_nodes, int32_t *tree_parent2, uint64_t *anc_mask,
                                 int32_t *depth, int32_t *pos_ids, uint32_t *dev_status, void *stream);

/*
 * Greedy acceptance after the verify pass (Sec. 1 and Sec. 2: the target model
 * checks all drafted tokens in parallel and keeps those that match its own
 * output, which leaves the output unchanged).  A node agrees if its token equals
 * the target's next token at its parent (target_root[b], the target's next token
 * after the context, for a root); the accepted path is the longest root path all
 * of whose nodes agree, the one ending in the smallest node index on ties.
 *     tokens      [B][N] int32 device  drafted token of node i (nodes >= n_cand,
 *                                      the extra tokens of Prepare, are never candidates)
 *     target_next [B][N] int32 device  the target's next token after node i's path
 *     accepted    [B][N] int32 device  out: path nodes from the root down, then -1
 *     n_accept    [B]    int32 device  out: the acceptance length of this step
 *     bonus       [B]    int32 device  out: the target's next token after the path
 *     last        [B]    int32 device  out: last accepted node or -1; with a tree
 *                                      from owl_prepare_spec_tree, row n + last of the
 *                                      verify pass is the extra token that follows the path
 * N <= 64, 0 <= n_cand <= N.  No host synchronisation.
 */
owl_status owl_accept_greedy(const int32_t *tokens, const int32_t *tree_parent, const int32_t *target_root,
                             const int32_t *target_next, int32_t batch, int32_t n_draft, int32_t n_cand,
                             int32_t *accepted, int32_t *n_accept, int32_t *bonus, int32_t *last,
                             uint32_t *dev_status, void *stream);

/*
 * Commit of the accepted tokens (Algorithm 1: the accepted draft is appended to
 * the context and the context length grows by its length): for every sequence
 * b, KV head g and i < n_accept[b], the K and V rows at logical position
 * ctx_lens[b] + accepted[b][i] move to ctx_lens[b] + i, in place, in the cache
 * described by desc (same layout and paging as owl_verify_attn; desc->n_draft
 * is the row length N of accepted[]).  All rows are read before any is written.
 * new_ctx_lens[b] = ctx_lens[b] + n_accept[b]; it may be NULL but must not be
 * ctx_lens itself.  accepted[b][0..n_accept) must be strictly increasing and in
 * [0, N) (a root path is), else nothing moves for b and OWL_DEV_BAD_ACCEPT is set.
 * Likewise, if a page-table entry under any source or destination row of b is
 * outside the pool (or the position lies beyond the table), nothing moves for
 * b, new_ctx_lens[b] = ctx_lens[b] and OWL_DEV_BAD_PAGE is set: a call that
 * writes never substitutes another page for a bad one.
 * The caches are written; everything else is read only.
 */
owl_status owl_commit_kv(const owl_verify_desc *desc, void *k_cache, void *v_cache, const int32_t *page_table,
                         const int32_t *ctx_lens, const int32_t *accepted, const int32_t *n_accept,
                         int32_t *new_ctx_lens, uint32_t *dev_status, void *stream);

/*
 * One step of the drafter's recurrent cell (Sec. 3.2.1, Eq. 1-8): from the token
 * t just predicted, the hidden state h it was predicted from and the running
 * cell state z,
 *     e   = E[t]                                                        (Eq. 1)
 *     s^m = W^m h + alpha e                m in {f, i, o, c}            (Eq. 2)
 *     g^m = sigmoid(s^m)                   m in {f, i, o}               (Eq. 5)
 *     c   = f(s^c) g^i                                                  (Eq. 6)
 *     z'  = z g^f + c                                                   (Eq. 7)
 *     h'  = f(z') g^o                                                   (Eq. 8)
 * where f is layer normalisation over the d channels (biased variance, eps under
 * the root, optional affine pair) followed by the exact GeLU x Phi(x).  The cell
 * never sees the context, so its cost does not depend on the context length
 * (Sec. 3.2.1); the step is a single read of the 4 d d_in weights.
 *
 * A step handles n_rows <= 64 rows that continue n_states <= 64 distinct states:
 * in tree drafting the children of a node share its (h, z) and differ in their
 * token, so W^m h is formed once per state and row r uses state parent_row[r].
 *
 *   h          [n_states][d_in]  dtype (OWL_BF16 or OWL_F16)
 *   z          [n_states][d]     float32 (all zeros at the first step, Sec. 3.2.1)
 *   tokens     [n_rows] int32
 *   parent_row [n_rows] int32, or NULL = identity (needs n_rows == n_states)
 *   w          W^f, W^i, W^o, W^c in this order, no bias: [4][d][d_in] dtype with
 *              one output channel's d_in weights contiguous (OWL_W_ROWS), or its
 *              tiled copy (OWL_W_TILED, see below)
 *   emb        [vocab][d] dtype, the embedding table E
 *   gamma_c, beta_c, gamma_z, beta_z   [d] float32 each or NULL (1 resp. 0): the
 *              affine pairs of f applied to s^c and of f applied to z'
 *   h_out      [n_rows][d] dtype (h' rounded to nearest even: the next step's h
 *              when d_in == d), h_out_f32 [n_rows][d] float32; either may be NULL
 *   z_out      [n_rows][d] float32
 *   workspace  >= owl_drafter_cell_workspace_size() bytes
 * Every pointer is 16-byte aligned.  Outputs must not overlap inputs.  d_in is a multiple of 32, d a multiple of 16
 * and at most 16384.  A token outside [0, vocab) contributes e = 0 and is flagged
 * (OWL_DEV_BAD_TOKEN); a parent_row outside [0, n_states) is read as 0 and flagged
 * (OWL_DEV_BAD_ROW).  `phases`: OWL_DRAFTER_PROJ forms W^m h into the workspace,
 * OWL_DRAFTER_GATES does the rest from the workspace; owl_drafter_cell runs both.
 */
typedef struct owl_drafter_desc {
    int32_t d_in;       /* width of the incoming hidden state h                     */
    int32_t d;          /* width of the cell (Sec. 4.1 uses 12288)                  */
    int32_t n_states;   /* P in [1, 64]                                             */
    int32_t n_rows;     /* M in [1, 64]                                             */
    int32_t vocab;      /* rows of emb                                              */
    int32_t dtype;      /* OWL_BF16 or OWL_F16: type of h, w, emb, h_out            */
    float alpha;        /* weight of the embedding, e.g. from owl_drafter_alpha     */
    float eps;          /* of the layer normalisation, e.g. 1e-5                    */
    int32_t w_layout;   /* OWL_W_ROWS or OWL_W_TILED: how `w` is stored             */
    int32_t reserved_;  /* set to 0                                                 */
} owl_drafter_desc;

/*
 * Layouts of the weights.  OWL_W_ROWS: w[m][j][k], m in the order f, i, o, c, a
 * plain [4 d][d_in] matrix.  OWL_W_TILED: the same numbers in the order the
 * projection kernel consumes them, which lets it stream HBM about 20 % faster
 * (one contiguous run per workgroup instead of 64 interleaved row streams).  In
 * units of 16 bytes (8 consecutive k of one row), element (row, k) of the
 * [4 d][d_in] matrix sits in granule
 *     ((row / 64 * (d_in / 32) + k / 32) * 4 + row % 64 / 16) * 64 + (k % 32 / 8) * 16 + row % 16
 * and the rows are padded with zeros to a multiple of 64.  Weights are constant,
 * so the copy is made once: owl_drafter_tile_weights does it on the device
 * (w_rows and w_tiled must not overlap; owl_drafter_tiled_weight_bytes gives the
 * size of w_tiled; only d_in, d and dtype of desc are used).
 */
#define OWL_W_ROWS 0
#define OWL_W_TILED 1
owl_status owl_drafter_tiled_weight_bytes(const owl_drafter_desc *desc, size_t *bytes);
owl_status owl_drafter_tile_weights(const owl_drafter_desc *desc, const void *w_rows, void *w_tiled, void *stream);

#define OWL_DRAFTER_PROJ 1
#define OWL_DRAFTER_GATES 2
#define OWL_DRAFTER_ALL 3

owl_status owl_drafter_cell_workspace_size(const owl_drafter_desc *desc, size_t *bytes);

owl_status owl_drafter_cell(const owl_drafter_desc *desc, const void *h, const float *z, const int32_t *tokens,
                            const int32_t *parent_row, const void *w, const void *emb, const float *gamma_c,
                            const float *beta_c, const float *gamma_z, const float *beta_z, void *h_out,
                            float *h_out_f32, float *z_out, void *workspace, size_t workspace_bytes,
                            uint32_t *dev_status, void *stream);

owl_status owl_drafter_cell_phases(const owl_drafter_desc *desc, const void *h, const float *z,
                                   const int32_t *tokens, const int32_t *parent_row, const void *w,
                                   const void *emb, const float *gamma_c, const float *beta_c,
                                   const float *gamma_z, const float *beta_z, void *h_out, float *h_out_f32,
                                   float *z_out, void *workspace, size_t workspace_bytes, uint32_t *dev_status,
                                   void *stream, int32_t phases);

/*
 * The weight of the embedding in Eq. 2, as Eq. 3-4 define it:
 *     alpha_0 = 2^(-1 / (2 n)),   alpha = 2 alpha_0 / ((1 - alpha_0^2) d),
 * n = the greatest tree depth to be drafted, d = the cell's width.  Host only;
 * evaluated in double precision, *alpha_host receives it rounded to float.
 */
owl_status owl_drafter_alpha(int32_t max_depth, int32_t d, float *alpha_host);

/* Host twin of owl_build_tree_mask for one tree; all pointers are HOST memory.
 * Validates the tree: OWL_ERR_BAD_TREE if some parent[i] is not in {-1} u [0,i). */
owl_status owl_build_tree_mask_host(const int32_t *tree_parent_host, int32_t n_draft,
                                    uint64_t *anc_mask_host, int32_t *depth_host);

/*
 * Paging on its own (the logical -> physical walk owl_verify_attn performs,
 * exposed so it can be checked bit for bit): copies n_tokens rows of sequence
 * `seq`, starting at logical position first_pos, of `cache` (K or V) into
 * dst[n_tokens][Hkv][D] in qkv_dtype.  Uses batch, n_kv_heads, head_dim,
 * page_size, max_pages_per_seq, qkv_dtype, strides and n_pool_pages of desc.
 */
owl_status owl_gather_kv(const owl_verify_desc *desc, const void *cache,
                         const int32_t *page_table, int32_t seq, int64_t first_pos,
                         int64_t n_tokens, void *dst, uint32_t *dev_status, void *stream);

/* Static string for a status code. */
const char *owl_status_str(owl_status s);

/* Library version, "major.minor". */
const char *owl_version(void);

#ifdef __cplusplus
}
#endif
#endif /* OWL_H_ */
