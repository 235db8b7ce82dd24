/*
 * libtreeattn -- tree attention for the verification step of tree-based
 * speculative decoding, hand-written for AMD MI355X (gfx950).
 *
 * The operation (paper section 3.1, "Tree attention"): the T draft tokens of a
 * speculation tree are flattened into one query sequence; node i of request b
 * must attend to the request's cached context (the prefix, L_b tokens) and to
 * the tree nodes on its own root-to-node path, itself included -- the result a
 * causal prefill over the unrolled path would give.  The paper computes it as
 * a mask-free prefix attention over the paged cache, a small tree-masked
 * suffix attention among the T tree tokens, and a merge of the partial results
 * through their log-sum-exp.  Paging applies to the cache (section 3.4, "Paged
 * KV with tree attention"); the tree tokens' K/V are expected at logical cache
 * positions L_b .. L_b+T-1, i.e. after they have been written back (or they
 * are handed over densely through ta_opts.k_new / v_new, which folds the
 * write-back into the call), and the page table must already cover them (the
 * paper's "tree padding").
 *
 * Conventions
 *   - Every `data` pointer is a DEVICE pointer unless stated otherwise; the
 *     caller owns all buffers, the library never frees or keeps them.
 *   - Strides are in ELEMENTS.  The innermost (head_dim) stride must be 1.
 *   - All entry points are asynchronous on `stream` (a hipStream_t passed as
 *     void*; NULL = the default stream), perform no device synchronisation and
 *     no device-to-host copy, and read seq_lens / page_table / tree_parent on
 *     the device only.
 *   - Calls that use the library-owned workspace of a device (tree_attn_fwd, and
 *     tree_attn_fwd_ex without ta_opts.workspace) share one buffer of partial
 *     results: they must not overlap in time, i.e. run on different streams of
 *     that device without ordering between them.  Concurrent calls each bring a
 *     workspace of their own.
 *   - Non-finite inputs.  A NaN or an infinity among the values a row attends to makes that output column NaN
 *     (an infinity may stay one), and with the 16-bit format of the partial results (the matrix-core kernels,
 *     i.e. bf16 inputs of head_dim 64 or 128; see tree_attn_plan) the whole output row NaN; NaNs in q or k reach out and lse through the
 *     scores.  Nothing else is affected.
 *   - Return value: TA_OK (0) or a negative ta_status.  Nothing throws or aborts.
 *     Problems visible on the host (null pointers, ranks, dtypes, shapes,
 *     strides) are reported before anything is launched.  Problems that only
 *     the data shows (a parent id outside [-1, T), a parent cycle, L_b < 0,
 *     L_b + T beyond max_pages*page_size, a page id outside the cache) cannot be
 *     seen without a synchronisation: the request's rows of `out` and `lse` are
 *     filled with NaN and a bit is set in a sticky per-device status word
 *     (tree_attn_last_status) and, if given, in the caller's own word
 *     (ta_opts.status).
 *   - Workspace lifetime.  A buffer of the library-owned workspace that has been
 *     handed to a launch is never freed or reused for anything else before
 *     tree_attn_release: when a later call needs more room the library allocates
 *     a larger buffer and keeps the old one, so a HIP graph captured earlier may
 *     be replayed at any time.  Under stream capture nothing is allocated: a call
 *     that would need a larger buffer than the device holds returns
 *     TA_ERR_WORKSPACE (call tree_attn_reserve before capturing, pass a workspace
 *     through ta_opts, or use tree_attn_fwd_static).
 */
#ifndef TREEATTN_H
#define TREEATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TREEATTN_VERSION 200      /* 0.2.0 */
#define TA_MAX_TREE 64            /* one 64-bit ancestor mask per node */
#define TA_MAX_HEAD_DIM 256
#define TA_MAX_BATCH 4096

typedef enum {
    TA_F32 = 0,
    TA_BF16 = 1,
    TA_I32 = 2,
    TA_U64 = 3
} ta_dtype;

typedef enum {
    TA_OK = 0,
    TA_ERR_NULL = -1,        /* a required descriptor or data pointer is NULL */
    TA_ERR_DTYPE = -2,       /* unsupported or mismatching element type */
    TA_ERR_RANK = -3,        /* wrong number of dimensions */
    TA_ERR_SHAPE = -4,       /* shapes disagree with each other */
    TA_ERR_STRIDE = -5,      /* innermost stride is not 1, or a stride is negative */
    TA_ERR_HEADS = -6,       /* Hq is not a multiple of Hkv */
    TA_ERR_HEAD_DIM = -7,    /* head_dim outside [1, TA_MAX_HEAD_DIM] */
    TA_ERR_TREE_SIZE = -8,   /* T outside [1, TA_MAX_TREE] */
    TA_ERR_PAGE_TABLE = -9,  /* max_pages * page_size cannot hold even the T tree tokens */
    TA_ERR_WORKSPACE = -10,  /* caller workspace too small or misaligned */
    TA_ERR_HIP = -11,        /* a HIP runtime call failed (no device, launch failure, allocation) */
    TA_ERR_BATCH = -12,      /* B outside [0, TA_MAX_BATCH] */
    TA_ERR_OPTS = -13        /* invalid field in ta_opts */
} ta_status;

/* Bits of the sticky device status word. */
#define TA_STATUS_BAD_PARENT 1   /* parent id outside [-1, T) or a parent cycle */
#define TA_STATUS_BAD_SEQLEN 2   /* L_b < 0 or L_b + T > max_pages * page_size */
#define TA_STATUS_BAD_PATH 4     /* tree_attn_compact: accepted length outside [0, A] or a node id outside [0, T) */
#define TA_STATUS_BAD_PAGE 8     /* a page_table entry the call needs lies outside [0, num_pages) */

typedef struct {
    void *data;           /* device pointer */
    int32_t dtype;        /* ta_dtype */
    int32_t ndim;
    int64_t shape[5];
    int64_t stride[5];    /* in elements */
} ta_tensor;

/* Kernel families (ta_opts.kernel).  AUTO picks MFMA when the shape allows it. */
#define TA_KERNEL_AUTO 0
#define TA_KERNEL_GENERIC 1   /* scalar fp32-accumulating kernel: any dtype, head_dim, page size */
#define TA_KERNEL_MFMA 2      /* bf16 matrix-core kernel: head_dim 128 or 64, power-of-two page size (or contiguous),
                                 16-byte aligned q/k/v rows, at most 256 query heads per KV head */
#define TA_KERNEL_MFMA_BASIC 3 /* as MFMA, but with the plain register-staged matrix-core kernel instead of the
                                 software-pipelined one (the library takes it by itself for head_dim 64, and when the
                                 batch is so large, B above ~1900, that the pipelined kernel's schedule does not fit
                                 beside the tiles in LDS) */

typedef struct {
    float scale;              /* softmax scale; <= 0 or NaN selects 1/sqrt(head_dim) */
    int32_t num_splits;       /* 0 = automatic; n > 0 = cut the batch's KV work into at most n workgroup shares */
    int32_t kernel;           /* TA_KERNEL_* */
    int32_t item_cost;        /* 0 = automatic.  n > 0: when the KV work is cut into workgroup shares, every
                                 (request, KV head) list counts n - 1 tiles more than it holds, which stands for
                                 the fixed work a workgroup spends per list it touches (1 = none).  Results do
                                 not depend on it beyond the order of the fp32 merge. */
    void *workspace;          /* device scratch, 256-byte aligned, or NULL = library-owned per-device buffer */
    size_t workspace_bytes;   /* size of `workspace` */
    void *events[3];          /* optional hipEvent_t handles (HOST values) recorded on `stream`: [0] before the
                                 KV pass, [1] between KV pass and merge pass, [2] after the merge pass; NULL
                                 entries are skipped.  For measurement harnesses. */
    const void *tree_masks;   /* optional DEVICE pointer to the ancestor masks tree_attn_encode wrote for these
                                 trees (64-bit words, node i of request b at [b * tree_masks_stride + i]); the
                                 call then reads them instead of walking tree_parent again -- for static trees
                                 (section 3.4, pre-computed static trees) that are encoded once and used for many
                                 steps.  Bits of nodes >= T are ignored.  tree_parent is still required (shape). */
    int64_t tree_masks_stride;/* words between the masks of consecutive requests; 0 = one tree for the batch */
    int32_t q_node_offset;    /* q, out and lse may hold fewer nodes than tree_parent describes: their row i is tree
                                 node q_node_offset + i, while all T nodes of the tree are keys (section 3.1: the
                                 same attention serves the drafting stage, where only the newest nodes ask).
                                 0 <= q_node_offset, q_node_offset + q.shape[1] <= T.  Default 0. */
    int32_t reserved;         /* must be 0 */
    const void *kv_start;     /* optional DEVICE pointer to int32 [B]: request b's nodes attend to prefix positions
                                 kv_start[b] .. L_b - 1 only (section 3.4, iRoPE for Llama4: on local-attention
                                 layers the prefix is the current sub-sequence), plus their tree path as always.
                                 0 <= kv_start[b] <= L_b, else the request is NaN-filled and TA_STATUS_BAD_SEQLEN
                                 is set.  NULL = 0. */
    const ta_tensor *k_new;   /* optional, with v_new (HOST descriptors, DEVICE data): the step's keys and values of the T
                                 tree tokens, [B, T, Hkv, D], dtype of the cache, unit D stride -- the write-back folded
                                 into the call (section 3.4, paged KV with tree attention: the step's keys and values
                                 are written back rather than fetched).  The call then takes the tree tokens' K/V from
                                 these tensors, never from the cache, and also stores them at logical positions
                                 L_b .. L_b+T-1 of k_cache / v_cache (which it therefore writes), exactly as
                                 tree_attn_append would have before the call; out and lse are bit for bit those of
                                 append followed by the plain call.  A request that is NaN-filled for a bad length
                                 is not written.  Both NULL = the tree tokens are already in the cache. */
    const ta_tensor *v_new;
    int32_t *status;          /* optional DEVICE pointer to one 32-bit word, 4-byte aligned: the call ORs the TA_STATUS_*
                                 bits of its own data-dependent problems into it (as well as into the device's sticky
                                 word), so that a captured graph or a caller with several streams can carry a status
                                 word of its own and read it whenever it likes.  The library never clears it. */
} ta_opts;

/*
 * Tree attention forward (section 3.1; cache addressing per section 3.4).
 *
 *   q           [B, T, Hq, D]  TA_BF16 or TA_F32; node i of request b, query head h (fewer nodes than the tree has:
 *               see ta_opts.q_node_offset)
 *   k_cache     [num_pages, Hkv, page_size, D] -- any 4-D strided view with unit D stride, dtype of q.
 *               Token at logical position t of request b, KV head g lives in page page_table[b][t / page_size],
 *               slot t % page_size.  Logical positions 0..L_b-1 are the prefix, L_b+i is tree node i.
 *   v_cache     same shape and dtype as k_cache (strides may differ)
 *   page_table  TA_I32 [B, max_pages], or NULL for the contiguous layout: request b owns page b, and
 *               page_size (the cache's slot dimension) is that request's capacity
 *   seq_lens    TA_I32 [B], prefix lengths L_b; the T tree tokens are NOT counted
 *   tree_parent TA_I32 [B, T] (stride[0] may be 0: one tree for the batch) or [T]; a negative parent marks a
 *               root; any node numbering is accepted (parents need not precede children)
 *   out         [B, T, Hq, D], dtype of q: softmax(scale * q K^T) V over prefix + path, rounded once
 *               (round to nearest even) from an fp32 accumulator
 *   lse         TA_F32 [B, Hq, T] or NULL: natural log of the sum of exp of the scaled scores
 *   stream      hipStream_t
 *
 * Query head h reads KV head h / (Hq / Hkv).  B == 0 is a no-op.  Uses the library-owned workspace of
 * the current device, grown on demand with hipMalloc: call tree_attn_reserve first (or pass a workspace
 * through tree_attn_fwd_ex) wherever allocation is not allowed, e.g. under stream capture.
 */
int tree_attn_fwd(const ta_tensor *q, const ta_tensor *k_cache, const ta_tensor *v_cache,
                  const ta_tensor *page_table, const ta_tensor *seq_lens, const ta_tensor *tree_parent,
                  ta_tensor *out, ta_tensor *lse, void *stream);

/* Same operation with explicit options (NULL opts = defaults). */
int tree_attn_fwd_ex(const ta_tensor *q, const ta_tensor *k_cache, const ta_tensor *v_cache,
                     const ta_tensor *page_table, const ta_tensor *seq_lens, const ta_tensor *tree_parent,
                     ta_tensor *out, ta_tensor *lse, void *stream, const ta_opts *opts);

/*
 * Upper bound, in bytes, of the scratch a call with these sizes needs (split-KV partial outputs and
 * their log-sum-exps; section 3.1, the partial results that the merge combines).  Host-only.
 * `num_cus` is the compute-unit count of the target device (0 = query the current device, 256 when
 * no device is present).  T counts the query nodes (q.shape[1]).  Returns 0 for invalid sizes.
 */
size_t tree_attn_workspace_bytes(int32_t B, int32_t T, int32_t Hq, int32_t Hkv, int32_t D,
                                 int32_t dtype, int32_t num_cus);

/* Grow the library-owned workspace of the current device to at least `bytes` (allocates; call outside
 * stream capture).  Never synchronises and never frees: a smaller buffer that earlier launches or captured graphs
 * may still use is kept until tree_attn_release.  Also performs the per-device set-up every entry point needs, so
 * that the first call under stream capture finds it done. */
int tree_attn_reserve(size_t bytes);

/* Free every buffer the library owns on the current device (the workspace and the buffers it outgrew).
 * Synchronises the device first.  Graphs captured with the library-owned workspace must not be replayed afterwards. */
int tree_attn_release(void);

/*
 * Tree-topology encoder alone (section 3.1: the tree mask, here one 64-bit word per node instead of an
 * explicit query x context mask tensor): masks[b][i] has bit j set iff node j lies on the path from a
 * root to node i, i included.  tree_parent TA_I32 [B,T] or [T]; masks TA_U64 of the same shape,
 * contiguous.  A malformed tree yields all-zero masks for that request and sets TA_STATUS_BAD_PARENT.
 */
int tree_attn_encode(const ta_tensor *tree_parent, ta_tensor *masks, void *stream);

/*
 * Write-back of the tree tokens' keys and values (section 3.4, paged KV with tree attention: the keys and values
 * computed in this step are written back to the cache, behind the prefix, where tree_attn_fwd reads them):
 * k_new, v_new [B, T, Hkv, D] (dtype of the cache, unit D stride) go to logical positions L_b .. L_b+T-1 of request b
 * in k_cache / v_cache, addressed through page_table exactly as in tree_attn_fwd (NULL = contiguous).  A request
 * with L_b < 0 or L_b + T beyond what its page-table row can address is skipped and TA_STATUS_BAD_SEQLEN is set.
 * One launch on `stream`, no allocation, no synchronisation.
 */
int tree_attn_append(const ta_tensor *k_new, const ta_tensor *v_new, ta_tensor *k_cache, ta_tensor *v_cache,
                     const ta_tensor *page_table, const ta_tensor *seq_lens, void *stream);

/*
 * Bookkeeping after acceptance (section 3, stage 6: the KV cache is rewound to the position the accepted length
 * gives; with a tree, node i of request b sits at logical position L_b + i, so the accepted path is first made
 * contiguous): the K/V rows of nodes accepted[b][0 .. n_b-1] (node ids, path order, root first; n_b =
 * n_accepted[b]) become logical positions L_b .. L_b+n_b-1 of request b, addressed through page_table exactly as in
 * tree_attn_fwd (NULL = contiguous).  Every row is read before any is written, so sources and destinations may
 * overlap; nothing else in the caches changes.
 *
 *   accepted      TA_I32 [B, A], 1 <= A <= TA_MAX_TREE, unit inner stride; entries past n_b are not read
 *   n_accepted    TA_I32 [B]
 *   tree_size     T: node ids must lie in [0, T); 1 <= T <= TA_MAX_TREE
 *   seq_lens_out  TA_I32 [B] or NULL: receives L_b + n_b.  May be seq_lens itself (same pointer and stride), must not
 *                 overlap it otherwise.
 *
 * A request with L_b < 0, L_b + T beyond what its page-table row can address (TA_STATUS_BAD_SEQLEN), n_b outside
 * [0, A] or a node id outside [0, T) (TA_STATUS_BAD_PATH) is left alone and its length is passed through unchanged.
 * One launch on `stream` (one workgroup per request), no allocation, no synchronisation.
 */
int tree_attn_compact(ta_tensor *k_cache, ta_tensor *v_cache, const ta_tensor *page_table, const ta_tensor *seq_lens,
                      const ta_tensor *accepted, const ta_tensor *n_accepted, int32_t tree_size,
                      ta_tensor *seq_lens_out, void *stream);

/* Read and clear the sticky status word of the current device.  Synchronises `stream`.
 * *host_status receives an OR of TA_STATUS_* bits (HOST pointer). */
int tree_attn_last_status(int32_t *host_status, void *stream);

/*
 * Host-only launch plan for a call (no device access): which kernel family would run and how the work
 * is cut (section 3.4, "Attention kernel": the choice by batch size, tree size and GPU; here one row of the
 * library's dispatch table, see tree_attn_dispatch_row).  plan[0] = kernel family, plan[1] = workgroups of the
 * KV pass, plan[2] = threads per workgroup, plan[3] = KV tokens per tile, plan[4] = row groups, plan[5] = padded
 * rows per group, plan[6] = partial slots, plan[7] = workgroups of the merge pass, plan[8] = smallest share of
 * tiles per workgroup, plan[9] = schedule units a list counts (item_cost), plan[10] = merge kernel (0 general,
 * 1 head_dim 128, 2 head_dim 128 with one workgroup per row), plan[11] = row of the dispatch table that was
 * taken (-1: the options fixed everything), plan[12] = workspace bytes the call needs, plan[13] = format
 * of the partial results (0: fp32; 1: 16-bit fixed point with one fp32 scale per row), plan[14..15] = 0.
 * HOST pointers.
 */
int tree_attn_plan(const ta_tensor *q, const ta_tensor *k_cache, const ta_tensor *v_cache,
                   const ta_tensor *page_table, const ta_tensor *seq_lens, const ta_tensor *tree_parent,
                   const ta_tensor *out, const ta_tensor *lse, const ta_opts *opts, int32_t num_cus,
                   int64_t plan[16]);

/*
 * Row `index` of the dispatch table (host-only; returns TA_ERR_OPTS past the last row): row[0] = kernel family,
 * row[1] = applies to row groups of up to this many rows, row[2] = and to at most this many (request, KV head)
 * lists, row[3] = KV-pass workgroups per compute unit in quarters, row[4] = smallest share of tiles,
 * row[5] = item_cost, row[6] = partials per list from which the one-workgroup-per-row merge takes over (0 = never),
 * row[7] = as long as the batch has at most this many output rows.  The first row that matches a call is taken.
 */
int tree_attn_dispatch_row(int32_t index, int64_t row[8]);

/*
 * For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): tree_attn_fwd_ex with its split-KV partial results in a fixed scratch area inside the
 * library image (TA_STATIC_SCRATCH_BYTES of device memory that every GPU the library runs on holds until the
 * process ends) instead of an allocated workspace.  Calls no hipMalloc / hipFree and no allocating library routine.
 * The call needs tree_attn_plan's plan[12] bytes of scratch; beyond TA_STATIC_SCRATCH_BYTES it returns
 * TA_ERR_WORKSPACE and launches nothing.  ta_opts.workspace must be NULL.  Every call on a device shares that
 * device's one scratch area: calls that overlap in time on one device (different streams without ordering) race,
 * exactly as with the library-owned workspace.  Nothing in the area has to survive from call to call.
 * Results are bit for bit those of tree_attn_fwd_ex.
 */
#define TA_STATIC_SCRATCH_BYTES (48u << 20)
int tree_attn_fwd_static(const ta_tensor *q, const ta_tensor *k_cache, const ta_tensor *v_cache,
                         const ta_tensor *page_table, const ta_tensor *seq_lens, const ta_tensor *tree_parent,
                         ta_tensor *out, ta_tensor *lse, void *stream, const ta_opts *opts);

/*
 * Measurement aid (no part of the method): a plain streaming read of `bytes` bytes of device memory at `buf`
 * (16-byte aligned, bytes a multiple of 16), one launch on `stream` -- the read rate this device attains, against
 * which the KV pass's rate is set beside the published peak.  `sink` is a DEVICE pointer to 4 bytes the kernel may
 * write.
 */
int tree_attn_stream_read(const void *buf, size_t bytes, void *sink, void *stream);

/*
 * Measurement aid (no part of the method): one launch that does nothing but bf16 matrix-core instructions on
 * registers, eight waves per compute unit, 32 * iters instructions of 32768 flop per wave (1 <= iters <= 2^20) --
 * the matrix-core rate this device sustains, which its power limit holds below the published peak.  *flop (HOST
 * pointer, may be NULL) receives the flop of the launch; `sink` is a DEVICE pointer to 4 bytes.
 */
int tree_attn_mfma_probe(int32_t iters, void *sink, int64_t *flop, void *stream);

const char *tree_attn_strerror(int status);
int tree_attn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TREEATTN_H */
