// Plain-data side of libtreeattn: the parameter blocks the host fills and the kernels read, the launch plan and its
// dispatch table.  No HIP types in here, so that the host logic (ta_host.cpp) also builds with an ordinary C++
// compiler, e.g. under -fsanitize=address,undefined.
#pragma once

#include <stddef.h>
#include <stdint.h>

#include "../../include/treeattn.h"

#define TA_WAVE 64
#define TA_TILE 64            // KV tokens per tile of the KV pass (the tree tokens form one more tile)
#define TA_MERGE_ROWS 4       // rows per workgroup of the general merge kernel (one per wave)
#define TA_MERGE128_ROWS 8    // rows per workgroup of the head_dim-128 merge kernel (half a wave per row)
#define TA_ROW_GROUP 256      // rows (tree nodes x query heads of one KV head) one workgroup keeps
#define TA_STATUS_BYTES 256

struct TAParams {
    const void *q, *k, *v;
    void *out;
    float *lse;
    const int32_t *page_table, *seq_lens, *parent;
    int64_t q_sb, q_st, q_sh;
    int64_t o_sb, o_st, o_sh;
    int64_t k_sp, k_sh, k_ss;
    int64_t v_sp, v_sh, v_ss;
    int64_t lse_sb, lse_sh, lse_st;
    int64_t pt_sb, par_sb, sl_s;
    int32_t B, T, Hq, Hkv, G, D;
    int32_t ps, ps_shift;      // page size; log2 of it, or -1 when it is not a power of two
    int32_t capacity;          // logical positions one request can address
    int32_t n_pages;           // pages the caches hold (page ids must lie in [0, n_pages))
    int32_t rows;              // T * G
    int32_t rows_grp;          // rows per row group (the last group may hold fewer)
    int32_t n_rg;              // row groups
    int32_t n_wg;              // workgroups of the KV pass along x
    int32_t min_q;             // smallest share of tiles a workgroup takes
    int32_t pad;               // schedule units a list counts on top of its tiles (fixed cost per list)
    uint32_t g_magic;          // 2^24 / G + 1: R / G == mulhi(R << 8, g_magic) for R * G < 2^24 (matrix-core kernels)
    const int32_t *kv_start;   // [B] window starts, or null
    int32_t q_off;             // row r of q, out and lse is tree node q_off + r / G (rows = Tq * G)
    const unsigned long long *masks_in;   // ancestor masks encoded earlier (or null: walk the parents in the call)
    int64_t masks_sb;          // words between the masks of consecutive requests
    int32_t is_bf16;
    float scale_log2e;         // softmax scale * log2(e): scores are kept in the base-2 domain
    float *ws_o;               // partial outputs  [slot][rg][rows_grp][D], normalised; fp32, or int16 when part_q15
    float *ws_lse;             // partial log2-sum-exp2 [slot][rg][rows_grp]; with part_q15 [slot][rg][rows_grp][2]:
                               // the log-sum-exp and the scale of the row's 16-bit values side by side
    int32_t ls;                // floats per row in ws_lse: 1, or 2 with part_q15
    int32_t *ws_parts;         // [B * Hkv][2]: first and last workgroup that hold partial results of a list; written
                               // by the KV pass (the owners of the list's first and last tile), read by the merge
    int32_t *status;           // sticky status word of the device
    int32_t *status2;          // the caller's own status word (ta_opts.status), or null
    int32_t basic;             // 256-row groups: use the register-staged MFMA kernel, not the pipelined one
    int32_t merge_kind;        // TA_MERGE_*: which merge kernel follows the KV pass
    int32_t part_q15;          // the partial outputs in ws_o are 16-bit fixed point with one scale per row
                               // (matrix-core kernels) rather than fp32
    // write-back folded into the call: the tree tokens' K/V come from these dense tensors [B, T, Hkv, D] (element
    // strides), the KV pass reads them there and the merge pass copies them behind the prefix in the caches
    const void *kn, *vn;
    int64_t kn_sb, kn_st, kn_sh, vn_sb, vn_st, vn_sh;
    int32_t kn_vec;            // rows can be copied in 16-byte pieces
};

struct TAAppend {
    const void *k_new, *v_new;         // [B, T, Hkv, D]
    void *k, *v;                       // caches
    const int32_t *page_table, *seq_lens;
    int64_t kn_sb, kn_st, kn_sh, vn_sb, vn_st, vn_sh;
    int64_t k_sp, k_sh, k_ss, v_sp, v_sh, v_ss, pt_sb, sl_s;
    int32_t B, T, Hkv, D, ps, capacity, n_pages, elem_bytes;
    int32_t *status;
};

struct TACompact {
    void *k, *v;                       // caches
    const int32_t *page_table, *seq_lens, *accepted, *n_accepted;
    int32_t *seq_lens_out;             // or nullptr
    int64_t k_sp, k_sh, k_ss, v_sp, v_sh, v_ss, pt_sb, sl_s, acc_sb, na_s, slo_s;
    int32_t B, T, A, Hkv, D, ps, capacity, n_pages, elem_bytes;
    int32_t *status;
};

// Which merge kernel combines the partial results.
#define TA_MERGE_GENERAL 0    // one wave per output row, any head_dim and alignment
#define TA_MERGE_D128 1       // head_dim 128, aligned outputs: half a wave per row, eight rows per workgroup
#define TA_MERGE_D128_WIDE 2  // the same shapes when few lists are cut into many shares: one workgroup per row

// ---------------------------------------------------------------------------------------------
// Dispatch table (section 3.4, "Attention kernel": the kernel and its split are chosen by a heuristic on batch size,
// tree size and GPU).  A call is classified by its kernel family, the query rows one KV head serves (T * G, rounded
// up to the row group the matrix-core kernel carries) and the number of (request, KV head) lists, and the first
// matching row fixes how the KV work is cut: workgroups per compute unit, the smallest share, the per-list cost
// of the schedule, and from how many partials per list on the row-per-workgroup merge takes over.
// ---------------------------------------------------------------------------------------------
struct TADispatchRow {
    int32_t family;            // TA_KERNEL_GENERIC, TA_KERNEL_MFMA or TA_KERNEL_MFMA_BASIC
    int32_t rows_grp_max;      // row applies to row groups of up to this many rows ...
    int32_t lists_max;         // ... and to batches of up to this many lists (INT32_MAX = any)
    int32_t wg_per_cu_x4;      // KV-pass workgroups per compute unit and row group, in quarters (4 = one per CU)
    int32_t min_share;         // smallest share of tiles per workgroup
    int32_t item_cost;         // schedule units per list on top of its tiles, plus one (ta_opts.item_cost)
    int32_t wide_from_parts;   // partials per list from which the row-per-workgroup merge is taken (0 = never)
    int32_t wide_max_rows;     // ... as long as the batch has at most this many output rows
};

struct TAPlan {
    int32_t kernel;            // TA_KERNEL_GENERIC or TA_KERNEL_MFMA (basic is a flag of the parameters)
    int32_t n_wg, threads, n_rg, rows_grp, n_slots, min_q, merge_wgs;
    int32_t item_cost, merge_kind, table_row;
};

struct TAProblem {
    TAParams p;
    TAPlan plan;
    size_t ws_o_bytes, ws_lse_bytes, ws_bytes;
    size_t ws_ls_off;          // byte offset of ws_lse inside the workspace: behind the partial outputs, or with
                               // part_q15 inside the half of their area that 16-bit rows leave unused
};

// Host logic shared by every entry point (ta_host.cpp).  None of these touches a device.
extern "C++" {
int ta_host_build_problem(const ta_tensor *q, const ta_tensor *k, const ta_tensor *v, const ta_tensor *pt,
                          const ta_tensor *sl, const ta_tensor *par, const ta_tensor *out, const ta_tensor *lse,
                          const ta_opts *opts, int num_cus, TAProblem *pr);
int ta_host_check_encode(const ta_tensor *tree_parent, const ta_tensor *masks, int *B, int *T, int64_t *par_sb);
int ta_host_check_append(const ta_tensor *k_new, const ta_tensor *v_new, const ta_tensor *k_cache,
                         const ta_tensor *v_cache, const ta_tensor *page_table, const ta_tensor *seq_lens, TAAppend *a);
int ta_host_check_compact(const ta_tensor *k_cache, const ta_tensor *v_cache, const ta_tensor *page_table,
                          const ta_tensor *seq_lens, const ta_tensor *accepted, const ta_tensor *n_accepted,
                          int32_t tree_size, const ta_tensor *seq_lens_out, TACompact *c);
size_t ta_host_workspace_bytes(int32_t B, int32_t T, int32_t Hq, int32_t Hkv, int32_t D, int32_t dtype, int32_t num_cus);
void ta_host_fill_plan(const TAProblem &pr, int64_t plan[16]);
const TADispatchRow *ta_host_dispatch_table(int *n_rows);
int ta_host_merge_rows(const TAParams &p);       // output rows one workgroup of the merge pass handles
size_t ta_host_align_up(size_t x, size_t a);
}
