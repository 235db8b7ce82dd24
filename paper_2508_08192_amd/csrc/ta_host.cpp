// Host logic of libtreeattn: descriptor validation, launch planning and the dispatch table.  Plain C++ with no
// device runtime behind it, so this file also builds with g++ under -fsanitize=address,undefined
// (see build.py: build_host_checked) and every rule in it can be exercised on a machine without a GPU.
// See include/treeattn.h for the contract of every entry point.
#include <initializer_list>
#include <limits.h>
#include <math.h>
#include <string.h>

#include "ta_params.h"

size_t ta_host_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

namespace {

bool strides_ok(const ta_tensor *t)
{
    for (int i = 0; i < t->ndim; ++i)
        if (t->stride[i] < 0)
            return false;
    return t->stride[t->ndim - 1] == 1 || t->shape[t->ndim - 1] <= 1;
}

// rows of a dense K/V tensor as the matrix-core kernels load them: 16-byte aligned, strides within 32 bits
bool new_rows_aligned(const ta_tensor *n)
{
    return ((uintptr_t)n->data % 16) == 0 && n->stride[0] % 8 == 0 && n->stride[1] % 8 == 0 && n->stride[2] % 8 == 0 &&
           n->stride[0] < INT32_MAX && n->stride[1] < INT32_MAX;
}

int mfma_rows_group(int rows)
{
    // 32 rows per wave; workgroups of 1, 2, 4 or 8 such waves, at most TA_ROW_GROUP rows.
    int grp = 32;
    while (grp < rows && grp < TA_ROW_GROUP)
        grp *= 2;
    return grp;
}

// Section 3.4, "Attention kernel": the split is chosen per batch size and tree size.  First matching row wins.
//   family, rows <=, lists <=, workgroups per CU x4, smallest share, item cost, wide merge from parts, wide max rows
// The pipelined matrix-core kernel runs one workgroup per compute unit (its tile rings fill the LDS).  A partial
// result costs rows * D * 4 bytes written and read again against TA_TILE * D * 4 bytes per tile of keys and values,
// hence the longer smallest shares of the larger row groups; the fixed work of entering a list is worth about eight
// tiles' time there (two for the register-staged kernel, nothing for the scalar one).  With few lists cut over the
// whole chip (batch size one) the merge becomes a latency problem and one workgroup per output row is faster from
// 13 partials per list on, while the batch has at most 1024 output rows.
const TADispatchRow kTable[] = {
    {TA_KERNEL_MFMA, 64, INT32_MAX, 4, 1, 9, 13, 1024},
    {TA_KERNEL_MFMA, 128, INT32_MAX, 4, 2, 9, 13, 1024},
    {TA_KERNEL_MFMA, 256, INT32_MAX, 4, 4, 9, 13, 1024},
    {TA_KERNEL_MFMA_BASIC, 64, INT32_MAX, 4, 1, 3, 13, 1024},
    {TA_KERNEL_MFMA_BASIC, 128, INT32_MAX, 4, 2, 3, 13, 1024},
    {TA_KERNEL_MFMA_BASIC, 256, INT32_MAX, 4, 4, 3, 13, 1024},
    {TA_KERNEL_GENERIC, 256, INT32_MAX, 16, 1, 1, 13, 1024},
};
constexpr int kTableRows = (int)(sizeof(kTable) / sizeof(kTable[0]));

int find_row(int family, int rows_grp, int64_t lists)
{
    for (int i = 0; i < kTableRows; ++i)
        if (kTable[i].family == family && rows_grp <= kTable[i].rows_grp_max && lists <= kTable[i].lists_max)
            return i;
    return -1;
}

}  // namespace

const TADispatchRow *ta_host_dispatch_table(int *n_rows)
{
    *n_rows = kTableRows;
    return kTable;
}

int ta_host_merge_rows(const TAParams &p)
{
    return p.merge_kind == TA_MERGE_D128_WIDE ? 1 : p.merge_kind == TA_MERGE_D128 ? TA_MERGE128_ROWS : TA_MERGE_ROWS;
}

// Everything that can be decided from the descriptors alone.
int ta_host_build_problem(const ta_tensor *q, const ta_tensor *k, const ta_tensor *v, const ta_tensor *pt,
                          const ta_tensor *sl, const ta_tensor *par, const ta_tensor *out, const ta_tensor *lse,
                          const ta_opts *opts, int num_cus, TAProblem *pr)
{
    if (!q || !k || !v || !sl || !par || !out)
        return TA_ERR_NULL;
    if (q->dtype != TA_BF16 && q->dtype != TA_F32)
        return TA_ERR_DTYPE;
    if (k->dtype != q->dtype || v->dtype != q->dtype || out->dtype != q->dtype)
        return TA_ERR_DTYPE;
    if (sl->dtype != TA_I32 || par->dtype != TA_I32 || (pt && pt->dtype != TA_I32) || (lse && lse->dtype != TA_F32))
        return TA_ERR_DTYPE;
    if (q->ndim != 4 || k->ndim != 4 || v->ndim != 4 || out->ndim != 4 || sl->ndim != 1 ||
        (par->ndim != 1 && par->ndim != 2) || (pt && pt->ndim != 2) || (lse && lse->ndim != 3))
        return TA_ERR_RANK;
    // T: nodes of the tree, all of them keys; Tq: the nodes that ask, q_off .. q_off+Tq-1 (all of them by default)
    const int64_t B = q->shape[0], Tq = q->shape[1], Hq = q->shape[2], D = q->shape[3];
    const int64_t T = par->shape[par->ndim - 1], q_off = opts ? opts->q_node_offset : 0;
    const int64_t n_pages = k->shape[0], Hkv = k->shape[1], ps = k->shape[2];
    if (B < 0 || B > TA_MAX_BATCH)
        return TA_ERR_BATCH;
    if (T < 1 || T > TA_MAX_TREE || Tq < 1 || Tq > TA_MAX_TREE)
        return TA_ERR_TREE_SIZE;
    if (Tq > T)
        return TA_ERR_SHAPE;                     // more query nodes than the tree has
    if (q_off < 0 || q_off + Tq > T)
        return TA_ERR_OPTS;
    if (D < 1 || D > TA_MAX_HEAD_DIM)
        return TA_ERR_HEAD_DIM;
    if (Hq < 1 || Hkv < 1 || Hq % Hkv != 0)
        return TA_ERR_HEADS;
    if (Hq > 65535 || ps < 1 || ps > (1 << 30) || n_pages < 0 || n_pages > INT32_MAX)
        return TA_ERR_SHAPE;
    if (k->shape[3] != D)
        return TA_ERR_SHAPE;
    for (int i = 0; i < 4; ++i)
        if (v->shape[i] != k->shape[i] || out->shape[i] != q->shape[i])
            return TA_ERR_SHAPE;
    if (sl->shape[0] != B)
        return TA_ERR_SHAPE;
    if (par->ndim == 2 && par->shape[0] != B)
        return TA_ERR_SHAPE;
    if (lse && (lse->shape[0] != B || lse->shape[1] != Hq || lse->shape[2] != Tq))
        return TA_ERR_SHAPE;
    if (pt && pt->shape[0] != B)
        return TA_ERR_SHAPE;
    if (!pt && n_pages < B)
        return TA_ERR_SHAPE;
    if (!strides_ok(q) || !strides_ok(k) || !strides_ok(v) || !strides_ok(out) || !strides_ok(par) ||
        (pt && !strides_ok(pt)))
        return TA_ERR_STRIDE;
    if (lse)
        for (int i = 0; i < 3; ++i)
            if (lse->stride[i] < 0)
                return TA_ERR_STRIDE;
    if (sl->stride[0] < 0)
        return TA_ERR_STRIDE;
    const int64_t capacity = pt ? pt->shape[1] * ps : ps;
    if (capacity < T)
        return TA_ERR_PAGE_TABLE;
    if (capacity > INT32_MAX)
        return TA_ERR_SHAPE;
    if (B > 0) {
        if (!q->data || !k->data || !v->data || !sl->data || !par->data || !out->data ||
            (pt && !pt->data) || (lse && !lse->data))
            return TA_ERR_NULL;
    }
    int kernel = TA_KERNEL_AUTO, num_splits = 0, item_cost = 0;
    const ta_tensor *kn = nullptr, *vn = nullptr;
    float scale = 0.f;
    void *user_ws = nullptr;
    size_t user_ws_bytes = 0;
    if (opts) {
        if (opts->item_cost < 0 || opts->item_cost > 4096 || opts->reserved != 0 || opts->num_splits < 0 ||
            opts->kernel < TA_KERNEL_AUTO ||
            opts->kernel > TA_KERNEL_MFMA_BASIC)
            return TA_ERR_OPTS;
        kernel = opts->kernel;
        num_splits = opts->num_splits;
        item_cost = opts->item_cost;
        if (opts->tree_masks && (((uintptr_t)opts->tree_masks % 8) != 0 || opts->tree_masks_stride < 0))
            return TA_ERR_OPTS;
        if (opts->kv_start && ((uintptr_t)opts->kv_start % 4) != 0)
            return TA_ERR_OPTS;
        if (opts->status && ((uintptr_t)opts->status % 4) != 0)
            return TA_ERR_OPTS;
        if ((opts->k_new != nullptr) != (opts->v_new != nullptr))
            return TA_ERR_OPTS;
        if (opts->k_new) {
            // the tree tokens' K/V of this step, dense: [B, T, Hkv, D] in the cache's dtype, rows contiguous
            for (const ta_tensor *n : {opts->k_new, opts->v_new}) {
                if (n->dtype != k->dtype)
                    return TA_ERR_DTYPE;
                if (n->ndim != 4)
                    return TA_ERR_RANK;
                if (n->shape[0] != B || n->shape[1] != T || n->shape[2] != Hkv || n->shape[3] != D)
                    return TA_ERR_SHAPE;
                if (!strides_ok(n) || n->stride[3] != 1)
                    return TA_ERR_STRIDE;
                if (B > 0 && !n->data)
                    return TA_ERR_NULL;
            }
            kn = opts->k_new;
            vn = opts->v_new;
        }
        scale = opts->scale;
        user_ws = opts->workspace;
        user_ws_bytes = opts->workspace_bytes;
        if (user_ws && ((uintptr_t)user_ws % 256) != 0)
            return TA_ERR_WORKSPACE;
    }
    if (!(scale > 0.f) || !isfinite(scale))
        scale = 1.0f / sqrtf((float)D);

    int ps_shift = -1;
    for (int s = 0; s <= 30; ++s)
        if (((int64_t)1 << s) == ps)
            ps_shift = s;
    const bool mfma_ok = q->dtype == TA_BF16 && (D == 128 || D == 64) && (!pt || ps_shift >= 0) &&
                         q->stride[2] % 8 == 0 && q->stride[1] % 8 == 0 && q->stride[0] % 8 == 0 &&
                         k->stride[0] % 8 == 0 && k->stride[1] % 8 == 0 && k->stride[2] % 8 == 0 &&
                         v->stride[0] % 8 == 0 && v->stride[1] % 8 == 0 && v->stride[2] % 8 == 0 &&
                         ((uintptr_t)q->data % 16) == 0 && ((uintptr_t)k->data % 16) == 0 &&
                         ((uintptr_t)v->data % 16) == 0 && k->stride[0] < INT32_MAX && k->stride[2] < INT32_MAX &&
                         v->stride[0] < INT32_MAX && v->stride[2] < INT32_MAX && Hq / Hkv <= 256 &&
                         (!kn || (new_rows_aligned(kn) && new_rows_aligned(vn)));
    int basic = kernel == TA_KERNEL_MFMA_BASIC ? 1 : 0;
    if (basic)
        kernel = TA_KERNEL_MFMA;
    if (kernel == TA_KERNEL_MFMA && !mfma_ok)
        return TA_ERR_OPTS;
    if (kernel == TA_KERNEL_AUTO)
        kernel = mfma_ok ? TA_KERNEL_MFMA : TA_KERNEL_GENERIC;
    if (kernel == TA_KERNEL_MFMA && D != 128)
        basic = 1;                               // the pipelined kernel is written for head_dim 128 only

    TAParams &p = pr->p;
    memset(&p, 0, sizeof p);
    p.basic = basic;
    p.q = q->data; p.k = k->data; p.v = v->data; p.out = out->data;
    p.lse = lse ? (float *)lse->data : nullptr;
    p.page_table = pt ? (const int32_t *)pt->data : nullptr;
    p.seq_lens = (const int32_t *)sl->data;
    p.parent = (const int32_t *)par->data;
    p.q_sb = q->stride[0]; p.q_st = q->stride[1]; p.q_sh = q->stride[2];
    p.o_sb = out->stride[0]; p.o_st = out->stride[1]; p.o_sh = out->stride[2];
    p.k_sp = k->stride[0]; p.k_sh = k->stride[1]; p.k_ss = k->stride[2];
    p.v_sp = v->stride[0]; p.v_sh = v->stride[1]; p.v_ss = v->stride[2];
    if (lse) { p.lse_sb = lse->stride[0]; p.lse_sh = lse->stride[1]; p.lse_st = lse->stride[2]; }
    p.pt_sb = pt ? pt->stride[0] : 0;
    p.par_sb = par->ndim == 2 ? par->stride[0] : 0;
    p.sl_s = sl->stride[0];
    p.B = (int)B; p.T = (int)T; p.Hq = (int)Hq; p.Hkv = (int)Hkv; p.G = (int)(Hq / Hkv); p.D = (int)D;
    p.ps = (int)ps; p.ps_shift = ps_shift; p.capacity = (int)capacity; p.n_pages = (int)n_pages;
    p.rows = (int)Tq * p.G;
    p.q_off = (int)q_off;
    p.g_magic = (1u << 24) / (uint32_t)p.G + 1u;
    p.masks_in = opts ? (const unsigned long long *)opts->tree_masks : nullptr;
    p.masks_sb = opts ? opts->tree_masks_stride : 0;
    p.kv_start = opts ? (const int32_t *)opts->kv_start : nullptr;
    p.status2 = opts ? opts->status : nullptr;
    p.is_bf16 = q->dtype == TA_BF16;
    if (kn) {
        p.kn = kn->data; p.vn = vn->data;
        p.kn_sb = kn->stride[0]; p.kn_st = kn->stride[1]; p.kn_sh = kn->stride[2];
        p.vn_sb = vn->stride[0]; p.vn_st = vn->stride[1]; p.vn_sh = vn->stride[2];
        const int es = p.is_bf16 ? 2 : 4;
        const int per16 = 16 / es;
        auto vec_ok = [&](const void *ptr, int64_t a, int64_t b2, int64_t c) {
            return ((uintptr_t)ptr % 16) == 0 && a % per16 == 0 && b2 % per16 == 0 && c % per16 == 0;
        };
        p.kn_vec = D % per16 == 0 && vec_ok(kn->data, kn->stride[0], kn->stride[1], kn->stride[2]) &&
                   vec_ok(vn->data, vn->stride[0], vn->stride[1], vn->stride[2]) &&
                   vec_ok(k->data, k->stride[0], k->stride[1], k->stride[2]) &&
                   vec_ok(v->data, v->stride[0], v->stride[1], v->stride[2]);
    }
    p.scale_log2e = scale * 1.4426950408889634f;

    // ---- the launch plan: one row of the dispatch table, unless the options fix a value
    TAPlan &pl = pr->plan;
    pl.kernel = kernel;
    const int family = kernel == TA_KERNEL_MFMA ? (basic ? TA_KERNEL_MFMA_BASIC : TA_KERNEL_MFMA) : TA_KERNEL_GENERIC;
    if (kernel == TA_KERNEL_MFMA) {
        pl.rows_grp = mfma_rows_group(p.rows);
        pl.threads = 512;                                   // always eight waves
    } else {
        pl.rows_grp = p.rows < TA_ROW_GROUP ? p.rows : TA_ROW_GROUP;
        pl.threads = 256;
    }
    pl.n_rg = (p.rows + pl.rows_grp - 1) / pl.rows_grp;
    const int64_t lists = B * Hkv;
    const int row = find_row(family, pl.rows_grp, lists);
    if (row < 0)
        return TA_ERR_OPTS;                                 // cannot happen: every family ends in a catch-all row
    const TADispatchRow &dr = kTable[row];
    pl.table_row = row;
    pl.item_cost = item_cost > 0 ? item_cost : dr.item_cost;
    p.pad = pl.item_cost - 1;
    const int64_t tiles_cap = lists * ((capacity - T + TA_TILE - 1) / TA_TILE + 1);
    if (tiles_cap + lists * p.pad > INT32_MAX)              // schedule units are counted in 32 bits
        return TA_ERR_SHAPE;
    int64_t want = (int64_t)num_cus * dr.wg_per_cu_x4 / 4;
    if (kernel == TA_KERNEL_MFMA)
        want /= pl.n_rg;                                    // the row groups of a list run side by side
    if (want < 1)
        want = 1;
    pl.n_wg = (int)(num_splits > 0 ? num_splits : want);
    pl.min_q = num_splits > 0 ? 1 : dr.min_share;
    if (pl.n_wg > tiles_cap)
        pl.n_wg = (int)(tiles_cap > 0 ? tiles_cap : 1);
    pl.n_slots = pl.n_wg + (int)lists;
    p.rows_grp = pl.rows_grp; p.n_rg = pl.n_rg; p.n_wg = pl.n_wg; p.min_q = pl.min_q;

    // merge kernel: partials per list the schedule produces on average = the KV pass's workgroups spread over the
    // lists, plus the one boundary each list shares with its neighbour
    const bool out_aligned = ((uintptr_t)out->data % 16) == 0 && p.o_sb % 4 == 0 && p.o_st % 4 == 0 && p.o_sh % 4 == 0;
    pl.merge_kind = TA_MERGE_GENERAL;
    if (D == 128 && out_aligned) {
        const int64_t l1 = lists > 0 ? lists : 1;
        const int64_t parts = (pl.n_wg + l1 - 1) / l1 + 1;
        const bool wide = dr.wide_from_parts > 0 && parts >= dr.wide_from_parts && lists * p.rows <= dr.wide_max_rows;
        pl.merge_kind = wide ? TA_MERGE_D128_WIDE : TA_MERGE_D128;
    }
    // Partial format of the matrix-core kernels: 16-bit fixed point with a scale per row, which halves what the KV pass
    // writes (C3 128.6 -> 125.0 us, p4 215.1 -> 210.2, C2 26.5 -> 24.1; batch-one shapes 1 to 2 us of 35).  The scalar
    // kernel, whose inputs may be fp32, keeps fp32 partials.
    p.part_q15 = kernel == TA_KERNEL_MFMA ? 1 : 0;
    p.merge_kind = pl.merge_kind;
    const int mrows = ta_host_merge_rows(p);
    pl.merge_wgs = (int)lists * ((p.rows + mrows - 1) / mrows);

    const size_t rows_total = (size_t)pl.n_slots * pl.n_rg * pl.rows_grp;
    pr->ws_o_bytes = ta_host_align_up(rows_total * D * sizeof(float), 256);
    pr->ws_lse_bytes = ta_host_align_up(rows_total * sizeof(float), 256);
    // (with 16-bit partials: rows_total * 8 bytes of {log-sum-exp, scale} fit into the unused half of the ws_o area)
    pr->ws_ls_off = p.part_q15 ? ta_host_align_up(rows_total * D * 2, 256) : pr->ws_o_bytes;
    p.ls = p.part_q15 ? 2 : 1;
    pr->ws_bytes = pr->ws_o_bytes + pr->ws_lse_bytes + ta_host_align_up((size_t)lists * 2 * sizeof(int32_t), 256);
    if (user_ws) {
        if (user_ws_bytes < pr->ws_bytes)
            return TA_ERR_WORKSPACE;
        p.ws_o = (float *)user_ws;
        p.ws_lse = (float *)((char *)user_ws + pr->ws_ls_off);
        p.ws_parts = (int32_t *)((char *)user_ws + pr->ws_o_bytes + pr->ws_lse_bytes);
    }
    return TA_OK;
}

void ta_host_fill_plan(const TAProblem &pr, int64_t plan[16])
{
    for (int i = 0; i < 16; ++i)
        plan[i] = 0;
    plan[0] = pr.plan.kernel;
    plan[1] = pr.plan.n_wg;
    plan[2] = pr.plan.threads;
    plan[3] = TA_TILE;
    plan[4] = pr.plan.n_rg;
    plan[5] = pr.plan.rows_grp;
    plan[6] = pr.plan.n_slots;
    plan[7] = pr.plan.merge_wgs;
    plan[8] = pr.plan.min_q;
    plan[9] = pr.plan.item_cost;
    plan[10] = pr.plan.merge_kind;
    plan[11] = pr.plan.table_row;
    plan[12] = (int64_t)pr.ws_bytes;
    plan[13] = pr.p.part_q15;
}

size_t ta_host_workspace_bytes(int32_t B, int32_t T, int32_t Hq, int32_t Hkv, int32_t D, int32_t dtype, int32_t num_cus)
{
    if (B < 0 || B > TA_MAX_BATCH || T < 1 || T > TA_MAX_TREE || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || D < 1 ||
        D > TA_MAX_HEAD_DIM || (dtype != TA_BF16 && dtype != TA_F32) || num_cus <= 0)
        return 0;
    // Worst case over the dispatch table: most workgroups per CU of any row, rows padded to the MFMA row group.
    int per_cu_x4 = 4;
    for (int i = 0; i < kTableRows; ++i)
        per_cu_x4 = kTable[i].wg_per_cu_x4 > per_cu_x4 ? kTable[i].wg_per_cu_x4 : per_cu_x4;
    const int rows = T * (Hq / Hkv);
    const int rows_grp = mfma_rows_group(rows);
    const size_t n_rg = (rows + rows_grp - 1) / rows_grp;
    const size_t slots = (size_t)num_cus * per_cu_x4 / 4 + (size_t)B * Hkv;
    const size_t rows_total = slots * n_rg * rows_grp;
    return ta_host_align_up(rows_total * D * sizeof(float), 256) + ta_host_align_up(rows_total * sizeof(float), 256) +
           ta_host_align_up((size_t)B * Hkv * 2 * sizeof(int32_t), 256);
}

int ta_host_check_encode(const ta_tensor *tree_parent, const ta_tensor *masks, int *B_out, int *T_out, int64_t *par_sb)
{
    if (!tree_parent || !masks)
        return TA_ERR_NULL;
    if (tree_parent->dtype != TA_I32 || masks->dtype != TA_U64)
        return TA_ERR_DTYPE;
    if ((tree_parent->ndim != 1 && tree_parent->ndim != 2) || masks->ndim != tree_parent->ndim)
        return TA_ERR_RANK;
    const int nd = tree_parent->ndim;
    const int64_t B = nd == 2 ? tree_parent->shape[0] : 1, T = tree_parent->shape[nd - 1];
    if (T < 1 || T > TA_MAX_TREE)
        return TA_ERR_TREE_SIZE;
    if (B < 0 || B > TA_MAX_BATCH)
        return TA_ERR_BATCH;
    for (int i = 0; i < nd; ++i)
        if (masks->shape[i] != tree_parent->shape[i])
            return TA_ERR_SHAPE;
    if (!strides_ok(tree_parent) || !strides_ok(masks) || (nd == 2 && masks->stride[0] != T && B > 1))
        return TA_ERR_STRIDE;
    if (B > 0 && (!tree_parent->data || !masks->data))
        return TA_ERR_NULL;
    *B_out = (int)B;
    *T_out = (int)T;
    *par_sb = nd == 2 ? tree_parent->stride[0] : 0;
    return TA_OK;
}

int ta_host_check_append(const ta_tensor *kn, const ta_tensor *vn, const ta_tensor *k, const ta_tensor *v,
                         const ta_tensor *pt, const ta_tensor *sl, TAAppend *out)
{
    if (!kn || !vn || !k || !v || !sl)
        return TA_ERR_NULL;
    if ((kn->dtype != TA_BF16 && kn->dtype != TA_F32) || vn->dtype != kn->dtype || k->dtype != kn->dtype ||
        v->dtype != kn->dtype || sl->dtype != TA_I32 || (pt && pt->dtype != TA_I32))
        return TA_ERR_DTYPE;
    if (kn->ndim != 4 || vn->ndim != 4 || k->ndim != 4 || v->ndim != 4 || sl->ndim != 1 || (pt && pt->ndim != 2))
        return TA_ERR_RANK;
    const int64_t B = kn->shape[0], T = kn->shape[1], Hkv = kn->shape[2], D = kn->shape[3], ps = k->shape[2];
    if (B < 0 || B > TA_MAX_BATCH)
        return TA_ERR_BATCH;
    if (T < 1 || T > TA_MAX_TREE)
        return TA_ERR_TREE_SIZE;
    if (D < 1 || D > TA_MAX_HEAD_DIM)
        return TA_ERR_HEAD_DIM;
    for (int i = 0; i < 4; ++i)
        if (vn->shape[i] != kn->shape[i] || v->shape[i] != k->shape[i])
            return TA_ERR_SHAPE;
    if (Hkv < 1 || k->shape[1] != Hkv || k->shape[3] != D || ps < 1 || sl->shape[0] != B || k->shape[0] < 0 ||
        k->shape[0] > INT32_MAX)
        return TA_ERR_SHAPE;
    if (pt ? (pt->shape[0] != B || pt->shape[1] < 1) : k->shape[0] < B)
        return TA_ERR_PAGE_TABLE;
    if (!strides_ok(kn) || !strides_ok(vn) || !strides_ok(k) || !strides_ok(v) || !strides_ok(sl) ||
        (pt && !strides_ok(pt)) || kn->stride[3] != 1 || vn->stride[3] != 1 || k->stride[3] != 1 || v->stride[3] != 1 ||
        (pt && pt->stride[1] != 1))
        return TA_ERR_STRIDE;
    const int64_t capacity = pt ? pt->shape[1] * ps : ps;
    if (capacity < T)
        return TA_ERR_PAGE_TABLE;
    if (capacity > INT32_MAX)
        return TA_ERR_SHAPE;
    if (B > 0 && (!kn->data || !vn->data || !k->data || !v->data || !sl->data || (pt && !pt->data)))
        return TA_ERR_NULL;
    TAAppend &a = *out;
    memset(&a, 0, sizeof a);
    a.k_new = kn->data; a.v_new = vn->data; a.k = k->data; a.v = v->data;
    a.page_table = pt ? (const int32_t *)pt->data : nullptr;
    a.seq_lens = (const int32_t *)sl->data;
    a.kn_sb = kn->stride[0]; a.kn_st = kn->stride[1]; a.kn_sh = kn->stride[2];
    a.vn_sb = vn->stride[0]; a.vn_st = vn->stride[1]; a.vn_sh = vn->stride[2];
    a.k_sp = k->stride[0]; a.k_sh = k->stride[1]; a.k_ss = k->stride[2];
    a.v_sp = v->stride[0]; a.v_sh = v->stride[1]; a.v_ss = v->stride[2];
    a.pt_sb = pt ? pt->stride[0] : 0;
    a.sl_s = sl->stride[0];
    a.B = (int)B; a.T = (int)T; a.Hkv = (int)Hkv; a.D = (int)D; a.ps = (int)ps; a.capacity = (int)capacity;
    a.n_pages = (int)k->shape[0];
    a.elem_bytes = kn->dtype == TA_BF16 ? 2 : 4;
    return TA_OK;
}

int ta_host_check_compact(const ta_tensor *k, const ta_tensor *v, const ta_tensor *pt, const ta_tensor *sl,
                          const ta_tensor *ac, const ta_tensor *na, int32_t tree_size, const ta_tensor *so,
                          TACompact *out)
{
    if (!k || !v || !sl || !ac || !na)
        return TA_ERR_NULL;
    if ((k->dtype != TA_BF16 && k->dtype != TA_F32) || v->dtype != k->dtype || sl->dtype != TA_I32 ||
        ac->dtype != TA_I32 || na->dtype != TA_I32 || (pt && pt->dtype != TA_I32) || (so && so->dtype != TA_I32))
        return TA_ERR_DTYPE;
    if (k->ndim != 4 || v->ndim != 4 || sl->ndim != 1 || ac->ndim != 2 || na->ndim != 1 || (pt && pt->ndim != 2) ||
        (so && so->ndim != 1))
        return TA_ERR_RANK;
    const int64_t B = ac->shape[0], A = ac->shape[1], Hkv = k->shape[1], D = k->shape[3], ps = k->shape[2];
    const int64_t T = tree_size;
    if (B < 0 || B > TA_MAX_BATCH)
        return TA_ERR_BATCH;
    if (T < 1 || T > TA_MAX_TREE || A < 1 || A > TA_MAX_TREE)
        return TA_ERR_TREE_SIZE;
    if (D < 1 || D > TA_MAX_HEAD_DIM)
        return TA_ERR_HEAD_DIM;
    for (int i = 0; i < 4; ++i)
        if (v->shape[i] != k->shape[i])
            return TA_ERR_SHAPE;
    if (Hkv < 1 || ps < 1 || sl->shape[0] != B || na->shape[0] != B || (so && so->shape[0] != B) || k->shape[0] < 0 ||
        k->shape[0] > INT32_MAX)
        return TA_ERR_SHAPE;
    if (pt ? (pt->shape[0] != B || pt->shape[1] < 1) : k->shape[0] < B)
        return TA_ERR_PAGE_TABLE;
    if (!strides_ok(k) || !strides_ok(v) || !strides_ok(ac) || (pt && !strides_ok(pt)) || k->stride[3] != 1 ||
        v->stride[3] != 1 || (pt && pt->stride[1] != 1) || sl->stride[0] < 0 || na->stride[0] < 0 ||
        (so && so->stride[0] < 0))
        return TA_ERR_STRIDE;
    const int64_t capacity = pt ? pt->shape[1] * ps : ps;
    if (capacity < T)
        return TA_ERR_PAGE_TABLE;
    if (capacity > INT32_MAX)
        return TA_ERR_SHAPE;
    if (B > 0 && (!k->data || !v->data || !sl->data || !ac->data || !na->data || (pt && !pt->data) || (so && !so->data)))
        return TA_ERR_NULL;
    if (so && B > 1) {
        // the lengths may be updated in place; any other overlap of the two arrays would let one request's new length
        // be read as another's old one
        const bool same = so->data == sl->data && so->stride[0] == sl->stride[0];
        const uintptr_t a0 = (uintptr_t)sl->data, a1 = a0 + (uintptr_t)((B - 1) * sl->stride[0] + 1) * 4;
        const uintptr_t b0 = (uintptr_t)so->data, b1 = b0 + (uintptr_t)((B - 1) * so->stride[0] + 1) * 4;
        if (!same && a0 < b1 && b0 < a1)
            return TA_ERR_STRIDE;
    }
    TACompact &c = *out;
    memset(&c, 0, sizeof c);
    c.k = k->data; c.v = v->data;
    c.page_table = pt ? (const int32_t *)pt->data : nullptr;
    c.seq_lens = (const int32_t *)sl->data;
    c.accepted = (const int32_t *)ac->data;
    c.n_accepted = (const int32_t *)na->data;
    c.seq_lens_out = so ? (int32_t *)so->data : nullptr;
    c.k_sp = k->stride[0]; c.k_sh = k->stride[1]; c.k_ss = k->stride[2];
    c.v_sp = v->stride[0]; c.v_sh = v->stride[1]; c.v_ss = v->stride[2];
    c.pt_sb = pt ? pt->stride[0] : 0;
    c.sl_s = sl->stride[0]; c.acc_sb = ac->stride[0]; c.na_s = na->stride[0]; c.slo_s = so ? so->stride[0] : 0;
    c.B = (int)B; c.T = (int)T; c.A = (int)A; c.Hkv = (int)Hkv; c.D = (int)D; c.ps = (int)ps; c.capacity = (int)capacity;
    c.n_pages = (int)k->shape[0];
    c.elem_bytes = k->dtype == TA_BF16 ? 2 : 4;
    return TA_OK;
}

// ---- entry points that need no device at all
extern "C" {

int tree_attn_version(void) { return TREEATTN_VERSION; }

const char *tree_attn_strerror(int status)
{
    switch (status) {
    case TA_OK: return "ok";
    case TA_ERR_NULL: return "a required descriptor or data pointer is NULL";
    case TA_ERR_DTYPE: return "unsupported or mismatching element type";
    case TA_ERR_RANK: return "wrong number of dimensions";
    case TA_ERR_SHAPE: return "shapes disagree";
    case TA_ERR_STRIDE: return "innermost stride must be 1 and strides must be non-negative";
    case TA_ERR_HEADS: return "query heads must be a multiple of KV heads";
    case TA_ERR_HEAD_DIM: return "head_dim out of range";
    case TA_ERR_TREE_SIZE: return "tree size must be in [1, 64]";
    case TA_ERR_PAGE_TABLE: return "page table cannot hold the tree tokens";
    case TA_ERR_WORKSPACE: return "workspace too small or misaligned, or it would have to grow under stream capture";
    case TA_ERR_HIP: return "HIP runtime call failed";
    case TA_ERR_BATCH: return "batch size out of range";
    case TA_ERR_OPTS: return "invalid option";
    default: return "unknown status";
    }
}

int tree_attn_plan(const ta_tensor *q, const ta_tensor *k_cache, const ta_tensor *v_cache,
                   const ta_tensor *page_table, const ta_tensor *seq_lens, const ta_tensor *tree_parent,
                   const ta_tensor *out, const ta_tensor *lse, const ta_opts *opts, int32_t num_cus,
                   int64_t plan[16])
{
    if (!plan)
        return TA_ERR_NULL;
    TAProblem pr;
    ta_opts o;
    if (opts) {
        o = *opts;
        o.workspace = nullptr;      // planning never needs the scratch itself
        o.workspace_bytes = 0;
    }
    int rc = ta_host_build_problem(q, k_cache, v_cache, page_table, seq_lens, tree_parent, out, lse,
                                   opts ? &o : nullptr, num_cus > 0 ? num_cus : 256, &pr);
    if (rc != TA_OK)
        return rc;
    ta_host_fill_plan(pr, plan);
    return TA_OK;
}

int tree_attn_dispatch_row(int32_t index, int64_t row[8])
{
    if (!row)
        return TA_ERR_NULL;
    if (index < 0 || index >= kTableRows)
        return TA_ERR_OPTS;
    const TADispatchRow &r = kTable[index];
    row[0] = r.family; row[1] = r.rows_grp_max; row[2] = r.lists_max; row[3] = r.wg_per_cu_x4;
    row[4] = r.min_share; row[5] = r.item_cost; row[6] = r.wide_from_parts; row[7] = r.wide_max_rows;
    return TA_OK;
}

}  // extern "C"
