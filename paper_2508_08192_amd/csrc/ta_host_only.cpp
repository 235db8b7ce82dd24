// The launching entry points of libtreeattn without a device behind them: every call is validated and planned by
// the same host code as in the real library (ta_host.cpp) and then stops with TA_ERR_HIP where the real one would
// touch the GPU.  Linked with ta_host.cpp into the checking build of the host logic (g++ with
// -fsanitize=address,undefined; see build.py: build_host_checked), which the CPU tests load in place of the real
// library.  Never part of libtreeattn.so.
#include "ta_params.h"

extern "C" {

size_t tree_attn_workspace_bytes(int32_t B, int32_t T, int32_t Hq, int32_t Hkv, int32_t D, int32_t dtype,
                                 int32_t num_cus)
{
    return ta_host_workspace_bytes(B, T, Hq, Hkv, D, dtype, num_cus > 0 ? num_cus : 256);
}

int tree_attn_reserve(size_t) { return TA_ERR_HIP; }
int tree_attn_release(void) { return TA_ERR_HIP; }

int tree_attn_fwd_ex(const ta_tensor *q, const ta_tensor *k_cache, const ta_tensor *v_cache,
                     const ta_tensor *page_table, const ta_tensor *seq_lens, const ta_tensor *tree_parent,
                     ta_tensor *out, ta_tensor *lse, void *, const ta_opts *opts)
{
    TAProblem pr;
    int rc = ta_host_build_problem(q, k_cache, v_cache, page_table, seq_lens, tree_parent, out, lse, opts, 256, &pr);
    if (rc != TA_OK)
        return rc;
    return pr.p.B == 0 ? TA_OK : TA_ERR_HIP;
}

int tree_attn_fwd(const ta_tensor *q, const ta_tensor *k_cache, const ta_tensor *v_cache,
                  const ta_tensor *page_table, const ta_tensor *seq_lens, const ta_tensor *tree_parent,
                  ta_tensor *out, ta_tensor *lse, void *stream)
{
    return tree_attn_fwd_ex(q, k_cache, v_cache, page_table, seq_lens, tree_parent, out, lse, stream, nullptr);
}

int tree_attn_fwd_static(const ta_tensor *q, const ta_tensor *k_cache, const ta_tensor *v_cache,
                         const ta_tensor *page_table, const ta_tensor *seq_lens, const ta_tensor *tree_parent,
                         ta_tensor *out, ta_tensor *lse, void *stream, const ta_opts *opts)
{
    if (opts && opts->workspace)
        return TA_ERR_OPTS;
    TAProblem pr;
    int rc = ta_host_build_problem(q, k_cache, v_cache, page_table, seq_lens, tree_parent, out, lse, opts, 256, &pr);
    if (rc != TA_OK)
        return rc;
    if (pr.p.B == 0)
        return TA_OK;
    (void)stream;
    return pr.ws_bytes > (size_t)TA_STATIC_SCRATCH_BYTES ? TA_ERR_WORKSPACE : TA_ERR_HIP;
}

int tree_attn_encode(const ta_tensor *tree_parent, ta_tensor *masks, void *)
{
    int B = 0, T = 0;
    int64_t par_sb = 0;
    int rc = ta_host_check_encode(tree_parent, masks, &B, &T, &par_sb);
    return rc != TA_OK || B == 0 ? rc : TA_ERR_HIP;
}

int tree_attn_append(const ta_tensor *k_new, const ta_tensor *v_new, ta_tensor *k_cache, ta_tensor *v_cache,
                     const ta_tensor *page_table, const ta_tensor *seq_lens, void *)
{
    TAAppend a;
    int rc = ta_host_check_append(k_new, v_new, k_cache, v_cache, page_table, seq_lens, &a);
    return rc != TA_OK || a.B == 0 ? rc : TA_ERR_HIP;
}

int tree_attn_compact(ta_tensor *k_cache, ta_tensor *v_cache, const ta_tensor *page_table, const ta_tensor *seq_lens,
                      const ta_tensor *accepted, const ta_tensor *n_accepted, int32_t tree_size,
                      ta_tensor *seq_lens_out, void *)
{
    TACompact c;
    int rc = ta_host_check_compact(k_cache, v_cache, page_table, seq_lens, accepted, n_accepted, tree_size,
                                   seq_lens_out, &c);
    return rc != TA_OK || c.B == 0 ? rc : TA_ERR_HIP;
}

int tree_attn_last_status(int32_t *host_status, void *) { return host_status ? TA_ERR_HIP : TA_ERR_NULL; }

int tree_attn_stream_read(const void *buf, size_t bytes, void *sink, void *)
{
    if (!buf || !sink)
        return TA_ERR_NULL;
    if (((uintptr_t)buf % 16) != 0 || bytes % 16 != 0 || ((uintptr_t)sink % 4) != 0)
        return TA_ERR_STRIDE;
    return bytes == 0 ? TA_OK : TA_ERR_HIP;
}

int tree_attn_mfma_probe(int32_t iters, void *sink, int64_t *, void *)
{
    if (!sink)
        return TA_ERR_NULL;
    if (iters < 1 || iters > (1 << 20) || ((uintptr_t)sink % 4) != 0)
        return TA_ERR_OPTS;
    return TA_ERR_HIP;
}

}  // extern "C"
