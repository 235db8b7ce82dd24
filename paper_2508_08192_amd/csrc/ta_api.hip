// C-ABI of libtreeattn: per-device state and the entry points that launch.  Descriptor validation, planning and the
// dispatch table are plain host code in ta_host.cpp; this file adds what needs the HIP runtime.
// See include/treeattn.h for the contract of every entry point.
#include <mutex>
#include <vector>

#include "ta_common.h"

namespace {

// The sticky status word of a device lives in the library image (every device holds its own copy of the array at its
// own address), so that no entry point has to allocate it.
__device__ __align__(256) int32_t ta_status_words[TA_STATUS_BYTES / 4];

// Scratch of tree_attn_fwd_static: the split-KV partial results of a call, for callers that cannot allocate.  In host
// code this name is only a handle for hipGetSymbolAddress; the device address of each GPU's copy is kept per device.
__device__ __align__(256) unsigned char scratch[TA_STATIC_SCRATCH_BYTES];

struct DeviceState {
    std::once_flag once;
    int init_rc = TA_ERR_HIP;
    int num_cus = 0;
    int32_t *status = nullptr;
    void *scratch_ptr = nullptr;       // this device's copy of `scratch`
    // library-owned workspace: grown under ws_mu; buffers it outgrew stay allocated (launches and captured graphs
    // may still hold their addresses) until tree_attn_release
    std::mutex ws_mu;
    void *ws = nullptr;
    size_t ws_bytes = 0;
    std::vector<void *> retired;
};

constexpr int kMaxDevices = 64;
DeviceState g_dev[kMaxDevices];

// State of the current device; the first call on a device resolves its status word and reads its size.  Allocates
// nothing.
int device_state(DeviceState **out, int *dev_out = nullptr)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return TA_ERR_HIP;
    }
    DeviceState &s = g_dev[dev];
    std::call_once(s.once, [&]() {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            return;
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(ta_status_words)) != hipSuccess || !ptr)
            return;
        void *sptr = nullptr;
        if (hipGetSymbolAddress(&sptr, HIP_SYMBOL(scratch)) != hipSuccess || !sptr)
            return;
        s.scratch_ptr = sptr;
        s.status = (int32_t *)ptr;
        s.num_cus = cus;
        s.init_rc = TA_OK;
    });
    if (s.init_rc != TA_OK) {
        (void)hipGetLastError();
        return s.init_rc;
    }
    *out = &s;
    if (dev_out)
        *dev_out = dev;
    return TA_OK;
}

// Grows the library-owned workspace (caller holds ws_mu).  The old buffer is kept, never freed here.
int reserve_locked(DeviceState *s, size_t bytes)
{
    if (bytes <= s->ws_bytes)
        return TA_OK;
    bytes = ta_host_align_up(bytes, (size_t)1 << 20);
    void *fresh = nullptr;
    if (hipMalloc(&fresh, bytes) != hipSuccess) {
        (void)hipGetLastError();
        return TA_ERR_HIP;
    }
    if (s->ws)
        s->retired.push_back(s->ws);
    s->ws = fresh;
    s->ws_bytes = bytes;
    return TA_OK;
}

void place_workspace(TAProblem &pr, void *ws)
{
    pr.p.ws_o = (float *)ws;
    pr.p.ws_lse = (float *)((char *)ws + pr.ws_ls_off);
    pr.p.ws_parts = (int32_t *)((char *)ws + pr.ws_o_bytes + pr.ws_lse_bytes);
}

// KV pass and merge pass of a planned call on `stream`.
int launch_call(const TAProblem &pr, hipStream_t st, int dev, void *const *ev)
{
    if (ev && ev[0] && hipEventRecord((hipEvent_t)ev[0], st) != hipSuccess)
        return TA_ERR_HIP;
    hipError_t e = pr.plan.kernel == TA_KERNEL_MFMA ? ta_launch_mfma(pr.p, st, dev) : ta_launch_generic(pr.p, st, dev);
    if (e != hipSuccess)
        return TA_ERR_HIP;
    if (ev && ev[1] && hipEventRecord((hipEvent_t)ev[1], st) != hipSuccess)
        return TA_ERR_HIP;
    e = ta_launch_merge(pr.p, st);
    if (e != hipSuccess)
        return TA_ERR_HIP;
    if (ev && ev[2] && hipEventRecord((hipEvent_t)ev[2], st) != hipSuccess)
        return TA_ERR_HIP;
    return TA_OK;
}

}  // namespace

extern "C" {

size_t tree_attn_workspace_bytes(int32_t B, int32_t T, int32_t Hq, int32_t Hkv, int32_t D, int32_t dtype,
                                 int32_t num_cus)
{
    if (num_cus <= 0) {
        DeviceState *s = nullptr;
        num_cus = device_state(&s) == TA_OK ? s->num_cus : 256;
    }
    return ta_host_workspace_bytes(B, T, Hq, Hkv, D, dtype, num_cus);
}

int tree_attn_reserve(size_t bytes)
{
    DeviceState *s = nullptr;
    int rc = device_state(&s);
    if (rc != TA_OK)
        return rc;
    std::lock_guard<std::mutex> lk(s->ws_mu);
    return reserve_locked(s, bytes);
}

int tree_attn_release(void)
{
    DeviceState *s = nullptr;
    int rc = device_state(&s);
    if (rc != TA_OK)
        return rc;
    std::lock_guard<std::mutex> lk(s->ws_mu);
    if (hipDeviceSynchronize() != hipSuccess)
        return TA_ERR_HIP;
    for (void *ptr : s->retired)
        (void)hipFree(ptr);
    s->retired.clear();
    if (s->ws)
        (void)hipFree(s->ws);
    s->ws = nullptr;
    s->ws_bytes = 0;
    return TA_OK;
}

int tree_attn_fwd_ex(const ta_tensor *q, const ta_tensor *k_cache, const ta_tensor *v_cache,
                     const ta_tensor *page_table, const ta_tensor *seq_lens, const ta_tensor *tree_parent,
                     ta_tensor *out, ta_tensor *lse, void *stream, const ta_opts *opts)
{
    TAProblem pr;
    // First pass with a nominal CU count: host-visible errors are reported before any HIP call.
    int rc = ta_host_build_problem(q, k_cache, v_cache, page_table, seq_lens, tree_parent, out, lse, opts, 256, &pr);
    if (rc != TA_OK)
        return rc;
    if (pr.p.B == 0)
        return TA_OK;
    DeviceState *s = nullptr;
    int dev = 0;
    rc = device_state(&s, &dev);
    if (rc != TA_OK)
        return rc;
    rc = ta_host_build_problem(q, k_cache, v_cache, page_table, seq_lens, tree_parent, out, lse, opts, s->num_cus, &pr);
    if (rc != TA_OK)
        return rc;
    hipStream_t st = (hipStream_t)stream;
    if (!pr.p.ws_o) {
        std::lock_guard<std::mutex> lk(s->ws_mu);
        if (pr.ws_bytes > s->ws_bytes) {
            // growing means hipMalloc, which stream capture forbids: such a caller reserves beforehand
            hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
            if (hipStreamIsCapturing(st, &cap) != hipSuccess) {
                (void)hipGetLastError();
                return TA_ERR_HIP;
            }
            if (cap != hipStreamCaptureStatusNone)
                return TA_ERR_WORKSPACE;
            rc = reserve_locked(s, pr.ws_bytes);
            if (rc != TA_OK)
                return rc;
        }
        place_workspace(pr, s->ws);
    }
    pr.p.status = s->status;
    return launch_call(pr, st, dev, opts ? opts->events : nullptr);
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
    DeviceState *s = nullptr;
    int dev = 0;
    rc = device_state(&s, &dev);
    if (rc != TA_OK)
        return rc;
    rc = ta_host_build_problem(q, k_cache, v_cache, page_table, seq_lens, tree_parent, out, lse, opts, s->num_cus, &pr);
    if (rc != TA_OK)
        return rc;
    if (pr.ws_bytes > (size_t)TA_STATIC_SCRATCH_BYTES)
        return TA_ERR_WORKSPACE;
    // Nothing in the scratch has to start at zero: the KV pass writes every partial result and every list's range of
    // partials before the merge pass, which follows it on the same stream, reads them.
    place_workspace(pr, s->scratch_ptr);
    pr.p.status = s->status;
    return launch_call(pr, (hipStream_t)stream, dev, opts ? opts->events : nullptr);
}

int tree_attn_fwd(const ta_tensor *q, const ta_tensor *k_cache, const ta_tensor *v_cache,
                  const ta_tensor *page_table, const ta_tensor *seq_lens, const ta_tensor *tree_parent,
                  ta_tensor *out, ta_tensor *lse, void *stream)
{
    return tree_attn_fwd_ex(q, k_cache, v_cache, page_table, seq_lens, tree_parent, out, lse, stream, nullptr);
}

int tree_attn_encode(const ta_tensor *tree_parent, ta_tensor *masks, void *stream)
{
    int B = 0, T = 0;
    int64_t par_sb = 0;
    int rc = ta_host_check_encode(tree_parent, masks, &B, &T, &par_sb);
    if (rc != TA_OK || B == 0)
        return rc;
    DeviceState *s = nullptr;
    rc = device_state(&s);
    if (rc != TA_OK)
        return rc;
    hipError_t e = ta_launch_encode((const int32_t *)tree_parent->data, par_sb, B, T, (unsigned long long *)masks->data,
                                    s->status, (hipStream_t)stream);
    return e == hipSuccess ? TA_OK : TA_ERR_HIP;
}

int tree_attn_append(const ta_tensor *k_new, const ta_tensor *v_new, ta_tensor *k_cache, ta_tensor *v_cache,
                     const ta_tensor *page_table, const ta_tensor *seq_lens, void *stream)
{
    TAAppend a;
    int rc = ta_host_check_append(k_new, v_new, k_cache, v_cache, page_table, seq_lens, &a);
    if (rc != TA_OK || a.B == 0)
        return rc;
    DeviceState *s = nullptr;
    rc = device_state(&s);
    if (rc != TA_OK)
        return rc;
    a.status = s->status;
    return ta_launch_append(a, (hipStream_t)stream) == hipSuccess ? TA_OK : TA_ERR_HIP;
}

int tree_attn_compact(ta_tensor *k_cache, ta_tensor *v_cache, const ta_tensor *page_table, const ta_tensor *seq_lens,
                      const ta_tensor *accepted, const ta_tensor *n_accepted, int32_t tree_size,
                      ta_tensor *seq_lens_out, void *stream)
{
    TACompact c;
    int rc = ta_host_check_compact(k_cache, v_cache, page_table, seq_lens, accepted, n_accepted, tree_size,
                                   seq_lens_out, &c);
    if (rc != TA_OK || c.B == 0)
        return rc;
    DeviceState *s = nullptr;
    int dev = 0;
    rc = device_state(&s, &dev);
    if (rc != TA_OK)
        return rc;
    c.status = s->status;
    return ta_launch_compact(c, (hipStream_t)stream, dev) == hipSuccess ? TA_OK : TA_ERR_HIP;
}

int tree_attn_last_status(int32_t *host_status, void *stream)
{
    if (!host_status)
        return TA_ERR_NULL;
    DeviceState *s = nullptr;
    int rc = device_state(&s);
    if (rc != TA_OK)
        return rc;
    hipStream_t st = (hipStream_t)stream;
    if (hipMemcpyAsync(host_status, s->status, sizeof(int32_t), hipMemcpyDeviceToHost, st) != hipSuccess)
        return TA_ERR_HIP;
    if (hipMemsetAsync(s->status, 0, sizeof(int32_t), st) != hipSuccess)
        return TA_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess)
        return TA_ERR_HIP;
    return TA_OK;
}

int tree_attn_stream_read(const void *buf, size_t bytes, void *sink, void *stream)
{
    if (!buf || !sink)
        return TA_ERR_NULL;
    if (((uintptr_t)buf % 16) != 0 || bytes % 16 != 0 || ((uintptr_t)sink % 4) != 0)
        return TA_ERR_STRIDE;
    if (bytes == 0)
        return TA_OK;
    DeviceState *s = nullptr;
    int rc = device_state(&s);
    if (rc != TA_OK)
        return rc;
    return ta_launch_stream_read(buf, bytes, sink, s->num_cus, (hipStream_t)stream) == hipSuccess ? TA_OK : TA_ERR_HIP;
}

int tree_attn_mfma_probe(int32_t iters, void *sink, int64_t *flop, void *stream)
{
    if (!sink)
        return TA_ERR_NULL;
    if (iters < 1 || iters > (1 << 20) || ((uintptr_t)sink % 4) != 0)
        return TA_ERR_OPTS;
    DeviceState *s = nullptr;
    int rc = device_state(&s);
    if (rc != TA_OK)
        return rc;
    if (flop)
        *flop = (int64_t)s->num_cus * 8 * 32 * (int64_t)iters * 32768;
    return ta_launch_mfma_probe(iters, sink, s->num_cus, (hipStream_t)stream) == hipSuccess ? TA_OK : TA_ERR_HIP;
}

}  // extern "C"
