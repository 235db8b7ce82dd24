// Shared declarations of the libtreeattn device code: kernel parameters and the device-side work
// schedule.  Everything here is specific to gfx950 (64-wide wavefronts).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/treeattn.h"

#define TA_WAVE 64
#define TA_TILE 64            // KV tokens per tile of the KV pass (the tree tokens form one more tile)
#define TA_MERGE_ROWS 4       // rows per workgroup of the merge pass (one per wave)
#define TA_ROW_GROUP 256
#ifdef TA_TUNING
#define TA_STATUS_BYTES 65536   // room for per-workgroup timestamps
#else
#define TA_STATUS_BYTES 256
#endif      // rows (tree nodes x query heads of one KV head) one workgroup keeps

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
    float *ws_o;               // partial outputs  [slot][rg][rows_grp][D], normalised, fp32
    float *ws_lse;             // partial log2-sum-exp2 [slot][rg][rows_grp]
    int32_t *ws_parts;         // [B * Hkv][2]: first and last workgroup that hold partial results of a list; written
                               // by the KV pass (the owners of the list's first and last tile), read by the merge
    int32_t *status;           // sticky status word
    int32_t basic;             // 256-row groups: use the register-staged MFMA kernel, not the pipelined one
    // write-back folded into the call: the tree tokens' K/V come from these dense tensors [B, T, Hkv, D] (element
    // strides), the KV pass reads them there and the merge pass copies them behind the prefix in the caches
    const void *kn, *vn;
    int64_t kn_sb, kn_st, kn_sh, vn_sb, vn_st, vn_sh;
    int32_t kn_vec;            // rows can be copied in 16-byte pieces
#ifdef TA_TUNING
    int32_t dbg;               // bit flags that switch parts of a kernel off (results become wrong)
#endif
};

// Ablation switches for tuning builds (-DTA_TUNING, flags from the TREEATTN_DBG environment variable): a set
// bit removes one part of the 256-row KV kernel so that its share of the time can be read off.  A regular
// build compiles every switch to `false`.
#ifdef TA_TUNING
#define TA_OFF(bit) ((p.dbg & (bit)) != 0)
#else
#define TA_OFF(bit) false
#endif

// ---------------------------------------------------------------------------------------------
// Work schedule.  The KV pass walks, for every (request b, KV head g), a list of tiles:
// ceil(L_b / TA_TILE) prefix tiles followed by one tile holding the T tree tokens.  A malformed
// request owns a single tile (it only poisons its outputs).  All tile lists are laid end to end,
// (b major, g minor), and workgroup w takes the contiguous share [w*share, (w+1)*share).  A share
// may start or end inside a list; every (workgroup, list) overlap produces one partial result in
// slot w + (b*Hkv + g), which is unique because both terms grow along the walk.
// The prefix lengths live on the device, so every workgroup derives the schedule itself.
// ---------------------------------------------------------------------------------------------

// S: first prefix position the request's nodes still attend to (section 3.4, iRoPE for Llama4: the prefix is the current
// sub-sequence only); 0 unless the caller gave kv_start.
__device__ __forceinline__ int ta_kv_start(const TAParams &p, int b)
{
    return p.kv_start ? p.kv_start[b] : 0;
}

__device__ __forceinline__ bool ta_request_ok(const TAParams &p, int L, int S)
{
    return L >= 0 && (int64_t)L + p.T <= (int64_t)p.capacity && S >= 0 && S <= L;
}

// Tiles of one list: the 64-token tiles that hold prefix positions S..L-1 (tile S/64 is the first), then the tree
// tile.  A malformed request owns one tile.
__device__ __forceinline__ int ta_list_tiles(const TAParams &p, int L, int S)
{
    if (!ta_request_ok(p, L, S))
        return 1;
    return (S < L ? (L + TA_TILE - 1) / TA_TILE - S / TA_TILE : 0) + 1;
}

// The KV work of the batch is one line of schedule units: request after request, KV head after KV head, and
// per (request, KV head) list one unit per tile (prefix tiles, then the tree tile) followed by p.pad units of
// padding.  Workgroup w takes units [w * share, (w + 1) * share).  The padding stands for the fixed cost of starting
// on a list: every workgroup pays that once for the list it begins in, whether at its first tile or in its middle,
// and once more per list boundary inside its range -- which is exactly where it meets a padding.  A workgroup whose
// range touches only the padding of a list has no work in it and writes no partial result.
//
// cum[0..B]: exclusive prefix sums of the per-request unit counts (per KV head).  Needs blockDim.x >= 64; ends
// with a barrier.  If `lens` is given, it also receives the B prefix lengths as they were read, and `starts` the B
// window starts.
__device__ __forceinline__ void ta_build_schedule(const TAParams &p, int *cum, int *lens = nullptr,
                                                  int *starts = nullptr)
{
    const int tid = threadIdx.x;
    for (int b = tid; b < p.B; b += blockDim.x) {
        const int L = p.seq_lens[(int64_t)b * p.sl_s];
        const int S = ta_kv_start(p, b);
        cum[b + 1] = ta_list_tiles(p, L, S) + p.pad;
        if (lens)
            lens[b] = L;
        if (starts)
            starts[b] = S;
    }
    if (tid == 0)
        cum[0] = 0;
    __syncthreads();
    if (tid < TA_WAVE) {
        int carry = 0;
        for (int base = 0; base < p.B; base += TA_WAVE) {
            int idx = base + tid;
            int x = idx < p.B ? cum[idx + 1] : 0;
            for (int off = 1; off < TA_WAVE; off <<= 1) {
                int y = __shfl_up(x, off, TA_WAVE);
                if (tid >= off)
                    x += y;
            }
            if (idx < p.B)
                cum[idx + 1] = x + carry;
            carry += __shfl(x, TA_WAVE - 1, TA_WAVE);
        }
    }
    __syncthreads();
}

__device__ __forceinline__ int ta_share(const TAParams &p, int total)
{
    int share = (total + p.n_wg - 1) / p.n_wg;
    return share < p.min_q ? p.min_q : share;
}

// Request whose tile lists contain global tile t (0 <= t < Hkv * cum[B]).
__device__ __forceinline__ int ta_find_request(const TAParams &p, const int *cum, int t)
{
    int lo = 0, hi = p.B;                 // invariant: Hkv*cum[lo] <= t < Hkv*cum[hi]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if ((int64_t)p.Hkv * cum[mid] <= t)
            lo = mid;
        else
            hi = mid;
    }
    return lo;
}

// The KV pass tells the merge pass which workgroups hold partial results of list (b, g): the owner of the list's
// first tile and the owner of its last one say so (row group 0 speaks for all).  Saves the merge pass rebuilding
// the schedule from the prefix lengths in each of its many small workgroups.
__device__ __forceinline__ void ta_note_owner(const TAParams &p, int b, int g, int w, int j0, int j1, int n_b)
{
    if (threadIdx.x == 0 && blockIdx.y == 0) {
        int wv = w;
        asm volatile("" : "+s"(wv));              // made where it is stored: a copy kept in a vector register across
                                                  // the caller's item loop would be spilled there
        if (j0 == 0)
            p.ws_parts[2 * (b * p.Hkv + g)] = wv;
        if (j1 == n_b)
            p.ws_parts[2 * (b * p.Hkv + g) + 1] = wv;
    }
}

// Bit k set: token k of the prefix tile that starts at position pos0 lies inside [S, L).
__device__ __forceinline__ unsigned long long ta_prefix_tile_mask(int pos0, int L, int S)
{
    const int rem = L - pos0, lo = S - pos0;
    unsigned long long m = rem < TA_TILE ? (1ull << rem) - 1ull : ~0ull;
    if (lo > 0)
        m &= ~((1ull << lo) - 1ull);
    return m;
}

__device__ __forceinline__ int64_t ta_ws_row(const TAParams &p, int slot, int rg, int r)
{
    return ((int64_t)slot * p.n_rg + rg) * p.rows_grp + r;
}

// Element offset of logical position pos of request b, KV head g in a cache with strides (sp, sh, ss).
__device__ __forceinline__ int64_t ta_cache_offset(const TAParams &p, int b, int g, int pos,
                                                   int64_t sp, int64_t sh, int64_t ss)
{
    int64_t page, slot;
    if (p.page_table) {
        int pi = p.ps_shift >= 0 ? (pos >> p.ps_shift) : (pos / p.ps);
        slot = p.ps_shift >= 0 ? (pos & (p.ps - 1)) : (pos - pi * p.ps);
        page = p.page_table[(int64_t)b * p.pt_sb + pi];
    } else {
        page = b;
        slot = pos;
    }
    return page * sp + (int64_t)g * sh + slot * ss;
}

// Ancestor masks of one request's tree into masks[0..T): bit j of masks[i] is set iff node j is on the
// path from a root to node i (i included).  The T parent ids are first copied to shared memory in one
// round trip (`par_s`, T ints), then threads 0..T-1 each walk one node upwards there; a parent id >= T
// or a walk longer than T nodes marks the tree as malformed.  Returns (to every thread, after a barrier)
// whether the tree is well formed; `flag` is one int of shared memory.
__device__ __forceinline__ bool ta_encode_tree(const int32_t *parent, int T, unsigned long long *masks, int *flag,
                                               int *par_s)
{
    const int tid = threadIdx.x;
    if (tid == 0)
        *flag = 0;
    if (tid < T)
        par_s[tid] = parent[tid];
    __syncthreads();
    if (tid < T) {
        unsigned long long m = 0;
        int cur = tid, steps = 0;
        bool bad = false;
        while (cur >= 0) {
            if (cur >= T || steps >= T) {
                bad = true;
                break;
            }
            m |= 1ull << cur;
            cur = par_s[cur];
            ++steps;
        }
        masks[tid] = bad ? 0ull : m;
        if (bad)
            atomicOr(flag, 1);
    }
    __syncthreads();
    return *flag == 0;
}

// Masks that were encoded before the call: node tid's word of request b, bits of nodes >= T dropped.
__device__ __forceinline__ unsigned long long ta_given_mask(const TAParams &p, int b, int tid)
{
    const unsigned long long m = p.masks_in[(int64_t)b * p.masks_sb + tid];
    return p.T >= 64 ? m : m & ((1ull << p.T) - 1ull);
}

// The walk itself: par_s[0..T) and *flag = 0 are already in LDS and visible to the workgroup.  Ends with a barrier.
// tid: threadIdx.x (a parameter so that a caller short of registers can keep the compiler from hoisting its uses).
__device__ __forceinline__ bool ta_encode_tree_lds(int tid, int T, unsigned long long *masks, int *flag,
                                                   const int *par_s)
{
    if (tid < T) {
        unsigned long long m = 0;
        int cur = tid, steps = 0;
        bool bad = false;
        while (cur >= 0) {
            if (cur >= T || steps >= T) {
                bad = true;
                break;
            }
            m |= 1ull << cur;
            cur = par_s[cur];
            ++steps;
        }
        masks[tid] = bad ? 0ull : m;
        if (bad)
            atomicOr(flag, 1);
    }
    __syncthreads();
    return *flag == 0;
}

// Same, for a caller that has already loaded the parent id of node threadIdx.x (any value for threads >= T).
__device__ __forceinline__ bool ta_encode_tree_from(int parent_of_tid, int T, unsigned long long *masks, int *flag,
                                                    int *par_s)
{
    const int tid = threadIdx.x;
    if (tid == 0)
        *flag = 0;
    if (tid < T)
        par_s[tid] = parent_of_tid;
    __syncthreads();
    return ta_encode_tree_lds(tid, T, masks, flag, par_s);
}

__device__ __forceinline__ float ta_wave_max(float x)
{
    for (int off = TA_WAVE / 2; off > 0; off >>= 1)
        x = fmaxf(x, __shfl_xor(x, off, TA_WAVE));
    return x;
}

__device__ __forceinline__ float ta_wave_sum(float x)
{
    for (int off = TA_WAVE / 2; off > 0; off >>= 1)
        x += __shfl_xor(x, off, TA_WAVE);
    return x;
}

__device__ __forceinline__ float ta_bf16_to_f32(uint16_t b)
{
    return __uint_as_float((uint32_t)b << 16);
}

// Round to nearest, ties to even; NaN stays NaN.
__device__ __forceinline__ uint16_t ta_f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// The write-back of ta_opts.k_new / v_new for one (request, KV head) list: its T rows go to logical positions
// L_b .. L_b+T-1 of the caches.  Every workgroup of the merge pass takes part (workgroup `part` of the `parts` that
// serve the list moves the tokens part, part + parts, ...); nothing in the same call reads those cache positions (the
// KV pass takes the tree tokens from the dense tensors).  The work comes in three steps so that a merge kernel can
// hide it behind its own loads: ta_scatter_load issues the loads that depend on nothing (the request's length and
// this thread's first 16-byte piece), ta_scatter_locate looks the destination up in the page table once the length
// is there, ta_scatter_store writes -- and moves what the first piece per thread does not cover (more pieces than
// threads, or rows that are not 16-byte aligned) in a plain loop.
struct TAScatter {
    uint4 v;                   // this thread's first piece
    int64_t dst;               // its byte offset in the cache
    int L, S, i, c, mine, per_row;
    bool is_v, live, ok;
};

__device__ __forceinline__ void ta_scatter_load(const TAParams &p, int b, int g, int part, int parts, TAScatter &s)
{
    s.L = p.seq_lens[(int64_t)b * p.sl_s];
    s.S = ta_kv_start(p, b);
    s.live = false;
    s.ok = false;
    s.mine = part < p.T ? (p.T - part + parts - 1) / parts : 0;            // tokens of this workgroup
    const int es = p.is_bf16 ? 2 : 4;
    s.per_row = p.kn_vec ? p.D * es / 16 : p.D;                           // pieces of a row
    const int x = threadIdx.x;
    if (p.kn_vec && x < 2 * s.mine * s.per_row) {
        s.is_v = x >= s.mine * s.per_row;
        const int y = s.is_v ? x - s.mine * s.per_row : x;
        s.i = part + (y / s.per_row) * parts;
        s.c = y % s.per_row;
        const int64_t src = s.is_v ? (int64_t)b * p.vn_sb + (int64_t)s.i * p.vn_st + (int64_t)g * p.vn_sh
                                   : (int64_t)b * p.kn_sb + (int64_t)s.i * p.kn_st + (int64_t)g * p.kn_sh;
        s.v = *(const uint4 *)((const char *)(s.is_v ? p.vn : p.kn) + src * es + 16 * s.c);
        s.live = true;
    }
}

__device__ __forceinline__ void ta_scatter_locate(const TAParams &p, int b, int g, TAScatter &s)
{
    s.ok = s.mine > 0 && ta_request_ok(p, s.L, s.S);
    if (s.ok && s.live) {
        const int es = p.is_bf16 ? 2 : 4;
        s.dst = (s.is_v ? ta_cache_offset(p, b, g, s.L + s.i, p.v_sp, p.v_sh, p.v_ss)
                        : ta_cache_offset(p, b, g, s.L + s.i, p.k_sp, p.k_sh, p.k_ss)) * es + 16 * s.c;
    }
}

__device__ __forceinline__ void ta_scatter_store(const TAParams &p, int b, int g, int part, int parts, const TAScatter &s)
{
    if (!s.ok)
        return;
    if (s.live)
        *(uint4 *)((char *)(s.is_v ? p.v : p.k) + s.dst) = s.v;
    const int es = p.is_bf16 ? 2 : 4;
    for (int x = threadIdx.x + (p.kn_vec ? blockDim.x : 0); x < 2 * s.mine * s.per_row; x += blockDim.x) {
        const int is_v = x >= s.mine * s.per_row;
        const int y = is_v ? x - s.mine * s.per_row : x;
        const int i = part + (y / s.per_row) * parts, c = y % s.per_row;
        const int64_t src = is_v ? (int64_t)b * p.vn_sb + (int64_t)i * p.vn_st + (int64_t)g * p.vn_sh
                                 : (int64_t)b * p.kn_sb + (int64_t)i * p.kn_st + (int64_t)g * p.kn_sh;
        const int64_t dst = is_v ? ta_cache_offset(p, b, g, s.L + i, p.v_sp, p.v_sh, p.v_ss)
                                 : ta_cache_offset(p, b, g, s.L + i, p.k_sp, p.k_sh, p.k_ss);
        const char *sp = (const char *)(is_v ? p.vn : p.kn) + src * es;
        char *dp = (char *)(is_v ? p.v : p.k) + dst * es;
        if (p.kn_vec)
            *(uint4 *)(dp + 16 * c) = *(const uint4 *)(sp + 16 * c);
        else if (p.is_bf16)
            *(uint16_t *)(dp + 2 * c) = *(const uint16_t *)(sp + 2 * c);
        else
            *(uint32_t *)(dp + 4 * c) = *(const uint32_t *)(sp + 4 * c);
    }
}

// Launchers implemented next to their kernels.
hipError_t ta_launch_generic(const TAParams &p, hipStream_t stream);
hipError_t ta_launch_mfma(const TAParams &p, hipStream_t stream);
hipError_t ta_launch_merge(const TAParams &p, hipStream_t stream);
int ta_merge_rows(const TAParams &p);            // output rows one workgroup of the merge pass handles
struct TAAppend {
    const void *k_new, *v_new;         // [B, T, Hkv, D]
    void *k, *v;                       // caches
    const int32_t *page_table, *seq_lens;
    int64_t kn_sb, kn_st, kn_sh, vn_sb, vn_st, vn_sh;
    int64_t k_sp, k_sh, k_ss, v_sp, v_sh, v_ss, pt_sb, sl_s;
    int32_t B, T, Hkv, D, ps, capacity, elem_bytes;
    int32_t *status;
};
hipError_t ta_launch_append(const TAAppend &a, hipStream_t stream);
struct TACompact {
    void *k, *v;                       // caches
    const int32_t *page_table, *seq_lens, *accepted, *n_accepted;
    int32_t *seq_lens_out;             // or nullptr
    int64_t k_sp, k_sh, k_ss, v_sp, v_sh, v_ss, pt_sb, sl_s, acc_sb, na_s, slo_s;
    int32_t B, T, A, Hkv, D, ps, capacity, elem_bytes;
    int32_t *status;
};
hipError_t ta_launch_compact(const TACompact &c, hipStream_t stream);
hipError_t ta_launch_encode(const int32_t *parent, int64_t par_sb, int B, int T, unsigned long long *masks,
                            int32_t *status, hipStream_t stream);
