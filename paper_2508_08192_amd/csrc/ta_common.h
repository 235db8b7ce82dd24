// Shared declarations of the libtreeattn device code: kernel parameters and the device-side work
// schedule.  Everything here is specific to gfx950 (64-wide wavefronts).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ta_params.h"

// A data-dependent problem of the call: the bit goes into the device's sticky status word and into the caller's own
// word, if it gave one (ta_opts.status).  One thread of a workgroup calls this.
__device__ __forceinline__ void ta_raise(const TAParams &p, int bits)
{
    atomicOr(p.status, bits);
    if (p.status2)
        atomicOr(p.status2, bits);
}

// ---------------------------------------------------------------------------------------------
// Work schedule.  The KV pass walks, for every (request b, KV head g), a list of tiles:
// ceil(L_b / TA_TILE) prefix tiles followed by one tile holding the T tree tokens.  A malformed
// request owns a single tile (it only poisons its outputs).  All tile lists are laid end to end,
// (b major, g minor), and workgroup w takes a contiguous share of them (ta_wg_range).  A share
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
// padding.  Workgroup w takes a contiguous range of units (ta_wg_range).  The padding stands for the fixed cost of starting
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

// Units [t, t_end) of workgroup w.  The line is cut evenly, at floor(k * total / n_act), among the n_act workgroups
// that have work: all of them when that gives each at least TA_EVEN_CUT_FROM units (and the smallest share), else
// as many as whole shares of ceil(total / n_wg) units (at least min_q) fill, so that a small batch is not cut into
// more partial results than it needs.  Whole shares alone would drift against lists of equal length whenever a list
// is not a whole number of shares (128 lists of 265 units over 256 workgroups: shares of 133, so that workgroup 2j-1
// ends j tiles inside list j and almost every workgroup enters a second list for a few tiles, at the full fixed cost
// of an item); cut evenly, every second boundary falls on a list's edge.
#define TA_EVEN_CUT_FROM 8
__device__ __forceinline__ void ta_wg_range(const TAParams &p, int total, int w, int &t, int &t_end)
{
    const int share = ta_share(p, total);
    const int floor_share = p.min_q > TA_EVEN_CUT_FROM ? p.min_q : TA_EVEN_CUT_FROM;
    const int n_act = (int64_t)p.n_wg * floor_share <= total ? p.n_wg : (total + share - 1) / share;
    // floor(k * total / n_act) = k * q + floor(k * r / n_act) with total = q * n_act + r: 32-bit divisions (k * r stays
    // below n_act squared) instead of two 64-bit ones, which cost every workgroup most of a microsecond at its start
    if (n_act <= 0xffff) {
        const unsigned n = n_act > 0 ? (unsigned)n_act : 1u, q = (unsigned)total / n, r = (unsigned)total - q * n;
        t = w >= n_act ? total : (int)((unsigned)w * q + (unsigned)w * r / n);
        t_end = w + 1 >= n_act ? total : (int)((unsigned)(w + 1) * q + (unsigned)(w + 1) * r / n);
    } else {
        t = w >= n_act ? total : (int)((int64_t)w * total / n_act);
        t_end = w + 1 >= n_act ? total : (int)((int64_t)(w + 1) * total / n_act);
    }
}

// Request whose tile lists contain global tile t (0 <= t < Hkv * cum[B]): the number of requests whose lists end at
// or before t (cum does not decrease), counted 64 requests at a time by the lanes of each wave -- one LDS read and a
// ballot instead of a binary search's chain of dependent reads.  Every lane of the wave calls this together.
__device__ __forceinline__ int ta_find_request(const TAParams &p, const int *cum, int t)
{
    int x = threadIdx.x;
    asm volatile("" : "+v"(x));           // derived here: a caller short of registers must not keep the lane id alive
    const int lane = x & (TA_WAVE - 1);
    int b = 0;
    for (int base = 0; base < p.B; base += TA_WAVE) {
        const int idx = base + lane;
        const bool before = idx < p.B && (int64_t)p.Hkv * cum[idx + 1] <= t;
        const int n = __popcll(__ballot(before));
        b += n;
        if (n < TA_WAVE)
            break;
    }
    return b;
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

// Partial outputs.  The matrix-core kernels keep them as 16-bit fixed point, one fp32 scale per row (value = scale *
// int16, scale = largest magnitude of the row / 32767): every byte written here costs the KV pass several bytes of
// its read stream (halving the partials took 4.5 % off the KV pass of batches with many short lists), the error is at
// most 2^-16 of the row's largest value (fp16 would give 2^-11 of each value, too coarse beside the final rounding to
// bf16 when outputs reach 2 and more), and there is no range to overflow.  A row with a NaN gets a NaN scale.
// The scalar kernel, whose inputs may be fp32, keeps fp32 partials.
typedef short ta_s4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ char *ta_part_row(const TAParams &p, int64_t wrow)      // first byte of partial row wrow
{
    return (char *)p.ws_o + wrow * (int64_t)p.D * (p.part_q15 ? 2 : 4);
}

__device__ __forceinline__ float ta_part_get(const TAParams &p, int64_t wrow, int d)
{
    return p.part_q15 ? p.ws_lse[2 * wrow + 1] * (float)((const short *)p.ws_o)[wrow * p.D + d] : p.ws_o[wrow * p.D + d];
}

// Scale of a row whose largest magnitude is amax (NaN if the row holds one), and the factor that maps its values to
// int16.  An all-zero row keeps scale 0.
__device__ __forceinline__ void ta_q15_scale(float amax, bool has_nan, float &scale, float &to_q)
{
    scale = has_nan ? __uint_as_float(0x7fc00000u) : amax * (1.f / 32767.f);
    to_q = amax > 0.f ? 32767.f / amax : 0.f;
}

__device__ __forceinline__ uint32_t ta_q15_pack(float a, float b, float to_q)      // two values -> two int16
{
    const int qa = __float2int_rn(a * to_q), qb = __float2int_rn(b * to_q);
    return ((uint32_t)qa & 0xffffu) | ((uint32_t)qb << 16);
}

// A page id comes from the caller's page table: one outside the cache must never become an address.
__device__ __forceinline__ bool ta_page_ok(const TAParams &p, int page)
{
    return (uint32_t)page < (uint32_t)p.n_pages;
}

// Element offset of logical position pos of request b, KV head g in a cache with strides (sp, sh, ss); -1 if the
// page table names a page the cache does not have.
__device__ __forceinline__ int64_t ta_cache_offset(const TAParams &p, int b, int g, int pos,
                                                   int64_t sp, int64_t sh, int64_t ss)
{
    int64_t page, slot;
    if (p.page_table) {
        int pi = p.ps_shift >= 0 ? (pos >> p.ps_shift) : (pos / p.ps);
        slot = p.ps_shift >= 0 ? (pos & (p.ps - 1)) : (pos - pi * p.ps);
        const int id = p.page_table[(int64_t)b * p.pt_sb + pi];
        if (!ta_page_ok(p, id))
            return -1;
        page = id;
    } else {
        page = b;
        slot = pos;
    }
    return page * sp + (int64_t)g * sh + slot * ss;
}

// Are the page-table entries that hold logical positions pos_lo .. pos_hi of request b all pages of the cache?
// Every thread of the workgroup calls this; *flag is one int of shared memory; two barriers inside.
__device__ __forceinline__ bool ta_pages_ok(const TAParams &p, int b, int pos_lo, int pos_hi, int *flag)
{
    if (!p.page_table || pos_hi < pos_lo)
        return true;
    if (threadIdx.x == 0)
        *flag = 0;
    __syncthreads();
    const int first = p.ps_shift >= 0 ? (pos_lo >> p.ps_shift) : (pos_lo / p.ps);
    const int last = p.ps_shift >= 0 ? (pos_hi >> p.ps_shift) : (pos_hi / p.ps);
    for (int k = first + (int)threadIdx.x; k <= last; k += (int)blockDim.x)
        if (!ta_page_ok(p, p.page_table[(int64_t)b * p.pt_sb + k]))
            atomicOr(flag, 1);
    __syncthreads();
    return *flag == 0;
}

// First and last logical position whose pages the item (tiles j0 .. j1-1 of a list with n_b tiles, first prefix tile
// tile0, window start S, length L) reads.
__device__ __forceinline__ void ta_item_positions(const TAParams &p, int j0, int j1, int n_b, int tile0, int L, int S,
                                                  int &pos_lo, int &pos_hi)
{
    const int first = (tile0 + j0) * TA_TILE;
    pos_lo = j0 == n_b - 1 ? L : (first > S ? first : S);
    const int end = (tile0 + j1) * TA_TILE;
    pos_hi = j1 == n_b ? L + p.T - 1 : (end < L ? end : L) - 1;
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

// A word of masks given by the caller is taken as it is, except that a node always lies on its own path: a word
// without its own bit (what tree_attn_encode writes for a malformed tree) marks the request as malformed.
__device__ __forceinline__ bool ta_given_mask_ok(unsigned long long m, int node)
{
    return ((m >> node) & 1ull) != 0;
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
        const int64_t off = s.is_v ? ta_cache_offset(p, b, g, s.L + s.i, p.v_sp, p.v_sh, p.v_ss)
                                   : ta_cache_offset(p, b, g, s.L + s.i, p.k_sp, p.k_sh, p.k_ss);
        s.dst = off * es + 16 * s.c;
        s.live = off >= 0;             // a page the cache does not have is not written (the KV pass reports it)
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
        if (dst < 0)
            continue;
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
// (`dev`: index of the current device, which the caller already knows)
hipError_t ta_launch_generic(const TAParams &p, hipStream_t stream, int dev);
hipError_t ta_launch_mfma(const TAParams &p, hipStream_t stream, int dev);
hipError_t ta_launch_merge(const TAParams &p, hipStream_t stream);
hipError_t ta_launch_append(const TAAppend &a, hipStream_t stream);
hipError_t ta_launch_compact(const TACompact &c, hipStream_t stream, int dev);
hipError_t ta_launch_stream_read(const void *buf, size_t bytes, void *sink, int num_cus, hipStream_t stream);
hipError_t ta_launch_mfma_probe(int iters, void *sink, int num_cus, hipStream_t stream);
hipError_t ta_launch_encode(const int32_t *parent, int64_t par_sb, int B, int T, unsigned long long *masks,
                            int32_t *status, hipStream_t stream);
