// Matrix-core KV pass of libtreeattn for gfx950: bf16 inputs, head_dim 128, fp32 accumulation.
//
// One workgroup keeps up to 256 query rows of one (request, KV head) -- the T tree nodes times the
// G query heads that share the KV head (GQA packing) -- and streams its share of that head's tile
// list through LDS: prefix tiles of 64 cached tokens (mask-free; section 3.1, prefix attention) and,
// last in every list, the tile of the T tree tokens, whose scores are masked in registers with the
// row's 64-bit ancestor mask (section 3.1, suffix attention).  Prefix and suffix partials that meet in
// one workgroup are merged on the fly by the running softmax, which is the same log-sum-exp merge the
// merge pass applies across workgroups.
//
// Two kernels share this scheme: ta_mfma_sp_kernel (the one that normally runs: per-tile instruction streams
// written in assembly, tiles loaded straight into LDS) and ta_mfma_kv_kernel (plain, compiler-scheduled,
// register-staged tiles; the fallback).
//
// Each wave owns a block of 32 rows.  Both contractions are issued in transposed form so that
// a lane owns one query row per block throughout (row statistics never leave the lane):
//     S^T[token, row] = K[token, :] . Q[row, :]      A = K fragment (LDS),  B = Q fragment (registers)
//     O^T[d, row]    += V^T[d, token] . P^T[token, row]   A = V^T fragment (LDS), B = P (registers)
// with v_mfma_f32_32x32x16_bf16.  The accumulator layout of S^T (lane = row, registers = tokens) is,
// up to a fixed permutation of the 16 contraction slots, the B-operand layout the second product
// needs; V is stored in LDS with the same slot permutation, token-minor, so its A fragments are
// single 16-byte reads.
#include <stdlib.h>

#include "ta_common.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define MF_D 128
#define MF_TILE_BYTES (TA_TILE * MF_D * 2)       // one K or V tile in LDS: 16 KB
#define MF_STAGES 2
#define MF_UNITS 512                             // staging units per tile: 256 for K, 256 for V

static_assert(TA_TILE == 64, "the fragment maps below assume 64-token tiles");

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v)
{
    return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    f32x2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

// Staging unit u of a tile: 4 consecutive tokens (quad) x 8 consecutive head-dim elements (chunk),
// i.e. four 16-byte global loads.  Units 0..255 carry K, 256..511 carry V.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
struct Unit {
    uint4 r[4];
};

// Loads one unit.  tbase already points at (KV head, 8-element chunk) of the cache; pos0 = logical
// position of the unit's first token; of its four tokens those with index n_skip .. n_valid-1 exist for
// this call (tokens before a window start and past the end are staged as zeros and never loaded, so stale
// cache contents -- NaN included -- never reach a product and released pages are never touched).  Page and slot
// strides fit 32 bits (checked on the host), which keeps the address arithmetic to a few instructions.
__device__ __forceinline__ void load_unit(const TAParams &p, Unit &u, const uint16_t *tbase, uint32_t sp, uint32_t ss,
                                          int b, int pos0, int n_valid, bool contiguous, int n_skip = 0)
{
    const uint16_t *ptr[4];
    if (n_valid > n_skip) {
        if (contiguous) {
            const uint16_t *p0 = tbase + (uint64_t)(uint32_t)b * sp + (uint64_t)(uint32_t)pos0 * ss;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                ptr[k] = p0 + (uint32_t)k * ss;
        } else if (p.ps_shift >= 2 && (pos0 & 3) == 0) {
            // (one page holds all four tokens, and at least one of them exists: the page id is a checked one)
            const uint32_t page = (uint32_t)p.page_table[(int64_t)b * p.pt_sb + (pos0 >> p.ps_shift)];
            const uint16_t *p0 = tbase + (uint64_t)page * sp + (uint32_t)(pos0 & (p.ps - 1)) * ss;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                ptr[k] = p0 + (uint32_t)k * ss;
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int pos = pos0 + (k < n_valid && k >= n_skip ? k : n_skip);
                const uint32_t page = (uint32_t)p.page_table[(int64_t)b * p.pt_sb + (pos >> p.ps_shift)];
                ptr[k] = tbase + (uint64_t)page * sp + (uint32_t)(pos & (p.ps - 1)) * ss;
            }
        }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        if (k < n_valid && k >= n_skip)
            // keys and values are read once: the non-temporal hint keeps them from displacing the partial results
            u.r[k] = __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4 *)ptr[k]));
        else
            u.r[k] = make_uint4(0, 0, 0, 0);
    }
}

// K tile in LDS: [token 0..63][DH / 8 chunks of 16 B], chunk index XOR-swizzled with the token's low bits so that
// the 16-byte fragment reads of different tokens at one chunk hit distinct banks.
template <int DH>
__device__ __forceinline__ void store_k_unit(char *ktile, const Unit &u, int quad, int chunk)
{
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int row = quad * 4 + k;
        *(uint4 *)(ktile + row * (DH * 2) + ((chunk ^ (row & (DH / 8 - 1))) << 4)) = u.r[k];
    }
}

// V tile in LDS, token-minor: [kb 0..3][half 0..1][DH head-dim slots][8 tokens] of bf16, where the 8
// tokens of (kb, half) are 16kb + 4half + {0,1,2,3} and 16kb + 8 + 4half + {0,1,2,3}: exactly the
// contraction slots a lane of that half feeds to the second MFMA.  The head-dim slot of column d is
// d ^ ((d >> 4) & 7), which spreads the eight 8-byte writes of a staging thread over the banks.
template <int DH>
__device__ __forceinline__ void store_v_unit(char *vtile, const Unit &u, int quad, int chunk)
{
    const int kb = quad >> 2, half = quad & 1, sec = (quad >> 1) & 1;
    char *base = vtile + ((kb * 2 + half) * DH) * 16 + sec * 8;
    const uint32_t *r0 = (const uint32_t *)&u.r[0], *r1 = (const uint32_t *)&u.r[1];
    const uint32_t *r2 = (const uint32_t *)&u.r[2], *r3 = (const uint32_t *)&u.r[3];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        // dword w of every token holds columns 8*chunk + 2w (low half) and 2w+1 (high half)
        uint2 lo, hi;
        lo.x = (r0[w] & 0xffffu) | (r1[w] << 16);
        lo.y = (r2[w] & 0xffffu) | (r3[w] << 16);
        hi.x = (r0[w] >> 16) | (r1[w] & 0xffff0000u);
        hi.y = (r2[w] >> 16) | (r3[w] & 0xffff0000u);
        const int d_lo = chunk * 8 + 2 * w, d_hi = d_lo + 1;
        *(uint2 *)(base + ((d_lo ^ ((d_lo >> 4) & 7)) << 4)) = lo;
        *(uint2 *)(base + ((d_hi ^ ((d_hi >> 4) & 7)) << 4)) = hi;
    }
}


__device__ __forceinline__ void lds_barrier()
{
    // LDS traffic of this wave must have landed before the others proceed; global loads stay in flight.
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ float max3(float a, float b, float c)
{
    // one instruction; the generic fmaxf would first quiet every operand
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

__device__ __forceinline__ float half_swap_max(float x)
{
    // max over the two lanes that share a query row (lane and lane ^ 32)
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Scores of tokens that do not exist for this lane's row become -inf.  Bit k of vm covers the register
// with token offset k = 32tb + 8(i/4) + (i%4) (the lane's half offset 4hf is already shifted out).
__device__ __forceinline__ void mask_scores(f32x16 (&acc_s)[2], unsigned long long vm)
{
    const uint32_t lo = (uint32_t)vm, hi = (uint32_t)(vm >> 32);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int bit = 8 * (i / 4) + (i % 4);
        if (!((lo >> bit) & 1u))
            acc_s[0][i] = -INFINITY;
        if (!((hi >> bit) & 1u))
            acc_s[1][i] = -INFINITY;
    }
}

// Running-softmax bookkeeping of one 64-token tile for one 32-row block: s holds the lane's 32 raw
// (unscaled) scores, c = softmax scale * log2(e).  Produces P as four bf16 B-operands and updates the
// running max (raw units), the lane's shares of the running sums -- l of the probabilities (for the log-sum-exp)
// and l2 of their bf16 roundings, the weights the second product really applies (O is normalised by l2, which makes
// the output an exact weighted mean of V rows) -- and (rarely) rescales O.
template <int NDB>
__device__ __forceinline__ void softmax_tile(const f32x16 (&s)[2], float c, float &m_run, float &l_run, float &l2_run,
                                             f32x16 (&acc_o)[NDB], uint4 (&pb)[4])
{
    float tmax = fmaxf(s[0][0], s[1][0]);
#pragma unroll
    for (int i = 1; i < 16; ++i)
        tmax = max3(tmax, s[0][i], s[1][i]);
    tmax = half_swap_max(tmax);
    const float m_new = fmaxf(m_run, tmax);
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
    const float neg_mc = -m_new * c;
    m_run = m_new;
    float psum = 0.f, psum2 = 0.f;
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
        float e[8];
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            e[jj] = __builtin_amdgcn_exp2f(fmaf(s[kb >> 1][8 * (kb & 1) + jj], c, neg_mc));
            psum += e[jj];
        }
        pb[kb].x = pack_bf16(e[0], e[1]);
        pb[kb].y = pack_bf16(e[2], e[3]);
        pb[kb].z = pack_bf16(e[4], e[5]);
        pb[kb].w = pack_bf16(e[6], e[7]);
        const uint32_t w4[4] = {pb[kb].x, pb[kb].y, pb[kb].z, pb[kb].w};
#pragma unroll
        for (int k = 0; k < 4; ++k)
            psum2 += __uint_as_float(w4[k] << 16) + __uint_as_float(w4[k] & 0xffff0000u);
    }
    l_run = l_run * alpha + psum;
    l2_run = l2_run * alpha + psum2;
    if (__any(alpha != 1.0f)) {
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                acc_o[db][i] *= alpha;
    }
}

// NCW compute waves of RB 32-row blocks each (rows per workgroup = 32*RB*NCW), NT threads in all
// (NT/64 - NCW waves only help with staging).  DH: head dimension, 64 or 128.
template <int NCW, int RB, int NT, int DH>
__global__ __launch_bounds__(NT) void ta_mfma_kv_kernel(TAParams p)
{
    constexpr int CH = DH / 8;                    // 16-byte chunks of a row
    constexpr int UNITS_K = 16 * CH;              // staging units of the K tile (as many again for V)
    constexpr int UPT = (2 * UNITS_K + NT - 1) / NT;   // staging units per thread
    constexpr int TILE_BYTES = TA_TILE * DH * 2;
    constexpr int NKK = DH / 16, NDB = DH / 32;   // contraction steps of the first product, head-dim blocks of the second
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char *tiles = smem;                                                   // [MF_STAGES][K tile | V tile]
    unsigned long long *masks = (unsigned long long *)(smem + MF_STAGES * 2 * TILE_BYTES);   // [64]
    int *flag = (int *)(masks + TA_MAX_TREE);
    int *par_s = flag + 4;                                                // [TA_MAX_TREE]
    int *cum = par_s + TA_MAX_TREE;                                       // [B + 1]

    ta_build_schedule(p, cum);
    const int total = __builtin_amdgcn_readfirstlane(p.Hkv * cum[p.B]);
    const int w = blockIdx.x, rg = blockIdx.y;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);           // wave-uniform, lives in SGPRs
    const int r32 = lane & 31, hf = lane >> 5;
    const bool compute_wave = wave < NCW;
    int t, t_end;
    ta_wg_range(p, total, w, t, t_end);
    t = __builtin_amdgcn_readfirstlane(t);
    t_end = __builtin_amdgcn_readfirstlane(t_end);
    const int rows_here = min(p.rows_grp, p.rows - rg * p.rows_grp);
    const float c = p.scale_log2e;
    // LDS byte offsets of this lane's fragments inside a tile
    const int sw = r32 & (CH - 1);
    const int krow_off = r32 * (DH * 2);                                  // + tb*32 rows + (((2kk+hf)^sw) << 4)
    int vcol_off[NDB];                                                    // + kb * 2 * DH * 16
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
        const int d = db * 32 + r32;
        vcol_off[db] = (hf * DH + (d ^ ((d >> 4) & 7))) << 4;
    }

    while (t < t_end) {
        // the schedule comes out of LDS, which the compiler treats as lane-varying: pin it to SGPRs
        const int b = __builtin_amdgcn_readfirstlane(ta_find_request(p, cum, t));
        const int n_u = __builtin_amdgcn_readfirstlane(cum[b + 1] - cum[b]);   // schedule units of one list
        const int cum_b = __builtin_amdgcn_readfirstlane(cum[b]);
        const int g = (t - p.Hkv * cum_b) / n_u;
        const int seg_start = p.Hkv * cum_b + g * n_u;                         // unit of the list's tile 0
        const int n_b = n_u - p.pad;
        const int j0 = t - seg_start;
        const int j1 = min(n_b, t_end - seg_start);
        if (j1 <= j0) {
            t = seg_start + n_u;                              // t lies in the list's trailing padding
            continue;
        }
        const int slot = w + b * p.Hkv + g;
        ta_note_owner(p, b, g, w, j0, j1, n_b);
        const int L = __builtin_amdgcn_readfirstlane(p.seq_lens[(int64_t)b * p.sl_s]);
        const int S = __builtin_amdgcn_readfirstlane(ta_kv_start(p, b));
        bool poison = !ta_request_ok(p, L, S);
        const int tile0 = poison ? 0 : S / TA_TILE;                // absolute index of the list's first prefix tile
        if (poison && tid == 0)
            ta_raise(p, TA_STATUS_BAD_SEQLEN);
        const bool has_tree_tile = (j1 == n_b);
        if (!poison) {
            int pos_lo, pos_hi;
            ta_item_positions(p, j0, j1, n_b, tile0, L, S, pos_lo, pos_hi);
            if (!ta_pages_ok(p, b, pos_lo, pos_hi, flag)) {
                poison = true;
                if (tid == 0)
                    ta_raise(p, TA_STATUS_BAD_PAGE);
            }
        }
        if (has_tree_tile && !poison && p.masks_in) {
            if (tid == 0)
                *flag = 0;
            __syncthreads();
            if ((int)threadIdx.x < p.T) {
                const unsigned long long m = ta_given_mask(p, b, threadIdx.x);
                masks[threadIdx.x] = m;
                if (!ta_given_mask_ok(m, threadIdx.x))
                    atomicOr(flag, 1);
            }
            __syncthreads();
            if (*flag != 0) {
                poison = true;
                if (tid == 0)
                    ta_raise(p, TA_STATUS_BAD_PARENT);
            }
        } else if (has_tree_tile && !poison) {
            if (!ta_encode_tree(p.parent + (int64_t)b * p.par_sb, p.T, masks, flag, par_s)) {
                poison = true;
                if (tid == 0)
                    ta_raise(p, TA_STATUS_BAD_PARENT);
            }
        }

        if (poison) {
            if (compute_wave) {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    const int row = (wave * RB + rb) * 32 + r32;
                    if (row < rows_here) {
                        const int64_t wrow = ta_ws_row(p, slot, rg, row);
                        for (int o = hf * DH; o < (hf + 1) * DH; o += 16)          // DH 16-bit values per row
                            *(float4 *)(ta_part_row(p, wrow) + o) = make_float4(0.f, 0.f, 0.f, 0.f);
                        if (hf == 0)
                            p.ws_lse[2 * wrow] = __uint_as_float(0x7fc00000u);
                    }
                }
            }
            __syncthreads();
            t = seg_start + (j1 == n_b ? n_u : j1);
            continue;
        }

        // Q fragments (B operand of the first product): row r32 of each block, head-dim 16kk + 8hf .. +8.
        uint4 qf[RB][NKK];
        unsigned long long tree_mask[RB];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int row = (wave * RB + rb) * 32 + r32;
            const int R = rg * p.rows_grp + row;
            const bool row_ok = compute_wave && row < rows_here;
            const int node = row_ok ? R / p.G : 0;
            if (row_ok) {
                const uint16_t *qp = (const uint16_t *)p.q + (int64_t)b * p.q_sb + (int64_t)node * p.q_st +
                                     (int64_t)(g * p.G + R % p.G) * p.q_sh + hf * 8;
#pragma unroll
                for (int kk = 0; kk < NKK; ++kk)
                    qf[rb][kk] = *(const uint4 *)(qp + kk * 16);
            } else {
#pragma unroll
                for (int kk = 0; kk < NKK; ++kk)
                    qf[rb][kk] = make_uint4(0, 0, 0, 0);
            }
            // Rows of padding keep an all-ones mask so that their (discarded) softmax stays finite.
            tree_mask[rb] = (has_tree_tile && row_ok) ? masks[p.q_off + node] : ~0ull;
        }

        f32x16 acc_o[RB][NDB];
        float m_run[RB], l_run[RB], l2_run[RB];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            m_run[rb] = -INFINITY;
            l_run[rb] = 0.f;
            l2_run[rb] = 0.f;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    acc_o[rb][db][i] = 0.f;
        }

        // ---- staging: which units this thread carries, and loading tile j into registers
        Unit stage[UPT];
        auto load_tile = [&](int j) {
            const bool tree_tile = (j == n_b - 1);
            const int tile_pos0 = tree_tile ? L : (tile0 + j) * TA_TILE;
            const int limit = tree_tile ? L + p.T : L;
#pragma unroll
            for (int s = 0; s < UPT; ++s) {
                const int u = tid + s * NT;
                if (u >= 2 * UNITS_K)
                    continue;
                const int uu = u < UNITS_K ? u : u - UNITS_K, quad = uu / CH, chunk = uu % CH;
                const int pos0 = tile_pos0 + quad * 4;
                const int n_valid = max(0, min(4, limit - pos0));
                const int n_skip = tree_tile ? 0 : max(0, min(4, S - pos0));      // tokens before the window start
                if (tree_tile && p.kn) {
                    // write-back folded into the call: the tree tokens sit in the dense tensors of this step, which
                    // are addressed like a contiguous cache -- request stride for the page, token stride for the slot
                    if (u < UNITS_K)
                        load_unit(p, stage[s], (const uint16_t *)p.kn + (int64_t)g * p.kn_sh + chunk * 8,
                                  (uint32_t)p.kn_sb, (uint32_t)p.kn_st, b, pos0 - L, n_valid, true);
                    else
                        load_unit(p, stage[s], (const uint16_t *)p.vn + (int64_t)g * p.vn_sh + chunk * 8,
                                  (uint32_t)p.vn_sb, (uint32_t)p.vn_st, b, pos0 - L, n_valid, true);
                } else if (u < UNITS_K) {
                    load_unit(p, stage[s], (const uint16_t *)p.k + (int64_t)g * p.k_sh + chunk * 8, (uint32_t)p.k_sp,
                              (uint32_t)p.k_ss, b, pos0, n_valid, !p.page_table, n_skip);
                } else {
                    load_unit(p, stage[s], (const uint16_t *)p.v + (int64_t)g * p.v_sh + chunk * 8, (uint32_t)p.v_sp,
                              (uint32_t)p.v_ss, b, pos0, n_valid, !p.page_table, n_skip);
                }
            }
        };
        auto store_tile = [&](int buf) {
            char *kt = tiles + buf * 2 * TILE_BYTES, *vt = kt + TILE_BYTES;
#pragma unroll
            for (int s = 0; s < UPT; ++s) {
                const int u = tid + s * NT;
                if (u >= 2 * UNITS_K)
                    continue;
                const int uu = u < UNITS_K ? u : u - UNITS_K, quad = uu / CH, chunk = uu % CH;
                if (u < UNITS_K)
                    store_k_unit<DH>(kt, stage[s], quad, chunk);
                else
                    store_v_unit<DH>(vt, stage[s], quad, chunk);
            }
        };

        load_tile(j0);
        store_tile(0);
        lds_barrier();

        for (int j = j0; j < j1; ++j) {
            const int buf = (j - j0) & 1;
            if (j + 1 < j1)
                load_tile(j + 1);                              // in flight while this tile is computed

            if (compute_wave) {
                const char *kt = tiles + buf * 2 * TILE_BYTES, *vt = kt + TILE_BYTES;
                constexpr int TB_OFF = 32 * DH * 2;            // second block of 32 tokens in the K tile
                // ---- S^T = K . Q^T for the two 32-token blocks of the tile, each K fragment feeding RB blocks
                f32x16 acc_s[RB][2];
                const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                uint4 kf[3][2];
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    const int co = ((2 * kk + hf) ^ sw) << 4;
                    kf[kk][0] = *(const uint4 *)(kt + krow_off + co);
                    kf[kk][1] = *(const uint4 *)(kt + TB_OFF + krow_off + co);
                }
#pragma unroll
                for (int kk = 0; kk < NKK; ++kk) {
                    if (kk + 2 < NKK) {
                        const int co = ((2 * (kk + 2) + hf) ^ sw) << 4;
                        kf[(kk + 2) % 3][0] = *(const uint4 *)(kt + krow_off + co);
                        kf[(kk + 2) % 3][1] = *(const uint4 *)(kt + TB_OFF + krow_off + co);
                    }
#pragma unroll
                    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                        for (int rb = 0; rb < RB; ++rb)
                            acc_s[rb][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                as_bf16x8(kf[kk % 3][tb]), as_bf16x8(qf[rb][kk]), kk == 0 ? zero16 : acc_s[rb][tb],
                                0, 0, 0);
                }
                // ---- which of this lane's 32 tokens count, then the running softmax per row block
                const bool tree_tile = (j == n_b - 1);
                const int pos0 = (tile0 + j) * TA_TILE;            // a prefix tile holds positions pos0 .. pos0+63,
                const bool partial = L - pos0 < TA_TILE || pos0 < S;   // of which those in [S, L) count
                uint4 pb[RB][4];
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    if (tree_tile || partial)
                        mask_scores(acc_s[rb], (tree_tile ? tree_mask[rb] : ta_prefix_tile_mask(pos0, L, S)) >> (4 * hf));
                    softmax_tile<NDB>(acc_s[rb], c, m_run[rb], l_run[rb], l2_run[rb], acc_o[rb], pb[rb]);
                }
                // ---- O^T += V^T . P^T, each V fragment feeding RB blocks
                constexpr int KB_OFF = 2 * DH * 16;            // token slab kb of the V tile; step s = kb * NDB + db
                uint4 vf[4];
#pragma unroll
                for (int s = 0; s < 3; ++s)
                    vf[s] = *(const uint4 *)(vt + (s / NDB) * KB_OFF + vcol_off[s % NDB]);
#pragma unroll
                for (int s = 0; s < 4 * NDB; ++s) {
                    if (s + 3 < 4 * NDB)
                        vf[(s + 3) & 3] = *(const uint4 *)(vt + ((s + 3) / NDB) * KB_OFF + vcol_off[(s + 3) % NDB]);
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
                        acc_o[rb][s % NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            as_bf16x8(vf[s & 3]), as_bf16x8(pb[rb][s / NDB]), acc_o[rb][s % NDB], 0, 0, 0);
                }
            }

            if (j + 1 < j1)
                store_tile(buf ^ 1);
            lds_barrier();
        }

        // ---- partial result of this (workgroup, list) overlap: normalised O and base-2 log-sum-exp
        if (compute_wave) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                const int row = (wave * RB + rb) * 32 + r32;
                if (row < rows_here) {
                    const int64_t wrow = ta_ws_row(p, slot, rg, row);
                    const float l_tot = l_run[rb] + __shfl_xor(l_run[rb], 32, TA_WAVE);
                    const float inv = 1.f / (l2_run[rb] + __shfl_xor(l2_run[rb], 32, TA_WAVE));
                    // 16-bit fixed point with the row's own scale: the two lanes of a row find its largest magnitude
                    float amax = 0.f;
                    bool has_nan = false;
#pragma unroll
                    for (int db = 0; db < NDB; ++db)
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            const float x = acc_o[rb][db][i] * inv;
                            amax = fmaxf(amax, fabsf(x));
                            has_nan |= x != x;
                        }
                    amax = fmaxf(amax, __shfl_xor(amax, 32, TA_WAVE));
                    has_nan |= __shfl_xor((int)has_nan, 32, TA_WAVE) != 0;
                    float scale, to_q;
                    ta_q15_scale(amax, has_nan, scale, to_q);
                    to_q *= inv;
#pragma unroll
                    for (int db = 0; db < NDB; ++db) {
#pragma unroll
                        for (int i4 = 0; i4 < 4; ++i4) {
                            uint2 o;
                            o.x = ta_q15_pack(acc_o[rb][db][4 * i4 + 0], acc_o[rb][db][4 * i4 + 1], to_q);
                            o.y = ta_q15_pack(acc_o[rb][db][4 * i4 + 2], acc_o[rb][db][4 * i4 + 3], to_q);
                            *(uint2 *)(ta_part_row(p, wrow) + 2 * (db * 32 + 8 * i4 + 4 * hf)) = o;
                        }
                    }
                    if (hf == 0)
                        *(float2 *)&p.ws_lse[2 * wrow] = make_float2(m_run[rb] * c + log2f(l_tot), scale);
                }
            }
        }
        __syncthreads();                                       // masks and tiles are reused by the next item
        t = seg_start + (j1 == n_b ? n_u : j1);
    }
}

#define PP_PAGES 2048                             // page ids cached in LDS per span of tiles
#define SP_OWN_FIRST 32                           // see issue_first in ta_mfma_sp_kernel

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// every lane moves 16 bytes from its own global address to LDS offset lds_wave_base + 16*lane
__device__ __forceinline__ void dma16(const void *gptr, uint32_t lds_wave_base)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt" ::"v"(gptr), "s"(lds_wave_base)
                 : "memory");          // M0 is not used by anything else in these kernels
}

template <int N>
__device__ __forceinline__ void vm_wait()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// ---------------------------------------------------------------------------------------------
// 256-row variant, software-pipelined inside every wave: 8 waves of 32 rows, two per SIMD.
//
// Block i of a wave is one instruction stream that interleaves the 16 MFMAs of O^T += V^T(i-1).P^T(i-1), the
// 16 MFMAs of S^T(i+1) = K(i+1).Q^T and the running softmax of S^T(i) (see gen_sp_block.py), so the wave feeds the
// matrix pipe and the vector ALU at once and needs no phase skew; one workgroup barrier per tile remains.
// K and V tiles travel global -> LDS without touching registers (global_load_lds_dwordx4), three blocks
// ahead of their first use, into a ring of 3 K tiles and a ring of 5 V tiles.  Both lie there as in the cache, one
// 256-byte row per token, with the 16-byte pieces of a row XOR-placed (K by token & 15, V in 32-byte blocks by
// token & 7) so that the fragment reads are free of bank conflicts; the V fragments of the second product, whose
// contraction runs over tokens, come out of the row-major tile through transposing LDS reads (see gen_sp_block.py).
//
//   start of block i : issue the loads of tile i+3        (K slot (i+3)%3: last read by S(i) in block i-1,
//                                                          V slot (i+3)%5: last read by PV(i-2) in block i-1)
//   block i          : PV(i-1) | S(i+1) | softmax(i)
//   tail i           : rescale O if the softmax reference moved; mask S(i+1) if tile i+1 is ragged or the
//                      tree tile; wait for this wave's part of tile i+2; barrier
// ---------------------------------------------------------------------------------------------
#define SP_RK 3
#define SP_RV 5
#define SP_V_OFF (SP_RK * MF_TILE_BYTES)
#define SP_AUX_OFF ((SP_RK + SP_RV) * MF_TILE_BYTES)

typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));

#include "ta_sp_block.inc"

// every lane moves 16 bytes from base + off to LDS offset lds_wave_base + 16*lane (base is wave-uniform)
__device__ __forceinline__ void dma16s(const void *base, uint32_t off, uint32_t lds_wave_base)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt" ::"v"(off), "s"(base),
                 "s"(lds_wave_base)
                 : "memory");
}

template <bool V>
struct SpTag {
    static constexpr bool value = V;
};

// amdgpu_num_vgpr(16): the register allocator stays in v0..v31; v32..v255 belong to the asm blocks (see gen_sp_block.py)
// NEW: the tree tokens' K/V come from the dense tensors of ta_opts.k_new / v_new (an instance of its own, so that the
// ordinary call carries none of that addressing).
template <bool NEW>
__global__ __launch_bounds__(512) __attribute__((amdgpu_num_vgpr(16))) void ta_mfma_sp_kernel(TAParams p)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    unsigned long long *masks = (unsigned long long *)(smem + SP_AUX_OFF);
    int *flag = (int *)(masks + TA_MAX_TREE);
    int *par_s = flag + 4;                                                // [TA_MAX_TREE]
    int *pcache = par_s + TA_MAX_TREE;                                    // [PP_PAGES] page ids of the current span
    int *cum = pcache + PP_PAGES;                                         // [B + 1] schedule, then [B] prefix lengths
    int *lens = cum + p.B + 1;
    int *starts = lens + p.B;                                             // [B] window starts
    const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) char *)smem);

    if (threadIdx.x == 0)
        flag[1] = 0;                   // set by an item that meets a bad page id or a bad given mask; see `bad` below
    ta_build_schedule(p, cum, lens, starts);
    const int total = __builtin_amdgcn_readfirstlane(p.Hkv * cum[p.B]);
    const int w = blockIdx.x, rg = blockIdx.y;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r32 = lane & 31, hf = lane >> 5;
    int t, t_end;
    {
        int t0, t1;
        ta_wg_range(p, total, w, t0, t1);
        t = __builtin_amdgcn_readfirstlane(t0);
        t_end = __builtin_amdgcn_readfirstlane(t1);
    }
    const int rows_here = min(p.rows_grp, p.rows - rg * p.rows_grp);
    const float c = p.scale_log2e;
    const bool paged = p.page_table != nullptr;
    const uint32_t ksp = (uint32_t)p.k_sp, kss = (uint32_t)p.k_ss, vsp = (uint32_t)p.v_sp, vss = (uint32_t)p.v_ss;
    // Lane constants of the blocks (LDS byte offsets), kept in their fixed registers:
    //   K fragment of step kk: row r32, 16-byte slot (2kk + hf) ^ (r32 & 15), i.e. base ^ 32kk inside the tile
    //   V fragment of head-dim block db (transposing read, groups of 16 lanes): the lane names the 8-byte piece
    //   p = lane & 3 of 32-byte block (2db + h16) ^ tk of token row tk = 4hf + k', with h16 = (lane >> 4) & 1 the
    //   half of the head-dim block the group serves and k' = (lane >> 2) & 3; i.e. (base ^ 64db) + 4096kb (+ 2048)
    {
        const int h16 = (lane >> 4) & 1, tk = 4 * hf + ((lane >> 2) & 3), pc = lane & 3;
        sp_set_bases(lds0 + SP_V_OFF + (uint32_t)(tk * 256 + ((h16 ^ tk) << 5) + pc * 8),
                     lds0 + (uint32_t)(r32 * 256 + ((hf ^ (r32 & 15)) << 4)));
    }
    // Cache-load role of a lane: tile rows drow and drow+4, 16-byte slot dslot; the source chunk is the slot
    // XOR-ed with the row's placement (K: row & 15; V: 2 * (row & 7)).
    // Only the byte offsets of the common case stay in registers; the rare paths derive their lane roles again
    // from the thread id (fresh_tid keeps the compiler from hoisting them into long-lived registers).
    auto fresh_tid = [&]() {
        int x = tid;
        asm volatile("" : "+v"(x));
        return x;
    };
    // (recomputed where needed rather than kept: a value that lives across the whole walk would be spilled, and a
    // reload from scratch memory waits for every cache load in flight)
    auto lane_offsets = [&](uint32_t &koff0, uint32_t &koff1, uint32_t &voff0, uint32_t &voff1, int wv) {
        const int ln = fresh_tid() & 63;
        // relative to the first of the wave's eight token rows (tile rows 8 wv .. 8 wv + 7): the wave's loads start
        // from that row's address, so that a tile may span several pages as long as these eight rows share one
        const int lrow = ln >> 4, drow = wv * 8 + lrow, dslot = ln & 15;
        koff0 = (uint32_t)(lrow * kss + (dslot ^ (drow & 15)) * 8) * 2u;
        koff1 = (uint32_t)((lrow + 4) * kss + (dslot ^ ((drow + 4) & 15)) * 8) * 2u;
        voff0 = (uint32_t)(lrow * vss + (dslot ^ (2 * (drow & 7))) * 8) * 2u;
        voff1 = (uint32_t)((lrow + 4) * vss + (dslot ^ (2 * ((drow + 4) & 7))) * 8) * 2u;
    };
    // a page (or the contiguous cache) holds the eight aligned token rows a wave loads of a tile, i.e. pages of eight
    // tokens and more; and lane offsets fit 32 bits
    const bool fast_geom = (!paged || p.ps_shift >= 3) && kss < (1u << 22) && vss < (1u << 22);

    int b_next = -1;                                   // request of the previous item
    while (t < t_end) {
        // Items after the first start where the previous list ended: the same request's next KV head or the next
        // request, so only the first one needs the search.
        int b = b_next;
        if (b < 0)
            b = ta_find_request(p, cum, t);
        else if ((int64_t)p.Hkv * cum[b + 1] <= t)
            ++b;
        b = __builtin_amdgcn_readfirstlane(b);
        b_next = b;
        const int n_u = __builtin_amdgcn_readfirstlane(cum[b + 1] - cum[b]);   // schedule units of one list
        const int cum_b = __builtin_amdgcn_readfirstlane(cum[b]);
        const int g = (t - p.Hkv * cum_b) / n_u;
        const int seg_start = p.Hkv * cum_b + g * n_u;                         // unit of the list's tile 0
        const int n_b = n_u - p.pad;
        const int j0 = t - seg_start;
        const int j1 = min(n_b, t_end - seg_start);
        if (j1 <= j0) {
            t = seg_start + n_u;                              // t lies in the list's trailing padding
            continue;
        }
        const int n = j1 - j0;
        const int slot = w + b * p.Hkv + g;
        ta_note_owner(p, b, g, w, j0, j1, n_b);
        const int L = __builtin_amdgcn_readfirstlane(lens[b]);
        const int S = __builtin_amdgcn_readfirstlane(starts[b]);
        bool poison = !ta_request_ok(p, L, S);
        const int tile0 = poison ? 0 : S / TA_TILE;                // absolute index of the list's first prefix tile
        if (poison && tid == 0)
            ta_raise(p, TA_STATUS_BAD_SEQLEN);
        const bool has_tree_tile = (j1 == n_b);
        // tile ti of this item: first logical position and number of tokens it holds
        auto tile_pos0 = [&](int ti) { return (j0 + ti == n_b - 1) ? L : (tile0 + j0 + ti) * TA_TILE; };
        auto tile_count = [&](int ti) {
            return (j0 + ti == n_b - 1) ? p.T : min(TA_TILE, L - (tile0 + j0 + ti) * TA_TILE);
        };
        // The item is walked in spans of tiles whose page ids fit the LDS cache (one span unless the pages are
        // tiny and the share very long).
        const int span_tiles = !paged ? n
                               : (p.ps_shift >= 6 ? PP_PAGES - 2 : max(1, ((PP_PAGES - 2) << p.ps_shift) / TA_TILE));
        // (lane roles inside an item come from fresh_tid(): nothing lane-dependent is carried from item to item)
        // A wave whose 32 rows all lie beyond the row group (T*G < 256) computes nothing; it still loads and
        // re-lays out its share of every tile and takes part in every barrier.
        const bool active = wave * 32 < rows_here;

        auto write_poison = [&]() {                        // a NaN log-sum-exp poisons the rows in the merge
            const int x = fresh_tid();
            const int prow = (x >> 6) * 32 + (x & 31), ph = (x >> 5) & 1;
            if (prow < rows_here) {
                const int64_t wrow = ta_ws_row(p, slot, rg, prow);
                for (int o = ph * 128; o < (ph + 1) * 128; o += 16)    // 128 16-bit values
                    *(float4 *)(ta_part_row(p, wrow) + o) = make_float4(0.f, 0.f, 0.f, 0.f);
                if (ph == 0)
                    p.ws_lse[2 * wrow] = __uint_as_float(0x7fc00000u);
            }
        };
        if (poison) {
            write_poison();
            __syncthreads();
            t = seg_start + (j1 == n_b ? n_u : j1);
            continue;
        }

        if (active) {
            // Q of this lane's row goes straight into its fixed registers; it is first read after the wait for the
            // first tile, which these loads precede.  Rows past the group's end read the group's first row (their
            // results are never stored).
            const int xl = fresh_tid();
            const int row = (xl >> 6) * 32 + (xl & 31), hfl = (xl >> 5) & 1;
            const int R = rg * p.rows_grp + (row < rows_here ? row : 0);
            const int node = (int)__umulhi((uint32_t)R << 8, p.g_magic);                 // R / G
            sp_load_q((const uint16_t *)p.q + (int64_t)b * p.q_sb + (int64_t)node * p.q_st +
                      (int64_t)(g * p.G + R - node * p.G) * p.q_sh + hfl * 8);
        }
        const uint16_t *kgp = (const uint16_t *)p.k + (int64_t)g * p.k_sh;
        const uint16_t *vgp = (const uint16_t *)p.v + (int64_t)g * p.v_sh;

        // bits of the tokens tile ti really holds for this lane's half, or all ones when nothing is to mask
        auto tile_mask = [&](int ti) -> unsigned long long {
            const int x = fresh_tid();
            const int rw = (x >> 6) * 32 + (x & 31), h = (x >> 5) & 1;
            const int j = j0 + ti;
            if (j == n_b - 1)
                return (rw < rows_here ? masks[p.q_off + __umulhi((uint32_t)(rg * p.rows_grp + rw) << 8, p.g_magic)]
                                       : ~0ull) >> (4 * h);
            return ta_prefix_tile_mask((tile0 + j) * TA_TILE, L, S) >> (4 * h);
        };
        // tiles that need a mask: the tree tile, a last prefix tile that is not full, a first one that begins before S
        auto tile_ragged = [&](int ti) {
            const int pos0 = (tile0 + j0 + ti) * TA_TILE;
            return j0 + ti == n_b - 1 || L - pos0 < TA_TILE || pos0 < S;
        };
        int span_first_page = 0;
        // Cache loads of tile ti into K slot ks and V slot vs: four 16-byte loads per lane.  Rows past the tile's
        // end, and rows before a window start, re-read its first attended token (their probabilities are exactly zero).
        // (wsel: the wave whose eight token rows are loaded -- this one's, or an active wave's that a helper serves)
        auto issue_rows = [&](int ti, int ks, int vs, int wsel) {
            const uint32_t kdst = lds0 + ks * MF_TILE_BYTES + wsel * 2048;
            const uint32_t vdst = lds0 + SP_V_OFF + vs * MF_TILE_BYTES + wsel * 2048;
            const int pos0 = tile_pos0(ti), cnt = tile_count(ti);
            if (fast_geom && !tile_ragged(ti)) {
                const int posw = pos0 + 8 * wsel;              // first of that wave's eight rows
                uint32_t pg = (uint32_t)b, sl = (uint32_t)posw;
                if (paged) {
                    pg = (uint32_t)__builtin_amdgcn_readfirstlane(pcache[(posw >> p.ps_shift) - span_first_page]);
                    sl = (uint32_t)(posw & (p.ps - 1));
                }
                const uint16_t *kb_ = kgp + (uint64_t)pg * ksp + (uint64_t)sl * kss;
                const uint16_t *vb_ = vgp + (uint64_t)pg * vsp + (uint64_t)sl * vss;
                uint32_t koff0, koff1, voff0, voff1;
                lane_offsets(koff0, koff1, voff0, voff1, wsel);
                dma16s(kb_, koff0, kdst);
                dma16s(kb_, koff1, kdst + 1024);
                dma16s(vb_, voff0, vdst);
                dma16s(vb_, voff1, vdst + 1024);
            } else {
                const int x = fresh_tid();
                const int drow = wsel * 8 + ((x & 63) >> 4), dslot = x & 15;
                // rows past the tile's end and rows before the window start read the tile's first attended token
                const int lo = max(0, S - pos0);
                auto row_pos = [&](int r) { return pos0 + (r < cnt && r >= lo ? r : lo); };
                const int pk[2] = {row_pos(drow), row_pos(drow + 4)};
                // With the write-back folded into the call the tree tokens come from the dense tensors of this step:
                // addressed like a contiguous cache, request stride for the page, token stride for the slot.
                bool from_new = false;
                if constexpr (NEW)
                    from_new = j0 + ti == n_b - 1;
                const uint16_t *kb0 = from_new ? (const uint16_t *)p.kn + (int64_t)g * p.kn_sh : kgp;
                const uint16_t *vb0 = from_new ? (const uint16_t *)p.vn + (int64_t)g * p.vn_sh : vgp;
                const uint64_t ksp_ = from_new ? (uint64_t)p.kn_sb : ksp, kss_ = from_new ? (uint64_t)p.kn_st : kss;
                const uint64_t vsp_ = from_new ? (uint64_t)p.vn_sb : vsp, vss_ = from_new ? (uint64_t)p.vn_st : vss;
                uint64_t ke[2], ve[2];
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    uint32_t pg = (uint32_t)b, sl = (uint32_t)pk[k];         // K and V rows hold the same tokens
                    if (from_new) {
                        sl -= (uint32_t)L;
                    } else if (paged) {
                        pg = (uint32_t)pcache[(pk[k] >> p.ps_shift) - span_first_page];
                        sl = (uint32_t)(pk[k] & (p.ps - 1));
                    }
                    ke[k] = (uint64_t)pg * ksp_ + (uint64_t)sl * kss_ + (dslot ^ ((drow + 4 * k) & 15)) * 8;
                    ve[k] = (uint64_t)pg * vsp_ + (uint64_t)sl * vss_ + (dslot ^ (2 * ((drow + 4 * k) & 7))) * 8;
                }
                dma16(kb0 + ke[0], kdst);
                dma16(kb0 + ke[1], kdst + 1024);
                dma16(vb0 + ve[0], vdst);
                dma16(vb0 + ve[1], vdst + 1024);
            }
        };
        // Outside the steady-state loop, where these loads are ordinary code in front of a wave's block, the waves
        // with query rows load nothing as long as there are as many waves without (row groups of up to 128 rows):
        // wave 8 - n_active + w, which only moves tiles anyway, loads the rows of active wave w on top of its own.
        const int n_active = (rows_here + 31) >> 5;
        const bool shift_loads = n_active <= 4;
        const int takeover = shift_loads ? wave - (8 - n_active) : -1;
        auto issue_tile = [&](int ti, int ks, int vs) {
            if (shift_loads && active)
                return;
            issue_rows(ti, ks, vs, wave);
            if (takeover >= 0)
                issue_rows(ti, ks, vs, takeover);
        };
        // The first three tiles of a span of up to SP_OWN_FIRST tiles are different: every wave loads its own rows of
        // them, the waves with query rows too -- they have nothing else to do yet, and the helper waves, which would
        // issue twice the loads, are what the first tile waits for (half a microsecond per item; p5 20.2 -> 19.6 us,
        // p1 33.6 -> 33.0).  Spans of a hundred tiles and more ran 1.5 % slower with it (uniform 16k lists: 168 ->
        // 170.5 us, in their steady state), so they keep the helpers' loads from the first tile on.
        auto issue_first = [&](int ti, int ks, int vs) { issue_rows(ti, ks, vs, wave); };
        auto wait_first = [&](int tiles_in_flight) {           // four loads per tile in every wave; Q is older
            if (tiles_in_flight >= 2)
                vm_wait<8>();
            else if (tiles_in_flight == 1)
                vm_wait<4>();
            else
                vm_wait<0>();
        };
        // all but the loads of the youngest tiles_in_flight tiles are done (four loads per tile and set of rows; a
        // wave that loads nothing has only its first tiles, its Q loads and earlier stores to wait for).  The youngest
        // tiles here are always ones that issue_tile has loaded.
        auto wait_loads = [&](int tiles_in_flight) {
            if (shift_loads && active) {
                vm_wait<0>();
            } else if (takeover >= 0) {
                if (tiles_in_flight >= 2)
                    vm_wait<16>();
                else if (tiles_in_flight == 1)
                    vm_wait<8>();
                else
                    vm_wait<0>();
            } else if (tiles_in_flight >= 2) {
                vm_wait<8>();
            } else if (tiles_in_flight == 1) {
                vm_wait<4>();
            } else {
                vm_wait<0>();
            }
        };

        int bad = 0;                                       // TA_STATUS_* bits this item has to report
        float m_run = -INFINITY, l_run = 0.f, l2_run = 0.f;   // l2: sum of the bf16-rounded probabilities

        for (int s0 = 0; s0 < n; s0 += span_tiles) {
            const int ns = min(span_tiles, n - s0);            // tiles s0 .. s0+ns-1 of the item; i is span-local
            // Page ids of the span and (first span) the parent ids, global memory -> LDS.  Q is on its way meanwhile;
            // everything here is used at once, so nothing lane-dependent has to be kept across the item.
            {
                const int x = fresh_tid();
                if (paged) {
                    // (positions before the window start are never read: their pages may be gone already)
                    span_first_page = max(tile_pos0(s0), S) >> p.ps_shift;
                    const int last_page = (tile_pos0(s0 + ns - 1) + tile_count(s0 + ns - 1) - 1) >> p.ps_shift;
                    for (int k = x; k <= last_page - span_first_page; k += 512) {
                        int id = p.page_table[(int64_t)b * p.pt_sb + span_first_page + k];
                        if (!ta_page_ok(p, id)) {              // must never become an address
                            atomicOr(&flag[1], TA_STATUS_BAD_PAGE);
                            id = 0;
                        }
                        pcache[k] = id;
                    }
                } else if (x == 0) {
                    pcache[0] = b;                             // the steady-state loop sees one page: the request's cache
                }
                const int xt = x;
                if (s0 == 0 && has_tree_tile && p.masks_in) {
                    if (xt < p.T) {
                        const unsigned long long gm = ta_given_mask(p, b, xt);     // encoded before the call
                        masks[xt] = gm;
                        if (!ta_given_mask_ok(gm, xt))
                            atomicOr(&flag[1], TA_STATUS_BAD_PARENT);
                    }
                } else if (s0 == 0 && has_tree_tile) {
                    if (x == 0)
                        *flag = 0;
                    if (xt < p.T)
                        par_s[xt] = p.parent[(int64_t)b * p.par_sb + xt];
                }
            }
            __syncthreads();
            bad = __builtin_amdgcn_readfirstlane(flag[1]);
            if (bad != 0) {
                vm_wait<0>();                                  // Q is still on its way into its registers
                break;
            }
            // ring positions: next slots to load into, K slot of tile i+1, V slots of tiles i and i-1
            int ik = 0, iv = 0, issued = 0;
            const bool own_first = ns <= SP_OWN_FIRST;
            for (; issued < min(ns, 3); ++issued) {
                if (own_first)
                    issue_first(s0 + issued, ik, iv);
                else
                    issue_tile(s0 + issued, ik, iv);
                ik = ik == SP_RK - 1 ? 0 : ik + 1;
                iv = iv == SP_RV - 1 ? 0 : iv + 1;
            }
            if (s0 == 0) {
                // while the first tiles are on their way: O = 0 and the ancestor masks
                sp_zero_o();
                if (has_tree_tile && !p.masks_in && !ta_encode_tree_lds(fresh_tid(), p.T, masks, flag, par_s)) {
                    bad = TA_STATUS_BAD_PARENT;
                    vm_wait<0>();                              // nothing may still land in the rings after this item
                    break;
                }
            }
            if (own_first)
                wait_first(issued - 1);                        // tile 0 and Q have landed
            else
                wait_loads(issued - 1);
            lds_barrier();
            if (active)
                sp_s_first(0u);
            if (active && tile_ragged(s0)) {
                const unsigned long long vm = tile_mask(s0);
                sp_mask_A((uint32_t)vm, (uint32_t)(vm >> 32));
            }
            if (ns > 1 && own_first)
                wait_first(issued - 2);                        // tile 1 has landed
            else if (ns > 1)
                wait_loads(issued - 2);
            lds_barrier();

            int kn = 1, vp = SP_RV - 1;                        // K slot of tile i+1, V slot of tile i-1
            auto step = [&](auto tag, int i) {
                constexpr bool A = decltype(tag)::value;       // S^T(i) sits in buffer A
                if (i + 3 < ns) {
                    issue_tile(s0 + i + 3, ik, iv);
                    ik = ik == SP_RK - 1 ? 0 : ik + 1;
                    iv = iv == SP_RV - 1 ? 0 : iv + 1;
                }
                const bool has_next = i + 1 < ns;
                const uint32_t ska = kn * MF_TILE_BYTES, sva = vp * MF_TILE_BYTES;
                float alpha = 1.f;
                if (!active) {
                } else if constexpr (A) {
                    if (i == 0) {
                        if (has_next)
                            sp_head_A(m_run, l_run, l2_run, alpha, c, ska);
                        else
                            sp_only_A(m_run, l_run, l2_run, alpha, c);
                    } else if (has_next) {
                        sp_full_A(sva, m_run, l_run, l2_run, alpha, c, ska);
                    } else {
                        sp_last_A(sva, m_run, l_run, l2_run, alpha, c);
                    }
                } else {
                    if (has_next)
                        sp_full_B(sva, m_run, l_run, l2_run, alpha, c, ska);
                    else
                        sp_last_B(sva, m_run, l_run, l2_run, alpha, c);
                }
                if (__any(alpha != 1.0f))
                    sp_scale_o(alpha);             // O still holds sums relative to the old reference
                if (active && has_next && tile_ragged(s0 + i + 1)) {
                    const unsigned long long vm = tile_mask(s0 + i + 1);
                    if constexpr (A)
                        sp_mask_B((uint32_t)vm, (uint32_t)(vm >> 32));
                    else
                        sp_mask_A((uint32_t)vm, (uint32_t)(vm >> 32));
                }
                if (i + 2 < ns)
                    wait_loads(i + 3 < ns ? 1 : 0);            // this wave's part of tile i+2 has landed
                lds_barrier();
                kn = kn == SP_RK - 1 ? 0 : kn + 1;
                vp = vp == SP_RV - 1 ? 0 : vp + 1;
            };
            // Steady state: every tile involved is a full prefix tile inside one page (or the contiguous cache), so
            // whole pairs of tiles run inside sp_fast_loop, which does its own loads and bookkeeping.
            const int n_plain = max(0, min(ns, L / TA_TILE - (tile0 + j0 + s0)));     // leading full prefix tiles of the span
            int i = 0;
#pragma unroll 1
            while (i < ns) {
                if (!(i & 1) && i >= 2 && fast_geom && i + 4 < n_plain) {
                    const uint32_t pairs = (uint32_t)((n_plain - 5 - i) / 2 + 1);
                    // (the loop looks pages up by `pos`, per wave: the position of the wave's first row of tile i+3)
                    uint32_t cnt = pairs, pos = (uint32_t)((tile0 + j0 + s0 + i + 3) * TA_TILE + 8 * wave);
                    uint32_t ik_o = ik * MF_TILE_BYTES, iv_o = iv * MF_TILE_BYTES, kn_o = kn * MF_TILE_BYTES;
                    uint32_t vp_o = vp * MF_TILE_BYTES;
                    const uint32_t pshift = paged ? (uint32_t)p.ps_shift : 31u;
                    const uint32_t pmask = paged ? (uint32_t)(p.ps - 1) : 0x7fffffffu;
                    const uint32_t pc_lds = lds0 + (uint32_t)((char *)pcache - smem) - 4u * (uint32_t)span_first_page;
                    const uint64_t c_kg = (uint64_t)(uintptr_t)kgp, c_vg = (uint64_t)(uintptr_t)vgp;
                    const uint64_t c_sp = (uint64_t)(ksp * 2u) | ((uint64_t)(vsp * 2u) << 32);
                    const uint64_t c_ss = (uint64_t)(kss * 2u) | ((uint64_t)(vss * 2u) << 32);
                    const uint64_t c_pp = (uint64_t)pshift | ((uint64_t)pmask << 32);
                    const uint64_t c_pc = (uint64_t)pc_lds | ((uint64_t)__float_as_uint(c) << 32);
                    const uint64_t c_dst = (uint64_t)(lds0 + wave * 2048) | ((uint64_t)(lds0 + SP_V_OFF + wave * 2048) << 32);
                    uint32_t koff0, koff1, voff0, voff1;
                    lane_offsets(koff0, koff1, voff0, voff1, wave);
                    if (active)
                        sp_fast_loop(m_run, l_run, l2_run, ik_o, iv_o, kn_o, vp_o, pos, cnt, c_kg, c_vg, c_sp, c_ss, c_pp, c_pc, c_dst,
                                     koff0, koff1, voff0, voff1);
                    else
                        sp_fast_loop_helper(ik_o, iv_o, kn_o, vp_o, pos, cnt, c_kg, c_vg, c_sp, c_ss, c_pp, c_pc, c_dst, koff0,
                                            koff1, voff0, voff1);
                    ik = ik_o / MF_TILE_BYTES;
                    iv = iv_o / MF_TILE_BYTES;
                    kn = kn_o / MF_TILE_BYTES;
                    vp = vp_o / MF_TILE_BYTES;
                    i += 2 * (int)pairs;
                } else {
                    if (i & 1)
                        step(SpTag<false>{}, i);
                    else
                        step(SpTag<true>{}, i);
                    ++i;
                }
            }
            if (active)
                sp_pv(vp * MF_TILE_BYTES);
            lds_barrier();                                     // the rings are free for the next span or item
        }
        if (bad != 0) {
            if (tid == 0)
                ta_raise(p, bad);
            write_poison();
            __syncthreads();                               // every thread has read flag[1] ...
            if (tid == 0)
                flag[1] = 0;
            __syncthreads();                               // ... and the next item starts from a clear one
            t = seg_start + (j1 == n_b ? n_u : j1);
            continue;
        }

        {
            // Partial result of this (workgroup, list) overlap, as 16-bit fixed point with one scale per row (see
            // ta_part_row).  A lane holds four-value pieces of one row, eight values apart; written like that,
            // every store would touch 64 cache lines.  So each wave first turns its 32 x 128 block into row-major
            // order in its part of the (now idle) K/V rings and then stores whole rows.
            const int x = fresh_tid();
            const int ln = x & 63, wv = x >> 6;
            const int r32_ = ln & 31, h = ln >> 5;
            const float l_tot = l_run + __shfl_xor(l_run, 32, TA_WAVE);
            const float l2_tot = l2_run + __shfl_xor(l2_run, 32, TA_WAVE);
            // The wave that stores the staged rows of active wave w: w itself, or -- row groups of up to 128 rows --
            // the helper wave that also loads w's rows, so that w goes on to the next item meanwhile.
            const int stores_for = shift_loads ? takeover : (active ? wv : -1);
            if (active) {
                // 16-byte chunk c of row r sits at chunk c ^ (r & 15); the lane's eight bytes of it at 8 h
                float scale;
                sp_put_q15(1.f / l2_tot, lds0 + (uint32_t)(wv * 16384 + r32_ * 256 + ((r32_ & 15) << 4) + 8 * h), scale);
                if (h == 0 && wv * 32 + r32_ < rows_here) {
                    const int64_t wrow = ta_ws_row(p, slot, rg, wv * 32 + r32_);
                    *(float2 *)&p.ws_lse[2 * wrow] = make_float2(m_run + log2f(l_tot), scale);
                }
            }
            if (shift_loads)
                lds_barrier();                             // the staged rows are visible to the wave that stores them
            else
                __builtin_amdgcn_wave_barrier();
            if (stores_for >= 0) {
                const char *stage = smem + stores_for * 16384;
                const int rw0 = stores_for * 32;
                const int cc = ln & 15, rq = ln >> 4;                  // 16 lanes store one row, four rows per round
#pragma unroll 2
                for (int it = 0; it < 8; ++it) {
                    const int rr = 4 * it + rq;
                    const uint4 val = *(const uint4 *)(stage + rr * 256 + ((cc ^ (rr & 15)) << 4));
                    if (rw0 + rr < rows_here)
                        *(uint4 *)(ta_part_row(p, ta_ws_row(p, slot, rg, rw0 + rr)) + 16 * cc) = val;
                }
            }
        }
        // The staging area is ring space again once its rows have been read: after the barrier below, or -- when helper
        // waves store -- after the barrier that every item and every poisoned one has before it loads a tile (the waves
        // with rows are already on their way to it).
        if (!shift_loads)
            lds_barrier();
        t = seg_start + (j1 == n_b ? n_u : j1);
    }
}

template <int NCW, int RB, int NT, int DH>
static hipError_t launch_variant(const TAParams &p, hipStream_t stream, int dev)
{
    const size_t smem = MF_STAGES * 2 * (TA_TILE * DH * 2) + sizeof(unsigned long long) * TA_MAX_TREE + 16 +
                        sizeof(int) * TA_MAX_TREE + sizeof(int) * (p.B + 2);
    static bool attr_set[64] = {};      // per device and variant; setting it twice is harmless
    if (dev < 0 || dev >= 64)
        return hipErrorInvalidDevice;
    if (!attr_set[dev]) {
        hipError_t e = hipFuncSetAttribute((const void *)ta_mfma_kv_kernel<NCW, RB, NT, DH>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 512);
        if (e != hipSuccess)
            return e;
        attr_set[dev] = true;
    }
    hipLaunchKernelGGL((ta_mfma_kv_kernel<NCW, RB, NT, DH>), dim3(p.n_wg, p.n_rg), dim3(NT), smem, stream, p);
    return hipGetLastError();
}

hipError_t ta_launch_mfma(const TAParams &p, hipStream_t stream, int dev)
{
    if (p.rows_grp != 32 && p.rows_grp != 64 && p.rows_grp != 128 && p.rows_grp != 256)
        return hipErrorInvalidValue;
    if (!p.part_q15 || p.ls != 2)                          // the one partial format these kernels write
        return hipErrorInvalidValue;
    if (p.D == 64)                                         // the register-staged kernel is the only one for this head dim
        return launch_variant<8, 1, 512, 64>(p, stream, dev);
    // One kernel for every row group: with fewer than 256 rows some of its eight waves only move tiles.
    const size_t smem = SP_AUX_OFF + sizeof(unsigned long long) * TA_MAX_TREE + 16 + sizeof(int) * TA_MAX_TREE +
                        sizeof(int) * PP_PAGES + sizeof(int) * (3 * p.B + 2);
    if (p.basic || smem > 160 * 1024 - 512)
        return launch_variant<8, 1, 512, 128>(p, stream, dev);   // register-staged kernel: very large batches, or on request
    static bool attr_set[64] = {};
    if (dev < 0 || dev >= 64)
        return hipErrorInvalidDevice;
    if (!attr_set[dev]) {
        for (const void *fn : {(const void *)ta_mfma_sp_kernel<false>, (const void *)ta_mfma_sp_kernel<true>}) {
            hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 512);
            if (e != hipSuccess)
                return e;
        }
        attr_set[dev] = true;
    }
    const dim3 grid(p.n_wg, p.n_rg);
    if (p.kn)
        hipLaunchKernelGGL((ta_mfma_sp_kernel<true>), grid, dim3(512), smem, stream, p);
    else
        hipLaunchKernelGGL((ta_mfma_sp_kernel<false>), grid, dim3(512), smem, stream, p);
    return hipGetLastError();
}
