// Scalar (vector-ALU, fp32-accumulating) kernels of libtreeattn: the any-shape KV pass, the merge pass
// and the stand-alone tree encoder.  The KV pass here is the portable path (fp32 inputs, head dims other
// than 128, page sizes that are not powers of two); the matrix-core path lives in ta_mfma.hip and shares
// the schedule and the merge.
#include "ta_common.h"

#define GEN_THREADS 256
#define GEN_WAVES (GEN_THREADS / TA_WAVE)
#define GEN_DCHUNKS (TA_MAX_HEAD_DIM / TA_WAVE)

template <bool BF16>
__device__ __forceinline__ float load_elem(const void *base, int64_t idx)
{
    if (BF16)
        return ta_bf16_to_f32(((const uint16_t *)base)[idx]);
    return ((const float *)base)[idx];
}

// The same in two steps -- the bits as they lie in memory, and their value -- for loads that stay in flight while
// other work goes on: a conversion next to the load would wait for it.
template <bool BF16>
__device__ __forceinline__ uint32_t load_bits(const void *base, int64_t row, uint32_t d)   // element d of the row
{
    // (row start and column apart: with a wave-uniform row the address is a scalar base plus a 32-bit lane offset)
    if (BF16)
        return ((const uint16_t *)base + row)[d];
    return ((const uint32_t *)base + row)[d];
}

template <bool BF16>
__device__ __forceinline__ float bits_value(uint32_t x)
{
    return BF16 ? ta_bf16_to_f32((uint16_t)x) : __uint_as_float(x);
}

// Barrier for data exchanged through LDS only: this wave's LDS traffic has landed, its global loads stay in flight
// (__syncthreads would wait for them as well).
__device__ __forceinline__ void gen_lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}


// KV pass for any shape.  A workgroup walks its share of a (request, KV head) tile list once per block of
// GEN_WAVES * RB query rows: every tile (64 tokens; section 3.1: prefix tiles are mask-free, the tree tile
// keeps only a row's ancestors) is staged in LDS as fp32, rows of tokens read coalesced, and then each wave
// updates its rows -- lanes are the tile's tokens for the scores, then head-dim columns for the weighted sum
// of V.  Running max / sum per row (base-2 domain).  Tokens that do not exist are staged as zeros.
// DCH = 64-column chunks of the head dimension a lane carries (1, 2 or 4).  A wave carries RB query rows at a time
// (eight with one chunk, which halves the passes over the tile list of the small-head shapes) and stages sixteen
// tokens of every tile; their loads go out one tile ahead, so that a tile's global round trip runs under the
// arithmetic of the tile before it, and Q's under the first tile's.
template <bool BF16, int DCH>
__global__ __launch_bounds__(GEN_THREADS) void ta_generic_kv_kernel(TAParams p)
{
    constexpr int RB = DCH == 1 ? 8 : 4;
    extern __shared__ int smem_i[];
    int *cum = smem_i;                                                   // [B + 1]
    int *lens = cum + ((p.B + 2) & ~1);                                  // [B] prefix lengths
    int *starts = lens + ((p.B + 1) & ~1);                               // [B] window starts
    unsigned long long *masks = (unsigned long long *)(starts + ((p.B + 1) & ~1));   // [64]
    int *flag = (int *)(masks + TA_MAX_TREE);                            // flag[4], then par_s[TA_MAX_TREE]
    int *par_s = flag + 4;
    float *qrow = (float *)(par_s + TA_MAX_TREE);                        // [GEN_WAVES * RB][D]
    float *kt = qrow + GEN_WAVES * RB * p.D;                         // [64][D + 1]: a lane reads its token's row
    float *vt = kt + TA_TILE * (p.D + 1);                                // [64][D]
    const int ldk = p.D + 1;

    ta_build_schedule(p, cum, lens, starts);
    const int total = p.Hkv * cum[p.B];
    const int w = blockIdx.x, rg = blockIdx.y;
    // (the wave index as a scalar: the addresses of a wave's rows and tokens are then scalar arithmetic)
    const int lane = threadIdx.x % TA_WAVE, wave = __builtin_amdgcn_readfirstlane(threadIdx.x / TA_WAVE);
    int t, t_end;
    ta_wg_range(p, total, w, t, t_end);
    const int rows_here = min(p.rows_grp, p.rows - rg * p.rows_grp);

    while (t < t_end) {
        const int b = ta_find_request(p, cum, t);
        const int n_u = cum[b + 1] - cum[b];                       // schedule units of one list of request b
        const int g = (t - p.Hkv * cum[b]) / n_u;
        const int seg_start = p.Hkv * cum[b] + g * n_u;            // unit of the list's tile 0
        const int n_b = n_u - p.pad;
        const int j0 = t - seg_start;
        const int j1 = min(n_b, t_end - seg_start);
        if (j1 <= j0) {
            t = seg_start + n_u;                              // t lies in the list's trailing padding
            continue;
        }
        const int slot = w + b * p.Hkv + g;
        ta_note_owner(p, b, g, w, j0, j1, n_b);
        const int L = lens[b];                                     // read once, by the schedule
        const int S = starts[b];
        bool poison = !ta_request_ok(p, L, S);
        const int tile0 = poison ? 0 : S / TA_TILE;               // absolute index of the list's first prefix tile
        if (poison && threadIdx.x == 0)
            ta_raise(p, TA_STATUS_BAD_SEQLEN);
        const bool has_tree_tile = (j1 == n_b);
        if (!poison) {
            int pos_lo, pos_hi;
            ta_item_positions(p, j0, j1, n_b, tile0, L, S, pos_lo, pos_hi);
            if (!ta_pages_ok(p, b, pos_lo, pos_hi, flag)) {
                poison = true;
                if (threadIdx.x == 0)
                    ta_raise(p, TA_STATUS_BAD_PAGE);
            }
        }
        if (has_tree_tile && !poison && p.masks_in) {
            if (threadIdx.x == 0)
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
                if (threadIdx.x == 0)
                    ta_raise(p, TA_STATUS_BAD_PARENT);
            }
        } else if (has_tree_tile && !poison) {
            if (!ta_encode_tree(p.parent + (int64_t)b * p.par_sb, p.T, masks, flag, par_s)) {
                poison = true;
                if (threadIdx.x == 0)
                    ta_raise(p, TA_STATUS_BAD_PARENT);
            }
        }
        for (int r0 = 0; r0 < rows_here; r0 += GEN_WAVES * RB) {
            int rr[RB];
            bool rok[RB];
            unsigned long long mask[RB];
            float m[RB], l[RB], acc[RB][DCH];
#pragma unroll
            for (int i = 0; i < RB; ++i) {
                rr[i] = r0 + wave * RB + i;
                rok[i] = rr[i] < rows_here;
                m[i] = -INFINITY;
                l[i] = 0.f;
#pragma unroll
                for (int c = 0; c < DCH; ++c)
                    acc[i][c] = 0.f;
                mask[i] = 0ull;
            }
            if (poison) {
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    if (!rok[i])
                        continue;
                    const int64_t wrow = ta_ws_row(p, slot, rg, rr[i]);
                    for (int d = lane; d < p.D; d += TA_WAVE)
                        p.ws_o[wrow * p.D + d] = 0.f;
                    if (lane == 0)
                        p.ws_lse[wrow] = __uint_as_float(0x7fc00000u);
                }
                continue;
            }
            // Q of the wave's rows: loaded here, written to LDS (rows only this wave reads) once the first tile's loads
            // are on their way as well.
            uint32_t qbits[RB][DCH];
#pragma unroll
            for (int i = 0; i < RB; ++i) {
#pragma unroll
                for (int c = 0; c < DCH; ++c)
                    qbits[i][c] = 0u;
                if (!rok[i])
                    continue;
                const int R = rg * p.rows_grp + rr[i];
                const int node = (int)__umulhi((uint32_t)R << 8, p.g_magic);          // R / G
                const int h = g * p.G + R - node * p.G;
                const int64_t qoff = (int64_t)b * p.q_sb + (int64_t)node * p.q_st + (int64_t)h * p.q_sh;
#pragma unroll
                for (int c = 0; c < DCH; ++c)
                    if (lane + c * TA_WAVE < p.D)
                        qbits[i][c] = load_bits<BF16>(p.q, qoff, (uint32_t)(lane + c * TA_WAVE));
                mask[i] = has_tree_tile ? masks[p.q_off + node] : 0ull;
            }
            // Wave w stages tokens 16w .. 16w+15 of every tile: their loads are issued a tile ahead and stay in flight
            // while the tile before is computed.  Tokens that do not exist are staged as zeros.
            constexpr int TOK = TA_TILE / GEN_WAVES;
            uint32_t kbits[TOK][DCH], vbits[TOK][DCH];
            auto load_tile = [&](int j) {
                const bool tree_tile = (j == n_b - 1);
#pragma unroll
                for (int u = 0; u < TOK; ++u) {
                    const int tk = wave * TOK + u;
                    const int pos = tree_tile ? L + tk : (tile0 + j) * TA_TILE + tk;
                    const bool exists = tree_tile ? tk < p.T : (pos >= S && pos < L);
                    // with the write-back folded in, the tree tokens come from the dense tensors of this step
                    const bool from_new = tree_tile && p.kn != nullptr;
                    const void *kb = from_new ? p.kn : p.k, *vb = from_new ? p.vn : p.v;
                    int64_t koff = 0, voff = 0;
                    if (exists && from_new) {
                        koff = (int64_t)b * p.kn_sb + (int64_t)tk * p.kn_st + (int64_t)g * p.kn_sh;
                        voff = (int64_t)b * p.vn_sb + (int64_t)tk * p.vn_st + (int64_t)g * p.vn_sh;
                    } else if (exists) {
                        koff = ta_cache_offset(p, b, g, pos, p.k_sp, p.k_sh, p.k_ss);
                        voff = ta_cache_offset(p, b, g, pos, p.v_sp, p.v_sh, p.v_ss);
                    }
#pragma unroll
                    for (int c = 0; c < DCH; ++c) {
                        const int d = lane + c * TA_WAVE;
                        const bool ld = exists && d < p.D && koff >= 0 && voff >= 0;
                        kbits[u][c] = ld ? load_bits<BF16>(kb, koff, (uint32_t)d) : 0u;
                        vbits[u][c] = ld ? load_bits<BF16>(vb, voff, (uint32_t)d) : 0u;
                    }
                }
            };
            load_tile(j0);
            for (int j = j0; j < j1; ++j) {
                const bool tree_tile = (j == n_b - 1);
                gen_lds_barrier();                                   // the previous tile has been consumed
#pragma unroll
                for (int u = 0; u < TOK; ++u)
#pragma unroll
                    for (int c = 0; c < DCH; ++c) {
                        const int d = lane + c * TA_WAVE;
                        if (d < p.D) {
                            kt[(wave * TOK + u) * ldk + d] = bits_value<BF16>(kbits[u][c]);
                            vt[(wave * TOK + u) * p.D + d] = bits_value<BF16>(vbits[u][c]);
                        }
                    }
                if (j == j0) {
#pragma unroll
                    for (int i = 0; i < RB; ++i)
#pragma unroll
                        for (int c = 0; c < DCH; ++c)
                            if (rok[i] && lane + c * TA_WAVE < p.D)
                                qrow[(wave * RB + i) * p.D + lane + c * TA_WAVE] = bits_value<BF16>(qbits[i][c]);
                }
                gen_lds_barrier();
                if (j + 1 < j1)
                    load_tile(j + 1);
                // Scores of the wave's rows against the lane's token: one LDS read of K serves all rows; q[d]
                // comes out of the lane that holds it as a scalar operand.
                float qreg[RB][DCH], dot[RB];
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    const float *qs = qrow + (wave * RB + i) * p.D;
                    dot[i] = 0.f;
#pragma unroll
                    for (int c = 0; c < DCH; ++c)
                        qreg[i][c] = (rok[i] && lane + c * TA_WAVE < p.D) ? qs[lane + c * TA_WAVE] : 0.f;
                }
                const float *kr = kt + lane * ldk;
#pragma unroll
                for (int c = 0; c < DCH; ++c) {
                    const int dn = min(TA_WAVE, p.D - c * TA_WAVE);              // columns of this chunk (<= 0: none)
#pragma unroll 4
                    for (int dd = 0; dd < dn; ++dd) {
                        const float kd = kr[c * TA_WAVE + dd];
#pragma unroll
                        for (int i = 0; i < RB; ++i)
                            dot[i] = fmaf(__int_as_float(__builtin_amdgcn_readlane(__float_as_int(qreg[i][c]), dd)), kd,
                                          dot[i]);
                    }
                }
                float pr[RB];
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    const int pos_l = (tile0 + j) * TA_TILE + lane;
                    const bool valid = rok[i] && (tree_tile ? (lane < p.T && ((mask[i] >> lane) & 1ull))
                                                            : (pos_l >= S && pos_l < L));
                    const float s = valid ? dot[i] * p.scale_log2e : -INFINITY;
                    // rows that exist always see a valid token in a tile; padding rows keep m = -inf, pr = 0
                    const float m_new = fmaxf(m[i], ta_wave_max(s));
                    const float alpha = rok[i] ? exp2f(m[i] - m_new) : 1.f;
                    pr[i] = valid ? exp2f(s - m_new) : 0.f;
                    l[i] = l[i] * alpha + ta_wave_sum(pr[i]);
                    m[i] = m_new;
#pragma unroll
                    for (int c = 0; c < DCH; ++c)
                        acc[i][c] *= alpha;
                }
#pragma unroll 4
                for (int jj = 0; jj < TA_TILE; ++jj) {
                    float vj[DCH];
#pragma unroll
                    for (int c = 0; c < DCH; ++c)
                        vj[c] = lane + c * TA_WAVE < p.D ? vt[jj * p.D + lane + c * TA_WAVE] : 0.f;
#pragma unroll
                    for (int i = 0; i < RB; ++i) {
                        const float pj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pr[i]), jj));  // scalar
#pragma unroll
                        for (int c = 0; c < DCH; ++c)
                            acc[i][c] = fmaf(pj, vj[c], acc[i][c]);
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < RB; ++i) {
                if (!rok[i])
                    continue;
                const int64_t wrow = ta_ws_row(p, slot, rg, rr[i]);
                const float inv = 1.f / l[i];
#pragma unroll
                for (int c = 0; c < DCH; ++c) {
                    const int d = lane + c * TA_WAVE;
                    if (d < p.D)
                        p.ws_o[wrow * p.D + d] = acc[i][c] * inv;
                }
                if (lane == 0)
                    p.ws_lse[wrow] = m[i] + log2f(l[i]);
            }
        }
        __syncthreads();               // masks / flag and the tiles are reused by the next item
        t = seg_start + (j1 == n_b ? n_u : j1);
    }
}

template <bool BF16, int DCH>
static hipError_t launch_generic_instance(const TAParams &p, hipStream_t stream, bool *attr_done)
{
    constexpr int RB = DCH == 1 ? 8 : 4;
    const size_t smem = sizeof(int) * (((p.B + 2) & ~1) + 2 * ((p.B + 1) & ~1)) + sizeof(unsigned long long) * TA_MAX_TREE + 16 +
                        sizeof(int) * TA_MAX_TREE +
                        sizeof(float) * ((size_t)GEN_WAVES * RB * p.D + (size_t)TA_TILE * (2 * p.D + 1));
    if (smem > 160 * 1024 - 512)
        return hipErrorInvalidValue;
    if (!*attr_done) {
        hipError_t e = hipFuncSetAttribute((const void *)ta_generic_kv_kernel<BF16, DCH>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 512);
        if (e != hipSuccess)
            return e;
        *attr_done = true;
    }
    hipLaunchKernelGGL((ta_generic_kv_kernel<BF16, DCH>), dim3(p.n_wg, p.n_rg), dim3(GEN_THREADS), smem, stream, p);
    return hipGetLastError();
}

hipError_t ta_launch_generic(const TAParams &p, hipStream_t stream, int dev)
{
    static bool attr_set[64][2][3] = {};
    if (dev < 0 || dev >= 64)
        return hipErrorInvalidDevice;
    const int bf = p.is_bf16 ? 1 : 0;
    if (p.D <= TA_WAVE)
        return bf ? launch_generic_instance<true, 1>(p, stream, &attr_set[dev][1][0])
                  : launch_generic_instance<false, 1>(p, stream, &attr_set[dev][0][0]);
    if (p.D <= 2 * TA_WAVE)
        return bf ? launch_generic_instance<true, 2>(p, stream, &attr_set[dev][1][1])
                  : launch_generic_instance<false, 2>(p, stream, &attr_set[dev][0][1]);
    return bf ? launch_generic_instance<true, 4>(p, stream, &attr_set[dev][1][2])
              : launch_generic_instance<false, 4>(p, stream, &attr_set[dev][0][2]);
}

// Merge pass (section 3.1: full attention from partial attentions over disjoint chunks of the keys,
// through their log-sum-exps).  One wave per output row: lanes first span the partials of the row
// (wave-wide max and sum of the partial log-sum-exps give every partial its weight), then span
// head-dim columns, with the loads of several partials in flight at once.
template <bool NEW>
__global__ __launch_bounds__(GEN_THREADS) void ta_merge_kernel(TAParams p)
{
    const int seg = blockIdx.x;
    const int b = seg / p.Hkv, g = seg % p.Hkv;
    const int lane = threadIdx.x % TA_WAVE, wave = threadIdx.x / TA_WAVE;
    const int w_first = p.ws_parts[2 * seg];                             // left by the KV pass
    const int n_parts = p.ws_parts[2 * seg + 1] - w_first + 1;
    const float LN2 = 0.6931471805599453f;
    const float QNAN = __uint_as_float(0x7fc00000u);

    if constexpr (NEW) {
        TAScatter sc;
        ta_scatter_load(p, b, g, blockIdx.y, gridDim.y, sc);
        ta_scatter_locate(p, b, g, sc);
        ta_scatter_store(p, b, g, blockIdx.y, gridDim.y, sc);
    }
    const int R = blockIdx.y * TA_MERGE_ROWS + wave;
    if (R >= p.rows)
        return;
    const int rg = R / p.rows_grp, r = R % p.rows_grp;
    const int node = R / p.G, h = g * p.G + R % p.G;
    const int64_t row0 = ta_ws_row(p, w_first + seg, rg, r);              // partial k of this row: row0 + k*pstride
    const int64_t pstride = (int64_t)p.n_rg * p.rows_grp;

    float acc[GEN_DCHUNKS];
#pragma unroll
    for (int c = 0; c < GEN_DCHUNKS; ++c)
        acc[c] = 0.f;
    float lse2;
    if (n_parts <= TA_WAVE) {
        // lane k owns partial k
        const float lk = lane < n_parts ? p.ws_lse[(row0 + lane * pstride) * p.ls] : -INFINITY;
        const bool nan_seen = __any(lk != lk);
        const float mx = ta_wave_max(lk);
        const float ek = exp2f(lk - mx);                                  // 0 for the idle lanes
        const float den = ta_wave_sum(ek);
        lse2 = nan_seen ? QNAN : mx + log2f(den);
        const float wk = nan_seen ? QNAN : ek / den;
        int k = 0;
        for (; k + 4 <= n_parts; k += 4) {
            float v[4][GEN_DCHUNKS];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int c = 0; c < GEN_DCHUNKS; ++c) {
                    const int d = lane + c * TA_WAVE;
                    v[u][c] = d < p.D ? ta_part_get(p, row0 + (k + u) * pstride, d) : 0.f;
                }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float wgt = __shfl(wk, k + u, TA_WAVE);
#pragma unroll
                for (int c = 0; c < GEN_DCHUNKS; ++c)
                    acc[c] = fmaf(wgt, v[u][c], acc[c]);
            }
        }
        for (; k < n_parts; ++k) {
            const float wgt = __shfl(wk, k, TA_WAVE);
#pragma unroll
            for (int c = 0; c < GEN_DCHUNKS; ++c) {
                const int d = lane + c * TA_WAVE;
                if (d < p.D)
                    acc[c] = fmaf(wgt, ta_part_get(p, row0 + k * pstride, d), acc[c]);
            }
        }
    } else {
        // more partials than lanes: two sweeps over the log-sum-exps, then one over the outputs
        float mx = -INFINITY;
        bool nan_seen = false;
        for (int q0 = 0; q0 < n_parts; q0 += TA_WAVE) {
            const int k = q0 + lane;
            if (k < n_parts) {
                const float v = p.ws_lse[(row0 + k * pstride) * p.ls];
                nan_seen |= (v != v);
                mx = fmaxf(mx, v);
            }
        }
        mx = ta_wave_max(mx);
        nan_seen = __any(nan_seen);
        float den = 0.f;
        for (int q0 = 0; q0 < n_parts; q0 += TA_WAVE) {
            const int k = q0 + lane;
            if (k < n_parts)
                den += exp2f(p.ws_lse[(row0 + k * pstride) * p.ls] - mx);
        }
        den = ta_wave_sum(den);
        lse2 = nan_seen ? QNAN : mx + log2f(den);
        for (int k = 0; k < n_parts; ++k) {
            const float wgt = exp2f(p.ws_lse[(row0 + k * pstride) * p.ls] - lse2);  // same address in every lane
#pragma unroll
            for (int c = 0; c < GEN_DCHUNKS; ++c) {
                const int d = lane + c * TA_WAVE;
                if (d < p.D)
                    acc[c] = fmaf(wgt, ta_part_get(p, row0 + k * pstride, d), acc[c]);
            }
        }
    }
    const int64_t ooff = (int64_t)b * p.o_sb + (int64_t)node * p.o_st + (int64_t)h * p.o_sh;
#pragma unroll
    for (int c = 0; c < GEN_DCHUNKS; ++c) {
        const int d = lane + c * TA_WAVE;
        if (d < p.D) {
            if (p.is_bf16)
                ((uint16_t *)p.out)[ooff + d] = ta_f32_to_bf16(acc[c]);
            else
                ((float *)p.out)[ooff + d] = acc[c];
        }
    }
    if (p.lse && lane == 0)
        p.lse[(int64_t)b * p.lse_sb + (int64_t)h * p.lse_sh + (int64_t)node * p.lse_st] = lse2 * LN2;
}

// The same merge for head_dim 128 and 16-byte aligned outputs: half a wave per output row, so that a lane holds four
// neighbouring columns (one 16-byte load per partial and lane) and a workgroup of four waves merges eight rows.
#define MG_ROWS TA_MERGE128_ROWS

__device__ __forceinline__ float ta_half_max(float x)          // over the 32 lanes of this lane's half-wave
{
    for (int off = 16; off > 0; off >>= 1)
        x = fmaxf(x, __shfl_xor(x, off, TA_WAVE));
    return x;
}

__device__ __forceinline__ float ta_half_sum(float x)
{
    for (int off = 16; off > 0; off >>= 1)
        x += __shfl_xor(x, off, TA_WAVE);
    return x;
}

// Four neighbouring columns of one partial row: fp32, or (HP) int16, which the caller's weight carries the scale of.
// The load returns the bits as they lie in memory and the conversion happens where the values are used: a conversion
// next to the load would make every load wait for its data, and the loads of a round are meant to be in flight together.
template <bool HP>
struct ta_part_raw { typedef float4 type; };
template <>
struct ta_part_raw<true> { typedef ta_s4 type; };

template <bool HP>
__device__ __forceinline__ typename ta_part_raw<HP>::type ta_part_load4(const char *ptr)
{
    return *(const typename ta_part_raw<HP>::type *)ptr;
}

__device__ __forceinline__ float4 ta_part_f4(const float4 &x) { return x; }
__device__ __forceinline__ float4 ta_part_f4(const ta_s4 &x)
{
    return make_float4((float)x.x, (float)x.y, (float)x.z, (float)x.w);
}

template <bool NEW, bool HP>
__global__ __launch_bounds__(256) void ta_merge128_kernel(TAParams p)
{
    const int seg = blockIdx.x;
    const int b = seg / p.Hkv, g = seg % p.Hkv;
    const int lane = threadIdx.x % TA_WAVE, wave = threadIdx.x / TA_WAVE;
    const int hl = lane & 31, half = lane >> 5;
    const int w_first = p.ws_parts[2 * seg];                             // left by the KV pass
    const int n_parts = p.ws_parts[2 * seg + 1] - w_first + 1;
    const float LN2 = 0.6931471805599453f;
    const float QNAN = __uint_as_float(0x7fc00000u);

    TAScatter sc;                                          // write-back folded into the call: see ta_scatter_load
    if constexpr (NEW)
        ta_scatter_load(p, b, g, blockIdx.y, gridDim.y, sc);
    const int R_raw = blockIdx.y * MG_ROWS + wave * 2 + half;
    if (R_raw - half >= p.rows) {                          // the whole wave is past the last row
        if constexpr (NEW) {
            ta_scatter_locate(p, b, g, sc);
            ta_scatter_store(p, b, g, blockIdx.y, gridDim.y, sc);
        }
        return;
    }
    const bool live = R_raw < p.rows;
    const int R = live ? R_raw : p.rows - 1;               // an odd last row: its idle partner half repeats it
    const int rg = R / p.rows_grp, r = R % p.rows_grp;
    const int node = R / p.G, h = g * p.G + R % p.G;
    const int64_t row0 = ta_ws_row(p, w_first + seg, rg, r);              // partial k of this row: row0 + k*pstride
    const int64_t pstride = (int64_t)p.n_rg * p.rows_grp;
    constexpr int EB = HP ? 2 : 4;                         // bytes per element of a partial output
    constexpr int LS = HP ? 2 : 1;                         // floats per row of ws_lse: {log-sum-exp, scale} or the former
    const char *o0 = (const char *)p.ws_o + (row0 * 128 + 4 * hl) * EB;
    const int64_t ostride = pstride * 128 * EB;

    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float lse2;
    if (n_parts <= 32) {
        // lane k of the half owns partial k
        float lk = -INFINITY, sk = 1.f;                                   // sk: scale of the partial's 16-bit values
        if (hl < n_parts) {
            if constexpr (HP) {
                const float2 t = *(const float2 *)&p.ws_lse[(row0 + hl * pstride) * LS];
                lk = t.x;
                sk = t.y;
            } else {
                lk = p.ws_lse[(row0 + hl * pstride) * LS];
            }
        }
        if constexpr (NEW)
            ta_scatter_locate(p, b, g, sc);
        const bool nan_seen = ta_half_max(lk != lk ? 1.f : 0.f) > 0.f;
        const float mx = ta_half_max(lk);
        const float ek = exp2f(lk - mx);                                  // 0 for the idle lanes
        const float den = ta_half_sum(ek);
        lse2 = nan_seen ? QNAN : mx + log2f(den);
        const float wk = nan_seen ? QNAN : ek / den * sk;
        const int src0 = lane & 32;
        int k = 0;
        for (; k + 4 <= n_parts; k += 4) {
            typename ta_part_raw<HP>::type v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                v[u] = ta_part_load4<HP>(o0 + (k + u) * ostride);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float wgt = __shfl(wk, src0 + k + u, TA_WAVE);
                const float4 x = ta_part_f4(v[u]);
                acc.x = fmaf(wgt, x.x, acc.x);
                acc.y = fmaf(wgt, x.y, acc.y);
                acc.z = fmaf(wgt, x.z, acc.z);
                acc.w = fmaf(wgt, x.w, acc.w);
            }
        }
        // The tail's loads go out together as well.  (Both halves of a wave merge rows of the same list, so
        // n_parts and with it every branch here is uniform over the wave.)
        typename ta_part_raw<HP>::type v[3];
#pragma unroll
        for (int u = 0; u < 3; ++u)
            if (k + u < n_parts)
                v[u] = ta_part_load4<HP>(o0 + (k + u) * ostride);
#pragma unroll
        for (int u = 0; u < 3; ++u)
            if (k + u < n_parts) {
                const float wgt = __shfl(wk, src0 + k + u, TA_WAVE);
                const float4 x = ta_part_f4(v[u]);
                acc.x = fmaf(wgt, x.x, acc.x);
                acc.y = fmaf(wgt, x.y, acc.y);
                acc.z = fmaf(wgt, x.z, acc.z);
                acc.w = fmaf(wgt, x.w, acc.w);
            }
    } else {
        if constexpr (NEW)
            ta_scatter_locate(p, b, g, sc);
        // more partials than lanes in a half: two sweeps over the log-sum-exps, then one over the outputs
        float mx = -INFINITY, bad = 0.f;
        for (int q0 = 0; q0 < n_parts; q0 += 32) {
            const int k = q0 + hl;
            if (k < n_parts) {
                const float v = p.ws_lse[(row0 + k * pstride) * LS];
                bad = v != v ? 1.f : bad;
                mx = fmaxf(mx, v);
            }
        }
        mx = ta_half_max(mx);
        const bool nan_seen = ta_half_max(bad) > 0.f;
        float den = 0.f;
        for (int q0 = 0; q0 < n_parts; q0 += 32) {
            const int k = q0 + hl;
            if (k < n_parts)
                den += exp2f(p.ws_lse[(row0 + k * pstride) * LS] - mx);
        }
        den = ta_half_sum(den);
        lse2 = nan_seen ? QNAN : mx + log2f(den);
        for (int k = 0; k < n_parts; ++k) {
            float wgt = exp2f(p.ws_lse[(row0 + k * pstride) * LS] - lse2);        // same address in every lane of the half
            if constexpr (HP)
                wgt *= p.ws_lse[(row0 + k * pstride) * LS + 1];
            const float4 v = ta_part_f4(ta_part_load4<HP>(o0 + k * ostride));
            acc.x = fmaf(wgt, v.x, acc.x);
            acc.y = fmaf(wgt, v.y, acc.y);
            acc.z = fmaf(wgt, v.z, acc.z);
            acc.w = fmaf(wgt, v.w, acc.w);
        }
    }
    if constexpr (NEW)
        ta_scatter_store(p, b, g, blockIdx.y, gridDim.y, sc);
    if (!live)
        return;
    const int64_t ooff = (int64_t)b * p.o_sb + (int64_t)node * p.o_st + (int64_t)h * p.o_sh + 4 * hl;
    if (p.is_bf16) {
        uint2 o;
        o.x = (uint32_t)ta_f32_to_bf16(acc.x) | ((uint32_t)ta_f32_to_bf16(acc.y) << 16);
        o.y = (uint32_t)ta_f32_to_bf16(acc.z) | ((uint32_t)ta_f32_to_bf16(acc.w) << 16);
        *(uint2 *)((uint16_t *)p.out + ooff) = o;
    } else {
        *(float4 *)((float *)p.out + ooff) = acc;
    }
    if (p.lse && hl == 0)
        p.lse[(int64_t)b * p.lse_sb + (int64_t)h * p.lse_sh + (int64_t)node * p.lse_st] = lse2 * LN2;
}

// Many partials per list (few lists cut over the whole chip: the batch-size-one regime): one workgroup per output row,
// its eight half-waves take every eighth partial each, up to MW_FLIGHT loads in flight per lane, and their sums meet
// in LDS.  The loads of the first round are issued before the log-sum-exps are reduced, so the two latencies overlap.
// (With the kernel above a half-wave walks all partials of its row alone: 256 partials took 38 us, now about 7.)
constexpr int MW_HALVES = 8, MW_FLIGHT = 8;

template <bool NEW, bool HP>
__global__ __launch_bounds__(256) void ta_merge128_wide_kernel(TAParams p)
{
    __shared__ float red[8];
    __shared__ float4 part[MW_HALVES][32];
    const int seg = blockIdx.x, R = blockIdx.y;
    const int b = seg / p.Hkv, g = seg % p.Hkv;
    const int tid = threadIdx.x, hw = tid >> 5, hl = tid & 31, wave = tid >> 6;
    const int w_first = p.ws_parts[2 * seg];                             // left by the KV pass
    const int n_parts = p.ws_parts[2 * seg + 1] - w_first + 1;
    const float LN2 = 0.6931471805599453f;
    const float QNAN = __uint_as_float(0x7fc00000u);
    TAScatter sc;                                          // write-back folded into the call: see ta_scatter_load
    if constexpr (NEW)
        ta_scatter_load(p, b, g, blockIdx.y, gridDim.y, sc);
    const int rg = R / p.rows_grp, r = R % p.rows_grp;
    const int node = R / p.G, h = g * p.G + R % p.G;
    const int64_t row0 = ta_ws_row(p, w_first + seg, rg, r);              // partial k of this row: row0 + k*pstride
    const int64_t pstride = (int64_t)p.n_rg * p.rows_grp;
    constexpr int EB = HP ? 2 : 4;                         // bytes per element of a partial output
    constexpr int LS = HP ? 2 : 1;                         // floats per row of ws_lse: {log-sum-exp, scale} or the former
    const char *o0 = (const char *)p.ws_o + (row0 * 128 + 4 * hl) * EB;
    const int64_t ostride = pstride * 128 * EB;

    // first round of this half-wave's partials (hw, hw + 8, ...): outputs and their log-sum-exps
    typename ta_part_raw<HP>::type v[MW_FLIGHT];
    float2 ls[MW_FLIGHT];                                  // log-sum-exps and (16-bit partials: one 8-byte load) scales
#pragma unroll
    for (int u = 0; u < MW_FLIGHT; ++u) {
        const int k = hw + MW_HALVES * u;
        if (k < n_parts) {
            v[u] = ta_part_load4<HP>(o0 + k * ostride);
            if constexpr (HP)
                ls[u] = *(const float2 *)&p.ws_lse[(row0 + k * pstride) * LS];
            else
                ls[u].x = p.ws_lse[(row0 + k * pstride) * LS];
        }
    }
    if constexpr (NEW)
        ta_scatter_locate(p, b, g, sc);
    // log-sum-exp of the row over all partials (thread t keeps partial t's value for the second sweep; only with
    // more than 256 partials is anything read twice)
    const float x_own = tid < n_parts ? p.ws_lse[(row0 + tid * pstride) * LS] : -INFINITY;
    float mx = x_own, bad = x_own != x_own ? 1.f : 0.f;
    for (int k = tid + 256; k < n_parts; k += 256) {
        const float x = p.ws_lse[(row0 + k * pstride) * LS];
        bad = x != x ? 1.f : bad;
        mx = fmaxf(mx, x);
    }
    mx = ta_wave_max(mx);
    bad = ta_wave_max(bad);
    if ((tid & 63) == 0) {
        red[wave] = mx;
        red[4 + wave] = bad;
    }
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const bool nan_seen = fmaxf(fmaxf(red[4], red[5]), fmaxf(red[6], red[7])) > 0.f;
    __syncthreads();
    float den = tid < n_parts ? exp2f(x_own - mx) : 0.f;
    for (int k = tid + 256; k < n_parts; k += 256)
        den += exp2f(p.ws_lse[(row0 + k * pstride) * LS] - mx);
    den = ta_wave_sum(den);
    if ((tid & 63) == 0)
        red[wave] = den;
    __syncthreads();
    den = (red[0] + red[1]) + (red[2] + red[3]);
    const float lse2 = nan_seen ? QNAN : mx + log2f(den);

    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int k0 = hw; k0 < n_parts; k0 += MW_HALVES * MW_FLIGHT) {
        if (k0 != hw) {
#pragma unroll
            for (int u = 0; u < MW_FLIGHT; ++u) {
                const int k = k0 + MW_HALVES * u;
                if (k < n_parts) {
                    v[u] = ta_part_load4<HP>(o0 + k * ostride);
                    if constexpr (HP)
                        ls[u] = *(const float2 *)&p.ws_lse[(row0 + k * pstride) * LS];
                    else
                        ls[u].x = p.ws_lse[(row0 + k * pstride) * LS];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < MW_FLIGHT; ++u) {
            if (k0 + MW_HALVES * u < n_parts) {
                const float wgt = nan_seen ? QNAN : exp2f(ls[u].x - lse2) * (HP ? ls[u].y : 1.f);
                const float4 x = ta_part_f4(v[u]);
                acc.x = fmaf(wgt, x.x, acc.x);
                acc.y = fmaf(wgt, x.y, acc.y);
                acc.z = fmaf(wgt, x.z, acc.z);
                acc.w = fmaf(wgt, x.w, acc.w);
            }
        }
    }
    part[hw][hl] = acc;
    if constexpr (NEW)
        ta_scatter_store(p, b, g, blockIdx.y, gridDim.y, sc);
    __syncthreads();
    if (tid >= 32)
        return;
    acc = part[0][hl];
#pragma unroll
    for (int k = 1; k < MW_HALVES; ++k) {
        const float4 x = part[k][hl];
        acc.x += x.x;
        acc.y += x.y;
        acc.z += x.z;
        acc.w += x.w;
    }
    const int64_t ooff = (int64_t)b * p.o_sb + (int64_t)node * p.o_st + (int64_t)h * p.o_sh + 4 * hl;
    if (p.is_bf16) {
        uint2 o;
        o.x = (uint32_t)ta_f32_to_bf16(acc.x) | ((uint32_t)ta_f32_to_bf16(acc.y) << 16);
        o.y = (uint32_t)ta_f32_to_bf16(acc.z) | ((uint32_t)ta_f32_to_bf16(acc.w) << 16);
        *(uint2 *)((uint16_t *)p.out + ooff) = o;
    } else {
        *(float4 *)((float *)p.out + ooff) = acc;
    }
    if (p.lse && hl == 0)
        p.lse[(int64_t)b * p.lse_sb + (int64_t)h * p.lse_sh + (int64_t)node * p.lse_st] = lse2 * LN2;
}

hipError_t ta_launch_merge(const TAParams &p, hipStream_t stream)
{
    const size_t smem = 0;
    const int rows_wg = ta_host_merge_rows(p);             // the plan chose the kernel (p.merge_kind)
    dim3 grid(p.B * p.Hkv, (p.rows + rows_wg - 1) / rows_wg);
    // (the instances with the write-back folded in also copy the tree tokens' K/V into the caches)
    if (p.merge_kind == TA_MERGE_D128_WIDE) {
        if (p.kn && p.part_q15)
            hipLaunchKernelGGL((ta_merge128_wide_kernel<true, true>), grid, dim3(256), smem, stream, p);
        else if (p.kn)
            hipLaunchKernelGGL((ta_merge128_wide_kernel<true, false>), grid, dim3(256), smem, stream, p);
        else if (p.part_q15)
            hipLaunchKernelGGL((ta_merge128_wide_kernel<false, true>), grid, dim3(256), smem, stream, p);
        else
            hipLaunchKernelGGL((ta_merge128_wide_kernel<false, false>), grid, dim3(256), smem, stream, p);
    } else if (p.merge_kind == TA_MERGE_D128) {
        if (p.kn && p.part_q15)
            hipLaunchKernelGGL((ta_merge128_kernel<true, true>), grid, dim3(256), smem, stream, p);
        else if (p.kn)
            hipLaunchKernelGGL((ta_merge128_kernel<true, false>), grid, dim3(256), smem, stream, p);
        else if (p.part_q15)
            hipLaunchKernelGGL((ta_merge128_kernel<false, true>), grid, dim3(256), smem, stream, p);
        else
            hipLaunchKernelGGL((ta_merge128_kernel<false, false>), grid, dim3(256), smem, stream, p);
    } else {
        if (p.kn)
            hipLaunchKernelGGL(ta_merge_kernel<true>, grid, dim3(GEN_THREADS), smem, stream, p);
        else
            hipLaunchKernelGGL(ta_merge_kernel<false>, grid, dim3(GEN_THREADS), smem, stream, p);
    }
    return hipGetLastError();
}

// Stand-alone tree encoder: one workgroup per request.
__global__ __launch_bounds__(TA_WAVE) void ta_encode_kernel(const int32_t *parent, int64_t par_sb, int T,
                                                            unsigned long long *masks, int32_t *status)
{
    __shared__ unsigned long long sm[TA_MAX_TREE];
    __shared__ int flag;
    __shared__ int par_s[TA_MAX_TREE];
    const int b = blockIdx.x;
    const bool ok = ta_encode_tree(parent + (int64_t)b * par_sb, T, sm, &flag, par_s);
    if (threadIdx.x < T)
        masks[(int64_t)b * T + threadIdx.x] = ok ? sm[threadIdx.x] : 0ull;
    if (!ok && threadIdx.x == 0)
        atomicOr(status, TA_STATUS_BAD_PARENT);
}

hipError_t ta_launch_encode(const int32_t *parent, int64_t par_sb, int B, int T, unsigned long long *masks,
                            int32_t *status, hipStream_t stream)
{
    hipLaunchKernelGGL(ta_encode_kernel, dim3(B), dim3(TA_WAVE), 0, stream, parent, par_sb, T, masks, status);
    return hipGetLastError();
}

// Write-back of the tree tokens' K and V rows (section 3.4, paged KV with tree attention): one workgroup per
// (request, node), threads over (KV head, head-dim element).
template <typename E>
__global__ __launch_bounds__(256) void ta_append_kernel(TAAppend a)
{
    const int b = blockIdx.x, i = blockIdx.y;
    const int L = a.seq_lens[(int64_t)b * a.sl_s];
    if (L < 0 || (int64_t)L + a.T > (int64_t)a.capacity) {
        if (threadIdx.x == 0 && i == 0)
            atomicOr(a.status, TA_STATUS_BAD_SEQLEN);
        return;
    }
    const int pos = L + i;
    int64_t page = b, slot = pos;
    if (a.page_table) {
        page = a.page_table[(int64_t)b * a.pt_sb + pos / a.ps];
        slot = pos % a.ps;
        if (page < 0 || page >= a.n_pages) {               // no such page in the cache: this token is not written
            if (threadIdx.x == 0)
                atomicOr(a.status, TA_STATUS_BAD_PAGE);
            return;
        }
    }
    for (int x = threadIdx.x; x < a.Hkv * a.D; x += blockDim.x) {
        const int g = x / a.D, d = x % a.D;
        ((E *)a.k)[page * a.k_sp + g * a.k_sh + slot * a.k_ss + d] =
            ((const E *)a.k_new)[b * a.kn_sb + i * a.kn_st + g * a.kn_sh + d];
        ((E *)a.v)[page * a.v_sp + g * a.v_sh + slot * a.v_ss + d] =
            ((const E *)a.v_new)[b * a.vn_sb + i * a.vn_st + g * a.vn_sh + d];
    }
}

// Bookkeeping after acceptance (section 3, stage 6): the accepted path's K/V rows move behind the prefix.  One
// workgroup per request.  The rows of one phase -- as many (KV head, K or V) units of n rows as fit the staging
// buffer -- are all read into LDS before any of them is written back, and no two phases touch the same bytes, so
// sources that are also destinations are safe.
constexpr int CP_STAGE_BYTES = 64 * 1024;

template <typename E>
__global__ __launch_bounds__(256) void ta_compact_kernel(TACompact c)
{
    extern __shared__ __attribute__((aligned(16))) char cp_stage[];
    __shared__ int ids[TA_MAX_TREE];
    __shared__ int bad;
    const int b = blockIdx.x, tid = threadIdx.x;
    const int L = c.seq_lens[(int64_t)b * c.sl_s];
    const int n = c.n_accepted[(int64_t)b * c.na_s];
    if (tid == 0)
        bad = 0;
    __syncthreads();
    const bool len_ok = L >= 0 && (int64_t)L + c.T <= (int64_t)c.capacity;
    const bool n_ok = n >= 0 && n <= c.A;
    if (n_ok && tid < n) {
        const int id = c.accepted[(int64_t)b * c.acc_sb + tid];
        ids[tid] = id;
        if (id < 0 || id >= c.T)
            atomicOr(&bad, 1);
    }
    __syncthreads();
    const bool path_ok = n_ok && (bad & 1) == 0;
    // every page a row may come from or go to (positions L .. L+T-1) must be a page of the cache
    if (len_ok && c.page_table && tid < c.T) {
        const int id = c.page_table[(int64_t)b * c.pt_sb + (L + tid) / c.ps];
        if (id < 0 || id >= c.n_pages)
            atomicOr(&bad, 2);
    }
    __syncthreads();
    const bool pages_ok = (bad & 2) == 0;
    if (!len_ok || !path_ok || !pages_ok) {
        if (tid == 0) {
            atomicOr(c.status, !len_ok ? TA_STATUS_BAD_SEQLEN : !path_ok ? TA_STATUS_BAD_PATH : TA_STATUS_BAD_PAGE);
            if (c.seq_lens_out)
                c.seq_lens_out[(int64_t)b * c.slo_s] = L;
        }
        return;
    }
    E *stage = (E *)cp_stage;
    const int unit = n * c.D;                                      // elements of one (KV head, K or V) unit
    const int units = 2 * c.Hkv;
    const int per_phase = unit > 0 ? max(1, (int)(CP_STAGE_BYTES / sizeof(E)) / unit) : units;
    for (int u0 = 0; u0 < units && unit > 0; u0 += per_phase) {
        const int nu = min(per_phase, units - u0);
        for (int pass = 0; pass < 2; ++pass) {                     // 0: cache -> LDS (sources), 1: LDS -> cache
            for (int x = tid; x < nu * unit; x += blockDim.x) {
                const int u = u0 + x / unit, r = x % unit;
                const int j = r / c.D, d = r % c.D;
                const int g = u >> 1;
                const int pos = L + (pass == 0 ? ids[j] : j);
                int64_t page = b, slot = pos;
                if (c.page_table) {
                    page = c.page_table[(int64_t)b * c.pt_sb + pos / c.ps];
                    slot = pos % c.ps;
                }
                E *row = (u & 1) ? (E *)c.v + page * c.v_sp + g * c.v_sh + slot * c.v_ss
                                 : (E *)c.k + page * c.k_sp + g * c.k_sh + slot * c.k_ss;
                if (pass == 0)
                    stage[x] = row[d];
                else
                    row[d] = stage[x];
            }
            __syncthreads();
        }
    }
    if (tid == 0 && c.seq_lens_out)
        c.seq_lens_out[(int64_t)b * c.slo_s] = L + n;
}

hipError_t ta_launch_compact(const TACompact &c, hipStream_t stream, int dev)
{
    // staging: one phase holds at most CP_STAGE_BYTES; a single unit (A rows of D elements) never exceeds that
    const size_t unit_bytes = (size_t)c.A * c.D * c.elem_bytes;
    if (unit_bytes > (size_t)CP_STAGE_BYTES)
        return hipErrorInvalidValue;
    const size_t smem = CP_STAGE_BYTES;                            // with the static part just above the 64 KB default
    static bool attr_set[64] = {};
    if (dev < 0 || dev >= 64)
        return hipErrorInvalidDevice;
    if (!attr_set[dev]) {
        for (const void *fn : {(const void *)ta_compact_kernel<uint16_t>, (const void *)ta_compact_kernel<uint32_t>}) {
            hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            if (e != hipSuccess)
                return e;
        }
        attr_set[dev] = true;
    }
    if (c.elem_bytes == 2)
        hipLaunchKernelGGL(ta_compact_kernel<uint16_t>, dim3(c.B), dim3(256), smem, stream, c);
    else
        hipLaunchKernelGGL(ta_compact_kernel<uint32_t>, dim3(c.B), dim3(256), smem, stream, c);
    return hipGetLastError();
}

hipError_t ta_launch_append(const TAAppend &a, hipStream_t stream)
{
    if (a.elem_bytes == 2)
        hipLaunchKernelGGL(ta_append_kernel<uint16_t>, dim3(a.B, a.T), dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL(ta_append_kernel<uint32_t>, dim3(a.B, a.T), dim3(256), 0, stream, a);
    return hipGetLastError();
}

// Measurement aid: a plain streaming read.  Every workgroup walks its contiguous part of the buffer with four
// 16-byte non-temporal loads per lane in flight, the access pattern of a KV scan without any arithmetic behind it.
__global__ __launch_bounds__(512) void ta_stream_read_kernel(const uint4 *__restrict__ src, size_t n_vec, unsigned *sink)
{
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    const size_t per = (n_vec + gridDim.x - 1) / gridDim.x;
    const size_t lo = (size_t)blockIdx.x * per, hi = lo + per < n_vec ? lo + per : n_vec;
    unsigned acc = 0;
    size_t i = lo + threadIdx.x;
    for (; i + 3 * 512 < hi; i += 4 * 512) {
        u32x4_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            v[u] = __builtin_nontemporal_load((const u32x4_t *)(src + i + u * 512));
#pragma unroll
        for (int u = 0; u < 4; ++u)
            acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < hi; i += 512) {
        const u32x4_t v = __builtin_nontemporal_load((const u32x4_t *)(src + i));
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x9e3779b9u)            // practically never: keeps the loads alive without a store per lane
        *sink = acc;
}

// Measurement aid: nothing but dependent-free chains of v_mfma_f32_32x32x16_bf16 on registers, eight waves per compute
// unit -- the matrix-core rate this device sustains under its power limit, against which the KV pass's rate is set
// beside the published peak.  Each wave issues 32 * iters matrix instructions (32768 flop each per wave).
__global__ __launch_bounds__(512) void ta_mfma_probe_kernel(int iters, float *sink)
{
    typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
    typedef float f32x16_t __attribute__((ext_vector_type(16)));
    f32x16_t acc[4];
    bf16x8_t a, b;
    // operands with the bit patterns of real data (a hash of the lane: values in (-2, 2)); matrix cores fed with
    // zeros and ones draw far less power and would show a rate no real kernel sees
    uint32_t h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    for (int i = 0; i < 8; ++i) {
        h = h * 1664525u + 1013904223u;
        a[i] = (__bf16)((float)(int)(h >> 8 & 0xffff) * (1.f / 16384.f) - 2.f);
        h = h * 1664525u + 1013904223u;
        b[i] = (__bf16)((float)(int)(h >> 8 & 0xffff) * (1.f / 16384.f) - 2.f);
    }
    for (int k = 0; k < 4; ++k)
        for (int i = 0; i < 16; ++i)
            acc[k][i] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 32; ++r)
            acc[r & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[r & 3], 0, 0, 0);
    }
    float x = 0.f;
    for (int k = 0; k < 4; ++k)
        for (int i = 0; i < 16; ++i)
            x += acc[k][i];
    if (x == 1.2345678f)               // practically never: keeps the results alive without a store per lane
        *sink = x;
}

hipError_t ta_launch_mfma_probe(int iters, void *sink, int num_cus, hipStream_t stream)
{
    hipLaunchKernelGGL(ta_mfma_probe_kernel, dim3(num_cus), dim3(512), 0, stream, iters, (float *)sink);
    return hipGetLastError();
}

hipError_t ta_launch_stream_read(const void *buf, size_t bytes, void *sink, int num_cus, hipStream_t stream)
{
    const int wgs = num_cus * 4;
    hipLaunchKernelGGL(ta_stream_read_kernel, dim3(wgs), dim3(512), 0, stream, (const uint4 *)buf, bytes / 16,
                       (unsigned *)sink);
    return hipGetLastError();
}
