/*
 * fp64 CPU oracle for tree attention in the verification step of tree-based
 * speculative decoding.  TEST INFRASTRUCTURE ONLY: nothing on the product path
 * may call it; it shares no code with the HIP kernels.
 *
 * What it computes (paper section 3.1 "Tree attention", first paragraph, and
 * section 3.4 "Paged KV with tree attention"): every node of the flattened
 * draft-token tree must produce the attention output it would get if its
 * root-to-node path were unrolled into an ordinary sequence behind the cached
 * context and run as a causal prefill.  So for request b, node i, query head h
 * the key list is
 *
 *     positions 0 .. L_b-1 of the request's cache            (the prefix)
 *     positions L_b + j, for j on the path root -> i, i last (the node's own path)
 *
 * and the result is plain softmax attention of q[b,i,h,:] over that list,
 * evaluated as the textbook definition: all scores, subtract their maximum,
 * exponentiate, normalise, weighted sum of the value rows.  There is no
 * prefix/suffix split, no bitmask, no running softmax and no tiling here; the
 * ancestor set is found by walking parent[] from the node up to a root.
 *
 * Readings the paper leaves open (each also listed in the design notes):
 *   - a node attends to itself (causal attention includes the diagonal);
 *   - every tree node, the root included, is a query and has its K/V in the
 *     cache at logical position L_b + (node id);
 *   - seq_lens[b] = L_b counts the cached prefix only;
 *   - a node with parent < 0 is a root; several roots are allowed;
 *   - query head h reads KV head h / (Hq / Hkv);
 *   - lse is the natural log of the sum of exp of the scaled scores.
 *
 * Data-dependent faults (parent id out of range, a parent cycle, negative
 * L_b, L_b + T beyond the page table) poison the whole request: its out and
 * lse are NaN and the return value counts such requests.
 *
 * Pins (tests that fix this file to something other than itself): chain tree
 * == masked causal attention from a library routine, single node == decode
 * attention, q = 0 closed forms, planted keys, per-head constant V, path
 * unrolling, node relabelling, page permutation, and an independent
 * pure-Python brute force over every tree shape of up to 5 nodes.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC tree_attn_oracle.c -o libtreeattn_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

typedef struct {
    const void *q;            /* [B,T,Hq,D], strides in elements, D contiguous */
    const void *k_cache;      /* [num_pages,Hkv,ps,D] view, strides in elements */
    const void *v_cache;
    int32_t dtype;            /* ORACLE_F32 or ORACLE_BF16 (raw 16-bit patterns) */
    int32_t B, T, Hq, Hkv, D;
    int64_t q_stride[3];      /* b, t, h */
    int64_t k_stride[3];      /* page, head, slot */
    int64_t v_stride[3];
    int32_t page_size;
    int32_t max_pages;        /* page_table row length; contiguous mode: 1 */
    const int32_t *page_table;/* [B,max_pages] or NULL: request b owns page b */
    const int32_t *seq_lens;  /* [B] prefix lengths L_b */
    const int32_t *tree_parent;
    int64_t parent_stride_b;  /* T, or 0 when one tree serves the whole batch */
    double scale;
    int32_t Tq, q_off;        /* q, out and lse hold the Tq nodes q_off .. q_off+Tq-1 of the T-node tree (section 3.1:
                                 the same attention serves the drafting stage, where only the newest nodes are
                                 queries and all nodes so far are keys); Tq = 0 means all T nodes */
    const int32_t *kv_start;  /* [B] or NULL: first prefix position a request's nodes still attend to (section 3.4,
                                 iRoPE for Llama4: the prefix is restricted to the current sub-sequence); NULL = 0 */
} oracle_problem;

static double widen(const void *base, int dtype, int64_t idx)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    /* bf16 is the upper half of an IEEE binary32 */
    uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* Root-to-node path of node i (node ids, root first, i last).  Returns its
 * length, or -1 when parent[] is malformed. */
static int root_path(const int32_t *parent, int T, int i, int32_t *path)
{
    int32_t up[64 + 1];
    int n = 0, cur = i;
    while (cur >= 0) {
        if (cur >= T || n >= T)
            return -1;               /* id out of range, or a cycle */
        up[n++] = cur;
        cur = parent[cur];
    }
    for (int a = 0; a < n; ++a)
        path[a] = up[n - 1 - a];
    return n;
}

static int64_t cache_offset(const oracle_problem *p, const int64_t *stride, int b, int g, int64_t pos)
{
    int64_t page, slot;
    if (p->page_table) {
        page = p->page_table[(int64_t)b * p->max_pages + pos / p->page_size];
        slot = pos % p->page_size;
    } else {
        page = b;
        slot = pos;
    }
    return page * stride[0] + g * stride[1] + slot * stride[2];
}

static int request_is_valid(const oracle_problem *p, int b)
{
    int64_t L = p->seq_lens[b];
    int64_t cap = (int64_t)p->max_pages * p->page_size;
    if (L < 0 || L + p->T > cap)
        return 0;
    if (p->kv_start && (p->kv_start[b] < 0 || p->kv_start[b] > L))
        return 0;
    const int32_t *par = p->tree_parent + b * p->parent_stride_b;
    int32_t path[64];
    for (int i = 0; i < p->T; ++i)
        if (root_path(par, p->T, i, path) < 0)
            return 0;
    return 1;
}

/* One (request, node, head): out_row[D], *lse_out.  `scores` has room for L_b + T doubles. */
static void attend_one(const oracle_problem *p, int b, int i, int h,
                       double *scores, double *out_row, double *lse_out)
{
    const int D = p->D;
    const int g = h / (p->Hq / p->Hkv);
    const int64_t L = p->seq_lens[b];
    const int32_t *par = p->tree_parent + b * p->parent_stride_b;
    int32_t path[64];
    const int plen = root_path(par, p->T, p->q_off + i, path);   /* query i is tree node q_off + i */
    const int64_t S = p->kv_start ? p->kv_start[b] : 0;   /* keys: prefix positions S..L-1, then the path */
    const int64_t W = L - S;
    const int64_t nkeys = W + plen;
    const int64_t qoff = b * p->q_stride[0] + i * p->q_stride[1] + h * p->q_stride[2];

    double smax = -INFINITY;
    for (int64_t t = 0; t < nkeys; ++t) {
        int64_t pos = t < W ? S + t : L + path[t - W];
        int64_t ko = cache_offset(p, p->k_stride, b, g, pos);
        double dot = 0.0;
        for (int d = 0; d < D; ++d)
            dot += widen(p->q, p->dtype, qoff + d) * widen(p->k_cache, p->dtype, ko + d);
        scores[t] = p->scale * dot;
        if (scores[t] > smax)
            smax = scores[t];
    }
    double denom = 0.0;
    for (int64_t t = 0; t < nkeys; ++t) {
        scores[t] = exp(scores[t] - smax);
        denom += scores[t];
    }
    for (int d = 0; d < D; ++d)
        out_row[d] = 0.0;
    for (int64_t t = 0; t < nkeys; ++t) {
        int64_t pos = t < W ? S + t : L + path[t - W];
        int64_t vo = cache_offset(p, p->v_stride, b, g, pos);
        double w = scores[t] / denom;
        for (int d = 0; d < D; ++d)
            out_row[d] += w * widen(p->v_cache, p->dtype, vo + d);
    }
    *lse_out = smax + log(denom);
}

static int check_shapes(const oracle_problem *p)
{
    if (!p || !p->q || !p->k_cache || !p->v_cache || !p->seq_lens || !p->tree_parent)
        return -1;
    if (p->B < 0 || p->T < 1 || p->T > 64 || p->Hq < 1 || p->Hkv < 1 || p->D < 1)
        return -1;
    if (p->Hq % p->Hkv != 0 || p->page_size < 1 || p->max_pages < 1)
        return -1;
    if (p->dtype != ORACLE_F32 && p->dtype != ORACLE_BF16)
        return -1;
    if (p->Tq < 0 || p->q_off < 0 || (p->Tq ? p->Tq : p->T) + p->q_off > p->T)
        return -1;
    return 0;
}

/* Selected outputs: triples[n][3] = (b, node, head); out[n][D], lse[n].
 * Returns the number of triples that fall in poisoned requests, or -1 on bad arguments. */
int tree_attn_oracle_sample(const oracle_problem *p, const int32_t *triples, int64_t n,
                            double *out, double *lse)
{
    if (check_shapes(p) || (n > 0 && (!triples || !out || !lse)))
        return -1;
    int64_t maxL = 0;
    for (int b = 0; b < p->B; ++b)
        if (p->seq_lens[b] > maxL)
            maxL = p->seq_lens[b];
    int poisoned = 0;
#pragma omp parallel reduction(+ : poisoned)
    {
        double *scores = (double *)malloc(sizeof(double) * (size_t)(maxL + p->T + 1));
#pragma omp for schedule(dynamic, 1)
        for (int64_t s = 0; s < n; ++s) {
            int b = triples[3 * s], i = triples[3 * s + 1], h = triples[3 * s + 2];
            double *row = out + s * p->D;
            if (b < 0 || b >= p->B || i < 0 || i >= (p->Tq ? p->Tq : p->T) || h < 0 || h >= p->Hq ||
                !request_is_valid(p, b)) {
                for (int d = 0; d < p->D; ++d)
                    row[d] = NAN;
                lse[s] = NAN;
                poisoned += 1;
                continue;
            }
            attend_one(p, b, i, h, scores, row, &lse[s]);
        }
        free(scores);
    }
    return poisoned;
}

/* Every output: out[B,Tq,Hq,D], lse[B,Hq,Tq] (both dense, fp64).
 * Returns the number of poisoned requests, or -1 on bad arguments. */
int tree_attn_oracle(const oracle_problem *p, double *out, double *lse)
{
    if (check_shapes(p) || !out || !lse)
        return -1;
    int64_t maxL = 0;
    int poisoned = 0;
    for (int b = 0; b < p->B; ++b) {
        if (p->seq_lens[b] > maxL)
            maxL = p->seq_lens[b];
        if (!request_is_valid(p, b))
            poisoned += 1;
    }
    const int Tq = p->Tq ? p->Tq : p->T;                 /* rows of q, out and lse per request */
    const int64_t per_b = (int64_t)p->Hq * Tq;
    const int64_t total = per_b * p->B;
#pragma omp parallel
    {
        double *scores = (double *)malloc(sizeof(double) * (size_t)(maxL + p->T + 1));
#pragma omp for schedule(dynamic, 1)
        for (int64_t w = 0; w < total; ++w) {
            int b = (int)(w / per_b);
            int h = (int)((w % per_b) / Tq);
            int i = (int)(w % Tq);
            double *row = out + (((int64_t)b * Tq + i) * p->Hq + h) * p->D;
            double *l = lse + ((int64_t)b * p->Hq + h) * Tq + i;
            if (!request_is_valid(p, b)) {
                for (int d = 0; d < p->D; ++d)
                    row[d] = NAN;
                *l = NAN;
                continue;
            }
            attend_one(p, b, i, h, scores, row, l);
        }
        free(scores);
    }
    return poisoned;
}

int tree_attn_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
