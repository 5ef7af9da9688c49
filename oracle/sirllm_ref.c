/*
 * sirllm_ref.c -- CPU oracle of the SirLLM retention step.  TEST INFRASTRUCTURE ONLY:
 * called by the tests, the smoke check and the benchmark's CPU-baseline leg, never by the
 * product path.  Plain C, host memory, double-precision accumulation, no blocking, no
 * fusion: each function is the definition in the paper written out.
 *
 * Readings taken where the paper leaves a choice (each is checked by a test):
 *   - "token entropy" is the printed formula, the surprisal of the token that occurred
 *     (Sec. 3.2), not the Shannon entropy of the row; natural logarithm.
 *   - index sets are 0-based and half open: sinks [0, n_sink), recent [n_cand-n_recent, n_cand)
 *     (Sec. 3.1 prints n_sink+1 indices, but Sec. 4.1 fixes the sink size at 4 and the worked
 *     example of Sec. 3.3 has sinks 0,1,2,3).
 *   - Top_k runs over the slots that are neither sink nor recent, so the three sets are
 *     disjoint and the cache holds exactly the budget after an eviction.
 *   - kept slots are listed in ascending slot order (Sec. 3.3's example is ascending).
 *   - "E <- E + E_t" in Algorithm 1 appends; the decay multiplies only the scores that were
 *     already held when the turn began (new scores enter the selection undecayed).
 *   - the eviction trigger is "n_cand > budget" (Algorithm 1: cache size > L).
 *   - equal scores: the lower slot wins.
 *
 * Parity status: every function below is pinned by tests/test_oracle_*.py against closed
 * forms, library routines, brute force and the paper's worked example.  What is NOT pinned:
 * the paper prints no numeric score, kept set or cache content from its experiments, so
 * agreement with the authors' own runs is "parity unpinned".
 */
#include "sirllm_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

static int g_threads = 1;

int sirllm_ref_set_threads(int n)
{
    if (n < 1) n = 1;
#ifdef _OPENMP
    g_threads = n;
#else
    g_threads = 1;
#endif
    return g_threads;
}

int sirllm_ref_get_threads(void) { return g_threads; }

/* ------------------------------------------------------------------------------------ */
/* Sec. 3.2:  e = -log P(x) = logsumexp(z) - z[x]                                        */
/* ------------------------------------------------------------------------------------ */

static double logit_at(const void* logits, int dtype, int64_t index)
{
    if (dtype == SIRLLM_REF_F32)
        return (double)((const float*)logits)[index];
    if (dtype == SIRLLM_REF_BF16) {
        /* bfloat16 is the top half of a binary32 */
        uint32_t bits = (uint32_t)((const uint16_t*)logits)[index] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
    /* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits */
    const uint16_t h = ((const uint16_t*)logits)[index];
    const int sign = h >> 15, expo = (h >> 10) & 31, frac = h & 1023;
    double mag;
    if (expo == 31) mag = frac ? (double)NAN : (double)INFINITY;
    else if (expo == 0) mag = ldexp((double)frac, -24);              /* subnormal: frac * 2^-10 * 2^-14 */
    else mag = ldexp(1.0 + frac / 1024.0, expo - 15);
    return sign ? -mag : mag;
}

int sirllm_ref_score(const void* logits, int dtype, int64_t n_rows, int32_t vocab, int64_t ld,
                     const int32_t* token_ids, float* scores_out)
{
    if (n_rows < 0 || vocab < 1 || ld < vocab) return -1;
    if (dtype != SIRLLM_REF_F32 && dtype != SIRLLM_REF_BF16 && dtype != SIRLLM_REF_F16) return -1;
    if (n_rows == 0) return 0;
    if (!logits || !token_ids || !scores_out) return -1;

    int64_t r;
#ifdef _OPENMP
#pragma omp parallel for num_threads(g_threads) schedule(static)
#endif
    for (r = 0; r < n_rows; ++r) {
        const int64_t base = r * ld;
        const int32_t tok = token_ids[r];
        if (tok < 0 || tok >= vocab) {          /* no such token: no probability to take the log of */
            scores_out[r] = (float)NAN;
            continue;
        }
        double m = -INFINITY;
        for (int32_t v = 0; v < vocab; ++v) {
            double z = logit_at(logits, dtype, base + v);
            if (z > m) m = z;
        }
        double s = 0.0;
        for (int32_t v = 0; v < vocab; ++v)
            s += exp(logit_at(logits, dtype, base + v) - m);
        double e = (m - logit_at(logits, dtype, base + tok)) + log(s);
        scores_out[r] = (float)e;
    }
    return 0;
}

/* ------------------------------------------------------------------------------------ */
/* Sec. 3.2 with the logits written out as the language-model head's product:             */
/* z[r][v] = sum_k h[r][k] * W[v][k]  (the model's last linear layer, no bias), then the   */
/* same e = logsumexp(z[r]) - z[r][x_r].  Inputs are widened exactly, products and sums    */
/* are taken in double in index order, nothing is rounded before the final score.          */
/* ------------------------------------------------------------------------------------ */

int sirllm_ref_lmhead_score(const void* hidden, int64_t ld_h, const void* weight, int64_t ld_w, int dtype,
                            int32_t d_model, int64_t n_rows, int32_t vocab,
                            const int32_t* token_ids, float* scores_out)
{
    if (n_rows < 0 || vocab < 1 || d_model < 1 || ld_h < d_model || ld_w < d_model) return -1;
    if (dtype != SIRLLM_REF_F32 && dtype != SIRLLM_REF_BF16 && dtype != SIRLLM_REF_F16) return -1;
    if (n_rows == 0) return 0;
    if (!hidden || !weight || !token_ids || !scores_out) return -1;

    int failed = 0;
    int64_t r;
#ifdef _OPENMP
#pragma omp parallel for num_threads(g_threads) schedule(dynamic, 1)
#endif
    for (r = 0; r < n_rows; ++r) {
        const int32_t tok = token_ids[r];
        if (tok < 0 || tok >= vocab) {
            scores_out[r] = (float)NAN;
            continue;
        }
        double* h = (double*)malloc(sizeof(double) * (size_t)d_model);
        double* z = (double*)malloc(sizeof(double) * (size_t)vocab);
        if (!h || !z) {
            free(h);
            free(z);
            failed = 1;
            continue;
        }
        for (int32_t k = 0; k < d_model; ++k) h[k] = logit_at(hidden, dtype, r * ld_h + k);
        for (int32_t v = 0; v < vocab; ++v) {
            double acc = 0.0;
            for (int32_t k = 0; k < d_model; ++k)
                acc += h[k] * logit_at(weight, dtype, (int64_t)v * ld_w + k);
            z[v] = acc;
        }
        double m = -INFINITY;
        for (int32_t v = 0; v < vocab; ++v)
            if (z[v] > m) m = z[v];
        double s = 0.0;
        for (int32_t v = 0; v < vocab; ++v) s += exp(z[v] - m);
        scores_out[r] = (float)((m - z[tok]) + log(s));
        free(h);
        free(z);
    }
    return failed ? -1 : 0;
}

/* ------------------------------------------------------------------------------------ */
/* Sec. 3.3 / 3.1: decay, Top_k, sink and recent sets                                     */
/* ------------------------------------------------------------------------------------ */

typedef struct { float score; int32_t slot; } scored_slot;

/* -1: x is a NaN with the sign bit set, +1: a NaN with it clear, 0: a number */
static int nan_class(float x)
{
    if (x == x) return 0;
    return signbit(x) ? -1 : 1;
}

/* >0 when a ranks above b, <0 when below, 0 when they tie.  Numbers by IEEE comparison
 * (+0 ties with -0).  NaNs have no IEEE order, so they are placed by bit pattern: sign-clear
 * NaNs above everything, sign-set NaNs below everything, and within a class in the order
 * their magnitude bits would have if they were numbers of that sign. */
static int rank_cmp(float a, float b)
{
    int ca = nan_class(a), cb = nan_class(b);
    if (ca == 0 && cb == 0) return (a > b) - (a < b);
    if (ca != cb) return (ca > cb) - (ca < cb);
    uint32_t ua, ub;
    memcpy(&ua, &a, 4);
    memcpy(&ub, &b, 4);
    ua &= 0x7fffffffu;
    ub &= 0x7fffffffu;
    int mag = (ua > ub) - (ua < ub);
    return ca > 0 ? mag : -mag;
}

/* qsort order: higher score first; among equals the lower slot first */
static int by_score_then_slot(const void* pa, const void* pb)
{
    const scored_slot* a = (const scored_slot*)pa;
    const scored_slot* b = (const scored_slot*)pb;
    int c = rank_cmp(a->score, b->score);
    if (c != 0) return -c;
    return (a->slot > b->slot) - (a->slot < b->slot);
}

static int policy_ok(const sirllm_ref_policy* p)
{
    return p && p->n_sink >= 0 && p->n_topk >= 0 && p->n_recent >= 0;
}

int sirllm_ref_decay_select(const float* scores, int64_t scores_stride,
                            int32_t n_streams, int32_t n_held, int32_t n_new,
                            const sirllm_ref_policy* policy,
                            int32_t* kept_idx, int64_t idx_stride,
                            float* scores_out, int64_t out_stride)
{
    if (n_streams < 0 || n_held < 0 || n_new < 0 || !policy_ok(policy)) return -1;
    const int64_t n_cand = (int64_t)n_held + n_new;
    const int64_t budget = (int64_t)policy->n_sink + policy->n_topk + policy->n_recent;
    if (n_streams == 0 || n_cand == 0) return 0;
    if (!scores || !kept_idx || !scores_out) return -1;
    const float eta = policy->decay;

    for (int32_t s = 0; s < n_streams; ++s) {
        const float* E_in = scores + (int64_t)s * scores_stride;
        int32_t* idx = kept_idx + (int64_t)s * idx_stride;
        float* E_out = scores_out + (int64_t)s * out_stride;

        /* E: the entropy cache after "append" and "decay" */
        float* E = (float*)malloc((size_t)n_cand * sizeof(float));
        char* keep = (char*)calloc((size_t)n_cand, 1);
        if (!E || !keep) { free(E); free(keep); return -1; }
        for (int64_t i = 0; i < n_cand; ++i) {
            if (i < n_held) {
                volatile float prod = E_in[i] * eta;   /* one binary32 multiply, rounded to nearest even */
                E[i] = prod;
            } else {
                E[i] = E_in[i];
            }
        }

        if (n_cand <= budget) {
            for (int64_t i = 0; i < n_cand; ++i) keep[i] = 1;       /* trigger not reached */
        } else {
            const int64_t mid_lo = policy->n_sink;
            const int64_t mid_hi = n_cand - policy->n_recent;
            for (int64_t i = 0; i < mid_lo; ++i) keep[i] = 1;        /* Id_sink   */
            for (int64_t i = mid_hi; i < n_cand; ++i) keep[i] = 1;   /* Id_recent */
            const int64_t n_mid = mid_hi - mid_lo;
            scored_slot* mid = (scored_slot*)malloc((size_t)(n_mid > 0 ? n_mid : 1) * sizeof(scored_slot));
            if (!mid) { free(E); free(keep); return -1; }
            for (int64_t i = 0; i < n_mid; ++i) {
                mid[i].score = E[mid_lo + i];
                mid[i].slot = (int32_t)(mid_lo + i);
            }
            qsort(mid, (size_t)n_mid, sizeof(scored_slot), by_score_then_slot);
            for (int64_t i = 0; i < policy->n_topk; ++i) keep[mid[i].slot] = 1;   /* Id_entropy */
            free(mid);
        }

        int64_t j = 0;
        for (int64_t i = 0; i < n_cand; ++i) {
            if (keep[i]) {
                idx[j] = (int32_t)i;
                E_out[j] = E[i];
                ++j;
            }
        }
        free(E);
        free(keep);
    }
    return 0;
}

/* ------------------------------------------------------------------------------------ */
/* Sec. 4.1: the baseline policies (StreamLLM, IntervalLLM, RandomLLM)                    */
/* ------------------------------------------------------------------------------------ */

/* One round: two 32x32 -> 64 bit products, the high halves are mixed with the other counter
 * words and the round key, the low halves pass through; the key then steps by the Weyl constants. */
void sirllm_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

typedef struct { uint32_t key; int32_t slot; } keyed_slot;

static int by_key_then_slot(const void* pa, const void* pb)
{
    const keyed_slot* a = (const keyed_slot*)pa;
    const keyed_slot* b = (const keyed_slot*)pb;
    if (a->key != b->key) return a->key > b->key ? -1 : 1;      /* larger key first */
    return (a->slot > b->slot) - (a->slot < b->slot);
}

int sirllm_ref_baseline_select(int kind, int32_t n_streams, int32_t n_cand, const sirllm_ref_policy* policy,
                               uint64_t seed, uint64_t turn, int32_t* kept_idx, int64_t idx_stride,
                               int32_t* n_keep_out)
{
    if (kind < 0 || kind > 2 || n_streams < 0 || n_cand < 0 || !policy_ok(policy)) return -1;
    const int64_t k = kind == 0 ? 0 : policy->n_topk;
    const int64_t budget = (int64_t)policy->n_sink + k + policy->n_recent;
    const int64_t n_keep = n_cand < budget ? n_cand : budget;
    if (n_keep_out) *n_keep_out = (int32_t)n_keep;
    if (n_streams == 0 || n_cand == 0) return 0;
    if (!kept_idx) return -1;

    for (int32_t s = 0; s < n_streams; ++s) {
        int32_t* idx = kept_idx + (int64_t)s * idx_stride;
        char* keep = (char*)calloc((size_t)n_cand, 1);
        if (!keep) return -1;
        if (n_cand <= budget) {
            for (int64_t i = 0; i < n_cand; ++i) keep[i] = 1;
        } else {
            const int64_t mid_lo = policy->n_sink, mid_hi = n_cand - policy->n_recent;
            const int64_t M = mid_hi - mid_lo;
            for (int64_t i = 0; i < mid_lo; ++i) keep[i] = 1;
            for (int64_t i = mid_hi; i < n_cand; ++i) keep[i] = 1;
            if (kind == 1 && k > 0) {
                int64_t interval = M / k;
                if (interval < 1) interval = 1;
                for (int64_t j = 0; j < k; ++j) keep[mid_hi - 1 - j * interval] = 1;
            } else if (kind == 2 && k > 0) {
                keyed_slot* mid = (keyed_slot*)malloc((size_t)M * sizeof(keyed_slot));
                if (!mid) { free(keep); return -1; }
                const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
                for (int64_t i = 0; i < M; ++i) {
                    const uint32_t ctr[4] = {(uint32_t)(mid_lo + i), (uint32_t)s, (uint32_t)turn, (uint32_t)(turn >> 32)};
                    uint32_t r[4];
                    sirllm_ref_philox4x32_10(ctr, key, r);
                    mid[i].key = r[0];
                    mid[i].slot = (int32_t)(mid_lo + i);
                }
                qsort(mid, (size_t)M, sizeof(keyed_slot), by_key_then_slot);
                for (int64_t j = 0; j < k; ++j) keep[mid[j].slot] = 1;
                free(mid);
            }
        }
        int64_t j = 0;
        for (int64_t i = 0; i < n_cand; ++i)
            if (keep[i]) idx[j++] = (int32_t)i;
        free(keep);
    }
    return 0;
}

/* ------------------------------------------------------------------------------------ */
/* Sec. 3.3: KV_cache <- KV_cache[Id]                                                    */
/* ------------------------------------------------------------------------------------ */

static int layout_ok(const sirllm_ref_kv_layout* L)
{
    return L && L->n_layers >= 0 && L->n_kv_heads >= 0 && L->head_dim >= 0 && L->elem_bytes > 0 &&
           L->stride_stream >= 0 && L->stride_layer >= 0 && L->stride_head >= 0 && L->stride_pos >= 0;
}

static void gather_one(const char* src, const sirllm_ref_kv_layout* S, int32_t n_src,
                       char* dst, const sirllm_ref_kv_layout* D,
                       const int32_t* kept_idx, int64_t idx_stride, int32_t n_streams, int32_t n_keep)
{
    const size_t row_bytes = (size_t)S->head_dim * (size_t)S->elem_bytes;
    const int64_t planes = (int64_t)n_streams * S->n_layers * S->n_kv_heads;
    int64_t p;
#ifdef _OPENMP
#pragma omp parallel for num_threads(g_threads) schedule(static)
#endif
    for (p = 0; p < planes; ++p) {
        const int64_t h = p % S->n_kv_heads;
        const int64_t l = (p / S->n_kv_heads) % S->n_layers;
        const int64_t s = p / ((int64_t)S->n_kv_heads * S->n_layers);
        const char* sp = src + (size_t)S->elem_bytes * (size_t)(s * S->stride_stream + l * S->stride_layer + h * S->stride_head);
        char* dp = dst + (size_t)D->elem_bytes * (size_t)(s * D->stride_stream + l * D->stride_layer + h * D->stride_head);
        const int32_t* idx = kept_idx + s * idx_stride;
        for (int32_t j = 0; j < n_keep; ++j) {
            char* drow = dp + (size_t)D->elem_bytes * (size_t)((int64_t)j * D->stride_pos);
            const int32_t i = idx[j];
            if (i < 0 || i >= n_src)
                memset(drow, 0, row_bytes);      /* no such slot: defined as an all-zero row */
            else
                memcpy(drow, sp + (size_t)S->elem_bytes * (size_t)((int64_t)i * S->stride_pos), row_bytes);
        }
    }
}

int sirllm_ref_compact_kv(const void* k_src, const void* v_src, const sirllm_ref_kv_layout* src, int32_t n_src,
                          void* k_dst, void* v_dst, const sirllm_ref_kv_layout* dst,
                          const int32_t* kept_idx, int64_t idx_stride,
                          int32_t n_streams, int32_t n_keep)
{
    if (!layout_ok(src) || !layout_ok(dst) || n_streams < 0 || n_keep < 0 || n_src < 0) return -1;
    if (src->n_layers != dst->n_layers || src->n_kv_heads != dst->n_kv_heads ||
        src->head_dim != dst->head_dim || src->elem_bytes != dst->elem_bytes) return -1;
    if (n_streams == 0 || n_keep == 0) return 0;
    if (!k_src || !k_dst || !kept_idx) return -1;
    if ((v_src == NULL) != (v_dst == NULL)) return -1;
    gather_one((const char*)k_src, src, n_src, (char*)k_dst, dst, kept_idx, idx_stride, n_streams, n_keep);
    if (v_src)
        gather_one((const char*)v_src, src, n_src, (char*)v_dst, dst, kept_idx, idx_stride, n_streams, n_keep);
    return 0;
}

/* In place: every plane is first set aside whole, then its kept rows are copied back to the front. */
static int gather_one_inplace(char* buf, const sirllm_ref_kv_layout* S, int32_t n_src,
                              const int32_t* kept_idx, int64_t idx_stride, int32_t n_streams, int32_t n_keep)
{
    const size_t row_bytes = (size_t)S->head_dim * (size_t)S->elem_bytes;
    char* old = (char*)malloc(row_bytes * (size_t)(n_src > 0 ? n_src : 1));
    if (!old) return -1;
    for (int64_t s = 0; s < n_streams; ++s)
        for (int64_t l = 0; l < S->n_layers; ++l)
            for (int64_t h = 0; h < S->n_kv_heads; ++h) {
                char* p = buf + (size_t)S->elem_bytes * (size_t)(s * S->stride_stream + l * S->stride_layer + h * S->stride_head);
                for (int32_t i = 0; i < n_src; ++i)
                    memcpy(old + row_bytes * (size_t)i, p + (size_t)S->elem_bytes * (size_t)((int64_t)i * S->stride_pos), row_bytes);
                const int32_t* idx = kept_idx + s * idx_stride;
                for (int32_t j = 0; j < n_keep; ++j) {
                    char* drow = p + (size_t)S->elem_bytes * (size_t)((int64_t)j * S->stride_pos);
                    if (idx[j] < 0 || idx[j] >= n_src) memset(drow, 0, row_bytes);
                    else memcpy(drow, old + row_bytes * (size_t)idx[j], row_bytes);
                }
            }
    free(old);
    return 0;
}

int sirllm_ref_compact_kv_inplace(void* k, void* v, const sirllm_ref_kv_layout* layout, int32_t n_src,
                                  const int32_t* kept_idx, int64_t idx_stride,
                                  int32_t n_streams, int32_t n_keep)
{
    if (!layout_ok(layout) || n_streams < 0 || n_keep < 0 || n_src < 0 || n_keep > n_src) return -1;
    if (n_streams == 0 || n_keep == 0) return 0;
    if (!k || !kept_idx) return -1;
    int rc = gather_one_inplace((char*)k, layout, n_src, kept_idx, idx_stride, n_streams, n_keep);
    if (rc == 0 && v) rc = gather_one_inplace((char*)v, layout, n_src, kept_idx, idx_stride, n_streams, n_keep);
    return rc;
}

/* ------------------------------------------------------------------------------------ */
/* Algorithm 1, one turn                                                                 */
/* ------------------------------------------------------------------------------------ */

int sirllm_ref_step(const void* logits, int dtype, int32_t vocab, int64_t ld, const int32_t* token_ids,
                    float* scores, int64_t scores_stride,
                    int32_t n_streams, int32_t n_held, int32_t n_new,
                    const sirllm_ref_policy* policy,
                    const void* k_src, const void* v_src, const sirllm_ref_kv_layout* src,
                    void* k_dst, void* v_dst, const sirllm_ref_kv_layout* dst,
                    int32_t* kept_idx, int64_t idx_stride,
                    float* scores_out, int64_t out_stride)
{
    if (n_streams < 0 || n_held < 0 || n_new < 0 || !policy_ok(policy)) return -1;
    const int64_t n_cand = (int64_t)n_held + n_new;
    const int64_t budget = (int64_t)policy->n_sink + policy->n_topk + policy->n_recent;
    if (n_streams == 0 || n_cand == 0) return 0;
    if (!scores) return -1;

    /* E_t = Entropy([I_t, R_t]);  E <- E ++ E_t */
    for (int32_t s = 0; s < n_streams && n_new > 0; ++s) {
        const size_t esz = dtype == SIRLLM_REF_F32 ? 4 : 2;   /* bfloat16 and binary16 are two bytes */
        const char* rows = (const char*)logits + esz * (size_t)((int64_t)s * n_new * ld);
        int rc = sirllm_ref_score(rows, dtype, n_new, vocab, ld, token_ids + (int64_t)s * n_new,
                                  scores + (int64_t)s * scores_stride + n_held);
        if (rc) return rc;
    }
    /* E <- E * eta (held part), Top_k, index list, E <- E[Id] */
    int rc = sirllm_ref_decay_select(scores, scores_stride, n_streams, n_held, n_new, policy,
                                     kept_idx, idx_stride, scores_out, out_stride);
    if (rc) return rc;
    /* KV <- KV[Id], only when the cache is over budget */
    if (n_cand > budget) {
        rc = sirllm_ref_compact_kv(k_src, v_src, src, (int32_t)n_cand, k_dst, v_dst, dst,
                                   kept_idx, idx_stride, n_streams, (int32_t)budget);
        if (rc) return rc;
    }
    return 0;
}
