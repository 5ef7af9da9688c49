/* Drives the CPU oracle through its awkward corners in a build with AddressSanitizer and
 * UndefinedBehaviorSanitizer (tests/test_oracle_sanitizers.py compiles oracle/sirllm_ref.c together with this
 * file).  Every buffer is allocated at exactly the size the call may touch, so a read or write one element beyond
 * it is reported.  The checks of values are few on purpose -- the pins live in the other oracle tests -- but each
 * call's result is looked at, so that nothing is optimised away.  Prints "SANITIZED OK" and exits 0. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "sirllm_ref.h"

#define CHECK(cond)                                                              \
    do {                                                                         \
        if (!(cond)) { fprintf(stderr, "line %d: %s\n", __LINE__, #cond); exit(2); } \
    } while (0)

static uint32_t lcg_state = 12345u;
static uint32_t lcg(void) { lcg_state = lcg_state * 1664525u + 1013904223u; return lcg_state >> 8; }
static float frand(void) { return (float)(lcg() % 10000) / 1000.0f; }

/* element count a layout with n_pos slots touches, from the base pointer */
static int64_t extent(const sirllm_ref_kv_layout* L, int n_streams, int n_pos)
{
    return (int64_t)(n_streams - 1) * L->stride_stream + (int64_t)(L->n_layers - 1) * L->stride_layer +
           (int64_t)(L->n_kv_heads - 1) * L->stride_head + (int64_t)(n_pos - 1) * L->stride_pos + L->head_dim;
}

static void score_cases(void)
{
    /* padded rows (ld > vocab), all three element types, vocab = 1, a token at the last column, non-finite logits */
    const int n_rows = 5, vocab = 37, ld = 41;
    float* z = malloc(sizeof(float) * ((n_rows - 1) * ld + vocab));          /* the last row has no padding behind it */
    uint16_t* zb = malloc(sizeof(uint16_t) * ((n_rows - 1) * ld + vocab));
    int32_t tok[5] = {0, 36, 5, 36, 1};
    float out[5];
    for (int r = 0; r < n_rows; ++r)
        for (int v = 0; v < (r == n_rows - 1 ? vocab : ld); ++v) {
            z[r * ld + v] = v < vocab ? frand() - 5.0f : 1.0e30f;
            union { float f; uint32_t u; } c = {z[r * ld + v]};
            zb[r * ld + v] = (uint16_t)(c.u >> 16);
        }
    z[2 * ld + 3] = -INFINITY;
    z[3 * ld + 36] = -INFINITY;                                               /* the token's own logit: +inf score */
    CHECK(sirllm_ref_score(z, SIRLLM_REF_F32, n_rows, vocab, ld, tok, out) == 0);
    CHECK(isfinite(out[0]) && out[0] > 0 && isinf(out[3]));
    CHECK(sirllm_ref_score(zb, SIRLLM_REF_BF16, n_rows, vocab, ld, tok, out) == 0);
    CHECK(isfinite(out[1]));
    uint16_t one_h[3] = {0x3c00, 0x3c00, 0x3c00};                             /* binary16 1.0, vocab = 1, three rows */
    int32_t t0[3] = {0, 0, 0};
    CHECK(sirllm_ref_score(one_h, SIRLLM_REF_F16, 3, 1, 1, t0, out) == 0 && out[0] == 0.0f);
    CHECK(sirllm_ref_score(z, SIRLLM_REF_F32, 0, vocab, ld, tok, out) == 0);  /* no rows */
    int32_t bad[5] = {-1, 37, 1 << 30, 0, 0};                                /* ids with no column must not be read */
    CHECK(sirllm_ref_score(z, SIRLLM_REF_F32, n_rows, vocab, ld, bad, out) == 0 && isnan(out[0]) && isnan(out[1]) && isnan(out[2]));
    free(z); free(zb);
}

static void lmhead_cases(void)
{
    /* padded leading dimensions; the last rows end exactly with their d_model elements */
    const int n_rows = 3, vocab = 11, d = 8, ld_h = 10, ld_w = 9;
    uint16_t* h = malloc(sizeof(uint16_t) * ((n_rows - 1) * ld_h + d));
    uint16_t* w = malloc(sizeof(uint16_t) * ((vocab - 1) * ld_w + d));
    for (int i = 0; i < (n_rows - 1) * ld_h + d; ++i) h[i] = (uint16_t)(0x3f80 + (lcg() % 64));   /* bfloat16 around 1 */
    for (int i = 0; i < (vocab - 1) * ld_w + d; ++i) w[i] = (uint16_t)(0x3e80 + (lcg() % 64));
    int32_t tok[3] = {0, 10, 4};
    float out[3];
    CHECK(sirllm_ref_lmhead_score(h, ld_h, w, ld_w, SIRLLM_REF_BF16, d, n_rows, vocab, tok, out) == 0);
    CHECK(isfinite(out[0]) && isfinite(out[1]) && isfinite(out[2]));
    free(h); free(w);
}

static void select_cases(void)
{
    /* strided score rows and outputs of exactly the needed size; k = 0, M = k + 1, n_recent = 0, no sinks,
       under budget, NaNs and signed zeros, n_new = 0, n_held = 0 */
    const struct { int n_streams, n_held, n_new, sink, k, recent; } cases[] = {
        {2, 40, 10, 4, 0, 6}, {1, 30, 11, 4, 36, 0}, {3, 17, 5, 0, 7, 0}, {2, 10, 5, 4, 20, 8},
        {1, 50, 0, 4, 20, 8}, {2, 0, 33, 2, 9, 3}, {1, 1, 0, 1, 0, 0}, {1, 64, 64, 0, 127, 0},
    };
    for (unsigned c = 0; c < sizeof(cases) / sizeof(cases[0]); ++c) {
        const int S = cases[c].n_streams, n_cand = cases[c].n_held + cases[c].n_new;
        const int budget = cases[c].sink + cases[c].k + cases[c].recent;
        const int n_keep = n_cand < budget ? n_cand : budget;
        const int64_t ss = n_cand + 3, is = n_keep + 1, os = n_keep + 2;
        float* E = malloc(sizeof(float) * ((S - 1) * ss + n_cand));
        int32_t* idx = malloc(sizeof(int32_t) * ((S - 1) * is + n_keep + (n_keep == 0)));
        float* Eo = malloc(sizeof(float) * ((S - 1) * os + n_keep + (n_keep == 0)));
        for (int64_t i = 0; i < (S - 1) * ss + n_cand; ++i) E[i] = (float)(lcg() % 7) / 2.0f;
        if (n_cand > 9) {
            union { uint32_t u; float f; } q = {0x7fc00000u}, m = {0xffc00000u};
            E[2] = q.f; E[5] = m.f; E[7] = -0.0f; E[8] = 0.0f; E[9] = INFINITY;
        }
        sirllm_ref_policy p = {cases[c].sink, cases[c].k, cases[c].recent, 0.75f};
        CHECK(sirllm_ref_decay_select(E, ss, S, cases[c].n_held, cases[c].n_new, &p, idx, is, Eo, os) == 0);
        for (int s = 0; s < S; ++s)
            for (int j = 1; j < n_keep; ++j) CHECK(idx[s * is + j] > idx[s * is + j - 1] && idx[s * is + j] < n_cand);
        free(E); free(idx); free(Eo);
    }
}

static void baseline_cases(void)
{
    for (int kind = 0; kind < 3; ++kind) {
        const int S = 2, n_cand = 300;
        sirllm_ref_policy p = {4, 100, 16, 0.0f};
        const int n_keep = kind == 0 ? 20 : 120;
        int32_t* idx = malloc(sizeof(int32_t) * ((S - 1) * (n_keep + 5) + n_keep));
        int32_t got = -1;
        CHECK(sirllm_ref_baseline_select(kind, S, n_cand, &p, 0x123456789abcdefULL, 77, idx, n_keep + 5, &got) == 0 && got == n_keep);
        for (int j = 1; j < n_keep; ++j) CHECK(idx[j] > idx[j - 1] && idx[j] < n_cand);
        free(idx);
        int32_t small[10];
        sirllm_ref_policy q = {4, 20, 8, 0.0f};
        CHECK(sirllm_ref_baseline_select(kind, 1, 10, &q, 1, 2, small, 10, &got) == 0 && got == 10);   /* under budget */
    }
}

static void gather_cases(void)
{
    /* padded heads, slots and channels on both sides, n_src below what is allocated, indices without a source slot,
       V absent; buffers end exactly where the layouts end */
    const int S = 2, L = 2, H = 3, D = 5, n_src = 9, n_keep = 6;
    sirllm_ref_kv_layout src = {L, H, D, 2, 0, 0, 0, 0}, dst = {L, H, D, 2, 0, 0, 0, 0};
    src.stride_pos = D + 2; src.stride_head = (n_src + 1) * src.stride_pos; src.stride_layer = (H + 1) * src.stride_head;
    src.stride_stream = L * src.stride_layer + 7;
    dst.stride_pos = D; dst.stride_head = n_keep * D + 1; dst.stride_layer = H * dst.stride_head; dst.stride_stream = L * dst.stride_layer;
    const int64_t ne_src = extent(&src, S, n_src), ne_dst = extent(&dst, S, n_keep);
    uint16_t *ks = malloc(2 * ne_src), *vs = malloc(2 * ne_src), *kd = malloc(2 * ne_dst), *vd = malloc(2 * ne_dst);
    for (int64_t i = 0; i < ne_src; ++i) { ks[i] = (uint16_t)lcg(); vs[i] = (uint16_t)lcg(); }
    memset(kd, 0x77, 2 * ne_dst); memset(vd, 0x77, 2 * ne_dst);
    int32_t kept[2][8] = {{0, 3, 8, 9, -1, 5, 0, 0}, {1, 2, 2147483647, 4, 7, 8, 0, 0}};     /* 9, -1, 2^31-1: no such slot */
    CHECK(sirllm_ref_compact_kv(ks, vs, &src, n_src, kd, vd, &dst, &kept[0][0], 8, S, n_keep) == 0);
    CHECK(kd[0] == ks[0] && kd[3 * D] == 0);                                                   /* row 3 of stream 0 is a zero row */
    CHECK(sirllm_ref_compact_kv(ks, NULL, &src, n_src, kd, NULL, &dst, &kept[0][0], 8, S, n_keep) == 0);
    CHECK(sirllm_ref_compact_kv(ks, vs, &src, n_src, kd, vd, &dst, &kept[0][0], 8, S, 0) == 0);   /* nothing kept */
    /* in place: ascending lists, n_keep = n_src - 1 (everything shifts by one behind the first hole), all kept,
       and a list with slots that do not exist */
    int32_t asc[2][8] = {{0, 1, 2, 4, 5, 6, 7, 8}, {1, 2, 3, 4, 5, 6, 7, 8}};
    CHECK(sirllm_ref_compact_kv_inplace(ks, vs, &src, n_src, &asc[0][0], 8, S, n_src - 1) == 0);
    int32_t all[2][9];
    for (int s = 0; s < 2; ++s) for (int j = 0; j < 9; ++j) all[s][j] = j;
    CHECK(sirllm_ref_compact_kv_inplace(ks, NULL, &src, n_src, &all[0][0], 9, S, n_src) == 0);
    int32_t holes[2][4] = {{2, 5, 9, 100}, {0, 8, 2147483647, 2147483647}};
    CHECK(sirllm_ref_compact_kv_inplace(ks, vs, &src, n_src, &holes[0][0], 4, S, 4) == 0);
    free(ks); free(vs); free(kd); free(vd);
}

static void step_cases(void)
{
    /* one whole turn with eviction and one under budget (K/V destination absent), tight buffers throughout */
    for (int round = 0; round < 2; ++round) {
        const int S = 2, n_held = round ? 3 : 20, n_new = round ? 4 : 15, vocab = 19, L = 1, H = 2, D = 4;
        const int n_cand = n_held + n_new;
        sirllm_ref_policy p = {2, 10, 6, 0.9f};
        const int n_keep = n_cand < 18 ? n_cand : 18;
        sirllm_ref_kv_layout lay = {L, H, D, 4, (int64_t)L * H * n_cand * D, (int64_t)H * n_cand * D, (int64_t)n_cand * D, D};
        sirllm_ref_kv_layout out = {L, H, D, 4, (int64_t)L * H * n_keep * D, (int64_t)H * n_keep * D, (int64_t)n_keep * D, D};
        float* z = malloc(sizeof(float) * S * n_new * vocab);
        int32_t* tok = malloc(sizeof(int32_t) * S * n_new);
        float* E = malloc(sizeof(float) * S * n_cand);
        float* k = malloc(sizeof(float) * extent(&lay, S, n_cand));
        float* v = malloc(sizeof(float) * extent(&lay, S, n_cand));
        float* kd = malloc(sizeof(float) * extent(&out, S, n_keep));
        float* vd = malloc(sizeof(float) * extent(&out, S, n_keep));
        int32_t* idx = malloc(sizeof(int32_t) * S * n_keep);
        float* Eo = malloc(sizeof(float) * S * n_keep);
        for (int i = 0; i < S * n_new * vocab; ++i) z[i] = frand();
        for (int i = 0; i < S * n_new; ++i) tok[i] = (int32_t)(lcg() % vocab);
        for (int i = 0; i < S * n_cand; ++i) E[i] = frand();
        for (int64_t i = 0; i < extent(&lay, S, n_cand); ++i) { k[i] = frand(); v[i] = frand(); }
        const int evict = n_cand > 18;
        CHECK(sirllm_ref_step(z, SIRLLM_REF_F32, vocab, vocab, tok, E, n_cand, S, n_held, n_new, &p, k, v, &lay,
                              evict ? kd : NULL, evict ? vd : NULL, &out, idx, n_keep, Eo, n_keep) == 0);
        CHECK(idx[0] == 0 && idx[n_keep - 1] == n_cand - 1);
        free(z); free(tok); free(E); free(k); free(v); free(kd); free(vd); free(idx); free(Eo);
    }
}

int main(void)
{
    for (int threads = 1; threads <= 4; threads += 3) {
        sirllm_ref_set_threads(threads);
        score_cases();
        lmhead_cases();
        select_cases();
        baseline_cases();
        gather_cases();
        step_cases();
    }
    uint32_t ctr[4] = {0, 0, 0, 0}, key[2] = {0, 0}, r[4];
    sirllm_ref_philox4x32_10(ctr, key, r);
    CHECK(r[0] != 0 || r[1] != 0);
    puts("SANITIZED OK");
    return 0;
}
