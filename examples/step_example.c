/*
 * A caller of libsirllm from plain C with nothing but the HIP runtime: allocate device buffers,
 * run one retention step (paper Sec. 3.2 score, Sec. 3.3 decay + Top_k + compaction), read the kept
 * slots back.  Build (from the repository root):
 *   hipcc -x c examples/step_example.c -Iinclude -Lpaper_2405_12528_amd -lsirllm \
 *         -Wl,-rpath,$PWD/paper_2405_12528_amd -o examples/step_example
 * Prints "ok" and the kept slots; exits non-zero on any error.
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include "sirllm.h"

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
    fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_)); return 2; } } while (0)

int main(void)
{
    enum { V = 512, N_HELD = 24, N_NEW = 16, N_CAND = N_HELD + N_NEW, LAYERS = 2, HEADS = 2, DIM = 32 };
    const sirllm_policy pol = { 2, 10, 4, 0.9f };                 /* budget 16 */
    const int n_keep = 16;

    /* host inputs: every row uniform except one preferred column; token = that column for even rows */
    float* logits = (float*)calloc((size_t)N_NEW * V, sizeof(float));
    int32_t tok[N_NEW];
    float held[N_CAND];
    for (int r = 0; r < N_NEW; ++r) { logits[(size_t)r * V + 7 * r] = 6.0f; tok[r] = (r % 2) ? 3 : 7 * r; }
    for (int i = 0; i < N_HELD; ++i) held[i] = (float)((i * 37) % 11);
    const size_t kv_elems = (size_t)LAYERS * HEADS * N_CAND * DIM;
    float* kv = (float*)malloc(kv_elems * sizeof(float));
    for (size_t i = 0; i < kv_elems; ++i) kv[i] = (float)i;

    float *d_logits, *d_scores, *d_out, *d_k, *d_v, *d_k2, *d_v2;
    int32_t *d_tok, *d_idx;
    HIP_OK(hipMalloc((void**)&d_logits, (size_t)N_NEW * V * 4));
    HIP_OK(hipMalloc((void**)&d_tok, N_NEW * 4));
    HIP_OK(hipMalloc((void**)&d_scores, N_CAND * 4));
    HIP_OK(hipMalloc((void**)&d_out, n_keep * 4));
    HIP_OK(hipMalloc((void**)&d_idx, n_keep * 4));
    HIP_OK(hipMalloc((void**)&d_k, kv_elems * 4));
    HIP_OK(hipMalloc((void**)&d_v, kv_elems * 4));
    HIP_OK(hipMalloc((void**)&d_k2, kv_elems * 4));
    HIP_OK(hipMalloc((void**)&d_v2, kv_elems * 4));
    HIP_OK(hipMemcpy(d_logits, logits, (size_t)N_NEW * V * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_tok, tok, N_NEW * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_scores, held, N_HELD * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_k, kv, kv_elems * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_v, kv, kv_elems * 4, hipMemcpyHostToDevice));

    const sirllm_kv_layout src = { LAYERS, HEADS, DIM, 4, 0, (int64_t)HEADS * N_CAND * DIM, (int64_t)N_CAND * DIM, DIM };
    const sirllm_kv_layout dst = { LAYERS, HEADS, DIM, 4, 0, (int64_t)HEADS * n_keep * DIM, (int64_t)n_keep * DIM, DIM };
    const int rc = sirllm_step(d_logits, SIRLLM_F32, V, V, d_tok, d_scores, N_CAND, 1, N_HELD, N_NEW, &pol,
                               d_k, d_v, &src, d_k2, d_v2, &dst, d_idx, n_keep, d_out, n_keep, NULL, 0, NULL);
    if (rc != SIRLLM_OK) { fprintf(stderr, "sirllm_step: %s\n", sirllm_status_string(rc)); return 3; }
    HIP_OK(hipDeviceSynchronize());

    int32_t idx[16];
    float new_scores[N_NEW], k_row0;
    HIP_OK(hipMemcpy(idx, d_idx, sizeof idx, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(new_scores, d_scores + N_HELD, sizeof new_scores, hipMemcpyDeviceToHost));
    /* closed form (Sec. 3.2): one logit a = 6 among V-1 zeros */
    const double logZ = log(exp(6.0) + V - 1);
    for (int r = 0; r < N_NEW; ++r) {
        const double want = (r % 2) ? logZ : logZ - 6.0;
        if (fabs(new_scores[r] - want) > 1e-6 + 1e-5 * want) { fprintf(stderr, "score %d off\n", r); return 4; }
    }
    if (idx[0] != 0 || idx[1] != 1 || idx[n_keep - 1] != N_CAND - 1) { fprintf(stderr, "sinks/recent wrong\n"); return 5; }
    /* compacted row 5 of plane 0 must be the source row idx[5] */
    HIP_OK(hipMemcpy(&k_row0, d_k2 + 5 * DIM, 4, hipMemcpyDeviceToHost));
    if (k_row0 != (float)(idx[5] * DIM)) { fprintf(stderr, "gather wrong\n"); return 6; }
    printf("ok: libsirllm %s kept", sirllm_version());
    for (int j = 0; j < n_keep; ++j) printf(" %d", idx[j]);
    printf("\n");
    return 0;
}
