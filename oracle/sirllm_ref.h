/*
 * sirllm_ref.h -- CPU oracle of the SirLLM retention step.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, host-memory implementation of what one dialogue turn of the method
 * computes outside the language model (paper: Sec. 3.1, 3.2, 3.3, Algorithm 1).  It exists
 * so that tests, the smoke check and the benchmark's CPU-baseline leg have something to
 * compare the GPU library with; nothing on the product path may call it.  It shares no
 * source, header or table with the GPU library: the structs below are declared here on
 * their own.
 *
 * All pointers are HOST pointers.  All functions return 0, or -1 for an argument they
 * cannot make sense of (null pointer, negative size).
 */
#ifndef SIRLLM_REF_H
#define SIRLLM_REF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { SIRLLM_REF_F32 = 0, SIRLLM_REF_BF16 = 1, SIRLLM_REF_F16 = 2 };

typedef struct {
    int32_t n_sink, n_topk, n_recent;
    float   decay;
} sirllm_ref_policy;

/* element (s,l,h,p,d) at base + elem_bytes*(s*stride_stream + l*stride_layer + h*stride_head + p*stride_pos + d) */
typedef struct {
    int32_t n_layers, n_kv_heads, head_dim, elem_bytes;
    int64_t stride_stream, stride_layer, stride_head, stride_pos;
} sirllm_ref_kv_layout;

/* Sec. 3.2: e_r = -log softmax(logits[r])[token_ids[r]], accumulated in double, rounded once. */
int sirllm_ref_score(const void* logits, int dtype, int64_t n_rows, int32_t vocab, int64_t ld,
                     const int32_t* token_ids, float* scores_out);

/* Sec. 3.2 with the logits never stored: z[r][v] = sum_k hidden[r][k] * weight[v][k] (the language-model
 * head, weight row v = the output embedding of token v), e_r = logsumexp(z[r]) - z[r][token_ids[r]].
 * hidden is [n_rows][ld_h], weight is [vocab][ld_w], both of element type `dtype`; everything in double. */
int sirllm_ref_lmhead_score(const void* hidden, int64_t ld_h, const void* weight, int64_t ld_w, int dtype,
                            int32_t d_model, int64_t n_rows, int32_t vocab,
                            const int32_t* token_ids, float* scores_out);

/* Sec. 3.3 + Sec. 3.1: decay the held scores, pick sink + top-k + recent, list them ascending. */
int sirllm_ref_decay_select(const float* scores, int64_t scores_stride,
                            int32_t n_streams, int32_t n_held, int32_t n_new,
                            const sirllm_ref_policy* policy,
                            int32_t* kept_idx, int64_t idx_stride,
                            float* scores_out, int64_t out_stride);

/* Sec. 3.3: KV_cache <- KV_cache[Id] for every stream, layer, head; K and V. */
int sirllm_ref_compact_kv(const void* k_src, const void* v_src, const sirllm_ref_kv_layout* src, int32_t n_src,
                          void* k_dst, void* v_dst, const sirllm_ref_kv_layout* dst,
                          const int32_t* kept_idx, int64_t idx_stride,
                          int32_t n_streams, int32_t n_keep);

/* The same, written back into the buffer it reads: slots [0, n_keep) become the kept rows, slots
 * >= n_keep keep their content. */
int sirllm_ref_compact_kv_inplace(void* k, void* v, const sirllm_ref_kv_layout* layout, int32_t n_src,
                                  const int32_t* kept_idx, int64_t idx_stride,
                                  int32_t n_streams, int32_t n_keep);

/* Algorithm 1, one turn, in the order score -> append -> decay held -> select -> compact. */
int sirllm_ref_step(const void* logits, int dtype, int32_t vocab, int64_t ld, const int32_t* token_ids,
                    float* scores, int64_t scores_stride,
                    int32_t n_streams, int32_t n_held, int32_t n_new,
                    const sirllm_ref_policy* policy,
                    const void* k_src, const void* v_src, const sirllm_ref_kv_layout* src,
                    void* k_dst, void* v_dst, const sirllm_ref_kv_layout* dst,
                    int32_t* kept_idx, int64_t idx_stride,
                    float* scores_out, int64_t out_stride);

/* Sec. 4.1 baselines: kind 0 = sink + recent only (StreamLLM), 1 = every interval-th middle slot
 * counted back from the newest one (IntervalLLM), 2 = a uniformly random subset of the middle slots
 * keyed by Philox4x32-10 (RandomLLM).  Writes the kept slots ascending; returns the kept count per
 * stream through *n_keep_out. */
int sirllm_ref_baseline_select(int kind, int32_t n_streams, int32_t n_cand, const sirllm_ref_policy* policy,
                               uint64_t seed, uint64_t turn, int32_t* kept_idx, int64_t idx_stride,
                               int32_t* n_keep_out);

/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC'11):
 * out[0..3] = ten rounds of the bijection on counter ctr[0..3] under key key[0..1]. */
void sirllm_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* Threads used by the loops over rows / planes (1 = serial).  Returns the count in effect. */
int sirllm_ref_set_threads(int n);
int sirllm_ref_get_threads(void);

#ifdef __cplusplus
}
#endif
#endif
