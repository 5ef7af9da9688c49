/*
 * sirllm.h -- C ABI of the SirLLM memory-retention hot path for AMD MI355X (gfx950).
 *
 * One dialogue turn of the method (paper: Section 3.2 "Token Entropy", Section 3.3
 * "Streaming Infinite Retentive LLM", Algorithm 1) adds four data-parallel operations
 * around the language model's forward pass:
 *
 *   score    e_i = -log P(x_i | x_<i)            token entropy of every new token   (Sec. 3.2)
 *   decay    E <- E * eta_decay                  once per dialogue round            (Sec. 3.3, Alg. 1 last line)
 *   select   Id_sink, Id_entropy = Top_k(E), Id_recent                              (Sec. 3.1, Sec. 3.3)
 *   compact  KV <- KV[Id], E <- E[Id]            for every layer and KV head        (Sec. 3.3, Alg. 1 eviction branch)
 *
 * The language model itself is not part of this library: logits, token ids and the K/V
 * tensors are inputs.
 *
 * General conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller, valid on the device that
 *     is current when the call is made.  Policy and layout structs are HOST pointers and are
 *     read before the call returns.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     enqueue work on it and return without synchronising.  The library allocates nothing and
 *     creates no streams.  Nothing a call computes depends on an earlier call; what the process keeps
 *     is bookkeeping only: per kernel and device, that the runtime has been told once about its LDS
 *     size; per device, the address of the static scratch of sirllm_decay_select_static; and whether
 *     the launch-shape overrides below are switched on.
 *   - Launch-shape overrides, for sweeps.  If the environment variable SIRLLM_TUNE is set to a non-empty
 *     value when the process makes its first call into the library, every launch reads the following
 *     variables (integers; unset = the default in brackets) -- otherwise none of them is ever read:
 *       SIRLLM_SCORE_BLOCK [by row length: 1024, 512 or 256]  threads per scored row
 *       SIRLLM_SCORE_NT [1], SIRLLM_GATHER_NT [1], SIRLLM_INPLACE_NT [1]   non-temporal (1) or cached (0) accesses
 *       SIRLLM_GATHER_BLOCK [64 for rows of 256 or 512 bytes or a power of two from 1 KB on, else 128] (or 64, 128, 256, 512), SIRLLM_GATHER_UNROLL [1] (or 2; 64 threads:
 *                                1, non-temporal only)   threads and 16-byte vectors per lane of a gather tile
 *       SIRLLM_GATHER_SCALAR_IDX [1], SIRLLM_GATHER_ROTATE [1 when the source planes lie a power of two apart and a compacted plane has 1 MiB or more, else 0]
 *                                rows of 256 bytes in tiles of 64 or 128 threads: kept indices by scalar loads (1) or per lane (0);
 *                                tiles of each group of eight exchanged by the plane index (1) or not (0)
 *       SIRLLM_FUSE_SELECT [1]   0: score and select in separate launches even when they are independent
 *       SIRLLM_LMHEAD_WIDE [1]   LM-head score of up to 128 rows (256 against a vocabulary below 65536 rows) with d_model a multiple of 64: pipeline stages of 64 (1) or 32 (0)
 *                                K elements, i.e. whole or half 128-byte lines of the embedding matrix per load
 *       SIRLLM_INPLACE_BLOCK [1024] (512, 256), SIRLLM_INPLACE_UNROLL [4] (2, 8), SIRLLM_INPLACE_PARTS [by plane count]
 *                                threads, vectors per lane and column parts of the in-place walk
 *       SIRLLM_INPLACE_TICKET [1 from 8192 planes on, else 0]   planes by ticket (1) or by block index (0) when a workspace is given
 *     Results do not depend on any of them (every setting is tested against the oracle); timings do.
 *   - All shapes are host integers and are uniform over the `n_streams` independent dialogue
 *     streams of a call.
 *   - Return value: SIRLLM_OK (0) or a negative sirllm_status.  Arguments are validated on
 *     the host before anything is enqueued; on a validation error nothing has been launched.
 *   - Alignment: no alignment beyond the natural alignment of the element type is required.
 *     The kernels take the widest access (16, 8, 4, 2 or 1 bytes) that all of a call's
 *     pointers and strides allow; 16-byte aligned pointers, strides and rows run fastest.
 *
 * Notation (used throughout):
 *   n_held   slots already in the cache, each with a score          n_new   tokens this turn
 *   n_cand   = n_held + n_new                                        budget  = n_sink + n_topk + n_recent
 *   n_keep   = min(n_cand, budget)
 */
#ifndef SIRLLM_H
#define SIRLLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SIRLLM_OK              =  0,
    SIRLLM_ERR_INVALID_ARG = -1,  /* null pointer, negative size, inconsistent shapes, overlapping src/dst */
    SIRLLM_ERR_UNSUPPORTED = -2,  /* a size above a documented limit, unknown dtype */
    SIRLLM_ERR_WORKSPACE   = -3,  /* workspace smaller than sirllm_workspace_bytes() or misaligned */
    SIRLLM_ERR_HIP         = -4   /* the HIP runtime refused a launch; hipGetLastError() has the detail */
} sirllm_status;

typedef enum {
    SIRLLM_F32  = 0,              /* IEEE binary32 */
    SIRLLM_BF16 = 1,              /* bfloat16: the upper 16 bits of a binary32 */
    SIRLLM_F16  = 2               /* IEEE binary16 */
} sirllm_dtype;

/* Retention policy (Sec. 3.1: n_sink, n_recent; Sec. 3.3: k of Top_k and eta_decay).
 * Any of the three sizes may be 0.  decay must be finite and >= 0. */
typedef struct {
    int32_t n_sink;     /* first n_sink cache slots are always kept */
    int32_t n_topk;     /* k: how many of the remaining slots are kept by decayed score */
    int32_t n_recent;   /* last n_recent candidate slots are always kept */
    float   decay;      /* eta_decay, multiplied once into every held score per call */
} sirllm_policy;

/* Addressing of a K or V cache.  Element (stream s, layer l, kv head h, slot p, channel d)
 * lives at  base + elem_bytes * (s*stride_stream + l*stride_layer + h*stride_head
 *                                + p*stride_pos + d),   0 <= d < head_dim  (channels contiguous).
 * Strides are in elements and must be >= 0; stride_pos >= head_dim.  The K/V payload is
 * treated as opaque bytes.  Any order of the four outer dimensions can be described; when the heads of a slot
 * lie back to back (stride_head == head_dim: [slot][head][dim] caches), and likewise the layers, in both the
 * source and the destination, the compaction copies them as one longer row. */
typedef struct {
    int32_t n_layers;
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t elem_bytes;   /* 1, 2, 4 or 8 */
    int64_t stride_stream;
    int64_t stride_layer;
    int64_t stride_head;
    int64_t stride_pos;
} sirllm_kv_layout;

/* Largest n_cand = n_held + n_new per stream that decay_select / step accept.  Up to 32768 slots a
 * stream is selected by one workgroup without any scratch; above that the selection runs as a
 * multi-workgroup radix select and needs the workspace (see sirllm_workspace_bytes). */
#define SIRLLM_MAX_CAND 16777216

/*
 * Token entropy (Sec. 3.2, the displayed definition of e_i):
 *     scores_out[r] = logsumexp_v(logits[r][0:vocab]) - logits[r][token_ids[r]],   0 <= r < n_rows
 * with the natural logarithm, i.e. minus the log-softmax probability of the token that
 * actually occurred.  Row r of `logits` starts at element r*ld (ld >= vocab) and is the
 * next-token distribution from which token_ids[r] was drawn; the library does no shifting.
 * Inputs (binary32, bfloat16 or binary16) are widened exactly to binary32; max, sum and log are
 * accumulated in binary32.
 *   logits      device, n_rows x ld elements of `dt`, read once
 *   token_ids   device, n_rows int32; an id outside [0, vocab) yields a quiet NaN score
 *   scores_out  device, n_rows float
 * -inf logits are allowed and contribute 0.  A row with no finite maximum (all -inf, any
 * +inf, any NaN) yields NaN.  n_rows == 0 is a no-op.
 * workspace: sirllm_workspace_bytes(0, 0, n_rows, vocab) bytes, 256-byte aligned (may be
 * NULL when that is 0).
 */
int sirllm_score(const void* logits, sirllm_dtype dt, int64_t n_rows, int32_t vocab, int64_t ld,
                 const int32_t* token_ids, float* scores_out,
                 void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Token entropy of rows that arrive in CHUNKS OF COLUMNS -- the shards of a vocabulary-parallel
 * LM head, or the tiles of an LM head that never materialises a whole row.  Softmax statistics
 * form a monoid: a chunk is summarised by (m, s) = (max, sum of exp(z - m)), two summaries merge as
 * m = max(m1, m2), s = s1*exp(m1 - m) + s2*exp(m2 - m), and the chunk that holds the token's column
 * also reports z_tok.  Merging all chunks gives exactly the quantity of Sec. 3.2,
 * e = (m - z_tok) + log s; across GPUs the merge is one all-reduce of 3 floats per row.
 *   sirllm_score_partial   columns [v_begin, v_begin + n_cols) of every row: logits_chunk is
 *                          n_rows x ld elements whose column c is vocabulary entry v_begin + c;
 *                          token_ids are GLOBAL ids; writes partial[3*r + {0,1,2}] = m, s, z_tok
 *                          (z_tok = NaN when the token is not in this chunk).
 *   sirllm_score_merge     n_parts partial arrays, part p at partials + p*part_stride floats
 *                          (part_stride >= 3*n_rows) -> scores_out[n_rows].  A token that no chunk
 *                          holds scores NaN.
 */
int sirllm_score_partial(const void* logits_chunk, sirllm_dtype dt, int64_t n_rows, int32_t n_cols, int64_t ld,
                         int32_t v_begin, const int32_t* token_ids, float* partial, void* hip_stream);
int sirllm_score_merge(const float* partials, int32_t n_parts, int64_t part_stride, int64_t n_rows,
                       float* scores_out, void* hip_stream);

/*
 * Token entropy straight from the language-model head.  Sec. 3.2 takes the probabilities from the
 * model's own softmax output, i.e. from logits z = h W^T that the model computes anyway (the paper's
 * remark that the metric needs no additional computation).  This entry point computes
 *     scores_out[r] = logsumexp_v(z[r][0:vocab]) - z[r][token_ids[r]],   z[r][v] = sum_k hidden[r][k] * weight[v][k]
 * on the matrix cores and reduces every tile of z to softmax statistics in registers, so the
 * n_rows x vocab logits are never written to or read from memory.
 *   hidden      device, n_rows x ld_h elements of `dt` (the final hidden state of each scored token's row)
 *   weight      device, vocab x ld_w elements of `dt`; row v is the output embedding of token v (no bias)
 *   dt          SIRLLM_BF16 or SIRLLM_F16 (products exact, accumulation in binary32); SIRLLM_F32 is
 *               SIRLLM_ERR_UNSUPPORTED
 *   d_model     inner dimension; d_model, ld_h and ld_w must be multiples of 8 and both base pointers
 *               16-byte aligned (else SIRLLM_ERR_UNSUPPORTED); ld_h, ld_w < 2^21
 *   token_ids   device, n_rows int32; an id outside [0, vocab) yields a quiet NaN score
 *   scores_out  device, n_rows float
 *   workspace   device scratch of sirllm_lmhead_workspace_bytes(n_rows, vocab) bytes, 256-byte aligned,
 *               required (SIRLLM_ERR_WORKSPACE); overwritten, carries nothing between calls; calls that
 *               share it must be ordered on one stream.
 * n_rows == 0 is a no-op.  A non-finite product makes that row's score NaN.  Results are deterministic for
 * given arguments; the order of the binary32 sums depends on the tile shape chosen from n_rows and vocab, so the
 * same row can differ in its last bits between calls with different n_rows.
 */
int sirllm_lmhead_score(const void* hidden, int64_t ld_h, const void* weight, int64_t ld_w, sirllm_dtype dt,
                        int32_t d_model, int64_t n_rows, int32_t vocab, const int32_t* token_ids,
                        float* scores_out, void* workspace, size_t workspace_bytes, void* hip_stream);
size_t sirllm_lmhead_workspace_bytes(int64_t n_rows, int32_t vocab);

/*
 * Decay, select and index build (Sec. 3.3: E <- E*eta, Id_entropy = Top_k(E), E <- E[Id];
 * Sec. 3.1: Id_sink, Id_recent; Alg. 1 eviction branch and its trigger "cache size > L").
 * For every stream s, with E = scores + s*scores_stride:
 *   1. E[i] <- fl32(E[i] * decay) for i < n_held (one rounded binary32 multiply, denormals
 *      kept); the n_new entries E[n_held : n_cand) are this turn's scores and enter undecayed.
 *      The input array is not modified; the decayed values appear in scores_out.
 *   2. If n_cand <= budget nothing is evicted: kept_idx = 0..n_cand-1.
 *      Otherwise kept = [0, n_sink)  U  Top_k of the middle region [n_sink, n_cand-n_recent)
 *      U  [n_cand-n_recent, n_cand).  Top_k takes the n_topk largest decayed scores; equal
 *      scores (IEEE ==, so +0 == -0) go to the lower slot.  NaNs are ordered by bit pattern:
 *      a NaN with the sign bit clear ranks above +inf, one with it set below -inf.
 *   3. kept_idx[s*idx_stride + j], j < n_keep, lists the kept slots in ascending order (the
 *      in-cache position j of Sec. 3.3's worked example), and
 *      scores_out[s*out_stride + j] = E[kept_idx[j]].
 * Limits: n_cand <= SIRLLM_MAX_CAND (else SIRLLM_ERR_UNSUPPORTED).  n_streams == 0 or
 * n_cand == 0 is a no-op.  scores_out must not overlap scores.
 * workspace: sirllm_workspace_bytes(n_streams, n_cand, 0, 0) bytes of device scratch, 256-byte aligned;
 * that is 0 (NULL accepted) up to 32768 slots per stream.  Above, the scratch is required
 * (SIRLLM_ERR_WORKSPACE without it); it is cleared by the call itself and carries nothing over, but
 * calls that share it must be ordered on one stream.
 */
int sirllm_decay_select(const float* scores, int64_t scores_stride,
                        int32_t n_streams, int32_t n_held, int32_t n_new,
                        const sirllm_policy* policy,
                        int32_t* kept_idx, int64_t idx_stride,
                        float* scores_out, int64_t out_stride,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * sirllm_decay_select for callers that cannot allocate device memory or size a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and limits as
 * sirllm_decay_select, minus the workspace: the scratch of the multi-workgroup selection (more than 32768 slots
 * per stream) lives in a static device array of SIRLLM_STATIC_SCRATCH_BYTES inside the library, which every GPU
 * the library runs on holds until the process ends.  The call allocates nothing and frees nothing.
 *   - Sizes whose scratch does not fit (sirllm_workspace_bytes(n_streams, n_cand, 0, 0) >
 *     SIRLLM_STATIC_SCRATCH_BYTES, e.g. more than 240 streams of 131072 slots, or more than 51 streams of
 *     SIRLLM_MAX_CAND slots) return SIRLLM_ERR_UNSUPPORTED; nothing is launched.
 *   - All calls on one GPU share that GPU's array.  The call clears what it needs itself (with a kernel), so
 *     nothing carries over from one call to the next; but two calls that overlap in time on one GPU (two streams,
 *     two host threads) race on it.  Order them on one stream, or use sirllm_decay_select with workspaces of
 *     their own.  Up to 32768 slots per stream no scratch is used and nothing is shared.
 *   - The address of the array is looked up (hipGetSymbolAddress) the first time the call needs it on a device;
 *     make one call outside any graph capture first.
 */
#define SIRLLM_STATIC_SCRATCH_BYTES 1048576
int sirllm_decay_select_static(const float* scores, int64_t scores_stride,
                               int32_t n_streams, int32_t n_held, int32_t n_new,
                               const sirllm_policy* policy,
                               int32_t* kept_idx, int64_t idx_stride,
                               float* scores_out, int64_t out_stride, void* hip_stream);

/*
 * KV compaction (Sec. 3.3: KV_cache <- KV_cache[Id], for the keys and the values of every
 * layer and head).  Out of place:
 *     dst(s, l, h, j, :) = src(s, l, h, kept_idx[s*idx_stride + j], :),   0 <= j < n_keep
 * for K (k_src -> k_dst) and V (v_src -> v_dst).  src and dst layouts must agree in
 * n_layers, n_kv_heads, head_dim and elem_bytes; strides may differ.  v_src/v_dst may both be
 * NULL to move one tensor only.  Source and destination must not overlap, and kept_idx must lie outside every
 * destination buffer (it is read while they are written; not checked).
 *   n_src   number of valid slots per (stream, layer, head) in the source; an index outside
 *           [0, n_src) cannot be reported without a device read-back, so the destination row
 *           is zero-filled instead of reading out of bounds.
 * Limit: n_keep * head_dim * elem_bytes (the bytes of one compacted plane) must stay below
 * 2 GiB, else SIRLLM_ERR_UNSUPPORTED.  n_keep == 0 or n_streams == 0 is a no-op.
 */
int sirllm_compact_kv(const void* k_src, const void* v_src, const sirllm_kv_layout* src, int32_t n_src,
                      void* k_dst, void* v_dst, const sirllm_kv_layout* dst,
                      const int32_t* kept_idx, int64_t idx_stride,
                      int32_t n_streams, int32_t n_keep, void* hip_stream);

/*
 * The same compaction (Sec. 3.3) for a cache held as one K and one V buffer PER LAYER, the usual shape of a model's
 * past keys and values: k_src[l], v_src[l], k_dst[l], v_dst[l] are device pointers to layer l's buffers, and the four
 * arrays of src->n_layers pointers themselves are HOST memory (they travel in the kernels' arguments, 32 layers per
 * launch; nothing is staged in device memory and the call can be captured).  `src` and `dst` describe ONE layer:
 * stride_stream, stride_head, stride_pos as in sirllm_kv_layout, stride_layer is ignored, n_layers is the number of
 * entries of the arrays.  v_src and v_dst may both be NULL.  Everything else as for sirllm_compact_kv; no destination
 * buffer may overlap a source buffer or another destination buffer (SIRLLM_ERR_INVALID_ARG).
 */
int sirllm_compact_kv_layers(const void* const* k_src, const void* const* v_src, const sirllm_kv_layout* src,
                             int32_t n_src, void* const* k_dst, void* const* v_dst, const sirllm_kv_layout* dst,
                             const int32_t* kept_idx, int64_t idx_stride,
                             int32_t n_streams, int32_t n_keep, void* hip_stream);

/*
 * The same compaction, written back into the buffer it reads (Sec. 3.3): after the call slots
 * [0, n_keep) of every plane hold the rows kept_idx[0 : n_keep), slots >= n_keep keep whatever
 * they held.  Needs kept_idx strictly ascending per stream with entries in [0, n_src) -- which is
 * what sirllm_decay_select and sirllm_baseline_select produce -- because rows then only move
 * towards the front; for any other list the result is unspecified (but nothing outside the
 * n_src slots of a plane is touched, and entries outside [0, n_src) give zero rows).  Rows that
 * already sit in their place are not touched at all.  Halves the K/V memory of the out-of-place
 * call at the same traffic per moved row.  v may be NULL.  Limits as for sirllm_compact_kv.
 *   workspace   optional device scratch, 256-byte aligned (else SIRLLM_ERR_WORKSPACE).  With at least
 *               SIRLLM_INPLACE_WORKSPACE_BYTES the workgroups that compact the (stream, layer, tensor, head) planes
 *               take their planes in the order in which they start (a ticket counter in the scratch, cleared by the
 *               call itself) instead of by block index, which keeps the planes in flight next to each other in
 *               memory: up to 7 % faster on batches of tens of thousands of planes.  The library does so from 8192
 *               planes on (streams x layers x tensors x heads); below that, and with NULL or a smaller workspace,
 *               planes go by block index.  Results are identical either way.  Calls that share a workspace must be
 *               ordered on one stream.
 */
#define SIRLLM_INPLACE_WORKSPACE_BYTES 256
int sirllm_compact_kv_inplace(void* k, void* v, const sirllm_kv_layout* layout, int32_t n_src,
                              const int32_t* kept_idx, int64_t idx_stride,
                              int32_t n_streams, int32_t n_keep,
                              void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * sirllm_compact_kv_inplace for a cache held as one K and one V buffer per layer: k[l], v[l] are device pointers to
 * layer l's buffers, the two arrays of layout->n_layers pointers are HOST memory (see sirllm_compact_kv_layers); `layout`
 * describes one layer, stride_layer is ignored.  v may be NULL.  No two buffers may overlap.
 */
int sirllm_compact_kv_inplace_layers(void* const* k, void* const* v, const sirllm_kv_layout* layout, int32_t n_src,
                                     const int32_t* kept_idx, int64_t idx_stride,
                                     int32_t n_streams, int32_t n_keep,
                                     void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * One whole retention step (Alg. 1 with the loop rotated so that a call is
 * score -> decay held -> select -> compact; multiplying every candidate by the same
 * eta > 0 cannot change a comparison, so the kept sets equal those of the printed order).
 *   logits, token_ids   n_streams*n_new rows, row s*n_new + r belongs to stream s, token r
 *   scores              per stream: [0, n_held) held scores (input, unchanged),
 *                       [n_held, n_cand) receives this turn's scores (output)
 *   k_src, v_src        caches holding n_cand slots per stream (the new tokens' K/V already
 *                       appended at slots [n_held, n_cand))
 *   kept_idx, scores_out, k_dst, v_dst   as in sirllm_decay_select / sirllm_compact_kv
 * When n_cand <= budget nothing is evicted: kept_idx = 0..n_cand-1, scores_out holds the
 * decayed and new scores, k_dst/v_dst are NOT written (they may be NULL) and the cache
 * stays in k_src/v_src.
 * workspace: sirllm_workspace_bytes(n_streams, n_cand, n_streams*n_new, vocab) bytes.
 */
int sirllm_step(const void* logits, sirllm_dtype dt, int32_t vocab, int64_t ld,
                const int32_t* token_ids,
                float* scores, int64_t scores_stride,
                int32_t n_streams, int32_t n_held, int32_t n_new,
                const sirllm_policy* policy,
                const void* k_src, const void* v_src, const sirllm_kv_layout* src,
                void* k_dst, void* v_dst, const sirllm_kv_layout* dst,
                int32_t* kept_idx, int64_t idx_stride,
                float* scores_out, int64_t out_stride,
                void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The step without its K/V movement (Alg. 1: the entropy, decay and selection lines): exactly what sirllm_step does in
 * front of its compaction, including the shared launch of scoring and selection when no new token can compete in
 * Top_k.  For callers that move their caches themselves -- per-layer tensors through sirllm_compact_kv_layers or
 * sirllm_compact_kv_inplace_layers, paged caches, a cache on another device.  Arguments, limits and workspace as for
 * sirllm_step.  kept_idx / scores_out hold min(n_cand, budget) entries per stream afterwards.
 */
int sirllm_score_select(const void* logits, sirllm_dtype dt, int32_t vocab, int64_t ld,
                        const int32_t* token_ids,
                        float* scores, int64_t scores_stride,
                        int32_t n_streams, int32_t n_held, int32_t n_new,
                        const sirllm_policy* policy,
                        int32_t* kept_idx, int64_t idx_stride, float* scores_out, int64_t out_stride,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * One dialogue turn with the scores taken straight from the language-model head: sirllm_step with its first
 * stage replaced by sirllm_lmhead_score (Alg. 1, one loop iteration; Sec. 3.2 for the score).  hidden holds
 * n_streams * n_new rows, stream s owning rows [s*n_new, (s+1)*n_new); every other argument, the results and the
 * under-budget behaviour are those of sirllm_step; the restrictions on hidden / weight / dt / d_model are those
 * of sirllm_lmhead_score.  workspace: sirllm_step_lmhead_workspace_bytes(n_streams, n_held + n_new,
 * n_streams * n_new, vocab) bytes of device scratch, 256-byte aligned, required.
 */
int sirllm_step_lmhead(const void* hidden, int64_t ld_h, const void* weight, int64_t ld_w, sirllm_dtype dt,
                       int32_t d_model, int32_t vocab, const int32_t* token_ids,
                       float* scores, int64_t scores_stride, int32_t n_streams, int32_t n_held, int32_t n_new,
                       const sirllm_policy* policy,
                       const void* k_src, const void* v_src, const sirllm_kv_layout* src,
                       void* k_dst, void* v_dst, const sirllm_kv_layout* dst,
                       int32_t* kept_idx, int64_t idx_stride, float* scores_out, int64_t out_stride,
                       void* workspace, size_t workspace_bytes, void* hip_stream);
size_t sirllm_step_lmhead_workspace_bytes(int32_t n_streams, int32_t n_cand, int64_t n_rows, int32_t vocab);

/*
 * One retention step for a RAGGED batch, compacting in place: every stream has its own cache fill
 * and its own number of new tokens, as in a serving batch whose dialogues are at different turns.
 * Per stream s (Alg. 1, same order and readings as sirllm_step):
 *     n_new[s]  = cu_new[s+1] - cu_new[s]        its rows of `logits` / `token_ids` are [cu_new[s], cu_new[s+1])
 *     n_cand[s] = n_held[s] + n_new[s]
 *   - the new scores are written to scores[s*scores_stride + n_held[s] + t];
 *   - held scores are decayed; if n_cand[s] > budget the stream is selected and its K/V compacted in
 *     place to `budget` slots, else everything is kept and its K/V is not touched;
 *   - kept_idx / scores_out rows as in sirllm_decay_select; n_keep_out[s] = min(n_cand[s], budget)
 *     is written to DEVICE memory (it is the stream's n_held for the next turn).
 *   n_held, cu_new, n_keep_out   device arrays of n_streams, n_streams+1, n_streams int32
 *   total_new                    host copy of cu_new[n_streams]
 *   max_cand, max_new            host upper bounds of n_cand[s] and n_new[s]; they size the launches.  A
 *                                stream whose sizes exceed them (or are negative) gets n_keep_out[s] = -1:
 *                                its kept_idx row and its K/V are left alone, its score rows are
 *                                unspecified.  When max_new <= n_recent no new token can compete in
 *                                Top_k, and scoring and selection share one launch.
 *   k, v, layout                 caches holding n_cand[s] slots of stream s (new tokens already appended);
 *                                rewritten in place as by sirllm_compact_kv_inplace.  v may be NULL.
 * scores_stride >= max_cand; idx_stride, out_stride >= min(max_cand, budget).  max_cand <= SIRLLM_MAX_CAND, else
 * SIRLLM_ERR_UNSUPPORTED.
 * workspace: 256-byte aligned.  Up to max_cand = 32768 every stream is selected by one workgroup and the workspace
 * is optional (NULL accepted); with at least SIRLLM_INPLACE_WORKSPACE_BYTES the compaction takes its planes in
 * ticket order, as described at sirllm_compact_kv_inplace.  Above 32768 the streams are selected by the
 * multi-workgroup kernels and sirllm_workspace_bytes(n_streams, max_cand, 0, 0) bytes are required
 * (SIRLLM_ERR_WORKSPACE otherwise); the compaction reuses them for its ticket.
 */
int sirllm_step_ragged(const void* logits, sirllm_dtype dt, int32_t vocab, int64_t ld,
                       const int32_t* token_ids,
                       float* scores, int64_t scores_stride,
                       int32_t n_streams, const int32_t* n_held, const int32_t* cu_new,
                       int64_t total_new, int32_t max_cand, int32_t max_new,
                       const sirllm_policy* policy,
                       void* k, void* v, const sirllm_kv_layout* layout,
                       int32_t* kept_idx, int64_t idx_stride,
                       float* scores_out, int64_t out_stride, int32_t* n_keep_out,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * sirllm_step_ragged with the K/V movement out of place (Alg. 1 per stream; Sec. 3.3): every stream the selection accepts
 * has its kept slots written to the destination buffers,
 *     dst(s, l, h, j, :) = src(s, l, h, kept_idx[s*idx_stride + j], :),   0 <= j < n_keep_out[s],
 * compacted to the budget when it holds more, all of its slots in their order while it holds less, so that after the
 * call the whole batch lives in the destination and a caller alternates two buffer pairs wholesale.  It is the kernel
 * of sirllm_compact_kv (5 to 14 % faster than the in-place walk, for a second pair of buffers).  A flagged stream
 * (n_keep_out[s] = -1) has nothing written.  Source and destination layouts must agree in n_layers, n_kv_heads,
 * head_dim and elem_bytes; the destination holds min(max_cand, budget) slots per plane; no destination buffer may
 * overlap a source buffer, the other destination buffer or kept_idx.  Everything else -- scores, sizes, bounds,
 * flags, workspace -- as for sirllm_step_ragged (the workspace is only the selection's: required above 32768 slots per
 * stream).
 */
int sirllm_step_ragged_out_of_place(const void* logits, sirllm_dtype dt, int32_t vocab, int64_t ld,
                                    const int32_t* token_ids,
                                    float* scores, int64_t scores_stride,
                                    int32_t n_streams, const int32_t* n_held, const int32_t* cu_new,
                                    int64_t total_new, int32_t max_cand, int32_t max_new,
                                    const sirllm_policy* policy,
                                    const void* k_src, const void* v_src, const sirllm_kv_layout* src,
                                    void* k_dst, void* v_dst, const sirllm_kv_layout* dst,
                                    int32_t* kept_idx, int64_t idx_stride,
                                    float* scores_out, int64_t out_stride, int32_t* n_keep_out,
                                    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * sirllm_step_ragged with its scores taken straight from the LM head (Alg. 1 per stream; Sec. 3.2): the rows of
 * `hidden` / `token_ids` of stream s are [cu_new[s], cu_new[s+1]), the score of its token t is written to
 * scores[s*scores_stride + n_held[s] + t], and everything behind the scores is sirllm_step_ragged's.  Operands
 * and their limits as for sirllm_lmhead_score; sizes, bounds, flags and in-place compaction as for
 * sirllm_step_ragged.  workspace: required, 256-byte aligned, at least
 * sirllm_step_lmhead_ragged_workspace_bytes(n_streams, max_cand, total_new, vocab) bytes (the LM head's per-tile
 * triples, then the selection's scratch or the compaction's ticket).
 */
int sirllm_step_lmhead_ragged(const void* hidden, int64_t ld_h, const void* weight, int64_t ld_w,
                              sirllm_dtype dt, int32_t d_model, int32_t vocab, const int32_t* token_ids,
                              float* scores, int64_t scores_stride,
                              int32_t n_streams, const int32_t* n_held, const int32_t* cu_new,
                              int64_t total_new, int32_t max_cand, int32_t max_new,
                              const sirllm_policy* policy,
                              void* k, void* v, const sirllm_kv_layout* layout,
                              int32_t* kept_idx, int64_t idx_stride,
                              float* scores_out, int64_t out_stride, int32_t* n_keep_out,
                              void* workspace, size_t workspace_bytes, void* hip_stream);
size_t sirllm_step_lmhead_ragged_workspace_bytes(int32_t n_streams, int32_t max_cand, int64_t total_new,
                                                 int32_t vocab);

/*
 * The ragged step from hidden states with a second buffer pair: sirllm_step_lmhead_ragged's scoring operands,
 * workspace and rules, sirllm_step_ragged_out_of_place's K/V arguments and its copy-all rule (every accepted stream's
 * kept slots land in k_dst / v_dst, a flagged stream's destination is left as it was, nothing of k_src / v_src is
 * written).  Paper Algorithm 1 per stream; Sec. 3.2 for where the score comes from.
 */
int sirllm_step_lmhead_ragged_out_of_place(const void* hidden, int64_t ld_h, const void* weight, int64_t ld_w,
                                           sirllm_dtype dt, int32_t d_model, int32_t vocab, const int32_t* token_ids,
                                           float* scores, int64_t scores_stride,
                                           int32_t n_streams, const int32_t* n_held, const int32_t* cu_new,
                                           int64_t total_new, int32_t max_cand, int32_t max_new,
                                           const sirllm_policy* policy,
                                           const void* k_src, const void* v_src, const sirllm_kv_layout* src,
                                           void* k_dst, void* v_dst, const sirllm_kv_layout* dst,
                                           int32_t* kept_idx, int64_t idx_stride,
                                           float* scores_out, int64_t out_stride, int32_t* n_keep_out,
                                           void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Baseline retention policies on the same compaction path (Sec. 4.1 "Baselines"): they pick the
 * n_topk slots of the middle region [n_sink, n_cand - n_recent) without looking at any score;
 * sinks and the recent window are kept as in sirllm_decay_select, and kept_idx comes out in the
 * same ascending order, ready for sirllm_compact_kv.  policy->decay is ignored.
 *   SIRLLM_BASELINE_STREAM    no middle slot at all: sinks + recent window only (StreamLLM);
 *                             the kept count is n_sink + n_recent, whatever n_topk says.
 *   SIRLLM_BASELINE_INTERVAL  every interval-th middle slot, interval = max(1, floor(M / n_topk)),
 *                             M the size of the middle region (IntervalLLM).  The paper does not
 *                             say where the comb is anchored; here it is anchored at the newest
 *                             middle slot and runs towards older ones until n_topk slots are
 *                             taken, so a stream keeps absorbing new tokens when interval is 1.
 *   SIRLLM_BASELINE_RANDOM    a uniformly random n_topk-subset of the middle slots (RandomLLM):
 *                             slot i of stream s gets the key Philox4x32-10(counter = {i, s,
 *                             turn low word, turn high word}, key = {seed low, seed high}) word 0,
 *                             and the n_topk largest keys are kept (equal keys: lower slot).
 * When n_cand <= the kept count nothing is evicted: kept_idx = 0..n_cand-1.
 * Returns, through *n_keep_out (host pointer, may be NULL), the number of kept slots per stream.
 * Limits as for sirllm_decay_select.  workspace: only SIRLLM_BASELINE_RANDOM with more than 32768 slots per
 * stream uses it (the multi-workgroup selection on the generator's draws) and then needs
 * sirllm_workspace_bytes(n_streams, n_cand, 0, 0) bytes, 256-byte aligned (SIRLLM_ERR_WORKSPACE otherwise);
 * everywhere else NULL / 0 is accepted.
 */
typedef enum {
    SIRLLM_BASELINE_STREAM   = 0,
    SIRLLM_BASELINE_INTERVAL = 1,
    SIRLLM_BASELINE_RANDOM   = 2
} sirllm_baseline;

int sirllm_baseline_select(sirllm_baseline kind, int32_t n_streams, int32_t n_cand,
                           const sirllm_policy* policy, uint64_t seed, uint64_t turn,
                           int32_t* kept_idx, int64_t idx_stride, int32_t* n_keep_out,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/* Bytes of device workspace the calls above need for these sizes (pass 0 for the sizes a
 * call does not have): 0 unless n_cand exceeds 32768, then about 4 KB + n_cand/1024 bytes per stream.
 * Never fails; the result is a multiple of 256. */
size_t sirllm_workspace_bytes(int32_t n_streams, int32_t n_cand, int64_t n_rows, int32_t vocab);

/* Static, NUL-terminated description of a status code. */
const char* sirllm_status_string(int status);

/* Library version, "major.minor.patch". */
const char* sirllm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SIRLLM_H */
