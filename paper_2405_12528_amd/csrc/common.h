// Internal declarations shared by the HIP translation units of libsirllm (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sirllm.h"

namespace sirllm {

constexpr int kWave = 64;                    // CDNA wavefront width

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// ---- cross-lane moves inside a wavefront ------------------------------------------------
// Data-parallel-primitive (DPP) moves run on the vector ALU, without the round trip through the LDS crossbar that a
// general lane shuffle takes; the reductions at the end of every latency-bound kernel here are chains of them.
// A wave is four rows of 16 lanes.  dpp_move<CTRL, ROW_MASK>(v, fill): every lane of the rows enabled in ROW_MASK
// receives v from the lane CTRL names, or `fill` when that lane does not exist or its own row is not enabled.
constexpr int kDppRowShr1 = 0x111, kDppRowShr2 = 0x112, kDppRowShr4 = 0x114, kDppRowShr8 = 0x118;   // lane i <- lane i - n of its row
constexpr int kDppRowBcast15 = 0x142;   // lane 15 of each row -> every lane of the next row
constexpr int kDppRowBcast31 = 0x143;   // lane 31 -> every lane of rows 2 and 3

template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ uint32_t dpp_move(uint32_t v, uint32_t fill)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)fill, (int)v, CTRL, ROW_MASK, 0xf, false);
}

// Inclusive prefix sum over the 64 lanes: Hillis-Steele inside each row, then the row totals carried forward.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t v)
{
    v += dpp_move<kDppRowShr1>(v, 0u);
    v += dpp_move<kDppRowShr2>(v, 0u);
    v += dpp_move<kDppRowShr4>(v, 0u);
    v += dpp_move<kDppRowShr8>(v, 0u);
    v += dpp_move<kDppRowBcast15, 0xa>(v, 0u);
    v += dpp_move<kDppRowBcast31, 0xc>(v, 0u);
    return v;
}

// Sum over the 64 lanes, the same value in every lane.
__device__ __forceinline__ uint32_t wave_sum(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)wave_inclusive_sum(v), kWave - 1);
}

// ---- score.hip --------------------------------------------------------------------------
// Token entropy of n_rows rows.  Row `row` belongs to stream row / rows_per_stream, token
// t = row % rows_per_stream; its score goes to out_a[stream*stride_a + t] and, when out_b is
// not null, also to out_b[stream*stride_b + t].
// Ragged batches (cu_rows != null): stream s owns rows [cu_rows[s], cu_rows[s+1]) and its token t
// goes to out_a[s*stride_a + held_dev[s] + t].
struct ScoreArgs {
    const void* logits;
    int64_t ld;               // elements between rows
    int32_t vocab;
    const int32_t* token_ids;
    int64_t n_rows;
    int64_t rows_per_stream;  // >= 1
    float* out_a;
    int64_t stride_a;
    float* out_b;
    int64_t stride_b;
    float* partial;           // not null: the row is a chunk of columns starting at v_begin; write (m, s, z_tok)
    int32_t v_begin;          //           triples to partial[3*row ..] instead of a finished score
    const int32_t* cu_rows;   // device [n_streams_r + 1], or null for uniform batches
    const int32_t* held_dev;  // device [n_streams_r]
    int32_t n_streams_r;
    int32_t budget_r;         // ragged + out_b: token t of stream s also goes to out_b[s*stride_b + n_keep[s] - n_new[s] + t]
};
hipError_t launch_score(const ScoreArgs& a, sirllm_dtype dt, hipStream_t stream);
// Merges n_parts sets of (m, s, z_tok) triples (set p starts at partials + p*part_stride) into scores.
hipError_t launch_score_merge(const float* partials, int32_t n_parts, int64_t part_stride, int64_t n_rows,
                              float* scores_out, hipStream_t stream);

// ---- lmhead.hip -------------------------------------------------------------------------
// Token entropy from hidden states and the output embedding matrix, logits never stored.
struct LmHeadArgs {
    const void* hidden;       // [n_rows][ld_h], 2-byte elements
    const void* weight;       // [vocab][ld_w]
    int64_t ld_h, ld_w;       // elements between rows, multiples of 8
    int32_t d_model;          // multiple of 8
    int32_t vocab;
    int64_t n_rows;
    const int32_t* token_ids;
    float* partial;           // scratch: [n_vtiles][part_stride] floats, (m, s, z_tok) per row
    int64_t part_stride;      // >= 3 * n_rows
    int32_t n_vtiles, n_ttiles;   // filled in by the launcher
};
// Upper bound on the number of vocabulary tiles (sets of triples in the scratch) for these sizes.
int lmhead_tiles_vocab(int64_t n_rows, int32_t vocab);
// Ragged batches: stream s owns rows [cu_rows[s], cu_rows[s+1]) and holds held_dev[s] slots already.
struct LmHeadRagged {
    const int32_t* cu_rows;   // device [n_streams + 1]
    const int32_t* held_dev;  // device [n_streams]
    int32_t n_streams;
};
// Row r is token r % rows_per_stream of stream r / rows_per_stream; its score goes to out[stream*out_stride + token].
// With `ragged`, row r is token t = r - cu_rows[s] of the stream s that owns it and goes to
// out[s*out_stride + held_dev[s] + t] (dropped when that lies outside [0, out_stride)).
hipError_t launch_lmhead_score(const LmHeadArgs& a, sirllm_dtype dt, float* out, int64_t rows_per_stream,
                               int64_t out_stride, hipStream_t stream, const LmHeadRagged* ragged = nullptr);

// ---- select.hip -------------------------------------------------------------------------
struct SelectArgs {
    const float* scores;      // [n_streams][scores_stride]
    int64_t scores_stride;
    int32_t n_streams, n_held, n_cand;
    int32_t n_sink, n_topk, n_recent;
    float decay;
    int32_t* kept_idx;
    int64_t idx_stride;
    float* scores_out;
    int64_t out_stride;
    uint32_t seed_lo, seed_hi, turn_lo, turn_hi;   // RandomLLM baseline only
    // Ragged batches: per-stream sizes in device memory (n_held / n_cand above are then upper bounds).
    const int32_t* held_dev;  // [n_streams]
    const int32_t* cu_new_dev;// [n_streams + 1]
    int32_t* n_keep_dev;      // [n_streams], written: min(n_cand[s], budget), or -1 when n_cand[s] exceeds the bound
    int32_t max_new;          // ragged: the caller's bound on n_new[s] (a stream above it is flagged like one above n_cand)
};
// n_cand > budget: decay + radix select + index build, one workgroup per stream.
hipError_t launch_select(const SelectArgs& a, hipStream_t stream);
// n_cand <= budget: identity index list, decayed scores.
hipError_t launch_keep_all(const SelectArgs& a, hipStream_t stream);
// Ragged batches: every stream takes its own branch (keep all, or select) on its own sizes.
hipError_t launch_select_ragged(const SelectArgs& a, hipStream_t stream);

// ---- select_large.hip -------------------------------------------------------------------
// One workgroup holds at most this many candidate slots of a stream in registers; larger caches go
// through the multi-workgroup path, which needs scratch.
#define SIRLLM_SINGLE_WG_CAND 32768
size_t select_large_scratch_bytes(int32_t n_streams, int32_t n_cand);
// Serves ragged batches too (a.held_dev set: per-stream sizes, a.n_cand the bound, a.n_keep_dev written), and with
// random_keys the RandomLLM baseline (no score read or written).
hipError_t launch_select_large(const SelectArgs& a, void* scratch, hipStream_t stream, bool random_keys = false);

// ---- gather.hip -------------------------------------------------------------------------
struct GatherArgs {
    const char* src[2];       // K, V (V may be null: then only tensor 0 is moved)
    char* dst[2];
    int64_t s_stream, s_layer, s_head, s_pos;   // source strides in bytes
    int64_t d_stream, d_layer, d_head, d_pos;   // destination strides in bytes
    int32_t n_layers, n_heads, n_tensors;
    int32_t n_streams, n_keep, n_src;
    int32_t row_bytes;
    const int32_t* kept_idx;
    int64_t idx_stride;
};
// Copies destination rows [row_begin, row_end) of every plane.
hipError_t launch_gather(const GatherArgs& a, int row_begin, int row_end, hipStream_t stream);
// The same for a cache held as one buffer per layer and tensor: a.src / a.dst and the layer strides of `a` are not
// used, layer l of tensor x starts at t.src[x][l] / t.dst[x][l]; a.n_layers <= kLayerTable.  The table travels in the
// kernel arguments (1 KB), so nothing has to be staged in device memory.
constexpr int kLayerTable = 32;
struct LayerTable {
    const char* src[2][kLayerTable];
    char* dst[2][kLayerTable];
};
hipError_t launch_gather_layers(const GatherArgs& a, const LayerTable& t, hipStream_t stream);
// Ragged batches, out of place: stream s holds held_dev[s] + (cu_new_dev[s+1] - cu_new_dev[s]) slots; its n_keep_dev[s] kept
// rows go to the destination (all of its rows while it is within its budget), nothing of a stream the selection flagged
// (n_keep_dev[s] < 0); a.n_keep and a.n_src are upper bounds.
hipError_t launch_gather_ragged(const GatherArgs& a, const int32_t* held_dev, const int32_t* cu_new_dev,
                                const int32_t* n_keep_dev, int32_t budget, hipStream_t stream);

// ---- gather_inplace.hip -----------------------------------------------------------------
// src and dst of `a` are the same buffers and layouts; kept_idx must be strictly ascending.  `scratch` is optional:
// with at least SIRLLM_INPLACE_WORKSPACE_BYTES of device memory the workgroups take their planes in ticket order
// (the call clears the counter itself), without it by block index.
hipError_t launch_gather_inplace(const GatherArgs& a, void* scratch, size_t scratch_bytes, hipStream_t stream);
// The same for a cache held as one buffer per layer and tensor (t.dst; a.n_layers <= kLayerTable).
hipError_t launch_gather_inplace_layers(const GatherArgs& a, const LayerTable& t, void* scratch, size_t scratch_bytes,
                                        hipStream_t stream);
// Ragged batches: stream s holds held_dev[s] + (cu_new_dev[s+1] - cu_new_dev[s]) slots and is compacted
// to `budget` slots only when it holds more and the selection did not flag it (n_keep_dev[s] >= 0); a.n_keep and
// a.n_src are upper bounds.
hipError_t launch_gather_inplace_ragged(const GatherArgs& a, const int32_t* held_dev, const int32_t* cu_new_dev,
                                        const int32_t* n_keep_dev, int32_t budget, void* scratch, size_t scratch_bytes,
                                        hipStream_t stream);

// ---- baseline.hip -----------------------------------------------------------------------
// kept_idx of the score-free policies; n_topk of `a` is the number of middle slots to keep.
hipError_t launch_baseline_comb(const SelectArgs& a, int interval, hipStream_t stream);   // stream / interval / keep-all
hipError_t launch_baseline_random(const SelectArgs& a, hipStream_t stream);               // needs n_cand > budget

// ---- fused.hip --------------------------------------------------------------------------
// Scoring and selection in one launch; only valid when score_select_fusable() says so (the new
// tokens all fall inside the recent window, so the selection never reads this turn's scores).
// The caller points sa.out_b at the tail of scores_out where the new scores belong.
bool score_select_fusable(const ScoreArgs& sa, const SelectArgs& se);
// The same for a ragged batch whose streams all bring at most n_recent new tokens (se.max_new <= se.n_recent).
bool score_select_ragged_fusable(const ScoreArgs& sa, const SelectArgs& se);
hipError_t launch_score_select_ragged(const ScoreArgs& sa, const SelectArgs& se, sirllm_dtype dt, hipStream_t stream);
hipError_t launch_score_select(const ScoreArgs& sa, const SelectArgs& se, sirllm_dtype dt, hipStream_t stream);

}  // namespace sirllm
