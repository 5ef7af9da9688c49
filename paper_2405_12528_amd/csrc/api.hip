// The exported C ABI of libsirllm (declared in sirllm.h): host-side argument validation and
// the order in which the kernels of one retention step are enqueued.
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "common.h"
#include "tuning.h"

namespace sirllm {
namespace tuning {
int get(const char* name, int dflt)
{
    static const bool active = [] {
        const char* t = std::getenv("SIRLLM_TUNE");
        return t && *t;
    }();
    if (!active) return dflt;
    const char* v = std::getenv(name);
    return (v && *v) ? std::atoi(v) : dflt;
}
}  // namespace tuning

namespace {

constexpr size_t kWorkspaceAlign = 256;

bool policy_ok(const sirllm_policy* p)
{
    if (!p) return false;
    if (p->n_sink < 0 || p->n_topk < 0 || p->n_recent < 0) return false;
    if (!(p->decay >= 0.0f) || std::isinf(p->decay)) return false;       // rejects NaN too
    return true;
}

int64_t budget_of(const sirllm_policy* p) { return (int64_t)p->n_sink + p->n_topk + p->n_recent; }

bool layout_ok(const sirllm_kv_layout* L)
{
    if (!L) return false;
    if (L->n_layers < 0 || L->n_kv_heads < 0 || L->head_dim < 0) return false;
    if (L->elem_bytes != 1 && L->elem_bytes != 2 && L->elem_bytes != 4 && L->elem_bytes != 8) return false;
    if (L->stride_stream < 0 || L->stride_layer < 0 || L->stride_head < 0 || L->stride_pos < 0) return false;
    if (L->stride_pos < L->head_dim) return false;
    return true;
}

// Bytes from the base pointer to one past the last byte a layout with n_pos slots can touch.
int64_t extent_bytes(const sirllm_kv_layout* L, int32_t n_streams, int32_t n_pos)
{
    if (n_streams <= 0 || n_pos <= 0 || L->n_layers <= 0 || L->n_kv_heads <= 0 || L->head_dim <= 0) return 0;
    const int64_t last = (int64_t)(n_streams - 1) * L->stride_stream + (int64_t)(L->n_layers - 1) * L->stride_layer +
                         (int64_t)(L->n_kv_heads - 1) * L->stride_head + (int64_t)(n_pos - 1) * L->stride_pos +
                         L->head_dim;
    return last * L->elem_bytes;
}

bool ranges_overlap(const void* a, int64_t a_bytes, const void* b, int64_t b_bytes)
{
    if (!a || !b || a_bytes <= 0 || b_bytes <= 0) return false;
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + (uint64_t)b_bytes && b0 < a0 + (uint64_t)a_bytes;
}

int workspace_check(void* workspace, size_t workspace_bytes, size_t need)
{
    if (need == 0) return SIRLLM_OK;
    if (!workspace || workspace_bytes < need) return SIRLLM_ERR_WORKSPACE;
    if (((uintptr_t)workspace & (kWorkspaceAlign - 1)) != 0) return SIRLLM_ERR_WORKSPACE;
    return SIRLLM_OK;
}

int validate_score(const void* logits, sirllm_dtype dt, int64_t n_rows, int32_t vocab, int64_t ld,
                   const int32_t* token_ids)
{
    if (dt != SIRLLM_F32 && dt != SIRLLM_BF16 && dt != SIRLLM_F16) return SIRLLM_ERR_UNSUPPORTED;
    if (n_rows < 0 || vocab < 1 || ld < vocab) return SIRLLM_ERR_INVALID_ARG;
    if (n_rows > 0x7fffffffLL) return SIRLLM_ERR_UNSUPPORTED;
    if (n_rows > 0 && (!logits || !token_ids)) return SIRLLM_ERR_INVALID_ARG;
    const uintptr_t esize = dt == SIRLLM_F32 ? 4 : 2;
    if (((uintptr_t)logits & (esize - 1)) != 0) return SIRLLM_ERR_INVALID_ARG;
    return SIRLLM_OK;
}

int validate_select(const float* scores, int64_t scores_stride, int32_t n_streams, int32_t n_held, int32_t n_new,
                    const sirllm_policy* policy, const int32_t* kept_idx, int64_t idx_stride,
                    const float* scores_out, int64_t out_stride)
{
    if (!policy_ok(policy)) return SIRLLM_ERR_INVALID_ARG;
    if (n_streams < 0 || n_held < 0 || n_new < 0) return SIRLLM_ERR_INVALID_ARG;
    const int64_t n_cand = (int64_t)n_held + n_new;
    if (n_cand > SIRLLM_MAX_CAND) return SIRLLM_ERR_UNSUPPORTED;
    if (n_streams == 0 || n_cand == 0) return SIRLLM_OK;
    if (!scores || !kept_idx || !scores_out) return SIRLLM_ERR_INVALID_ARG;
    const int64_t n_keep = n_cand < budget_of(policy) ? n_cand : budget_of(policy);
    if (scores_stride < n_cand || idx_stride < n_keep || out_stride < n_keep) return SIRLLM_ERR_INVALID_ARG;
    if (ranges_overlap(scores, ((int64_t)(n_streams - 1) * scores_stride + n_cand) * 4,
                       scores_out, ((int64_t)(n_streams - 1) * out_stride + n_keep) * 4))
        return SIRLLM_ERR_INVALID_ARG;
    return SIRLLM_OK;
}

int validate_compact(const void* k_src, const void* v_src, const sirllm_kv_layout* src, int32_t n_src,
                     void* k_dst, void* v_dst, const sirllm_kv_layout* dst, const int32_t* kept_idx,
                     int64_t idx_stride, int32_t n_streams, int32_t n_keep)
{
    if (!layout_ok(src) || !layout_ok(dst)) return SIRLLM_ERR_INVALID_ARG;
    if (src->n_layers != dst->n_layers || src->n_kv_heads != dst->n_kv_heads || src->head_dim != dst->head_dim ||
        src->elem_bytes != dst->elem_bytes)
        return SIRLLM_ERR_INVALID_ARG;
    if (n_streams < 0 || n_keep < 0 || n_src < 0) return SIRLLM_ERR_INVALID_ARG;
    if (n_streams == 0 || n_keep == 0) return SIRLLM_OK;
    if (!k_src || !k_dst || !kept_idx) return SIRLLM_ERR_INVALID_ARG;
    if ((v_src == nullptr) != (v_dst == nullptr)) return SIRLLM_ERR_INVALID_ARG;
    if (idx_stride < n_keep) return SIRLLM_ERR_INVALID_ARG;
    if ((int64_t)src->head_dim * src->elem_bytes * n_keep > 0x7fff0000LL) return SIRLLM_ERR_UNSUPPORTED;  // per-plane bytes
    const uintptr_t em = (uintptr_t)src->elem_bytes - 1;
    if (((uintptr_t)k_src & em) || ((uintptr_t)k_dst & em) || ((uintptr_t)v_src & em) || ((uintptr_t)v_dst & em))
        return SIRLLM_ERR_INVALID_ARG;
    const int64_t sb = extent_bytes(src, n_streams, n_src), db = extent_bytes(dst, n_streams, n_keep);
    const void* srcs[2] = {k_src, v_src};
    const void* dsts[2] = {k_dst, v_dst};
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 2; ++j)
            if (ranges_overlap(srcs[i], sb, dsts[j], db)) return SIRLLM_ERR_INVALID_ARG;
    if (ranges_overlap(k_dst, db, v_dst, db)) return SIRLLM_ERR_INVALID_ARG;
    return SIRLLM_OK;
}

SelectArgs make_select_args(const float* scores, int64_t scores_stride, int32_t n_streams, int32_t n_held,
                            int32_t n_new, const sirllm_policy* p, int32_t* kept_idx, int64_t idx_stride,
                            float* scores_out, int64_t out_stride)
{
    SelectArgs a;
    a.scores = scores; a.scores_stride = scores_stride;
    a.n_streams = n_streams; a.n_held = n_held; a.n_cand = n_held + n_new;
    a.n_sink = p->n_sink; a.n_topk = p->n_topk; a.n_recent = p->n_recent; a.decay = p->decay;
    a.kept_idx = kept_idx; a.idx_stride = idx_stride;
    a.scores_out = scores_out; a.out_stride = out_stride;
    a.seed_lo = a.seed_hi = a.turn_lo = a.turn_hi = 0;
    a.held_dev = nullptr; a.cu_new_dev = nullptr; a.n_keep_dev = nullptr; a.max_new = 0x7fffffff;
    return a;
}

GatherArgs make_gather_args(const void* k_src, const void* v_src, const sirllm_kv_layout* src, int32_t n_src,
                            void* k_dst, void* v_dst, const sirllm_kv_layout* dst, const int32_t* kept_idx,
                            int64_t idx_stride, int32_t n_streams, int32_t n_keep)
{
    GatherArgs g;
    const int64_t eb = src->elem_bytes;
    g.src[0] = (const char*)k_src; g.src[1] = (const char*)v_src;
    g.dst[0] = (char*)k_dst; g.dst[1] = (char*)v_dst;
    g.s_stream = src->stride_stream * eb; g.s_layer = src->stride_layer * eb;
    g.s_head = src->stride_head * eb; g.s_pos = src->stride_pos * eb;
    g.d_stream = dst->stride_stream * eb; g.d_layer = dst->stride_layer * eb;
    g.d_head = dst->stride_head * eb; g.d_pos = dst->stride_pos * eb;
    g.n_layers = src->n_layers; g.n_heads = src->n_kv_heads; g.n_tensors = v_src ? 2 : 1;
    g.n_streams = n_streams; g.n_keep = n_keep; g.n_src = n_src;
    g.row_bytes = (int32_t)((int64_t)src->head_dim * eb);
    g.kept_idx = kept_idx; g.idx_stride = idx_stride;
    // Slot-major caches ([slot][head][dim], or [slot][layer][head][dim]): the rows of consecutive heads (and then
    // of consecutive layers) of one slot lie back to back in both layouts, so they are one longer row of one
    // plane -- the copy then streams whole slots instead of head_dim-sized pieces a slot stride apart.
    const int64_t kMaxRowSpan = 0x7fffffffLL - 8192;      // keeps n_keep * (vectors per row) inside 32 bits for any vector width
    auto fits = [&](int64_t row) {
        return row <= g.s_pos && row <= g.d_pos && row <= (1 << 24) && (int64_t)n_keep * row <= kMaxRowSpan;
    };
    if (g.n_heads > 1 && g.s_head == g.row_bytes && g.d_head == g.row_bytes && fits((int64_t)g.row_bytes * g.n_heads)) {
        g.row_bytes *= g.n_heads;
        g.n_heads = 1;
    }
    if (g.n_heads == 1) {
        g.s_head = g.s_layer; g.d_head = g.d_layer;        // one head per layer: planes are a plain walk over layers
        if (g.n_layers > 1 && g.s_layer == g.row_bytes && g.d_layer == g.row_bytes &&
            fits((int64_t)g.row_bytes * g.n_layers)) {
            g.row_bytes *= g.n_layers;
            g.n_layers = 1;
        }
    }
    return g;
}

int hip_status(hipError_t e) { return e == hipSuccess ? SIRLLM_OK : SIRLLM_ERR_HIP; }

}  // namespace
}  // namespace sirllm

// ---- scratch of sirllm_decay_select_static ---------------------------------------------------
// Device memory that lives in the library's code object: every GPU the library runs on holds its own
// copy, at its own address, from module load until the process ends.  In host code the array's name is
// only a handle for hipGetSymbolAddress; the address it returns for the current device is what kernels,
// and everything else on the host, are given.
static __device__ __align__(256) uint32_t sirllm_static_scratch[SIRLLM_STATIC_SCRATCH_BYTES / sizeof(uint32_t)];

namespace sirllm {
namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};        // per device, resolved on the first call made with that device current

int static_scratch_of_current_device(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return SIRLLM_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return SIRLLM_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(sirllm_static_scratch)) != hipSuccess || !p) return SIRLLM_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return SIRLLM_OK;
}

}  // namespace
}  // namespace sirllm

using namespace sirllm;

extern "C" {

size_t sirllm_workspace_bytes(int32_t n_streams, int32_t n_cand, int64_t n_rows, int32_t vocab)
{
    (void)n_rows; (void)vocab;
    // Only the selection over more than 32768 slots per stream needs scratch (global histograms and per-tile
    // counts of its multi-workgroup radix select); every other kernel keeps its partial results in
    // registers and LDS.
    if (n_streams < 0 || n_cand < 0) return 0;
    return (select_large_scratch_bytes(n_streams, n_cand) + 255) / 256 * 256;
}

const char* sirllm_status_string(int status)
{
    switch (status) {
    case SIRLLM_OK:              return "ok";
    case SIRLLM_ERR_INVALID_ARG: return "invalid argument (null pointer, negative size, inconsistent shapes or overlapping buffers)";
    case SIRLLM_ERR_UNSUPPORTED: return "unsupported (size above a documented limit or unknown dtype)";
    case SIRLLM_ERR_WORKSPACE:   return "workspace too small or not 256-byte aligned";
    case SIRLLM_ERR_HIP:         return "HIP runtime error at kernel launch";
    default:                     return "unknown status";
    }
}

const char* sirllm_version(void) { return "0.1.0"; }

int sirllm_score(const void* logits, sirllm_dtype dt, int64_t n_rows, int32_t vocab, int64_t ld,
                 const int32_t* token_ids, float* scores_out, void* workspace, size_t workspace_bytes,
                 void* hip_stream)
{
    int rc = validate_score(logits, dt, n_rows, vocab, ld, token_ids);
    if (rc) return rc;
    if (n_rows == 0) return SIRLLM_OK;
    if (!scores_out) return SIRLLM_ERR_INVALID_ARG;
    rc = workspace_check(workspace, workspace_bytes, sirllm_workspace_bytes(0, 0, n_rows, vocab));
    if (rc) return rc;
    ScoreArgs a;
    a.logits = logits; a.ld = ld; a.vocab = vocab; a.token_ids = token_ids;
    a.n_rows = n_rows; a.rows_per_stream = n_rows;
    a.out_a = scores_out; a.stride_a = 0; a.out_b = nullptr; a.stride_b = 0;
    a.partial = nullptr; a.v_begin = 0; a.cu_rows = nullptr; a.held_dev = nullptr; a.n_streams_r = 0; a.budget_r = 0;
    return hip_status(launch_score(a, dt, (hipStream_t)hip_stream));
}

int sirllm_score_partial(const void* logits_chunk, sirllm_dtype dt, int64_t n_rows, int32_t n_cols, int64_t ld,
                         int32_t v_begin, const int32_t* token_ids, float* partial, void* hip_stream)
{
    int rc = validate_score(logits_chunk, dt, n_rows, n_cols, ld, token_ids);
    if (rc) return rc;
    if (v_begin < 0) return SIRLLM_ERR_INVALID_ARG;
    if (n_rows == 0) return SIRLLM_OK;
    if (!partial) return SIRLLM_ERR_INVALID_ARG;
    ScoreArgs a;
    a.logits = logits_chunk; a.ld = ld; a.vocab = n_cols; a.token_ids = token_ids;
    a.n_rows = n_rows; a.rows_per_stream = n_rows;
    a.out_a = nullptr; a.stride_a = 0; a.out_b = nullptr; a.stride_b = 0;
    a.partial = partial; a.v_begin = v_begin; a.cu_rows = nullptr; a.held_dev = nullptr; a.n_streams_r = 0; a.budget_r = 0;
    return hip_status(launch_score(a, dt, (hipStream_t)hip_stream));
}

int sirllm_score_merge(const float* partials, int32_t n_parts, int64_t part_stride, int64_t n_rows,
                       float* scores_out, void* hip_stream)
{
    if (n_parts < 1 || n_rows < 0 || n_rows > 0x7fffffffLL) return SIRLLM_ERR_INVALID_ARG;
    if (n_rows == 0) return SIRLLM_OK;
    if (!partials || !scores_out) return SIRLLM_ERR_INVALID_ARG;
    if (n_parts > 1 && part_stride < 3 * n_rows) return SIRLLM_ERR_INVALID_ARG;
    return hip_status(launch_score_merge(partials, n_parts, part_stride, n_rows, scores_out, (hipStream_t)hip_stream));
}

size_t sirllm_lmhead_workspace_bytes(int64_t n_rows, int32_t vocab)
{
    if (n_rows <= 0 || vocab <= 0) return 0;
    // one (m, s, z_tok) triple per row and vocabulary tile, each tile's block padded to 256 bytes
    const size_t per_tile = ((size_t)n_rows * 3 * sizeof(float) + 255) & ~(size_t)255;
    return per_tile * (size_t)lmhead_tiles_vocab(n_rows, vocab);
}

namespace {

int validate_lmhead(const void* hidden, int64_t ld_h, const void* weight, int64_t ld_w, sirllm_dtype dt,
                    int32_t d_model, int64_t n_rows, int32_t vocab, const int32_t* token_ids)
{
    if (n_rows < 0 || n_rows > 0x7fffffffLL || vocab < 1 || d_model < 1 || ld_h < d_model || ld_w < d_model)
        return SIRLLM_ERR_INVALID_ARG;
    if (dt != SIRLLM_F32 && dt != SIRLLM_BF16 && dt != SIRLLM_F16) return SIRLLM_ERR_INVALID_ARG;
    if (n_rows == 0) return SIRLLM_OK;
    if (!hidden || !weight || !token_ids) return SIRLLM_ERR_INVALID_ARG;
    if (dt == SIRLLM_F32) return SIRLLM_ERR_UNSUPPORTED;
    if ((d_model & 7) || (ld_h & 7) || (ld_w & 7) || ld_h >= (1 << 21) || ld_w >= (1 << 21) ||
        ((uintptr_t)hidden & 15) || ((uintptr_t)weight & 15))
        return SIRLLM_ERR_UNSUPPORTED;
    return SIRLLM_OK;
}

LmHeadArgs make_lmhead_args(const void* hidden, int64_t ld_h, const void* weight, int64_t ld_w, int32_t d_model,
                            int64_t n_rows, int32_t vocab, const int32_t* token_ids, void* workspace)
{
    LmHeadArgs a;
    a.hidden = hidden; a.weight = weight; a.ld_h = ld_h; a.ld_w = ld_w; a.d_model = d_model; a.vocab = vocab;
    a.n_rows = n_rows; a.token_ids = token_ids; a.partial = (float*)workspace;
    a.part_stride = (int64_t)((((size_t)n_rows * 3 * sizeof(float) + 255) & ~(size_t)255) / sizeof(float));
    a.n_vtiles = 0; a.n_ttiles = 0;
    return a;
}

}  // namespace

int sirllm_lmhead_score(const void* hidden, int64_t ld_h, const void* weight, int64_t ld_w, sirllm_dtype dt,
                        int32_t d_model, int64_t n_rows, int32_t vocab, const int32_t* token_ids,
                        float* scores_out, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    int rc = validate_lmhead(hidden, ld_h, weight, ld_w, dt, d_model, n_rows, vocab, token_ids);
    if (rc) return rc;
    if (n_rows == 0) return SIRLLM_OK;
    if (!scores_out) return SIRLLM_ERR_INVALID_ARG;
    rc = workspace_check(workspace, workspace_bytes, sirllm_lmhead_workspace_bytes(n_rows, vocab));
    if (rc) return rc;
    const LmHeadArgs a = make_lmhead_args(hidden, ld_h, weight, ld_w, d_model, n_rows, vocab, token_ids, workspace);
    return hip_status(launch_lmhead_score(a, dt, scores_out, n_rows, 0, (hipStream_t)hip_stream));
}

int sirllm_decay_select(const float* scores, int64_t scores_stride, int32_t n_streams, int32_t n_held,
                        int32_t n_new, const sirllm_policy* policy, int32_t* kept_idx, int64_t idx_stride,
                        float* scores_out, int64_t out_stride, void* workspace, size_t workspace_bytes,
                        void* hip_stream)
{
    int rc = validate_select(scores, scores_stride, n_streams, n_held, n_new, policy, kept_idx, idx_stride,
                             scores_out, out_stride);
    if (rc) return rc;
    const int32_t n_cand = n_held + n_new;
    if (n_streams == 0 || n_cand == 0) return SIRLLM_OK;
    rc = workspace_check(workspace, workspace_bytes, sirllm_workspace_bytes(n_streams, n_cand, 0, 0));
    if (rc) return rc;
    const SelectArgs a = make_select_args(scores, scores_stride, n_streams, n_held, n_new, policy, kept_idx,
                                          idx_stride, scores_out, out_stride);
    if ((int64_t)n_cand <= budget_of(policy)) return hip_status(launch_keep_all(a, (hipStream_t)hip_stream));
    if (n_cand > SIRLLM_SINGLE_WG_CAND) return hip_status(launch_select_large(a, workspace, (hipStream_t)hip_stream));
    return hip_status(launch_select(a, (hipStream_t)hip_stream));
}

int sirllm_decay_select_static(const float* scores, int64_t scores_stride, int32_t n_streams, int32_t n_held,
                               int32_t n_new, const sirllm_policy* policy, int32_t* kept_idx, int64_t idx_stride,
                               float* scores_out, int64_t out_stride, void* hip_stream)
{
    int rc = validate_select(scores, scores_stride, n_streams, n_held, n_new, policy, kept_idx, idx_stride,
                             scores_out, out_stride);
    if (rc) return rc;
    const int32_t n_cand = n_held + n_new;
    if (n_streams == 0 || n_cand == 0) return SIRLLM_OK;
    const SelectArgs a = make_select_args(scores, scores_stride, n_streams, n_held, n_new, policy, kept_idx,
                                          idx_stride, scores_out, out_stride);
    if ((int64_t)n_cand <= budget_of(policy)) return hip_status(launch_keep_all(a, (hipStream_t)hip_stream));
    if (n_cand <= SIRLLM_SINGLE_WG_CAND) return hip_status(launch_select(a, (hipStream_t)hip_stream));
    // the multi-workgroup selection: its histograms and per-tile counts go into the static array, which the
    // first launch of the call clears (a kernel, not a memset)
    if (select_large_scratch_bytes(n_streams, n_cand) > (size_t)SIRLLM_STATIC_SCRATCH_BYTES) return SIRLLM_ERR_UNSUPPORTED;
    void* scratch = nullptr;
    rc = static_scratch_of_current_device(&scratch);
    if (rc) return rc;
    return hip_status(launch_select_large(a, scratch, (hipStream_t)hip_stream));
}

int sirllm_baseline_select(sirllm_baseline kind, int32_t n_streams, int32_t n_cand, const sirllm_policy* policy,
                           uint64_t seed, uint64_t turn, int32_t* kept_idx, int64_t idx_stride,
                           int32_t* n_keep_out, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (kind != SIRLLM_BASELINE_STREAM && kind != SIRLLM_BASELINE_INTERVAL && kind != SIRLLM_BASELINE_RANDOM)
        return SIRLLM_ERR_UNSUPPORTED;
    if (!policy || policy->n_sink < 0 || policy->n_topk < 0 || policy->n_recent < 0) return SIRLLM_ERR_INVALID_ARG;
    if (n_streams < 0 || n_cand < 0) return SIRLLM_ERR_INVALID_ARG;
    if (n_cand > SIRLLM_MAX_CAND) return SIRLLM_ERR_UNSUPPORTED;
    sirllm_policy p = *policy;
    p.decay = 1.0f;
    if (kind == SIRLLM_BASELINE_STREAM) p.n_topk = 0;
    const int64_t budget = budget_of(&p);
    const int32_t n_keep = (int32_t)((int64_t)n_cand < budget ? n_cand : budget);
    if (n_keep_out) *n_keep_out = n_keep;
    if (n_streams == 0 || n_cand == 0) return SIRLLM_OK;
    if (!kept_idx || idx_stride < n_keep) return SIRLLM_ERR_INVALID_ARG;
    SelectArgs a = make_select_args(nullptr, 0, n_streams, n_cand, 0, &p, kept_idx, idx_stride, nullptr, 0);
    a.seed_lo = (uint32_t)seed; a.seed_hi = (uint32_t)(seed >> 32);
    a.turn_lo = (uint32_t)turn; a.turn_hi = (uint32_t)(turn >> 32);
    hipStream_t stream = (hipStream_t)hip_stream;
    if ((int64_t)n_cand <= budget) return hip_status(launch_baseline_comb(a, 0, stream));
    if (kind == SIRLLM_BASELINE_RANDOM && p.n_topk > 0) {
        if (n_cand <= SIRLLM_SINGLE_WG_CAND) return hip_status(launch_baseline_random(a, stream));
        // more slots than one workgroup holds: the multi-workgroup selection on the generator's draws
        const int rc = workspace_check(workspace, workspace_bytes, sirllm_workspace_bytes(n_streams, n_cand, 0, 0));
        if (rc) return rc;
        return hip_status(launch_select_large(a, workspace, stream, true));
    }
    int interval = 1;
    if (p.n_topk > 0) {
        interval = (n_cand - p.n_sink - p.n_recent) / p.n_topk;
        if (interval < 1) interval = 1;
    }
    return hip_status(launch_baseline_comb(a, interval, stream));
}

int sirllm_compact_kv(const void* k_src, const void* v_src, const sirllm_kv_layout* src, int32_t n_src,
                      void* k_dst, void* v_dst, const sirllm_kv_layout* dst, const int32_t* kept_idx,
                      int64_t idx_stride, int32_t n_streams, int32_t n_keep, void* hip_stream)
{
    int rc = validate_compact(k_src, v_src, src, n_src, k_dst, v_dst, dst, kept_idx, idx_stride, n_streams, n_keep);
    if (rc) return rc;
    if (n_streams == 0 || n_keep == 0) return SIRLLM_OK;
    const GatherArgs g = make_gather_args(k_src, v_src, src, n_src, k_dst, v_dst, dst, kept_idx, idx_stride,
                                          n_streams, n_keep);
    return hip_status(launch_gather(g, 0, n_keep, (hipStream_t)hip_stream));
}

int sirllm_compact_kv_layers(const void* const* k_src, const void* const* v_src, const sirllm_kv_layout* src,
                             int32_t n_src, void* const* k_dst, void* const* v_dst, const sirllm_kv_layout* dst,
                             const int32_t* kept_idx, int64_t idx_stride, int32_t n_streams, int32_t n_keep,
                             void* hip_stream)
{
    if (!layout_ok(src) || !layout_ok(dst)) return SIRLLM_ERR_INVALID_ARG;
    if (src->n_layers != dst->n_layers || src->n_kv_heads != dst->n_kv_heads || src->head_dim != dst->head_dim ||
        src->elem_bytes != dst->elem_bytes)
        return SIRLLM_ERR_INVALID_ARG;
    if (n_streams < 0 || n_keep < 0 || n_src < 0) return SIRLLM_ERR_INVALID_ARG;
    const int32_t n_layers = src->n_layers;
    if (n_streams == 0 || n_keep == 0 || n_layers == 0) return SIRLLM_OK;
    if (!k_src || !k_dst || !kept_idx || idx_stride < n_keep) return SIRLLM_ERR_INVALID_ARG;
    if ((v_src == nullptr) != (v_dst == nullptr)) return SIRLLM_ERR_INVALID_ARG;
    if ((int64_t)src->head_dim * src->elem_bytes * n_keep > 0x7fff0000LL) return SIRLLM_ERR_UNSUPPORTED;
    // one layer of either side: the layouts with the layer dimension taken out
    sirllm_kv_layout s1 = *src, d1 = *dst;
    s1.n_layers = d1.n_layers = 1;
    s1.stride_layer = d1.stride_layer = 0;
    const int64_t sb = extent_bytes(&s1, n_streams, n_src), db = extent_bytes(&d1, n_streams, n_keep);
    const uintptr_t em = (uintptr_t)src->elem_bytes - 1;
    const int n_tensors = v_src ? 2 : 1;
    const void* const* srcs[2] = {k_src, v_src};
    void* const* dsts[2] = {k_dst, v_dst};
    for (int x = 0; x < n_tensors; ++x)
        for (int l = 0; l < n_layers; ++l) {
            if (!srcs[x][l] || !dsts[x][l]) return SIRLLM_ERR_INVALID_ARG;
            if (((uintptr_t)srcs[x][l] & em) || ((uintptr_t)dsts[x][l] & em)) return SIRLLM_ERR_INVALID_ARG;
        }
    // no destination buffer may overlap a source buffer or another destination buffer
    for (int x = 0; x < n_tensors; ++x)
        for (int l = 0; l < n_layers; ++l)
            for (int y = 0; y < n_tensors; ++y)
                for (int m = 0; m < n_layers; ++m) {
                    if (ranges_overlap(dsts[x][l], db, srcs[y][m], sb)) return SIRLLM_ERR_INVALID_ARG;
                    if ((x != y || l != m) && ranges_overlap(dsts[x][l], db, dsts[y][m], db)) return SIRLLM_ERR_INVALID_ARG;
                }
    // the layers go into the kernel's arguments kLayerTable at a time
    for (int l0 = 0; l0 < n_layers; l0 += kLayerTable) {
        const int nl = n_layers - l0 < kLayerTable ? n_layers - l0 : kLayerTable;
        s1.n_layers = d1.n_layers = nl;
        GatherArgs g = make_gather_args(k_src[l0], v_src ? v_src[l0] : nullptr, &s1, n_src, k_dst[l0],
                                        v_dst ? v_dst[l0] : nullptr, &d1, kept_idx, idx_stride, n_streams, n_keep);
        g.src[0] = g.src[1] = nullptr;                       // the table below is what the kernel reads
        g.dst[0] = g.dst[1] = nullptr;
        LayerTable t;
        for (int x = 0; x < 2; ++x)
            for (int l = 0; l < kLayerTable; ++l) {
                const bool live = x < n_tensors && l < nl;
                t.src[x][l] = live ? (const char*)srcs[x][l0 + l] : nullptr;
                t.dst[x][l] = live ? (char*)dsts[x][l0 + l] : nullptr;
            }
        const int rc = hip_status(launch_gather_layers(g, t, (hipStream_t)hip_stream));
        if (rc) return rc;
    }
    return SIRLLM_OK;
}

int sirllm_compact_kv_inplace(void* k, void* v, const sirllm_kv_layout* layout, int32_t n_src,
                              const int32_t* kept_idx, int64_t idx_stride, int32_t n_streams, int32_t n_keep,
                              void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!layout_ok(layout)) return SIRLLM_ERR_INVALID_ARG;
    if (n_streams < 0 || n_keep < 0 || n_src < 0 || n_keep > n_src) return SIRLLM_ERR_INVALID_ARG;
    if (n_streams == 0 || n_keep == 0) return SIRLLM_OK;
    if (!k || !kept_idx || idx_stride < n_keep) return SIRLLM_ERR_INVALID_ARG;
    if ((int64_t)layout->head_dim * layout->elem_bytes * n_keep > 0x7fff0000LL) return SIRLLM_ERR_UNSUPPORTED;
    const uintptr_t em = (uintptr_t)layout->elem_bytes - 1;
    if (((uintptr_t)k & em) || ((uintptr_t)v & em)) return SIRLLM_ERR_INVALID_ARG;
    if (ranges_overlap(k, extent_bytes(layout, n_streams, n_src), v, extent_bytes(layout, n_streams, n_src)))
        return SIRLLM_ERR_INVALID_ARG;
    if (workspace && ((uintptr_t)workspace & (kWorkspaceAlign - 1)) != 0) return SIRLLM_ERR_WORKSPACE;
    const GatherArgs g = make_gather_args(k, v, layout, n_src, k, v, layout, kept_idx, idx_stride, n_streams, n_keep);
    return hip_status(launch_gather_inplace(g, workspace, workspace ? workspace_bytes : 0, (hipStream_t)hip_stream));
}

int sirllm_compact_kv_inplace_layers(void* const* k, void* const* v, const sirllm_kv_layout* layout, int32_t n_src,
                                     const int32_t* kept_idx, int64_t idx_stride, int32_t n_streams, int32_t n_keep,
                                     void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!layout_ok(layout)) return SIRLLM_ERR_INVALID_ARG;
    if (n_streams < 0 || n_keep < 0 || n_src < 0 || n_keep > n_src) return SIRLLM_ERR_INVALID_ARG;
    const int32_t n_layers = layout->n_layers;
    if (n_streams == 0 || n_keep == 0 || n_layers == 0) return SIRLLM_OK;
    if (!k || !kept_idx || idx_stride < n_keep) return SIRLLM_ERR_INVALID_ARG;
    if ((int64_t)layout->head_dim * layout->elem_bytes * n_keep > 0x7fff0000LL) return SIRLLM_ERR_UNSUPPORTED;
    if (workspace && ((uintptr_t)workspace & (kWorkspaceAlign - 1)) != 0) return SIRLLM_ERR_WORKSPACE;
    sirllm_kv_layout one = *layout;                          // one layer: the layout with the layer dimension taken out
    one.n_layers = 1;
    one.stride_layer = 0;
    const int64_t bytes = extent_bytes(&one, n_streams, n_src);
    const uintptr_t em = (uintptr_t)layout->elem_bytes - 1;
    const int n_tensors = v ? 2 : 1;
    void* const* bufs[2] = {k, v};
    for (int x = 0; x < n_tensors; ++x)
        for (int l = 0; l < n_layers; ++l) {
            if (!bufs[x][l] || ((uintptr_t)bufs[x][l] & em)) return SIRLLM_ERR_INVALID_ARG;
            for (int y = 0; y <= x; ++y)
                for (int m = 0; m < (y == x ? l : n_layers); ++m)
                    if (ranges_overlap(bufs[x][l], bytes, bufs[y][m], bytes)) return SIRLLM_ERR_INVALID_ARG;
        }
    for (int l0 = 0; l0 < n_layers; l0 += kLayerTable) {
        const int nl = n_layers - l0 < kLayerTable ? n_layers - l0 : kLayerTable;
        one.n_layers = nl;
        GatherArgs g = make_gather_args(k[l0], v ? v[l0] : nullptr, &one, n_src, k[l0], v ? v[l0] : nullptr, &one, kept_idx,
                                        idx_stride, n_streams, n_keep);
        g.src[0] = g.src[1] = nullptr;                       // the table below is what the kernel reads
        g.dst[0] = g.dst[1] = nullptr;
        LayerTable t;
        for (int x = 0; x < 2; ++x)
            for (int l = 0; l < kLayerTable; ++l) {
                char* p = (x < n_tensors && l < nl) ? (char*)bufs[x][l0 + l] : nullptr;
                t.src[x][l] = p;
                t.dst[x][l] = p;
            }
        const int rc = hip_status(launch_gather_inplace_layers(g, t, workspace, workspace ? workspace_bytes : 0,
                                                               (hipStream_t)hip_stream));
        if (rc) return rc;
    }
    return SIRLLM_OK;
}

namespace {

// The part of a step in front of the K/V movement: E_t = Entropy(new tokens) behind the held scores, E <- E * eta on
// the held part, Id = sink + Top_k + recent, E <- E[Id].  All arguments are validated by the caller.
int score_and_select(const void* logits, sirllm_dtype dt, int32_t vocab, int64_t ld, const int32_t* token_ids,
                     float* scores, int64_t scores_stride, int32_t n_streams, int32_t n_held, int32_t n_new,
                     const sirllm_policy* policy, int32_t* kept_idx, int64_t idx_stride, float* scores_out,
                     int64_t out_stride, void* workspace, hipStream_t stream)
{
    const int64_t n_rows = (int64_t)n_streams * n_new;
    const int32_t n_cand = n_held + n_new;
    const bool evict = (int64_t)n_cand > budget_of(policy);
    const int32_t n_keep = evict ? (int32_t)budget_of(policy) : n_cand;
    ScoreArgs a;
    a.logits = logits; a.ld = ld; a.vocab = vocab; a.token_ids = token_ids;
    a.n_rows = n_rows; a.rows_per_stream = n_new > 0 ? n_new : 1;
    a.out_a = scores + n_held; a.stride_a = scores_stride; a.out_b = nullptr; a.stride_b = 0;
    a.partial = nullptr; a.v_begin = 0; a.cu_rows = nullptr; a.held_dev = nullptr; a.n_streams_r = 0; a.budget_r = 0;
    const SelectArgs s = make_select_args(scores, scores_stride, n_streams, n_held, n_new, policy, kept_idx,
                                          idx_stride, scores_out, out_stride);
    if (evict && score_select_fusable(a, s)) {
        // The new tokens all sit in the recent window: Top_k does not look at this turn's scores, so
        // one launch scores the rows and selects at the same time.  New token t of a stream ends up
        // at in-cache position n_keep - n_new + t; the scoring workgroups write it there themselves.
        a.out_b = scores_out + (n_keep - n_new); a.stride_b = out_stride;
        return hip_status(launch_score_select(a, s, dt, stream));
    }
    if (n_rows > 0) {
        const int rc = hip_status(launch_score(a, dt, stream));
        if (rc) return rc;
    }
    if (!evict) return hip_status(launch_keep_all(s, stream));
    return hip_status(n_cand > SIRLLM_SINGLE_WG_CAND ? launch_select_large(s, workspace, stream) : launch_select(s, stream));
}

}  // namespace

int sirllm_score_select(const void* logits, sirllm_dtype dt, int32_t vocab, int64_t ld, const int32_t* token_ids,
                        float* scores, int64_t scores_stride, int32_t n_streams, int32_t n_held, int32_t n_new,
                        const sirllm_policy* policy, int32_t* kept_idx, int64_t idx_stride,
                        float* scores_out, int64_t out_stride, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (n_streams < 0 || n_held < 0 || n_new < 0) return SIRLLM_ERR_INVALID_ARG;
    int rc = validate_score(logits, dt, (int64_t)n_streams * n_new, vocab, ld, token_ids);
    if (rc) return rc;
    rc = validate_select(scores, scores_stride, n_streams, n_held, n_new, policy, kept_idx, idx_stride,
                         scores_out, out_stride);
    if (rc) return rc;
    if (n_streams == 0 || n_held + n_new == 0) return SIRLLM_OK;
    rc = workspace_check(workspace, workspace_bytes, sirllm_workspace_bytes(n_streams, n_held + n_new, 0, 0));
    if (rc) return rc;
    return score_and_select(logits, dt, vocab, ld, token_ids, scores, scores_stride, n_streams, n_held, n_new, policy,
                            kept_idx, idx_stride, scores_out, out_stride, workspace, (hipStream_t)hip_stream);
}

int sirllm_step(const void* logits, sirllm_dtype dt, int32_t vocab, int64_t ld, const int32_t* token_ids,
                float* scores, int64_t scores_stride, int32_t n_streams, int32_t n_held, int32_t n_new,
                const sirllm_policy* policy, const void* k_src, const void* v_src, const sirllm_kv_layout* src,
                void* k_dst, void* v_dst, const sirllm_kv_layout* dst, int32_t* kept_idx, int64_t idx_stride,
                float* scores_out, int64_t out_stride, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (n_streams < 0 || n_held < 0 || n_new < 0) return SIRLLM_ERR_INVALID_ARG;
    const int64_t n_rows = (int64_t)n_streams * n_new;
    int rc = validate_score(logits, dt, n_rows, vocab, ld, token_ids);
    if (rc) return rc;
    rc = validate_select(scores, scores_stride, n_streams, n_held, n_new, policy, kept_idx, idx_stride,
                         scores_out, out_stride);
    if (rc) return rc;
    const int32_t n_cand = n_held + n_new;
    if (n_streams == 0 || n_cand == 0) return SIRLLM_OK;
    const bool evict = (int64_t)n_cand > budget_of(policy);
    const int32_t n_keep = evict ? (int32_t)budget_of(policy) : n_cand;
    if (evict) {
        rc = validate_compact(k_src, v_src, src, n_cand, k_dst, v_dst, dst, kept_idx, idx_stride, n_streams, n_keep);
        if (rc) return rc;
    }
    rc = workspace_check(workspace, workspace_bytes, sirllm_workspace_bytes(n_streams, n_cand, n_rows, vocab));
    if (rc) return rc;
    hipStream_t stream = (hipStream_t)hip_stream;
    rc = score_and_select(logits, dt, vocab, ld, token_ids, scores, scores_stride, n_streams, n_held, n_new, policy,
                          kept_idx, idx_stride, scores_out, out_stride, workspace, stream);
    if (rc || !evict) return rc;
    // KV <- KV[Id]
    const GatherArgs g = make_gather_args(k_src, v_src, src, n_cand, k_dst, v_dst, dst, kept_idx, idx_stride,
                                          n_streams, n_keep);
    return hip_status(launch_gather(g, 0, n_keep, stream));
}

size_t sirllm_step_lmhead_workspace_bytes(int32_t n_streams, int32_t n_cand, int64_t n_rows, int32_t vocab)
{
    return sirllm_lmhead_workspace_bytes(n_rows, vocab) + sirllm_workspace_bytes(n_streams, n_cand, 0, 0);
}

int sirllm_step_lmhead(const void* hidden, int64_t ld_h, const void* weight, int64_t ld_w, sirllm_dtype dt,
                       int32_t d_model, int32_t vocab, const int32_t* token_ids,
                       float* scores, int64_t scores_stride, int32_t n_streams, int32_t n_held, int32_t n_new,
                       const sirllm_policy* policy, const void* k_src, const void* v_src, const sirllm_kv_layout* src,
                       void* k_dst, void* v_dst, const sirllm_kv_layout* dst, int32_t* kept_idx, int64_t idx_stride,
                       float* scores_out, int64_t out_stride, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (n_streams < 0 || n_held < 0 || n_new < 0) return SIRLLM_ERR_INVALID_ARG;
    const int64_t n_rows = (int64_t)n_streams * n_new;
    int rc = validate_lmhead(hidden, ld_h, weight, ld_w, dt, d_model, n_rows, vocab, token_ids);
    if (rc) return rc;
    rc = validate_select(scores, scores_stride, n_streams, n_held, n_new, policy, kept_idx, idx_stride,
                         scores_out, out_stride);
    if (rc) return rc;
    const int32_t n_cand = n_held + n_new;
    if (n_streams == 0 || n_cand == 0) return SIRLLM_OK;
    const bool evict = (int64_t)n_cand > budget_of(policy);
    const int32_t n_keep = evict ? (int32_t)budget_of(policy) : n_cand;
    if (evict) {
        rc = validate_compact(k_src, v_src, src, n_cand, k_dst, v_dst, dst, kept_idx, idx_stride, n_streams, n_keep);
        if (rc) return rc;
    }
    const size_t lm_bytes = sirllm_lmhead_workspace_bytes(n_rows, vocab);
    rc = workspace_check(workspace, workspace_bytes, sirllm_step_lmhead_workspace_bytes(n_streams, n_cand, n_rows, vocab));
    if (rc) return rc;
    hipStream_t stream = (hipStream_t)hip_stream;

    // E_t = Entropy(new tokens) from z = h W^T, appended behind the held scores
    if (n_rows > 0) {
        const LmHeadArgs a = make_lmhead_args(hidden, ld_h, weight, ld_w, d_model, n_rows, vocab, token_ids, workspace);
        rc = hip_status(launch_lmhead_score(a, dt, scores + n_held, n_new, scores_stride, stream));
        if (rc) return rc;
    }
    // E <- E * eta on the held part; Id = sink + Top_k + recent; E <- E[Id]
    const SelectArgs s = make_select_args(scores, scores_stride, n_streams, n_held, n_new, policy, kept_idx,
                                          idx_stride, scores_out, out_stride);
    if (!evict) return hip_status(launch_keep_all(s, stream));
    rc = hip_status(n_cand > SIRLLM_SINGLE_WG_CAND ? launch_select_large(s, (char*)workspace + lm_bytes, stream)
                                                     : launch_select(s, stream));
    if (rc) return rc;
    // KV <- KV[Id]
    const GatherArgs g = make_gather_args(k_src, v_src, src, n_cand, k_dst, v_dst, dst, kept_idx, idx_stride,
                                          n_streams, n_keep);
    return hip_status(launch_gather(g, 0, n_keep, stream));
}

namespace {

// What sirllm_step_ragged and sirllm_step_lmhead_ragged share: the checks of everything but the scoring operands ...
int validate_ragged(float* scores, int64_t scores_stride, int32_t n_streams, const int32_t* n_held,
                    const int32_t* cu_new, int64_t total_new, int32_t max_cand, int32_t max_new,
                    const sirllm_policy* policy, void* k, void* v, const sirllm_kv_layout* layout, int32_t* kept_idx,
                    int64_t idx_stride, float* scores_out, int64_t out_stride, int32_t* n_keep_out)
{
    if (n_streams < 0 || total_new < 0 || max_cand < 0 || max_new < 0 || max_new > max_cand) return SIRLLM_ERR_INVALID_ARG;
    if (!policy_ok(policy)) return SIRLLM_ERR_INVALID_ARG;
    if (max_cand > SIRLLM_MAX_CAND) return SIRLLM_ERR_UNSUPPORTED;
    if (n_streams == 0) return SIRLLM_OK;
    if (!n_held || !cu_new || !n_keep_out || !scores || !kept_idx || !scores_out) return SIRLLM_ERR_INVALID_ARG;
    const int64_t budget = budget_of(policy);
    const int64_t keep_bound = max_cand < budget ? max_cand : budget;
    if (scores_stride < max_cand || idx_stride < keep_bound || out_stride < keep_bound) return SIRLLM_ERR_INVALID_ARG;
    if (ranges_overlap(scores, ((int64_t)(n_streams - 1) * scores_stride + max_cand) * 4,
                       scores_out, ((int64_t)(n_streams - 1) * out_stride + keep_bound) * 4))
        return SIRLLM_ERR_INVALID_ARG;
    if (max_cand > budget) {
        if (!layout_ok(layout) || !k) return SIRLLM_ERR_INVALID_ARG;
        if ((int64_t)layout->head_dim * layout->elem_bytes * budget > 0x7fff0000LL) return SIRLLM_ERR_UNSUPPORTED;
        const uintptr_t em = (uintptr_t)layout->elem_bytes - 1;
        if (((uintptr_t)k & em) || ((uintptr_t)v & em)) return SIRLLM_ERR_INVALID_ARG;
        if (ranges_overlap(k, extent_bytes(layout, n_streams, max_cand), v, extent_bytes(layout, n_streams, max_cand)))
            return SIRLLM_ERR_INVALID_ARG;
    }
    return SIRLLM_OK;
}

SelectArgs make_ragged_select_args(float* scores, int64_t scores_stride, int32_t n_streams, const int32_t* n_held,
                                   const int32_t* cu_new, int32_t max_cand, int32_t max_new, const sirllm_policy* policy,
                                   int32_t* kept_idx, int64_t idx_stride, float* scores_out, int64_t out_stride,
                                   int32_t* n_keep_out)
{
    SelectArgs s = make_select_args(scores, scores_stride, n_streams, 0, max_cand, policy, kept_idx, idx_stride,
                                    scores_out, out_stride);
    s.held_dev = n_held; s.cu_new_dev = cu_new; s.n_keep_dev = n_keep_out; s.max_new = max_new;
    return s;
}

// ... and the part behind the scores: E <- E * eta, Id, E <- E[Id] per stream, then KV <- KV[Id] in place.
// `scratch` is the selection's scratch when a stream may hold more slots than one workgroup selects (then required
// and already checked), and the in-place compaction's ticket afterwards (stream order keeps the two uses apart).
// Where a ragged step compacts to: nowhere else (k_dst null: in place), or a second pair of buffers.
struct RaggedDst {
    void* k_dst;
    void* v_dst;
    const sirllm_kv_layout* layout;
};

// KV <- KV[Id] for the streams of a ragged batch that exceed their budget: in place, or into dst.
int ragged_compact(const SelectArgs& s, int32_t max_cand, int64_t budget, void* k, void* v, const sirllm_kv_layout* layout,
                   const RaggedDst& dst, void* scratch, size_t scratch_bytes, hipStream_t stream)
{
    if (dst.k_dst) {
        // every accepted stream moves: compacted when over its budget, as it is otherwise
        const int32_t keep_bound = (int32_t)(max_cand < budget ? max_cand : budget);
        if (keep_bound == 0) return SIRLLM_OK;
        const GatherArgs g = make_gather_args(k, v, layout, max_cand, dst.k_dst, dst.v_dst, dst.layout, s.kept_idx, s.idx_stride,
                                              s.n_streams, keep_bound);
        return hip_status(launch_gather_ragged(g, s.held_dev, s.cu_new_dev, s.n_keep_dev, (int32_t)budget, stream));
    }
    if (max_cand <= budget) return SIRLLM_OK;
    const GatherArgs g = make_gather_args(k, v, layout, max_cand, k, v, layout, s.kept_idx, s.idx_stride, s.n_streams,
                                          (int32_t)budget);
    // with a workspace the compacting workgroups take their planes in ticket order
    return hip_status(launch_gather_inplace_ragged(g, s.held_dev, s.cu_new_dev, s.n_keep_dev, (int32_t)budget, scratch,
                                                   scratch ? scratch_bytes : 0, stream));
}

int ragged_select_compact(const SelectArgs& s, int32_t max_cand, const sirllm_policy* policy, void* k, void* v,
                          const sirllm_kv_layout* layout, const RaggedDst& dst, void* scratch, size_t scratch_bytes,
                          hipStream_t stream)
{
    const int rc = hip_status(max_cand > SIRLLM_SINGLE_WG_CAND ? launch_select_large(s, scratch, stream)
                                                                : launch_select_ragged(s, stream));
    if (rc) return rc;
    return ragged_compact(s, max_cand, budget_of(policy), k, v, layout, dst, scratch, scratch_bytes, stream);
}

}  // namespace

namespace {

int step_ragged_common(const void* logits, sirllm_dtype dt, int32_t vocab, int64_t ld, const int32_t* token_ids,
                       float* scores, int64_t scores_stride, int32_t n_streams, const int32_t* n_held,
                       const int32_t* cu_new, int64_t total_new, int32_t max_cand, int32_t max_new,
                       const sirllm_policy* policy,
                       void* k, void* v, const sirllm_kv_layout* layout, const RaggedDst& dst,
                       int32_t* kept_idx, int64_t idx_stride,
                       float* scores_out, int64_t out_stride, int32_t* n_keep_out, void* workspace,
                       size_t workspace_bytes, void* hip_stream)
{
    using namespace sirllm;
    if (total_new < 0) return SIRLLM_ERR_INVALID_ARG;
    int rc = validate_score(logits, dt, total_new, vocab, ld, token_ids);
    if (rc) return rc;
    rc = validate_ragged(scores, scores_stride, n_streams, n_held, cu_new, total_new, max_cand, max_new, policy, k, v,
                         layout, kept_idx, idx_stride, scores_out, out_stride, n_keep_out);
    if (rc || n_streams == 0) return rc;
    rc = workspace_check(workspace, workspace_bytes, sirllm_workspace_bytes(n_streams, max_cand, total_new, vocab));
    if (rc) return rc;
    if (workspace && ((uintptr_t)workspace & (kWorkspaceAlign - 1)) != 0) return SIRLLM_ERR_WORKSPACE;
    hipStream_t stream = (hipStream_t)hip_stream;
    const int64_t budget = budget_of(policy);

    ScoreArgs a;
    a.logits = logits; a.ld = ld; a.vocab = vocab; a.token_ids = token_ids;
    a.n_rows = total_new; a.rows_per_stream = 1;
    a.out_a = scores; a.stride_a = scores_stride; a.out_b = nullptr; a.stride_b = 0;
    a.partial = nullptr; a.v_begin = 0;
    a.cu_rows = cu_new; a.held_dev = n_held; a.n_streams_r = n_streams; a.budget_r = (int32_t)(budget < 0x7fffffff ? budget : 0x7fffffff);
    const SelectArgs s = make_ragged_select_args(scores, scores_stride, n_streams, n_held, cu_new, max_cand, max_new,
                                                 policy, kept_idx, idx_stride, scores_out, out_stride, n_keep_out);
    if (score_select_ragged_fusable(a, s)) {
        // no stream brings more new tokens than the recent window holds: score and select in one launch
        a.out_b = scores_out; a.stride_b = out_stride;
        rc = hip_status(launch_score_select_ragged(a, s, dt, stream));
        if (rc) return rc;
        return ragged_compact(s, max_cand, budget, k, v, layout, dst, workspace, workspace ? workspace_bytes : 0, stream);
    }
    if (total_new > 0) {
        rc = hip_status(launch_score(a, dt, stream));
        if (rc) return rc;
    }
    return ragged_select_compact(s, max_cand, policy, k, v, layout, dst, workspace, workspace_bytes, stream);
}

// The destination side of a ragged step with two buffer pairs, and source against destination (the source side is
// checked with the rest of the step).
int validate_ragged_dst(int32_t max_cand, int32_t n_streams, const sirllm_policy* policy, const void* k_src, const void* v_src,
                        const sirllm_kv_layout* src, void* k_dst, void* v_dst, const sirllm_kv_layout* dst,
                        const int32_t* kept_idx, int64_t idx_stride)
{
    if (max_cand < 0 || n_streams < 0 || !policy_ok(policy)) return SIRLLM_ERR_INVALID_ARG;
    const int64_t budget = budget_of(policy);
    if (n_streams > 0 && max_cand > 0) {
        const int rc = validate_compact(k_src, v_src, src, max_cand, k_dst, v_dst, dst, kept_idx, idx_stride, n_streams,
                                        (int32_t)(max_cand < budget ? max_cand : budget));
        if (rc) return rc;
        if (budget > 0 && !k_dst) return SIRLLM_ERR_INVALID_ARG;
    }
    return SIRLLM_OK;
}

size_t lmhead_ragged_workspace_bytes(int32_t n_streams, int32_t max_cand, int64_t total_new, int32_t vocab)
{
    const size_t sel = sirllm_workspace_bytes(n_streams, max_cand, 0, 0);
    return sirllm_lmhead_workspace_bytes(total_new, vocab) +
           (sel > (size_t)SIRLLM_INPLACE_WORKSPACE_BYTES ? sel : (size_t)SIRLLM_INPLACE_WORKSPACE_BYTES);
}

int step_lmhead_ragged_common(const void* hidden, int64_t ld_h, const void* weight, int64_t ld_w, sirllm_dtype dt,
                              int32_t d_model, int32_t vocab, const int32_t* token_ids,
                              float* scores, int64_t scores_stride, int32_t n_streams, const int32_t* n_held,
                              const int32_t* cu_new, int64_t total_new, int32_t max_cand, int32_t max_new,
                              const sirllm_policy* policy, void* k, void* v, const sirllm_kv_layout* layout,
                              const RaggedDst& dst, int32_t* kept_idx, int64_t idx_stride, float* scores_out, int64_t out_stride,
                              int32_t* n_keep_out, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (total_new < 0) return SIRLLM_ERR_INVALID_ARG;
    int rc = validate_lmhead(hidden, ld_h, weight, ld_w, dt, d_model, total_new, vocab, token_ids);
    if (rc) return rc;
    rc = validate_ragged(scores, scores_stride, n_streams, n_held, cu_new, total_new, max_cand, max_new, policy, k, v,
                         layout, kept_idx, idx_stride, scores_out, out_stride, n_keep_out);
    if (rc || n_streams == 0) return rc;
    rc = workspace_check(workspace, workspace_bytes,
                         lmhead_ragged_workspace_bytes(n_streams, max_cand, total_new, vocab));
    if (rc) return rc;
    hipStream_t stream = (hipStream_t)hip_stream;
    const size_t lm_bytes = sirllm_lmhead_workspace_bytes(total_new, vocab);

    // E_t = Entropy(new tokens) from z = h W^T; token t of stream s lands behind that stream's held scores
    if (total_new > 0) {
        const LmHeadArgs a = make_lmhead_args(hidden, ld_h, weight, ld_w, d_model, total_new, vocab, token_ids, workspace);
        const LmHeadRagged rg = {cu_new, n_held, n_streams};
        rc = hip_status(launch_lmhead_score(a, dt, scores, 1, scores_stride, stream, &rg));
        if (rc) return rc;
    }
    const SelectArgs s = make_ragged_select_args(scores, scores_stride, n_streams, n_held, cu_new, max_cand, max_new,
                                                 policy, kept_idx, idx_stride, scores_out, out_stride, n_keep_out);
    return ragged_select_compact(s, max_cand, policy, k, v, layout, dst,
                                 (char*)workspace + lm_bytes, workspace_bytes - lm_bytes, stream);
}

}  // namespace

int sirllm_step_ragged(const void* logits, sirllm_dtype dt, int32_t vocab, int64_t ld, const int32_t* token_ids,
                       float* scores, int64_t scores_stride, int32_t n_streams, const int32_t* n_held,
                       const int32_t* cu_new, int64_t total_new, int32_t max_cand, int32_t max_new,
                       const sirllm_policy* policy,
                       void* k, void* v, const sirllm_kv_layout* layout, int32_t* kept_idx, int64_t idx_stride,
                       float* scores_out, int64_t out_stride, int32_t* n_keep_out, void* workspace,
                       size_t workspace_bytes, void* hip_stream)
{
    return step_ragged_common(logits, dt, vocab, ld, token_ids, scores, scores_stride, n_streams, n_held, cu_new, total_new,
                              max_cand, max_new, policy, k, v, layout, RaggedDst{nullptr, nullptr, nullptr}, kept_idx,
                              idx_stride, scores_out, out_stride, n_keep_out, workspace, workspace_bytes, hip_stream);
}

int sirllm_step_ragged_out_of_place(const void* logits, sirllm_dtype dt, int32_t vocab, int64_t ld, const int32_t* token_ids,
                                    float* scores, int64_t scores_stride, int32_t n_streams, const int32_t* n_held,
                                    const int32_t* cu_new, int64_t total_new, int32_t max_cand, int32_t max_new,
                                    const sirllm_policy* policy,
                                    const void* k_src, const void* v_src, const sirllm_kv_layout* src,
                                    void* k_dst, void* v_dst, const sirllm_kv_layout* dst,
                                    int32_t* kept_idx, int64_t idx_stride,
                                    float* scores_out, int64_t out_stride, int32_t* n_keep_out, void* workspace,
                                    size_t workspace_bytes, void* hip_stream)
{
    const int rc = validate_ragged_dst(max_cand, n_streams, policy, k_src, v_src, src, k_dst, v_dst, dst, kept_idx, idx_stride);
    if (rc) return rc;
    return step_ragged_common(logits, dt, vocab, ld, token_ids, scores, scores_stride, n_streams, n_held, cu_new, total_new,
                              max_cand, max_new, policy, const_cast<void*>(k_src), const_cast<void*>(v_src), src,
                              RaggedDst{k_dst, v_dst, dst}, kept_idx, idx_stride, scores_out, out_stride, n_keep_out, workspace,
                              workspace_bytes, hip_stream);
}

size_t sirllm_step_lmhead_ragged_workspace_bytes(int32_t n_streams, int32_t max_cand, int64_t total_new, int32_t vocab)
{
    return lmhead_ragged_workspace_bytes(n_streams, max_cand, total_new, vocab);
}

int sirllm_step_lmhead_ragged(const void* hidden, int64_t ld_h, const void* weight, int64_t ld_w, sirllm_dtype dt,
                              int32_t d_model, int32_t vocab, const int32_t* token_ids,
                              float* scores, int64_t scores_stride, int32_t n_streams, const int32_t* n_held,
                              const int32_t* cu_new, int64_t total_new, int32_t max_cand, int32_t max_new,
                              const sirllm_policy* policy, void* k, void* v, const sirllm_kv_layout* layout,
                              int32_t* kept_idx, int64_t idx_stride, float* scores_out, int64_t out_stride,
                              int32_t* n_keep_out, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return step_lmhead_ragged_common(hidden, ld_h, weight, ld_w, dt, d_model, vocab, token_ids, scores, scores_stride, n_streams,
                                     n_held, cu_new, total_new, max_cand, max_new, policy, k, v, layout,
                                     RaggedDst{nullptr, nullptr, nullptr}, kept_idx, idx_stride, scores_out, out_stride,
                                     n_keep_out, workspace, workspace_bytes, hip_stream);
}

int sirllm_step_lmhead_ragged_out_of_place(const void* hidden, int64_t ld_h, const void* weight, int64_t ld_w, sirllm_dtype dt,
                                           int32_t d_model, int32_t vocab, const int32_t* token_ids,
                                           float* scores, int64_t scores_stride, int32_t n_streams, const int32_t* n_held,
                                           const int32_t* cu_new, int64_t total_new, int32_t max_cand, int32_t max_new,
                                           const sirllm_policy* policy,
                                           const void* k_src, const void* v_src, const sirllm_kv_layout* src,
                                           void* k_dst, void* v_dst, const sirllm_kv_layout* dst,
                                           int32_t* kept_idx, int64_t idx_stride, float* scores_out, int64_t out_stride,
                                           int32_t* n_keep_out, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    const int rc = validate_ragged_dst(max_cand, n_streams, policy, k_src, v_src, src, k_dst, v_dst, dst, kept_idx, idx_stride);
    if (rc) return rc;
    return step_lmhead_ragged_common(hidden, ld_h, weight, ld_w, dt, d_model, vocab, token_ids, scores, scores_stride, n_streams,
                                     n_held, cu_new, total_new, max_cand, max_new, policy, const_cast<void*>(k_src),
                                     const_cast<void*>(v_src), src, RaggedDst{k_dst, v_dst, dst}, kept_idx, idx_stride,
                                     scores_out, out_stride, n_keep_out, workspace, workspace_bytes, hip_stream);
}

}  // extern "C"
