// Launch of the token-entropy score kernel (paper Sec. 3.2): one workgroup per vocabulary row.
// HBM-read bound.
#include "common.h"
#include "score_device.h"
#include "tuning.h"

namespace sirllm {
namespace {

template <int DT, int BLOCK, int UNROLL, bool NT>
__global__ __launch_bounds__(BLOCK) void score_rows_kernel(ScoreArgs a)
{
    __shared__ score_dev::ScoreSmem<BLOCK> sm;
    score_dev::score_row<DT, BLOCK, UNROLL, NT>(a, (int64_t)blockIdx.x, sm);
}

// One thread per row: fold the chunks' (m, s) with the same merge the lanes use, pick the chunk that
// saw the token's logit, finish e = (m - z_tok) + log s.
__global__ __launch_bounds__(256) void score_merge_kernel(const float* partials, int n_parts, int64_t part_stride,
                                                          int64_t n_rows, float* out)
{
    const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (row >= n_rows) return;
    score_dev::MS acc = {-INFINITY, 0.0f};
    float zt = __uint_as_float(0x7fc00000u);
    for (int p = 0; p < n_parts; ++p) {
        const float* t = partials + p * part_stride + 3 * row;
        acc = score_dev::merge(acc, score_dev::MS{t[0], t[1]});
        const float z = t[2];
        if (zt != zt && z == z) zt = z;
    }
    out[row] = (acc.m - zt) + logf(acc.s);
}

template <int DT, int BLOCK>
hipError_t launch_one(const ScoreArgs& a, hipStream_t stream, bool nt)
{
    const dim3 grid((unsigned)a.n_rows), block(BLOCK);
    if (nt) hipLaunchKernelGGL((score_rows_kernel<DT, BLOCK, 4, true>), grid, block, 0, stream, a);
    else    hipLaunchKernelGGL((score_rows_kernel<DT, BLOCK, 4, false>), grid, block, 0, stream, a);
    return hipGetLastError();
}

template <int DT>
hipError_t launch_esize(const ScoreArgs& a, hipStream_t stream)
{
    // Long rows take the widest workgroup (most waves per CU on few rows); short rows a narrower
    // one, so that lanes are not left without a single 16-byte vector.
    const int64_t vecs = (int64_t)a.vocab * score_dev::Elem<DT>::kSize / 16;
    int block = vecs >= 2048 ? 1024 : (vecs >= 1024 ? 512 : 256);
    block = tuning::get("SIRLLM_SCORE_BLOCK", block);
    const bool nt = tuning::get("SIRLLM_SCORE_NT", 1) != 0;
    switch (block) {
    case 256:  return launch_one<DT, 256>(a, stream, nt);
    case 512:  return launch_one<DT, 512>(a, stream, nt);
    default:   return launch_one<DT, 1024>(a, stream, nt);
    }
}

}  // namespace

hipError_t launch_score(const ScoreArgs& a, sirllm_dtype dt, hipStream_t stream)
{
    if (a.n_rows <= 0) return hipSuccess;
    switch (dt) {
    case SIRLLM_F32:  return launch_esize<SIRLLM_F32>(a, stream);
    case SIRLLM_BF16: return launch_esize<SIRLLM_BF16>(a, stream);
    default:          return launch_esize<SIRLLM_F16>(a, stream);
    }
}

hipError_t launch_score_merge(const float* partials, int32_t n_parts, int64_t part_stride, int64_t n_rows,
                              float* scores_out, hipStream_t stream)
{
    if (n_rows <= 0) return hipSuccess;
    const int64_t blocks = (n_rows + 255) / 256;
    hipLaunchKernelGGL(score_merge_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, partials, n_parts,
                       part_stride, n_rows, scores_out);
    return hipGetLastError();
}

}  // namespace sirllm
