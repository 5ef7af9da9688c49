// Launch of the token-entropy score kernel (paper Sec. 3.2): one workgroup per vocabulary row.
// HBM-read bound.
#include "common.h"
#include "score_device.h"
#include "tuning.h"

namespace sirllm {
namespace {

template <int ESIZE, int BLOCK, int UNROLL, bool NT>
__global__ __launch_bounds__(BLOCK) void score_rows_kernel(ScoreArgs a)
{
    __shared__ score_dev::ScoreSmem<BLOCK> sm;
    score_dev::score_row<ESIZE, BLOCK, UNROLL, NT>(a, (int64_t)blockIdx.x, sm);
}

template <int ESIZE, int BLOCK>
hipError_t launch_one(const ScoreArgs& a, hipStream_t stream, bool nt)
{
    const dim3 grid((unsigned)a.n_rows), block(BLOCK);
    if (nt) hipLaunchKernelGGL((score_rows_kernel<ESIZE, BLOCK, 4, true>), grid, block, 0, stream, a);
    else    hipLaunchKernelGGL((score_rows_kernel<ESIZE, BLOCK, 4, false>), grid, block, 0, stream, a);
    return hipGetLastError();
}

template <int ESIZE>
hipError_t launch_esize(const ScoreArgs& a, hipStream_t stream)
{
    // Long rows take the widest workgroup (most waves per CU on few rows); short rows a narrower
    // one, so that lanes are not left without a single 16-byte vector.
    const int64_t vecs = (int64_t)a.vocab * ESIZE / 16;
    int block = vecs >= 2048 ? 1024 : (vecs >= 1024 ? 512 : 256);
    block = tuning::get("SIRLLM_SCORE_BLOCK", block);
    const bool nt = tuning::get("SIRLLM_SCORE_NT", 1) != 0;
    switch (block) {
    case 256:  return launch_one<ESIZE, 256>(a, stream, nt);
    case 512:  return launch_one<ESIZE, 512>(a, stream, nt);
    default:   return launch_one<ESIZE, 1024>(a, stream, nt);
    }
}

}  // namespace

hipError_t launch_score(const ScoreArgs& a, sirllm_dtype dt, hipStream_t stream)
{
    if (a.n_rows <= 0) return hipSuccess;
    return dt == SIRLLM_F32 ? launch_esize<4>(a, stream) : launch_esize<2>(a, stream);
}

}  // namespace sirllm
