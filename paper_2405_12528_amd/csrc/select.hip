// Launch of decay + Top_k selection + index build (paper Sec. 3.3, Sec. 3.1): one workgroup of
// 1024 threads per dialogue stream, and the trivial keep-everything kernel for a cache that is
// still within its budget.
#include "common.h"
#include "select_device.h"
#include "tuning.h"

namespace sirllm {
namespace {

template <int BLOCK, int KPT>
__global__ __launch_bounds__(BLOCK) void select_kernel(SelectArgs a)
{
    __shared__ select_dev::SelectSmem<BLOCK> sm;
    select_dev::select_stream<BLOCK, KPT, false>(a, (int)blockIdx.x, sm);
}

template <int BLOCK, int KPT>
__global__ __launch_bounds__(BLOCK) void select_ragged_kernel(SelectArgs a)
{
    __shared__ select_dev::SelectSmem<BLOCK> sm;
    select_dev::select_ragged_stream<BLOCK, KPT, false>(a, (int)blockIdx.x, sm);
}

__global__ __launch_bounds__(256) void keep_all_kernel(SelectArgs a)
{
    const int64_t total = (int64_t)a.n_streams * a.n_cand;
    for (int64_t w = (int64_t)blockIdx.x * 256 + threadIdx.x; w < total; w += (int64_t)gridDim.x * 256) {
        const int64_t s = w / a.n_cand;
        const int i = (int)(w - s * a.n_cand);
        float e = a.scores[s * a.scores_stride + i];
        if (i < a.n_held) e = __fmul_rn(e, a.decay);
        a.kept_idx[s * a.idx_stride + i] = i;
        a.scores_out[s * a.out_stride + i] = e;
    }
}

}  // namespace

hipError_t launch_select(const SelectArgs& a, hipStream_t stream)
{
    if (a.n_streams <= 0 || a.n_cand <= 0) return hipSuccess;
    constexpr int B = 1024;
    const dim3 grid((unsigned)a.n_streams), block(B);
    const int need = (a.n_cand + B - 1) / B;      // slots per thread
#define SIRLLM_SELECT_LAUNCH(K) hipLaunchKernelGGL((select_kernel<B, K>), grid, block, 0, stream, a)
    if (need <= 1)       SIRLLM_SELECT_LAUNCH(1);
    else if (need <= 2)  SIRLLM_SELECT_LAUNCH(2);
    else if (need <= 4)  SIRLLM_SELECT_LAUNCH(4);
    else if (need <= 8)  SIRLLM_SELECT_LAUNCH(8);
    else if (need <= 16) SIRLLM_SELECT_LAUNCH(16);
    else if (need <= 32) SIRLLM_SELECT_LAUNCH(32);
    else return hipErrorInvalidValue;             // above SIRLLM_MAX_CAND; the API layer rejects it first
#undef SIRLLM_SELECT_LAUNCH
    return hipGetLastError();
}

hipError_t launch_select_ragged(const SelectArgs& a, hipStream_t stream)
{
    if (a.n_streams <= 0) return hipSuccess;
    constexpr int B = 1024;
    const dim3 grid((unsigned)a.n_streams), block(B);
    const int need = (a.n_cand + B - 1) / B;      // a.n_cand is the caller's upper bound
#define SIRLLM_SELECT_LAUNCH(K) hipLaunchKernelGGL((select_ragged_kernel<B, K>), grid, block, 0, stream, a)
    if (need <= 2)       SIRLLM_SELECT_LAUNCH(2);
    else if (need <= 8)  SIRLLM_SELECT_LAUNCH(8);
    else if (need <= 16) SIRLLM_SELECT_LAUNCH(16);
    else if (need <= 32) SIRLLM_SELECT_LAUNCH(32);
    else return hipErrorInvalidValue;
#undef SIRLLM_SELECT_LAUNCH
    return hipGetLastError();
}

hipError_t launch_keep_all(const SelectArgs& a, hipStream_t stream)
{
    const int64_t total = (int64_t)a.n_streams * a.n_cand;
    if (total <= 0) return hipSuccess;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(keep_all_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace sirllm
