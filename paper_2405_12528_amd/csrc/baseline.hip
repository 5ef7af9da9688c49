// The score-free retention policies the paper compares against (Sec. 4.1 "Baselines"), producing
// the same ascending kept_idx list as the entropy policy so that the same compaction follows:
// StreamLLM (sinks + recent window), IntervalLLM (a fixed-interval comb over the middle region,
// anchored at its newest slot) and RandomLLM (a uniformly random subset of the middle region,
// drawn with Philox4x32-10 keys and the radix select of the entropy policy).
#include "common.h"
#include "select_device.h"

namespace sirllm {
namespace {

// One thread per kept position j.  interval == 0: keep everything (n_cand <= budget).
__global__ __launch_bounds__(256) void comb_kernel(SelectArgs a, int interval)
{
    const int n_keep = interval == 0 ? a.n_cand : a.n_sink + a.n_topk + a.n_recent;
    const int64_t total = (int64_t)a.n_streams * n_keep;
    for (int64_t w = (int64_t)blockIdx.x * 256 + threadIdx.x; w < total; w += (int64_t)gridDim.x * 256) {
        const int64_t s = w / n_keep;
        const int j = (int)(w - s * n_keep);
        int i;
        if (interval == 0 || j < a.n_sink) {
            i = j;                                                      // keep-all, or Id_sink
        } else if (j >= a.n_sink + a.n_topk) {
            i = a.n_cand - (n_keep - j);                                // Id_recent
        } else {
            const int m = j - a.n_sink;                                 // m-th oldest tooth of the comb
            i = (a.n_cand - a.n_recent - 1) - (a.n_topk - 1 - m) * interval;
        }
        a.kept_idx[s * a.idx_stride + j] = i;
    }
}

template <int BLOCK, int KPT>
__global__ __launch_bounds__(BLOCK) void random_select_kernel(SelectArgs a)
{
    __shared__ select_dev::SelectSmem<BLOCK> sm;
    select_dev::select_stream<BLOCK, KPT, false, true>(a, (int)blockIdx.x, sm);
}

}  // namespace

hipError_t launch_baseline_comb(const SelectArgs& a, int interval, hipStream_t stream)
{
    const int n_keep = interval == 0 ? a.n_cand : a.n_sink + a.n_topk + a.n_recent;
    const int64_t total = (int64_t)a.n_streams * n_keep;
    if (total <= 0) return hipSuccess;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(comb_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, a, interval);
    return hipGetLastError();
}

hipError_t launch_baseline_random(const SelectArgs& a, hipStream_t stream)
{
    if (a.n_streams <= 0 || a.n_cand <= 0) return hipSuccess;
    constexpr int B = 1024;
    const dim3 grid((unsigned)a.n_streams), block(B);
    const int need = (a.n_cand + B - 1) / B;
#define SIRLLM_RANDOM_LAUNCH(K) hipLaunchKernelGGL((random_select_kernel<B, K>), grid, block, 0, stream, a)
    if (need <= 1)       SIRLLM_RANDOM_LAUNCH(1);
    else if (need <= 4)  SIRLLM_RANDOM_LAUNCH(4);
    else if (need <= 8)  SIRLLM_RANDOM_LAUNCH(8);
    else if (need <= 16) SIRLLM_RANDOM_LAUNCH(16);
    else if (need <= 32) SIRLLM_RANDOM_LAUNCH(32);
    else return hipErrorInvalidValue;
#undef SIRLLM_RANDOM_LAUNCH
    return hipGetLastError();
}

}  // namespace sirllm
