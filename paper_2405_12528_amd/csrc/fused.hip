// One launch for "score the new tokens" and "decay + select + index build" when the two do not
// depend on each other: with n_new <= n_recent every new token lies inside the recent window,
// so Top_k (paper Sec. 3.3) only looks at held scores and can run while the vocabulary rows are
// still being scanned (Sec. 3.2).  The first n_streams workgroups do the selection of one
// stream each, all others score one row each; the scorers also drop the new scores straight
// into their known places at the tail of the compacted score cache.  The latency-bound
// selection thereby hides behind the HBM-bound scan.
#include "common.h"
#include "score_device.h"
#include "select_device.h"
#include "tuning.h"

namespace sirllm {
namespace {

constexpr int kBlock = 1024;
// Most slots per lane of a selecting workgroup inside the shared launch: with 16 the kernel still fits 64 registers,
// so two workgroups of 1024 threads share a CU as in the scoring kernel proper; 32 slots per lane need 128 registers
// (one workgroup per CU, and spills), so caches above 16384 slots take the three launches.
constexpr int kMaxKpt = 16;

template <int DT, int KPT, bool NT>
__global__ __launch_bounds__(kBlock) void score_select_kernel(ScoreArgs sa, SelectArgs se)
{
    __shared__ union {
        select_dev::SelectSmem<kBlock> sel;
        score_dev::ScoreSmem<kBlock> sc;
    } sm;
    if ((int)blockIdx.x < se.n_streams) {
        select_dev::select_stream<kBlock, KPT, true>(se, (int)blockIdx.x, sm.sel);
    } else {
        score_dev::score_row<DT, kBlock, 4, NT>(sa, (int64_t)blockIdx.x - se.n_streams, sm.sc);
    }
}

// Ragged batch: the same split of roles, every selecting workgroup on its stream's own sizes.
template <int DT, int KPT, bool NT>
__global__ __launch_bounds__(kBlock) void score_select_ragged_kernel(ScoreArgs sa, SelectArgs se)
{
    __shared__ union {
        select_dev::SelectSmem<kBlock> sel;
        score_dev::ScoreSmem<kBlock> sc;
    } sm;
    if ((int)blockIdx.x < se.n_streams) {
        select_dev::select_ragged_stream<kBlock, KPT, true>(se, (int)blockIdx.x, sm.sel);
    } else {
        score_dev::score_row<DT, kBlock, 4, NT>(sa, (int64_t)blockIdx.x - se.n_streams, sm.sc);
    }
}

template <int DT, int KPT>
hipError_t launch_ragged_kpt(const ScoreArgs& sa, const SelectArgs& se, hipStream_t stream)
{
    const dim3 grid((unsigned)(sa.n_rows + se.n_streams)), block(kBlock);
    if (tuning::get("SIRLLM_SCORE_NT", 1) != 0)
        hipLaunchKernelGGL((score_select_ragged_kernel<DT, KPT, true>), grid, block, 0, stream, sa, se);
    else
        hipLaunchKernelGGL((score_select_ragged_kernel<DT, KPT, false>), grid, block, 0, stream, sa, se);
    return hipGetLastError();
}

template <int DT>
hipError_t launch_ragged_esize(const ScoreArgs& sa, const SelectArgs& se, hipStream_t stream)
{
    const int need = (se.n_cand + kBlock - 1) / kBlock;
    if (need <= 2) return launch_ragged_kpt<DT, 2>(sa, se, stream);
    if (need <= 8) return launch_ragged_kpt<DT, 8>(sa, se, stream);
    return launch_ragged_kpt<DT, 16>(sa, se, stream);
}

template <int DT, int KPT>
hipError_t launch_kpt(const ScoreArgs& sa, const SelectArgs& se, hipStream_t stream)
{
    const dim3 grid((unsigned)(sa.n_rows + se.n_streams)), block(kBlock);
    if (tuning::get("SIRLLM_SCORE_NT", 1) != 0)
        hipLaunchKernelGGL((score_select_kernel<DT, KPT, true>), grid, block, 0, stream, sa, se);
    else
        hipLaunchKernelGGL((score_select_kernel<DT, KPT, false>), grid, block, 0, stream, sa, se);
    return hipGetLastError();
}

template <int DT>
hipError_t launch_esize(const ScoreArgs& sa, const SelectArgs& se, hipStream_t stream)
{
    const int need = (se.n_cand + kBlock - 1) / kBlock;
    if (need <= 2) return launch_kpt<DT, 2>(sa, se, stream);
    if (need <= 8) return launch_kpt<DT, 8>(sa, se, stream);
    return launch_kpt<DT, 16>(sa, se, stream);
}

}  // namespace

bool score_select_fusable(const ScoreArgs& sa, const SelectArgs& se)
{
    if (tuning::get("SIRLLM_FUSE_SELECT", 1) == 0) return false;
    const int n_new = se.n_cand - se.n_held;
    return sa.n_rows > 0 && n_new <= se.n_recent && se.n_cand <= kBlock * kMaxKpt &&
           sa.n_rows + se.n_streams <= 0x7fffffffLL;
}

bool score_select_ragged_fusable(const ScoreArgs& sa, const SelectArgs& se)
{
    if (tuning::get("SIRLLM_FUSE_SELECT", 1) == 0) return false;
    return sa.n_rows > 0 && se.max_new <= se.n_recent && se.n_cand <= kBlock * kMaxKpt &&
           sa.n_rows + se.n_streams <= 0x7fffffffLL;
}

hipError_t launch_score_select_ragged(const ScoreArgs& sa, const SelectArgs& se, sirllm_dtype dt, hipStream_t stream)
{
    switch (dt) {
    case SIRLLM_F32:  return launch_ragged_esize<SIRLLM_F32>(sa, se, stream);
    case SIRLLM_BF16: return launch_ragged_esize<SIRLLM_BF16>(sa, se, stream);
    default:          return launch_ragged_esize<SIRLLM_F16>(sa, se, stream);
    }
}

hipError_t launch_score_select(const ScoreArgs& sa, const SelectArgs& se, sirllm_dtype dt, hipStream_t stream)
{
    switch (dt) {
    case SIRLLM_F32:  return launch_esize<SIRLLM_F32>(sa, se, stream);
    case SIRLLM_BF16: return launch_esize<SIRLLM_BF16>(sa, se, stream);
    default:          return launch_esize<SIRLLM_F16>(sa, se, stream);
    }
}

}  // namespace sirllm
