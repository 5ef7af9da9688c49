// KV compaction KV <- KV[Id]  (paper Sec. 3.3): an out-of-place gather of cache rows for
// every stream, layer, K|V tensor and KV head.  A workgroup copies one tile of consecutive
// destination rows of one plane; every lane moves 16-byte vectors (narrower ones only when the
// caller's pointers or strides are not 16-byte multiples), issuing all loads of its tile before
// the first store.  HBM bound: each kept row is read once and written once; dropped rows are
// never touched.
#include "common.h"
#include "tuning.h"

namespace sirllm {
namespace {

constexpr int kBlock = 256;

template <typename VecT, bool NT>
__device__ __forceinline__ VecT ld(const char* p)
{
    if constexpr (NT) return __builtin_nontemporal_load((const VecT*)p);
    else return *(const VecT*)p;
}
template <typename VecT, bool NT>
__device__ __forceinline__ void st(char* p, VecT v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, (VecT*)p);
    else *(VecT*)p = v;
}

// vpr: vectors per row; shift >= 0 when vpr is a power of two.
template <typename VecT, int UNROLL, bool NT>
__global__ __launch_bounds__(kBlock) void gather_rows_kernel(GatherArgs a, int vpr, int shift, int n_tiles)
{
    const int planes = a.n_tensors * a.n_layers * a.n_heads;
    const uint32_t b = blockIdx.x;
    const int tile = (int)(b % (uint32_t)n_tiles);
    const uint32_t rest = b / (uint32_t)n_tiles;
    const int plane = (int)(rest % (uint32_t)planes);
    const int stream = (int)(rest / (uint32_t)planes);
    const int h = plane % a.n_heads;
    const int l = (plane / a.n_heads) % a.n_layers;
    const int tensor = plane / (a.n_heads * a.n_layers);

    const char* sp = a.src[tensor] + stream * a.s_stream + l * a.s_layer + h * a.s_head;
    char* dp = a.dst[tensor] + stream * a.d_stream + l * a.d_layer + h * a.d_head;
    const int32_t* idx = a.kept_idx + stream * a.idx_stride;

    const int64_t n_items = (int64_t)a.n_keep * vpr;
    const int64_t w0 = (int64_t)tile * (kBlock * UNROLL) + threadIdx.x;

    VecT v[UNROLL];
    int64_t doff[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t w = w0 + u * kBlock;
        doff[u] = -1;
        v[u] = VecT{};
        if (w < n_items) {
            int64_t j, c;
            if (shift >= 0) { j = w >> shift; c = w & (vpr - 1); }
            else            { j = w / vpr;    c = w - j * vpr; }
            const int32_t i = idx[j];
            doff[u] = j * a.d_pos + c * (int64_t)sizeof(VecT);
            if (i >= 0 && i < a.n_src)       // an index with no source slot leaves a zero row
                v[u] = ld<VecT, NT>(sp + i * a.s_pos + c * (int64_t)sizeof(VecT));
        }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
        if (doff[u] >= 0) st<VecT, NT>(dp + doff[u], v[u]);
}

template <typename VecT>
hipError_t launch_vec(const GatherArgs& a, hipStream_t stream)
{
    const int vpr = a.row_bytes / (int)sizeof(VecT);
    int shift = -1;
    if ((vpr & (vpr - 1)) == 0) { shift = 0; while ((1 << shift) < vpr) ++shift; }
    const int unroll = tuning::get("SIRLLM_GATHER_UNROLL", 8);
    const bool nt = tuning::get("SIRLLM_GATHER_NT", 1) != 0;
    const int64_t n_items = (int64_t)a.n_keep * vpr;
    const int64_t per_block = (int64_t)kBlock * unroll;
    const int64_t n_tiles = (n_items + per_block - 1) / per_block;
    const int64_t blocks = n_tiles * a.n_tensors * a.n_layers * a.n_heads * a.n_streams;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffffLL || n_tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks), block(kBlock);
#define SIRLLM_GATHER_LAUNCH(U, N) \
    hipLaunchKernelGGL((gather_rows_kernel<VecT, U, N>), grid, block, 0, stream, a, vpr, shift, (int)n_tiles)
    if (unroll == 4)      { if (nt) SIRLLM_GATHER_LAUNCH(4, true); else SIRLLM_GATHER_LAUNCH(4, false); }
    else if (unroll == 2) { if (nt) SIRLLM_GATHER_LAUNCH(2, true); else SIRLLM_GATHER_LAUNCH(2, false); }
    else                  { if (nt) SIRLLM_GATHER_LAUNCH(8, true); else SIRLLM_GATHER_LAUNCH(8, false); }
#undef SIRLLM_GATHER_LAUNCH
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gather(const GatherArgs& a, hipStream_t stream)
{
    if (a.n_keep <= 0 || a.n_streams <= 0 || a.row_bytes <= 0 || a.n_layers <= 0 || a.n_heads <= 0)
        return hipSuccess;
    // widest access that every address in the call is a multiple of
    uint64_t bits = (uint64_t)a.row_bytes | (uint64_t)a.s_stream | (uint64_t)a.s_layer | (uint64_t)a.s_head |
                    (uint64_t)a.s_pos | (uint64_t)a.d_stream | (uint64_t)a.d_layer | (uint64_t)a.d_head |
                    (uint64_t)a.d_pos;
    for (int t = 0; t < a.n_tensors; ++t) bits |= (uint64_t)(uintptr_t)a.src[t] | (uint64_t)(uintptr_t)a.dst[t];
    const int tuned = tuning::get("SIRLLM_GATHER_VEC", 16);
    if ((bits & 15) == 0 && tuned >= 16) return launch_vec<u32x4>(a, stream);
    if ((bits & 7) == 0 && tuned >= 8)   return launch_vec<u32x2>(a, stream);
    if ((bits & 3) == 0 && tuned >= 4)   return launch_vec<uint32_t>(a, stream);
    if ((bits & 1) == 0 && tuned >= 2)   return launch_vec<uint16_t>(a, stream);
    return launch_vec<uint8_t>(a, stream);
}

}  // namespace sirllm
