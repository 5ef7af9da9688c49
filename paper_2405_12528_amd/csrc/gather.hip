// KV compaction KV <- KV[Id]  (paper Sec. 3.3): an out-of-place gather of cache rows for
// every stream, layer, K|V tensor and KV head.  Grid = (row tiles, planes, streams); a
// workgroup copies one tile of consecutive destination rows of one plane.  A row is covered by
// consecutive lanes, each moving one 16-byte vector (narrower ones only when the caller's
// pointers or strides are not 16-byte multiples); all of a lane's loads are issued before its
// first store.  The kernel is kept to a few dozen instructions per lane on purpose: at 16 bytes
// per lane the copy is as close to instruction-issue bound as to HBM bound.
// HBM traffic: each kept row is read once and written once; dropped rows are never touched.
#include <type_traits>

#include "common.h"
#include "tuning.h"

namespace sirllm {
namespace {

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

struct GatherLaunch {
    GatherArgs a;
    int32_t vpr;          // vectors per row
    int32_t shift;        // log2(vpr) when POW2
    int32_t n_items;      // n_keep * vpr
    int32_t plane0;       // first plane of this launch (grids are cut into <= 65535 planes)
    int32_t stream0;      // first stream of this launch
    int32_t lh;           // n_layers * n_heads
    int32_t uniform;      // 1: s_layer == n_heads*s_head and d_layer == n_heads*d_head
};

// POW2: vpr is a power of two.  OFF64: offsets inside a plane need more than 32 bits.
template <typename VecT, int BLOCK, int UNROLL, bool NT, bool POW2, bool OFF64>
__global__ __launch_bounds__(BLOCK) void gather_rows_kernel(GatherLaunch g)
{
    const GatherArgs& a = g.a;
    using off_t = typename std::conditional<OFF64, int64_t, uint32_t>::type;

    // plane -> base pointers (uniform over the workgroup: scalar arithmetic)
    const int plane = g.plane0 + (int)blockIdx.y;
    const int stream = g.stream0 + (int)blockIdx.z;
    const int tensor = plane >= g.lh ? 1 : 0;
    const int ph = plane - tensor * g.lh;
    int64_t so, dof;
    if (g.uniform) {
        so = ph * a.s_head;
        dof = ph * a.d_head;
    } else {
        const int l = ph / a.n_heads, h = ph - l * a.n_heads;
        so = l * a.s_layer + h * a.s_head;
        dof = l * a.d_layer + h * a.d_head;
    }
    const char* sp = a.src[tensor] + stream * a.s_stream + so;
    char* dp = a.dst[tensor] + stream * a.d_stream + dof;
    const int32_t* idx = a.kept_idx + stream * a.idx_stride;

    const int w0 = (int)blockIdx.x * (BLOCK * UNROLL) + (int)threadIdx.x;
    VecT v[UNROLL];
    off_t doff[UNROLL];
    bool live[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int w = w0 + u * BLOCK;
        live[u] = w < g.n_items;
        v[u] = VecT{};
        doff[u] = 0;
        if (live[u]) {
            int j, c;
            if constexpr (POW2) { j = w >> g.shift; c = w & (g.vpr - 1); }
            else                { j = w / g.vpr;    c = w - j * g.vpr; }
            const uint32_t i = (uint32_t)idx[j];
            doff[u] = (off_t)j * (off_t)a.d_pos + (off_t)(c * (int)sizeof(VecT));
            if (i < (uint32_t)a.n_src)       // an index with no source slot leaves a zero row
                v[u] = ld<VecT, NT>(sp + ((off_t)i * (off_t)a.s_pos + (off_t)(c * (int)sizeof(VecT))));
        }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
        if (live[u]) st<VecT, NT>(dp + doff[u], v[u]);
}

template <typename VecT, int BLOCK, int UNROLL, bool NT>
void launch_shape(const GatherLaunch& g, dim3 grid, bool pow2, bool off64, hipStream_t stream)
{
    const dim3 block(BLOCK);
    if (pow2) {
        if (off64) hipLaunchKernelGGL((gather_rows_kernel<VecT, BLOCK, UNROLL, NT, true, true>), grid, block, 0, stream, g);
        else       hipLaunchKernelGGL((gather_rows_kernel<VecT, BLOCK, UNROLL, NT, true, false>), grid, block, 0, stream, g);
    } else {
        if (off64) hipLaunchKernelGGL((gather_rows_kernel<VecT, BLOCK, UNROLL, NT, false, true>), grid, block, 0, stream, g);
        else       hipLaunchKernelGGL((gather_rows_kernel<VecT, BLOCK, UNROLL, NT, false, false>), grid, block, 0, stream, g);
    }
}

template <typename VecT>
hipError_t launch_vec(const GatherArgs& a, hipStream_t stream)
{
    GatherLaunch g;
    g.a = a;
    g.vpr = a.row_bytes / (int)sizeof(VecT);
    const int64_t n_items = (int64_t)a.n_keep * g.vpr;
    if (n_items > 0x7fffffffLL - 4096) return hipErrorInvalidValue;   // the API layer rejects this first
    g.n_items = (int32_t)n_items;
    const bool pow2 = (g.vpr & (g.vpr - 1)) == 0;
    g.shift = 0;
    while (pow2 && (1 << g.shift) < g.vpr) ++g.shift;
    g.lh = a.n_layers * a.n_heads;
    g.uniform = (a.s_layer == a.n_heads * a.s_head && a.d_layer == a.n_heads * a.d_head) ? 1 : 0;
    // 32-bit offsets inside a plane when both planes are below 4 GiB
    const bool off64 = (int64_t)a.n_src * a.s_pos + a.row_bytes > 0xffffffffLL ||
                       (int64_t)a.n_keep * a.d_pos + a.row_bytes > 0xffffffffLL;

    const int block = tuning::get("SIRLLM_GATHER_BLOCK", 512);
    const int unroll = tuning::get("SIRLLM_GATHER_UNROLL", 1);
    const bool nt = tuning::get("SIRLLM_GATHER_NT", 1) != 0;
    const int per_block = block * unroll;
    const unsigned n_tiles = (unsigned)((n_items + per_block - 1) / per_block);
    const int planes = a.n_tensors * g.lh;
    constexpr int kMaxDim = 65535;
    for (int s0 = 0; s0 < a.n_streams; s0 += kMaxDim) {
        for (int p0 = 0; p0 < planes; p0 += kMaxDim) {
            g.stream0 = s0;
            g.plane0 = p0;
            const dim3 grid(n_tiles, (unsigned)min(kMaxDim, planes - p0), (unsigned)min(kMaxDim, a.n_streams - s0));
            if (block == 512) {
                if (unroll == 2) { if (nt) launch_shape<VecT, 512, 2, true>(g, grid, pow2, off64, stream); else launch_shape<VecT, 512, 2, false>(g, grid, pow2, off64, stream); }
                else             { if (nt) launch_shape<VecT, 512, 1, true>(g, grid, pow2, off64, stream); else launch_shape<VecT, 512, 1, false>(g, grid, pow2, off64, stream); }
            } else {
                if (unroll == 2) { if (nt) launch_shape<VecT, 256, 2, true>(g, grid, pow2, off64, stream); else launch_shape<VecT, 256, 2, false>(g, grid, pow2, off64, stream); }
                else             { if (nt) launch_shape<VecT, 256, 1, true>(g, grid, pow2, off64, stream); else launch_shape<VecT, 256, 1, false>(g, grid, pow2, off64, stream); }
            }
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
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
    if ((bits & 15) == 0) return launch_vec<u32x4>(a, stream);
    if ((bits & 7) == 0)  return launch_vec<u32x2>(a, stream);
    if ((bits & 3) == 0)  return launch_vec<uint32_t>(a, stream);
    if ((bits & 1) == 0)  return launch_vec<uint16_t>(a, stream);
    return launch_vec<uint8_t>(a, stream);
}

}  // namespace sirllm
