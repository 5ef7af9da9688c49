// Device code of the KV compaction KV <- KV[Id]  (paper Sec. 3.3): one workgroup copies one tile
// of consecutive destination rows of one plane (one stream, layer, K|V tensor, KV head).  A row
// is covered by consecutive lanes, each moving one 16-byte vector (narrower ones only when the
// caller's pointers or strides are not 16-byte multiples); all of a lane's loads are issued before
// its first store.  Kept to a few dozen instructions per lane on purpose: at 16 bytes per lane the
// copy is as close to instruction-issue bound as to HBM bound.
#pragma once

#include <type_traits>

#include "common.h"

namespace sirllm {
namespace gather_dev {

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
    int32_t row_begin;    // destination rows [row_begin, row_end) are copied by this launch
    int32_t row_end;
    int32_t plane0;       // first plane of this launch (grids are cut into <= 65535 planes)
    int32_t stream0;      // first stream of this launch
    int32_t lh;           // n_layers * n_heads
    int32_t uniform;      // 1: s_layer == n_heads*s_head and d_layer == n_heads*d_head
};

// One tile of destination rows of the plane that starts at sp (source) / dp (destination) and belongs to `stream`.
// POW2: vpr is a power of two.  OFF64: offsets inside a plane need more than 32 bits.
template <typename VecT, int BLOCK, int UNROLL, bool NT, bool POW2, bool OFF64>
__device__ __forceinline__ void gather_tile_at(const GatherLaunch& g, int tile, const char* sp, char* dp, int stream)
{
    const GatherArgs& a = g.a;
    using off_t = typename std::conditional<OFF64, int64_t, uint32_t>::type;
    const int32_t* idx = a.kept_idx + stream * a.idx_stride;

    const int n_items = (g.row_end - g.row_begin) * g.vpr;
    const int w0 = tile * (BLOCK * UNROLL) + (int)threadIdx.x;
    VecT v[UNROLL];
    off_t doff[UNROLL];
    bool live[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int w = w0 + u * BLOCK;
        live[u] = w < n_items;
        v[u] = VecT{};
        doff[u] = 0;
        if (live[u]) {
            int j, c;
            if constexpr (POW2) { j = w >> g.shift; c = w & (g.vpr - 1); }
            else                { j = w / g.vpr;    c = w - j * g.vpr; }
            j += g.row_begin;
            doff[u] = (off_t)j * (off_t)a.d_pos + (off_t)(c * (int)sizeof(VecT));
            const uint32_t i = (uint32_t)idx[j];
            if (i < (uint32_t)a.n_src)       // an index with no source slot leaves a zero row
                v[u] = ld<VecT, NT>(sp + ((off_t)i * (off_t)a.s_pos + (off_t)(c * (int)sizeof(VecT))));
        }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
        if (live[u]) st<VecT, NT>(dp + doff[u], v[u]);
}

// The cache is one buffer per tensor: plane -> base pointers by the layout's strides (uniform over the workgroup:
// scalar arithmetic).
template <typename VecT, int BLOCK, int UNROLL, bool NT, bool POW2, bool OFF64>
__device__ __forceinline__ void gather_tile(const GatherLaunch& g, int tile, int plane, int stream)
{
    const GatherArgs& a = g.a;
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
    gather_tile_at<VecT, BLOCK, UNROLL, NT, POW2, OFF64>(g, tile, a.src[tensor] + stream * a.s_stream + so,
                                                         a.dst[tensor] + stream * a.d_stream + dof, stream);
}

// The cache is one buffer per layer and tensor (the table rides in the kernel arguments): plane -> (tensor, layer,
// head), base pointer of that layer's buffer, then the stream and head strides.
template <typename VecT, int BLOCK, int UNROLL, bool NT, bool POW2, bool OFF64>
__device__ __forceinline__ void gather_tile_layers(const GatherLaunch& g, const LayerTable& t, int tile, int plane, int stream)
{
    const GatherArgs& a = g.a;
    const int tensor = plane >= g.lh ? 1 : 0;
    const int ph = plane - tensor * g.lh;
    const int l = ph / a.n_heads, h = ph - l * a.n_heads;
    gather_tile_at<VecT, BLOCK, UNROLL, NT, POW2, OFF64>(g, tile, t.src[tensor][l] + stream * a.s_stream + h * a.s_head,
                                                         t.dst[tensor][l] + stream * a.d_stream + h * a.d_head, stream);
}

// Host side: fills everything of a GatherLaunch that depends on the vector width.
template <typename VecT>
inline bool fill_launch(GatherLaunch& g, const GatherArgs& a, int row_begin, int row_end, bool* pow2, bool* off64)
{
    g.a = a;
    g.vpr = a.row_bytes / (int)sizeof(VecT);
    if ((int64_t)a.n_keep * g.vpr > 0x7fffffffLL - 4096) return false;   // the API layer rejects this first
    *pow2 = (g.vpr & (g.vpr - 1)) == 0;
    g.shift = 0;
    while (*pow2 && (1 << g.shift) < g.vpr) ++g.shift;
    g.row_begin = row_begin;
    g.row_end = row_end;
    g.plane0 = 0;
    g.stream0 = 0;
    g.lh = a.n_layers * a.n_heads;
    g.uniform = (a.s_layer == a.n_heads * a.s_head && a.d_layer == a.n_heads * a.d_head) ? 1 : 0;
    // 32-bit offsets inside a plane when both planes are below 4 GiB
    *off64 = (int64_t)a.n_src * a.s_pos + a.row_bytes > 0xffffffffLL ||
             (int64_t)a.n_keep * a.d_pos + a.row_bytes > 0xffffffffLL;
    return true;
}

// Widest power-of-two access (<= 16 bytes) that every number OR-ed into `bits` is a multiple of.
inline int widest_access(uint64_t bits)
{
    if ((bits & 15) == 0) return 16;
    if ((bits & 7) == 0) return 8;
    if ((bits & 3) == 0) return 4;
    if ((bits & 1) == 0) return 2;
    return 1;
}

// ... that every address of the call is a multiple of (with_layer_stride = false: the layers are separate buffers).
inline int vector_bytes(const GatherArgs& a, bool with_layer_stride = true)
{
    uint64_t bits = (uint64_t)a.row_bytes | (uint64_t)a.s_stream | (uint64_t)a.s_head | (uint64_t)a.s_pos |
                    (uint64_t)a.d_stream | (uint64_t)a.d_head | (uint64_t)a.d_pos;
    if (with_layer_stride) {
        bits |= (uint64_t)a.s_layer | (uint64_t)a.d_layer;
        for (int t = 0; t < a.n_tensors; ++t) bits |= (uint64_t)(uintptr_t)a.src[t] | (uint64_t)(uintptr_t)a.dst[t];
    }
    return widest_access(bits);
}

}  // namespace gather_dev
}  // namespace sirllm
