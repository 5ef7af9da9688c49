// Launch of the KV compaction KV <- KV[Id]  (paper Sec. 3.3): an out-of-place gather of cache rows
// for every stream, layer, K|V tensor and KV head.  Grid = (row tiles, planes, streams).
// HBM traffic: each kept row is read once and written once; dropped rows are never touched.
#include "common.h"
#include "gather_device.h"
#include "tuning.h"

namespace sirllm {
namespace {

using gather_dev::GatherLaunch;

template <typename VecT, int BLOCK, int UNROLL, bool NT, bool POW2, bool OFF64>
__global__ __launch_bounds__(BLOCK) void gather_rows_kernel(GatherLaunch g)
{
    gather_dev::gather_tile<VecT, BLOCK, UNROLL, NT, POW2, OFF64>(
        g, (int)blockIdx.x, g.plane0 + (int)blockIdx.y, g.stream0 + (int)blockIdx.z);
}

// Rows of sixteen 16-byte vectors (256 bytes), one vector per lane: the kept indices come through the scalar cache.
using gather_dev::WaveRowsArgs;

template <int BLOCK, bool OFF64>
__global__ __launch_bounds__(BLOCK) void gather_rows16_kernel(WaveRowsArgs w)
{
    gather_dev::gather_tile_wave_rows<BLOCK, true, OFF64, 4>(w, (int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z);
}

// The same for rows of 32 vectors (LV = 5) and for rows of 64 vectors and more (LV = 6), single-wave tiles.
template <int LV, bool OFF64>
__global__ __launch_bounds__(64) void gather_wave_rows_kernel(WaveRowsArgs w)
{
    gather_dev::gather_tile_wave_rows<64, true, OFF64, LV>(w, (int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z);
}

// Ragged batches (per-stream slot and row counts in device memory; streams flagged by the selection are left alone): the
// single-wave tile for rows of 16, 32 or >= 64 vectors, the general tile for everything else.
template <int LV, bool OFF64>
__global__ __launch_bounds__(64) void gather_wave_rows_ragged_kernel(WaveRowsArgs w)
{
    gather_dev::gather_tile_wave_rows<64, true, OFF64, LV, false, true>(w, (int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z);
}

template <typename VecT, bool POW2, bool OFF64>
__global__ __launch_bounds__(128) void gather_rows_ragged_kernel(GatherLaunch g, gather_dev::Ragged rg)
{
    const int stream = g.stream0 + (int)blockIdx.z;
    int rows = 0;
    const int n_src = gather_dev::ragged_rows(rg, stream, g.a.n_src, g.row_end - g.row_begin, rows);
    if (n_src < 0) return;
    g.a.n_src = n_src;
    g.row_end = g.row_begin + rows;
    gather_dev::gather_tile<VecT, 128, 1, true, POW2, OFF64>(g, (int)blockIdx.x, g.plane0 + (int)blockIdx.y, stream);
}

template <bool OFF64>
__global__ __launch_bounds__(64) void gather_rows16_layers_kernel(WaveRowsArgs w, LayerTable t)
{
    gather_dev::gather_tile_wave_rows<64, true, OFF64, 4, true>(w, (int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z, &t);
}

template <typename VecT, bool POW2, bool OFF64>
__global__ __launch_bounds__(128) void gather_rows_layers_kernel(GatherLaunch g, LayerTable t)
{
    gather_dev::gather_tile_layers<VecT, 128, 1, true, POW2, OFF64>(g, t, (int)blockIdx.x, g.plane0 + (int)blockIdx.y,
                                                                   g.stream0 + (int)blockIdx.z);
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
hipError_t launch_vec(const GatherArgs& a, int row_begin, int row_end, hipStream_t stream)
{
    GatherLaunch g;
    bool pow2, off64;
    if (!gather_dev::fill_launch<VecT>(g, a, row_begin, row_end, &pow2, &off64)) return hipErrorInvalidValue;
    const int64_t n_items = (int64_t)(row_end - row_begin) * g.vpr;

    // Small workgroups: a workgroup's wave slots come free only when its slowest wave is done, and a tile of one or two
    // waves wastes fewer of them than one of eight (128 threads against 512 on the workloads of bench.py: 1 to 6.5 %
    // less time, never more).  Rows of 256 bytes (sixteen vectors) have a kernel of their own that fetches the kept
    // indices by scalar loads; it runs best as single waves (64 threads: another 2 to 6 % on all but one workload).
    const bool rows16_shape = sizeof(VecT) == 16 && g.vpr == 16;
    // ... and so do longer rows that are a power of two of vectors (512 bytes: +2.5 %, 2 KB: +2 %; rows of 128 bytes, eight to
    // a wave, measured 1.4 % slower than with per-lane index loads and stay with the general kernel)
    const bool wave_rows_shape = sizeof(VecT) == 16 && pow2 && g.vpr >= 32;
    int block = tuning::get("SIRLLM_GATHER_BLOCK", rows16_shape || wave_rows_shape ? 64 : 128);
    if (block != 64 && block != 256 && block != 512) block = 128;
    const int unroll = block == 64 ? 1 : (tuning::get("SIRLLM_GATHER_UNROLL", 1) == 2 ? 2 : 1);
    const bool nt = block == 64 || tuning::get("SIRLLM_GATHER_NT", 1) != 0;
    const bool scalar_idx = tuning::get("SIRLLM_GATHER_SCALAR_IDX", 1) != 0;
    const bool rows16 = rows16_shape && unroll == 1 && nt && (block == 64 || block == 128) && scalar_idx;
    const bool wave_rows = wave_rows_shape && block == 64 && scalar_idx;
    // source planes a power of two apart: see gather_tile_wave_rows
    // (and compacted planes of 1 MiB and more: below that the dips only show on lists that are one run, and the
    // exchange costs 3-6 % on scattered lists once there are thousands of planes)
    const bool pow2_planes = a.s_head > 0 && (a.s_head & (a.s_head - 1)) == 0 && (int64_t)a.n_keep * a.d_pos >= (1 << 20);
    const bool rotate = tuning::get("SIRLLM_GATHER_ROTATE", pow2_planes ? 1 : 0) != 0;
    const int per_block = block * unroll;
    const unsigned n_tiles = (unsigned)((n_items + per_block - 1) / per_block);
    g.rotate = rotate ? (int)(n_tiles & ~7u) : 0;
    const int planes = a.n_tensors * g.lh;
    constexpr int kMaxDim = 65535;
    for (int s0 = 0; s0 < a.n_streams; s0 += kMaxDim) {
        for (int p0 = 0; p0 < planes; p0 += kMaxDim) {
            g.stream0 = s0;
            g.plane0 = p0;
            const dim3 grid(n_tiles, (unsigned)min(kMaxDim, planes - p0), (unsigned)min(kMaxDim, a.n_streams - s0));
            const WaveRowsArgs w = gather_dev::wave_rows_args(g, nullptr);
            if (wave_rows) {
                if (g.vpr == 32) {
                    if (off64) hipLaunchKernelGGL((gather_wave_rows_kernel<5, true>), grid, dim3(64), 0, stream, w);
                    else       hipLaunchKernelGGL((gather_wave_rows_kernel<5, false>), grid, dim3(64), 0, stream, w);
                } else {
                    if (off64) hipLaunchKernelGGL((gather_wave_rows_kernel<6, true>), grid, dim3(64), 0, stream, w);
                    else       hipLaunchKernelGGL((gather_wave_rows_kernel<6, false>), grid, dim3(64), 0, stream, w);
                }
            } else if (rows16) {
                if (block == 64) {
                    if (off64) hipLaunchKernelGGL((gather_rows16_kernel<64, true>), grid, dim3(64), 0, stream, w);
                    else       hipLaunchKernelGGL((gather_rows16_kernel<64, false>), grid, dim3(64), 0, stream, w);
                } else {
                    if (off64) hipLaunchKernelGGL((gather_rows16_kernel<128, true>), grid, dim3(128), 0, stream, w);
                    else       hipLaunchKernelGGL((gather_rows16_kernel<128, false>), grid, dim3(128), 0, stream, w);
                }
            } else if (block == 64) {
                launch_shape<VecT, 64, 1, true>(g, grid, pow2, off64, stream);
            } else if (block == 256) {
                if (unroll == 2) { if (nt) launch_shape<VecT, 256, 2, true>(g, grid, pow2, off64, stream); else launch_shape<VecT, 256, 2, false>(g, grid, pow2, off64, stream); }
                else             { if (nt) launch_shape<VecT, 256, 1, true>(g, grid, pow2, off64, stream); else launch_shape<VecT, 256, 1, false>(g, grid, pow2, off64, stream); }
            } else if (block == 512) {
                if (unroll == 2) { if (nt) launch_shape<VecT, 512, 2, true>(g, grid, pow2, off64, stream); else launch_shape<VecT, 512, 2, false>(g, grid, pow2, off64, stream); }
                else             { if (nt) launch_shape<VecT, 512, 1, true>(g, grid, pow2, off64, stream); else launch_shape<VecT, 512, 1, false>(g, grid, pow2, off64, stream); }
            } else {
                if (unroll == 2) { if (nt) launch_shape<VecT, 128, 2, true>(g, grid, pow2, off64, stream); else launch_shape<VecT, 128, 2, false>(g, grid, pow2, off64, stream); }
                else             { if (nt) launch_shape<VecT, 128, 1, true>(g, grid, pow2, off64, stream); else launch_shape<VecT, 128, 1, false>(g, grid, pow2, off64, stream); }
            }
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

// Per-layer buffers: the default launch shapes only (one vector per lane, non-temporal accesses).
template <typename VecT>
hipError_t launch_vec_layers(const GatherArgs& a, const LayerTable& t, hipStream_t stream)
{
    GatherLaunch g;
    bool pow2, off64;
    if (!gather_dev::fill_launch<VecT>(g, a, 0, a.n_keep, &pow2, &off64)) return hipErrorInvalidValue;
    const int64_t n_items = (int64_t)a.n_keep * g.vpr;
    // rows of 256 bytes: single-wave tiles with scalar index loads, as in launch_vec
    const bool rows16 = sizeof(VecT) == 16 && g.vpr == 16;
    const bool pow2_planes = a.s_head > 0 && (a.s_head & (a.s_head - 1)) == 0 && (int64_t)a.n_keep * a.d_pos >= (1 << 20);
    const unsigned n_tiles = (unsigned)((n_items + (rows16 ? 63 : 127)) / (rows16 ? 64 : 128));
    g.rotate = rows16 && pow2_planes ? (int)(n_tiles & ~7u) : 0;
    const int planes = a.n_tensors * g.lh;            // at most 2 * 32 * n_heads
    constexpr int kMaxDim = 65535;
    const dim3 block(rows16 ? 64 : 128);
    for (int s0 = 0; s0 < a.n_streams; s0 += kMaxDim) {
        for (int p0 = 0; p0 < planes; p0 += kMaxDim) {
            g.stream0 = s0;
            g.plane0 = p0;
            const dim3 grid(n_tiles, (unsigned)min(kMaxDim, planes - p0), (unsigned)min(kMaxDim, a.n_streams - s0));
            if (rows16) {
                const WaveRowsArgs w = gather_dev::wave_rows_args(g, nullptr);
                if (off64) hipLaunchKernelGGL((gather_rows16_layers_kernel<true>), grid, block, 0, stream, w, t);
                else       hipLaunchKernelGGL((gather_rows16_layers_kernel<false>), grid, block, 0, stream, w, t);
            } else if (pow2) {
                if (off64) hipLaunchKernelGGL((gather_rows_layers_kernel<VecT, true, true>), grid, block, 0, stream, g, t);
                else       hipLaunchKernelGGL((gather_rows_layers_kernel<VecT, true, false>), grid, block, 0, stream, g, t);
            } else {
                if (off64) hipLaunchKernelGGL((gather_rows_layers_kernel<VecT, false, true>), grid, block, 0, stream, g, t);
                else       hipLaunchKernelGGL((gather_rows_layers_kernel<VecT, false, false>), grid, block, 0, stream, g, t);
            }
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

// Ragged batches: default launch shapes only.
template <typename VecT>
hipError_t launch_vec_ragged(const GatherArgs& a, const gather_dev::Ragged& rg, hipStream_t stream)
{
    GatherLaunch g;
    bool pow2, off64;
    if (!gather_dev::fill_launch<VecT>(g, a, 0, a.n_keep, &pow2, &off64)) return hipErrorInvalidValue;
    const int64_t n_items = (int64_t)a.n_keep * g.vpr;
    const bool wave_rows = sizeof(VecT) == 16 && pow2 && g.vpr >= 16;
    const bool pow2_planes = a.s_head > 0 && (a.s_head & (a.s_head - 1)) == 0 && (int64_t)a.n_keep * a.d_pos >= (1 << 20);
    const int per_block = wave_rows ? 64 : 128;
    const unsigned n_tiles = (unsigned)((n_items + per_block - 1) / per_block);
    g.rotate = wave_rows && pow2_planes ? (int)(n_tiles & ~7u) : 0;
    const int planes = a.n_tensors * g.lh;
    constexpr int kMaxDim = 65535;
    const dim3 block(per_block);
    for (int s0 = 0; s0 < a.n_streams; s0 += kMaxDim) {
        for (int p0 = 0; p0 < planes; p0 += kMaxDim) {
            g.stream0 = s0;
            g.plane0 = p0;
            const dim3 grid(n_tiles, (unsigned)min(kMaxDim, planes - p0), (unsigned)min(kMaxDim, a.n_streams - s0));
            if (wave_rows) {
                const WaveRowsArgs w = gather_dev::wave_rows_args(g, &rg);
                const int lv = g.vpr == 16 ? 4 : g.vpr == 32 ? 5 : 6;
                if (lv == 4) {
                    if (off64) hipLaunchKernelGGL((gather_wave_rows_ragged_kernel<4, true>), grid, block, 0, stream, w);
                    else       hipLaunchKernelGGL((gather_wave_rows_ragged_kernel<4, false>), grid, block, 0, stream, w);
                } else if (lv == 5) {
                    if (off64) hipLaunchKernelGGL((gather_wave_rows_ragged_kernel<5, true>), grid, block, 0, stream, w);
                    else       hipLaunchKernelGGL((gather_wave_rows_ragged_kernel<5, false>), grid, block, 0, stream, w);
                } else {
                    if (off64) hipLaunchKernelGGL((gather_wave_rows_ragged_kernel<6, true>), grid, block, 0, stream, w);
                    else       hipLaunchKernelGGL((gather_wave_rows_ragged_kernel<6, false>), grid, block, 0, stream, w);
                }
            } else if (pow2) {
                if (off64) hipLaunchKernelGGL((gather_rows_ragged_kernel<VecT, true, true>), grid, block, 0, stream, g, rg);
                else       hipLaunchKernelGGL((gather_rows_ragged_kernel<VecT, true, false>), grid, block, 0, stream, g, rg);
            } else {
                if (off64) hipLaunchKernelGGL((gather_rows_ragged_kernel<VecT, false, true>), grid, block, 0, stream, g, rg);
                else       hipLaunchKernelGGL((gather_rows_ragged_kernel<VecT, false, false>), grid, block, 0, stream, g, rg);
            }
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

}  // namespace

hipError_t launch_gather_ragged(const GatherArgs& a, const int32_t* held_dev, const int32_t* cu_new_dev,
                                const int32_t* n_keep_dev, int32_t budget, hipStream_t stream)
{
    if (a.n_keep <= 0 || a.n_streams <= 0 || a.row_bytes <= 0 || a.n_layers <= 0 || a.n_heads <= 0) return hipSuccess;
    const gather_dev::Ragged rg{held_dev, cu_new_dev, n_keep_dev, budget};
    switch (gather_dev::vector_bytes(a)) {
    case 16: return launch_vec_ragged<u32x4>(a, rg, stream);
    case 8:  return launch_vec_ragged<u32x2>(a, rg, stream);
    case 4:  return launch_vec_ragged<uint32_t>(a, rg, stream);
    case 2:  return launch_vec_ragged<uint16_t>(a, rg, stream);
    default: return launch_vec_ragged<uint8_t>(a, rg, stream);
    }
}

hipError_t launch_gather_layers(const GatherArgs& a, const LayerTable& t, hipStream_t stream)
{
    if (a.n_keep <= 0 || a.n_streams <= 0 || a.row_bytes <= 0 || a.n_layers <= 0 || a.n_heads <= 0) return hipSuccess;
    if (a.n_layers > kLayerTable) return hipErrorInvalidValue;
    // the widest access every address of the call is a multiple of: strides and row size, and every layer's pointers
    uint64_t bits = (uint64_t)gather_dev::vector_bytes(a, false);
    for (int x = 0; x < a.n_tensors; ++x)
        for (int l = 0; l < a.n_layers; ++l) bits |= (uint64_t)(uintptr_t)t.src[x][l] | (uint64_t)(uintptr_t)t.dst[x][l];
    switch (gather_dev::widest_access(bits)) {
    case 16: return launch_vec_layers<u32x4>(a, t, stream);
    case 8:  return launch_vec_layers<u32x2>(a, t, stream);
    case 4:  return launch_vec_layers<uint32_t>(a, t, stream);
    case 2:  return launch_vec_layers<uint16_t>(a, t, stream);
    default: return launch_vec_layers<uint8_t>(a, t, stream);
    }
}

hipError_t launch_gather(const GatherArgs& a, int row_begin, int row_end, hipStream_t stream)
{
    if (row_end <= row_begin || a.n_streams <= 0 || a.row_bytes <= 0 || a.n_layers <= 0 || a.n_heads <= 0)
        return hipSuccess;
    switch (gather_dev::vector_bytes(a)) {
    case 16: return launch_vec<u32x4>(a, row_begin, row_end, stream);
    case 8:  return launch_vec<u32x2>(a, row_begin, row_end, stream);
    case 4:  return launch_vec<uint32_t>(a, row_begin, row_end, stream);
    case 2:  return launch_vec<uint16_t>(a, row_begin, row_end, stream);
    default: return launch_vec<uint8_t>(a, row_begin, row_end, stream);
    }
}

}  // namespace sirllm
