// In-place KV compaction (paper Sec. 3.3: KV_cache <- KV_cache[Id], written back into the same
// buffer).  The kept list is strictly ascending, so row j always comes from a slot kept_idx[j] >= j:
// rows only move towards the front, and a row that has been written is never read again.  The one hazard is
// write-after-read: row j may be overwritten only after whoever needs the old row j as a source -- a
// destination row j' <= j -- has read it.  One workgroup owns one plane (stream, layer, K|V, head) and
// walks it front to back in chunks: every lane loads its vectors of the chunk, the workgroup waits
// until all of those loads have landed, then stores; the loads of the next chunk are already in flight
// by then.  A chunk writes rows [c0, c1) and reads rows >= c0; the next chunk reads rows >= c1 only, so
// nothing a chunk writes is ever read again and no ordering between workgroups is needed.  Rows that stay where
// they are (the sinks, any leading run of kept slots) are neither read nor written.  Same HBM traffic per moved
// row as the out-of-place gather, half the K/V memory.
//
// Which workgroup walks which plane: by block index, or -- given four bytes of scratch for a counter -- by a ticket
// drawn when the workgroup starts.  Block indices are dealt to the chip's eight dies round-robin and every die works
// through its share at its own pace; over a batch of tens of thousands of planes the dies drift apart and the
// workgroups in flight end up walking planes that lie gigabytes apart.  With tickets the planes being walked at any
// moment are always neighbours, which the memory system serves faster (32 streams x 2048 planes: 5.6 -> 6.0 TB/s;
// no difference for a few thousand planes, so the launcher uses tickets from 8192 planes on).
#include "common.h"
#include "gather_device.h"
#include "tuning.h"

namespace sirllm {
namespace {

using gather_dev::GatherLaunch;

using gather_dev::Ragged;
using gather_dev::ragged_n_src;

// Base address of plane `plane` of stream `stream` (uniform over the workgroup: scalar arithmetic).
__device__ __forceinline__ char* plane_base(const GatherLaunch& g, int plane, int stream)
{
    const GatherArgs& a = g.a;
    const int tensor = plane >= g.lh ? 1 : 0;
    const int ph = plane - tensor * g.lh;
    int64_t so;
    if (g.uniform) {
        so = ph * a.s_head;
    } else {
        const int l = ph / a.n_heads, h = ph - l * a.n_heads;
        so = l * a.s_layer + h * a.s_head;
    }
    return a.dst[tensor] + stream * a.s_stream + so;
}

// A kernel, not a memset: the call may be recorded into a HIP graph.
__global__ void ticket_clear_kernel(int32_t* ticket) { *ticket = 0; }

// The walk of one plane by one workgroup.  base_of(plane, stream) is where that plane starts: by the layout's strides
// when the cache is one buffer per tensor, from a table of pointers when it is one buffer per layer.
template <typename VecT, int BLOCK, int UNROLL, bool NT, bool POW2, bool OFF64, typename BaseOf>
__device__ __forceinline__ void inplace_walk(GatherLaunch g, const Ragged& rg, int32_t* ticket, BaseOf base_of)
{
    // Which plane: by block index, or -- with a ticket counter -- the next one in the order in which workgroups
    // actually start, so that the workgroups in flight always walk neighbouring planes.  Every ticket below the
    // grid size is drawn exactly once, so every plane is walked exactly once.
    int bx = (int)blockIdx.x, by = (int)blockIdx.y, bz = (int)blockIdx.z;
    if (ticket) {
        __shared__ int s_t;
        if (threadIdx.x == 0) s_t = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        const uint32_t t = (uint32_t)s_t;
        if (t >= gridDim.x * gridDim.y * gridDim.z) return;            // cannot happen with a cleared counter
        bx = (int)(t % gridDim.x);
        by = (int)((t / gridDim.x) % gridDim.y);
        bz = (int)(t / (gridDim.x * gridDim.y));
    }
    if (rg.held_dev) {
        // ragged batch: this stream's own slot count decides whether anything moves at all
        const int n_cand = ragged_n_src(rg, g.stream0 + by, g.a.n_src);
        if (n_cand < 0) return;                                        // uniform over the workgroup
        g.a.n_src = n_cand;
    }
    const GatherArgs& a = g.a;
    using off_t = typename std::conditional<OFF64, int64_t, uint32_t>::type;
    const int stream = g.stream0 + by;
    // bz picks one column part of the rows: parts never share a byte, so they need no ordering
    char* base = base_of(g.plane0 + bx, stream) + (int64_t)bz * (g.vpr * (int)sizeof(VecT));
    const int32_t* idx = a.kept_idx + stream * a.idx_stride;

    const int n_items = (g.row_end - g.row_begin) * g.vpr;
    constexpr int CH = BLOCK * UNROLL;
    // The destination offsets and move flags ride through the waits in registers on purpose: at the default shape
    // (1024 threads x 4 vectors) that puts the kernel at 72 vector registers, i.e. ONE workgroup per CU.  The same
    // kernel trimmed to 40 registers (offsets recomputed at store time), two workgroups per CU, measured 3-5 %
    // slower on every shape: with a walk per workgroup, more walks in flight serve the memory system worse.
    VecT va[UNROLL], vb[UNROLL];
    off_t da[UNROLL], db[UNROLL];
    bool ma[UNROLL], mb[UNROLL];
    // Every wave issues UNROLL row loads per chunk (and the UNROLL kept_idx loads their addresses need), whatever
    // its rows need: a lane past the end, a row that stays in place or an index with no source slot re-reads a
    // harmless address and drops the data.  The loads are unconditional instructions -- no branch may ever skip
    // one -- because the wait below counts instructions.
    auto load_chunk = [&](VecT (&v)[UNROLL], off_t (&doff)[UNROLL], bool (&moved)[UNROLL], int c0) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int w = c0 + u * BLOCK + (int)threadIdx.x;
            const bool in = w < n_items;
            const int wc = in ? w : n_items - 1;
            int j, c;
            if constexpr (POW2) { j = wc >> g.shift; c = wc & (g.vpr - 1); }
            else                { j = wc / g.vpr;    c = wc - j * g.vpr; }
            j += g.row_begin;
            const uint32_t i = (uint32_t)idx[j];
            const bool ok = i < (uint32_t)a.n_src;                     // an index with no source slot leaves a zero row
            moved[u] = in && i != (uint32_t)j;
            doff[u] = (off_t)j * (off_t)a.s_pos + (off_t)(c * (int)sizeof(VecT));
            const uint32_t isrc = (moved[u] && ok) ? i : (uint32_t)j;
            const VecT x = gather_dev::ld<VecT, NT>(base + ((off_t)isrc * (off_t)a.s_pos + (off_t)(c * (int)sizeof(VecT))));
            v[u] = (moved[u] && !ok) ? VecT{} : x;
        }
    };
    auto store_chunk = [&](const VecT (&v)[UNROLL], const off_t (&doff)[UNROLL], const bool (&moved)[UNROLL]) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            if (moved[u]) gather_dev::st<VecT, NT>(base + doff[u], v[u]);
    };
    // A chunk's sources lie at or behind its own first row, i.e. behind every row an earlier chunk writes: loads may
    // run ahead of stores, and only a chunk's own stores have to wait for its own loads (of the whole workgroup).
    // So the loads of chunk c + 1 go out before the workgroup waits for chunk c.
    //
    // The wait.  vmcnt is the wave's count of vector-memory instructions (loads and stores) that have not completed;
    // loads complete in the order they were issued (stores may overtake or lag loads, which does not matter here).
    // At `s_waitcnt vmcnt(UNROLL)` the wave has issued, after the last row load of chunk c, at least the UNROLL
    // row loads of chunk c + 1.  If a load of chunk c were still outstanding, so would be all UNROLL younger row
    // loads, UNROLL + 1 operations in all; hence "at most UNROLL outstanding" implies chunk c has landed in this
    // wave, and the barrier extends that to the workgroup.  What an edit must keep: (1) between the loads of
    // chunk c and the wait, every wave issues at least UNROLL further vector-memory LOADS, unconditionally (they
    // may be more: the kept_idx loads of chunk c + 1 also count, and so do the stores of chunk c - 1, which only
    // makes the wait stricter); (2) nothing that completes out of order with the row loads (an LDS-direct load,
    // a scalar load of row data) may carry row data; (3) the barrier stays directly behind the wait, the stores
    // behind the barrier.  The compiler adds waits of its own for the data it stores; they can only be stricter.
    load_chunk(va, da, ma, 0);
    for (int c0 = 0; c0 < n_items; c0 += 2 * CH) {
        load_chunk(vb, db, mb, c0 + CH);
        asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(UNROLL) : "memory");
        store_chunk(va, da, ma);
        __builtin_amdgcn_sched_barrier(0);
        load_chunk(va, da, ma, c0 + 2 * CH);
        asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(UNROLL) : "memory");
        store_chunk(vb, db, mb);
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <typename VecT, int BLOCK, int UNROLL, bool NT, bool POW2, bool OFF64>
__global__ __launch_bounds__(BLOCK) void gather_inplace_kernel(GatherLaunch g, Ragged rg, int32_t* ticket)
{
    inplace_walk<VecT, BLOCK, UNROLL, NT, POW2, OFF64>(g, rg, ticket,
                                                      [&](int plane, int stream) { return plane_base(g, plane, stream); });
}

// One buffer per layer and tensor: the default launch shape only; the table of base pointers rides in the kernel
// arguments (t.dst; t.src is not used, source and destination are the same buffers).
template <typename VecT, bool POW2, bool OFF64>
__global__ __launch_bounds__(1024) void gather_inplace_layers_kernel(GatherLaunch g, Ragged rg, int32_t* ticket, LayerTable t)
{
    inplace_walk<VecT, 1024, 4, true, POW2, OFF64>(g, rg, ticket, [&](int plane, int stream) {
        const int tensor = plane >= g.lh ? 1 : 0;
        const int ph = plane - tensor * g.lh;
        const int l = ph / g.a.n_heads, h = ph - l * g.a.n_heads;
        return t.dst[tensor][l] + stream * g.a.s_stream + h * g.a.s_head;
    });
}

template <typename VecT, int BLOCK, int UNROLL>
void launch_shape(const GatherLaunch& g, const Ragged& rg, dim3 grid, bool pow2, bool off64, int32_t* ticket, hipStream_t stream)
{
    const dim3 block(BLOCK);
    if (tuning::get("SIRLLM_INPLACE_NT", 1) == 0) {
        if (pow2 && !off64) hipLaunchKernelGGL((gather_inplace_kernel<VecT, BLOCK, UNROLL, false, true, false>), grid, block, 0, stream, g, rg, ticket);
        else hipLaunchKernelGGL((gather_inplace_kernel<VecT, BLOCK, UNROLL, false, false, true>), grid, block, 0, stream, g, rg, ticket);
        return;
    }
    if (pow2) {
        if (off64) hipLaunchKernelGGL((gather_inplace_kernel<VecT, BLOCK, UNROLL, true, true, true>), grid, block, 0, stream, g, rg, ticket);
        else       hipLaunchKernelGGL((gather_inplace_kernel<VecT, BLOCK, UNROLL, true, true, false>), grid, block, 0, stream, g, rg, ticket);
    } else {
        if (off64) hipLaunchKernelGGL((gather_inplace_kernel<VecT, BLOCK, UNROLL, true, false, true>), grid, block, 0, stream, g, rg, ticket);
        else       hipLaunchKernelGGL((gather_inplace_kernel<VecT, BLOCK, UNROLL, true, false, false>), grid, block, 0, stream, g, rg, ticket);
    }
}

template <typename VecT>
hipError_t launch_vec(const GatherArgs& a, const Ragged& rg, int32_t* ticket, const LayerTable* layers, hipStream_t stream)
{
    GatherLaunch g;
    bool pow2, off64;
    if (!gather_dev::fill_launch<VecT>(g, a, 0, a.n_keep, &pow2, &off64)) return hipErrorInvalidValue;
    const int block = tuning::get("SIRLLM_INPLACE_BLOCK", 1024);
    const int unroll = tuning::get("SIRLLM_INPLACE_UNROLL", 4);
    const int planes = a.n_tensors * g.lh;
    // Few planes cannot fill the chip with one workgroup each: cut every row into column parts that are
    // compacted by workgroups of their own (only when vectors per row is a power of two).
    int parts = 1;
    while (pow2 && parts < g.vpr && (int64_t)planes * a.n_streams * parts < 512) parts <<= 1;
    parts = tuning::get("SIRLLM_INPLACE_PARTS", parts);
    while (parts > 1 && (!pow2 || g.vpr % parts != 0)) parts >>= 1;
    if (parts < 1) parts = 1;
    g.vpr /= parts;
    g.shift = 0;
    while (pow2 && (1 << g.shift) < g.vpr) ++g.shift;
    constexpr int kMaxDim = 65535;
    for (int s0 = 0; s0 < a.n_streams; s0 += kMaxDim) {
        g.stream0 = s0;
        g.plane0 = 0;
        const dim3 grid((unsigned)planes, (unsigned)min(kMaxDim, a.n_streams - s0), (unsigned)parts);
        if (ticket) hipLaunchKernelGGL(ticket_clear_kernel, dim3(1), dim3(1), 0, stream, ticket);
        if (layers) {
            const dim3 blk(1024);
            if (pow2) {
                if (off64) hipLaunchKernelGGL((gather_inplace_layers_kernel<VecT, true, true>), grid, blk, 0, stream, g, rg, ticket, *layers);
                else       hipLaunchKernelGGL((gather_inplace_layers_kernel<VecT, true, false>), grid, blk, 0, stream, g, rg, ticket, *layers);
            } else {
                hipLaunchKernelGGL((gather_inplace_layers_kernel<VecT, false, true>), grid, blk, 0, stream, g, rg, ticket, *layers);
            }
        } else if (block == 1024) {
            if (unroll == 2)      launch_shape<VecT, 1024, 2>(g, rg, grid, pow2, off64, ticket, stream);
            else if (unroll == 8) launch_shape<VecT, 1024, 8>(g, rg, grid, pow2, off64, ticket, stream);
            else                  launch_shape<VecT, 1024, 4>(g, rg, grid, pow2, off64, ticket, stream);
        } else if (block == 256) {
            if (unroll == 2)      launch_shape<VecT, 256, 2>(g, rg, grid, pow2, off64, ticket, stream);
            else if (unroll == 8) launch_shape<VecT, 256, 8>(g, rg, grid, pow2, off64, ticket, stream);
            else                  launch_shape<VecT, 256, 4>(g, rg, grid, pow2, off64, ticket, stream);
        } else {
            if (unroll == 2)      launch_shape<VecT, 512, 2>(g, rg, grid, pow2, off64, ticket, stream);
            else if (unroll == 8) launch_shape<VecT, 512, 8>(g, rg, grid, pow2, off64, ticket, stream);
            else                  launch_shape<VecT, 512, 4>(g, rg, grid, pow2, off64, ticket, stream);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_any(const GatherArgs& a, const Ragged& rg, void* scratch, size_t scratch_bytes, const LayerTable* layers,
                      hipStream_t stream)
{
    if (a.n_keep <= 0 || a.n_streams <= 0 || a.row_bytes <= 0 || a.n_layers <= 0 || a.n_heads <= 0)
        return hipSuccess;
    // Ticket order pays once the batch has so many planes that the dies drift apart while they work through them; for
    // a few thousand planes it changes nothing and the launch that clears the counter would only cost its 2-4 us.
    constexpr int64_t kTicketPlanes = 8192;
    const int64_t planes_total = (int64_t)a.n_streams * a.n_tensors * a.n_layers * a.n_heads;
    int32_t* ticket = nullptr;
    const int want = tuning::get("SIRLLM_INPLACE_TICKET", planes_total >= kTicketPlanes ? 1 : 0);
    if (scratch && scratch_bytes >= (size_t)SIRLLM_INPLACE_WORKSPACE_BYTES && want != 0) ticket = (int32_t*)scratch;
    int width = gather_dev::vector_bytes(a, layers == nullptr);
    if (layers) {
        uint64_t bits = (uint64_t)width;
        for (int x = 0; x < a.n_tensors; ++x)
            for (int l = 0; l < a.n_layers; ++l) bits |= (uint64_t)(uintptr_t)layers->dst[x][l];
        width = gather_dev::widest_access(bits);
    }
    switch (width) {
    case 16: return launch_vec<u32x4>(a, rg, ticket, layers, stream);
    case 8:  return launch_vec<u32x2>(a, rg, ticket, layers, stream);
    case 4:  return launch_vec<uint32_t>(a, rg, ticket, layers, stream);
    case 2:  return launch_vec<uint16_t>(a, rg, ticket, layers, stream);
    default: return launch_vec<uint8_t>(a, rg, ticket, layers, stream);
    }
}

}  // namespace

// a.src and a.dst name the same buffers; the s_* strides are used for both sides.
hipError_t launch_gather_inplace(const GatherArgs& a, void* scratch, size_t scratch_bytes, hipStream_t stream)
{
    return launch_any(a, Ragged{nullptr, nullptr, nullptr, 0}, scratch, scratch_bytes, nullptr, stream);
}

// One buffer per layer and tensor: t.dst[x][l] is layer l of tensor x (a.src / a.dst and the layer stride of `a` are
// not used; a.n_layers <= kLayerTable).
hipError_t launch_gather_inplace_layers(const GatherArgs& a, const LayerTable& t, void* scratch, size_t scratch_bytes,
                                        hipStream_t stream)
{
    if (a.n_layers > kLayerTable) return hipErrorInvalidValue;
    return launch_any(a, Ragged{nullptr, nullptr, nullptr, 0}, scratch, scratch_bytes, &t, stream);
}

hipError_t launch_gather_inplace_ragged(const GatherArgs& a, const int32_t* held_dev, const int32_t* cu_new_dev,
                                        const int32_t* n_keep_dev, int32_t budget, void* scratch, size_t scratch_bytes,
                                        hipStream_t stream)
{
    return launch_any(a, Ragged{held_dev, cu_new_dev, n_keep_dev, budget}, scratch, scratch_bytes, nullptr, stream);
}

}  // namespace sirllm
