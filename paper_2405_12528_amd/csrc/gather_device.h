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

// A streaming store of bytes that this launch never touches again: base (wave uniform) + off.  16-byte vectors go
// out at agent scope with the non-temporal hint (`sc1 nt`): written through instead of left dirty in the L2, which
// measured 6.7 against 6.3 TB/s for a plain 1 GiB fill and 1 % on the gather; the other widths take the compiler's
// non-temporal store.
// The instruction is written out, so the compiler does not see a store there.  What it would otherwise look after is
// spelled out around it: five wait states in front (a scalar base that a vector instruction has just written, e.g. a
// v_readfirstlane, must not be read sooner) and two behind (a store of more than 8 bytes must have read its data
// registers before they are overwritten; a kernel that ends right after the store does not need them, one that loops
// does).  A few cycles in a wave that lives for microseconds: no difference in time (159.0 us either way).
template <typename VecT, typename OffT>
__device__ __forceinline__ void st_stream(char* base, OffT off, VecT v)
{
    if constexpr (sizeof(VecT) == 16 && sizeof(OffT) == 4) {
        asm volatile("s_nop 4\n\tglobal_store_dwordx4 %0, %1, %2 sc1 nt\n\ts_nop 1" ::"v"(off), "v"(v), "s"(base) : "memory");
    } else if constexpr (sizeof(VecT) == 16) {
        char* p = base + off;
        asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
    } else {
        __builtin_nontemporal_store(v, (VecT*)(base + off));
    }
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
    int32_t rotate;       // single-wave tiles: tiles below this index (a multiple of eight; 0: none) are exchanged inside their
                          // group of eight, differently from plane to plane
};

// Ragged batches: per-stream slot counts in device memory.
struct Ragged {
    const int32_t* held_dev;    // null: uniform batch
    const int32_t* cu_new_dev;
    const int32_t* n_keep_dev;  // written by the selection launch that precedes this one on the stream
    int32_t budget;
};

// Ragged batch: does stream s compact at all?  A stream the selection flagged (sizes negative or beyond the
// caller's bounds: n_keep = -1) has no kept list of this call; its K/V stays as it is.  So does a stream that
// is within its budget.  Returns the stream's slot count, or -1 when nothing moves.
__device__ __forceinline__ int ragged_n_src(const Ragged& rg, int s, int n_src_bound)
{
    const int n_cand = rg.held_dev[s] + (rg.cu_new_dev[s + 1] - rg.cu_new_dev[s]);
    if (rg.n_keep_dev[s] < 0 || n_cand <= rg.budget || n_cand > n_src_bound) return -1;
    return n_cand;
}

// Ragged batch, out of place: every stream the selection accepted is moved, its n_keep_dev[s] kept rows (all of its
// rows, in place order, while it is within its budget), so that afterwards the whole batch lives in the destination.
// Returns the stream's slot count and its row count, or -1 for a flagged stream (nothing of it is touched).
__device__ __forceinline__ int ragged_rows(const Ragged& rg, int s, int n_src_bound, int n_rows_bound, int& n_rows)
{
    const int n_cand = rg.held_dev[s] + (rg.cu_new_dev[s + 1] - rg.cu_new_dev[s]);
    const int nk = rg.n_keep_dev[s];
    if (nk < 0 || n_cand > n_src_bound) return -1;
    n_rows = nk < n_rows_bound ? nk : n_rows_bound;
    return n_cand;
}

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
        if (live[u]) {
            if constexpr (NT) st_stream<VecT, off_t>(dp, doff[u], v[u]);
            else st<VecT, false>(dp + doff[u], v[u]);
        }
}

// A tile for rows that are a power of two of 16-byte vectors, at least sixteen (256 bytes), one vector per lane.
// LV = log2(vectors per row) for rows of 16 or 32 vectors: a wave covers 4 or 2 whole rows; LV = 6 stands for
// every row of 64 vectors or more (the real shift is g.shift): a wave covers 64 consecutive vectors of ONE row.  Either
// way the wave's kept indices are wave-uniform, so they come through the scalar cache (scalar loads from clamped
// positions, the list read through the constant address space) instead of one vector load per lane; each lane then
// picks its row's index.  Every kernel argument the wave needs is requested in one batch at its start, the indices in
// a second one: two scalar round trips, then the wave's first vector memory operation is the row load itself.  The
// kept list must not be written while the launch runs, which every caller of the compaction already guarantees:
// destination buffers and kept list may not overlap.
// LAYERS: the cache is one buffer per layer and tensor, `table` holds their base pointers (else it is not read).
// RAGGED: every stream has its own slot and row counts in device memory, a flagged stream is left alone.
//
// The arguments of such a tile, packed so that every dword a wave fetches is one it needs (the compiler then has no
// dead lane of a wide scalar load to reuse for a later load, which would force a wait in between).
struct WaveRowsArgs {
    uint64_t idx_base;                 // kept_idx
    int64_t idx_stride;
    uint64_t src0, src1, dst0, dst1;   // K | V bases (unused with LAYERS)
    int64_t s_stream, d_stream, s_head, d_head, s_layer, d_layer, s_pos, d_pos;
    int32_t row_begin, row_end, lh, uniform, n_heads, n_src, shift, rotate, plane0, stream0;
    uint64_t rg_held, rg_cu, rg_keep;  // RAGGED: n_held, cu_new, n_keep per stream
};

inline WaveRowsArgs wave_rows_args(const GatherLaunch& g, const Ragged* rg)
{
    WaveRowsArgs w;
    const GatherArgs& a = g.a;
    w.idx_base = (uint64_t)(uintptr_t)a.kept_idx; w.idx_stride = a.idx_stride;
    w.src0 = (uint64_t)(uintptr_t)a.src[0]; w.src1 = (uint64_t)(uintptr_t)a.src[1];
    w.dst0 = (uint64_t)(uintptr_t)a.dst[0]; w.dst1 = (uint64_t)(uintptr_t)a.dst[1];
    w.s_stream = a.s_stream; w.d_stream = a.d_stream; w.s_head = a.s_head; w.d_head = a.d_head;
    w.s_layer = a.s_layer; w.d_layer = a.d_layer; w.s_pos = a.s_pos; w.d_pos = a.d_pos;
    w.row_begin = g.row_begin; w.row_end = g.row_end; w.lh = g.lh; w.uniform = g.uniform; w.n_heads = a.n_heads;
    w.n_src = a.n_src; w.shift = g.shift; w.rotate = g.rotate; w.plane0 = g.plane0; w.stream0 = g.stream0;
    w.rg_held = rg ? (uint64_t)(uintptr_t)rg->held_dev : 0;
    w.rg_cu = rg ? (uint64_t)(uintptr_t)rg->cu_new_dev : 0;
    w.rg_keep = rg ? (uint64_t)(uintptr_t)rg->n_keep_dev : 0;
    return w;
}

template <int BLOCK, bool NT, bool OFF64, int LV, bool LAYERS = false, bool RAGGED = false>
__device__ __forceinline__ void gather_tile_wave_rows(const WaveRowsArgs& w, int tile, int plane_in_launch, int stream_in_launch,
                                                      const LayerTable* table = nullptr)
{
    static_assert(BLOCK % 64 == 0 && LV >= 4 && LV <= 6, "whole waves; rows of 16, 32 or >= 64 vectors");
    constexpr int R = 64 >> LV;                                       // whole rows per wave (1: one row, or a part of one)
    using VecT = u32x4;
    using off_t = typename std::conditional<OFF64, int64_t, uint32_t>::type;
    typedef const __attribute__((address_space(4))) int32_t* const_idx_t;     // read-only for the whole launch: scalar loads
    typedef const __attribute__((address_space(1))) char* gsrc_t;
    typedef __attribute__((address_space(1))) char* gdst_t;
    // one batch of scalar loads from the argument block
    uint64_t idx_base = w.idx_base;
    int64_t idx_stride = w.idx_stride;
    int row_begin = w.row_begin, row_end = w.row_end, lh = w.lh, uniform = w.uniform, n_heads = w.n_heads, n_src = w.n_src;
    int shift = LV < 6 ? LV : w.shift, rotate_below = w.rotate, plane = w.plane0 + plane_in_launch,
        stream = w.stream0 + stream_in_launch;
    uint64_t src0 = w.src0, src1 = w.src1, dst0 = w.dst0, dst1 = w.dst1;
    int64_t s_stream = w.s_stream, d_stream = w.d_stream, s_head = w.s_head, d_head = w.d_head, s_layer = w.s_layer,
            d_layer = w.d_layer, s_pos = w.s_pos, d_pos = w.d_pos;
    uint64_t rg_held = RAGGED ? w.rg_held : 0, rg_cu = RAGGED ? w.rg_cu : 0, rg_keep = RAGGED ? w.rg_keep : 0;
    asm volatile("" : "+s"(idx_base), "+s"(idx_stride), "+s"(src0), "+s"(src1), "+s"(dst0), "+s"(dst1));
    asm volatile("" : "+s"(s_stream), "+s"(d_stream), "+s"(s_head), "+s"(d_head), "+s"(s_layer), "+s"(d_layer), "+s"(s_pos), "+s"(d_pos));
    asm volatile("" : "+s"(row_begin), "+s"(row_end), "+s"(lh), "+s"(uniform), "+s"(n_heads), "+s"(n_src), "+s"(shift),
                      "+s"(rotate_below), "+s"(plane), "+s"(stream));
    if constexpr (RAGGED) asm volatile("" : "+s"(rg_held), "+s"(rg_cu), "+s"(rg_keep));

    int n_rows = row_end - row_begin;                                // ragged batch: an upper bound until the stream's own count is in
    const int lane = (int)threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    // Workgroups are dealt to the eight XCDs round robin and a plane holds a multiple of eight tiles, so XCD x would
    // copy tile 8 m + x of EVERY plane: one fixed eighth of the addresses modulo eight tiles.  When the planes also lie
    // a power of two apart, an XCD's traffic then keeps falling on the same few channels (measured: 5.2-5.9 instead of
    // 6.5 TB/s on long runs of kept slots).  Exchanging the tiles of each group of eight by the plane index gives every
    // XCD every residue in turn.  It costs 3-7 % where nothing needs curing (many planes, strides that are no power of
    // two), so the launcher asks for it only where it pays (rotate_below: the end of the last whole group, or 0).
    if (tile < rotate_below) tile ^= plane & 7;
    const int item0 = (tile * (BLOCK / 64) + wave) * 64;             // the wave's first vector, counted over the plane's rows
    const int r0 = item0 >> shift;                                   // its first row (relative to row_begin)
    if (r0 >= n_rows) return;                                        // wave-uniform
    const int last = n_rows - 1;
    const int tensor = plane >= lh ? 1 : 0;
    const int ph = plane - tensor * lh;
    const_idx_t idx = (const_idx_t)(idx_base + (uint64_t)((stream * idx_stride + row_begin) * 4));
    int32_t iv[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) iv[q] = q < R ? idx[min(r0 + q, last)] : 0;
    if constexpr (RAGGED) {
        // The stream's own sizes, in the same batch of scalar loads as the indices (which were clamped by the bound:
        // the kept list has that many entries for every stream).  Inputs of the launch, or written by the selection
        // launch before it: read-only here.
        int32_t held = ((const_idx_t)rg_held)[stream];
        int32_t cu0 = ((const_idx_t)rg_cu)[stream], cu1 = ((const_idx_t)rg_cu)[stream + 1];
        int32_t nk = ((const_idx_t)rg_keep)[stream];
        asm volatile("" : "+s"(held), "+s"(cu0), "+s"(cu1), "+s"(nk), "+s"(iv[0]), "+s"(iv[1]), "+s"(iv[2]), "+s"(iv[3]));
        const int n_cand = held + (cu1 - cu0);
        if (nk < 0 || n_cand > n_src) return;                        // a stream the selection flagged: nothing of it is touched
        n_src = n_cand;
        n_rows = nk < n_rows ? nk : n_rows;
        if (r0 >= n_rows) return;
    }
    uint64_t sbase, dbase;
    int64_t so, dof;
    if constexpr (LAYERS) {
        const int l = ph / n_heads, h = ph - l * n_heads;
        sbase = (uint64_t)(uintptr_t)table->src[tensor][l];          // second batch, together with the indices
        dbase = (uint64_t)(uintptr_t)table->dst[tensor][l];
        asm volatile("" : "+s"(sbase), "+s"(dbase));
        so = h * s_head;
        dof = h * d_head;
    } else {
        sbase = tensor ? src1 : src0;
        dbase = tensor ? dst1 : dst0;
        if (uniform) {
            so = ph * s_head;
            dof = ph * d_head;
        } else {
            const int l = ph / n_heads, h = ph - l * n_heads;
            so = l * s_layer + h * s_head;
            dof = l * d_layer + h * d_head;
        }
    }
    // every index requested before any is looked at
    if constexpr (R == 4) asm volatile("" : "+s"(iv[0]), "+s"(iv[1]), "+s"(iv[2]), "+s"(iv[3]));
    else if constexpr (R == 2) asm volatile("" : "+s"(iv[0]), "+s"(iv[1]));
    else asm volatile("" : "+s"(iv[0]));
    const gsrc_t sp = (gsrc_t)(sbase + (uint64_t)(stream * s_stream + so));
    const gdst_t dp = (gdst_t)(dbase + (uint64_t)(stream * d_stream + dof));

    const int r = R > 1 ? lane >> (LV < 6 ? LV : 0) : 0;             // which of the wave's rows
    const int c = (item0 + lane) & ((1 << shift) - 1);               // which vector of the row
    uint32_t i = (uint32_t)iv[0];
#pragma unroll
    for (int q = 1; q < R; ++q) i = r == q ? (uint32_t)iv[q] : i;
    if (r0 + r >= n_rows) return;
    const int j = row_begin + r0 + r;
    VecT v = VecT{};
    if (i < (uint32_t)n_src) {                                       // an index with no source slot leaves a zero row
        const auto* p = (const __attribute__((address_space(1))) VecT*)(sp + ((off_t)i * (off_t)s_pos + (off_t)(c * 16)));
        v = NT ? __builtin_nontemporal_load(p) : *p;
    }
    const off_t qoff = (off_t)j * (off_t)d_pos + (off_t)(c * 16);
    if constexpr (NT) st_stream<VecT, off_t>((char*)(uintptr_t)(uint64_t)dp, qoff, v);
    else *(__attribute__((address_space(1))) VecT*)(dp + qoff) = v;
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
    g.rotate = 0;
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
