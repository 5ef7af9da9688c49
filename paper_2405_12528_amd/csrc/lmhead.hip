// Token entropy taken straight from the language-model head (paper Sec. 3.2: the probabilities are the
// model's own softmax output, so the logits are z = h W^T).  The product is never stored: a workgroup
// computes a 256 (vocabulary) x 256 (tokens) tile of z on the matrix cores, reduces it in registers to one
// (max, sum of exponentials, logit of the token) triple per token, and a second small kernel folds the
// triples of all vocabulary tiles with the same monoid the logits scan uses.
//
// MFMA mapping (v_mfma_f32_32x32x16 bf16 / f16, one wave = 64 lanes):
//   operand "A" = 32 vocabulary rows of W, operand "B" = 32 token rows of h, both K-contiguous: lane l holds
//   row l % 32, elements k = 8 * (l / 32) .. + 7 of the 16-wide K slice (one 16-byte LDS read each).
//   The result block D[vocab i][token j] leaves lane l with token j = l % 32 and the 16 vocabulary rows
//   i = 8 * (r / 4) + 4 * (l / 32) + r % 4, r = 0..15: the reduction over the vocabulary is lane-local but
//   for one exchange between the two half waves.
#include "common.h"
#include "score_device.h"

namespace sirllm {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

constexpr int BV = 256;                       // vocabulary rows per workgroup tile
constexpr int BT = 256;                       // token rows per workgroup tile
constexpr int BK = 64;                        // K elements per pipeline stage (128 bytes per row)
constexpr int kRowBytes = BK * 2;
constexpr int kTileBytes = BV * kRowBytes;    // 32 KB; the token tile has the same size (BT == BV)
constexpr int kStageBytes = 2 * kTileBytes;   // W tile, then h tile
constexpr int kRedFloats = 2 * BT * 3;        // (m, s, z_tok) of both vocabulary halves
constexpr int kLdsBytes = 2 * kStageBytes + kRedFloats * 4;

template <int DT>
__device__ __forceinline__ f32x16 mfma(u32x4 a, u32x4 b, f32x16 c)
{
    if constexpr (DT == SIRLLM_BF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// Byte offset of 16-byte chunk `c` (0..7) of tile row `r` inside a tile.  The LDS has 64 banks of 4 bytes and
// serves a 16-byte-per-lane read 16 lanes at a time, so the 16 rows a quarter wave reads from one chunk column
// must land in 16 different 16-byte slots of the 256-byte bank line: rows are 128 bytes (two per bank line), and
// the chunk index is XOR-ed with bits 1..3 of the row.
__device__ __forceinline__ int tile_offset(int r, int c) { return r * kRowBytes + ((c ^ ((r >> 1) & 7)) << 4); }

// Tile coordinates of a workgroup.  Workgroups are dealt to the 8 XCDs round robin; an XCD takes every 8th
// vocabulary tile and walks all token tiles of it back to back, so a weight tile is fetched into one L2 only
// and the (small) hidden-state matrix is what the XCDs share.
__device__ __forceinline__ bool tile_of_block(const LmHeadArgs& a, int& vt, int& tt)
{
    const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
    tt = q % a.n_ttiles;
    vt = (q / a.n_ttiles) * 8 + xcd;
    return vt < a.n_vtiles;
}

// Reduces the wave's 128 x 128 block of logits to per-token softmax statistics, merges the two vocabulary
// halves through LDS and writes one (m, s, z_tok) triple per token of the tile.
__device__ __forceinline__ void tile_epilogue(const LmHeadArgs& a, f32x16 (&acc)[4][4], float* red, int vt, int v0,
                                              int64_t t0, int wv, int wt, int lane, int tid)
{
    const int frag_row = lane & 31, khalf = lane >> 5;
#pragma unroll
    for (int tb = 0; tb < 4; ++tb) {
        const int T = wt * 128 + tb * 32 + frag_row;
        const int64_t row = t0 + T;
        int32_t tok = (row < a.n_rows) ? a.token_ids[row] : -1;
        if (tok >= a.vocab) tok = -1;
        float z[64];
        float zt = __uint_as_float(0x7fc00000u);
#pragma unroll
        for (int vb = 0; vb < 4; ++vb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int v = v0 + wv * 128 + vb * 32 + 8 * (r >> 2) + 4 * khalf + (r & 3);
                float x = acc[vb][tb][r];
                if (v >= a.vocab) x = -INFINITY;
                if (v == tok) zt = x;
                z[vb * 16 + r] = x;
            }
        score_dev::MS ms = {-INFINITY, 0.0f};
        score_dev::accumulate<64>(z, ms);
        const score_dev::MS o = {__shfl_xor(ms.m, 32, kWave), __shfl_xor(ms.s, 32, kWave)};
        ms = score_dev::merge(ms, o);
        const float zo = __shfl_xor(zt, 32, kWave);
        if (zt != zt) zt = zo;
        if (khalf == 0) {
            float* p = red + (wv * BT + T) * 3;
            p[0] = ms.m;
            p[1] = ms.s;
            p[2] = zt;
        }
    }
    __syncthreads();
    const int64_t row = t0 + tid;
    if (row < a.n_rows) {
        const float* p0 = red + tid * 3;
        const float* p1 = red + (BT + tid) * 3;
        const score_dev::MS ms = score_dev::merge(score_dev::MS{p0[0], p0[1]}, score_dev::MS{p1[0], p1[1]});
        const float zt = (p0[2] == p0[2]) ? p0[2] : p1[2];
        float* out = a.partial + (int64_t)vt * a.part_stride + 3 * row;
        out[0] = ms.m;
        out[1] = ms.s;
        out[2] = zt;
    }
}

// General kernel (any d_model that is a multiple of 8): tiles staged global -> registers -> LDS, two LDS
// buffers, the compiler's own schedule.
template <int DT>
__global__ __launch_bounds__(256) void lmhead_score_general_kernel(LmHeadArgs a)
{
    extern __shared__ __align__(16) char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wv = wave & 1, wt = wave >> 1;          // which 128 vocabulary rows / 128 tokens this wave owns

    int vt, tt;
    if (!tile_of_block(a, vt, tt)) return;
    const int v0 = vt * BV;
    const int64_t t0 = (int64_t)tt * BT;

    // ---- global -> register -> LDS staging: thread owns chunk c of rows r_in + 32 i, i = 0..7, of both tiles
    const int c = tid & 7, r_in = tid >> 3;
    const char* wbase = (const char*)a.weight + (int64_t)v0 * a.ld_w * 2 + c * 16;
    const char* hbase = (const char*)a.hidden + t0 * a.ld_h * 2 + c * 16;
    int off_w[8], off_h[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int rw = r_in + 32 * i, rh = rw;
        if (v0 + rw >= a.vocab) rw = a.vocab - 1 - v0;                   // rows past the end re-read the last row
        if (t0 + rh >= a.n_rows) rh = (int)(a.n_rows - 1 - t0);
        off_w[i] = rw * (int)a.ld_w * 2;
        off_h[i] = rh * (int)a.ld_h * 2;
    }
    const int st_off = tile_offset(r_in, c);          // + i * 32 rows * 128 bytes

    u32x4 gw[8], gh[8];
    auto load_global = [&](int k0) {
        const bool in = k0 + c * 8 < a.d_model;       // d_model is a multiple of 8: a chunk is all in or all out
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const u32x4 zero = {0u, 0u, 0u, 0u};
            gw[i] = in ? *(const u32x4*)(wbase + off_w[i] + k0 * 2) : zero;
            gh[i] = in ? *(const u32x4*)(hbase + off_h[i] + k0 * 2) : zero;
        }
    };
    auto store_lds = [&](int buf) {
        char* s = lds + buf * kStageBytes + st_off;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            *(u32x4*)(s + i * 32 * kRowBytes) = gw[i];
            *(u32x4*)(s + kTileBytes + i * 32 * kRowBytes) = gh[i];
        }
    };

    // ---- fragment addresses: row = 128 * (wave half) + 32 * block + lane % 32, chunk = 2 kk + lane / 32
    const int frag_row = lane & 31, khalf = lane >> 5;
    const int a_base = (wv * 128 + frag_row) * kRowBytes;
    const int b_base = kTileBytes + (wt * 128 + frag_row) * kRowBytes;
    int cpos[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) cpos[kk] = ((2 * kk + khalf) ^ ((frag_row >> 1) & 7)) << 4;

    f32x16 acc[4][4];
#pragma unroll
    for (int vb = 0; vb < 4; ++vb)
#pragma unroll
        for (int tb = 0; tb < 4; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[vb][tb][r] = 0.0f;

    const int nk = (a.d_model + BK - 1) / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int ks = 0; ks < nk; ++ks) {
        if (ks + 1 < nk) load_global((ks + 1) * BK);
        const char* s = lds + (ks & 1) * kStageBytes;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            u32x4 af[4], bf[4];
#pragma unroll
            for (int vb = 0; vb < 4; ++vb) af[vb] = *(const u32x4*)(s + a_base + vb * 32 * kRowBytes + cpos[kk]);
#pragma unroll
            for (int tb = 0; tb < 4; ++tb) bf[tb] = *(const u32x4*)(s + b_base + tb * 32 * kRowBytes + cpos[kk]);
#pragma unroll
            for (int vb = 0; vb < 4; ++vb)
#pragma unroll
                for (int tb = 0; tb < 4; ++tb) acc[vb][tb] = mfma<DT>(af[vb], bf[tb], acc[vb][tb]);
        }
        if (ks + 1 < nk) store_lds((ks + 1) & 1);
        __syncthreads();
    }

    tile_epilogue(a, acc, (float*)(lds + 2 * kStageBytes), vt, v0, t0, wv, wt, lane, tid);
}

// 16 bytes per lane straight from global memory into LDS (global_load_lds_dwordx4): lane l's chunk lands at
// lds_block + 16 l, so one wave instruction fills 1 KB = 8 tile rows.  lds_block must be wave uniform.
__device__ __forceinline__ void load_to_lds(const char* g, char* lds_block)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                     (__attribute__((address_space(3))) void*)lds_block, 16, 0, 0);
}

// Fast kernel (d_model a multiple of 32): tiles go from global memory straight into LDS, no staging
// registers, through a ring of five 32 KB buffers (stage = 32 K elements of both tiles; buffer = stage % 5;
// all 160 KB of the LDS).  One stage is two 16-wide slices = 32 MFMAs per wave:
//   slice 0: MFMAs under the LDS reads of slice 1 and under 4 of this wave's 8 loads of stage ks + 4
//   wait until this wave's loads of stage ks + 1 have landed (the 24 younger ones may stay in flight), barrier:
//   every wave has finished reading stage ks, so its buffer is free for stage ks + 5
//   slice 1: MFMAs under the LDS reads of slice 0 of stage ks + 1 and under the first 4 loads of stage ks + 5.
// What bounds this kernel is the L2 -> LDS path: a CU gets bandwidth in proportion to the bytes it keeps in
// flight (measured: ~46 GB/s per CU with 128 KB in flight), so the ring is as deep as the LDS allows (up to
// 3.5 stages = 112 KB in flight) and loads are issued one per four MFMAs rather than in bursts.
constexpr int FK = 32;
constexpr int kFastRow = FK * 2;                       // 64 bytes per tile row
constexpr int kFastTile = BV * kFastRow;               // 16 KB
constexpr int kFastStage = 2 * kFastTile;              // 32 KB
constexpr int kRing = 5;
constexpr int kFastLds = kRing * kFastStage;      // the epilogue's scratch reuses the ring

// wait for all but the n youngest vector-memory operations and for every LDS operation, then barrier
#define SIRLLM_WAIT_BARRIER(n) asm volatile("s_waitcnt vmcnt(" #n ") lgkmcnt(0)\n\ts_barrier" ::: "memory")

template <int DT>
__global__ __launch_bounds__(256) void lmhead_score_kernel(LmHeadArgs a)
{
    extern __shared__ __align__(16) char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wv = wave & 1, wt = wave >> 1;
    int vt, tt;
    if (!tile_of_block(a, vt, tt)) return;
    const int v0 = vt * BV;
    const int64_t t0 = (int64_t)tt * BT;

    // ---- loads: a stage is 32 blocks of 1 KB (16 rows x 64 B): blocks 0..15 the W tile, 16..31 the h tile.
    // Wave w issues blocks 8 w + j, j = 0..7 (waves 0, 1: W; waves 2, 3: h).  Within a block lane l fills
    // row l / 4, chunk position l % 4, which holds chunk (l % 4) ^ ((row / 4) % 4) of that row: rows are 64
    // bytes, four to a 256-byte bank line, and the 16 rows a quarter wave reads from one chunk column land in
    // 16 different 16-byte slots.
    const bool is_w = wave < 2;
    const int ld2 = (int)(is_w ? a.ld_w : a.ld_h) * 2;
    const int rows_left = is_w ? a.vocab - v0 : (int)((a.n_rows - t0 < BT) ? a.n_rows - t0 : BT);
    const char* gbase = is_w ? (const char*)a.weight + (int64_t)v0 * a.ld_w * 2
                             : (const char*)a.hidden + t0 * a.ld_h * 2;
    gbase += (((lane & 3) ^ ((lane >> 4) & 3)) << 4);
    int goff[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        int r = ((wave & 1) * 8 + j) * 16 + (lane >> 2);
        if (r >= rows_left) r = rows_left - 1;                            // rows past the end re-read the last row
        goff[j] = r * ld2;
    }
    char* const my_blocks = lds + wave * 8 * 1024;
    const int nk = a.d_model / FK;             // >= 1
    // ---- fragments: row = 128 * (wave half) + 32 * block + lane % 32, chunk = 2 kk + lane / 32
    const int frag_row = lane & 31, khalf = lane >> 5;
    const int a_base = (wv * 128 + frag_row) * kFastRow;
    const int b_base = kFastTile + (wt * 128 + frag_row) * kFastRow;
    int cpos[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) cpos[kk] = ((2 * kk + khalf) ^ ((frag_row >> 2) & 3)) << 4;

    f32x16 acc[4][4];
#pragma unroll
    for (int vb = 0; vb < 4; ++vb)
#pragma unroll
        for (int tb = 0; tb < 4; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[vb][tb][r] = 0.0f;

    u32x4 af[2][4], bf[2][4];
    // fragment i of slice kk: i = 0..3 the W blocks, 4..7 the h blocks
    auto read_frag = [&](const char* s, int kk, int set, int i) {
        if (i < 4) af[set][i] = *(const u32x4*)(s + a_base + i * 32 * kFastRow + cpos[kk]);
        else bf[set][i - 4] = *(const u32x4*)(s + b_base + (i - 4) * 32 * kFastRow + cpos[kk]);
    };
    auto load_frags = [&](const char* s, int kk, int set) {
#pragma unroll
        for (int i = 0; i < 8; ++i) read_frag(s, kk, set, i);
    };
    // load j of stage ks into ring buffer `buf` (a stage past the end re-reads the last one into a buffer
    // nobody reads)
    auto issue_load = [&](int ks, int buf, int j) {
        const char* g = gbase + (int64_t)(ks < nk ? ks : nk - 1) * (FK * 2);
        load_to_lds(g + goff[j], my_blocks + buf * kFastStage + j * 1024);
    };
    // One slice: 16 MFMAs on fragment set `use`, and in their shadow the 8 LDS reads of the next slice (into
    // the other set) and 4 loads, at most one of them behind each MFMA.  The order is pinned: a matrix
    // instruction keeps its pipe busy for 32 cycles, one LDS read or one load issues within that time, and
    // loads that arrive at the memory pipeline one at a time do not stall the wave that issues them (a burst of
    // four costs ~120 cycles, sixteen ~900).
    auto slice = [&](int use, const char* rs, int rkk, int ls, int lbuf, int lj0) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc[g][i] = mfma<DT>(af[use][g], bf[use][i], acc[g][i]);
                __builtin_amdgcn_sched_barrier(0);
                if (i < 2) read_frag(rs, rkk, use ^ 1, 2 * g + i);
                else if (i == 2) issue_load(ls, lbuf, lj0 + g);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    for (int st = 0; st < 4; ++st)
#pragma unroll
        for (int j = 0; j < 8; ++j) issue_load(st, st, j);
#pragma unroll
    for (int j = 0; j < 4; ++j) issue_load(4, 4, j);
    SIRLLM_WAIT_BARRIER(28);                   // stage 0 landed (stages 1..3 and half of 4 may be in flight)
    load_frags(lds, 0, 0);
    int bcur = 0;                              // ks % kRing
    for (int ks = 0; ks < nk; ++ks) {
        const int bnext = bcur == kRing - 1 ? 0 : bcur + 1;
        const int blast = bcur == 0 ? kRing - 1 : bcur - 1;            // (ks + 4) % kRing
        const char* cur = lds + bcur * kFastStage;
        const char* nxt = lds + bnext * kFastStage;
        slice(0, cur, 1, ks + 4, blast, 4);
        SIRLLM_WAIT_BARRIER(24);               // stage ks + 1 landed; all reads of stage ks done
        slice(1, nxt, 0, ks + 5, bcur, 0);
        bcur = bnext;
    }
    SIRLLM_WAIT_BARRIER(0);                    // no load may still be landing when the LDS is reused
    tile_epilogue(a, acc, (float*)lds, vt, v0, t0, wv, wt, lane, tid);
}

// Folds the n_parts triples of every row: 16 rows per workgroup, 16 lanes per row striding over the parts.
// Row `row` belongs to stream row / rows_per_stream and is its token t = row % rows_per_stream; the score goes
// to out[stream * out_stride + t].
__global__ __launch_bounds__(256) void lmhead_merge_kernel(const float* partials, int n_parts, int64_t part_stride,
                                                           int64_t n_rows, float* out, int64_t rows_per_stream,
                                                           int64_t out_stride)
{
    __shared__ float sm[16][16][3];
    const int r = threadIdx.x & 15, pl = threadIdx.x >> 4;
    const int64_t row = (int64_t)blockIdx.x * 16 + r;
    score_dev::MS acc = {-INFINITY, 0.0f};
    float zt = __uint_as_float(0x7fc00000u);
    if (row < n_rows) {
        for (int p = pl; p < n_parts; p += 16) {
            const float* t = partials + p * part_stride + 3 * row;
            acc = score_dev::merge(acc, score_dev::MS{t[0], t[1]});
            const float z = t[2];
            if (zt != zt && z == z) zt = z;
        }
    }
    sm[pl][r][0] = acc.m;
    sm[pl][r][1] = acc.s;
    sm[pl][r][2] = zt;
    __syncthreads();
    if (pl == 0 && row < n_rows) {
#pragma unroll
        for (int i = 1; i < 16; ++i) {
            acc = score_dev::merge(acc, score_dev::MS{sm[i][r][0], sm[i][r][1]});
            const float z = sm[i][r][2];
            if (zt != zt && z == z) zt = z;
        }
        const int64_t stream = row / rows_per_stream;
        out[stream * out_stride + (row - stream * rows_per_stream)] = (acc.m - zt) + logf(acc.s);
    }
}

}  // namespace

int lmhead_tiles_vocab(int32_t vocab) { return (vocab + BV - 1) / BV; }

hipError_t launch_lmhead_score(const LmHeadArgs& args, sirllm_dtype dt, float* out, int64_t rows_per_stream,
                               int64_t out_stride, hipStream_t stream)
{
    if (args.n_rows <= 0) return hipSuccess;
    LmHeadArgs a = args;
    a.n_vtiles = lmhead_tiles_vocab(a.vocab);
    a.n_ttiles = (int)((a.n_rows + BT - 1) / BT);
    const int64_t groups = (int64_t)((a.n_vtiles + 7) / 8) * a.n_ttiles * 8;
    if (groups > 0x7fffffff) return hipErrorInvalidValue;
    const bool fast = a.d_model % FK == 0;
    typedef void (*kernel_t)(LmHeadArgs);
    const kernel_t fn = fast ? (dt == SIRLLM_BF16 ? lmhead_score_kernel<SIRLLM_BF16> : lmhead_score_kernel<SIRLLM_F16>)
                             : (dt == SIRLLM_BF16 ? lmhead_score_general_kernel<SIRLLM_BF16>
                                                  : lmhead_score_general_kernel<SIRLLM_F16>);
    const int lds_bytes = fast ? kFastLds : kLdsBytes;
    hipError_t e = hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(fn, dim3((unsigned)groups), dim3(256), lds_bytes, stream, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(lmhead_merge_kernel, dim3((unsigned)((a.n_rows + 15) / 16)), dim3(256), 0, stream,
                       a.partial, a.n_vtiles, a.part_stride, a.n_rows, out, rows_per_stream > 0 ? rows_per_stream : 1, out_stride);
    return hipGetLastError();
}

}  // namespace sirllm
