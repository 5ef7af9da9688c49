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
#include <atomic>

#include "common.h"
#include "score_device.h"
#include "tuning.h"

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
// vocabulary tile, so a weight tile is fetched into one L2 only.  Token tiles come in groups of at most kTokenGroup:
// an XCD walks, group after group, all its vocabulary tiles and for each the token tiles of the group back to back.
// The 32 workgroups it runs at a time are then 4 vocabulary tiles x 8 token tiles, whose 12 operand tiles per stage
// fit its 4 MB L2 with a ring's worth of stages to spare; without the grouping 32 token tiles of one vocabulary tile
// would be in flight (33 operand tiles per stage, and every generation of workgroups pulls in all of h again).
constexpr int kTokenGroup = 8;
__host__ __device__ __forceinline__ int token_group(int n_ttiles) { return n_ttiles < kTokenGroup ? n_ttiles : kTokenGroup; }
// workgroups per XCD and token group
__host__ __device__ __forceinline__ int tiles_per_group(const LmHeadArgs& a) { return ((a.n_vtiles + 7) / 8) * token_group(a.n_ttiles); }

// q-th workgroup of XCD `xcd` -> tile; false when it falls off the ragged end of either axis
__device__ __forceinline__ bool tile_of(const LmHeadArgs& a, int q, int xcd, int& vt, int& tt)
{
    const int tg = token_group(a.n_ttiles), per = tiles_per_group(a);
    const int grp = q / per, r = q - grp * per;
    vt = (r / tg) * 8 + xcd;
    tt = grp * tg + r % tg;
    return vt < a.n_vtiles && tt < a.n_ttiles;
}

__device__ __forceinline__ bool tile_of_block(const LmHeadArgs& a, int& vt, int& tt)
{
    return tile_of(a, (int)(blockIdx.x >> 3), (int)(blockIdx.x & 7), vt, tt);
}

// Workgroups of a launch: 8 XCDs x token groups x (vocabulary tiles per XCD x token tiles per group).
inline int64_t lmhead_grid(const LmHeadArgs& a)
{
    const int tg = token_group(a.n_ttiles);
    return (int64_t)8 * ((a.n_ttiles + tg - 1) / tg) * tiles_per_group(a);
}

// Reduces a wave's (32 NVB) x (32 NTB) block of logits (vocabulary x tokens) to per-token softmax statistics,
// merges the two vocabulary halves of the tile through LDS and writes one (m, s, z_tok) triple per token of the tile.
template <int NVB, int NTB>
__device__ __forceinline__ void tile_epilogue(const LmHeadArgs& a, f32x16 (&acc)[NVB][NTB], float* red, int vt, int v0,
                                              int64_t t0, int wv, int wt, int lane, int tid)
{
    constexpr int TILE_T = 64 * NTB;
    const int frag_row = lane & 31, khalf = lane >> 5;
    const int v_wave = v0 + wv * (32 * NVB);           // first vocabulary row of this wave's blocks
    // Only the last vocabulary tile can hold rows past the end of the vocabulary: they are set to -inf in place, in
    // a pass of their own that every other tile jumps over (wave-uniform).
    if (v_wave + 32 * NVB > a.vocab) {
#pragma unroll
        for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int v = v_wave + vb * 32 + 8 * (r >> 2) + 4 * khalf + (r & 3);
                if (v >= a.vocab) {
#pragma unroll
                    for (int tb = 0; tb < NTB; ++tb) acc[vb][tb][r] = -INFINITY;
                }
            }
    }
#pragma unroll
    for (int tb = 0; tb < NTB; ++tb) {
        const int T = wt * (32 * NTB) + tb * 32 + frag_row;
        const int64_t row = t0 + T;
        int32_t tok = (row < a.n_rows) ? a.token_ids[row] : -1;
        if (tok >= a.vocab) tok = -1;
        // The token's logit: lane l holds vocabulary rows v_wave + 32 vb + 8 (r / 4) + 4 (l / 32) + r % 4, so the token
        // sits in this lane iff d = tok - v_wave is in [0, 32 NVB) and bit 2 of d is l / 32.  Few waves hold any of their
        // 32 tokens' logits in a given tile; the others skip the search (wave-uniform).
        const int d = tok - v_wave;
        const bool mine = tok >= 0 && d >= 0 && d < 32 * NVB && ((d >> 2) & 1) == khalf;
        float zt = __uint_as_float(0x7fc00000u);
        if (__builtin_amdgcn_ballot_w64(mine) != 0ull) {
            const int e = mine ? (d >> 5) * 16 + ((d >> 3) & 3) * 4 + (d & 3) : -1;
#pragma unroll
            for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (e == vb * 16 + r) zt = acc[vb][tb][r];
        }
        float z[16 * NVB];
#pragma unroll
        for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
            for (int r = 0; r < 16; ++r) z[vb * 16 + r] = acc[vb][tb][r];
        score_dev::MS ms = {-INFINITY, 0.0f};
        score_dev::accumulate<16 * NVB>(z, ms);
        const score_dev::MS o = {__shfl_xor(ms.m, 32, kWave), __shfl_xor(ms.s, 32, kWave)};
        ms = score_dev::merge(ms, o);
        const float zo = __shfl_xor(zt, 32, kWave);
        if (zt != zt) zt = zo;
        if (khalf == 0) {
            float* p = red + (wv * TILE_T + T) * 3;
            p[0] = ms.m;
            p[1] = ms.s;
            p[2] = zt;
        }
    }
    __syncthreads();
    const int64_t row = t0 + tid;
    if (tid < TILE_T && row < a.n_rows) {
        const float* p0 = red + tid * 3;
        const float* p1 = red + (TILE_T + tid) * 3;
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

    tile_epilogue<4, 4>(a, acc, (float*)(lds + 2 * kStageBytes), vt, v0, t0, wv, wt, lane, tid);
}

// 16 bytes per lane straight from global memory into LDS (global_load_lds_dwordx4): lane l's chunk lands at
// lds_block + 16 l, so one wave instruction fills 1 KB = 8 tile rows.  lds_block must be wave uniform.
// NT: with the non-temporal hint (bytes that are read exactly once).
template <bool NT = false>
__device__ __forceinline__ void load_to_lds(const char* g, char* lds_block)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                     (__attribute__((address_space(3))) void*)lds_block, 16, 0, NT ? 2 : 0);
}

// Fast kernel (d_model a multiple of 32).  The workgroup is 2 x 2 waves; a wave owns NVB x NTB result blocks of
// 32 x 32, so the tile is (64 NVB) vocabulary rows x (64 NTB) tokens:
//   NVB = NTB = 4   256 x 256, 256 accumulator registers per lane, one workgroup per CU: MFMA bound
//   NVB = 2, NTB = 4   128 x 256 for 129 to 256 rows against a vocabulary below 65536 rows
//   NVB = NTB = 2   128 x 128 for 65 to 128 rows (NVB = 4: 256 x 128 against a vocabulary of 65536 rows or more, there
//                   also for 257 to 384 rows)
//   NVB = 2, NTB = 1   128 x 64 for up to 64 rows (a turn of a dialogue): bound by streaming W from HBM
// Tiles go from global memory straight into LDS, no staging registers, through a ring of RING buffers (stage =
// 32 K elements of both tiles; buffer = stage % RING).  One stage is two 16-wide slices:
//   slice 0: MFMAs under the LDS reads of slice 1
//   wait until this wave's loads of stage ks + 1 have landed (the younger ones stay in flight), barrier: every
//   wave has finished reading stage ks, so its buffer is free for stage ks + RING
//   slice 1: MFMAs under the LDS reads of slice 0 of stage ks + 1 and under this wave's loads of stage ks + RING.
// The tiles for up to 128 rows take stages of 64 K elements instead when d_model allows (FKE = 64: tile rows of 128
// bytes, four slices, three of them in front of the barrier): a wave load then fetches whole 128-byte lines.
constexpr int FK = 32;

// Wait until at most N vector-memory operations of this wave are outstanding and every LDS operation is done, then
// barrier.  What the callers rely on, and what an edit must keep:
//  * vmcnt counts every vector-memory instruction of the wave (tile loads into LDS, the warm-up touches, stores) and
//    loads complete in issue order, so "at most N outstanding" means "everything but the N youngest has landed".
//  * N is therefore the number of vector-memory instructions the wave has issued AFTER the last load of the stage
//    it is about to read.  Every wave issues exactly kLpw tile loads per stage, unconditionally (rows past the end
//    of a tile load a clamped address), so that number is a compile-time constant.
//  * An extra instruction issued in between (the warm-up touch is one) makes the wait stricter by one, never
//    weaker: it is always safe to add one.  Dropping a load, or making one conditional per wave, is not: the
//    constant would then let a needed load count among the "youngest N" while still in flight.
//  * The barrier sits behind the wait, so a wave passes it only after its own share of the stage has landed, and
//    all waves have passed it before any reads the stage.
template <int N>
__device__ __forceinline__ void wait_barrier()
{
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

// FKE: K elements per stage, 32 or 64 (tile rows of 64 or 128 bytes).
template <int NVB, int NTB, int RING, int FKE = FK>
struct FastCfg {
    static_assert(FKE == 32 || FKE == 64, "tile rows of 64 or 128 bytes");
    static constexpr int kBV = 64 * NVB, kBT = 64 * NTB;
    static constexpr int kRow = FKE * 2;                           // bytes of a tile row
    static constexpr int kChunks = kRow / 16;                      // 16-byte chunks per row
    static constexpr int kRowsPerLine = 256 / kRow;                // rows per 256-byte bank line
    static constexpr int kRowsPerBlock = 1024 / kRow;              // rows one wave load fills
    static constexpr int kSlices = FKE / 16;                       // 16-wide MFMA slices per stage
    static constexpr int kTileW = kBV * kRow;                      // bytes of the W tile of one stage
    static constexpr int kStage = (kBV + kBT) * kRow;
    static constexpr int kLpw = (NVB + NTB) * kRow / 64;           // 1 KB loads per wave and stage
    static constexpr int kDump = 256;                              // where the L2 warm-up loads drop their bytes
    static constexpr int kLds = RING * kStage + kDump;             // the epilogue's scratch reuses the ring
    static_assert((RING - 1) * kLpw <= 63, "vmcnt is a 6-bit counter");
    static_assert(RING * kStage >= 2 * kBT * 3 * 4 && kLds <= 160 * 1024, "LDS budget");
};

template <int DT, int NVB, int NTB, int RING, bool PIN, bool WARM, int FKE = FK, bool WNT = false>
__global__ __launch_bounds__(256) void lmhead_score_kernel(LmHeadArgs a)
{
    using Cfg = FastCfg<NVB, NTB, RING, FKE>;
    static_assert(FKE == FK || (!PIN && !WARM), "the pinned schedule and the L2 touches are written for 64-byte tile rows");
    extern __shared__ __align__(16) char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wv = wave & 1, wt = wave >> 1;
    int vt, tt;
    if (!tile_of_block(a, vt, tt)) return;
    const int v0 = vt * Cfg::kBV;
    const int64_t t0 = (int64_t)tt * Cfg::kBT;

    // ---- loads: a stage is 4 kLpw blocks of 1 KB (16 rows x 64 B, or 8 rows x 128 B): first the W tile, then the h
    // tile.  Wave w issues blocks kLpw w + j.  With 64-byte rows lane l of a block fills row l / 4, chunk position
    // l % 4, which holds chunk (l % 4) ^ ((row / 4) % 4) of that row: four rows share a 256-byte bank line, and the 16
    // rows a quarter wave reads from one chunk column land in 16 different 16-byte slots (the LDS has 64 banks
    // and serves a 16-byte-per-lane read 16 lanes at a time).  With 128-byte rows (two to a bank line) it is row l / 8,
    // position l % 8, chunk (l % 8) ^ ((row / 2) % 8): again 16 different slots.  Then one wave load takes whole
    // 128-byte lines of W, which streams from HBM 20 % faster than half lines in two loads.
    const int rows_w = a.vocab - v0;
    const int rows_h = (int)((a.n_rows - t0 < Cfg::kBT) ? a.n_rows - t0 : Cfg::kBT);
    // A load address is a wave-uniform base (tile origin + stage offset, scalar registers) plus a 32-bit per-lane
    // offset (row * pitch + chunk): no vector arithmetic per load.
    constexpr int kWBlocks = Cfg::kBV / Cfg::kRowsPerBlock;               // blocks of the W tile
    const char* ubase[Cfg::kLpw];
    uint32_t goff[Cfg::kLpw];
#pragma unroll
    for (int j = 0; j < Cfg::kLpw; ++j) {
        const int blk = __builtin_amdgcn_readfirstlane(wave) * Cfg::kLpw + j;
        const bool is_w = blk < kWBlocks;
        const int tr = (is_w ? blk : blk - kWBlocks) * Cfg::kRowsPerBlock + lane / Cfg::kChunks;   // row of its tile
        const uint32_t lane_chunk = (uint32_t)(((lane % Cfg::kChunks) ^ ((tr / Cfg::kRowsPerLine) % Cfg::kChunks)) << 4);
        const int rows_left = is_w ? rows_w : rows_h;
        const int r = tr < rows_left ? tr : rows_left - 1;                // rows past the end re-read the last row
        ubase[j] = is_w ? (const char*)a.weight + (int64_t)v0 * a.ld_w * 2 : (const char*)a.hidden + t0 * a.ld_h * 2;
        goff[j] = (uint32_t)r * (uint32_t)((is_w ? a.ld_w : a.ld_h) * 2) + lane_chunk;
    }
    char* const my_blocks = lds + __builtin_amdgcn_readfirstlane(wave) * Cfg::kLpw * 1024;
    const int nk = a.d_model / FKE;            // >= 1
    // Workgroups start their walk over K at different stages (and wrap around): at any moment the chip then
    // reads many different column stripes of W instead of one 64-byte-wide stripe with a row pitch of d_model
    // elements, which would land on few memory channels.  A dot product does not care where its sum starts.
    // Only with a single token tile: otherwise the workgroups that share a W tile (or an h tile) must walk in
    // step, or they stop finding each other's lines in the L2.
    const int kstart = a.n_ttiles == 1 ? (int)(((unsigned)vt * 37u) % (unsigned)nk) : 0;
    // load j of stage ks into ring buffer `buf` (a stage past the end re-reads the last one into a buffer
    // nobody reads)
    auto issue_load = [&](int ks, int buf, int j) {
        int st = (ks < nk ? ks : nk - 1) + kstart;
        if (st >= nk) st -= nk;
        const char* g = ubase[j] + (int64_t)st * Cfg::kRow + goff[j];
        char* l = my_blocks + buf * Cfg::kStage + j * 1024;
        // blocks below kWBlocks belong to W: read exactly once when there is a single token tile
        if (WNT && __builtin_amdgcn_readfirstlane(wave) * Cfg::kLpw + j < kWBlocks) load_to_lds<true>(g, l);
        else load_to_lds<false>(g, l);
    };

    // ---- fragments: row = 32 NVB (or NTB) * (wave half) + 32 * block + lane % 32, chunk = 2 kk + lane / 32
    const int frag_row = lane & 31, khalf = lane >> 5;
    const int a_base = (wv * (32 * NVB) + frag_row) * Cfg::kRow;
    const int b_base = Cfg::kTileW + (wt * (32 * NTB) + frag_row) * Cfg::kRow;
    int cpos[Cfg::kSlices];
#pragma unroll
    for (int kk = 0; kk < Cfg::kSlices; ++kk)
        cpos[kk] = ((2 * kk + khalf) ^ ((frag_row / Cfg::kRowsPerLine) % Cfg::kChunks)) << 4;

    f32x16 acc[NVB][NTB];
#pragma unroll
    for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
        for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[vb][tb][r] = 0.0f;

    u32x4 af[2][NVB], bf[2][NTB];
    // fragment i of slice kk: i < NVB the W blocks, then the h blocks
    auto read_frag = [&](const char* s, int kk, int set, int i) {
        if (i < NVB) af[set][i] = *(const u32x4*)(s + a_base + i * 32 * Cfg::kRow + cpos[kk]);
        else bf[set][i - NVB] = *(const u32x4*)(s + b_base + (i - NVB) * 32 * Cfg::kRow + cpos[kk]);
    };
    // One slice: NVB x NTB MFMAs on fragment set `use`, and in their shadow the LDS reads of the next slice
    // (into the other set) and, in slice 1, the loads of a later stage.  With PIN the order is fixed: behind each
    // MFMA at most one read or one load (a matrix instruction keeps its pipe busy for 32 cycles, and one read or
    // load issues within that time); otherwise the compiler orders them (small tiles are not MFMA bound).
    auto slice = [&](int use, const char* rs, int rkk, int ls, int lbuf, int lj0, int ln) {
        if constexpr (PIN) {
            // reads and loads one per MFMA, a load behind every fourth MFMA: the four waves run in step, and four 1 KB
            // loads in a row from each of them would queue up in the CU's one address unit faster than it drains
            int ri = 0, li = 0;
#pragma unroll
            for (int g = 0; g < NVB; ++g)
#pragma unroll
                for (int i = 0; i < NTB; ++i) {
                    const int e = g * NTB + i;
                    acc[g][i] = mfma<DT>(af[use][g], bf[use][i], acc[g][i]);
                    __builtin_amdgcn_sched_barrier(0);
                    if ((e & 3) == 1 && li < ln) { issue_load(ls, lbuf, lj0 + li); ++li; }
                    else if (ri < NVB + NTB) { read_frag(rs, rkk, use ^ 1, ri); ++ri; }
                    else if (li < ln) { issue_load(ls, lbuf, lj0 + li); ++li; }
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
            for (; ri < NVB + NTB; ++ri) read_frag(rs, rkk, use ^ 1, ri);
#pragma unroll
            for (; li < Cfg::kLpw; ++li)
                if (li < ln) issue_load(ls, lbuf, lj0 + li);
            return;
        }
        int extra = 0;                                     // reads, then loads, one behind each MFMA; the compiler reorders
#pragma unroll
        for (int g = 0; g < NVB; ++g)
#pragma unroll
            for (int i = 0; i < NTB; ++i) {
                acc[g][i] = mfma<DT>(af[use][g], bf[use][i], acc[g][i]);
                if (extra < NVB + NTB) read_frag(rs, rkk, use ^ 1, extra);
                else if (extra - (NVB + NTB) < ln) issue_load(ls, lbuf, lj0 + extra - (NVB + NTB));
                ++extra;
            }
        // what did not fit behind an MFMA (tiles with fewer MFMAs than reads + loads)
#pragma unroll
        for (int e = NVB * NTB; e < NVB + NTB + Cfg::kLpw; ++e) {
            if (e < NVB + NTB) read_frag(rs, rkk, use ^ 1, e);
            else if (e - (NVB + NTB) < ln) issue_load(ls, lbuf, lj0 + e - (NVB + NTB));
        }
    };

    // PIN tiles split a stage's loads over both slices (second half of stage ks + RING - 1 in slice 0, first half of
    // stage ks + RING in slice 1, so that no slice issues more than one load per two MFMAs); the others issue a
    // whole stage in slice 1.
    constexpr int kHalf = PIN ? Cfg::kLpw / 2 : 0;
    static_assert(!PIN || Cfg::kLpw % 2 == 0, "split loads need an even count");
    for (int st = 0; st < RING - 1; ++st)
#pragma unroll
        for (int j = 0; j < Cfg::kLpw; ++j) issue_load(st, st, j);
#pragma unroll
    for (int j = 0; j < Cfg::kLpw - kHalf; ++j) issue_load(RING - 1, RING - 1, j);
    // issued so far: RING * kLpw - kHalf loads, stage 0's kLpw first: all but the rest may stay in flight
    wait_barrier<(RING - 1) * Cfg::kLpw - kHalf>();        // stage 0 landed (the others may be in flight)
#pragma unroll
    for (int i = 0; i < NVB + NTB; ++i) read_frag(lds, 0, 0, i);
    // ---- L2 warm-up (WARM): the W tile comes from HBM, and the ring's look-ahead (RING - 1 stages, ~2 us) does
    // not cover an HBM access under load.  Every 4 stages one wave touches, with a 4-byte-per-lane load whose data
    // goes to a dump area in LDS (no register, same in-order completion counter as the tile loads), the W lines of
    // stages ks + 12 .. ks + 15: one lane per 128-byte line, 32 rows x 2 lines per instruction.  The `ns`
    // workgroups that share a W tile (same vocabulary tile, consecutive token tiles, resident together on one XCD)
    // split its rows.  Past the end of K the lines of the tile this CU will take next are touched.
    const int swave = __builtin_amdgcn_readfirstlane(wave);
    const int tgs = token_group(a.n_ttiles);   // the workgroups that share a W tile: the token tiles of one group
    const int ns = (tgs & 7) == 0 ? 8 : (tgs & 3) == 0 ? 4 : (tgs & 1) == 0 ? 2 : 1;
    auto warm = [&](int stage) {
        int vt2 = vt, tt2 = tt;
        if (stage >= nk) {
            stage -= nk;
            if (!tile_of(a, (int)(blockIdx.x >> 3) + 32, (int)(blockIdx.x & 7), vt2, tt2) || stage >= nk) return;
        }
        const int rows_per = Cfg::kBV / ns;
        const int rows_left = a.vocab - vt2 * Cfg::kBV;
        int koff = stage * (FK * 2) + (lane & 1) * 128;
        if (koff >= a.d_model * 2) koff = stage * (FK * 2);                  // a row shorter than the 256 bytes touched
        const char* base = (const char*)a.weight + (int64_t)vt2 * Cfg::kBV * a.ld_w * 2 + koff;
        for (int r0 = 0; r0 < rows_per; r0 += 32) {
            int r = (tt2 % ns) * rows_per + r0 + (lane >> 1);
            if (r >= rows_left) r = rows_left - 1;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(base + (int64_t)r * a.ld_w * 2),
                                             (__attribute__((address_space(3))) void*)(lds + RING * Cfg::kStage), 4, 0, 0);
        }
    };

    int bcur = 0;                              // ks % RING
    for (int ks = 0; ks < nk; ++ks) {
        const int bnext = bcur == RING - 1 ? 0 : bcur + 1;
        const int blast = bcur == 0 ? RING - 1 : bcur - 1;             // (ks + RING - 1) % RING
        const char* cur = lds + bcur * Cfg::kStage;
        const char* nxt = lds + bnext * Cfg::kStage;
        if constexpr (Cfg::kSlices == 2) {
            slice(0, cur, 1, ks + RING - 1, blast, Cfg::kLpw - kHalf, kHalf);
        } else {                                           // four slices: three of them in front of the barrier
            slice(0, cur, 1, 0, 0, 0, 0);
            slice(1, cur, 2, 0, 0, 0, 0);
            slice(0, cur, 3, 0, 0, 0, 0);
        }
        // issued after stage ks + 1: stages ks + 2 .. ks + RING - 1 whole = (RING - 2) * kLpw loads (plus, for one
        // wave in four iterations, the touch below: a stricter wait, see wait_barrier)
        wait_barrier<(RING - 2) * Cfg::kLpw>();            // stage ks + 1 landed; all reads of stage ks done
        // (right after a wait: the touch has three stages to come back before a younger load is waited for)
        if (WARM && kstart == 0 && (ks & 3) == 0 && ((ks >> 2) & 3) == swave) warm(ks + 12);
        slice(1, nxt, 0, ks + RING, bcur, 0, Cfg::kLpw - kHalf);
        bcur = bnext;
    }
    wait_barrier<0>();                         // no load may still be landing when the LDS is reused
    tile_epilogue<NVB, NTB>(a, acc, (float*)lds, vt, v0, t0, wv, wt, lane, tid);
}

// Folds the n_parts triples of every row: 4 rows per workgroup, 64 lanes per row striding over the parts (the
// chain of dependent merges is n_parts / 64 long, then a shuffle tree inside each wave and one exchange through LDS).
// Row `row` belongs to stream row / rows_per_stream and is its token t = row % rows_per_stream; the score goes
// to out[stream * out_stride + t].  Ragged batches (rg.cu_rows not null): stream s owns rows
// [cu_rows[s], cu_rows[s+1]) and its token t goes to out[s * out_stride + held_dev[s] + t].
__global__ __launch_bounds__(256) void lmhead_merge_kernel(const float* partials, int n_parts, int64_t part_stride,
                                                           int64_t n_rows, float* out, int64_t rows_per_stream,
                                                           int64_t out_stride, LmHeadRagged rg)
{
    constexpr int R = 4, PL = 256 / R;           // rows per workgroup, part lanes per row
    __shared__ float sm[4][R][3];
    const int r = threadIdx.x & (R - 1), pl = threadIdx.x >> 2;
    const int64_t row = (int64_t)blockIdx.x * R + r;
    score_dev::MS acc = {-INFINITY, 0.0f};
    float zt = __uint_as_float(0x7fc00000u);
    if (row < n_rows) {
        const float* base = partials + 3 * row;
        for (int p0 = pl; p0 < n_parts; p0 += 4 * PL) {
            float t[4][3];
#pragma unroll
            for (int u = 0; u < 4; ++u) {         // the loads of four parts go out together
                const int p = p0 + u * PL;
                const float* q = base + (int64_t)min(p, n_parts - 1) * part_stride;
                t[u][0] = q[0]; t[u][1] = q[1]; t[u][2] = q[2];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (p0 + u * PL < n_parts) {
                    acc = score_dev::merge(acc, score_dev::MS{t[u][0], t[u][1]});
                    if (zt != zt && t[u][2] == t[u][2]) zt = t[u][2];
                }
            }
        }
    }
    // part lanes of one row sit R lanes apart inside a wave (16 of them per wave)
#pragma unroll
    for (int off = R; off < kWave; off <<= 1) {
        const score_dev::MS o = {__shfl_xor(acc.m, off, kWave), __shfl_xor(acc.s, off, kWave)};
        const float z = __shfl_xor(zt, off, kWave);
        acc = score_dev::merge(acc, o);
        if (zt != zt && z == z) zt = z;
    }
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & (kWave - 1)) < R) { sm[wave][r][0] = acc.m; sm[wave][r][1] = acc.s; sm[wave][r][2] = zt; }
    __syncthreads();
    if (threadIdx.x < R && row < n_rows) {
#pragma unroll
        for (int i = 1; i < 4; ++i) {
            acc = score_dev::merge(acc, score_dev::MS{sm[i][r][0], sm[i][r][1]});
            const float z = sm[i][r][2];
            if (zt != zt && z == z) zt = z;
        }
        const float e = (acc.m - zt) + logf(acc.s);
        if (rg.cu_rows) {
            int lo = 0, hi = rg.n_streams;                 // largest s with cu_rows[s] <= row
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if ((int64_t)rg.cu_rows[mid] <= row) lo = mid; else hi = mid;
            }
            const int64_t pos = (int64_t)rg.held_dev[lo] + (row - rg.cu_rows[lo]);
            if (pos >= 0 && pos < out_stride)              // sizes the caller did not promise are dropped, not written
                out[lo * out_stride + pos] = e;
        } else {
            const int64_t stream = row / rows_per_stream;
            out[stream * out_stride + (row - stream * rows_per_stream)] = e;
        }
    }
}

}  // namespace

namespace {

// Tile shape by row count: (vocabulary rows, token rows) of a workgroup tile.
void tile_shape(int64_t n_rows, int32_t vocab, int& bv, int& bt)
{
    // few rows: W is streamed once and h is re-read by every workgroup, so the tile is as tall as leaves enough
    // workgroups to fill the chip
    if (n_rows <= 64) { bv = vocab >= 65536 ? 256 : 128; bt = 64; }
    else if (n_rows <= 128) { bv = vocab >= 65536 ? 256 : 128; bt = 128; }
    // 129 to 256 rows: one token tile; a vocabulary below 65536 rows has too few 256-row tiles to fill the chip
    else if (n_rows <= 256 && vocab < 65536) { bv = 128; bt = 256; }
    // 257 to 384 rows against a large vocabulary: three token tiles of 128 rows waste fewer MFMAs than two of 256
    // (300 x 4096 x 128256: 541 -> 460 us); from 385 rows on the 256 x 256 tile's pinned schedule wins again
    else if (n_rows > 256 && n_rows <= 384 && vocab >= 65536) { bv = 256; bt = 128; }
    else { bv = 256; bt = 256; }
}

// A kernel that uses more than 64 KB of dynamic LDS has to be told so once per device; `done` (one bit per device,
// owned by the calling launcher, i.e. one per kernel) remembers where that has happened, so that the launch path of
// a small turn does not pay for the runtime call every time.
inline hipError_t allow_dynamic_lds(const void* fn, int bytes, std::atomic<uint64_t>& done)
{
    int dev = -1;
    const bool known = hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < 64;
    if (known && (done.load(std::memory_order_acquire) >> dev & 1ull)) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && known) done.fetch_or(1ull << dev, std::memory_order_release);
    return e;
}

template <int DT, int NVB, int NTB, int RING, bool PIN, bool WARM, int FKE = FK, bool WNT = false>
hipError_t launch_fast(const LmHeadArgs& a, hipStream_t stream)
{
    using Cfg = FastCfg<NVB, NTB, RING, FKE>;
    const int64_t groups = lmhead_grid(a);
    if (groups > 0x7fffffff) return hipErrorInvalidValue;
    auto fn = lmhead_score_kernel<DT, NVB, NTB, RING, PIN, WARM, FKE, WNT>;
    static std::atomic<uint64_t> lds_allowed{0};
    const hipError_t e = allow_dynamic_lds((const void*)fn, Cfg::kLds, lds_allowed);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(fn, dim3((unsigned)groups), dim3(256), Cfg::kLds, stream, a);
    return hipGetLastError();
}

template <int DT>
hipError_t launch_general(const LmHeadArgs& a, hipStream_t stream)
{
    const int64_t groups = lmhead_grid(a);
    if (groups > 0x7fffffff) return hipErrorInvalidValue;
    auto fn = lmhead_score_general_kernel<DT>;
    static std::atomic<uint64_t> lds_allowed{0};
    const hipError_t e = allow_dynamic_lds((const void*)fn, kLdsBytes, lds_allowed);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(fn, dim3((unsigned)groups), dim3(256), kLdsBytes, stream, a);
    return hipGetLastError();
}

template <int DT>
hipError_t launch_dtype(LmHeadArgs& a, hipStream_t stream)
{
    if (a.d_model % FK != 0) {                 // register-staged kernel, 256 x 256 tiles
        a.n_vtiles = (a.vocab + BV - 1) / BV;
        a.n_ttiles = (int)((a.n_rows + BT - 1) / BT);
        return launch_general<DT>(a, stream);
    }
    int bv, bt;
    tile_shape(a.n_rows, a.vocab, bv, bt);
    a.n_vtiles = (a.vocab + bv - 1) / bv;
    a.n_ttiles = (int)((a.n_rows + bt - 1) / bt);
    // Up to 128 rows the kernel is bound by streaming W, and whole 128-byte lines per load stream faster than halves
    // (tile rows of 64 K elements; d_model must be a multiple of 64).  With at most 64 rows there is one token tile, so
    // every byte of W is read exactly once and carries the non-temporal hint.
    const bool wide = a.d_model % 64 == 0 && tuning::get("SIRLLM_LMHEAD_WIDE", 1) != 0;
    if (bt == 64 && bv == 256)
        return wide ? launch_fast<DT, 4, 1, 3, false, false, 64, true>(a, stream) : launch_fast<DT, 4, 1, 4, false, false>(a, stream);
    if (bt == 64)
        return wide ? launch_fast<DT, 2, 1, 3, false, false, 64, true>(a, stream) : launch_fast<DT, 2, 1, 6, false, false>(a, stream);
    // 65 to 128 rows: 256 x 128 tiles against a large vocabulary (half the re-reads of h, twice the MFMAs per fragment
    // read: 7 to 10 % faster than 128 x 128 there), 128 x 128 otherwise (a small vocabulary has too few tall tiles)
    if (bt == 128 && bv == 256)
        return wide ? launch_fast<DT, 4, 2, 3, false, false, 64, false>(a, stream) : launch_fast<DT, 4, 2, 4, false, false>(a, stream);
    if (bt == 128 && wide) return launch_fast<DT, 2, 2, 3, false, false, 64, false>(a, stream);
    if (bt == 128) return launch_fast<DT, 2, 2, 5, false, false>(a, stream);
    // 128 x 256 tiles (129 to 256 rows against a small vocabulary): 129 x 4096 x 32000 114 -> 78 us, 256 rows 126 -> 90 us
    if (bt == 256 && bv == 128)
        return wide ? launch_fast<DT, 2, 4, 3, false, false, 64, false>(a, stream) : launch_fast<DT, 2, 4, 6, true, false>(a, stream);
    return launch_fast<DT, 4, 4, 4, true, true>(a, stream);
}

}  // namespace

// Upper bound on the number of vocabulary tiles (= sets of triples) a call with these sizes writes.
int lmhead_tiles_vocab(int64_t n_rows, int32_t vocab)
{
    int bv, bt;
    tile_shape(n_rows, vocab, bv, bt);
    return (vocab + bv - 1) / bv;
}

hipError_t launch_lmhead_score(const LmHeadArgs& args, sirllm_dtype dt, float* out, int64_t rows_per_stream,
                               int64_t out_stride, hipStream_t stream, const LmHeadRagged* ragged)
{
    LmHeadRagged rg = {nullptr, nullptr, 0};
    if (ragged) rg = *ragged;
    if (args.n_rows <= 0) return hipSuccess;
    LmHeadArgs a = args;
    hipError_t e = dt == SIRLLM_BF16 ? launch_dtype<SIRLLM_BF16>(a, stream) : launch_dtype<SIRLLM_F16>(a, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(lmhead_merge_kernel, dim3((unsigned)((a.n_rows + 3) / 4)), dim3(256), 0, stream,
                       a.partial, a.n_vtiles, a.part_stride, a.n_rows, out, rows_per_stream > 0 ? rows_per_stream : 1, out_stride, rg);
    return hipGetLastError();
}

}  // namespace sirllm
