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

// Byte offset of 16-byte chunk `c` (0..7) of tile row `r` inside a tile: rows are 128 bytes, the chunk
// index is XOR-ed with the low row bits so that 8 consecutive rows of one chunk column cover all banks.
__device__ __forceinline__ int tile_offset(int r, int c) { return r * kRowBytes + ((c ^ (r & 7)) << 4); }

template <int DT>
__global__ __launch_bounds__(256) void lmhead_score_kernel(LmHeadArgs a)
{
    extern __shared__ __align__(16) char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wv = wave & 1, wt = wave >> 1;          // which 128 vocabulary rows / 128 tokens this wave owns

    // Workgroups are dealt to the 8 XCDs round robin.  An XCD takes every 8th vocabulary tile and walks
    // all token tiles of it back to back, so a weight tile is fetched into one L2 only and the (small)
    // hidden-state matrix is what the XCDs share.
    const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
    const int tt = q % a.n_ttiles;
    const int vt = (q / a.n_ttiles) * 8 + xcd;
    if (vt >= a.n_vtiles) return;
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
    for (int kk = 0; kk < 4; ++kk) cpos[kk] = ((2 * kk + khalf) ^ (frag_row & 7)) << 4;

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

    // ---- epilogue: per token, (m, s) over this wave's 128 vocabulary rows and the token's own logit
    float* red = (float*)(lds + 2 * kStageBytes);
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
    {
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
}

// Folds the n_parts triples of every row: 16 rows per workgroup, 16 lanes per row striding over the parts.
__global__ __launch_bounds__(256) void lmhead_merge_kernel(const float* partials, int n_parts, int64_t part_stride,
                                                           int64_t n_rows, float* out)
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
        out[row] = (acc.m - zt) + logf(acc.s);
    }
}

}  // namespace

int lmhead_tiles_vocab(int32_t vocab) { return (vocab + BV - 1) / BV; }

hipError_t launch_lmhead_score(const LmHeadArgs& args, sirllm_dtype dt, float* scores_out, hipStream_t stream)
{
    if (args.n_rows <= 0) return hipSuccess;
    LmHeadArgs a = args;
    a.n_vtiles = lmhead_tiles_vocab(a.vocab);
    a.n_ttiles = (int)((a.n_rows + BT - 1) / BT);
    const int64_t groups = (int64_t)((a.n_vtiles + 7) / 8) * a.n_ttiles * 8;
    if (groups > 0x7fffffff) return hipErrorInvalidValue;
    const void* fn = dt == SIRLLM_BF16 ? (const void*)lmhead_score_kernel<SIRLLM_BF16>
                                       : (const void*)lmhead_score_kernel<SIRLLM_F16>;
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    if (dt == SIRLLM_BF16)
        hipLaunchKernelGGL(lmhead_score_kernel<SIRLLM_BF16>, dim3((unsigned)groups), dim3(256), kLdsBytes, stream, a);
    else
        hipLaunchKernelGGL(lmhead_score_kernel<SIRLLM_F16>, dim3((unsigned)groups), dim3(256), kLdsBytes, stream, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(lmhead_merge_kernel, dim3((unsigned)((a.n_rows + 15) / 16)), dim3(256), 0, stream,
                       a.partial, a.n_vtiles, a.part_stride, a.n_rows, scores_out);
    return hipGetLastError();
}

}  // namespace sirllm
