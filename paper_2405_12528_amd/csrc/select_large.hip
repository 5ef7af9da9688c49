// Decay + Top_k selection + index build (paper Sec. 3.3, Sec. 3.1) for caches too large for one
// workgroup's registers (more than 32768 candidate slots per stream): the same MSB-first radix
// select, spread over a grid.  Tiles of 8192 slots; per stream a scratch block holds four global
// 256-bin histograms (one per radix pass) and per-tile (greater, equal) counts.
//   zero      clears the histograms
//   hist<p>   pass p: every workgroup re-derives the digits chosen by passes < p from the finished
//             global histograms, builds the histogram of its tile in LDS, adds it to the global one
//   count     derives the threshold key tau and the tie quota, counts greater / equal per tile
//   scatter   prefix over the tiles before it + the in-tile prefix of the one-workgroup kernel give
//             every kept slot its in-cache position
// Kernel boundaries order the phases; nothing spins.  Latency bound (seven small launches).
// The same launches serve ragged batches (every stream's own sizes are read from device memory; a stream within
// its budget is only decayed, a stream beyond the promised bounds is flagged and left alone: Alg. 1 per stream) and
// the RandomLLM baseline of Sec. 4.1 (the keys are then draws of Philox4x32-10, no score is read or written).
#include "common.h"
#include "select_device.h"

namespace sirllm {
namespace {

using select_dev::order_key;
using select_dev::wave_inclusive_scan;

constexpr int kBlock = 1024;
constexpr int kKpt = 8;
constexpr int kTile = kBlock * kKpt;

struct LargeArgs {
    SelectArgs a;
    uint32_t* ws;          // per stream: [4][256] histograms, then n_tiles x {greater, equal}
    int64_t ws_stride;     // uint32 words per stream
    int32_t n_tiles;
    int32_t random_keys;   // keys are generator draws, not scores
};

// What a workgroup does for its stream.  Uniform batches: always the selection on the launch's sizes.
enum StreamMode { kSelect = 0, kKeepAll = 1, kFlagged = 2 };
struct StreamDims {
    int n_held, n_cand, mode;
};

__device__ __forceinline__ StreamDims dims_of(const SelectArgs& a, int s)
{
    StreamDims d = {a.n_held, a.n_cand, kSelect};
    if (a.held_dev) {
        const int64_t held = a.held_dev[s];
        const int64_t n_new = (int64_t)a.cu_new_dev[s + 1] - (int64_t)a.cu_new_dev[s];
        const int64_t cand = held + n_new;
        const bool fits = held >= 0 && n_new >= 0 && n_new <= a.max_new && cand <= a.n_cand;
        d.n_held = fits ? (int)held : 0;
        d.n_cand = fits ? (int)cand : 0;
        d.mode = !fits ? kFlagged : (cand <= (int64_t)a.n_sink + a.n_topk + a.n_recent ? kKeepAll : kSelect);
    }
    return d;
}

struct ScanSmem {
    uint32_t wave_tot[kBlock / kWave];
    uint32_t sel_digit, sel_above;
};

// Digits of passes [0, n_passes) from the finished global histograms: returns the key prefix they
// fix and how many of the n_topk are still to be found below it.  Called by the whole workgroup.
__device__ __forceinline__ void derive_prefix(const uint32_t* hist, int n_passes, uint32_t n_topk, ScanSmem& sm,
                                              uint32_t& prefix, uint32_t& mask, uint32_t& k_rem)
{
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    prefix = 0u; mask = 0u; k_rem = n_topk;
    for (int p = 0; p < n_passes; ++p) {
        const int shift = 24 - 8 * p;
        const uint32_t c = (tid < 256) ? hist[p * 256 + tid] : 0u;
        const uint32_t inc = wave_inclusive_scan(c);
        __syncthreads();                                   // sm is reused from the previous pass
        if (lane == kWave - 1) sm.wave_tot[wave] = inc;
        __syncthreads();
        if (tid < 256) {
            uint32_t below_waves = 0u, total = 0u;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const uint32_t t = sm.wave_tot[w];
                if (w < wave) below_waves += t;
                total += t;
            }
            const uint32_t above = total - (inc + below_waves);
            if (above < k_rem && k_rem <= above + c) { sm.sel_digit = (uint32_t)tid; sm.sel_above = above; }
        }
        __syncthreads();
        prefix |= sm.sel_digit << shift;
        mask |= 255u << shift;
        k_rem -= sm.sel_above;
    }
}

// Slot i of a stream: its value (the decayed score; 0 for the random policy) and the key it is ranked by.
__device__ __forceinline__ uint32_t slot_key(const LargeArgs& g, const float* E, int i, int n_held, int stream, float& val)
{
    if (g.random_keys) {
        val = 0.0f;
        return select_dev::philox4x32_10_word0((uint32_t)i, (uint32_t)stream, g.a.turn_lo, g.a.turn_hi, g.a.seed_lo,
                                               g.a.seed_hi);
    }
    float e = E[i];
    if (i < n_held) e = __fmul_rn(e, g.a.decay);           // one rounded multiply, never fused
    val = e;
    return order_key(e);
}

__global__ __launch_bounds__(256) void zero_kernel(LargeArgs g)
{
    const int64_t n = (int64_t)g.a.n_streams * g.ws_stride;       // histograms and tile counts alike
    for (int64_t w = (int64_t)blockIdx.x * 256 + threadIdx.x; w < n; w += (int64_t)gridDim.x * 256) g.ws[w] = 0u;
}

__global__ __launch_bounds__(kBlock) void hist_kernel(LargeArgs g, int pass)
{
    __shared__ ScanSmem sm;
    __shared__ uint32_t lh[256];
    const SelectArgs& a = g.a;
    const int tid = threadIdx.x, tile = blockIdx.x, stream = blockIdx.y;
    const StreamDims d = dims_of(a, stream);
    if (d.mode != kSelect || tile * kTile >= d.n_cand) return;      // uniform over the workgroup
    uint32_t* hist = g.ws + stream * g.ws_stride;
    uint32_t prefix, mask, k_rem;
    derive_prefix(hist, pass, (uint32_t)a.n_topk, sm, prefix, mask, k_rem);
    if (tid < 256) lh[tid] = 0u;
    __syncthreads();
    const float* E = a.scores + (int64_t)stream * a.scores_stride;
    const int mid_lo = a.n_sink, mid_hi = d.n_cand - a.n_recent;
    const int shift = 24 - 8 * pass;
#pragma unroll
    for (int q = 0; q < kKpt; ++q) {
        const int i = tile * kTile + q * kBlock + tid;     // coalesced: order does not matter for counting
        if (i >= mid_lo && i < mid_hi) {
            float val;
            const uint32_t key = slot_key(g, E, i, d.n_held, stream, val);
            if ((key & mask) == prefix) atomicAdd(&lh[(key >> shift) & 255u], 1u);
        }
    }
    __syncthreads();
    if (tid < 256 && lh[tid]) atomicAdd(&hist[pass * 256 + tid], lh[tid]);
}

__global__ __launch_bounds__(kBlock) void count_kernel(LargeArgs g)
{
    __shared__ ScanSmem sm;
    __shared__ uint32_t red[2][kBlock / kWave];
    const SelectArgs& a = g.a;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int tile = blockIdx.x, stream = blockIdx.y;
    const StreamDims d = dims_of(a, stream);
    if (d.mode != kSelect || tile * kTile >= d.n_cand) return;      // its counts stay zero
    uint32_t* hist = g.ws + stream * g.ws_stride;
    uint32_t tau, mask, quota;
    derive_prefix(hist, 4, (uint32_t)a.n_topk, sm, tau, mask, quota);
    const float* E = a.scores + (int64_t)stream * a.scores_stride;
    const int mid_lo = a.n_sink, mid_hi = d.n_cand - a.n_recent;
    uint32_t gt = 0u, eq = 0u;
#pragma unroll
    for (int q = 0; q < kKpt; ++q) {
        const int i = tile * kTile + q * kBlock + tid;
        if (i >= mid_lo && i < mid_hi) {
            float val;
            const uint32_t key = slot_key(g, E, i, d.n_held, stream, val);
            gt += key > tau;
            eq += key == tau;
        }
    }
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        gt += __shfl_xor(gt, off, kWave);
        eq += __shfl_xor(eq, off, kWave);
    }
    if (lane == 0) { red[0][wave] = gt; red[1][wave] = eq; }
    __syncthreads();
    if (tid == 0) {
        uint32_t G = 0u, Q = 0u;
        for (int w = 0; w < kBlock / kWave; ++w) { G += red[0][w]; Q += red[1][w]; }
        hist[1024 + 2 * tile] = G;
        hist[1024 + 2 * tile + 1] = Q;
    }
}

__global__ __launch_bounds__(kBlock) void scatter_kernel(LargeArgs g)
{
    __shared__ ScanSmem sm;
    __shared__ uint32_t red[2][kBlock / kWave];
    const SelectArgs& a = g.a;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    constexpr int NW = kBlock / kWave;
    const int tile = blockIdx.x, stream = blockIdx.y;
    const StreamDims d = dims_of(a, stream);
    const int budget = a.n_sink + a.n_topk + a.n_recent;
    if (a.n_keep_dev && tile == 0 && tid == 0)
        a.n_keep_dev[stream] = d.mode == kFlagged ? -1 : (d.n_cand < budget ? d.n_cand : budget);
    if (d.mode == kFlagged || tile * kTile >= d.n_cand) return;
    if (d.mode == kKeepAll) {                              // within the budget: identity list, E <- E * eta
        for (int i = tile * kTile + tid; i < min(d.n_cand, (tile + 1) * kTile); i += kBlock) {
            a.kept_idx[(int64_t)stream * a.idx_stride + i] = i;
            if (!g.random_keys) {
                float val;
                slot_key(g, a.scores + (int64_t)stream * a.scores_stride, i, d.n_held, stream, val);
                a.scores_out[(int64_t)stream * a.out_stride + i] = val;
            }
        }
        return;
    }
    uint32_t* hist = g.ws + stream * g.ws_stride;
    uint32_t tau, mask, quota;
    if (a.n_topk > 0) {
        derive_prefix(hist, 4, (uint32_t)a.n_topk, sm, tau, mask, quota);
    } else {
        tau = 0xffffffffu; quota = 0u;                     // nothing is greater, nothing equal is taken
    }
    // kept middle slots in the tiles before this one
    uint32_t g0 = 0u, e0 = 0u;
    for (int t = tid; t < tile; t += kBlock) { g0 += hist[1024 + 2 * t]; e0 += hist[1024 + 2 * t + 1]; }
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        g0 += __shfl_xor(g0, off, kWave);
        e0 += __shfl_xor(e0, off, kWave);
    }
    if (lane == 0) { red[0][wave] = g0; red[1][wave] = e0; }
    __syncthreads();
    g0 = 0u; e0 = 0u;
#pragma unroll
    for (int w = 0; w < NW; ++w) { g0 += red[0][w]; e0 += red[1][w]; }
    __syncthreads();                                       // red is reused below

    // this tile: every lane owns kKpt consecutive slots, as in the one-workgroup kernel
    const int n_cand = d.n_cand, mid_lo = a.n_sink, mid_hi = n_cand - a.n_recent;
    const int n_keep = budget;
    const float* E = a.scores + (int64_t)stream * a.scores_stride;
    const int i0 = tile * kTile + tid * kKpt;
    float val[kKpt];
    uint32_t key[kKpt];
    uint32_t mg = 0u, me = 0u;
#pragma unroll
    for (int q = 0; q < kKpt; ++q) {
        const int i = i0 + q;
        val[q] = 0.0f;
        key[q] = 0u;
        if (i < n_cand && (!g.random_keys || (i >= mid_lo && i < mid_hi))) key[q] = slot_key(g, E, i, d.n_held, stream, val[q]);
        if (i >= mid_lo && i < mid_hi) {
            mg += key[q] > tau;
            me += key[q] == tau;
        }
    }
    const uint32_t ig = wave_inclusive_scan(mg), ie = wave_inclusive_scan(me);
    if (lane == kWave - 1) { red[0][wave] = ig; red[1][wave] = ie; }
    __syncthreads();
    uint32_t gt = g0 + ig - mg, eq = e0 + ie - me;
#pragma unroll
    for (int w = 0; w < NW; ++w)
        if (w < wave) { gt += red[0][w]; eq += red[1][w]; }

    int32_t* idx = a.kept_idx + (int64_t)stream * a.idx_stride;
    float* Eo = a.scores_out + (int64_t)stream * a.out_stride;
#pragma unroll
    for (int q = 0; q < kKpt; ++q) {
        const int i = i0 + q;
        if (i >= n_cand) break;
        int pos = -1;
        if (i < mid_lo) {
            pos = i;                                            // Id_sink
        } else if (i >= mid_hi) {
            pos = n_keep - (n_cand - i);                        // Id_recent
        } else {
            if (key[q] > tau) {
                pos = mid_lo + (int)(gt + (eq < quota ? eq : quota));
                ++gt;
            } else if (key[q] == tau) {
                if (eq < quota) pos = mid_lo + (int)(gt + eq);  // Id_entropy, ties to the lower slot
                ++eq;
            }
        }
        if (pos >= 0 && pos < n_keep) {
            idx[pos] = i;
            if (!g.random_keys) Eo[pos] = val[q];
        }
    }
}

}  // namespace

size_t select_large_scratch_bytes(int32_t n_streams, int32_t n_cand)
{
    if (n_cand <= SIRLLM_SINGLE_WG_CAND || n_streams <= 0) return 0;
    const int64_t n_tiles = ((int64_t)n_cand + kTile - 1) / kTile;
    const int64_t words = (1024 + 2 * n_tiles + 63) / 64 * 64;
    return (size_t)(words * 4 * n_streams);
}

hipError_t launch_select_large(const SelectArgs& a, void* scratch, hipStream_t stream, bool random_keys)
{
    if (a.n_streams <= 0 || a.n_cand <= 0) return hipSuccess;
    LargeArgs g;
    g.a = a;
    g.n_tiles = (a.n_cand + kTile - 1) / kTile;
    g.ws = (uint32_t*)scratch;
    g.ws_stride = (1024 + 2 * (int64_t)g.n_tiles + 63) / 64 * 64;
    g.random_keys = random_keys ? 1 : 0;
    if (g.n_tiles > 65535 || a.n_streams > 65535) return hipErrorInvalidValue;
    const dim3 grid((unsigned)g.n_tiles, (unsigned)a.n_streams), block(kBlock);
    hipLaunchKernelGGL(zero_kernel, dim3((unsigned)min((int64_t)1024, (a.n_streams * g.ws_stride + 255) / 256)), dim3(256), 0, stream, g);
    if (a.n_topk > 0) {
        for (int pass = 0; pass < 4; ++pass) hipLaunchKernelGGL(hist_kernel, grid, block, 0, stream, g, pass);
        hipLaunchKernelGGL(count_kernel, grid, block, 0, stream, g);
    }
    hipLaunchKernelGGL(scatter_kernel, grid, block, 0, stream, g);
    return hipGetLastError();
}

}  // namespace sirllm
