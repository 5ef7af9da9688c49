// Device code of decay, Top_k selection and index build (paper Sec. 3.3: E <- E*eta,
// Id_entropy = Top_k(E), E <- E[Id]; Sec. 3.1: Id_sink, Id_recent) for ONE dialogue stream by
// one workgroup.  Every thread owns KPT consecutive candidate slots in registers.  The k-th
// largest key of the middle region is found by an MSB-first radix select (four 8-bit digits, one
// LDS histogram, two barriers per digit), which yields the threshold key and how many slots equal to it may still be
// taken (lowest slots first); one block-wide prefix sum over (greater, equal) counts then
// gives every kept slot its in-cache position, so the kept list comes out in ascending slot
// order without sorting anything.  Latency bound: a few tens of KB per stream.
#pragma once

#include "common.h"

// Phase marks: a file that includes this header to time the selection's phases defines SIRLLM_TSTAMP(k) beforehand
// (e.g. to store the cycle counter into slot k of a buffer); in the library it expands to nothing.
#ifndef SIRLLM_TSTAMP
#define SIRLLM_TSTAMP(k)
#endif

namespace sirllm {
namespace select_dev {

// Order-preserving map from binary32 to uint32: a > b as numbers <=> key(a) > key(b).
// -0 is folded onto +0 so that the two tie; NaNs land above +inf (sign clear) or below -inf (sign set).
__device__ __forceinline__ uint32_t order_key(float x)
{
    uint32_t b = __float_as_uint(x);
    if (b == 0x80000000u) b = 0u;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) { return wave_inclusive_sum(v); }

template <int BLOCK>
struct SelectSmem {
    uint32_t hist[256];
    uint32_t wave_tot[BLOCK / kWave];
    uint32_t sel_digit;
    uint32_t sel_above;
};

// Philox4x32-10 (Salmon et al., SC'11), word 0 of the output block.
__device__ __forceinline__ uint32_t philox4x32_10_word0(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                        uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return c0;
}

// RANDOM_KEYS: the keys are not scores but draws of a counter-based generator (the RandomLLM
// baseline, paper Sec. 4.1); no score is read or written.
// NEW_ELSEWHERE: the slots [n_held, n_cand) all lie in the recent window and their scores are
// being written by other workgroups at the same time; this workgroup then neither reads them nor
// writes their scores_out entries (only their kept_idx entries).
template <int BLOCK, int KPT, bool NEW_ELSEWHERE, bool RANDOM_KEYS = false>
__device__ __forceinline__ void select_stream(const SelectArgs& a, int stream, SelectSmem<BLOCK>& sm)
{
    static_assert(BLOCK >= 256 && BLOCK % kWave == 0, "histogram scan uses the first 256 threads");
    constexpr int NW = BLOCK / kWave;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;

    const int n_cand = a.n_cand;
    const int mid_lo = a.n_sink;
    const int mid_hi = n_cand - a.n_recent;
    const int n_keep = a.n_sink + a.n_topk + a.n_recent;      // this path runs only when n_cand > budget
    const int n_read = NEW_ELSEWHERE ? a.n_held : n_cand;
    const float* E = a.scores + (int64_t)stream * a.scores_stride;
    const int i0 = tid * KPT;

    // E <- E * eta for the held slots (one rounded multiply; never fused with anything)
    float val[KPT];
    if constexpr (RANDOM_KEYS) {
#pragma unroll
        for (int q = 0; q < KPT; ++q) {
            const int i = i0 + q;
            float e = 0.0f;
            if (i >= mid_lo && i < mid_hi)
                e = __uint_as_float(philox4x32_10_word0((uint32_t)i, (uint32_t)stream, a.turn_lo, a.turn_hi,
                                                        a.seed_lo, a.seed_hi));
            val[q] = e;
        }
    } else {
        // a lane's KPT consecutive scores in 16-byte pieces when the row allows it (uniform over the workgroup),
        // else one by one
        bool wide = false;
        if constexpr (KPT % 4 == 0) wide = (((uintptr_t)E) & 15) == 0;
        if (wide) {
            if constexpr (KPT % 4 == 0) {
#pragma unroll
                for (int q4 = 0; q4 < KPT; q4 += 4) {
                    const int i = i0 + q4;
                    u32x4 x = {0u, 0u, 0u, 0u};
                    if (i + 3 < n_read) {
                        x = *(const u32x4*)(E + i);
                    } else {
#pragma unroll
                        for (int t = 0; t < 4; ++t)
                            if (i + t < n_read) x[t] = __float_as_uint(E[i + t]);
                    }
#pragma unroll
                    for (int t = 0; t < 4; ++t) val[q4 + t] = __uint_as_float(x[t]);
                }
            }
        } else {
#pragma unroll
            for (int q = 0; q < KPT; ++q) val[q] = (i0 + q < n_read) ? E[i0 + q] : 0.0f;
        }
#pragma unroll
        for (int q = 0; q < KPT; ++q)
            if (i0 + q < a.n_held && i0 + q < n_read) val[q] = __fmul_rn(val[q], a.decay);
    }
    SIRLLM_TSTAMP(1);
    auto key_of = [](float v) -> uint32_t {
        if constexpr (RANDOM_KEYS) return __float_as_uint(v);
        else return order_key(v);
    };

    // ---- radix select of the n_topk-th largest key among the middle slots -------------------
    uint32_t prefix = 0xffffffffu, mask = 0xffffffffu;   // n_topk == 0: nothing is greater, quota 0
    uint32_t k_rem = 0;
    if (a.n_topk > 0) {
        prefix = 0u; mask = 0u; k_rem = (uint32_t)a.n_topk;
        if (tid < 256) sm.hist[tid] = 0u;
        __syncthreads();
        for (int shift = 24; shift >= 0; shift -= 8) {
            // A lane first folds its own slots: those whose digit equals the digit of its first live slot
            // go into the histogram with one add.  In the first pass (sign and high exponent bits, nearly
            // the same for every score) that is all of them; the wave then folds its lanes the same way: when
            // every live lane holds the same digit, one lane adds the wave's count.  That takes the pile-up on
            // one or two bins from one add per slot down to one per wave.  In later passes digits differ and
            // most slots add on their own.
            {
                uint32_t d0 = 0xffffffffu, n0 = 0u;
#pragma unroll
                for (int q = 0; q < KPT; ++q) {
                    const int i = i0 + q;
                    if (i >= mid_lo && i < mid_hi) {
                        const uint32_t key = key_of(val[q]);
                        if ((key & mask) == prefix) {
                            const uint32_t digit = (key >> shift) & 255u;
                            if (d0 == 0xffffffffu) d0 = digit;
                            if (digit == d0) ++n0;
                            else atomicAdd(&sm.hist[digit], 1u);
                        }
                    }
                }
                const unsigned long long live = __ballot(n0 != 0u);
                if (live != 0ull) {
                    const int first = __ffsll((long long)live) - 1;
                    const uint32_t ref = (uint32_t)__builtin_amdgcn_readlane((int)d0, first);
                    if (__ballot(n0 != 0u && d0 != ref) == 0ull) {
                        const uint32_t tot = wave_sum(n0);
                        if (lane == first) atomicAdd(&sm.hist[ref], tot);
                    } else if (n0) {
                        atomicAdd(&sm.hist[d0], n0);
                    }
                }
            }
            __syncthreads();
            // One wave finds the digit d with  #(digit > d) < k_rem <= #(digit >= d):  lane l owns bins 4l .. 4l+3,
            // a wave scan of the lanes' sums gives the count above each lane's bins.  It clears the bins for the next
            // pass on the way (every other wave is past its adds and waits at the barrier below).
            if (wave == 0) {
                uint32_t c[4];
#pragma unroll
                for (int b = 0; b < 4; ++b) { c[b] = sm.hist[4 * lane + b]; sm.hist[4 * lane + b] = 0u; }
                const uint32_t mine = (c[0] + c[1]) + (c[2] + c[3]);
                const uint32_t inc = wave_inclusive_scan(mine);
                const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)inc, kWave - 1);
                uint32_t above = total - inc;                       // slots in bins above this lane's four
#pragma unroll
                for (int b = 3; b >= 0; --b) {
                    if (above < k_rem && k_rem <= above + c[b]) { sm.sel_digit = (uint32_t)(4 * lane + b); sm.sel_above = above; }
                    above += c[b];
                }
            }
            __syncthreads();
            SIRLLM_TSTAMP(2 + (24 - shift) / 8);
            prefix |= sm.sel_digit << shift;
            mask |= 255u << shift;
            k_rem -= sm.sel_above;
        }
    }
    const uint32_t tau = prefix;       // key of the n_topk-th largest middle slot
    const uint32_t quota = k_rem;      // how many slots equal to tau are still taken, lowest first

    // ---- block-wide exclusive prefix sum of (greater, equal) counts ---------------------------
    uint32_t mine = 0u;                // greater in the low 16 bits, equal in the high 16
#pragma unroll
    for (int q = 0; q < KPT; ++q) {
        const int i = i0 + q;
        if (i >= mid_lo && i < mid_hi) {
            const uint32_t key = key_of(val[q]);
            mine += (key > tau) ? 1u : 0u;
            mine += (key == tau) ? 0x10000u : 0u;
        }
    }
    const uint32_t inc = wave_inclusive_scan(mine);
    if (lane == kWave - 1) sm.wave_tot[wave] = inc;
    __syncthreads();
    uint32_t before = inc - mine;
#pragma unroll
    for (int w = 0; w < NW; ++w)
        if (w < wave) before += sm.wave_tot[w];
    uint32_t g = before & 0xffffu, eq = before >> 16;
    SIRLLM_TSTAMP(6);

    // ---- index build: kept slot i goes to in-cache position pos; E_out[pos] = E[i] ------------
    int32_t* idx = a.kept_idx + (int64_t)stream * a.idx_stride;
    float* Eo = a.scores_out + (int64_t)stream * a.out_stride;
#pragma unroll
    for (int q = 0; q < KPT; ++q) {
        const int i = i0 + q;
        if (i >= n_cand) break;
        int pos = -1;
        if (i < mid_lo) {
            pos = i;                                            // Id_sink
        } else if (i >= mid_hi) {
            pos = n_keep - (n_cand - i);                        // Id_recent
        } else {
            const uint32_t key = key_of(val[q]);
            if (key > tau) {
                pos = mid_lo + (int)(g + (eq < quota ? eq : quota));
                ++g;
            } else if (key == tau) {
                if (eq < quota) pos = mid_lo + (int)(g + eq);   // Id_entropy, ties to the lower slot
                ++eq;
            }
        }
        if (pos >= 0 && pos < n_keep) {
            idx[pos] = i;
            if constexpr (!RANDOM_KEYS) {
                if (i < n_read) Eo[pos] = val[q];
            }
        }
    }
}

// One stream of a ragged batch: the workgroup reads the stream's own sizes, flags sizes beyond what the
// caller promised, then either keeps everything (decay only) or runs the selection.
template <int BLOCK, int KPT, bool NEW_ELSEWHERE>
__device__ __forceinline__ void select_ragged_stream(const SelectArgs& a, int s, SelectSmem<BLOCK>& sm)
{
    SelectArgs b = a;
    const int64_t held = a.held_dev[s];
    const int64_t n_new = (int64_t)a.cu_new_dev[s + 1] - (int64_t)a.cu_new_dev[s];
    const int64_t cand = held + n_new;                      // 64-bit: sizes that are garbage must not wrap into range
    const int budget = a.n_sink + a.n_topk + a.n_recent;
    const bool fits = held >= 0 && n_new >= 0 && n_new <= a.max_new && cand <= a.n_cand && cand <= BLOCK * KPT;
    if (threadIdx.x == 0) a.n_keep_dev[s] = !fits ? -1 : (int)(cand < budget ? cand : budget);
    if (!fits) return;                      // flagged, nothing written (uniform over the workgroup)
    b.n_held = (int)held;
    b.n_cand = (int)cand;
    if (b.n_cand <= budget) {
        const int n_read = NEW_ELSEWHERE ? b.n_held : b.n_cand;
        for (int i = threadIdx.x; i < b.n_cand; i += BLOCK) {
            a.kept_idx[(int64_t)s * a.idx_stride + i] = i;
            if (i < n_read) {
                float e = a.scores[(int64_t)s * a.scores_stride + i];
                if (i < b.n_held) e = __fmul_rn(e, a.decay);
                a.scores_out[(int64_t)s * a.out_stride + i] = e;
            }
        }
        return;
    }
    select_stream<BLOCK, KPT, NEW_ELSEWHERE>(b, s, sm);
}

}  // namespace select_dev
}  // namespace sirllm
