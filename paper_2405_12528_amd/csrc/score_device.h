// Device code of the token-entropy score e = logsumexp(z) - z[token]  (paper Sec. 3.2): a
// one-pass online (max, sum) reduction over one vocabulary row by one workgroup.  Every lane
// streams 16-byte vectors of the row and keeps a running (m, s) pair in registers; lanes are
// merged with wavefront shuffles, waves through LDS.  Each logit is read from HBM exactly once.
#pragma once

#include "common.h"

namespace sirllm {
namespace score_dev {

constexpr float kLog2e = 1.4426950408889634f;
constexpr uint32_t kNegInfBits = 0xff800000u;

__device__ __forceinline__ float exp2_hw(float x) { return __builtin_amdgcn_exp2f(x); }   // v_exp_f32

struct MS {
    float m;   // running maximum (-inf when nothing finite has been seen)
    float s;   // sum of exp(z - m) over what has been seen
};

// (m, s) pairs form a monoid under this merge; a side whose m equals the merged m is not rescaled,
// which also keeps the empty element (-inf, 0) neutral.
__device__ __forceinline__ MS merge(MS a, MS b)
{
    const float m = fmaxf(a.m, b.m);
    const float fa = (a.m == m) ? 1.0f : exp2_hw((a.m - m) * kLog2e);
    const float fb = (b.m == m) ? 1.0f : exp2_hw((b.m - m) * kLog2e);
    return {m, a.s * fa + b.s * fb};
}

// One step of a cross-lane reduction: every lane merges in the (m, s) of the lane CTRL names (the empty element
// where there is none).
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ MS merge_from(MS a)
{
    const MS o = {__uint_as_float(dpp_move<CTRL, ROW_MASK>(__float_as_uint(a.m), kNegInfBits)),
                  __uint_as_float(dpp_move<CTRL, ROW_MASK>(__float_as_uint(a.s), 0u))};
    return merge(a, o);
}

// Lane 16*r + 15 ends up with the merge of row r's sixteen lanes (rows are the wave's four groups of 16 lanes).
__device__ __forceinline__ MS row_reduce(MS a)
{
    a = merge_from<kDppRowShr1>(a);
    a = merge_from<kDppRowShr2>(a);
    a = merge_from<kDppRowShr4>(a);
    a = merge_from<kDppRowShr8>(a);
    return a;
}

// Lane 63 ends up with the merge of all 64 lanes.
__device__ __forceinline__ MS wave_reduce(MS a)
{
    a = row_reduce(a);
    a = merge_from<kDppRowBcast15, 0xa>(a);
    a = merge_from<kDppRowBcast31, 0xc>(a);
    return a;
}

template <int N>
__device__ __forceinline__ void accumulate(const float (&z)[N], MS& acc)
{
    float cm = z[0];
#pragma unroll
    for (int i = 1; i < N; ++i) cm = fmaxf(cm, z[i]);
    const float m_new = fmaxf(acc.m, cm);
    const float f = (acc.m == m_new) ? 1.0f : exp2_hw((acc.m - m_new) * kLog2e);
    // while no finite value has been seen the reference is 0: exp(-inf - 0) = 0, never inf - inf
    const float ref = (m_new == -INFINITY) ? 0.0f : m_new;
    float t[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int i = 0; i < N; ++i) t[i & 3] += exp2_hw((z[i] - ref) * kLog2e);
    acc.s = acc.s * f + ((t[0] + t[1]) + (t[2] + t[3]));
    acc.m = m_new;
}

// Element traits by sirllm_dtype code.
template <int DT> struct Elem;
template <> struct Elem<SIRLLM_F32> {
    static constexpr int kSize = 4;
    static constexpr int kVec = 4;
    static __device__ __forceinline__ float load1(const char* row, int i) { return ((const float*)row)[i]; }
    static __device__ __forceinline__ void unpack(u32x4 v, float* z)
    {
        z[0] = __uint_as_float(v.x); z[1] = __uint_as_float(v.y);
        z[2] = __uint_as_float(v.z); z[3] = __uint_as_float(v.w);
    }
    static __device__ __forceinline__ u32x4 neg_inf()
    {
        u32x4 v = {kNegInfBits, kNegInfBits, kNegInfBits, kNegInfBits};
        return v;
    }
};
template <> struct Elem<SIRLLM_BF16> {   // bfloat16: the upper half of a binary32
    static constexpr int kSize = 2;
    static constexpr int kVec = 8;
    static __device__ __forceinline__ float load1(const char* row, int i)
    {
        return __uint_as_float((uint32_t)((const uint16_t*)row)[i] << 16);
    }
    static __device__ __forceinline__ void unpack(u32x4 v, float* z)
    {
        z[0] = __uint_as_float(v.x << 16); z[1] = __uint_as_float(v.x & 0xffff0000u);
        z[2] = __uint_as_float(v.y << 16); z[3] = __uint_as_float(v.y & 0xffff0000u);
        z[4] = __uint_as_float(v.z << 16); z[5] = __uint_as_float(v.z & 0xffff0000u);
        z[6] = __uint_as_float(v.w << 16); z[7] = __uint_as_float(v.w & 0xffff0000u);
    }
    static __device__ __forceinline__ u32x4 neg_inf()
    {
        u32x4 v = {0xff80ff80u, 0xff80ff80u, 0xff80ff80u, 0xff80ff80u};
        return v;
    }
};

template <> struct Elem<SIRLLM_F16> {    // IEEE binary16, widened exactly by v_cvt_f32_f16
    static constexpr int kSize = 2;
    static constexpr int kVec = 8;
    typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ float load1(const char* row, int i)
    {
        return (float)__builtin_bit_cast(_Float16, ((const uint16_t*)row)[i]);
    }
    static __device__ __forceinline__ void unpack(u32x4 v, float* z)
    {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const half2_t h = __builtin_bit_cast(half2_t, w[i]);
            z[2 * i] = (float)h.x;
            z[2 * i + 1] = (float)h.y;
        }
    }
    static __device__ __forceinline__ u32x4 neg_inf()
    {
        u32x4 v = {0xfc00fc00u, 0xfc00fc00u, 0xfc00fc00u, 0xfc00fc00u};
        return v;
    }
};

template <bool NT>
__device__ __forceinline__ u32x4 load_vec(const u32x4* p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

template <int BLOCK>
struct ScoreSmem {
    float m[BLOCK / kWave];
    float s[BLOCK / kWave];
};

// Scores row `row` with the whole workgroup (BLOCK threads); thread 0 writes the result.
template <int DT, int BLOCK, int UNROLL, bool NT>
__device__ __forceinline__ void score_row(const ScoreArgs& a, int64_t row, ScoreSmem<BLOCK>& sm)
{
    using E = Elem<DT>;
    constexpr int VEC = E::kVec;
    constexpr int ESIZE = E::kSize;
    const int tid = threadIdx.x;
    const char* rowp = (const char*)a.logits + row * a.ld * ESIZE;
    const int V = a.vocab;

    // split the row into [0, head) scalar | nvec 16-byte aligned vectors | scalar tail
    int head = (int)(((16u - (uint32_t)((uintptr_t)rowp & 15u)) & 15u) / ESIZE);
    if (head > V) head = V;
    const int nvec = (V - head) / VEC;
    const int tail0 = head + nvec * VEC;

    // The token's own logit is fetched now, by the lane that finishes the row, so that its two dependent loads (the
    // id, then the logit) are over long before the reduction is: at the end of a short row they would be the
    // longest thing left.
    float z_tok = __uint_as_float(0x7fc00000u);            // NaN: no such token (or not in this chunk of columns)
    if (tid == 0) {
        const int64_t local = (int64_t)a.token_ids[row] - (a.partial ? a.v_begin : 0);
        if (local >= 0 && local < V) z_tok = E::load1(rowp, (int)local);
    }

    MS acc = {-INFINITY, 0.0f};
    {   // at most 2*(VEC-1) scalar elements, one per thread
        int e = -1;
        if (tid < head) e = tid;
        else if (tid - head < V - tail0) e = tail0 + (tid - head);
        if (e >= 0) {
            float z[1] = {E::load1(rowp, e)};
            accumulate<1>(z, acc);
        }
    }

    const u32x4* vp = (const u32x4*)(rowp + (size_t)head * ESIZE);
    int base = 0;
    for (; base + BLOCK * UNROLL <= nvec; base += BLOCK * UNROLL) {
        u32x4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) v[u] = load_vec<NT>(vp + base + u * BLOCK + tid);
        float z[UNROLL * VEC];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) E::unpack(v[u], z + u * VEC);
        accumulate<UNROLL * VEC>(z, acc);
    }
    if (base < nvec) {   // ragged last sweep: lanes past the end see -inf, which adds exactly 0
        u32x4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int i = base + u * BLOCK + tid;
            v[u] = (i < nvec) ? load_vec<NT>(vp + i) : E::neg_inf();
        }
        float z[UNROLL * VEC];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) E::unpack(v[u], z + u * VEC);
        accumulate<UNROLL * VEC>(z, acc);
    }

    // lanes -> wave (lane 63 holds the wave's result)
    acc = wave_reduce(acc);
    // waves -> workgroup
    constexpr int NW = BLOCK / kWave;
    static_assert(NW <= 16, "the second stage reduces one row of sixteen lanes");
    if constexpr (NW > 1) {
        if ((tid & (kWave - 1)) == kWave - 1) { sm.m[tid / kWave] = acc.m; sm.s[tid / kWave] = acc.s; }
        __syncthreads();
        if (tid < kWave) {
            acc = (tid < NW) ? MS{sm.m[tid], sm.s[tid]} : MS{-INFINITY, 0.0f};
            acc = row_reduce(acc);                                     // lanes 0..15 hold the waves: lane 15 has it all
            acc.m = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(acc.m), 15));
            acc.s = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(acc.s), 15));
        }
    } else {
        acc.m = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(acc.m), kWave - 1));
        acc.s = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(acc.s), kWave - 1));
    }
    if (tid == 0 && a.partial) {
        // a chunk of columns [v_begin, v_begin + V) of a longer row: leave the monoid element and, if the
        // token's column is in this chunk, its logit (NaN says "not in this chunk")
        a.partial[3 * row + 0] = acc.m;
        a.partial[3 * row + 1] = acc.s;
        a.partial[3 * row + 2] = z_tok;
        return;
    }
    if (tid == 0) {
        // a token id outside [0, V) left z_tok = NaN, and so is the score
        const float e = (acc.m - z_tok) + logf(acc.s);
        if (a.cu_rows) {
            // ragged batch: the stream whose row range holds `row` (largest s with cu_rows[s] <= row)
            int lo = 0, hi = a.n_streams_r;
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if ((int64_t)a.cu_rows[mid] <= row) lo = mid; else hi = mid;
            }
            const int64_t t = row - a.cu_rows[lo];
            const int64_t held = a.held_dev[lo];
            const int64_t pos = held + t;
            if (pos >= 0 && pos < a.stride_a)            // sizes the caller did not promise are dropped, not written
                a.out_a[lo * a.stride_a + pos] = e;
            if (a.out_b) {
                // the token's place in the compacted score cache: the new tokens are the tail of the kept list
                const int64_t n_new = a.cu_rows[lo + 1] - a.cu_rows[lo];
                const int64_t n_cand = held + n_new;
                const int64_t n_keep = n_cand < a.budget_r ? n_cand : a.budget_r;
                const int64_t posb = n_keep - n_new + t;
                if (posb >= 0 && posb < a.stride_b) a.out_b[lo * a.stride_b + posb] = e;
            }
        } else {
            const int64_t stream = row / a.rows_per_stream;
            const int64_t t = row - stream * a.rows_per_stream;
            a.out_a[stream * a.stride_a + t] = e;
            if (a.out_b) a.out_b[stream * a.stride_b + t] = e;
        }
    }
}

}  // namespace score_dev
}  // namespace sirllm
