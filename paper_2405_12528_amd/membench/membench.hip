// Plain streaming kernels that measure what this GPU's memory system gives a read-only scan, a write-only
// fill and a copy, with the same access shape the library's kernels use (one 16-byte vector per lane per step,
// non-temporal loads, stores at agent scope with the non-temporal hint), in workgroups of 64, 128 or 512 threads.  They are measurement references for bench.py, not part
// of the retention path: the score scan is compared with the read stream, the K/V gather with the copy.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// The store the library's gather uses for bytes it never touches again: written through (`sc1`) with the
// non-temporal hint; of the eight combinations of the sc0 / sc1 / nt modifiers the ones with sc1 fill 1 GiB fastest.
__device__ __forceinline__ void store_stream(u32x4* p, u32x4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt" ::"v"(p), "v"(v) : "memory");
}

// Every lane reads `per_lane` vectors a whole workgroup sweep apart; the XOR of what it read is stored only if
// it equals a value that random data never produces, so the loads cannot be dropped.
template <int kBlock, int UNROLL>
__global__ __launch_bounds__(kBlock) void read_kernel(const u32x4* src, uint64_t n_vec, uint32_t* sink)
{
    const uint64_t base = (uint64_t)blockIdx.x * (kBlock * UNROLL) + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const uint64_t i = base + (uint64_t)u * kBlock;
        if (i < n_vec) acc ^= __builtin_nontemporal_load(src + i);
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u && acc.x == 0x7f4a7c15u) sink[0] = acc.y;
}

template <int kBlock>
__global__ __launch_bounds__(kBlock) void write_kernel(u32x4* dst, uint64_t n_vec, uint32_t value)
{
    const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const u32x4 v = {value, value + 1u, value + 2u, value + 3u};
    if (i < n_vec) store_stream(dst + i, v);
}

template <int kBlock>
__global__ __launch_bounds__(kBlock) void copy_kernel(u32x4* dst, const u32x4* src, uint64_t n_vec)
{
    const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n_vec) store_stream(dst + i, __builtin_nontemporal_load(src + i));
}

bool shape_ok(int threads) { return threads == 64 || threads == 128 || threads == 512; }
bool aligned(const void* p, size_t bytes) { return ((uintptr_t)p & 15) == 0 && (bytes & 15) == 0 && bytes > 0 && bytes <= ((size_t)1 << 40); }

}  // namespace

extern "C" {

// All three: device pointers, 16-byte aligned, `bytes` a multiple of 16, `threads` (per workgroup) 64, 128 or 512; enqueue on
// `stream` and return at once.  Return 0, or -1 for bad arguments, -2 when the launch was refused.
int membench_read(const void* src, size_t bytes, void* sink, int threads, void* stream)
{
    if (!src || !sink || !aligned(src, bytes) || !shape_ok(threads)) return -1;
    const uint64_t n_vec = bytes / 16;
    constexpr int UNROLL = 4;
    const uint64_t blocks = (n_vec + (uint64_t)threads * UNROLL - 1) / ((uint64_t)threads * UNROLL);
    if (blocks > 0x7fffffffull) return -1;
    if (threads == 64)
        hipLaunchKernelGGL((read_kernel<64, UNROLL>), dim3((unsigned)blocks), dim3(64), 0, (hipStream_t)stream,
                           (const u32x4*)src, n_vec, (uint32_t*)sink);
    else if (threads == 128)
        hipLaunchKernelGGL((read_kernel<128, UNROLL>), dim3((unsigned)blocks), dim3(128), 0, (hipStream_t)stream,
                           (const u32x4*)src, n_vec, (uint32_t*)sink);
    else
        hipLaunchKernelGGL((read_kernel<512, UNROLL>), dim3((unsigned)blocks), dim3(512), 0, (hipStream_t)stream,
                           (const u32x4*)src, n_vec, (uint32_t*)sink);
    return hipGetLastError() == hipSuccess ? 0 : -2;
}

int membench_write(void* dst, size_t bytes, int threads, void* stream)
{
    if (!dst || !aligned(dst, bytes) || !shape_ok(threads)) return -1;
    const uint64_t n_vec = bytes / 16;
    const uint64_t blocks = (n_vec + threads - 1) / threads;
    if (blocks > 0x7fffffffull) return -1;
    if (threads == 64)
        hipLaunchKernelGGL(write_kernel<64>, dim3((unsigned)blocks), dim3(64), 0, (hipStream_t)stream, (u32x4*)dst, n_vec, 0x01020304u);
    else if (threads == 128)
        hipLaunchKernelGGL(write_kernel<128>, dim3((unsigned)blocks), dim3(128), 0, (hipStream_t)stream, (u32x4*)dst, n_vec, 0x01020304u);
    else
        hipLaunchKernelGGL(write_kernel<512>, dim3((unsigned)blocks), dim3(512), 0, (hipStream_t)stream, (u32x4*)dst, n_vec, 0x01020304u);
    return hipGetLastError() == hipSuccess ? 0 : -2;
}

int membench_copy(void* dst, const void* src, size_t bytes, int threads, void* stream)
{
    if (!dst || !src || !aligned(dst, bytes) || !aligned(src, bytes) || !shape_ok(threads)) return -1;
    const uint64_t n_vec = bytes / 16;
    const uint64_t blocks = (n_vec + threads - 1) / threads;
    if (blocks > 0x7fffffffull) return -1;
    if (threads == 64)
        hipLaunchKernelGGL(copy_kernel<64>, dim3((unsigned)blocks), dim3(64), 0, (hipStream_t)stream, (u32x4*)dst, (const u32x4*)src, n_vec);
    else if (threads == 128)
        hipLaunchKernelGGL(copy_kernel<128>, dim3((unsigned)blocks), dim3(128), 0, (hipStream_t)stream, (u32x4*)dst, (const u32x4*)src, n_vec);
    else
        hipLaunchKernelGGL(copy_kernel<512>, dim3((unsigned)blocks), dim3(512), 0, (hipStream_t)stream, (u32x4*)dst, (const u32x4*)src, n_vec);
    return hipGetLastError() == hipSuccess ? 0 : -2;
}

}  // extern "C"
