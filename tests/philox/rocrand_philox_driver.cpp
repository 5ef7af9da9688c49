// Test infrastructure (CPU only): prints Philox4x32-10 output blocks computed by the engine that ships in ROCm's
// rocRAND headers, which is callable from host code.  tests/test_oracle_philox_library.py compares the oracle's own
// generator (used by the RandomLLM baseline, paper Sec. 4.1) against it.  No GPU call is made.
//
// stdin: lines "seed subsequence block" (unsigned 64-bit decimals).  The engine seeded with (seed, subsequence,
// offset = 4 * block) returns as its next four numbers the output block of
//     counter = {block low word, block high word, subsequence low word, subsequence high word},
//     key     = {seed low word, seed high word}
// (rocRAND's documented state layout: an offset skips single numbers, four to a block; a subsequence advances the
// upper half of the counter).  stdout: the four words in hexadecimal, one block per line.
#include <hip/hip_runtime.h>
#include <rocrand/rocrand_philox4x32_10.h>

#include <cstdio>

int main()
{
    unsigned long long seed, subsequence, block;
    while (std::scanf("%llu %llu %llu", &seed, &subsequence, &block) == 3) {
        if (block >= (1ull << 62)) return 2;               // 4 * block must fit the 64-bit offset
        rocrand_device::philox4x32_10_engine engine(seed, subsequence, 4ull * block);
        const uint4 r = engine.next4();
        std::printf("%08x %08x %08x %08x\n", r.x, r.y, r.z, r.w);
    }
    return 0;
}
