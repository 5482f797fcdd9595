// Test helper (host only): prints Philox4x32-10 output blocks computed by
// rocRAND's own engine (AMD's published implementation), as an external
// reference for the oracle's generator.  Input lines: "seed subsequence offset"
// (decimal, unsigned 64-bit); output: four hex words per line.  With offset a
// multiple of 4 the engine's counter is (lo32(offset/4), hi32(offset/4),
// lo32(subsequence), hi32(subsequence)) and its key (lo32(seed), hi32(seed)).
#include <hip/hip_runtime.h>
#include <rocrand/rocrand_philox4x32_10.h>
#include <cstdio>

int main()
{
    unsigned long long seed, sub, off;
    while (std::scanf("%llu %llu %llu", &seed, &sub, &off) == 3) {
        rocrand_device::philox4x32_10_engine eng(seed, sub, off);
        uint4 r = eng.next4();
        std::printf("%08x %08x %08x %08x\n", r.x, r.y, r.z, r.w);
    }
    return 0;
}
