// Host-only witness for the Philox4x32-10 pins: it asks rocRAND's open-source
// engine (a library routine independent of both the oracle and the GPU kernels)
// for the four words at a given (seed, subsequence, offset) and prints them.
// Reads lines "seed subsequence offset" from stdin, numbers in C syntax.
#include <hip/hip_runtime.h>
#include <rocrand/rocrand_philox4x32_10.h>
#include <cstdio>
#include <cstdlib>

int main()
{
    char a[64], b[64], c[64];
    while (std::scanf("%63s %63s %63s", a, b, c) == 3) {
        unsigned long long seed = std::strtoull(a, nullptr, 0);
        unsigned long long sub = std::strtoull(b, nullptr, 0);
        unsigned long long off = std::strtoull(c, nullptr, 0);
        rocrand_state_philox4x32_10 st;
        rocrand_init(seed, sub, off, &st);
        uint4 r = rocrand4(&st);
        std::printf("%08x %08x %08x %08x\n", r.x, r.y, r.z, r.w);
    }
    return 0;
}
