// Prints rocRAND's Philox4x32-10 output words for given (seed, counter) tuples,
// running the vendor header's engine on the host.  Used only to pin the oracle's
// generator against a library routine; no GPU is touched.
// stdin: lines "seed c0 c1 c2 c3" (decimal);  stdout: four words per line.
#include <hip/hip_runtime.h>
#include <rocrand/rocrand_philox4x32_10.h>
#include <cstdio>
int main() {
    unsigned long long seed, c0, c1, c2, c3;
    while (std::scanf("%llu %llu %llu %llu %llu", &seed, &c0, &c1, &c2, &c3) == 5) {
        rocrand_state_philox4x32_10 st;
        // subsequence -> high 64 counter bits, offset/4 -> low 64 counter bits
        rocrand_init(seed, (c3 << 32) | c2, 4ULL * ((c1 << 32) | c0), &st);
        uint4 r = rocrand4(&st);
        std::printf("%u %u %u %u\n", r.x, r.y, r.z, r.w);
    }
    return 0;
}
