// Prints Philox4x32-10 blocks from rocRAND's own host-callable engine, for pinning the
// CPU oracle's generator against an independent library implementation.
// usage: rocrand_philox_host <seed> <subsequence> <first_counter> <count>
// Each output line: the four 32-bit words of the block whose 128-bit counter is
// (first_counter + i) in the low 64 bits and <subsequence> in the high 64 bits.
#include <hip/hip_runtime.h>
#include <rocrand/rocrand_philox4x32_10.h>
#include <cstdio>
#include <cstdlib>

int main(int argc, char** argv)
{
    if(argc != 5) return 2;
    unsigned long long seed  = strtoull(argv[1], nullptr, 0);
    unsigned long long subs  = strtoull(argv[2], nullptr, 0);
    unsigned long long first = strtoull(argv[3], nullptr, 0);
    unsigned long long count = strtoull(argv[4], nullptr, 0);
    for(unsigned long long i = 0; i < count; ++i)
    {
        // the engine's offset counts 32-bit outputs, four per block
        rocrand_device::philox4x32_10_engine eng(seed, subs, 4ull * (first + i));
        unsigned int a = eng.next(), b = eng.next(), c = eng.next(), d = eng.next();
        std::printf("%u %u %u %u\n", a, b, c, d);
    }
    return 0;
}
