// Test helper only: exposes AMD rocRAND's host-callable Philox4x32-10 engine so
// that the oracle's raw stream can be pinned against an independent
// implementation.  Not part of the product and not part of the oracle.
#include <hip/hip_runtime.h>
#include <rocrand/rocrand_philox4x32_10.h>
#include <stdint.h>

extern "C" void rocrand_ref_philox_block(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                         uint32_t k0, uint32_t k1, uint32_t* out)
{
    // engine(seed, subsequence, offset): key = seed, counter = (offset/4, subsequence);
    // c1 must stay below 2^30 so that 4*(c0 | c1<<32) fits 64 bits.
    unsigned long long seed = (unsigned long long)k0 | ((unsigned long long)k1 << 32);
    unsigned long long subseq = (unsigned long long)c2 | ((unsigned long long)c3 << 32);
    unsigned long long block = (unsigned long long)c0 | ((unsigned long long)c1 << 32);
    rocrand_device::philox4x32_10_engine e(seed, subseq, block * 4ull);
    uint4 r = e.next4();
    out[0] = r.x; out[1] = r.y; out[2] = r.z; out[3] = r.w;
}
