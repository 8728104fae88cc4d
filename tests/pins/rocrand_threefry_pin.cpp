// Test-only pin: exposes rocRAND's host-callable Threefry-2x32-20 engine (a third-party
// implementation of the published generator) through a C function, so the oracle's own block
// function can be checked against an independent implementation on the CPU.
// Not linked into the product or the oracle.
#include <hip/hip_runtime.h>
#include <rocrand/rocrand_threefry2x32_20.h>

extern "C" void pin_rocrand_threefry2x32_20(unsigned long long seed, unsigned long long subsequence,
                                            unsigned long long offset, int n, unsigned int* out)
{
    rocrand_state_threefry2x32_20 st;
    rocrand_init(seed, subsequence, offset, &st);
    for (int i = 0; i < n; ++i) out[i] = rocrand(&st);
}
