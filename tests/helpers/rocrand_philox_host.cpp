// Test helper: the i-th 32-bit output of rocRAND's Philox4x32-10 engine for a
// given (seed, subsequence, offset), computed on the HOST through rocRAND's
// public header (its engine functions are host-callable).  It is an independent
// implementation of the published generator, used to cross-check the oracle's
// own Philox; it launches no GPU work.
#include <hip/hip_runtime.h>
#include <rocrand/rocrand_philox4x32_10.h>

extern "C" void rocrand_philox_words(unsigned long long seed, unsigned long long subsequence,
                                     unsigned long long offset, unsigned int* out, int n) {
    rocrand_state_philox4x32_10 st;
    rocrand_init(seed, subsequence, offset, &st);
    for (int i = 0; i < n; ++i) out[i] = rocrand(&st);
}
