// Measurement helper, not a step of the method: the core clock the chip actually runs at while other kernels are
// busy.  One wave reads the shader-clock counter and the constant 100 MHz counter, sleeps until `ticks` ticks of
// the latter have passed (or an iteration cap is reached, so the wave always ends), and reads both again.
// Launched on a stream of its own next to the kernel under test, the ratio of the two differences is that
// kernel's core clock: the compute-bound products run the chip into its board power limit, and their
// throughput has to be read against the clock they get.
#include "fxp_internal.h"

namespace fxp {

__global__ __launch_bounds__(64) void k_clock_probe(unsigned long long* __restrict__ out, unsigned long long ticks) {
    if (threadIdx.x != 0) return;
    const unsigned long long t0 = wall_clock64(), c0 = clock64();
    unsigned long long t1 = t0;
    for (int i = 0; i < (1 << 22) && t1 - t0 < ticks; ++i) {       // one iteration sleeps about 2000 core cycles
        __builtin_amdgcn_s_sleep(32);
        t1 = wall_clock64();
    }
    const unsigned long long c1 = clock64();
    out[0] = t1 - t0;      // ticks of the constant 100 MHz counter
    out[1] = c1 - c0;      // core clock cycles in the same interval
}

}  // namespace fxp

extern "C" int fxp_clock_probe(uint64_t* out, uint32_t microseconds, void* stream) {
    if (!out) return FXP_ERR_NULL;
    if (!fxp::aligned(out, 8)) return FXP_ERR_ALIGN;
    if (microseconds == 0 || microseconds > 1000000u) return FXP_ERR_DIMS;
    hipLaunchKernelGGL(fxp::k_clock_probe, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream),
                       reinterpret_cast<unsigned long long*>(out), static_cast<unsigned long long>(microseconds) * 100ull);
    return fxp::launch_status();
}
