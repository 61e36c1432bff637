// Non-linear inverse mapping (paper Sec. 3.2, Fig. 1b) as a standalone streaming
// kernel: integer mantissas + one shared exponent (the sum of the operand exponents,
// Sec. 3.3) -> rounded, normalised, packed fp32.  The GEMM epilogue does the same in
// registers; this kernel serves int32 results that already sit in memory and mapped
// int8 tensors.  HBM-bound: 8 B (int32) or 5 B (int8) per element.
#include "fxp_internal.h"

namespace fxp {

__global__ __launch_bounds__(256) void k_unmap_i32(const int32_t* acc, size_t n, const int32_t* __restrict__ eA,
                                                   int bitsA, const int32_t* __restrict__ eB, int bitsB, float* out) {
    // acc and out may alias element-wise (each thread reads its elements before writing them)
    const int E = lsb_exponent(eA[0], bitsA) + (eB ? lsb_exponent(eB[0], bitsB) : 0);
    const size_t stride = static_cast<size_t>(gridDim.x) * 256;
    const size_t tid = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
    const bool vec = ((reinterpret_cast<uintptr_t>(acc) | reinterpret_cast<uintptr_t>(out)) & 15u) == 0;
    const size_t nvec = vec ? n >> 2 : 0;
    for (size_t i = tid; i < nvec; i += stride) {
        const int4 a = reinterpret_cast<const int4*>(acc)[i];
        float4 o;
        o.x = unmap_value(a.x, E);
        o.y = unmap_value(a.y, E);
        o.z = unmap_value(a.z, E);
        o.w = unmap_value(a.w, E);
        reinterpret_cast<float4*>(out)[i] = o;
    }
    for (size_t i = (nvec << 2) + tid; i < n; i += stride) out[i] = unmap_value(acc[i], E);
}

__global__ __launch_bounds__(256) void k_unmap_i8(const int8_t* __restrict__ q, size_t n, const int32_t* __restrict__ eA,
                                                  int bitsA, float* __restrict__ out) {
    const int E = lsb_exponent(eA[0], bitsA);
    const size_t stride = static_cast<size_t>(gridDim.x) * 256;
    for (size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x; i < n; i += stride)
        out[i] = unmap_value(static_cast<int>(q[i]), E);
}

static unsigned grid_for(size_t n, size_t per_thread) {
    size_t want = (n + 256 * per_thread - 1) / (256 * per_thread);
    return static_cast<unsigned>(want < 1 ? 1 : (want > 8192 ? 8192 : want));
}

}  // namespace fxp

extern "C" int fxp_unmap(const int32_t* acc, size_t n, const int32_t* eA, int bitsA, const int32_t* eB, int bitsB,
                         float* out, void* stream) {
    if (!eA || (n && (!acc || !out))) return FXP_ERR_NULL;
    if (bitsA < 2 || bitsA > 8 || (eB && (bitsB < 2 || bitsB > 8))) return FXP_ERR_BITS;
    if (!fxp::aligned(acc, 4) || !fxp::aligned(out, 4)) return FXP_ERR_ALIGN;
    if (n == 0) return FXP_OK;
    hipLaunchKernelGGL(fxp::k_unmap_i32, dim3(fxp::grid_for(n, 4)), dim3(256), 0, static_cast<hipStream_t>(stream), acc,
                       n, eA, bitsA, eB, bitsB, out);
    return fxp::launch_status();
}

extern "C" int fxp_unmap_i8(const int8_t* q, size_t n, const int32_t* eA, int bitsA, float* out, void* stream) {
    if (!eA || (n && (!q || !out))) return FXP_ERR_NULL;
    if (bitsA < 2 || bitsA > 8) return FXP_ERR_BITS;
    if (!fxp::aligned(out, 4)) return FXP_ERR_ALIGN;
    if (n == 0) return FXP_OK;
    hipLaunchKernelGGL(fxp::k_unmap_i8, dim3(fxp::grid_for(n, 1)), dim3(256), 0, static_cast<hipStream_t>(stream), q, n,
                       eA, bitsA, out);
    return fxp::launch_status();
}
