// Scale of a tensor: e_max = max_i e_i (paper Sec. 3.1).
//
// The exponent field is monotone in the magnitude bits, so the reduction is an
// unsigned integer max over (bits & 0x7fffffff); the field of the winner is the
// scale.  Two kernels: every block leaves the max of its grid-stride share in
// `partials`; a single block (or the map kernel, which folds this step) reduces
// those.  HBM-bound: 4 bytes read per element, 16-byte loads, no writes.
#include "fxp_internal.h"

namespace fxp {


// Up to two tensors per launch: the first blocks0 workgroups reduce tensor 0, the others tensor 1.
__global__ __launch_bounds__(kScaleThreads) void k_absmax_partials(const uint32_t* __restrict__ x0, size_t n0,
                                                                   uint32_t* __restrict__ partials0, unsigned blocks0,
                                                                   const uint32_t* __restrict__ x1, size_t n1,
                                                                   uint32_t* __restrict__ partials1) {
    __shared__ uint32_t lds[kScaleThreads / 64];
    if (blockIdx.x < blocks0) absmax_body(x0, n0, partials0, blockIdx.x, blocks0, lds);
    else absmax_body(x1, n1, partials1, blockIdx.x - blocks0, gridDim.x - blocks0, lds);
}

__global__ __launch_bounds__(kScaleThreads) void k_absmax_finish(const uint32_t* __restrict__ partials, int count,
                                                                 int32_t* __restrict__ e_max) {
    __shared__ uint32_t lds[kScaleThreads / 64];
    uint32_t m = 0;
    for (int i = threadIdx.x; i < count; i += kScaleThreads) m = max(m, partials[i]);
    m = block_max(m, lds);
    if (threadIdx.x == 0) e_max[0] = max(1, static_cast<int>(m >> 23));
}

// 16K elements or more per block (the map kernel re-reads every block maximum), at most kScaleBlocks
int scale_partial_count(size_t n) {
    const size_t want = (n + 16383) / 16384;
    return static_cast<int>(want < 1 ? 1 : (want > kScaleBlocks ? kScaleBlocks : want));
}

int scale_partials(const float* x, size_t n, uint32_t* partials, int* n_partials, hipStream_t s) {
    const int grid = scale_partial_count(n);
    hipLaunchKernelGGL(k_absmax_partials, dim3(grid), dim3(kScaleThreads), 0, s, reinterpret_cast<const uint32_t*>(x), n,
                       partials, static_cast<unsigned>(grid), static_cast<const uint32_t*>(nullptr), size_t{0},
                       static_cast<uint32_t*>(nullptr));
    *n_partials = grid;
    return launch_status();
}

int scale_partials2(const float* x0, size_t n0, uint32_t* partials0, int* n_partials0, const float* x1, size_t n1,
                    uint32_t* partials1, int* n_partials1, hipStream_t s) {
    const int g0 = scale_partial_count(n0), g1 = scale_partial_count(n1);
    hipLaunchKernelGGL(k_absmax_partials, dim3(g0 + g1), dim3(kScaleThreads), 0, s, reinterpret_cast<const uint32_t*>(x0),
                       n0, partials0, static_cast<unsigned>(g0), reinterpret_cast<const uint32_t*>(x1), n1, partials1);
    *n_partials0 = g0;
    *n_partials1 = g1;
    return launch_status();
}

int scale_finish(const uint32_t* partials, int n_partials, int32_t* e_max, hipStream_t s) {
    hipLaunchKernelGGL(k_absmax_finish, dim3(1), dim3(kScaleThreads), 0, s, partials, n_partials, e_max);
    return launch_status();
}

}  // namespace fxp

extern "C" int fxp_scale(const float* x, size_t n, int32_t* e_max, void* ws, size_t ws_bytes, void* stream) {
    if (!e_max || (n && !x)) return FXP_ERR_NULL;
    if (!ws || ws_bytes < fxp::kScaleWsBytes) return FXP_ERR_WORKSPACE;
    if (!fxp::aligned(x, 4) || !fxp::aligned(e_max, 4) || !fxp::aligned(ws, 4)) return FXP_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int np = 0;
    int rc = fxp::scale_partials(x, n, static_cast<uint32_t*>(ws), &np, s);
    if (rc) return rc;
    return fxp::scale_finish(static_cast<const uint32_t*>(ws), np, e_max, s);
}
