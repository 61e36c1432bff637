// Scale of a tensor: e_max = max_i e_i (paper Sec. 3.1).
//
// The exponent field is monotone in the magnitude bits, so the reduction is an
// unsigned integer max over (bits & 0x7fffffff); the field of the winner is the
// scale.  Two kernels: every block leaves the max of its grid-stride share in
// `partials`; a single block (or the map kernel, which folds this step) reduces
// those.  HBM-bound: 4 bytes read per element, 16-byte loads, no writes.
#include "fxp_internal.h"

namespace fxp {

__device__ inline uint32_t absmax4(const uint4 v) {
    const uint32_t kAbs = 0x7fffffffu;
    return max(max(v.x & kAbs, v.y & kAbs), max(v.z & kAbs, v.w & kAbs));
}

__global__ __launch_bounds__(kScaleThreads) void k_absmax_partials(const uint32_t* __restrict__ x, size_t n,
                                                                   uint32_t* __restrict__ partials) {
    __shared__ uint32_t lds[kScaleThreads / 64];
    const uint32_t kAbs = 0x7fffffffu;
    uint32_t m = 0;
    // scalar head up to 16-byte alignment, vector body, scalar tail
    const size_t mis = (reinterpret_cast<uintptr_t>(x) >> 2) & 3u;
    size_t head = mis ? 4 - mis : 0;
    if (head > n) head = n;
    const size_t nvec = (n - head) >> 2;
    const uint4* xv = reinterpret_cast<const uint4*>(x + head);
    const size_t tid = static_cast<size_t>(blockIdx.x) * kScaleThreads + threadIdx.x;
    const size_t stride = static_cast<size_t>(gridDim.x) * kScaleThreads;
    size_t i = tid;
    for (; i + 3 * stride < nvec; i += 4 * stride) {
        const uint4 a = xv[i], b = xv[i + stride], c = xv[i + 2 * stride], d = xv[i + 3 * stride];
        m = max(max(m, absmax4(a)), max(absmax4(b), max(absmax4(c), absmax4(d))));
    }
    for (; i < nvec; i += stride) m = max(m, absmax4(xv[i]));
    if (blockIdx.x == 0) {
        if (threadIdx.x < head) m = max(m, x[threadIdx.x] & kAbs);
        const size_t tail0 = head + (nvec << 2);
        if (tail0 + threadIdx.x < n) m = max(m, x[tail0 + threadIdx.x] & kAbs);
    }
    m = block_max(m, lds);
    if (threadIdx.x == 0) partials[blockIdx.x] = m;
}

__global__ __launch_bounds__(kScaleThreads) void k_absmax_finish(const uint32_t* __restrict__ partials, int count,
                                                                 int32_t* __restrict__ e_max) {
    __shared__ uint32_t lds[kScaleThreads / 64];
    uint32_t m = 0;
    for (int i = threadIdx.x; i < count; i += kScaleThreads) m = max(m, partials[i]);
    m = block_max(m, lds);
    if (threadIdx.x == 0) e_max[0] = max(1, static_cast<int>(m >> 23));
}

int scale_partials(const float* x, size_t n, uint32_t* partials, int* n_partials, hipStream_t s) {
    // 16K elements or more per block (the map kernel re-reads every block maximum), at most kMaxPartials
    size_t want = (n + 16383) / 16384;
    int grid = static_cast<int>(want < 1 ? 1 : (want > kMaxPartials ? kMaxPartials : want));
    hipLaunchKernelGGL(k_absmax_partials, dim3(grid), dim3(kScaleThreads), 0, s, reinterpret_cast<const uint32_t*>(x),
                       n, partials);
    *n_partials = grid;
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
