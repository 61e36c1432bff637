// Internal declarations shared by the HIP translation units of libfxp.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "../../include/fxp.h"

namespace fxp {

constexpr int kMaxPartials = 1024;        // capacity of a block-maxima scratch area (uint32 each)
// Workgroups of a scale reduction: one per CU, four 16-byte loads in flight per thread.  More requests in flight
// make the reduction slower, not faster (8192^3 layer, the step's two reductions over 805 MB: 147 us with 1024
// workgroups, 124 with two loads per thread, 115-117 with 256 workgroups x 4 loads, 512 x 2 or 1024 x 1 = 6.9 TB/s;
// 215 us with 256 x 1).
constexpr int kScaleBlocks = 256;
constexpr int kScaleThreads = 256;
constexpr size_t kScaleWsBytes = kMaxPartials * sizeof(uint32_t);
constexpr int64_t kMaxContraction = 133144;   // 127^2 * K < 2^31: the longest contraction one int32 sum can hold
// Longer contractions (a weight gradient over more rows than that) run as slices of at most kMaxSlice terms (a
// multiple of every K step), each summed exactly in int32 into its workspace slice; the slices are added in 64
// bits and the inverse mapping rounds that sum once.
constexpr int64_t kMaxSlice = 133120;

inline int launch_status() { return hipGetLastError() == hipSuccess ? FXP_OK : FXP_ERR_LAUNCH; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Launchers used by the layer composition (all enqueue on `s`, arguments already validated).
int scale_partials(const float* x, size_t n, uint32_t* partials, int* n_partials, hipStream_t s);
// the same for two tensors in one launch
int scale_partials2(const float* x0, size_t n0, uint32_t* partials0, int* n_partials0, const float* x1, size_t n1,
                    uint32_t* partials1, int* n_partials1, hipStream_t s);
int scale_finish(const uint32_t* partials, int n_partials, int32_t* e_max, hipStream_t s);
int scale_partial_count(size_t n);     // block maxima a reduction over n elements leaves (<= kScaleBlocks)

// One tensor to map: x[rows, cols] fp32 -> q (row-major) and / or qT (transposed), either may be null.  The
// scale comes from e_in (device) or, when partials is given, from the block maxima of a scale reduction, in
// which case the kernel finishes the reduction and publishes the scale to e_out.
struct MapTensor {
    const float* x;
    int64_t rows, cols;
    const int32_t* e_in;
    const uint32_t* partials;
    int n_partials;
    int32_t* e_out;
    int8_t* q;
    int8_t* qT;
    uint64_t stream_id;
};
int map_launch(const MapTensor& t, uint64_t seed, int rounding, int bits, hipStream_t s);
// scale + map in one pass with the previous scale as a guess (fxp_map.hip)
constexpr unsigned kGuessBlocks = 1008;            // workgroups of a guessing launch: their maxima and the guess fit one scratch area
constexpr int64_t kGuessMinElements = int64_t{1} << 22;
constexpr int kNoGuessPath = 2;
constexpr int kGuessOneByOne = 3;
int scale_map_guess_launch(const MapTensor& a, const MapTensor* b, uint32_t* area_a, uint32_t* area_b, uint64_t seed,
                           int rounding, int bits, hipStream_t s);
int map_launch2(const MapTensor& a, const MapTensor& b, uint64_t seed, int rounding, int bits, hipStream_t s);
int gemm_nt_batched_launch(int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda, int64_t strideA,
                           const int8_t* B, int64_t ldb, int64_t strideB, void* C, int64_t ldc, int64_t strideC,
                           int64_t batch, bool fp32_out, const int32_t* eA, int bitsA, const int32_t* eB, int bitsB,
                           hipStream_t s);
// The reduction that finishes a product split along K (sum of its int32 slices, inverse mapping), as a piece of
// work that can ride in the launch of ANOTHER product: `blocks` workgroups of that launch's grid.x do it instead
// of a tile.  A dependent launch costs about 4.5 us on this machine and the reduction is a few microseconds of
// reading, so the backward pass sends the weight gradient's reduction along with the input-gradient product.
// Where the product has several rounds of tiles the riders are its FIRST workgroups (they run beside the first
// round; as the last ones they were a tail of their own: ResNet layer 0.116 -> 0.110 ms); where its tiles leave
// CUs idle (150 tiles of 256 x 256 in the ViT layers) they are the LAST ones and run on the idle CUs at once - a
// rider occupies a whole workgroup slot of the product's kernel, so in front they would hold the tiles back.
// blocks = 0: nothing rides.
struct ReduceRider {
    const int32_t* parts = nullptr;
    int splits = 0;
    int64_t stride = 0;
    int M = 0, N = 0;
    void* C = nullptr;
    int64_t ldc = 0;
    int fp32_out = 0;
    const int32_t* eA = nullptr;
    int bitsA = 8;
    const int32_t* eB = nullptr;
    int bitsB = 8;
    uint32_t* amax = nullptr;
    int wide = 0;            // the contraction is longer than kMaxContraction: the slices are added in 64 bits
    unsigned blocks = 0;
    unsigned tiles = 0;      // set by the launcher: workgroups of the host product
    bool front = false;      // set by the launcher: riders before the tiles
};

int gemm_nt_launch(int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                   void* C, int64_t ldc, bool fp32_out, const int32_t* eA, int bitsA, const int32_t* eB, int bitsB,
                   void* ws, size_t ws_bytes, hipStream_t s, uint32_t* amax = nullptr, ReduceRider* ride = nullptr,
                   ReduceRider* defer = nullptr);
size_t gemm_split_ws_bytes(int64_t M, int64_t N, int64_t K);
// geometry of the patches an implicit-convolution GEMM reads: image H x W x C (channels-last), filter width
// KW, stride, padding (rows / columns), output Ho x Wo
struct ConvTaps {
    int H = 0, W = 0, C = 1, KW = 1, stride = 1, pad = 0, padw = 0, Ho = 1, Wo = 1;
};
constexpr int kNotApplicable = 1;
int conv_gemm_launch(const ConvTaps& ct, int KH, int64_t M, int64_t Cout, const int8_t* Xq, const int8_t* Wq, float* Y,
                     const int32_t* eA, int bitsA, const int32_t* eB, int bitsB, hipStream_t s, ReduceRider* ride = nullptr);
int splitk_reduce_launch(const ReduceRider& r, hipStream_t s);
size_t gemm_ws_worst(int64_t M, int64_t N, int64_t K);
int transpose_i8_launch(const int8_t* src, int64_t rows, int64_t cols, int64_t ld, int8_t* dst, hipStream_t s);

// max over the 64 lanes of a wave, the same value in every lane.  Data-parallel-primitive moves inside the
// vector ALU (within quads, within rows of 16, then row to row) instead of six round trips through the LDS
// crossbar; the total arrives in lane 63 and is read from there.
__device__ inline uint32_t wave_max(uint32_t v) {
    auto step = [](uint32_t x, auto ctrl, auto rows) {
        const int t = __builtin_amdgcn_update_dpp(static_cast<int>(x), static_cast<int>(x), decltype(ctrl)::value,
                                                  decltype(rows)::value, 0xf, false);
        return max(x, static_cast<uint32_t>(t));
    };
    using std::integral_constant;
    v = step(v, integral_constant<int, 0xB1>{}, integral_constant<int, 0xf>{});     // quad_perm [1,0,3,2]
    v = step(v, integral_constant<int, 0x4E>{}, integral_constant<int, 0xf>{});     // quad_perm [2,3,0,1]
    v = step(v, integral_constant<int, 0x141>{}, integral_constant<int, 0xf>{});    // row_half_mirror
    v = step(v, integral_constant<int, 0x140>{}, integral_constant<int, 0xf>{});    // row_mirror: every row of 16 done
    v = step(v, integral_constant<int, 0x142>{}, integral_constant<int, 0xa>{});    // row_bcast:15 into rows 1 and 3
    v = step(v, integral_constant<int, 0x143>{}, integral_constant<int, 0xc>{});    // row_bcast:31 into rows 2 and 3
    return static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(v), 63));
}

// max over a block of up to 1024 threads; lds holds blockDim.x / 64 words
__device__ inline uint32_t block_max(uint32_t v, uint32_t* lds) {
    v = wave_max(v);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = blockDim.x >> 6;
    if (lane == 0) lds[wave] = v;
    __syncthreads();
    uint32_t r = (lane < nw) ? lds[lane] : 0u;
    r = wave_max(r);
    __syncthreads();
    return r;
}

__device__ inline uint32_t absmax4(const uint4 v) {
    const uint32_t kAbs = 0x7fffffffu;
    return max(max(v.x & kAbs, v.y & kAbs), max(v.z & kAbs, v.w & kAbs));
}

// block maxima of one tensor: block `bid` of `nblocks`
__device__ inline void absmax_body(const uint32_t* __restrict__ x, size_t n, uint32_t* __restrict__ partials, unsigned bid,
                                   unsigned nblocks, uint32_t* lds) {
    const uint32_t kAbs = 0x7fffffffu;
    uint32_t m = 0;
    // scalar head up to 16-byte alignment, vector body, scalar tail
    const size_t mis = (reinterpret_cast<uintptr_t>(x) >> 2) & 3u;
    size_t head = mis ? 4 - mis : 0;
    if (head > n) head = n;
    const size_t nvec = (n - head) >> 2;
    const uint4* xv = reinterpret_cast<const uint4*>(x + head);
    const size_t tid = static_cast<size_t>(bid) * kScaleThreads + threadIdx.x;
    const size_t stride = static_cast<size_t>(nblocks) * kScaleThreads;
    // back to front: the map kernel that follows reads front to back, and what the last-level cache still
    // holds of a tensor near its size is what was read last here
    const uint4* xe = xv + nvec - 1;
    size_t i = tid;
    for (; i + 3 * stride < nvec; i += 4 * stride) {
        const uint4 a = *(xe - i), b = *(xe - (i + stride)), c = *(xe - (i + 2 * stride)), d = *(xe - (i + 3 * stride));
        m = max(max(m, absmax4(a)), max(absmax4(b), max(absmax4(c), absmax4(d))));
    }
    for (; i < nvec; i += stride) m = max(m, absmax4(*(xe - i)));
    if (bid == 0) {
        if (threadIdx.x < head) m = max(m, x[threadIdx.x] & kAbs);
        const size_t tail0 = head + (nvec << 2);
        if (tail0 + threadIdx.x < n) m = max(m, x[tail0 + threadIdx.x] & kAbs);
    }
    m = block_max(m, lds);
    if (threadIdx.x == 0) partials[bid] = m;
}

// byte permute: every byte of the result is byte (sel & 7) of the pair {hi, lo} (0-3 = lo, 4-7 = hi)
__device__ inline uint32_t perm(uint32_t hi, uint32_t lo, uint32_t sel) { return __builtin_amdgcn_perm(hi, lo, sel); }

// 4 x 4 byte transpose: o[r] holds columns 0..3 of row r; t[c] receives rows 0..3 of column c
__device__ inline void transpose4x4(const uint32_t (&o)[4], uint32_t (&t)[4]) {
    const uint32_t a = perm(o[1], o[0], 0x05010400u), b = perm(o[1], o[0], 0x07030602u);   // rows 0,1: columns 0,1 | 2,3
    const uint32_t c = perm(o[3], o[2], 0x05010400u), d = perm(o[3], o[2], 0x07030602u);   // rows 2,3
    t[0] = perm(c, a, 0x05040100u);
    t[1] = perm(c, a, 0x07060302u);
    t[2] = perm(d, b, 0x05040100u);
    t[3] = perm(d, b, 0x07060302u);
}

// Philox-4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): counter (c0..c3), key (k0, k1), ten rounds of two
// 32x32->64 multiplies with the Weyl key schedule.  Element i of a tensor stream uses word i % 4 of the
// block with counter (i / 4, stream id) and key = seed.
// a ^ b ^ c in one instruction (three-input bit operation with the parity truth table); the compiler
// leaves two v_xor_b32 when one input is wave-uniform, and the map kernels spend most of their VALU issue slots in these rounds
__device__ inline uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) { return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96); }

__device__ inline uint4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = static_cast<uint64_t>(0xD2511F53u) * c0;
        const uint64_t p1 = static_cast<uint64_t>(0xCD9E8D57u) * c2;
        const uint32_t n0 = xor3(static_cast<uint32_t>(p1 >> 32), c1, k0 + 0x9E3779B9u * r);
        const uint32_t n2 = xor3(static_cast<uint32_t>(p0 >> 32), c3, k1 + 0xBB67AE85u * r);
        c1 = static_cast<uint32_t>(p1);
        c3 = static_cast<uint32_t>(p0);
        c0 = n0;
        c2 = n2;
    }
    return make_uint4(c0, c1, c2, c3);
}

// scale + map of one tensor: block maxima, then the map kernel finishes the reduction and publishes *e
inline int scale_and_map(const float* x, int64_t rows, int64_t cols, int32_t* e, int8_t* q, int8_t* qT, uint64_t seed,
                         uint64_t sid, int rounding, int bits, uint32_t* partials, hipStream_t s) {
    int np = 0;
    int rc = scale_partials(x, static_cast<size_t>(rows * cols), partials, &np, s);
    if (rc) return rc;
    const MapTensor t{x, rows, cols, nullptr, partials, np, e, q, qT, sid};
    return map_launch(t, seed, rounding, bits, s);
}

// Scale + map of two tensors (the two operands of a forward pass) in two launches instead of four: one
// reduction launch and one map launch cover both.  t.partials must point at kMaxPartials words each; e_in and
// n_partials of the arguments are ignored.
inline int scale_and_map2(MapTensor a, MapTensor b, uint64_t seed, int rounding, int bits, hipStream_t s) {
    int rc = scale_partials2(a.x, static_cast<size_t>(a.rows * a.cols), const_cast<uint32_t*>(a.partials), &a.n_partials, b.x,
                             static_cast<size_t>(b.rows * b.cols), const_cast<uint32_t*>(b.partials), &b.n_partials, s);
    if (rc) return rc;
    a.e_in = b.e_in = nullptr;
    return map_launch2(a, b, seed, rounding, bits, s);
}


// exponent of one unit of a mapped tensor
__host__ __device__ inline int lsb_exponent(int e_max, int bits) { return e_max - 127 - (bits - 2); }

// fp32 nearest (ties to even, gradual underflow, overflow to Inf) to acc * 2^E: the
// inverse mapping of Sec. 3.2.  v_cvt_f32_i32 rounds the integer once to 24 bits; the
// power-of-two factor is exact whenever it is a normal float (then the product is
// normal or overflows, both as IEEE prescribes).  Outside that range one exact double
// carries the value to a single f64->f32 rounding.
__device__ inline float unmap_value(int acc, int E) {
    if (E >= -126 && E <= 127) {
        return static_cast<float>(acc) * __uint_as_float(static_cast<uint32_t>(E + 127) << 23);
    }
    return static_cast<float>(ldexp(static_cast<double>(acc), E));
}

// the same for a sum of slices that needs more than 32 bits (|acc| < 2^53: the conversion to double is exact, and
// so is the scaling; one rounding, double -> float)
__device__ inline float unmap_value64(int64_t acc, int E) { return static_cast<float>(ldexp(static_cast<double>(acc), E)); }

}  // namespace fxp
