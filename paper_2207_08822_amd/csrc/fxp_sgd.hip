// int16 weight update (paper Remark 5 and App. A.4: w_hat_{k+1} = w_hat_k + alpha_hat_k * g_hat, every term
// in fixed point, stochastic rounding).  The building block is one fixed-point "a times y plus x":
//   z = x_hat + SR(a_hat * y_hat)
// with x_hat, y_hat, a_hat the 16-bit instance of the mapping of Sec. 3.1 (15 magnitude bits: the 24-bit
// mantissa rounded with its low 9 bits), the product exact in int32 on the unit 2^(Ea + Ey), brought to the
// unit of x_hat by an integer shift (stochastic rounding of the magnitude when it is a right shift:
// up  <=>  word < floor(dropped * 2^32 / 2^s)), added in integer and sent through the inverse mapping of
// Sec. 3.2.  The paper leaves the alignment and the place of the rounding open; this is the reading the CPU
// oracle of this repository takes as well.  An SGD step with weight decay and momentum is three such lines.
//
// One kernel per line: 8 B read + 4 B written per element, two Philox blocks per four elements.  The
// scales of x and y arrive as block maxima (the kernel finishes the reduction, like the map kernel does), and
// the kernel leaves the block maxima of z behind, so a chain of lines needs no scale pass for intermediates.
#include "fxp_internal.h"

namespace fxp {

constexpr int kAxpyThreads = 256;
template <bool V>
struct IC {
    static constexpr bool value = V;
};
// streams (step << 8) | tag: x and y of one element round with bits 31..23 and 22..14 of ONE word of the
// operand stream, the update with a full word of its own stream, the scalar with word 0 of a third
constexpr uint32_t kTagAxpyXY = 3, kTagAxpyU = 4, kTagAxpyA = 5;
constexpr uint32_t kUpdateSat = (1u << 23) - (1u << 15);   // keeps x_hat + u an exact fp32 mantissa

// signed 16-bit fixed-point value of the float with bit pattern b on the scale e_max, every case;
// r9 = the 9-bit random number
template <bool STOCH>
__device__ inline int map16_full(uint32_t b, uint32_t r9, int e_max) {
    const uint32_t e = (b >> 23) & 0xffu, f = b & 0x7fffffu;
    uint32_t q;
    if (e == 255u) {
        q = f == 0u ? 32767u : 0u;                        // Inf saturates, NaN maps to 0
    } else {
        const int d = e_max - static_cast<int>(max(e, 1u));
        if (d < 0) {
            q = 32767u;
        } else {
            const uint32_t m = f | (e ? 0x800000u : 0u);
            const uint32_t ms = d >= 24 ? 0u : m >> d;
            q = STOCH ? (ms >> 9) + ((r9 < (ms & 511u)) ? 1u : 0u) : (ms + 256u) >> 9;
            q = min(q, 32767u);
        }
    }
    return (b >> 31) ? -static_cast<int>(q) : static_cast<int>(q);
}

// The same without branches for a finite element at or below the scale: the shifted mantissa m >> (e_max - e) is
// the integer part of |x| * 2^(150 - e_max) (an exact scaling by a power of two, sub-normal inputs included,
// then a truncating conversion), and the round-up is the carry of low + (511 - r9) out of the 9 dropped bits.
// `bad` collects, as a lane mask, the lanes holding an element the scale does not cover (exponent above it, Inf,
// NaN: everything that is not below `limit` = 2^(e_max - 126)); the caller redoes those quads with map16_full.
template <bool STOCH>
__device__ inline int map16_fast(uint32_t b, uint32_t r9, int to_units, float limit, uint64_t& bad) {
    const float ax = fabsf(__uint_as_float(b));
    bad |= __builtin_amdgcn_ballot_w64(!(ax < limit));
    const uint32_t ms = static_cast<uint32_t>(ldexpf(ax, to_units));
    const uint32_t q = min((ms + (STOCH ? (r9 ^ 511u) : 256u)) >> 9, 32767u);
    return (b >> 31) ? -static_cast<int>(q) : static_cast<int>(q);
}

// How the int32 product (unit 2^(Ea+Ey)) reaches the unit of x_hat, s = Ex - (Ea + Ey); all wave-uniform.
struct Align {
    int left;        // s <= 0: shift left by this much (24 = anything non-zero saturates)
    int right;       // 0 < s < 32: bits kept are m >> right; 32 when nothing is kept
    uint32_t mask;   // dropped bits of m
    int thr_left;    // threshold = dropped << thr_left   (s <= 32)
    int thr_right;   // threshold = dropped >> thr_right  (s > 32; 31 with mask 0 when s >= 63)
    int half;        // round-half-up: bit s-1 of m (31 = none)
};

__device__ inline Align make_align(int s) {
    Align a;
    a.left = s <= 0 ? min(-s, 24) : -1;
    a.right = s >= 32 ? 32 : max(s, 0);
    a.mask = s <= 0 ? 0u : (s >= 63 ? 0u : (s >= 32 ? 0xffffffffu : (1u << s) - 1u));
    a.thr_left = s <= 32 ? 32 - max(s, 1) : 0;
    a.thr_right = s > 32 ? min(s - 32, 31) : 0;
    a.half = (s >= 1 && s <= 31) ? s - 1 : 31;
    return a;
}

template <bool STOCH>
__device__ inline int update_on_grid(int p, const Align& a, uint32_t word) {
    const uint32_t m = static_cast<uint32_t>(p < 0 ? -p : p);     // < 2^30: bit 31 of m is never set
    uint32_t u;
    if (a.left >= 0) {
        u = a.left >= 24 ? (m ? kUpdateSat : 0u) : static_cast<uint32_t>(min<uint64_t>(static_cast<uint64_t>(m) << a.left, kUpdateSat));
    } else {
        const uint32_t dropped = m & a.mask;
        const uint32_t kept = a.right >= 32 ? 0u : m >> a.right;
        const uint32_t up = STOCH ? (word < ((dropped << a.thr_left) >> a.thr_right) ? 1u : 0u) : (m >> a.half) & 1u;
        u = min(kept + up, kUpdateSat);
    }
    return p < 0 ? -static_cast<int>(u) : static_cast<int>(u);
}

// one element, every case (tails, unaligned tensors, quads that hold a special value)
template <bool STOCH>
__device__ inline float axpy_one(uint32_t xb, uint32_t yb, uint32_t wxy, uint32_t wu, int ex, int ey, int a_hat,
                                 const Align& al, int Ex) {
    const int xh = map16_full<STOCH>(xb, wxy >> 23, ex);
    const int yh = map16_full<STOCH>(yb, (wxy >> 14) & 511u, ey);
    return unmap_value(xh + update_on_grid<STOCH>(a_hat * yh, al, wu), Ex);
}

__device__ inline uint32_t word_of(const uint4& r, uint32_t k) { return k == 0 ? r.x : k == 1 ? r.y : k == 2 ? r.z : r.w; }

// VEC: x, y, z are 16-byte aligned; a thread owns whole quads of four consecutive elements (16-byte loads and
// stores, both Philox blocks of the quad used in full) and block 0 finishes the n % 4 tail.  Otherwise one
// element per thread and iteration.
// Workgroup `bid` of the `nblocks` that share one line over one tensor.
template <bool STOCH, bool VEC>
__device__ __attribute__((always_inline)) inline void axpy16_body(const uint32_t* x, const uint32_t* y, uint32_t a_bits,
                                                                  uint64_t n, float* z, const uint32_t* __restrict__ px,
                                                                  int npx, const uint32_t* __restrict__ py, int npy,
                                                                  uint32_t* __restrict__ pz, int32_t* __restrict__ e_out,
                                                                  uint32_t key0, uint32_t key1, uint64_t step, unsigned bid,
                                                                  unsigned nblocks, uint32_t* red) {
    // scales of the two tensors from their block maxima, the scalar's from its own exponent
    uint32_t mx = 0, my = 0;
    for (int i = threadIdx.x; i < npx; i += kAxpyThreads) mx = max(mx, px[i]);
    for (int i = threadIdx.x; i < npy; i += kAxpyThreads) my = max(my, py[i]);
    // readfirstlane: the maxima are the same in every lane; as scalars, everything derived from them (shift
    // amounts, the alignment case, the range test of the inverse mapping) stays wave-uniform for the compiler
    const int ex = __builtin_amdgcn_readfirstlane(max(1, static_cast<int>(block_max(mx, red) >> 23)));
    const int ey = __builtin_amdgcn_readfirstlane(max(1, static_cast<int>(block_max(my, red) >> 23)));
    const int ea = max(1, static_cast<int>((a_bits >> 23) & 0xffu));
    if (e_out != nullptr && bid == 0 && threadIdx.x == 0) {
        e_out[0] = ex;
        e_out[1] = ey;
        e_out[2] = ea;
    }
    const uint32_t sid_hi = static_cast<uint32_t>(step >> 24);          // stream id = (step << 8) | tag
    const uint32_t sid_xy = static_cast<uint32_t>(step << 8) | kTagAxpyXY, sid_u = static_cast<uint32_t>(step << 8) | kTagAxpyU;
    const uint32_t wa = STOCH ? philox4x32_10(0u, 0u, static_cast<uint32_t>(step << 8) | kTagAxpyA, sid_hi, key0, key1).x : 0u;
    const int a_hat = map16_full<STOCH>(a_bits, wa >> 23, ea);
    const int Ex = lsb_exponent(ex, 16);
    const Align al = make_align(Ex - (lsb_exponent(ea, 16) + lsb_exponent(ey, 16)));
    auto blocks_of = [&](uint64_t q, uint4& rxy, uint4& ru) {
        rxy = ru = make_uint4(0, 0, 0, 0);
        if (STOCH) {
            rxy = philox4x32_10(static_cast<uint32_t>(q), static_cast<uint32_t>(q >> 32), sid_xy, sid_hi, key0, key1);
            ru = philox4x32_10(static_cast<uint32_t>(q), static_cast<uint32_t>(q >> 32), sid_u, sid_hi, key0, key1);
        }
    };

    uint32_t zmax = 0;
    const uint64_t stride = static_cast<uint64_t>(nblocks) * kAxpyThreads;
    const uint64_t first = static_cast<uint64_t>(bid) * kAxpyThreads + threadIdx.x;
    if (VEC) {
        const uint64_t quads = n >> 2;
        const uint4* xv = reinterpret_cast<const uint4*>(x);
        const uint4* yv = reinterpret_cast<const uint4*>(y);
        float4* zv = reinterpret_cast<float4*>(z);
        // The loop over whole quads, once for the usual alignment (the product sits 1..31 bits below the unit
        // of x_hat and 2^Ex is a normal float: straight-line 32-bit code) and once for every other case; the
        // choice is made here, outside the loop.
        auto quad_loop = [&](auto usual_c) __attribute__((always_inline)) {
            constexpr bool USUAL = decltype(usual_c)::value;
            const int sh = al.right;                                   // USUAL: 1..31
            const float unit = __uint_as_float(static_cast<uint32_t>(Ex + 127) << 23);
            // scale 255 (a non-finite element somewhere): the limit becomes -0 and every quad takes the full path
            const int ux = 150 - ex, uy = 150 - ey;
            const float limx = __uint_as_float(static_cast<uint32_t>(ex + 1) << 23);
            const float limy = __uint_as_float(static_cast<uint32_t>(ey + 1) << 23);
            uint4 xc = make_uint4(0, 0, 0, 0), yc = xc, xn = xc, yn = xc;
            if (first < quads) {
                xc = xv[first];
                yc = yv[first];
            }
            for (uint64_t q = first; q < quads; q += stride) {
                const uint64_t qn = min(q + stride, quads - 1);   // clamped: the last prefetch is simply not used
                xn = xv[qn];
                yn = yv[qn];
                uint4 rxy, ru;
                blocks_of(q, rxy, ru);
                const uint32_t xb[4] = {xc.x, xc.y, xc.z, xc.w}, yb[4] = {yc.x, yc.y, yc.z, yc.w};
                const uint32_t wxy[4] = {rxy.x, rxy.y, rxy.z, rxy.w}, wu[4] = {ru.x, ru.y, ru.z, ru.w};
                uint64_t bad = 0;                                      // wave-uniform lane mask
                float zf[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int xh = map16_fast<STOCH>(xb[k], wxy[k] >> 23, ux, limx, bad);
                    const int yh = map16_fast<STOCH>(yb[k], (wxy[k] >> 14) & 511u, uy, limy, bad);
                    const int p = a_hat * yh;
                    if (USUAL) {
                        const uint32_t m = static_cast<uint32_t>(p < 0 ? -p : p);
                        const uint32_t up = STOCH ? (wu[k] < ((m & al.mask) << al.thr_left) ? 1u : 0u) : (m >> al.half) & 1u;
                        const int u = static_cast<int>(min((m >> sh) + up, kUpdateSat));
                        zf[k] = static_cast<float>(xh + (p < 0 ? -u : u)) * unit;
                    } else {
                        zf[k] = unmap_value(xh + update_on_grid<STOCH>(p, al, wu[k]), Ex);
                    }
                }
                if (bad != 0) {               // rare: a non-finite element (or one above a scale) in this wave's quads
#pragma unroll
                    for (int k = 0; k < 4; ++k) zf[k] = axpy_one<STOCH>(xb[k], yb[k], wxy[k], wu[k], ex, ey, a_hat, al, Ex);
                }
                zv[q] = make_float4(zf[0], zf[1], zf[2], zf[3]);
                zmax = max(max(zmax, __float_as_uint(zf[0]) & 0x7fffffffu),
                           max(max(__float_as_uint(zf[1]) & 0x7fffffffu, __float_as_uint(zf[2]) & 0x7fffffffu),
                               __float_as_uint(zf[3]) & 0x7fffffffu));
                xc = xn;
                yc = yn;
            }
        };
        if (al.left < 0 && al.right < 32 && Ex >= -126 && Ex <= 127) quad_loop(IC<true>{});
        else quad_loop(IC<false>{});
        const uint32_t tail = static_cast<uint32_t>(n & 3u);
        if (bid == 0 && threadIdx.x < tail) {
            uint4 rxy, ru;
            blocks_of(quads, rxy, ru);
            const uint64_t i = (quads << 2) + threadIdx.x;
            const float zf = axpy_one<STOCH>(x[i], y[i], word_of(rxy, threadIdx.x), word_of(ru, threadIdx.x), ex, ey, a_hat, al, Ex);
            z[i] = zf;
            zmax = max(zmax, __float_as_uint(zf) & 0x7fffffffu);
        }
    } else {
        for (uint64_t i = first; i < n; i += stride) {
            uint4 rxy, ru;
            blocks_of(i >> 2, rxy, ru);
            const uint32_t k = static_cast<uint32_t>(i & 3u);
            const float zf = axpy_one<STOCH>(x[i], y[i], word_of(rxy, k), word_of(ru, k), ex, ey, a_hat, al, Ex);
            z[i] = zf;
            zmax = max(zmax, __float_as_uint(zf) & 0x7fffffffu);
        }
    }
    zmax = block_max(zmax, red);
    if (pz != nullptr && threadIdx.x == 0) pz[bid] = zmax;
}

template <bool STOCH, bool VEC>
__global__ __launch_bounds__(kAxpyThreads) void k_axpy16(const uint32_t* x, const uint32_t* y, uint32_t a_bits, uint64_t n,
                                                         float* z, const uint32_t* __restrict__ px, int npx,
                                                         const uint32_t* __restrict__ py, int npy,
                                                         uint32_t* __restrict__ pz, int32_t* __restrict__ e_out,
                                                         uint32_t key0, uint32_t key1, uint64_t step) {
    __shared__ uint32_t red[kAxpyThreads / 64];
    axpy16_body<STOCH, VEC>(x, y, a_bits, n, z, px, npx, py, npy, pz, e_out, key0, key1, step, blockIdx.x, gridDim.x, red);
}

// ---- many parameter tensors per launch ------------------------------------------------------------------
// Up to kMaxJobs tensors travel in the kernel argument segment.  Tensor t owns workgroups
// [block0, block0 + blocks) of every launch of a step and the same range of each block-maxima array, so a
// line finds the scales of its operands (and leaves those of its result) without any launch in between.
constexpr int kMaxJobs = 64;
struct SgdJob {
    float* w;
    const float* g;
    float* v;
    float* tmp;
    uint64_t n;
    uint32_t block0, blocks;
    uint32_t index;      // position of the tensor in the caller's list: part of its random-stream id
};
struct SgdJobs {
    SgdJob j[kMaxJobs];
    int count;
};

__device__ inline int job_of_block(const SgdJobs& jobs, unsigned b) {   // last job whose block0 <= b
    int lo = 0, hi = jobs.count - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (jobs.j[mid].block0 <= b) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

// block maxima of w, g and (blockIdx.y == 2) v of every tensor
__global__ __launch_bounds__(kScaleThreads) void k_absmax_multi(const SgdJobs jobs, uint32_t* __restrict__ pw,
                                                                uint32_t* __restrict__ pg, uint32_t* __restrict__ pv) {
    __shared__ uint32_t lds[kScaleThreads / 64];
    const SgdJob& J = jobs.j[job_of_block(jobs, blockIdx.x)];
    const float* x = blockIdx.y == 0 ? J.w : (blockIdx.y == 1 ? J.g : J.v);
    uint32_t* p = blockIdx.y == 0 ? pw : (blockIdx.y == 1 ? pg : pv);
    absmax_body(reinterpret_cast<const uint32_t*>(x), J.n, p + J.block0, blockIdx.x - J.block0, J.blocks, lds);
}

// one line of the step for every tensor: line 0: tmp = g + wd w; 1: v = x1 + momentum v; 2: w = w + (-lr) d, where
// x1 is tmp when line 0 ran, else g, and d is v when line 1 ran, else x1.  px / py: block maxima of x / y; pz: of z.
template <bool STOCH>
__global__ __launch_bounds__(kAxpyThreads) void k_axpy16_multi(const SgdJobs jobs, int line, int have_wd, int have_mom,
                                                               uint32_t a_bits, const uint32_t* __restrict__ px,
                                                               const uint32_t* __restrict__ py, uint32_t* __restrict__ pz,
                                                               uint32_t key0, uint32_t key1, uint64_t step) {
    __shared__ uint32_t red[kAxpyThreads / 64];
    const int t = job_of_block(jobs, blockIdx.x);
    const SgdJob& J = jobs.j[t];
    const float* x1 = have_wd ? J.tmp : J.g;
    const float* x = line == 0 ? J.g : (line == 1 ? x1 : J.w);
    const float* y = line == 0 ? J.w : (line == 1 ? J.v : (have_mom ? J.v : x1));
    float* z = line == 0 ? J.tmp : (line == 1 ? J.v : J.w);
    // the random streams of tensor t: those of a single-tensor step with step (step << 16) | t, three lines each
    const uint64_t line_step = 3 * ((step << 16) | static_cast<uint64_t>(J.index)) + line;
    const bool vec = ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(y) | reinterpret_cast<uintptr_t>(z)) & 15u) == 0;
    const unsigned bid = blockIdx.x - J.block0;
    const uint32_t* xb = reinterpret_cast<const uint32_t*>(x);
    const uint32_t* yb = reinterpret_cast<const uint32_t*>(y);
    uint32_t* pzt = pz ? pz + J.block0 : nullptr;
    if (vec)
        axpy16_body<STOCH, true>(xb, yb, a_bits, J.n, z, px + J.block0, J.blocks, py + J.block0, J.blocks, pzt, nullptr, key0, key1,
                                 line_step, bid, J.blocks, red);
    else
        axpy16_body<STOCH, false>(xb, yb, a_bits, J.n, z, px + J.block0, J.blocks, py + J.block0, J.blocks, pzt, nullptr, key0, key1,
                                  line_step, bid, J.blocks, red);
}

// grid of one line over n elements: at most kAxpyBlocks workgroups (three per CU: 0.1104 -> 0.1066 ms per step
// of 11.7 M parameters against 1024; 512: 0.107, 384: 0.122 - the kernel is bound by VALU issue and needs the
// waves, the memory system prefers fewer requests in flight); pz fits a scale scratch area (kMaxPartials words)
constexpr int kAxpyBlocks = 768;
static_assert(kAxpyBlocks <= kMaxPartials, "block maxima of z go to a scale scratch area");
static int axpy_grid(uint64_t n) {
    const uint64_t want = (((n + 3) >> 2) + kAxpyThreads - 1) / kAxpyThreads;
    return static_cast<int>(want < 1 ? 1 : (want > kAxpyBlocks ? kAxpyBlocks : want));
}

// one line; px / py: block maxima of x / y (npx / npy of them); pz receives axpy_grid(n) block maxima of z
static int axpy16_launch(const float* x, const float* y, float a, uint64_t n, float* z, const uint32_t* px, int npx,
                         const uint32_t* py, int npy, uint32_t* pz, int32_t* e_out, uint64_t seed, uint64_t step,
                         int rounding, hipStream_t s) {
    uint32_t a_bits;
    __builtin_memcpy(&a_bits, &a, sizeof a_bits);
    const bool vec = aligned(x, 16) && aligned(y, 16) && aligned(z, 16);
    const dim3 grid(axpy_grid(n)), block(kAxpyThreads);
    const uint32_t k0 = static_cast<uint32_t>(seed), k1 = static_cast<uint32_t>(seed >> 32);
    const uint32_t* xb = reinterpret_cast<const uint32_t*>(x);
    const uint32_t* yb = reinterpret_cast<const uint32_t*>(y);
#define FXP_AXPY_LAUNCH(STOCH, VEC) \
    hipLaunchKernelGGL((k_axpy16<STOCH, VEC>), grid, block, 0, s, xb, yb, a_bits, n, z, px, npx, py, npy, pz, e_out, k0, k1, step)
    if (rounding == FXP_ROUND_STOCHASTIC) {
        if (vec) FXP_AXPY_LAUNCH(true, true);
        else FXP_AXPY_LAUNCH(true, false);
    } else {
        if (vec) FXP_AXPY_LAUNCH(false, true);
        else FXP_AXPY_LAUNCH(false, false);
    }
#undef FXP_AXPY_LAUNCH
    return launch_status();
}

static int check_common(size_t n, int rounding, const void* ws, size_t ws_bytes, size_t need) {
    if (n >= (size_t{1} << 40)) return FXP_ERR_DIMS;
    if (rounding != FXP_ROUND_STOCHASTIC && rounding != FXP_ROUND_NEAREST) return FXP_ERR_ROUNDING;
    if (!ws || ws_bytes < need) return FXP_ERR_WORKSPACE;
    if (!aligned(ws, 4)) return FXP_ERR_ALIGN;
    return FXP_OK;
}

}  // namespace fxp

extern "C" size_t fxp_sgd16_workspace_bytes(void) { return 5 * fxp::kScaleWsBytes; }

extern "C" int fxp_axpy16(const float* x, const float* y, float a, size_t n, float* z, int32_t* e_out, uint64_t seed,
                          uint64_t step, int rounding, void* ws, size_t ws_bytes, void* stream) {
    using namespace fxp;
    int rc = check_common(n, rounding, ws, ws_bytes, 2 * kScaleWsBytes);
    if (rc) return rc;
    if (n == 0) return FXP_OK;
    if (!x || !y || !z) return FXP_ERR_NULL;
    if (!aligned(x, 4) || !aligned(y, 4) || !aligned(z, 4) || !aligned(e_out, 4)) return FXP_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t* px = static_cast<uint32_t*>(ws);
    uint32_t* py = px + kMaxPartials;
    int npx = 0, npy = 0;
    if ((rc = scale_partials(x, n, px, &npx, s))) return rc;
    if ((rc = scale_partials(y, n, py, &npy, s))) return rc;
    return axpy16_launch(x, y, a, n, z, px, npx, py, npy, nullptr, e_out, seed, step, rounding, s);
}

extern "C" int fxp_sgd16_step(float* w, const float* g, float* v, size_t n, float lr, float momentum, float weight_decay,
                              float* tmp, uint64_t seed, uint64_t step, int rounding, void* ws, size_t ws_bytes,
                              void* stream) {
    using namespace fxp;
    int rc = check_common(n, rounding, ws, ws_bytes, fxp_sgd16_workspace_bytes());
    if (rc) return rc;
    if (step >= (uint64_t{1} << 54)) return FXP_ERR_DIMS;        // three stream steps per optimiser step
    if (n == 0) return FXP_OK;
    if (!w || !g || (momentum != 0.0f && !v) || (weight_decay != 0.0f && !tmp)) return FXP_ERR_NULL;
    if (!aligned(w, 4) || !aligned(g, 4) || !aligned(v, 4) || !aligned(tmp, 4)) return FXP_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t* pw = static_cast<uint32_t*>(ws);
    uint32_t* pg = pw + kMaxPartials;
    uint32_t* pv = pg + kMaxPartials;
    uint32_t* pt = pv + kMaxPartials;     // block maxima of g1 = g + wd * w
    uint32_t* pn = pt + kMaxPartials;     // block maxima of the new v
    int npw = 0, npg = 0, npv = 0;
    const int npz = axpy_grid(n);
    if ((rc = scale_partials(w, n, pw, &npw, s))) return rc;
    if ((rc = scale_partials(g, n, pg, &npg, s))) return rc;
    const float* g1 = g;
    const uint32_t* pg1 = pg;
    int npg1 = npg;
    if (weight_decay != 0.0f) {           // g1 = g + wd * w
        if ((rc = axpy16_launch(g, w, weight_decay, n, tmp, pg, npg, pw, npw, pt, nullptr, seed, 3 * step, rounding, s)))
            return rc;
        g1 = tmp; pg1 = pt; npg1 = npz;
    }
    const float* d = g1;
    const uint32_t* pd = pg1;
    int npd = npg1;
    if (momentum != 0.0f) {               // v = g1 + momentum * v
        if ((rc = scale_partials(v, n, pv, &npv, s))) return rc;
        if ((rc = axpy16_launch(g1, v, momentum, n, v, pg1, npg1, pv, npv, pn, nullptr, seed, 3 * step + 1, rounding, s)))
            return rc;
        d = v; pd = pn; npd = npz;
    }
    // w = w + (-lr) * d
    return axpy16_launch(w, d, -lr, n, w, pw, npw, pd, npd, nullptr, nullptr, seed, 3 * step + 2, rounding, s);
}

namespace fxp {
// workgroups of one tensor in every launch of a multi-tensor step: eight quads or more per thread (6: slower, 12 and
// 16: the same, 24: slower), at most 1024
static uint32_t multi_blocks(size_t n) {
    const uint64_t want = (((static_cast<uint64_t>(n) + 3) >> 2) + kAxpyThreads * 8 - 1) / (kAxpyThreads * 8);
    return static_cast<uint32_t>(want < 1 ? 1 : (want > 1024 ? 1024 : want));
}
}  // namespace fxp

extern "C" size_t fxp_sgd16_multi_workspace_bytes(const fxp_sgd_tensor* tensors, size_t count) {
    if (!tensors) return 0;
    size_t blocks = 0;
    for (size_t t = 0; t < count; ++t)
        if (tensors[t].n) blocks += fxp::multi_blocks(tensors[t].n);
    return 5 * sizeof(uint32_t) * (blocks ? blocks : 1);
}

extern "C" int fxp_sgd16_step_multi(const fxp_sgd_tensor* tensors, size_t count, float lr, float momentum, float weight_decay,
                                    uint64_t seed, uint64_t step, int rounding, void* ws, size_t ws_bytes, void* stream) {
    using namespace fxp;
    if (count > 65536 || step >= (uint64_t{1} << 32)) return FXP_ERR_DIMS;
    if (rounding != FXP_ROUND_STOCHASTIC && rounding != FXP_ROUND_NEAREST) return FXP_ERR_ROUNDING;
    if (count == 0) return FXP_OK;
    if (!tensors) return FXP_ERR_NULL;
    const bool have_wd = weight_decay != 0.0f, have_mom = momentum != 0.0f;
    size_t total_blocks = 0;
    for (size_t t = 0; t < count; ++t) {
        const fxp_sgd_tensor& T = tensors[t];
        if (T.n >= (size_t{1} << 40)) return FXP_ERR_DIMS;
        if (T.n == 0) continue;
        if (!T.w || !T.g || (have_mom && !T.v) || (have_wd && !T.tmp)) return FXP_ERR_NULL;
        if (!aligned(T.w, 4) || !aligned(T.g, 4) || !aligned(T.v, 4) || !aligned(T.tmp, 4)) return FXP_ERR_ALIGN;
        total_blocks += multi_blocks(T.n);
    }
    if (total_blocks == 0) return FXP_OK;
    if (!ws || ws_bytes < 5 * sizeof(uint32_t) * total_blocks) return FXP_ERR_WORKSPACE;
    if (!aligned(ws, 4)) return FXP_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t* pw = static_cast<uint32_t*>(ws);       // block maxima of w, g, v, g1 = g + wd w, and the new v
    uint32_t* pg = pw + total_blocks;
    uint32_t* pv = pg + total_blocks;
    uint32_t* pt = pv + total_blocks;
    uint32_t* pn = pt + total_blocks;
    const uint32_t k0 = static_cast<uint32_t>(seed), k1 = static_cast<uint32_t>(seed >> 32);
    auto bits_of = [](float a) {
        uint32_t b;
        __builtin_memcpy(&b, &a, sizeof b);
        return b;
    };
    size_t t = 0, block_base = 0;                    // block_base: offset of this launch group in the maxima arrays
    while (t < count) {
        SgdJobs jobs;
        jobs.count = 0;
        uint32_t blocks = 0;
        for (; t < count && jobs.count < kMaxJobs; ++t) {
            const fxp_sgd_tensor& T = tensors[t];
            if (T.n == 0) continue;
            SgdJob& J = jobs.j[jobs.count++];
            J.w = T.w; J.g = T.g; J.v = T.v; J.tmp = T.tmp; J.n = T.n;
            J.block0 = blocks;
            J.blocks = multi_blocks(T.n);
            J.index = static_cast<uint32_t>(t);
            blocks += J.blocks;
        }
        if (jobs.count == 0) break;
        uint32_t* w_ = pw + block_base; uint32_t* g_ = pg + block_base; uint32_t* v_ = pv + block_base;
        uint32_t* t_ = pt + block_base; uint32_t* n_ = pn + block_base;
        hipLaunchKernelGGL(k_absmax_multi, dim3(blocks, have_mom ? 3 : 2), dim3(kScaleThreads), 0, s, jobs, w_, g_, v_);
        int rc = launch_status();
        if (rc) return rc;
#define FXP_LINE(LINE, A, PX, PY, PZ)                                                                                      \
    do {                                                                                                                   \
        if (rounding == FXP_ROUND_STOCHASTIC)                                                                              \
            hipLaunchKernelGGL(k_axpy16_multi<true>, dim3(blocks), dim3(kAxpyThreads), 0, s, jobs, LINE, int(have_wd),      \
                               int(have_mom), bits_of(A), PX, PY, PZ, k0, k1, step);                                        \
        else                                                                                                               \
            hipLaunchKernelGGL(k_axpy16_multi<false>, dim3(blocks), dim3(kAxpyThreads), 0, s, jobs, LINE, int(have_wd),     \
                               int(have_mom), bits_of(A), PX, PY, PZ, k0, k1, step);                                        \
        if ((rc = launch_status())) return rc;                                                                             \
    } while (0)
        const uint32_t* x1 = have_wd ? t_ : g_;
        if (have_wd) FXP_LINE(0, weight_decay, g_, w_, t_);
        if (have_mom) FXP_LINE(1, momentum, x1, v_, n_);
        FXP_LINE(2, -lr, w_, (have_mom ? n_ : x1), static_cast<uint32_t*>(nullptr));
#undef FXP_LINE
        block_base += blocks;
    }
    return FXP_OK;
}
