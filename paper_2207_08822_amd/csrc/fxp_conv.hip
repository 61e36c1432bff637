// Integer convolution layer (paper Sec. 3.4: convolution layers are the same integer inner
// products as linear layers), channels-last, as an explicit int8 im2col around the GEMM kernels:
//   forward : scale+map X[N,H,W,C] ONCE (9x fewer fp32 bytes than mapping a 3x3 patch matrix),
//             scale+map W[Cout,KH,KW,C] (both orientations), int8 im2col -> col[M,K],
//             Y[M,Cout] = unmap(col * Wq^T)                         M = N*Ho*Wo, K = KH*KW*C
//   backward: scale+map dY[M,Cout] once (both orientations),
//             dW[Cout,K] = unmap(dYqT * colT^T) with colT[K,M] rebuilt from the saved int8 X,
//             dX: for stride 1 it is itself a convolution - im2col of dYq (padded by K-1-pad) times the
//             flipped weights WqF, inverse mapping fused in the GEMM; for other strides
//             dcol[M,K] = dYq * Wq (int32) and dX = unmap(col2im(dcol)) as a gather: every input
//             pixel sums the <= KH*KW patch entries that read it, so no atomics are needed.
// The saved state of a layer is the int8 activation itself (1 byte per element), not its patches.
#include <algorithm>

#include "fxp_internal.h"

namespace fxp {

struct ConvGeo {
    int N, H, W, C, Cout, KH, KW, stride, pad, padw, Ho, Wo;   // pad: rows, padw: columns
    __host__ __device__ int64_t M() const { return static_cast<int64_t>(N) * Ho * Wo; }
    __host__ __device__ int64_t K() const { return static_cast<int64_t>(KH) * KW * C; }
};

// col[m][(kh*KW + kw)*C + c] = X[n, ho*stride + kh - pad, wo*stride + kw - pad, c] (0 outside);
// one thread moves VEC bytes (16 when C % 16 == 0, else 1)
// top-left input coordinate of output pixel m and the offset of that pixel in X (may point outside
// the image: callers add the tap and test the bounds)
struct PatchRow {
    int h0, w0;
    int64_t base;   // ((n*H + h0)*W + w0)*C
};

__device__ inline PatchRow patch_row(const ConvGeo& g, uint32_t m) {
    const uint32_t t = m / static_cast<uint32_t>(g.Wo);
    const int wo = static_cast<int>(m - t * g.Wo);
    const uint32_t n = t / static_cast<uint32_t>(g.Ho);
    const int ho = static_cast<int>(t - n * g.Ho);
    PatchRow r;
    r.h0 = ho * g.stride - g.pad;
    r.w0 = wo * g.stride - g.padw;
    r.base = ((static_cast<int64_t>(n) * g.H + r.h0) * g.W + r.w0) * g.C;
    return r;
}

template <int VEC>
__global__ __launch_bounds__(256) void k_im2col_i8(const int8_t* __restrict__ Xq, ConvGeo g, int8_t* __restrict__ col) {
    // A block copies 32 consecutive patch rows.  Their pixel coordinates are worked out once (LDS table);
    // a thread then owns one (tap, channel vector) column of the patch matrix and every RSTEP-th row, so
    // the copy loop has no division.
    __shared__ PatchRow rows[32];
    const uint32_t cv = g.C / VEC;                               // vectors per pixel
    const uint32_t per_row = static_cast<uint32_t>(g.KH * g.KW) * cv;
    const uint32_t M = static_cast<uint32_t>(g.M()), m_first = blockIdx.x * 32u;
    const uint32_t rows_here = min(32u, M - m_first);
    const int64_t K = g.K();
    if (threadIdx.x < rows_here) rows[threadIdx.x] = patch_row(g, m_first + threadIdx.x);
    __syncthreads();
    const uint32_t cols_par = min(per_row, 256u);                // columns handled side by side
    const uint32_t rstep = 256u / cols_par;                      // rows handled side by side
    const uint32_t r_first = threadIdx.x / cols_par, lane_col = threadIdx.x - r_first * cols_par;
    if (r_first >= rstep) return;
    for (uint32_t colv = lane_col; colv < per_row; colv += cols_par) {
        const uint32_t tap = colv / cv, c = (colv - tap * cv) * VEC;
        const int kh = static_cast<int>(tap) / g.KW, kw = static_cast<int>(tap) - kh * g.KW;
        const int64_t tap_off = (static_cast<int64_t>(kh) * g.W + kw) * g.C + c;
        for (uint32_t r = r_first; r < rows_here; r += rstep) {
            const PatchRow pr = rows[r];
            const int h = pr.h0 + kh, w = pr.w0 + kw;
            const bool inside = h >= 0 && h < g.H && w >= 0 && w < g.W;
            int8_t* dst = col + (m_first + r) * K + static_cast<int64_t>(tap) * g.C + c;
            if (VEC == 16) {
                *reinterpret_cast<uint4*>(dst) = inside ? *reinterpret_cast<const uint4*>(Xq + pr.base + tap_off) : make_uint4(0, 0, 0, 0);
            } else {
                *dst = inside ? Xq[pr.base + tap_off] : static_cast<int8_t>(0);
            }
        }
    }
}

// WqF[c][(kh', kw', co)] = Wq[co][(KH-1-kh', KW-1-kw', c)]: the weights of the stride-1 input-gradient
// convolution (the upstream gradient correlated with the flipped kernel), contraction-contiguous
__device__ inline void flip_weights_body(const int8_t* __restrict__ Wq, const ConvGeo& g, int8_t* __restrict__ WqF, unsigned bid,
                                         unsigned nblocks) {
    const int64_t K = g.K(), Kf = static_cast<int64_t>(g.KH) * g.KW * g.Cout, total = static_cast<int64_t>(g.C) * Kf;
    for (int64_t id = static_cast<int64_t>(bid) * 256 + threadIdx.x; id < total; id += static_cast<int64_t>(nblocks) * 256) {
        const int c = static_cast<int>(id / Kf);
        const int rem = static_cast<int>(id - c * Kf);
        const int tap = rem / g.Cout, co = rem - tap * g.Cout;
        const int kh = tap / g.KW, kw = tap - kh * g.KW;
        WqF[id] = Wq[co * K + static_cast<int64_t>((g.KH - 1 - kh) * g.KW + (g.KW - 1 - kw)) * g.C + c];
    }
}

__global__ __launch_bounds__(256) void k_flip_weights_i8(const int8_t* __restrict__ Wq, ConvGeo g, int8_t* __restrict__ WqF) {
    flip_weights_body(Wq, g, WqF, blockIdx.x, gridDim.x);
}

// The launch that writes the transposed patches carries two more pieces of the backward pass that depend on
// nothing it writes: its first side.blocks workgroups reduce the block maxima of the incoming gradient (the
// scale reduction that would otherwise be a launch of its own, and the first one of the pass), and the workgroups
// beyond the tile_blocks tiles flip the weights for the input-gradient convolution (Wq -> WqF; possibly none).
struct SideScale {
    const uint32_t* x = nullptr;      // the gradient, as bit patterns
    size_t n = 0;
    uint32_t* partials = nullptr;     // side.blocks block maxima
    unsigned blocks = 0;
};

// true: this workgroup had one of the side roles and is done
__device__ inline bool side_roles(const SideScale& side, unsigned tile_blocks, const int8_t* __restrict__ Wq, const ConvGeo& g,
                                  int8_t* __restrict__ WqF) {
    if (blockIdx.x < side.blocks) {
        __shared__ uint32_t red[4];
        absmax_body(side.x, side.n, side.partials, blockIdx.x, side.blocks, red);
        return true;
    }
    const unsigned b = blockIdx.x - side.blocks;
    if (b >= tile_blocks) {
        flip_weights_body(Wq, g, WqF, b - tile_blocks, gridDim.x - side.blocks - tile_blocks);
        return true;
    }
    return false;
}

// colT[(tap*C + c)][m] for a tile of 128 consecutive m x TCH = 64 channels of one tap (128 bytes of a colT row: whole
// cache lines; 14.0 -> 12.0 us on the ResNet layer against 64-byte pieces; 128 channels per tile, whole lines on
// the read side too, or 256 output pixels changed nothing or lost).  Each thread reads
// 4 (m) x 4 (c) blocks as four dwords each, transposes them in registers (byte permutes), parks the "4 consecutive m of one
// channel" dwords in LDS and the block then writes 16-byte pieces along m.  Needs C % 4 == 0.
// A workgroup walks the KW taps of one filter row for its tile (the rows' patch coordinates are worked out once, and
// the loads of the next tap are in flight while this one is written out: 0.0645 -> 0.0633 ms per layer step on the
// ResNet layer; all KH * KW taps per workgroup leave too few workgroups: 0.071 ms).
// Workgroups beyond the tile_blocks tiles flip the weights for the input-gradient convolution (Wq -> WqF;
// flip_blocks of them, possibly 0): two independent pieces of the backward pass in one launch.
constexpr int kColTileM = 128;
template <int TCH>
__global__ __launch_bounds__(256) void k_im2col_t_i8(const int8_t* __restrict__ Xq, ConvGeo g, int8_t* __restrict__ colT,
                                                     int tiles_m, int tiles_c, unsigned tile_blocks,
                                                     const int8_t* __restrict__ Wq, int8_t* __restrict__ WqF, SideScale side) {
    if (side_roles(side, tile_blocks, Wq, g, WqF)) return;
    constexpr int TS = kColTileM / 4 + 1;                        // dwords per staged channel (+ 1 pad)
    constexpr int CG = TCH / 4, MG = 256 / CG;                   // channel groups x row groups per round
    constexpr int ROUNDS = kColTileM / 4 / MG;                   // groups of 4 rows per thread
    __shared__ uint32_t t[TCH * TS];                             // [channel][32 dwords of m]
    __shared__ PatchRow rows[kColTileM];
    int b = static_cast<int>(blockIdx.x - side.blocks);
    const int tc = b % tiles_c; b /= tiles_c;
    const int tm = b % tiles_m;
    const int kh = b / tiles_m;                                  // one filter row per workgroup, its KW taps in turn
    const int64_t m0 = static_cast<int64_t>(tm) * kColTileM, M = g.M();
    const int c0 = tc * TCH;
    const int cg = threadIdx.x % CG, mg = threadIdx.x / CG;
    if (threadIdx.x < kColTileM && m0 + threadIdx.x < M) rows[threadIdx.x] = patch_row(g, static_cast<uint32_t>(m0) + threadIdx.x);
    __syncthreads();
    uint32_t v[ROUNDS][4];
    auto load_tap = [&](int kw) {
        const int64_t tap_off = (static_cast<int64_t>(kh) * g.W + kw) * g.C + c0 + 4 * cg;
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            const int rg = mg + MG * r;                          // group of 4 rows
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                v[r][k] = 0;
                if (m0 + 4 * rg + k < M && c0 + 4 * cg < g.C) {
                    const PatchRow pr = rows[4 * rg + k];
                    const int h = pr.h0 + kh, w = pr.w0 + kw;
                    if (h >= 0 && h < g.H && w >= 0 && w < g.W) v[r][k] = *reinterpret_cast<const uint32_t*>(Xq + pr.base + tap_off);
                }
            }
        }
    };
    load_tap(0);
    for (int kw = 0; kw < g.KW; ++kw) {
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            uint32_t col[4];                                     // col[c] = 4 consecutive m of channel 4 * cg + c
            transpose4x4(v[r], col);
#pragma unroll
            for (int c = 0; c < 4; ++c) t[(4 * cg + c) * TS + mg + MG * r] = col[c];
        }
        __syncthreads();
        if (kw + 1 < g.KW) load_tap(kw + 1);                     // in flight while this tap is written out
        const int tap = kh * g.KW + kw;
        constexpr int PIECES = kColTileM / 16;                   // 16-byte pieces of a staged channel
#pragma unroll
        for (int it = 0; it < TCH * PIECES / 256; ++it) {
            const int id = it * 256 + threadIdx.x;
            const int c = id / PIECES, ch = id % PIECES;         // channel row, 16-byte piece along m
            if (c0 + c >= g.C) continue;
            int8_t* dst = colT + (static_cast<int64_t>(tap) * g.C + c0 + c) * M + m0 + 16 * ch;
            const uint32_t* src = t + c * TS + 4 * ch;
            if ((M & 15) == 0 && m0 + 16 * ch + 16 <= M) {
                *reinterpret_cast<uint4*>(dst) = make_uint4(src[0], src[1], src[2], src[3]);
            } else {
                for (int j = 0; j < 16; ++j)
                    if (m0 + 16 * ch + j < M) dst[j] = static_cast<int8_t>((src[j >> 2] >> (8 * (j & 3))) & 0xffu);
            }
        }
        __syncthreads();                                         // the staging area is free for the next tap
    }
}

// same, one byte at a time, for C % 4 != 0
__global__ __launch_bounds__(256) void k_im2col_t_i8_bytes(const int8_t* __restrict__ Xq, ConvGeo g, int8_t* __restrict__ colT,
                                                           int tiles_m, int tiles_c, unsigned tile_blocks,
                                                           const int8_t* __restrict__ Wq, int8_t* __restrict__ WqF, SideScale side) {
    if (side_roles(side, tile_blocks, Wq, g, WqF)) return;
    __shared__ int8_t t[64][65];
    int b = static_cast<int>(blockIdx.x - side.blocks);
    const int tc = b % tiles_c; b /= tiles_c;
    const int tm = b % tiles_m;
    const int tap = b / tiles_m;
    const int kh = tap / g.KW, kw = tap - kh * g.KW;
    const int64_t m0 = static_cast<int64_t>(tm) * 64, M = g.M();
    const int c0 = tc * 64;
    for (int id = threadIdx.x; id < 64 * 64; id += 256) {
        const int r = id >> 6, c = id & 63;
        const int64_t m = m0 + r;
        int8_t v = 0;
        if (m < M && c0 + c < g.C) {
            const int wo = static_cast<int>(m % g.Wo);
            const int64_t q = m / g.Wo;
            const int ho = static_cast<int>(q % g.Ho), n = static_cast<int>(q / g.Ho);
            const int h = ho * g.stride + kh - g.pad, w = wo * g.stride + kw - g.padw;
            if (h >= 0 && h < g.H && w >= 0 && w < g.W) v = Xq[((static_cast<int64_t>(n) * g.H + h) * g.W + w) * g.C + c0 + c];
        }
        t[r][c] = v;
    }
    __syncthreads();
    for (int id = threadIdx.x; id < 64 * 64; id += 256) {
        const int c = id >> 6, r = id & 63;
        if (m0 + r < M && c0 + c < g.C) colT[(static_cast<int64_t>(tap) * g.C + c0 + c) * M + m0 + r] = t[r][c];
    }
}

// dX[n,h,w,c] = unmap( sum over taps (kh,kw) with (h + pad - kh) = ho*stride, (w + pad - kw) = wo*stride of
//               dcol[(n,ho,wo)][tap*C + c] ); VEC channels per thread (4 when C % 4 == 0)
template <int VEC>
__global__ __launch_bounds__(256) void k_col2im_unmap(const int32_t* __restrict__ dcol, ConvGeo g, const int32_t* __restrict__ eA,
                                                      int bitsA, const int32_t* __restrict__ eB, int bitsB,
                                                      float* __restrict__ dX) {
    const int E = lsb_exponent(eA[0], bitsA) + lsb_exponent(eB[0], bitsB);
    const int cv = g.C / VEC;
    const int64_t total = static_cast<int64_t>(g.N) * g.H * g.W * cv, K = g.K();
    for (int64_t id = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; id < total; id += static_cast<int64_t>(gridDim.x) * 256) {
        const int c = static_cast<int>(id % cv) * VEC;
        int64_t p = id / cv;
        const int w = static_cast<int>(p % g.W); p /= g.W;
        const int h = static_cast<int>(p % g.H);
        const int n = static_cast<int>(p / g.H);
        int acc[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] = 0;
        for (int kh = 0; kh < g.KH; ++kh) {
            const int th = h + g.pad - kh;
            if (th < 0 || th % g.stride) continue;
            const int ho = th / g.stride;
            if (ho >= g.Ho) continue;
            for (int kw = 0; kw < g.KW; ++kw) {
                const int tw = w + g.padw - kw;
                if (tw < 0 || tw % g.stride) continue;
                const int wo = tw / g.stride;
                if (wo >= g.Wo) continue;
                const int32_t* src = dcol + ((static_cast<int64_t>(n) * g.Ho + ho) * g.Wo + wo) * K +
                                     static_cast<int64_t>(kh * g.KW + kw) * g.C + c;
                if constexpr (VEC == 4) {
                    const int4 q = *reinterpret_cast<const int4*>(src);
                    acc[0] += q.x; acc[1] += q.y; acc[2] += q.z; acc[3] += q.w;
                } else {
                    acc[0] += src[0];
                }
            }
        }
        float* dst = dX + ((static_cast<int64_t>(n) * g.H + h) * g.W + w) * g.C + c;
        if constexpr (VEC == 4) {
            *reinterpret_cast<float4*>(dst) = make_float4(unmap_value(acc[0], E), unmap_value(acc[1], E),
                                                          unmap_value(acc[2], E), unmap_value(acc[3], E));
        } else {
            dst[0] = unmap_value(acc[0], E);
        }
    }
}

// the input gradient of a stride-1 convolution is itself a convolution: of dY, padded by K-1-pad, with WqF
static bool dx_as_conv(const ConvGeo& g) { return g.stride == 1 && g.pad <= g.KH - 1 && g.padw <= g.KW - 1; }

static ConvGeo dx_geo(const ConvGeo& g) {
    ConvGeo d = g;
    d.H = g.Ho; d.W = g.Wo; d.C = g.Cout; d.Cout = g.C;
    d.pad = g.KH - 1 - g.pad; d.padw = g.KW - 1 - g.padw;
    d.Ho = g.H; d.Wo = g.W;
    return d;
}

static ConvTaps taps_of(const ConvGeo& g) {
    ConvTaps t;
    t.H = g.H; t.W = g.W; t.C = g.C; t.KW = g.KW; t.stride = g.stride; t.pad = g.pad; t.padw = g.padw; t.Ho = g.Ho; t.Wo = g.Wo;
    return t;
}

static unsigned grid_for(int64_t items) {
    const int64_t want = (items + 255) / 256;
    return static_cast<unsigned>(std::max<int64_t>(1, std::min<int64_t>(want, 16384)));
}

static int geo_of(const fxp_conv2d_shape* s, ConvGeo* g) {
    if (!s) return FXP_ERR_NULL;
    const int64_t lim = int64_t{1} << 30;
    if (s->N < 1 || s->H < 1 || s->W < 1 || s->C < 1 || s->Cout < 1 || s->KH < 1 || s->KW < 1 || s->stride < 1 || s->pad < 0)
        return FXP_ERR_DIMS;
    if (s->N > lim || s->H > lim || s->W > lim || s->C > lim || s->Cout > lim || s->KH > 64 || s->KW > 64 || s->stride > 64 ||
        s->pad > 64)
        return FXP_ERR_DIMS;
    if (s->H + 2 * s->pad < s->KH || s->W + 2 * s->pad < s->KW) return FXP_ERR_DIMS;
    g->N = static_cast<int>(s->N); g->H = static_cast<int>(s->H); g->W = static_cast<int>(s->W); g->C = static_cast<int>(s->C);
    g->Cout = static_cast<int>(s->Cout); g->KH = static_cast<int>(s->KH); g->KW = static_cast<int>(s->KW);
    g->stride = static_cast<int>(s->stride); g->pad = g->padw = static_cast<int>(s->pad);
    g->Ho = (g->H + 2 * g->pad - g->KH) / g->stride + 1;
    g->Wo = (g->W + 2 * g->pad - g->KW) / g->stride + 1;
    if (g->M() >= (int64_t{1} << 31) || g->K() >= (int64_t{1} << 31) || static_cast<int64_t>(g->N) * g->H * g->W >= (int64_t{1} << 31))
        return FXP_ERR_DIMS;
    // contractions of the forward and input-gradient products; the weight gradient sums over the M output pixels,
    // and beyond this many its workspace slices are added in 64 bits
    if (g->K() > kMaxContraction || static_cast<int64_t>(g->KH) * g->KW * g->Cout > kMaxContraction) return FXP_ERR_OVERFLOW;
    return FXP_OK;
}

static size_t conv_ws_fwd(const ConvGeo& g) {
    return 2 * round_up(kScaleWsBytes, 256) + round_up(static_cast<size_t>(g.M()) * g.K(), 256) +
           gemm_split_ws_bytes(g.M(), g.Cout, g.K());
}

static size_t conv_ws_bwd(const ConvGeo& g) {
    const size_t dw = round_up(static_cast<size_t>(g.K()) * g.M(), 256) + gemm_split_ws_bytes(g.Cout, g.K(), g.M());
    size_t dx;
    if (dx_as_conv(g)) {
        const ConvGeo d = dx_geo(g);
        dx = round_up(static_cast<size_t>(d.M()) * d.K(), 256) + gemm_split_ws_bytes(d.M(), d.Cout, d.K());
    } else {
        dx = round_up(static_cast<size_t>(g.M()) * g.K() * sizeof(int32_t), 256) + gemm_split_ws_bytes(g.M(), g.K(), g.Cout);
    }
    return round_up(kScaleWsBytes, 256) + std::max(dw, dx);
}

}  // namespace fxp

extern "C" size_t fxp_conv2d_workspace_bytes(const fxp_conv2d_shape* shape, int backward) {
    fxp::ConvGeo g;
    if (fxp::geo_of(shape, &g)) return 0;
    return backward ? fxp::conv_ws_bwd(g) : fxp::conv_ws_fwd(g);
}

extern "C" int fxp_conv2d_fwd(const float* X, const float* W, const fxp_conv2d_shape* shape, float* Y,
                              const fxp_conv_saved* saved, uint64_t seed, uint64_t step, int rounding, int bits, void* ws,
                              size_t ws_bytes, void* stream) {
    using namespace fxp;
    ConvGeo g;
    int rc = geo_of(shape, &g);
    if (rc) return rc;
    if (rounding != FXP_ROUND_STOCHASTIC && rounding != FXP_ROUND_NEAREST) return FXP_ERR_ROUNDING;
    if (bits < 2 || bits > 8) return FXP_ERR_BITS;
    if (!X || !W || !Y || !saved || !saved->Xq || !saved->Wq || !saved->WqT || !saved->WqF || !saved->eX || !saved->eW)
        return FXP_ERR_NULL;
    if (!ws || ws_bytes < conv_ws_fwd(g)) return FXP_ERR_WORKSPACE;
    if (!aligned(ws, 256) || !aligned(X, 4) || !aligned(W, 4) || !aligned(Y, 4) || !aligned(saved->Xq, 16)) return FXP_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t* w8 = static_cast<uint8_t*>(ws);
    uint32_t* pX = reinterpret_cast<uint32_t*>(w8);
    uint32_t* pW = reinterpret_cast<uint32_t*>(w8 + round_up(kScaleWsBytes, 256));
    int8_t* col = reinterpret_cast<int8_t*>(w8 + 2 * round_up(kScaleWsBytes, 256));
    uint8_t* rest = reinterpret_cast<uint8_t*>(col) + round_up(static_cast<size_t>(g.M()) * g.K(), 256);
    const int64_t M = g.M(), K = g.K(), pixels = static_cast<int64_t>(g.N) * g.H * g.W;
    const MapTensor tX{X, pixels, g.C, nullptr, pX, 0, saved->eX, saved->Xq, nullptr, (step << 8) | FXP_TAG_X};
    const MapTensor tW{W, g.Cout, K, nullptr, pW, 0, saved->eW, saved->Wq, saved->WqT, (step << 8) | FXP_TAG_W};
    if ((rc = scale_and_map2(tX, tW, seed, rounding, bits, s))) return rc;
    // patches read straight from the int8 image by the GEMM loader where the shape allows, else stored first
    rc = conv_gemm_launch(taps_of(g), g.KH, M, g.Cout, saved->Xq, saved->Wq, Y, saved->eX, bits, saved->eW, bits, s);
    if (rc != kNotApplicable) return rc;
    if (g.C % 16 == 0)
        hipLaunchKernelGGL(k_im2col_i8<16>, dim3(static_cast<unsigned>((M + 31) / 32)), dim3(256), 0, s, saved->Xq, g, col);
    else
        hipLaunchKernelGGL(k_im2col_i8<1>, dim3(static_cast<unsigned>((M + 31) / 32)), dim3(256), 0, s, saved->Xq, g, col);
    if ((rc = launch_status())) return rc;
    return gemm_nt_launch(M, g.Cout, K, col, K, saved->Wq, K, Y, g.Cout, true, saved->eX, bits, saved->eW, bits, rest,
                          ws_bytes - static_cast<size_t>(rest - w8), s);
}

extern "C" int fxp_conv2d_bwd(const float* dY, const fxp_conv_saved* saved, const fxp_conv2d_shape* shape, float* dX,
                              float* dW, int8_t* dYq, int8_t* dYqT, int32_t* e_dY, uint64_t seed, uint64_t step,
                              int rounding, int bits, void* ws, size_t ws_bytes, void* stream) {
    using namespace fxp;
    ConvGeo g;
    int rc = geo_of(shape, &g);
    if (rc) return rc;
    if (rounding != FXP_ROUND_STOCHASTIC && rounding != FXP_ROUND_NEAREST) return FXP_ERR_ROUNDING;
    if (bits < 2 || bits > 8) return FXP_ERR_BITS;
    if (!dY || !saved || !saved->Xq || !saved->Wq || !saved->WqT || !saved->WqF || !saved->eX || !saved->eW || !dYq || !dYqT ||
        !e_dY)
        return FXP_ERR_NULL;
    if (!ws || ws_bytes < conv_ws_bwd(g)) return FXP_ERR_WORKSPACE;
    if (!aligned(ws, 256) || !aligned(dY, 4) || !aligned(dX, 16) || !aligned(dW, 4)) return FXP_ERR_ALIGN;
    // the patch, flip and product kernels of this call read and write these with 4- and 16-byte accesses
    if (!aligned(saved->Xq, 16) || !aligned(saved->Wq, 16) || !aligned(saved->WqT, 16) || !aligned(saved->WqF, 16) ||
        !aligned(dYq, 16) || !aligned(dYqT, 16) || !aligned(saved->eX, 4) || !aligned(saved->eW, 4) || !aligned(e_dY, 4))
        return FXP_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t* w8 = static_cast<uint8_t*>(ws);
    uint8_t* area = w8 + round_up(kScaleWsBytes, 256);
    const size_t area_bytes = ws_bytes - round_up(kScaleWsBytes, 256);
    const int64_t M = g.M(), K = g.K();
    // With a weight gradient to compute, the block maxima of dY are reduced by the launch that writes the
    // transposed patches (below) and the map of dY follows it; otherwise the usual pair of launches.
    SideScale side;
    if (dW) {
        side.x = reinterpret_cast<const uint32_t*>(dY);
        side.n = static_cast<size_t>(M) * static_cast<size_t>(g.Cout);
        side.partials = reinterpret_cast<uint32_t*>(w8);
        side.blocks = static_cast<unsigned>(scale_partial_count(side.n));
    } else if ((rc = scale_and_map(dY, M, g.Cout, e_dY, dYq, dYqT, seed, (step << 8) | FXP_TAG_DY, rounding, bits,
                                   reinterpret_cast<uint32_t*>(w8), s))) {
        return rc;
    }
    const bool need_flip = dX && dx_as_conv(g);
    ReduceRider pending;                 // the weight gradient's split-K reduction while it waits for a launch to ride in
    if (need_flip && !dW) {
        hipLaunchKernelGGL(k_flip_weights_i8, dim3(grid_for(static_cast<int64_t>(g.Cout) * K)), dim3(256), 0, s, saved->Wq, g,
                           saved->WqF);
        if ((rc = launch_status())) return rc;
    }
    if (dW) {
        int8_t* colT = reinterpret_cast<int8_t*>(area);
        const bool quads = g.C % 4 == 0;                        // the dword kernel takes 128 output pixels per tile
        const int tch = 64;                                     // channels per tile
        const int tiles_m = static_cast<int>(quads ? (M + kColTileM - 1) / kColTileM : (M + 63) / 64), tiles_c = (g.C + tch - 1) / tch;
        // the dword kernel walks the KW taps of a filter row inside a workgroup, the byte kernel takes one tap
        const int64_t blocks = static_cast<int64_t>(g.KH) * (quads ? 1 : g.KW) * tiles_m * tiles_c;
        if (blocks >= (int64_t{1} << 31)) return FXP_ERR_DIMS;
        // the flipped weights of the input-gradient convolution ride along in the same launch
        const unsigned flip_blocks = need_flip ? grid_for(static_cast<int64_t>(g.Cout) * K) : 0u;
        if (blocks + flip_blocks + side.blocks >= (int64_t{1} << 31)) return FXP_ERR_DIMS;
        const dim3 tgrid(side.blocks + static_cast<unsigned>(blocks) + flip_blocks);
        if (quads)
            hipLaunchKernelGGL(k_im2col_t_i8<64>, tgrid, dim3(256), 0, s, saved->Xq, g, colT, tiles_m, tiles_c,
                               static_cast<unsigned>(blocks), saved->Wq, saved->WqF, side);
        else
            hipLaunchKernelGGL(k_im2col_t_i8_bytes, tgrid, dim3(256), 0, s, saved->Xq, g, colT, tiles_m, tiles_c,
                               static_cast<unsigned>(blocks), saved->Wq, saved->WqF, side);
        if ((rc = launch_status())) return rc;
        // dY: the map kernel finishes the reduction from the block maxima just written
        const MapTensor tdY{dY, M, g.Cout, nullptr, side.partials, static_cast<int>(side.blocks), e_dY, dYq, dYqT,
                            (step << 8) | FXP_TAG_DY};
        if ((rc = map_launch(tdY, seed, rounding, bits, s))) return rc;
        const size_t used = round_up(static_cast<size_t>(K) * M, 256);
        // dW[Cout, K] = dYqT[Cout, M] * colT[K, M]^T, contraction over all output pixels
        // (split along K: the sum of its slices rides in the launch of the input-gradient convolution when that
        // one reads its patches in the loader and leaves the workspace alone)
        if ((rc = gemm_nt_launch(g.Cout, K, M, dYqT, M, colT, M, dW, K, true, e_dY, bits, saved->eX, bits, area + used,
                                 area_bytes - used, s, nullptr, nullptr, dX && dx_as_conv(g) ? &pending : nullptr)))
            return rc;
    }
    if (dX && dx_as_conv(g)) {
        // stride 1: dX[N*H*W, C] = unmap( im2col(dYq, pad K-1-pad) * WqF^T ), the inverse mapping fused as usual
        const ConvGeo d = dx_geo(g);
        int8_t* colg = reinterpret_cast<int8_t*>(area);
        const int64_t Md = d.M(), Kd = d.K();
        rc = conv_gemm_launch(taps_of(d), d.KH, Md, g.C, dYq, saved->WqF, dX, e_dY, bits, saved->eW, bits, s, &pending);
        if (rc != kNotApplicable) {
            if (rc == FXP_OK && pending.blocks != 0) rc = splitk_reduce_launch(pending, s);
            return rc;
        }
        // the explicit path below reuses the workspace: the weight gradient's slices are summed first
        if (pending.blocks != 0) {
            if ((rc = splitk_reduce_launch(pending, s))) return rc;
            pending.blocks = 0;
        }
        if (d.C % 16 == 0)
            hipLaunchKernelGGL(k_im2col_i8<16>, dim3(static_cast<unsigned>((Md + 31) / 32)), dim3(256), 0, s, dYq, d, colg);
        else
            hipLaunchKernelGGL(k_im2col_i8<1>, dim3(static_cast<unsigned>((Md + 31) / 32)), dim3(256), 0, s, dYq, d, colg);
        if ((rc = launch_status())) return rc;
        const size_t used = round_up(static_cast<size_t>(Md) * Kd, 256);
        if ((rc = gemm_nt_launch(Md, g.C, Kd, colg, Kd, saved->WqF, Kd, dX, g.C, true, e_dY, bits, saved->eW, bits, area + used,
                                 area_bytes - used, s)))
            return rc;
    } else if (dX) {
        int32_t* dcol = reinterpret_cast<int32_t*>(area);
        const size_t used = round_up(static_cast<size_t>(M) * K * sizeof(int32_t), 256);
        // dcol[M, K] = dYq[M, Cout] * WqT[K, Cout]^T, kept as int32: the patch sum below must be exact
        if ((rc = gemm_nt_launch(M, K, g.Cout, dYq, g.Cout, saved->WqT, g.Cout, dcol, K, false, nullptr, bits, nullptr, bits,
                                 area + used, area_bytes - used, s)))
            return rc;
        const int64_t pixels = static_cast<int64_t>(g.N) * g.H * g.W;
        if (g.C % 4 == 0)
            hipLaunchKernelGGL(k_col2im_unmap<4>, dim3(grid_for(pixels * g.C / 4)), dim3(256), 0, s, dcol, g, e_dY, bits,
                               saved->eW, bits, dX);
        else
            hipLaunchKernelGGL(k_col2im_unmap<1>, dim3(grid_for(pixels * g.C)), dim3(256), 0, s, dcol, g, e_dY, bits,
                               saved->eW, bits, dX);
        if ((rc = launch_status())) return rc;
    }
    return FXP_OK;
}
