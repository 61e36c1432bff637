// Integer GEMM on the matrix cores (paper Sec. 3.3, Fig. 2: int8 x int8 products,
// int32 accumulation) with the non-linear inverse mapping of Sec. 3.2 fused into the
// epilogue.
//
// One kernel form: C[M,N] = A[M,K] * B[N,K]^T with BOTH operands contiguous along the
// contraction (the mapping kernel emits every tensor in both orientations, so the three
// GEMMs of a layer step all take this form).  v_mfma_i32_32x32x32_i8: a lane holds 16
// consecutive contraction bytes of one row (A) or one column (B); integer addition is
// order-free, so only "same bytes on both sides" matters for the contraction index.
//
//   * three kernels share the tile scheme and the epilogue: k_gemm_nt stages tiles through registers (two LDS
//     buffers, any alignment and leading dimension: the fallback), k_gemm_nt_dma loads global -> LDS directly in a
//     multi-stage pipeline (the workhorse for every tile shape but the largest), k_gemm_nt_ring keeps a five-slot
//     ring of 256 x 256 x 128 tiles for the MFMA-bound shapes;
//   * LDS rows are BK bytes; 16-byte pieces are XOR-swizzled by the row so that the
//     64-lane ds_read_b128 of a fragment (32 rows x 2 pieces) spreads over all banks;
//   * accumulator lanes run along N: each store instruction writes 128-byte runs;
//   * workgroups are renumbered so that each XCD (own L2) works on a compact patch of
//     tiles instead of every 8th tile;
//   * long-contraction / small-output shapes split K across grid.y: every slice stores its int32 tile into a
//     workspace slice and a reduction (its own launch, or riding in the next product's) sums them and applies the
//     inverse mapping; without workspace the slices add into C with int32 atomics (exact either way: integer
//     addition is associative).
// Roofline: MFMA-bound when 2MNK / (MK + NK + 4MN bytes) is above ~630 ops/B, else HBM.
#include <algorithm>
#include <type_traits>

#include "fxp_internal.h"

namespace fxp {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

enum { kStoreI32 = 0, kStoreF32 = 1, kAtomicI32 = 2 };

// batched product: `count` matrices, element strides between consecutive ones (grid.z)
struct Batch {
    unsigned count = 1;
    int64_t a = 0, b = 0, c = 0;
};

template <int V>
using IC = std::integral_constant<int, V>;

constexpr int kNumXcd = 8;

// Workgroup b runs on XCD b % 8.  Give XCD x the contiguous range of tile numbers
// [start(x), start(x+1)), then walk tiles in column-major groups of `group_m` tile rows
// so that concurrently resident tiles share A and B panels in that XCD's L2.
__device__ inline void tile_of_block(int b, int tiles_m, int tiles_n, int group_m, int* tm, int* tn) {
    const int total = tiles_m * tiles_n;
    const int q = total / kNumXcd, r = total % kNumXcd;
    const int xcd = b % kNumXcd, local = b / kNumXcd;
    const int t = (xcd < r) ? xcd * (q + 1) + local : r * (q + 1) + (xcd - r) * q + local;
    const int per_group = group_m * tiles_n;
    const int g = t / per_group, in_g = t % per_group;
    const int rows_here = min(group_m, tiles_m - g * group_m);
    *tm = g * group_m + in_g % rows_here;
    *tn = in_g / rows_here;
}

template <int BK>
__device__ inline int swizzle_of_row(int row) {
    constexpr int CPR = BK / 16;            // 16-byte pieces per LDS row
    return (row / (16 / CPR)) % CPR;        // period 16 rows: 16 rows x 16 B = all 64 banks once
}

// The wave's largest output magnitude -> one of the FXP_ABSMAX_WORDS words at amax (IEEE bits of a non-negative
// float order like unsigned integers): one device-scope atomic per wave, without a returned value and with no
// load before it - vector memory operations complete in order, so anything a wave has to WAIT for behind its
// stores (a look at the word first, to skip the atomic) keeps it alive until they have drained, and the
// output-bound products live on waves ending while their stores are still in flight; consecutive waves use
// words in different cache lines.
__device__ inline void publish_absmax(float m, uint32_t* amax) {
    const uint32_t b = wave_max(__float_as_uint(m));
    // (block and thread indices only: the launch dimensions would be LOADED, and a wave that waits for a load
    // behind its stores stays alive until they have drained)
    const unsigned slot = ((blockIdx.x + blockIdx.y * 37u) * 16u + (threadIdx.x >> 6)) % FXP_ABSMAX_WORDS;
    if ((threadIdx.x & 63) == 0) atomicMax(amax + (((slot & 7u) << 5) | (slot >> 3)), b);     // 8 lines of 32 words
}

// Epilogue of every product kernel: the wave's FM x FN fragments of 32 x 32 go to C (top-left element row0, col0
// of the wave's tile), as inverse-mapped fp32 (non-temporal: the output is not read again here), as int32, or
// added into int32 with atomics.  Accumulator register r of lane l is row 8 * (r / 4) + 4 * (l / 32) + r % 4,
// column l % 32 of its fragment.  AMAX: returns the largest magnitude this lane stored.
// GUARD = false: the wave's tile lies inside C - no bounds tests, row addresses a scalar multiple of ldc away from
// the lane's base.  PLAIN: 2^E is a normal float (or the output is int32) - one convert and one multiply per
// value.  The output-bound products spend a fifth of their time issuing this loop, so both tests are made once
// per wave, outside it.
template <int FM, int FN, int MODE, bool AMAX, bool GUARD, bool PLAIN>
__device__ inline float store_loop(const v16i (&acc)[FM][FN], void* __restrict__ Cv, int64_t ldc, int M, int N, int row0,
                                   int col0, int fhalf, int frow, int E) {
    float m = 0.0f;
    const float unit = __uint_as_float(static_cast<uint32_t>(PLAIN ? E + 127 : 127) << 23);
    const int64_t base = static_cast<int64_t>(row0 + 4 * fhalf) * ldc + col0 + frow;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int dr = 32 * i + 8 * (r >> 2) + (r & 3);            // row of this register below the lane's base row
            if (GUARD && row0 + 4 * fhalf + dr >= M) continue;
            const int64_t off_row = base + dr * ldc;
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                if (GUARD && col0 + 32 * j + frow >= N) continue;
                const int64_t off = off_row + 32 * j;
                if (MODE == kStoreF32) {
                    const float v = PLAIN ? static_cast<float>(acc[i][j][r]) * unit : unmap_value(acc[i][j][r], E);
                    __builtin_nontemporal_store(v, static_cast<float*>(Cv) + off);
                    if (AMAX) m = fmaxf(m, fabsf(v));
                } else if (MODE == kStoreI32) {
                    static_cast<int32_t*>(Cv)[off] = acc[i][j][r];
                } else {
                    atomicAdd(static_cast<int32_t*>(Cv) + off, acc[i][j][r]);
                }
            }
        }
    }
    return m;
}

template <int FM, int FN, int MODE, bool AMAX>
__device__ inline float store_fragments(const v16i (&acc)[FM][FN], void* __restrict__ Cv, int64_t ldc, int M, int N, int row0,
                                        int col0, int fhalf, int frow, int E) {
    const bool inside = row0 + 32 * FM <= M && col0 + 32 * FN <= N;                     // wave-uniform
    const bool plain = MODE != kStoreF32 || (E >= -126 && E <= 127);
    if (inside && plain) {
        float m = 0.0f;
        if (AMAX) {
            // the inverse mapping is monotone: the largest magnitude comes from the largest or the smallest sum,
            // found on the integers (one three-input max / min per value) before the store loop starts
            int hi = 0, lo = 0;
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; r += 2) {
                        hi = max(max(hi, acc[i][j][r]), acc[i][j][r + 1]);
                        lo = min(min(lo, acc[i][j][r]), acc[i][j][r + 1]);
                    }
            const float unit = __uint_as_float(static_cast<uint32_t>(E + 127) << 23);
            m = fmaxf(static_cast<float>(hi) * unit, -(static_cast<float>(lo) * unit));
        }
        store_loop<FM, FN, MODE, false, false, true>(acc, Cv, ldc, M, N, row0, col0, fhalf, frow, E);
        return m;
    }
    if (plain) return store_loop<FM, FN, MODE, AMAX, true, true>(acc, Cv, ldc, M, N, row0, col0, fhalf, frow, E);
    return store_loop<FM, FN, MODE, AMAX, true, false>(acc, Cv, ldc, M, N, row0, col0, fhalf, frow, E);
}

// Sum of the split-K slices of a product (int32, exact in any order) -> int32 or inverse-mapped fp32, by workgroup
// `b` of `nb`.  The slices are dense M x N matrices `stride` elements apart.  A dense, 16-byte aligned output is
// walked as one flat run of 16-byte pieces, anything else row by row.
__device__ inline void splitk_reduce_body(const ReduceRider& r, unsigned b, unsigned nb) {
    const unsigned nt = blockDim.x;                  // 256 stand-alone; the host product's workgroup size when riding
    float m = 0.0f;
    int E = 0;
    if (r.fp32_out) E = lsb_exponent(r.eA[0], r.bitsA) + (r.eB ? lsb_exponent(r.eB[0], r.bitsB) : 0);
    const int32_t* __restrict__ parts = r.parts;
    const int64_t stride = r.stride;
    const int splits = r.splits;
    auto one = [&](int acc, int32_t* dst) {
        if (r.fp32_out) {
            const float o = unmap_value(acc, E);
            *reinterpret_cast<float*>(dst) = o;
            m = fmaxf(m, fabsf(o));
        } else {
            *dst = acc;
        }
    };
    const int64_t total = static_cast<int64_t>(r.M) * r.N;
    const bool flat = r.ldc == r.N && (reinterpret_cast<uintptr_t>(r.C) & 15u) == 0;
    if (r.wide) {
        // contraction beyond what one int32 sum holds: 64-bit sum of the slices, one element per thread and round
        for (int64_t i = static_cast<int64_t>(b) * nt + threadIdx.x; i < total; i += static_cast<int64_t>(nb) * nt) {
            int64_t acc = 0;
            for (int sidx = 0; sidx < splits; ++sidx) acc += parts[sidx * stride + i];
            const float o = unmap_value64(acc, E);
            static_cast<float*>(r.C)[(i / r.N) * r.ldc + i % r.N] = o;
            m = fmaxf(m, fabsf(o));
        }
    } else if (flat) {
        const int64_t nvec = total >> 2;
        for (int64_t i = static_cast<int64_t>(b) * nt + threadIdx.x; i < nvec; i += static_cast<int64_t>(nb) * nt) {
            int4 acc = make_int4(0, 0, 0, 0);
#pragma unroll 8
            for (int sidx = 0; sidx < splits; ++sidx) {
                const int4 v = reinterpret_cast<const int4*>(parts + sidx * stride)[i];
                acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
            }
            if (r.fp32_out) {
                float4 o;
                o.x = unmap_value(acc.x, E); o.y = unmap_value(acc.y, E);
                o.z = unmap_value(acc.z, E); o.w = unmap_value(acc.w, E);
                reinterpret_cast<float4*>(r.C)[i] = o;
                m = fmaxf(fmaxf(m, fmaxf(fabsf(o.x), fabsf(o.y))), fmaxf(fabsf(o.z), fabsf(o.w)));
            } else {
                reinterpret_cast<int4*>(r.C)[i] = acc;
            }
        }
        if (b == 0 && threadIdx.x < (total & 3)) {                 // the slices are 16-byte aligned, the tail is not a piece
            const int64_t i = (nvec << 2) + threadIdx.x;
            int acc = 0;
            for (int sidx = 0; sidx < splits; ++sidx) acc += parts[sidx * stride + i];
            one(acc, static_cast<int32_t*>(r.C) + i);
        }
    } else {
        for (int row = static_cast<int>(b); row < r.M; row += static_cast<int>(nb)) {
            const int32_t* prow = parts + static_cast<int64_t>(row) * r.N;
            int32_t* crow = static_cast<int32_t*>(r.C) + static_cast<int64_t>(row) * r.ldc;
            for (int i = threadIdx.x; i < r.N; i += static_cast<int>(nt)) {
                int acc = 0;
                for (int sidx = 0; sidx < splits; ++sidx) acc += prow[sidx * stride + i];
                one(acc, crow + i);
            }
        }
    }
    if (r.fp32_out && r.amax != nullptr) publish_absmax(m, r.amax);
}

template <int BM, int BN, int BK, int WM, int WN, bool VEC, int MODE>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void k_gemm_nt(
    const int8_t* __restrict__ A, int64_t lda, const int8_t* __restrict__ B, int64_t ldb, void* __restrict__ Cv,
    int64_t ldc, int M, int N, int K, int k_per_split, const int32_t* __restrict__ eA, int bitsA,
    const int32_t* __restrict__ eB, int bitsB, int tiles_m, int tiles_n, int group_m, int64_t split_stride,
    int64_t batch_a, int64_t batch_b, int64_t batch_c, uint32_t* __restrict__ amax, ReduceRider rider) {
    int tile_block = static_cast<int>(blockIdx.x);
    if (rider.blocks != 0) {                                      // workgroup-uniform
        const unsigned first = rider.front ? 0u : rider.tiles;    // the riders are the first or the last workgroups
        if (blockIdx.x >= first && blockIdx.x < first + rider.blocks) {
            splitk_reduce_body(rider, blockIdx.x - first, rider.blocks);
            return;
        }
        if (rider.front) tile_block -= static_cast<int>(rider.blocks);
    }
    constexpr int NT = (BM / WM) * (BN / WN) * 64;
    constexpr int CPR = BK / 16;
    constexpr int NA = BM * CPR / NT, NB = BN * CPR / NT;   // 16-byte pieces per thread per step
    constexpr int FM = WM / 32, FN = WN / 32;               // 32x32 fragments per wave
    static_assert(BM * CPR % NT == 0 && BN * CPR % NT == 0, "tile does not divide over the threads");

    __shared__ __attribute__((aligned(16))) int8_t lds[2][(BM + BN) * BK];

    int tm, tn;
    tile_of_block(tile_block, tiles_m, tiles_n, group_m, &tm, &tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const int kb = blockIdx.y * k_per_split;
    // split-K into a workspace: slice y owns its own M x N int32 matrix (split_stride elements apart)
    Cv = static_cast<int32_t*>(Cv) + static_cast<int64_t>(blockIdx.y) * split_stride + static_cast<int64_t>(blockIdx.z) * batch_c;
    // batched product: matrix z of each operand lies batch_* elements further on
    A += static_cast<int64_t>(blockIdx.z) * batch_a;
    B += static_cast<int64_t>(blockIdx.z) * batch_b;
    const int ke = min(K, kb + k_per_split);
    const int nk = (ke - kb + BK - 1) / BK;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / (BN / WN)) * WM, wn0 = (wave % (BN / WN)) * WN;

    // ---- global -> register staging ------------------------------------------------
    const int8_t* pa[NA];
    const int8_t* pb[NB];
    int lds_a[NA], lds_b[NB], kc_a[NA], kc_b[NB];
#pragma unroll
    for (int j = 0; j < NA; ++j) {
        const int id = tid + j * NT, row = id / CPR, c = id % CPR;
        pa[j] = A + static_cast<int64_t>(min(m0 + row, M - 1)) * lda + c * 16;
        lds_a[j] = row * BK + ((c ^ swizzle_of_row<BK>(row)) * 16);
        kc_a[j] = c * 16;
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int id = tid + j * NT, row = id / CPR, c = id % CPR;
        pb[j] = B + static_cast<int64_t>(min(n0 + row, N - 1)) * ldb + c * 16;
        lds_b[j] = BM * BK + row * BK + ((c ^ swizzle_of_row<BK>(row)) * 16);
        kc_b[j] = c * 16;
    }
    uint4 ra[NA], rb[NB];

    auto load_piece = [&](const int8_t* p, int k_first) -> uint4 {
        // k_first: contraction index of the piece's first byte; bytes at or beyond ke read as 0
        if (VEC) {
            if (k_first < ke) return *reinterpret_cast<const uint4*>(p);
            return make_uint4(0, 0, 0, 0);
        }
        uint32_t w[4] = {0, 0, 0, 0};
        for (int b = 0; b < 16; ++b)
            if (k_first + b < ke) w[b >> 2] |= static_cast<uint32_t>(static_cast<uint8_t>(p[b])) << (8 * (b & 3));
        return make_uint4(w[0], w[1], w[2], w[3]);
    };
    auto load_step = [&](int kk) {
#pragma unroll
        for (int j = 0; j < NA; ++j) ra[j] = load_piece(pa[j] + kk, kk + kc_a[j]);
#pragma unroll
        for (int j = 0; j < NB; ++j) rb[j] = load_piece(pb[j] + kk, kk + kc_b[j]);
    };
    auto store_step = [&](int buf) {
#pragma unroll
        for (int j = 0; j < NA; ++j) *reinterpret_cast<uint4*>(&lds[buf][lds_a[j]]) = ra[j];
#pragma unroll
        for (int j = 0; j < NB; ++j) *reinterpret_cast<uint4*>(&lds[buf][lds_b[j]]) = rb[j];
    };

    // ---- fragment addressing ---------------------------------------------------------
    // lane l reads row (l % 32) of a fragment, contraction bytes 16 * (l / 32) .. +15 of a 32-byte step
    const int frow = lane & 31, fhalf = lane >> 5;
    const int fswz = swizzle_of_row<BK>(frow);     // fragment bases are multiples of 32 rows: same swizzle
    const int a_base = (wm0 + frow) * BK, b_base = BM * BK + (wn0 + frow) * BK;

    v16i acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    if (nk > 0) {
        load_step(kb);
        store_step(0);
    }
    __syncthreads();
    for (int it = 0; it < nk; ++it) {
        const int buf = it & 1;
        if (it + 1 < nk) load_step(kb + (it + 1) * BK);
#pragma unroll
        for (int ks = 0; ks < BK / 32; ++ks) {
            const int piece = ((2 * ks + fhalf) ^ fswz) * 16;
            v4i fa[FM], fb[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i) fa[i] = *reinterpret_cast<const v4i*>(&lds[buf][a_base + i * 32 * BK + piece]);
#pragma unroll
            for (int j = 0; j < FN; ++j) fb[j] = *reinterpret_cast<const v4i*>(&lds[buf][b_base + j * 32 * BK + piece]);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (it + 1 < nk) store_step(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue --------------------------------------------------------------------
    // accumulator register r of lane l is row 8 * (r / 4) + 4 * (l / 32) + r % 4, column l % 32
    int E = 0;
    if (MODE == kStoreF32) E = lsb_exponent(eA[0], bitsA) + (eB ? lsb_exponent(eB[0], bitsB) : 0);
    if (MODE == kStoreF32 && amax != nullptr)
        publish_absmax(store_fragments<FM, FN, MODE, true>(acc, Cv, ldc, M, N, m0 + wm0, n0 + wn0, fhalf, frow, E), amax);
    else
        store_fragments<FM, FN, MODE, false>(acc, Cv, ldc, M, N, m0 + wm0, n0 + wn0, fhalf, frow, E);
}

// s_waitcnt immediate (gfx9 encoding): wait until at most `vm` vector-memory operations
// and no LDS operation of this wave are outstanding.
__host__ __device__ constexpr int waitcnt_vm_lgkm0(int vm) { return (vm & 0xF) | ((vm >> 4) << 14) | 0x70; }

template <int VM>
__device__ inline void wait_loads_and_lds() {
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(VM));
}

// 256 zero bytes: where the patch rows of an implicit convolution read their padding from, and a partial last K step
// the pieces beyond the end of the contraction
__device__ __attribute__((aligned(256))) const uint8_t g_zero_page[256] = {0};

// Same product, fast path: K a multiple of BK, operands 16-byte aligned.  Global loads go
// straight into LDS (global_load_lds_dwordx4: each wave fills one contiguous 1 KiB region
// per instruction, no register staging, no ds_write), STAGES buffers deep, so loads for
// step k + STAGES - 1 are in flight while step k is multiplied.  The XOR swizzle of the
// LDS layout is applied on the global side: lane p of a region fetches the 16-byte piece
// that belongs in slot p.  One s_barrier per step, no fence: the only cross-wave traffic
// is LDS written by the loads (waited for with vmcnt before the barrier) and read by
// ds_read (waited for with lgkmcnt before the next barrier lets the buffer be refilled).
//
// CONV: the A operand is not a stored matrix but the patch matrix of a channels-last int8 image tensor
// (A points at X[N,H,W,C]; row m is output pixel m, contraction index (kh*KW + kw)*C + c): the loader
// works out, per K step, which input pixel a row reads (one tap of the filter, since C % BK == 0) and takes
// the bytes straight from the image, or from a page of zeros where the tap falls into the padding.  Nothing
// else differs from the plain product.
template <int BM, int BN, int BK, int WM, int WN, int STAGES, int MODE, bool SCHED, bool CONV = false>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void k_gemm_nt_dma(
    const int8_t* __restrict__ A, int64_t lda, const int8_t* __restrict__ B, int64_t ldb, void* __restrict__ Cv,
    int64_t ldc, int M, int N, int K, int k_per_split, const int32_t* __restrict__ eA, int bitsA,
    const int32_t* __restrict__ eB, int bitsB, int tiles_m, int tiles_n, int group_m, int64_t split_stride,
    int64_t batch_a, int64_t batch_b, int64_t batch_c, ConvTaps ct, uint32_t* __restrict__ amax, ReduceRider rider) {
    int tile_block = static_cast<int>(blockIdx.x);
    if (rider.blocks != 0) {                                      // workgroup-uniform
        const unsigned first = rider.front ? 0u : rider.tiles;    // the riders are the first or the last workgroups
        if (blockIdx.x >= first && blockIdx.x < first + rider.blocks) {
            splitk_reduce_body(rider, blockIdx.x - first, rider.blocks);
            return;
        }
        if (rider.front) tile_block -= static_cast<int>(rider.blocks);
    }
    constexpr int NW = (BM / WM) * (BN / WN);
    constexpr int CPR = BK / 16;                     // 16-byte pieces per LDS row
    constexpr int RROWS = 64 / CPR;                  // tile rows per 1 KiB region
    constexpr int REGIONS = (BM + BN) * BK / 1024;   // per stage: A rows first, then B rows
    constexpr int RPW = REGIONS / NW;                // load instructions per wave per step
    constexpr int STAGE_BYTES = (BM + BN) * BK;
    constexpr int FM = WM / 32, FN = WN / 32;
    static_assert(REGIONS % NW == 0, "regions do not divide over the waves");
    static_assert(STAGES >= 2 && STAGES <= 4, "2 to 4 stages");
    static_assert((STAGES - 1) * RPW < 64, "vmcnt is a 6-bit counter");
    static_assert((BK / 32) % 2 == 0, "two 32-byte steps per register buffer pair");
    static_assert(FM * FN >= (FM + FN) / 2, "wave tile too small for the interleave");

    __shared__ __attribute__((aligned(1024))) int8_t lds[STAGES * STAGE_BYTES];

    // Workgroups reach the XCDs round-robin in dispatch order (x fastest, then y, then z).  One product, one slice:
    // the tile walk of tile_of_block.  Split along K, or a batch of products: XCD c takes a contiguous run of
    // (slice or matrix, tile) pairs in slice-major order, so the tiles of one slice (which read the same K range of
    // B) or of one small matrix (which read the same operands) share that XCD's L2.
    int tm, tn, slice = 0, matrix = 0;
    const int outer = static_cast<int>(gridDim.y * gridDim.z);     // never both: a batch is not split
    if (outer == 1) {
        tile_of_block(tile_block, tiles_m, tiles_n, group_m, &tm, &tn);
    } else {
        const int64_t tiles = static_cast<int64_t>(tiles_m) * tiles_n, total = tiles * outer;
        const int64_t v = (static_cast<int64_t>(blockIdx.z) * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
        const int64_t q = total / kNumXcd, r = total % kNumXcd, xcd = v % kNumXcd, local = v / kNumXcd;
        const int64_t p = (xcd < r) ? xcd * (q + 1) + local : r * (q + 1) + (xcd - r) * q + local;
        const int o = static_cast<int>(p / tiles), t = static_cast<int>(p - o * tiles);
        if (gridDim.y > 1) slice = o;
        else matrix = o;
        tm = t % tiles_m;
        tn = t / tiles_m;
    }
    const int m0 = tm * BM, n0 = tn * BN;
    const int kb = slice * k_per_split;
    // split-K into a workspace: every slice owns its own M x N int32 matrix (split_stride elements apart)
    Cv = static_cast<int32_t*>(Cv) + static_cast<int64_t>(slice) * split_stride + static_cast<int64_t>(matrix) * batch_c;
    // batched product: matrix z of each operand lies batch_* elements further on
    A += static_cast<int64_t>(matrix) * batch_a;
    B += static_cast<int64_t>(matrix) * batch_b;
    const int ke = min(K, kb + k_per_split);
    // whole K steps, plus one partial step when the slice ends inside a step (K a multiple of 16, not of BK):
    // its missing 16-byte pieces are read from the page of zeros, so the multiply loop never sees a tail
    const int nk = (ke - kb + BK - 1) / BK;
    const int tail = (ke - kb) % BK;


    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: LDS targets stay in SGPRs
    const int wm0 = (wave / (BN / WN)) * WM, wn0 = (wave % (BN / WN)) * WN;

    const int8_t* gp[RPW];
    int kpiece[RPW];                                                 // offset of the lane's 16-byte piece inside a K step
    int a_h0[RPW], a_w0[RPW];                                        // CONV: top-left input coordinate of the row's patch
#pragma unroll
    for (int j = 0; j < RPW; ++j) {
        const int row_t = (wave + j * NW) * RROWS + lane / CPR;      // row in the stacked (A;B) tile
        const int piece = (lane % CPR) ^ swizzle_of_row<BK>(row_t);  // BM % 16 == 0: same swizzle for B rows
        kpiece[j] = piece * 16;
        a_h0[j] = a_w0[j] = 0;
        if (CONV && row_t < BM) {
            const uint32_t m = static_cast<uint32_t>(min(m0 + row_t, M - 1));
            const uint32_t t = m / static_cast<uint32_t>(ct.Wo), n = t / static_cast<uint32_t>(ct.Ho);
            a_h0[j] = static_cast<int>(t - n * ct.Ho) * ct.stride - ct.pad;
            a_w0[j] = static_cast<int>(m - t * ct.Wo) * ct.stride - ct.padw;
            gp[j] = A + static_cast<int64_t>(n) * ct.H * ct.W * ct.C + piece * 16;          // the row's image
        } else {
            gp[j] = (row_t < BM) ? A + static_cast<int64_t>(min(m0 + row_t, M - 1)) * lda + kb + piece * 16
                                 : B + static_cast<int64_t>(min(n0 + row_t - BM, N - 1)) * ldb + kb + piece * 16;
        }
    }
    auto issue = [&](int step, int stage) {
        int kh = 0, kw = 0, c0 = 0;                                  // CONV: the tap and channel offset of this K step
        if (CONV) {
            const int k0 = kb + step * BK, tap = k0 / ct.C;
            c0 = k0 - tap * ct.C;
            kh = tap / ct.KW;
            kw = tap - kh * ct.KW;
        }
        const bool partial = !CONV && tail != 0 && step == nk - 1;   // wave-uniform
#pragma unroll
        for (int j = 0; j < RPW; ++j) {
            const int8_t* src = gp[j] + static_cast<int64_t>(step) * BK;
            if (partial && kpiece[j] >= tail) src = reinterpret_cast<const int8_t*>(g_zero_page) + kpiece[j];
            if (CONV && (wave + j * NW) * RROWS < BM) {              // a region of A rows (wave-uniform)
                const int h = a_h0[j] + kh, w = a_w0[j] + kw;
                const bool inside = static_cast<unsigned>(h) < static_cast<unsigned>(ct.H) &&
                                    static_cast<unsigned>(w) < static_cast<unsigned>(ct.W);
                src = inside ? gp[j] + (static_cast<int64_t>(h) * ct.W + w) * ct.C + c0
                             : reinterpret_cast<const int8_t*>(g_zero_page) + kpiece[j];
            }
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)src,
                (__attribute__((address_space(3))) void*)(&lds[stage * STAGE_BYTES + (wave + j * NW) * 1024]),
                16, 0, 0);
        }
    };

    const int frow = lane & 31, fhalf = lane >> 5;
    const int fswz = swizzle_of_row<BK>(frow);
    const int a_base = (wm0 + frow) * BK, b_base = BM * BK + (wn0 + frow) * BK;

    v16i acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // Fragments are double-buffered in registers: the ds_reads of 32-byte step s+1 are
    // issued before the MFMAs of step s.  The barrier that publishes LDS stage it+1 sits
    // in front of the LAST 32-byte step of stage it, so the first fragments of the next
    // stage are already on their way while that last step is multiplied, and the stage
    // just finished (every wave is past its reads of it) is refilled at once: all STAGES
    // buffers stay in flight.
    constexpr int KS = BK / 32;
    v4i fa[2][FM], fb[2][FN];
    auto read_frags = [&](int buf, int stage, int ks) {
        const int8_t* st = lds + stage * STAGE_BYTES;
        const int piece = ((2 * ks + fhalf) ^ fswz) * 16;
#pragma unroll
        for (int i = 0; i < FM; ++i) fa[buf][i] = *reinterpret_cast<const v4i*>(&st[a_base + i * 32 * BK + piece]);
#pragma unroll
        for (int j = 0; j < FN; ++j) fb[buf][j] = *reinterpret_cast<const v4i*>(&st[b_base + j * 32 * BK + piece]);
    };
#pragma unroll
    for (int s = 0; s < STAGES; ++s)
        if (s < nk) issue(s, s);
    if (nk > 0) {
        if (nk >= STAGES) wait_loads_and_lds<(STAGES - 1) * RPW>();
        else wait_loads_and_lds<0>();
        __builtin_amdgcn_s_barrier();
        read_frags(0, 0, 0);
    }
    // MFMAs of one 32-byte step.  `reads` ds_reads and `loads` global->LDS loads issued just
    // before it are slotted behind its first MFMAs (the matrix core runs an MFMA for 32
    // cycles; the wave issues the memory instructions in its shadow).
    auto multiply = [&](int cur, auto reads_c, auto loads_c) {
        constexpr int reads = decltype(reads_c)::value, loads = decltype(loads_c)::value;
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[cur][i], fb[cur][j], acc[i][j], 0, 0, 0);
        if (SCHED) {
#pragma unroll
            for (int n = 0; n < reads / 2; ++n) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);   // 2 DS reads
            }
#pragma unroll
            for (int n = 0; n < loads; ++n) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // 1 VMEM read
            }
            __builtin_amdgcn_sched_group_barrier(0x008, FM * FN - reads / 2 - loads, 0);
        }
    };
    // One LDS stage: all 32-byte steps but the last, then the barrier that publishes the next
    // stage, the first fragments of that stage, the refill of the stage just finished, and the
    // last step.  The wait is one fixed instruction and the refill is unconditional inside a
    // loop variant, so everything between two barriers is one basic block the scheduler can
    // interleave.
    auto stage_body = [&](int it, auto wait_next, auto refill) {
        const int stage = it % STAGES;
#pragma unroll
        for (int ks = 0; ks + 1 < KS; ++ks) {
            read_frags((ks & 1) ^ 1, stage, ks + 1);
            multiply(ks & 1, IC<FM + FN>{}, IC<0>{});
        }
        wait_next();
        __builtin_amdgcn_s_barrier();
        read_frags(0, (it + 1) % STAGES, 0);          // KS is even: the last step used buffer 1
        multiply(1, IC<FM + FN>{}, refill(it + STAGES, stage));
    };
    auto steady_wait = [] { wait_loads_and_lds<(STAGES - 2) * RPW>(); };
    auto full_wait = [] { wait_loads_and_lds<0>(); };
    auto do_refill = [&](int step, int stage) {
        issue(step, stage);
        return IC<(RPW <= FM * FN - (FM + FN) / 2 ? RPW : 0)>{};
    };
    auto no_refill = [](int, int) { return IC<0>{}; };
    int it = 0;
    for (; it + STAGES < nk; ++it) stage_body(it, steady_wait, do_refill);     // steps it+2 .. it+STAGES-1 in flight
    for (; it + STAGES - 1 < nk; ++it) stage_body(it, steady_wait, no_refill);
    for (; it + 1 < nk; ++it) stage_body(it, full_wait, no_refill);            // drain
    if (nk > 0) {
        const int stage = (nk - 1) % STAGES;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (ks + 1 < KS) read_frags((ks & 1) ^ 1, stage, ks + 1);
            if (ks + 1 < KS) multiply(ks & 1, IC<FM + FN>{}, IC<0>{});
            else multiply(ks & 1, IC<0>{}, IC<0>{});
        }
    }

    int E = 0;
    if (MODE == kStoreF32) E = lsb_exponent(eA[0], bitsA) + (eB ? lsb_exponent(eB[0], bitsB) : 0);
    if (MODE == kStoreF32 && amax != nullptr)
        publish_absmax(store_fragments<FM, FN, MODE, true>(acc, Cv, ldc, M, N, m0 + wm0, n0 + wn0, fhalf, frow, E), amax);
    else
        store_fragments<FM, FN, MODE, false>(acc, Cv, ldc, M, N, m0 + wm0, n0 + wn0, fhalf, frow, E);
}

// 256 x 256 x 128 tile with LDS used as a RING of five 32 KiB half-stages instead of two
// full stages.  A half-stage is the 256 x 128-byte slice of one operand for one step:
// A(0) B(0) A(1) B(1) A(2) | B(2) A(3) ...; half-stage h lives in slot h % 5.  Full 128-byte
// rows keep every L2 request a whole cache line (half-line requests top out at ~60 % of the
// line rate), and the fifth slot lets the loads of a step be issued in two instalments:
// A(t+2) is spread thinly over the first three 32-byte steps of stage t (its slot was freed
// one barrier earlier) and only B(t+2) has to be issued in a burst behind the barrier that
// frees A(t)'s slot.  The load queue therefore never runs dry and never has to swallow a
// whole 64 KiB stage at once, which is what stalled the MFMA stream of the two-stage form.
template <int WM, int WN, int MODE, bool SCHED>
__global__ __launch_bounds__((256 / WM) * (256 / WN) * 64) void k_gemm_nt_ring(
    const int8_t* __restrict__ A, int64_t lda, const int8_t* __restrict__ B, int64_t ldb, void* __restrict__ Cv,
    int64_t ldc, int M, int N, int K, int k_per_split, const int32_t* __restrict__ eA, int bitsA,
    const int32_t* __restrict__ eB, int bitsB, int tiles_m, int tiles_n, int group_m, int64_t split_stride,
    int64_t batch_a, int64_t batch_b, int64_t batch_c, uint32_t* __restrict__ amax, ReduceRider rider) {
    int tile_block = static_cast<int>(blockIdx.x);
    if (rider.blocks != 0) {                                      // workgroup-uniform
        const unsigned first = rider.front ? 0u : rider.tiles;    // the riders are the first or the last workgroups
        if (blockIdx.x >= first && blockIdx.x < first + rider.blocks) {
            splitk_reduce_body(rider, blockIdx.x - first, rider.blocks);
            return;
        }
        if (rider.front) tile_block -= static_cast<int>(rider.blocks);
    }
    constexpr int BM = 256, BN = 256, BK = 128;
    constexpr int NW = (BM / WM) * (BN / WN);
    constexpr int SLOT = 256 * BK;                   // bytes of a half-stage
    constexpr int RPH = (SLOT / 1024) / NW;          // load instructions per wave per half-stage
    constexpr int FM = WM / 32, FN = WN / 32, KS = BK / 32;
    static_assert(RPH >= 3 && RPH * 2 < 64, "loads per half-stage");

    __shared__ __attribute__((aligned(1024))) int8_t lds[5 * SLOT];

    int tm, tn;
    tile_of_block(tile_block, tiles_m, tiles_n, group_m, &tm, &tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const int kb = blockIdx.y * k_per_split;
    // split-K into a workspace: slice y owns its own M x N int32 matrix (split_stride elements apart)
    Cv = static_cast<int32_t*>(Cv) + static_cast<int64_t>(blockIdx.y) * split_stride + static_cast<int64_t>(blockIdx.z) * batch_c;
    // batched product: matrix z of each operand lies batch_* elements further on
    A += static_cast<int64_t>(blockIdx.z) * batch_a;
    B += static_cast<int64_t>(blockIdx.z) * batch_b;
    const int ke = min(K, kb + k_per_split);
    const int nk = (ke - kb) / BK;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave / (BN / WN)) * WM, wn0 = (wave % (BN / WN)) * WN;

    // lane p of 1 KiB region g fetches row 8g + p/8, piece (p%8) ^ swizzle(row) of the 128-byte row
    const int8_t* ga[RPH];
    const int8_t* gb[RPH];
#pragma unroll
    for (int j = 0; j < RPH; ++j) {
        const int row = (wave + j * NW) * 8 + lane / 8;
        const int piece = (lane % 8) ^ swizzle_of_row<BK>(row);
        ga[j] = A + static_cast<int64_t>(min(m0 + row, M - 1)) * lda + kb + piece * 16;
        gb[j] = B + static_cast<int64_t>(min(n0 + row, N - 1)) * ldb + kb + piece * 16;
    }
    auto load_piece = [&](const int8_t* g, int step, int slot, int j) {
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void*)(g + static_cast<int64_t>(step) * BK),
            (__attribute__((address_space(3))) void*)(&lds[slot * SLOT + (wave + j * NW) * 1024]), 16, 0, 0);
    };
    auto issue_a = [&](int step, auto lo_c, auto hi_c) {        // loads [lo, hi) of A(step)
        const int slot = (2 * step) % 5;
#pragma unroll
        for (int j = decltype(lo_c)::value; j < decltype(hi_c)::value; ++j) load_piece(ga[j], step, slot, j);
    };
    auto issue_b = [&](int step) {
        const int slot = (2 * step + 1) % 5;
#pragma unroll
        for (int j = 0; j < RPH; ++j) load_piece(gb[j], step, slot, j);
    };

    const int frow = lane & 31, fhalf = lane >> 5;
    const int fswz = swizzle_of_row<BK>(frow);
    const int a_off = (wm0 + frow) * BK, b_off = (wn0 + frow) * BK;

    v16i acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    v4i fa[2][FM], fb[2][FN];
    auto read_frags = [&](int buf, int step, int ks) {
        const int8_t* sa = lds + ((2 * step) % 5) * SLOT + a_off;
        const int8_t* sb = lds + ((2 * step + 1) % 5) * SLOT + b_off;
        const int piece = ((2 * ks + fhalf) ^ fswz) * 16;
#pragma unroll
        for (int i = 0; i < FM; ++i) fa[buf][i] = *reinterpret_cast<const v4i*>(&sa[i * 32 * BK + piece]);
#pragma unroll
        for (int j = 0; j < FN; ++j) fb[buf][j] = *reinterpret_cast<const v4i*>(&sb[j * 32 * BK + piece]);
    };
    auto multiply = [&](int cur, auto reads_c, auto loads_c) {
        constexpr int reads = decltype(reads_c)::value, loads = decltype(loads_c)::value;
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[cur][i], fb[cur][j], acc[i][j], 0, 0, 0);
        if (SCHED) {
#pragma unroll
            for (int n = 0; n < reads / 2; ++n) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            }
#pragma unroll
            for (int n = 0; n < loads; ++n) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, FM * FN - reads / 2 - loads, 0);
        }
    };
    // thirds of a half-stage for the three early 32-byte steps
    constexpr int T1 = (RPH + 2) / 3, T2 = (2 * RPH + 2) / 3;
    // stage t, when step t+1 exists.  EARLY: A(t+2) is issued here (not for t = 0: the prologue
    // did it); LATE: B(t+2) is issued behind the barrier.
    auto stage_body = [&](int t, auto early_c, auto late_c, auto wait_next) {
        constexpr bool EARLY = decltype(early_c)::value != 0, LATE = decltype(late_c)::value != 0;
        read_frags(1, t, 1);
        if (EARLY) issue_a(t + 2, IC<0>{}, IC<T1>{});
        multiply(0, IC<FM + FN>{}, IC<(EARLY ? T1 : 0)>{});
        read_frags(0, t, 2);
        if (EARLY) issue_a(t + 2, IC<T1>{}, IC<T2>{});
        multiply(1, IC<FM + FN>{}, IC<(EARLY ? T2 - T1 : 0)>{});
        read_frags(1, t, 3);
        if (EARLY) issue_a(t + 2, IC<T2>{}, IC<RPH>{});
        multiply(0, IC<FM + FN>{}, IC<(EARLY ? RPH - T2 : 0)>{});
        wait_next();
        __builtin_amdgcn_s_barrier();
        read_frags(0, t + 1, 0);
        if (LATE) issue_b(t + 2);
        multiply(1, IC<FM + FN>{}, IC<(LATE ? RPH : 0)>{});
    };
    auto wait_one_half = [] { wait_loads_and_lds<RPH>(); };
    auto wait_all = [] { wait_loads_and_lds<0>(); };

    // prologue: A(0) B(0) A(1) B(1) A(2)
    if (nk > 0) { issue_a(0, IC<0>{}, IC<RPH>{}); issue_b(0); }
    if (nk > 1) { issue_a(1, IC<0>{}, IC<RPH>{}); issue_b(1); }
    if (nk > 2) issue_a(2, IC<0>{}, IC<RPH>{});
    if (nk > 0) {
        if (nk > 2) wait_loads_and_lds<3 * RPH>();
        else if (nk > 1) wait_loads_and_lds<2 * RPH>();
        else wait_loads_and_lds<0>();
        __builtin_amdgcn_s_barrier();
        read_frags(0, 0, 0);
    }
    int t = 0;
    if (nk > 2) {                                                   // t = 0: A(2) already in flight
        stage_body(0, IC<0>{}, IC<1>{}, wait_one_half);
        t = 1;
        for (; t + 2 < nk; ++t) stage_body(t, IC<1>{}, IC<1>{}, wait_one_half);
    }
    for (; t + 1 < nk; ++t) stage_body(t, IC<0>{}, IC<0>{}, wait_all);   // nothing left to issue
    if (nk > 0) {                                                   // last stage
        read_frags(1, t, 1);
        multiply(0, IC<FM + FN>{}, IC<0>{});
        read_frags(0, t, 2);
        multiply(1, IC<FM + FN>{}, IC<0>{});
        read_frags(1, t, 3);
        multiply(0, IC<FM + FN>{}, IC<0>{});
        multiply(1, IC<0>{}, IC<0>{});
    }

    int E = 0;
    if (MODE == kStoreF32) E = lsb_exponent(eA[0], bitsA) + (eB ? lsb_exponent(eB[0], bitsB) : 0);
    if (MODE == kStoreF32 && amax != nullptr)
        publish_absmax(store_fragments<FM, FN, MODE, true>(acc, Cv, ldc, M, N, m0 + wm0, n0 + wn0, fhalf, frow, E), amax);
    else
        store_fragments<FM, FN, MODE, false>(acc, Cv, ldc, M, N, m0 + wm0, n0 + wn0, fhalf, frow, E);
}

// split-K helpers over an M x N int32 / fp32 matrix with leading dimension ldc; grid.y walks
// rows when ldc != N, otherwise the matrix is one flat run (16-byte accesses when aligned)
__global__ __launch_bounds__(256) void k_zero_rows(int32_t* __restrict__ C, int64_t ldc, int rows, int cols) {
    for (int r = blockIdx.y; r < rows; r += gridDim.y) {
        int32_t* row = C + static_cast<int64_t>(r) * ldc;
        const bool vec = (reinterpret_cast<uintptr_t>(row) & 15u) == 0;
        const int nvec = vec ? cols >> 2 : 0;
        for (int i = blockIdx.x * 256 + threadIdx.x; i < nvec; i += gridDim.x * 256)
            reinterpret_cast<int4*>(row)[i] = make_int4(0, 0, 0, 0);
        for (int i = (nvec << 2) + blockIdx.x * 256 + threadIdx.x; i < cols; i += gridDim.x * 256) row[i] = 0;
    }
}

__global__ __launch_bounds__(256) void k_unmap_rows(int32_t* __restrict__ C, int64_t ldc, int rows, int cols,
                                                    const int32_t* __restrict__ eA, int bitsA,
                                                    const int32_t* __restrict__ eB, int bitsB, uint32_t* __restrict__ amax) {
    const int E = lsb_exponent(eA[0], bitsA) + (eB ? lsb_exponent(eB[0], bitsB) : 0);
    float m = 0.0f;
    for (int r = blockIdx.y; r < rows; r += gridDim.y) {
        int32_t* row = C + static_cast<int64_t>(r) * ldc;
        const bool vec = (reinterpret_cast<uintptr_t>(row) & 15u) == 0;
        const int nvec = vec ? cols >> 2 : 0;
        for (int i = blockIdx.x * 256 + threadIdx.x; i < nvec; i += gridDim.x * 256) {
            const int4 a = reinterpret_cast<const int4*>(row)[i];
            float4 o;
            o.x = unmap_value(a.x, E);
            o.y = unmap_value(a.y, E);
            o.z = unmap_value(a.z, E);
            o.w = unmap_value(a.w, E);
            reinterpret_cast<float4*>(row)[i] = o;
            m = fmaxf(fmaxf(m, fmaxf(fabsf(o.x), fabsf(o.y))), fmaxf(fabsf(o.z), fabsf(o.w)));
        }
        for (int i = (nvec << 2) + blockIdx.x * 256 + threadIdx.x; i < cols; i += gridDim.x * 256) {
            const float o = unmap_value(row[i], E);
            reinterpret_cast<float*>(row)[i] = o;
            m = fmaxf(m, fabsf(o));
        }
    }
    if (amax != nullptr) publish_absmax(m, amax);
}

// launch shape of the two helpers: a dense matrix is treated as one long row
static void rows_launch_shape(int64_t M, int64_t N, int64_t ldc, int* rows, int* cols, dim3* grid) {
    if (ldc == N && M * N < (int64_t{1} << 31)) {
        *rows = 1;
        *cols = static_cast<int>(M * N);
    } else {
        *rows = static_cast<int>(M);
        *cols = static_cast<int>(N);
    }
    const int gx = std::max(1, std::min(1024, (*cols / 4 + 255) / 256));
    *grid = dim3(gx, std::max(1, std::min(*rows, 65535)));
}

// int8 [rows, cols] (leading dimension ld) -> [cols, rows] contiguous, 64 x 64 tiles through LDS
__global__ __launch_bounds__(256) void k_transpose_i8(const int8_t* __restrict__ src, int64_t rows, int64_t cols,
                                                      int64_t ld, int8_t* __restrict__ dst, int tiles_c) {
    __shared__ int8_t t[64][65];
    const int64_t r0 = static_cast<int64_t>(blockIdx.x / tiles_c) * 64, c0 = static_cast<int64_t>(blockIdx.x % tiles_c) * 64;
    for (int id = threadIdx.x; id < 64 * 64; id += 256) {
        const int r = id >> 6, c = id & 63;
        if (r0 + r < rows && c0 + c < cols) t[r][c] = src[(r0 + r) * ld + c0 + c];
    }
    __syncthreads();
    for (int id = threadIdx.x; id < 64 * 64; id += 256) {
        const int c = id >> 6, r = id & 63;
        if (r0 + r < rows && c0 + c < cols) dst[(c0 + c) * rows + r0 + r] = t[r][c];
    }
}

int transpose_i8_launch(const int8_t* src, int64_t rows, int64_t cols, int64_t ld, int8_t* dst, hipStream_t s) {
    if (rows == 0 || cols == 0) return FXP_OK;
    const int64_t tr = (rows + 63) / 64, tc = (cols + 63) / 64;
    if (tr * tc >= (int64_t{1} << 31)) return FXP_ERR_DIMS;
    hipLaunchKernelGGL(k_transpose_i8, dim3(static_cast<unsigned>(tr * tc)), dim3(256), 0, s, src, rows, cols, ld, dst,
                       static_cast<int>(tc));
    return launch_status();
}

template <int BM, int BN, int BK, int WM, int WN>
static int launch_cfg(int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                      void* C, int64_t ldc, int mode, bool vec, int splits, const int32_t* eA, int bitsA,
                      const int32_t* eB, int bitsB, hipStream_t s, int64_t split_stride = 0, int* slices = nullptr,
                      Batch bt = Batch(), uint32_t* amax = nullptr, ReduceRider* ride = nullptr) {
    constexpr int NT = (BM / WM) * (BN / WN) * 64;
    const int tiles_m = static_cast<int>((M + BM - 1) / BM), tiles_n = static_cast<int>((N + BN - 1) / BN);
    int k_per_split = static_cast<int>((K + splits - 1) / splits);
    k_per_split = (k_per_split + BK - 1) / BK * BK;
    if (k_per_split == 0) k_per_split = BK;
    const int ny = K > 0 ? static_cast<int>((K + k_per_split - 1) / k_per_split) : 1;
    if (slices) *slices = ny;
    ReduceRider rider;                                          // rides only in an unsplit, unbatched launch
    if (ride != nullptr && ride->blocks != 0 && ny == 1 && bt.count == 1) {
        rider = *ride;
        rider.tiles = static_cast<unsigned>(tiles_m) * tiles_n;
        rider.front = rider.tiles >= 512;                       // several rounds of tiles: ride in the first one
        ride->blocks = 0;                                       // taken
    }
    const dim3 grid(static_cast<unsigned>(tiles_m) * tiles_n + rider.blocks, ny, bt.count), block(NT);
    const int group_m = 8;
#define FXP_GEMM_LAUNCH(VEC, MODE)                                                                                 \
    hipLaunchKernelGGL((k_gemm_nt<BM, BN, BK, WM, WN, VEC, MODE>), grid, block, 0, s, A, lda, B, ldb, C, ldc,       \
                       static_cast<int>(M), static_cast<int>(N), static_cast<int>(K), k_per_split, eA, bitsA, eB,   \
                       bitsB, tiles_m, tiles_n, group_m, split_stride, bt.a, bt.b, bt.c, amax, rider)
    if (vec) {
        if (mode == kStoreI32) FXP_GEMM_LAUNCH(true, kStoreI32);
        else if (mode == kStoreF32) FXP_GEMM_LAUNCH(true, kStoreF32);
        else FXP_GEMM_LAUNCH(true, kAtomicI32);
    } else {
        if (mode == kStoreI32) FXP_GEMM_LAUNCH(false, kStoreI32);
        else if (mode == kStoreF32) FXP_GEMM_LAUNCH(false, kStoreF32);
        else FXP_GEMM_LAUNCH(false, kAtomicI32);
    }
#undef FXP_GEMM_LAUNCH
    return launch_status();
}

template <int WM, int WN, bool SCHED = true>
static int launch_ring(int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                       void* C, int64_t ldc, int mode, int splits, const int32_t* eA, int bitsA, const int32_t* eB,
                       int bitsB, hipStream_t s, int64_t split_stride = 0, int* slices = nullptr,
                      Batch bt = Batch(), uint32_t* amax = nullptr, ReduceRider* ride = nullptr) {
    constexpr int NT = (256 / WM) * (256 / WN) * 64, BK = 128;
    const int tiles_m = static_cast<int>((M + 255) / 256), tiles_n = static_cast<int>((N + 255) / 256);
    int k_per_split = static_cast<int>((K + splits - 1) / splits);
    k_per_split = (k_per_split + BK - 1) / BK * BK;
    const int ny = static_cast<int>((K + k_per_split - 1) / k_per_split);
    if (slices) *slices = ny;
    ReduceRider rider;                                          // rides only in an unsplit, unbatched launch
    if (ride != nullptr && ride->blocks != 0 && ny == 1 && bt.count == 1) {
        rider = *ride;
        rider.tiles = static_cast<unsigned>(tiles_m) * tiles_n;
        rider.front = rider.tiles >= 512;                       // several rounds of tiles: ride in the first one
        ride->blocks = 0;                                       // taken
    }
    const dim3 grid(static_cast<unsigned>(tiles_m) * tiles_n + rider.blocks, ny, bt.count), block(NT);
    const int group_m = 8;
#define FXP_GEMM_LAUNCH(MODE)                                                                                    \
    hipLaunchKernelGGL((k_gemm_nt_ring<WM, WN, MODE, SCHED>), grid, block, 0, s, A, lda, B, ldb, C, ldc,          \
                       static_cast<int>(M), static_cast<int>(N), static_cast<int>(K), k_per_split, eA, bitsA, eB, \
                       bitsB, tiles_m, tiles_n, group_m, split_stride, bt.a, bt.b, bt.c, amax, rider)
    if (mode == kStoreI32) FXP_GEMM_LAUNCH(kStoreI32);
    else if (mode == kStoreF32) FXP_GEMM_LAUNCH(kStoreF32);
    else FXP_GEMM_LAUNCH(kAtomicI32);
#undef FXP_GEMM_LAUNCH
    return launch_status();
}

template <int BM, int BN, int BK, int WM, int WN, int STAGES, bool SCHED = true>
static int launch_dma(int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                      void* C, int64_t ldc, int mode, int splits, const int32_t* eA, int bitsA, const int32_t* eB,
                      int bitsB, hipStream_t s, int64_t split_stride = 0, int* slices = nullptr,
                      Batch bt = Batch(), uint32_t* amax = nullptr, ReduceRider* ride = nullptr) {
    constexpr int NT = (BM / WM) * (BN / WN) * 64;
    const int tiles_m = static_cast<int>((M + BM - 1) / BM), tiles_n = static_cast<int>((N + BN - 1) / BN);
    int k_per_split = static_cast<int>((K + splits - 1) / splits);
    k_per_split = (k_per_split + BK - 1) / BK * BK;
    const int ny = static_cast<int>((K + k_per_split - 1) / k_per_split);
    if (slices) *slices = ny;
    ReduceRider rider;                                          // rides only in an unsplit, unbatched launch
    if (ride != nullptr && ride->blocks != 0 && ny == 1 && bt.count == 1) {
        rider = *ride;
        rider.tiles = static_cast<unsigned>(tiles_m) * tiles_n;
        rider.front = rider.tiles >= 512;                       // several rounds of tiles: ride in the first one
        ride->blocks = 0;                                       // taken
    }
    const dim3 grid(static_cast<unsigned>(tiles_m) * tiles_n + rider.blocks, ny, bt.count), block(NT);
    const int group_m = 8;
#define FXP_GEMM_LAUNCH(MODE)                                                                                      \
    hipLaunchKernelGGL((k_gemm_nt_dma<BM, BN, BK, WM, WN, STAGES, MODE, SCHED>), grid, block, 0, s, A, lda, B, ldb, C, \
                       ldc,                                                                                        \
                       static_cast<int>(M), static_cast<int>(N), static_cast<int>(K), k_per_split, eA, bitsA, eB,   \
                       bitsB, tiles_m, tiles_n, group_m, split_stride, bt.a, bt.b, bt.c, ConvTaps(), amax, rider)
    if (mode == kStoreI32) FXP_GEMM_LAUNCH(kStoreI32);
    else if (mode == kStoreF32) FXP_GEMM_LAUNCH(kStoreF32);
    else FXP_GEMM_LAUNCH(kAtomicI32);
#undef FXP_GEMM_LAUNCH
    return launch_status();
}

__global__ __launch_bounds__(256) void k_splitk_reduce(ReduceRider r) { splitk_reduce_body(r, blockIdx.x, gridDim.x); }

// workgroups a reduction wants: one 16-byte piece of the output per thread (its loads over the slices are
// independent of each other), 256 threads per workgroup, at most 2048 workgroups
static unsigned reduce_blocks(int64_t M, int64_t N) {
    return static_cast<unsigned>(std::max<int64_t>(1, std::min<int64_t>(2048, (M * N / 4 + 255) / 256)));
}

int splitk_reduce_launch(const ReduceRider& r, hipStream_t s) {
    hipLaunchKernelGGL(k_splitk_reduce, dim3(r.blocks), dim3(256), 0, s, r);
    return launch_status();
}

// How a product is cut up.  Depends on the shape only, so that workspace sizing and launch agree.
struct GemmPlan {
    bool use256;   // 256 x 256 tiles, else 128 x 128
    int splits;    // slices of the contraction (grid.y)
    bool tall;     // split products only: 128 x 256 tiles (use256 is false then)
};

// no slice longer than one int32 sum can hold
static GemmPlan long_contraction(GemmPlan p, int64_t K) {
    if (K > kMaxContraction) p.splits = static_cast<int>(std::max<int64_t>(p.splits, (K + kMaxSlice - 1) / kMaxSlice));
    return p;
}

static GemmPlan plan_gemm(int64_t M, int64_t N, int64_t K) {
    const int num_cu = 256;
    const int64_t t256 = ((M + 255) / 256) * ((N + 255) / 256);
    const int64_t t128 = ((M + 127) / 128) * ((N + 127) / 128);
    const bool wide = M >= 256 && N >= 256;
    GemmPlan p{wide && t256 >= 96, 1, false};
    if (K >= 2048 && t256 < 64) {
        // small output, long contraction (a weight gradient): fill the chip along K, slices of 1024 or more
        if (wide && t256 >= 16) {
            // 128 x 256 tiles, about one workgroup per CU: measured on the ViT weight gradients (contraction 12608)
            // 768 x 2304: 30.8 us (4 slices) against 31.9 with 256 x 256 tiles and 7 slices; 768 x 3072: 39.0 (3)
            // against 39.5 (7) - and fewer slices to write and to sum afterwards.  Smaller outputs (768 x 768) stay
            // with 128 x 128 tiles: 19.6 us with the sum of their 7 slices against 22.0 (12 slices).
            const int64_t tiles = ((M + 127) / 128) * ((N + 255) / 256);
            p.use256 = false;
            p.tall = true;
            p.splits = static_cast<int>(std::max<int64_t>(1, std::min<int64_t>(num_cu / tiles, K / 1024)));
            return long_contraction(p, K);
        }
        p.use256 = false;
        p.splits = static_cast<int>(std::max<int64_t>(1, std::min<int64_t>((num_cu + t128 / 2) / t128, K / 1024)));
    }
    return long_contraction(p, K);
}

// elements between two workspace slices of an M x N product: a multiple of 4, so that every slice starts 16-byte
// aligned and the reduction can read all of them in 16-byte pieces
static int64_t slice_stride(int64_t M, int64_t N) { return (M * N + 3) / 4 * 4; }

// Output elements the busiest CU computes with 256 x 256 tiles (one workgroup per CU) and with 160 x 128 tiles
// (tiles dealt round-robin, two resident per CU): the smaller tiles win when they cut that by a quarter or more,
// i.e. when the large tiles leave many CUs idle or a last round nearly empty.
static bool fits_160x128(int64_t M, int64_t N) {
    const int64_t num_cu = 256;
    const int64_t t256 = ((M + 255) / 256) * ((N + 255) / 256), t160 = ((M + 159) / 160) * ((N + 127) / 128);
    const int64_t work256 = (t256 + num_cu - 1) / num_cu * (256 * 256), work160 = (t160 + num_cu - 1) / num_cu * (160 * 128);
    return 4 * work160 <= 3 * work256;
}

size_t gemm_split_ws_bytes(int64_t M, int64_t N, int64_t K) {
    const GemmPlan p = plan_gemm(M, N, K);
    return p.splits > 1 ? round_up(static_cast<size_t>(p.splits) * slice_stride(M, N) * sizeof(int32_t), 256) : 0;
}

// `batch` products of one shape in one launch (grid.z), never split along K.
int gemm_nt_batched_launch(int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda, int64_t strideA,
                           const int8_t* B, int64_t ldb, int64_t strideB, void* C, int64_t ldc, int64_t strideC,
                           int64_t batch, bool fp32_out, const int32_t* eA, int bitsA, const int32_t* eB, int bitsB,
                           hipStream_t s) {
    // the batch supplies the parallelism: no split along K, tiles chosen per matrix
    if (M == 0 || N == 0 || batch == 0) return FXP_OK;
    const bool vec = aligned(A, 16) && aligned(B, 16) && lda % 16 == 0 && ldb % 16 == 0 && K % 16 == 0 && strideA % 16 == 0 &&
                     strideB % 16 == 0;
    const bool dma = vec && K >= 64;   // K % 16 == 0: the direct-to-LDS kernels pad a partial last step with zeros
    const int64_t t256 = ((M + 255) / 256) * ((N + 255) / 256);
    const bool use256 = M >= 256 && N >= 256 && t256 * batch >= 96;
    const int mode = fp32_out ? kStoreF32 : kStoreI32;
    Batch bt;
    bt.count = static_cast<unsigned>(batch);
    bt.a = strideA; bt.b = strideB; bt.c = strideC;
#define FXP_BATCHED_ARGS M, N, K, A, lda, B, ldb, C, ldc, mode
#define FXP_BATCHED_TAIL 1, eA, bitsA, eB, bitsB, s, 0, nullptr, bt
    if (!dma) {
        // narrow outputs (head width 64 of the attention context and of dQ, dK, dV) take a tile of their own width
        if (N <= 64) return launch_cfg<128, 64, 64, 64, 32>(FXP_BATCHED_ARGS, vec, FXP_BATCHED_TAIL);
        if (M <= 64) return launch_cfg<64, 128, 64, 32, 64>(FXP_BATCHED_ARGS, vec, FXP_BATCHED_TAIL);
        return launch_cfg<128, 128, 64, 64, 64>(FXP_BATCHED_ARGS, vec, FXP_BATCHED_TAIL);
    }
    if (use256 && K % 128 == 0) return launch_ring<64, 128>(FXP_BATCHED_ARGS, FXP_BATCHED_TAIL);
    if (use256) return launch_dma<256, 256, 64, 64, 128, 4>(FXP_BATCHED_ARGS, FXP_BATCHED_TAIL);
    // narrow outputs (head width 64 of the attention context and of dQ, dK, dV): a tile of their own width
    if (N <= 64) return launch_dma<128, 64, 64, 64, 32, 4>(FXP_BATCHED_ARGS, FXP_BATCHED_TAIL);
    // one or two steps along K (scores = Q K^T with head width 64): two stages, more workgroups per CU
    if (K <= 128) return launch_dma<128, 128, 64, 64, 64, 2>(FXP_BATCHED_ARGS, FXP_BATCHED_TAIL);
    if (K % 128 == 0) return launch_dma<128, 128, 128, 64, 32, 4>(FXP_BATCHED_ARGS, FXP_BATCHED_TAIL);
    return launch_dma<128, 128, 64, 64, 64, 4>(FXP_BATCHED_ARGS, FXP_BATCHED_TAIL);
#undef FXP_BATCHED_ARGS
#undef FXP_BATCHED_TAIL
}

// C = A[M,K] * B[N,K]^T.  fp32_out: C receives the inverse-mapped fp32 values (eA, eB on
// the device), else the int32 sums.  C is overwritten in both cases.
//
// Kernel choice (measured on MI355X with mapped Gaussian operands):
//   * operands 16-byte aligned and K a multiple of 64 -> direct-to-LDS kernels, else the
//     register-staged 128 x 128 x 64 kernel with its element-wise loader;
//   * enough 256 x 256 tiles to fill the chip -> the ring kernel (K % 128 == 0) or the
//     four-stage 256 x 256 x 64 kernel; otherwise 128 x 128 tiles;
//   * output-bound products (below the ridge, wide and large output or a very short contraction) -> 128-row tiles
//     of 64 or 96 KiB of LDS, so that two workgroups are resident per CU and one stores while the other multiplies;
//   * long contraction and a small output (the weight gradient) -> split K over grid.y.
//     With workspace every slice stores its own int32 matrix and one pass sums the slices
//     and applies the inverse mapping; without it the slices add into the zeroed output
//     with int32 atomics (device-scope atomics are served at the memory side on this
//     multi-die part, about 4x slower) and a pass converts in place.  Both are exact.
//
// amax (fp32_out only, may be null): FXP_ABSMAX_WORDS device words raised so that their maximum is at least the
// IEEE bits of the largest |C| of this product.
// ride (may be null): a pending reduction of another product; if this product is launched unsplit it takes the
// reduction along (ride->blocks becomes 0), otherwise the caller still has to launch it.
// defer (may be null): if this product is split along K into workspace slices, its reduction is not launched but
// described in *defer (blocks != 0) for the caller to send along with a later launch or to launch by itself;
// the slices in ws must stay untouched until then.
int gemm_nt_launch(int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                   void* C, int64_t ldc, bool fp32_out, const int32_t* eA, int bitsA, const int32_t* eB, int bitsB,
                   void* ws, size_t ws_bytes, hipStream_t s, uint32_t* amax, ReduceRider* ride, ReduceRider* defer) {
    if (M == 0 || N == 0) return FXP_OK;
    if (!fp32_out) amax = nullptr;
    uint32_t* amax1 = nullptr;      // the product kernel publishes the maximum itself only when it writes the final fp32
    const bool vec = aligned(A, 16) && aligned(B, 16) && lda % 16 == 0 && ldb % 16 == 0 && K % 16 == 0;
    const bool dma = vec && K >= 64;   // K % 16 == 0: the direct-to-LDS kernels pad a partial last step with zeros
    const GemmPlan plan = plan_gemm(M, N, K);
    const int splits = plan.splits;
    const bool use256 = plan.use256;
    // HBM-bound by the roofline (below 625 operations per byte) with the output stream dominating: a very short
    // contraction or an output of 128 MB and more (measured: c2 dX 26.6 -> 25.0 us, ViT fc1 forward 59 -> 53 us; the
    // 256 x 256 ring kernel stays ahead on the narrower and smaller outputs)
    const bool hbm_bound = 2.0 * M * N * K < 625.0 * (static_cast<double>(M) * K + static_cast<double>(N) * K + 4.0 * M * N);
    const bool stream_out = hbm_bound && N >= 1024 && (K <= 256 || 4.0 * M * N >= 96.0 * 1024 * 1024);
    const bool to_ws = splits > 1 && ws != nullptr && aligned(ws, 16) && ws_bytes >= gemm_split_ws_bytes(M, N, K);
    const int first_mode = splits > 1 ? (to_ws ? kStoreI32 : kAtomicI32) : (fp32_out ? kStoreF32 : kStoreI32);
    void* dst = to_ws ? ws : C;
    const int64_t dst_ld = to_ws ? N : ldc;
    const int64_t split_stride = to_ws ? slice_stride(M, N) : 0;
    // beyond kMaxContraction only the 64-bit sum of workspace slices is exact
    if (K > kMaxContraction && !(to_ws && fp32_out)) return FXP_ERR_OVERFLOW;
    int hr, hc;
    dim3 hgrid;
    rows_launch_shape(M, N, ldc, &hr, &hc, &hgrid);
    if (splits == 1) amax1 = amax;
    const Batch one{};
    int rc, slices = 1;   // the launchers round a slice up to whole K steps, so fewer slices than planned may run
    if (splits > 1 && !to_ws) {
        hipLaunchKernelGGL(k_zero_rows, hgrid, dim3(256), 0, s, static_cast<int32_t*>(C), ldc, hr, hc);
        if ((rc = launch_status())) return rc;
    }
    if (!dma)
        rc = launch_cfg<128, 128, 64, 64, 64>(M, N, K, A, lda, B, ldb, dst, dst_ld, first_mode, vec, splits, eA, bitsA, eB, bitsB, s, split_stride, &slices, one, amax1, ride);
    else if (use256 && splits == 1 && stream_out && K % 128 == 0 && (K <= 256 || 4.0 * M * N < 128.0 * 1024 * 1024))
        // 64 KiB of LDS per workgroup keeps two resident per CU: one stores its tile while the other multiplies
        // (ResNet dX 25088 x 1152 x 128: 22.5 us against 27.3 with the 128 x 256 tile and 24.4 with the ring kernel;
        // ViT qkv forward 36.7 / 38.3 / 40.5; fc1 forward 48.1 / 46.9 / 54.7)
        rc = launch_dma<128, 128, 128, 64, 64, 2>(M, N, K, A, lda, B, ldb, dst, dst_ld, first_mode, 1, eA, bitsA, eB, bitsB, s, 0, nullptr, one, amax1, ride);
    else if (use256 && splits == 1 && stream_out)
        rc = launch_dma<128, 256, 64, 64, 64, 3>(M, N, K, A, lda, B, ldb, dst, dst_ld, first_mode, 1, eA, bitsA, eB, bitsB, s, 0, nullptr, one, amax1, ride);
    else if (use256 && K % 128 == 0 && splits == 1 && fits_160x128(M, N))
        // too few 256 x 256 tiles for the 256 CUs: 160 x 128 tiles, two workgroups resident per CU (one is at its
        // barrier or in its epilogue while the other multiplies).  ViT-B, 12608 x 768 outputs = 150 tiles of 256 x 256
        // against 474 of these: contraction 3072: 39.9 -> 35.2 us, 2304: 32.4 -> 28.1, 768: 16.8 -> 14.7
        rc = launch_dma<160, 128, 128, 160, 32, 2>(M, N, K, A, lda, B, ldb, dst, dst_ld, first_mode, 1, eA, bitsA, eB, bitsB, s, 0, nullptr, one, amax1, ride);
    else if (use256 && K % 128 == 0 && splits == 1)
        rc = launch_ring<64, 128>(M, N, K, A, lda, B, ldb, dst, dst_ld, first_mode, 1, eA, bitsA, eB, bitsB, s, 0, nullptr, one, amax1, ride);
    else if (plan.tall)
        rc = launch_dma<128, 256, 64, 64, 64, 3>(M, N, K, A, lda, B, ldb, dst, dst_ld, first_mode, splits, eA, bitsA, eB, bitsB, s, split_stride, &slices, one, amax1, ride);
    else if (use256)
        rc = launch_dma<256, 256, 64, 64, 128, 4>(M, N, K, A, lda, B, ldb, dst, dst_ld, first_mode, splits, eA, bitsA, eB, bitsB, s, split_stride, &slices, one, amax1, ride);
    else if (K % 128 == 0)
        rc = launch_dma<128, 128, 128, 64, 32, 4>(M, N, K, A, lda, B, ldb, dst, dst_ld, first_mode, splits, eA, bitsA, eB, bitsB, s, split_stride, &slices, one, amax1, ride);
    else
        rc = launch_dma<128, 128, 64, 64, 64, 4>(M, N, K, A, lda, B, ldb, dst, dst_ld, first_mode, splits, eA, bitsA, eB, bitsB, s, split_stride, &slices, one, amax1, ride);
    if (rc || splits == 1) return rc;
    if (to_ws) {
        ReduceRider r;
        r.parts = static_cast<const int32_t*>(ws);
        r.splits = slices;
        r.stride = split_stride;
        r.M = static_cast<int>(M);
        r.N = static_cast<int>(N);
        r.C = C;
        r.ldc = ldc;
        r.fp32_out = fp32_out ? 1 : 0;
        r.eA = eA; r.bitsA = bitsA; r.eB = eB; r.bitsB = bitsB;
        r.amax = amax;
        r.wide = K > kMaxContraction ? 1 : 0;
        r.blocks = reduce_blocks(M, N);
        if (defer != nullptr) {
            *defer = r;
            return FXP_OK;
        }
        return splitk_reduce_launch(r, s);
    }
    if (!fp32_out) return rc;
    hipLaunchKernelGGL(k_unmap_rows, hgrid, dim3(256), 0, s, static_cast<int32_t*>(C), ldc, hr, hc, eA, bitsA, eB, bitsB, amax);
    return launch_status();
}

// Y[M, Cout] = unmap(patches(Xq) * Wq^T) with the patch matrix never stored (see k_gemm_nt_dma, CONV): M output
// pixels, K = KH*KW*C.  Returns kNotApplicable when the shape needs the explicit patch matrix: channels not a
// multiple of 64 (the smallest K step), a product that plan_gemm would split along K or give 256 x 256 tiles.
template <int BK, int WN>
static int conv_gemm_launch_cfg(const ConvTaps& ct, int64_t K, int64_t M, int64_t Cout, const int8_t* Xq, const int8_t* Wq,
                                float* Y, const int32_t* eA, int bitsA, const int32_t* eB, int bitsB, hipStream_t s,
                                ReduceRider* ride) {
    constexpr int BM = 128, BN = 128, WM = 64, STAGES = 4;
    const int tiles_m = static_cast<int>((M + BM - 1) / BM), tiles_n = static_cast<int>((Cout + BN - 1) / BN);
    ReduceRider rider;
    if (ride != nullptr && ride->blocks != 0) {
        rider = *ride;
        rider.tiles = static_cast<unsigned>(tiles_m) * tiles_n;
        rider.front = rider.tiles >= 512;                       // several rounds of tiles: ride in the first one
        ride->blocks = 0;                                       // taken
    }
    const dim3 grid(static_cast<unsigned>(tiles_m) * tiles_n + rider.blocks), block((BM / WM) * (BN / WN) * 64);
    hipLaunchKernelGGL((k_gemm_nt_dma<BM, BN, BK, WM, WN, STAGES, kStoreF32, true, true>), grid, block, 0, s, Xq, K, Wq, K,
                       static_cast<void*>(Y), Cout, static_cast<int>(M), static_cast<int>(Cout), static_cast<int>(K),
                       static_cast<int>(K), eA, bitsA, eB, bitsB, tiles_m, tiles_n, 8, int64_t{0}, int64_t{0}, int64_t{0},
                       int64_t{0}, ct, static_cast<uint32_t*>(nullptr), rider);
    return launch_status();
}

int conv_gemm_launch(const ConvTaps& ct, int KH, int64_t M, int64_t Cout, const int8_t* Xq, const int8_t* Wq, float* Y,
                     const int32_t* eA, int bitsA, const int32_t* eB, int bitsB, hipStream_t s, ReduceRider* ride) {
    const int64_t K = static_cast<int64_t>(KH) * ct.KW * ct.C;
    if (ct.C % 64 != 0 || !aligned(Xq, 16) || !aligned(Wq, 16) || M <= 0 || Cout <= 0) return kNotApplicable;
    const GemmPlan plan = plan_gemm(M, Cout, K);
    if (plan.splits != 1 || plan.use256) return kNotApplicable;
    // one K step = one run of channels of one filter tap: 128 channels (8 waves) where C allows, else 64 (4 waves)
    if (ct.C % 128 == 0) return conv_gemm_launch_cfg<128, 32>(ct, K, M, Cout, Xq, Wq, Y, eA, bitsA, eB, bitsB, s, ride);
    return conv_gemm_launch_cfg<64, 64>(ct, K, M, Cout, Xq, Wq, Y, eA, bitsA, eB, bitsB, s, ride);
}

// long_k: the caller can take a contraction beyond kMaxContraction (fp32 output through workspace slices)
static int check_gemm_args(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, int transA, const void* B,
                           int64_t ldb, int transB, const void* C, int64_t ldc, bool long_k = false) {
    if (M < 0 || N < 0 || K < 0) return FXP_ERR_DIMS;
    if (M >= (int64_t{1} << 31) || N >= (int64_t{1} << 31) || K >= (int64_t{1} << 31)) return FXP_ERR_DIMS;
    if (K > kMaxContraction && !long_k) return FXP_ERR_OVERFLOW;
    if (lda < (transA ? M : K) || ldb < (transB ? K : N) || ldc < N) return FXP_ERR_DIMS;
    if ((M * N > 0 && !C) || (M * K > 0 && !A) || (N * K > 0 && !B)) return FXP_ERR_NULL;
    if (!aligned(C, 4)) return FXP_ERR_ALIGN;
    if (((M + 127) / 128) * ((N + 127) / 128) >= (int64_t{1} << 31)) return FXP_ERR_DIMS;
    return FXP_OK;
}

static size_t gemm_ws_bytes(int transA, int transB, int64_t M, int64_t N, int64_t K) {
    size_t b = 0;
    if (transA) b += round_up(static_cast<size_t>(M) * static_cast<size_t>(K), 256);
    if (!transB) b += round_up(static_cast<size_t>(N) * static_cast<size_t>(K), 256);
    return b;
}

size_t gemm_ws_worst(int64_t M, int64_t N, int64_t K) { return gemm_ws_bytes(1, 0, M, N, K) + gemm_split_ws_bytes(M, N, K); }

// Bring any operand form to the native one (transposed copies in ws), then run it.
static int gemm_any(int transA, int transB, int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda,
                    const int8_t* B, int64_t ldb, void* C, int64_t ldc, bool fp32_out, const int32_t* eA, int bitsA,
                    const int32_t* eB, int bitsB, void* ws, size_t ws_bytes, hipStream_t s, uint32_t* amax = nullptr) {
    if (M == 0 || N == 0) return FXP_OK;
    const size_t need = gemm_ws_bytes(transA, transB, M, N, K);
    if (need > 0 && (!ws || ws_bytes < need)) return FXP_ERR_WORKSPACE;
    if (ws && !aligned(ws, 256)) return FXP_ERR_ALIGN;
    // a contraction beyond one int32 sum needs the slice area behind the transposed copies (nothing is enqueued otherwise)
    if (K > kMaxContraction && (!fp32_out || !ws || ws_bytes < need + gemm_split_ws_bytes(M, N, K))) return FXP_ERR_OVERFLOW;
    int8_t* w = static_cast<int8_t*>(ws);
    int rc;
    if (transA && K > 0) {
        if ((rc = transpose_i8_launch(A, K, M, lda, w, s))) return rc;      // stored [K, M] -> [M, K]
        A = w;
        lda = K;
        w += round_up(static_cast<size_t>(M) * static_cast<size_t>(K), 256);
    }
    if (!transB && K > 0) {
        if ((rc = transpose_i8_launch(B, K, N, ldb, w, s))) return rc;      // stored [K, N] -> [N, K]
        B = w;
        ldb = K;
        w += round_up(static_cast<size_t>(N) * static_cast<size_t>(K), 256);
    }
    // what is left of the workspace serves the split-K slices (atomics are used if it is too small)
    const size_t used = static_cast<size_t>(w - static_cast<int8_t*>(ws));
    return gemm_nt_launch(M, N, K, A, lda, B, ldb, C, ldc, fp32_out, eA, bitsA, eB, bitsB, ws ? w : nullptr,
                          ws_bytes > used ? ws_bytes - used : 0, s, amax, nullptr, nullptr);
}

}  // namespace fxp

extern "C" int fxp_gemm(int transA, int transB, int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda,
                        const int8_t* B, int64_t ldb, int32_t* C, int64_t ldc, void* ws, size_t ws_bytes, void* stream) {
    int rc = fxp::check_gemm_args(M, N, K, A, lda, transA, B, ldb, transB, C, ldc);
    if (rc) return rc;
    return fxp::gemm_any(transA, transB, M, N, K, A, lda, B, ldb, C, ldc, false, nullptr, 8, nullptr, 8, ws, ws_bytes,
                         static_cast<hipStream_t>(stream));
}

extern "C" int fxp_gemm_unmap(int transA, int transB, int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda,
                              const int8_t* B, int64_t ldb, const int32_t* eA, int bitsA, const int32_t* eB, int bitsB,
                              float* C, int64_t ldc, void* ws, size_t ws_bytes, void* stream) {
    int rc = fxp::check_gemm_args(M, N, K, A, lda, transA, B, ldb, transB, C, ldc, true);
    if (rc) return rc;
    if (!eA) return FXP_ERR_NULL;
    if (bitsA < 2 || bitsA > 8 || (eB && (bitsB < 2 || bitsB > 8))) return FXP_ERR_BITS;
    return fxp::gemm_any(transA, transB, M, N, K, A, lda, B, ldb, C, ldc, true, eA, bitsA, eB, bitsB, ws, ws_bytes,
                         static_cast<hipStream_t>(stream));
}

extern "C" int fxp_gemm_unmap_absmax(int transA, int transB, int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda,
                                     const int8_t* B, int64_t ldb, const int32_t* eA, int bitsA, const int32_t* eB,
                                     int bitsB, float* C, int64_t ldc, uint32_t* out_absmax, void* ws, size_t ws_bytes,
                                     void* stream) {
    int rc = fxp::check_gemm_args(M, N, K, A, lda, transA, B, ldb, transB, C, ldc, true);
    if (rc) return rc;
    if (!eA || !out_absmax) return FXP_ERR_NULL;
    if (!fxp::aligned(out_absmax, 4)) return FXP_ERR_ALIGN;
    if (bitsA < 2 || bitsA > 8 || (eB && (bitsB < 2 || bitsB > 8))) return FXP_ERR_BITS;
    return fxp::gemm_any(transA, transB, M, N, K, A, lda, B, ldb, C, ldc, true, eA, bitsA, eB, bitsB, ws, ws_bytes,
                         static_cast<hipStream_t>(stream), out_absmax);
}

// Batched products for the attention matmuls (Q K^T and P V with per-tensor scales): `batch` independent
// C_b[M,N] = A_b[M,K] * B_b[N,K]^T, matrices of one operand strideX elements apart.
static int check_batched(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, int64_t strideA, const void* B,
                         int64_t ldb, int64_t strideB, const void* C, int64_t ldc, int64_t strideC, int64_t batch) {
    if (batch < 0 || batch > 65535 || strideA < 0 || strideB < 0 || strideC < 0) return FXP_ERR_DIMS;
    int rc = fxp::check_gemm_args(M, N, K, A, lda, 0, B, ldb, 1, C, ldc);
    if (rc) return rc;
    if (batch > 1 && M * N > 0 && strideC < (M - 1) * ldc + N) return FXP_ERR_DIMS;   // outputs must not overlap
    return FXP_OK;
}

extern "C" int fxp_gemm_batched(int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda, int64_t strideA,
                                const int8_t* B, int64_t ldb, int64_t strideB, int32_t* C, int64_t ldc, int64_t strideC,
                                int64_t batch, void* stream) {
    int rc = check_batched(M, N, K, A, lda, strideA, B, ldb, strideB, C, ldc, strideC, batch);
    if (rc) return rc;
    return fxp::gemm_nt_batched_launch(M, N, K, A, lda, strideA, B, ldb, strideB, C, ldc, strideC, batch, false, nullptr, 8,
                                       nullptr, 8, static_cast<hipStream_t>(stream));
}

extern "C" int fxp_gemm_unmap_batched(int64_t M, int64_t N, int64_t K, const int8_t* A, int64_t lda, int64_t strideA,
                                      const int8_t* B, int64_t ldb, int64_t strideB, const int32_t* eA, int bitsA,
                                      const int32_t* eB, int bitsB, float* C, int64_t ldc, int64_t strideC, int64_t batch,
                                      void* stream) {
    int rc = check_batched(M, N, K, A, lda, strideA, B, ldb, strideB, C, ldc, strideC, batch);
    if (rc) return rc;
    if (!eA) return FXP_ERR_NULL;
    if (bitsA < 2 || bitsA > 8 || (eB && (bitsB < 2 || bitsB > 8))) return FXP_ERR_BITS;
    return fxp::gemm_nt_batched_launch(M, N, K, A, lda, strideA, B, ldb, strideB, C, ldc, strideC, batch, true, eA, bitsA, eB,
                                       bitsB, static_cast<hipStream_t>(stream));
}
