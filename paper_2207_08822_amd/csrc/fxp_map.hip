// Linear fixed-point mapping fp32 -> int8 (paper Sec. 3.1) with the stochastic
// rounding of App. A.1 (Fig. 4): the 24-bit mantissa, shifted right by
// e_max - e, is cut after bits-1 magnitude bits and rounded up iff a random
// number is below the bits cut off.
//
// Kernel shape (HBM-bound by intent: 4 B read, 1 B written per copy per element;
// the Philox rounds make VALU the close second):
//   * one block = one 128 x 128 tile; each thread owns 4 x 4 element blocks, read
//     as four 16-byte loads along rows (one Philox call per load);
//   * q is written as packed dwords straight from registers (128 B per row per
//     half-wave);
//   * for the transposed copy the 4 x 4 block is transposed in registers, staged in
//     LDS as [col][row] bytes and written out in 16-byte pieces along rows of qT,
//     so both copies carry the same rounding decisions and both stores coalesce;
//   * the final step of the scale reduction (max over <= 1024 block maxima) can be
//     folded in, which saves a launch per tensor.
// The random word of element i is word (i mod 4) of Philox-4x32-10 with key = seed
// and counter = (i / 4, stream_id): nothing depends on the launch geometry.
#include <algorithm>

#include "fxp_internal.h"

namespace fxp {

constexpr int kMapThreads = 256;

struct MapCfg {
    int e_max;
    int cut;        // low bits dropped: 24 - (bits - 1)
    int rshift;     // 32 - cut: the random number is the top `cut` bits of the word
    uint32_t sat;   // 2^(bits-1) - 1
    uint32_t half;  // 2^(cut-1), the nearest-rounding increment
    uint32_t low_mask;  // 2^cut - 1
    float to_units;     // 2^(150 - e_max): |x| * to_units = the 24-bit mantissa shifted to the scale (e_max in [25, 254])
    float limit;        // 2^(e_max - 126): magnitudes from here on are above the scale (+Inf for e_max = 254)
};

// Magnitude of one element, every case: non-finite input, scale below the element.
template <bool STOCH>
__device__ inline uint32_t magnitude_full(uint32_t b, uint32_t word, const MapCfg& c) {
    const uint32_t e = (b >> 23) & 0xffu, f = b & 0x7fffffu;
    if (e == 255u) return f == 0u ? c.sat : 0u;
    const int d = c.e_max - static_cast<int>(max(e, 1u));
    if (d < 0) return c.sat;
    const uint32_t m = f | (e ? 0x800000u : 0u);
    const uint32_t mp = m >> min(d, 31);
    const uint32_t add = STOCH ? ((~word) >> c.rshift) : c.half;
    return min((mp + add) >> c.cut, c.sat);
}

// Same for the common case: e_max in [25, 254], no element above the scale, no result above the largest
// magnitude.  The shifted mantissa m >> (e_max - e) is the integer part of |x| * 2^(150 - e_max): the factor is a
// power of two (a normal float for these scales), so the product is exact whenever it is 1 or more and below 1
// otherwise, sub-normal inputs included, and the conversion truncates - two instructions for unpack, hidden
// bit, clamp and shift.  r < low  <=>  low + (2^cut - 1 - r) carries out of the cut.  `bad` collects, as a lane
// mask (one compare per element, accumulated on the scalar side), the lanes with an element the scale does not
// cover (exponent above it, Inf, NaN); the caller also ORs the results (a bit above the magnitude bits = needs
// the saturating path) and redoes the block with magnitude_full if either fires.
template <bool STOCH>
__device__ inline uint32_t magnitude_fast(uint32_t b, uint32_t word, const MapCfg& c, uint64_t& bad) {
    const float ax = fabsf(__uint_as_float(b));
    bad |= __builtin_amdgcn_ballot_w64(!(ax < c.limit));
    const uint32_t mp = static_cast<uint32_t>(ax * c.to_units);
    const uint32_t add = STOCH ? ((word >> c.rshift) ^ c.low_mask) : c.half;
    return (mp + add) >> c.cut;
}

__device__ inline uint32_t with_sign(uint32_t mag, uint32_t b) {
    const uint32_t sm = static_cast<uint32_t>(static_cast<int32_t>(b) >> 31);
    return (mag ^ sm) - sm;
}

// the four signed results of a 16-byte load as one dword, low bytes in element order
__device__ inline uint32_t pack4(uint32_t q0, uint32_t q1, uint32_t q2, uint32_t q3, const uint4 v) {
    const uint32_t p01 = perm(with_sign(q1, v.y), with_sign(q0, v.x), 0x0c0c0400u);
    const uint32_t p23 = perm(with_sign(q3, v.w), with_sign(q2, v.z), 0x0c0c0400u);
    return perm(p23, p01, 0x05040100u);
}


__device__ inline MapCfg make_cfg(int e_max, int bits) {
    MapCfg c;
    c.e_max = e_max;
    c.cut = 24 - (bits - 1);
    c.rshift = 32 - c.cut;
    c.sat = (1u << (bits - 1)) - 1u;
    c.half = 1u << (c.cut - 1);
    c.low_mask = (1u << c.cut) - 1u;
    const int e = min(max(e_max, 25), 254);                       // outside: the fast path is not taken
    c.to_units = __uint_as_float(static_cast<uint32_t>(277 - e) << 23);
    c.limit = __uint_as_float(static_cast<uint32_t>(e + 1) << 23);
    return c;
}

// One tensor of a map launch.  A launch carries up to two (the activation and the weight of a forward pass):
// the first `blocks` workgroups belong to job 0, the rest to job 1.
struct MapJob {
    const uint32_t* x;
    int64_t rows, cols;
    const int32_t* e_in;
    const uint32_t* partials;
    int n_partials;
    int32_t* e_out;
    int8_t* q;
    int8_t* qT;
    uint32_t sid0, sid1;
    int tiles_c;
    unsigned blocks;
    unsigned xcd_blocks;    // leading workgroups whose tiles are numbered per XCD (see tile_of_workgroup)
    // scale taken as a guess (see k_map_tile_guess): where the guess comes from, where the workgroup maxima of
    // the guessing launch go, and the word that records which guess the tensor was mapped with (0 = none)
    const int32_t* e_guess;
    uint32_t* guess_partials;
    int32_t* guess_used;
};
struct MapJobs {
    MapJob j[2];
};

// Row block and column block of workgroup `bid` of a tensor.  Plain numbering walks the column tiles of a row
// block first.  Where a row is not a whole number of 128-byte lines, neighbouring column tiles share the lines
// their boundary falls into, and workgroups are dealt to the eight XCDs in turn, each with an L2 of its own: such a
// tensor numbers its tiles so that the column tiles of one row block are eight workgroups apart - the same XCD,
// one after the other - and the shared lines come from that L2 the second time (row blocks beyond the last
// whole group of eight keep the plain numbering).
__device__ inline void tile_of_workgroup(const MapJob& J, unsigned bid, unsigned* rb, unsigned* cb) {
    const unsigned tc = static_cast<unsigned>(J.tiles_c);
    if (bid < J.xcd_blocks) {
        const unsigned group = bid / (8u * tc), local = bid % (8u * tc);
        *rb = group * 8u + (local & 7u);
        *cb = local >> 3;
    } else {
        const unsigned i = bid - J.xcd_blocks;
        *rb = J.xcd_blocks / tc + i / tc;
        *cb = i % tc;
    }
}

// scale of the tensor: either given, or the max of the per-block maxima (and then
// block 0 publishes it)
__device__ inline int resolve_scale(const int32_t* e_in, const uint32_t* partials, int n_partials, int32_t* e_out,
                                    uint32_t* red, bool publish) {
    if (partials == nullptr) return e_in[0];
    uint32_t m = 0;
    for (int i = threadIdx.x; i < n_partials; i += blockDim.x) m = max(m, partials[i]);
    m = block_max(m, red);
    const int e = max(1, static_cast<int>(m >> 23));
    if (publish && threadIdx.x == 0) e_out[0] = e;
    return e;
}

// One tile of TC columns (128, or 64 for tensors whose width pads less that way: head width 64 of the
// attention operands) and TR = 1024 / TC * 4 * PASSES rows: every thread owns 4 x 4 elements per pass, the 256
// threads of a pass cover 32 x 128 or 64 x 64.  PASSES = 4 for large tensors, 2 or 1 when the tensor is too small
// to fill the chip with the taller tiles.  EDGE = the tile sticks out of the tensor: loads are clamped to valid
// addresses and stores are predicated; interior tiles carry no bounds code at all.  All
// per-thread addressing is a 32-bit element offset from the tile's (wave-uniform) origin.
// GUESS: the scale is not resolved from block maxima but given (e_given; do_map = false: there is none, only the
// maximum is wanted), and the largest magnitude bits of the tile are accumulated into tile_max (clamped loads
// of an edge tile repeat elements of the tensor, which a maximum does not mind).
template <bool STOCH, bool EDGE, int PASSES, int TC, bool GUESS = false>
__device__ inline void map_tile_body(const uint32_t* __restrict__ x, int64_t rows, int64_t cols, const MapJob& J, int bits,
                                     bool publish, uint32_t* red, int8_t* __restrict__ q, int8_t* __restrict__ qT,
                                     uint32_t key0, uint32_t key1, uint32_t sid0, uint32_t sid1, int64_t r0, int64_t c0,
                                     uint32_t* stage, int e_given = 0, bool do_map = true, uint32_t* tile_max = nullptr) {
    constexpr int CG = TC / 4;                    // groups of 4 columns
    constexpr int RGP = kMapThreads / CG;         // groups of 4 rows per pass
    constexpr int TR = 4 * RGP * PASSES;          // rows of the tile
    constexpr int TS = RGP * PASSES + 1;          // dwords per staged column (TR row bytes + 4 pad)
    const int tid = threadIdx.x;
    const int cg = tid % CG;                      // group of 4 columns
    const int rgl = tid / CG;                     // group of 4 rows within a pass
    const uint32_t ucols = static_cast<uint32_t>(cols);
    const int64_t origin = r0 * cols + c0;        // element index of the tile's first element (multiple of 4)
    const uint32_t* xt = x + origin;
    int8_t* qt = q ? q + origin : nullptr;
    const uint64_t blk0 = static_cast<uint64_t>(origin) >> 2;
    const int rows_here = EDGE ? static_cast<int>(min<int64_t>(TR, rows - r0)) : TR;
    const int cols_here = EDGE ? static_cast<int>(min<int64_t>(TC, cols - c0)) : TC;
    const bool col_ok = !EDGE || 4 * cg < cols_here;
    const uint32_t col_ld = EDGE ? static_cast<uint32_t>(min(4 * cg, cols_here - 4)) : 4 * cg;

    // PASSES passes of 4 * RGP rows.  The loads of pass p+1 are issued before the arithmetic of pass
    // p, so a block keeps the memory pipe busy while it runs its Philox rounds.
    auto load_pass = [&](int p, uint4 (&v)[4]) {
        const int lrow = 4 * (p * RGP + rgl);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int rr = EDGE ? min(lrow + k, rows_here - 1) : lrow + k;
            v[k] = *reinterpret_cast<const uint4*>(xt + static_cast<uint32_t>(rr) * ucols + col_ld);
        }
    };
    uint4 cur[4], nxt[4];
    load_pass(0, cur);
    // the scale is resolved (block maxima re-read and reduced) while the first loads are in flight
    const MapCfg cfg = make_cfg(GUESS ? e_given : resolve_scale(J.e_in, J.partials, J.n_partials, J.e_out, red, publish), bits);
    const bool scale_ok = cfg.e_max >= 25 && cfg.e_max < 255;
    const uint32_t over_bits = ~cfg.sat;          // a fast-path result with any of these set needs saturation
    uint32_t seen = 0;                             // GUESS: largest magnitude bits this thread has loaded
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int rg = p * RGP + rgl;              // group of 4 rows
        const int lrow = 4 * rg;
        if (p + 1 < PASSES) load_pass(p + 1, nxt);
        if (GUESS) {
#pragma unroll
            for (int k = 0; k < 4; ++k) seen = max(seen, absmax4(cur[k]));
            if (!do_map) {                         // workgroup-uniform: no scale to map with, the maximum is all
#pragma unroll
                for (int k = 0; k < 4; ++k) cur[k] = nxt[k];
                continue;
            }
        }
        auto words_of = [&](int k) {
            const uint32_t off = static_cast<uint32_t>(lrow + k) * ucols + 4 * cg;   // element offset in the tile
            const uint64_t blk = blk0 + (off >> 2);
            return STOCH ? philox4x32_10(static_cast<uint32_t>(blk), static_cast<uint32_t>(blk >> 32), sid0, sid1, key0, key1)
                         : make_uint4(0, 0, 0, 0);
        };
        uint32_t o[4];
        uint32_t q_or = 0;
        uint64_t bad = 0;                          // wave-uniform: any lane with an uncovered element
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint4 w = words_of(k);
            const uint32_t m0 = magnitude_fast<STOCH>(cur[k].x, w.x, cfg, bad);
            const uint32_t m1 = magnitude_fast<STOCH>(cur[k].y, w.y, cfg, bad);
            const uint32_t m2 = magnitude_fast<STOCH>(cur[k].z, w.z, cfg, bad);
            const uint32_t m3 = magnitude_fast<STOCH>(cur[k].w, w.w, cfg, bad);
            q_or |= m0 | m1 | m2 | m3;
            o[k] = pack4(m0, m1, m2, m3, cur[k]);
        }
        if (!scale_ok || bad != 0 || (q_or & over_bits)) {
            // rare: an element above the scale, a saturating result, a non-finite input or a tiny
            // scale somewhere in this 4 x 4 block: redo it with the complete per-element path
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint4 w = words_of(k);
                o[k] = pack4(magnitude_full<STOCH>(cur[k].x, w.x, cfg), magnitude_full<STOCH>(cur[k].y, w.y, cfg),
                             magnitude_full<STOCH>(cur[k].z, w.z, cfg), magnitude_full<STOCH>(cur[k].w, w.w, cfg), cur[k]);
            }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (qt != nullptr && col_ok && (!EDGE || lrow + k < rows_here))
                *reinterpret_cast<uint32_t*>(qt + static_cast<uint32_t>(lrow + k) * ucols + 4 * cg) = o[k];
        if (qT != nullptr) {
            uint32_t t[4];                          // t[c] = column c of the block, rows in ascending byte order
            transpose4x4(o, t);
#pragma unroll
            for (int c = 0; c < 4; ++c) stage[(4 * cg + c) * TS + rg] = t[c];
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) cur[k] = nxt[k];
    }
    if (GUESS) *tile_max = max(*tile_max, seen);
    if (qT == nullptr || (GUESS && !do_map)) return;
    __syncthreads();
    int8_t* qTt = qT + c0 * rows + r0;             // element [c0][r0] of the transposed copy
    const uint32_t urows = static_cast<uint32_t>(rows);
    if ((rows & 15) == 0) {
        // 16 rows of one column = 16 contiguous bytes of qT
        constexpr int PIECES = TR / 16;                     // per column
#pragma unroll
        for (int it = 0; it < (TC * PIECES + kMapThreads - 1) / kMapThreads; ++it) {
            const int id = it * kMapThreads + tid;
            const int c = id / PIECES, ch = id % PIECES;
            if (c < TC && (!EDGE || (c < cols_here && 16 * ch < rows_here))) {
                const uint32_t* src = stage + c * TS + 4 * ch;
                *reinterpret_cast<uint4*>(qTt + static_cast<uint64_t>(c) * urows + 16 * ch) =
                    make_uint4(src[0], src[1], src[2], src[3]);
            }
        }
    } else {
        const uint8_t* bytes = reinterpret_cast<const uint8_t*>(stage);
        for (int id = tid; id < TC * TR; id += kMapThreads) {
            const int c = id / TR, r = id % TR;
            if (c < cols_here && r < rows_here)
                qTt[static_cast<uint64_t>(c) * urows + r] = static_cast<int8_t>(bytes[c * TS * 4 + r]);
        }
    }
}

template <bool STOCH, int PASSES, int TC>
__global__ __launch_bounds__(kMapThreads) void k_map_tile(const MapJobs jobs, uint32_t key0, uint32_t key1, int bits) {
    constexpr int RGP = kMapThreads / (TC / 4);
    constexpr int TR = 4 * RGP * PASSES;
    __shared__ uint32_t stage[TC * (RGP * PASSES + 1)];
    __shared__ uint32_t red[kMapThreads / 64];
    const bool second = blockIdx.x >= jobs.j[0].blocks;            // workgroup-uniform
    const MapJob& J = jobs.j[second ? 1 : 0];
    const unsigned bid = blockIdx.x - (second ? jobs.j[0].blocks : 0u);
    if (J.guess_used != nullptr) {
        // this launch follows k_map_tile_guess: the tensor is already mapped if the guess was its scale - then
        // the scale is published and nothing else is left to do; otherwise the tile is mapped now
        const int e = resolve_scale(nullptr, J.partials, J.n_partials, J.e_out, red, bid == 0);
        if (J.guess_used[0] == e) return;
    }
    const uint32_t* __restrict__ x = J.x;
    int8_t* __restrict__ q = J.q;
    int8_t* __restrict__ qT = J.qT;
    const int64_t rows = J.rows, cols = J.cols;
    unsigned rb, cb;
    tile_of_workgroup(J, bid, &rb, &cb);
    const int64_t r0 = static_cast<int64_t>(rb) * TR;
    const int64_t c0 = static_cast<int64_t>(cb) * TC;
    if (r0 + TR <= rows && c0 + TC <= cols)
        map_tile_body<STOCH, false, PASSES, TC>(x, rows, cols, J, bits, bid == 0, red, q, qT, key0, key1, J.sid0, J.sid1, r0, c0, stage);
    else
        map_tile_body<STOCH, true, PASSES, TC>(x, rows, cols, J, bits, bid == 0, red, q, qT, key0, key1, J.sid0, J.sid1, r0, c0, stage);
}

// Scale and map in ONE pass over the tensor, for a caller that has a guess of the scale (the tensor's scale of
// the previous training step: the largest exponent of a weight, an activation or a gradient tensor seldom moves
// from one step to the next).  Every workgroup maps its tiles with the guess and keeps the largest magnitude it
// saw; the launch leaves one maximum per workgroup (at most kGuessBlocks, so that the launch that follows can
// reduce them like block maxima) and the guess it used.  The launch that follows (k_map_tile with guess_used
// set) computes the true scale from the maxima: equal to the guess - the bytes written here are exactly what the
// two-pass path writes, and that launch ends at once; different, or no usable guess (outside 1 .. 255) - it
// maps the tensor again with the true scale.  4 B read + 2 B written per element instead of 8 + 2 on a hit.
template <bool STOCH, int PASSES, int TC>
__global__ __launch_bounds__(kMapThreads) void k_map_tile_guess(const MapJobs jobs, uint32_t key0, uint32_t key1, int bits) {
    constexpr int RGP = kMapThreads / (TC / 4);
    constexpr int TR = 4 * RGP * PASSES;
    __shared__ uint32_t stage[TC * (RGP * PASSES + 1)];
    __shared__ uint32_t red[kMapThreads / 64];
    int guess[2];
    uint32_t seen[2] = {0u, 0u};
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        guess[j] = jobs.j[j].blocks != 0 ? jobs.j[j].e_guess[0] : 0;
        if (guess[j] < 1 || guess[j] > 255) guess[j] = 0;
        if (jobs.j[j].blocks != 0 && blockIdx.x == 0 && threadIdx.x == 0) jobs.j[j].guess_used[0] = guess[j];
    }
    const unsigned total = jobs.j[0].blocks + jobs.j[1].blocks;
    for (unsigned tile = blockIdx.x; tile < total; tile += gridDim.x) {
        const int which = tile >= jobs.j[0].blocks ? 1 : 0;       // workgroup-uniform
        const MapJob& J = jobs.j[which];
        const unsigned bid = tile - (which ? jobs.j[0].blocks : 0u);
        unsigned rb, cb;
        tile_of_workgroup(J, bid, &rb, &cb);
        const int64_t r0 = static_cast<int64_t>(rb) * TR;
        const int64_t c0 = static_cast<int64_t>(cb) * TC;
        uint32_t m = 0;
        if (r0 + TR <= J.rows && c0 + TC <= J.cols)
            map_tile_body<STOCH, false, PASSES, TC, true>(J.x, J.rows, J.cols, J, bits, false, red, J.q, J.qT, key0, key1, J.sid0,
                                                          J.sid1, r0, c0, stage, guess[which], guess[which] != 0, &m);
        else
            map_tile_body<STOCH, true, PASSES, TC, true>(J.x, J.rows, J.cols, J, bits, false, red, J.q, J.qT, key0, key1, J.sid0,
                                                         J.sid1, r0, c0, stage, guess[which], guess[which] != 0, &m);
        seen[which] = max(seen[which], m);
        __syncthreads();      // the staging area is read by other threads than those that fill it for the next tile
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        if (jobs.j[j].blocks == 0) continue;
        const uint32_t m = block_max(seen[j], red);
        if (threadIdx.x == 0) jobs.j[j].guess_partials[blockIdx.x] = m;
    }
}

// One element per thread, any shape and alignment.
template <bool STOCH>
__global__ __launch_bounds__(kMapThreads) void k_map_generic(const uint32_t* __restrict__ x, int64_t rows, int64_t cols,
                                                             const int32_t* __restrict__ e_in,
                                                             const uint32_t* __restrict__ partials, int n_partials,
                                                             int32_t* __restrict__ e_out, int8_t* __restrict__ q,
                                                             int8_t* __restrict__ qT, uint32_t key0, uint32_t key1,
                                                             uint32_t sid0, uint32_t sid1, int bits) {
    __shared__ uint32_t red[kMapThreads / 64];
    const MapCfg cfg = make_cfg(resolve_scale(e_in, partials, n_partials, e_out, red, blockIdx.x == 0), bits);
    const uint64_t n = static_cast<uint64_t>(rows) * static_cast<uint64_t>(cols);
    for (uint64_t i = static_cast<uint64_t>(blockIdx.x) * kMapThreads + threadIdx.x; i < n;
         i += static_cast<uint64_t>(gridDim.x) * kMapThreads) {
        const uint32_t b = x[i];
        uint32_t word = 0;
        if (STOCH) {
            const uint64_t blk = i >> 2;
            const uint4 w = philox4x32_10(static_cast<uint32_t>(blk), static_cast<uint32_t>(blk >> 32), sid0, sid1, key0, key1);
            const uint32_t sel = static_cast<uint32_t>(i & 3u);
            word = sel == 0 ? w.x : sel == 1 ? w.y : sel == 2 ? w.z : w.w;
        }
        const int8_t v = static_cast<int8_t>(with_sign(magnitude_full<STOCH>(b, word, cfg), b));
        if (q) q[i] = v;
        if (qT) {
            const uint64_t r = i / static_cast<uint64_t>(cols), c = i % static_cast<uint64_t>(cols);
            qT[c * static_cast<uint64_t>(rows) + r] = v;
        }
    }
}

// how one tensor would be tiled
struct MapPlan {
    int tc;          // tile columns
    int passes;      // 4, 2 or 1
    bool tile_path;  // false: the one-element-per-thread kernel
};

static MapPlan plan_map(const MapTensor& t) {
    MapPlan p;
    // tile width: 64 when that pads the rows less than 128 does (cols = 64, 192, ...)
    p.tc = ((t.cols + 63) / 64) * 64 < ((t.cols + 127) / 128) * 128 ? 64 : 128;
    const int64_t tall = p.tc == 128 ? 128 : 256;   // rows of a 4-pass tile
    const int64_t tiles_c = (t.cols + p.tc - 1) / p.tc;
    // four passes per tile when that still gives a thousand workgroups (four per CU), else two, else single-pass
    // tiles (a sweep of the threshold from 512 to 8192 moved whole-step times by under 3 %)
    auto count = [&](int64_t tile_rows) { return ((t.rows + tile_rows - 1) / tile_rows) * tiles_c; };
    p.passes = count(tall) >= 1024 ? 4 : (count(tall / 2) >= 1024 ? 2 : 1);
    p.tile_path = (t.cols % 4 == 0) && aligned(t.x, 16) && (!t.q || aligned(t.q, 16)) && (!t.qT || aligned(t.qT, 16)) &&
                  t.rows > 0 && count(tall / 4) < (int64_t{1} << 30) && t.cols < (int64_t{1} << 22) &&   // 32-bit offsets inside a tile
                  t.rows < (int64_t{1} << 32);                        // and a 32-bit row count in the transposed copy's addressing
    return p;
}

static MapJob make_job(const MapTensor& t, int tc, int passes) {
    MapJob j;
    const int64_t tr = (tc == 128 ? 128 : 256) / 4 * passes;
    j.x = reinterpret_cast<const uint32_t*>(t.x);
    j.rows = t.rows;
    j.cols = t.cols;
    j.e_in = t.e_in;
    j.partials = t.partials;
    j.n_partials = t.n_partials;
    j.e_out = t.e_out;
    j.q = t.q;
    j.qT = t.qT;
    j.sid0 = static_cast<uint32_t>(t.stream_id);
    j.sid1 = static_cast<uint32_t>(t.stream_id >> 32);
    j.tiles_c = static_cast<int>((t.cols + tc - 1) / tc);
    j.blocks = static_cast<unsigned>(((t.rows + tr - 1) / tr) * j.tiles_c);
    const bool shared_lines = j.tiles_c > 1 && t.cols % 128 != 0;
    j.xcd_blocks = shared_lines ? static_cast<unsigned>((t.rows + tr - 1) / tr / 8 * 8 * j.tiles_c) : 0u;
    j.e_guess = nullptr;
    j.guess_partials = nullptr;
    j.guess_used = nullptr;
    return j;
}

static void launch_tiles(const MapJobs& jobs, int tc, int passes, bool stoch, uint32_t k0, uint32_t k1, int bits,
                         hipStream_t s) {
    const dim3 grid(jobs.j[0].blocks + jobs.j[1].blocks), block(kMapThreads);
#define FXP_MAP_LAUNCH(STOCH, PASSES, TC) \
    hipLaunchKernelGGL((k_map_tile<STOCH, PASSES, TC>), grid, block, 0, s, jobs, k0, k1, bits)
#define FXP_MAP_PICK(TC)                                   \
    if (stoch) {                                           \
        if (passes == 4) FXP_MAP_LAUNCH(true, 4, TC);      \
        else if (passes == 2) FXP_MAP_LAUNCH(true, 2, TC); \
        else FXP_MAP_LAUNCH(true, 1, TC);                  \
    } else {                                               \
        if (passes == 4) FXP_MAP_LAUNCH(false, 4, TC);     \
        else if (passes == 2) FXP_MAP_LAUNCH(false, 2, TC);\
        else FXP_MAP_LAUNCH(false, 1, TC);                 \
    }
    if (tc == 128) { FXP_MAP_PICK(128); }
    else { FXP_MAP_PICK(64); }
#undef FXP_MAP_PICK
#undef FXP_MAP_LAUNCH
}

static void launch_tiles_guess(const MapJobs& jobs, unsigned grid_x, int tc, int passes, bool stoch, uint32_t k0, uint32_t k1,
                               int bits, hipStream_t s) {
    const dim3 grid(grid_x), block(kMapThreads);
#define FXP_MAP_LAUNCH(STOCH, PASSES, TC) \
    hipLaunchKernelGGL((k_map_tile_guess<STOCH, PASSES, TC>), grid, block, 0, s, jobs, k0, k1, bits)
#define FXP_MAP_PICK(TC)                                   \
    if (stoch) {                                           \
        if (passes == 4) FXP_MAP_LAUNCH(true, 4, TC);      \
        else if (passes == 2) FXP_MAP_LAUNCH(true, 2, TC); \
        else FXP_MAP_LAUNCH(true, 1, TC);                  \
    } else {                                               \
        if (passes == 4) FXP_MAP_LAUNCH(false, 4, TC);     \
        else if (passes == 2) FXP_MAP_LAUNCH(false, 2, TC);\
        else FXP_MAP_LAUNCH(false, 1, TC);                 \
    }
    if (tc == 128) { FXP_MAP_PICK(128); }
    else { FXP_MAP_PICK(64); }
#undef FXP_MAP_PICK
#undef FXP_MAP_LAUNCH
}

// Scale + map of one or two tensors (b may be null) with the scales their e_out words hold on entry taken as
// guesses: one pass over the tensors and a launch that verifies (and repairs, should a guess be off).  area_a /
// area_b: kMaxPartials words of scratch each.  Returns kNoGuessPath when the tensors do not take the tiled
// kernel together or are too small for the guess to pay (the caller then takes the two-pass path).
int scale_map_guess_launch(const MapTensor& a, const MapTensor* b, uint32_t* area_a, uint32_t* area_b, uint64_t seed,
                           int rounding, int bits, hipStream_t s) {
    const MapPlan pa = plan_map(a);
    const MapPlan pb = b ? plan_map(*b) : pa;
    const int64_t na = a.rows * a.cols, nb = b ? b->rows * b->cols : 0;
    // below a few million elements a scale reduction costs what the verifying launch costs
    if (std::max(na, nb) < kGuessMinElements) return kNoGuessPath;
    if (!pa.tile_path || !pb.tile_path) return kNoGuessPath;
    if (pa.tc != pb.tc) return kGuessOneByOne;        // different tile widths: no common launch, but each may guess alone
    const int passes = na >= nb ? pa.passes : pb.passes;
    MapJobs jobs;
    jobs.j[0] = make_job(a, pa.tc, passes);
    if (b) jobs.j[1] = make_job(*b, pa.tc, passes);
    else { jobs.j[1] = jobs.j[0]; jobs.j[1].blocks = 0; }
    const uint64_t total = static_cast<uint64_t>(jobs.j[0].blocks) + jobs.j[1].blocks;
    if (total >= (uint64_t{1} << 31)) return kNoGuessPath;
    const unsigned grid = static_cast<unsigned>(std::min<uint64_t>(total, kGuessBlocks));
    uint32_t* areas[2] = {area_a, area_b};
    const MapTensor* ts[2] = {&a, b};
    for (int j = 0; j < 2; ++j) {
        if (jobs.j[j].blocks == 0) continue;
        jobs.j[j].e_guess = ts[j]->e_out;                                   // last step's scale, if the caller kept it
        jobs.j[j].guess_partials = areas[j];
        jobs.j[j].guess_used = reinterpret_cast<int32_t*>(areas[j] + kGuessBlocks);
        jobs.j[j].e_in = nullptr;
        jobs.j[j].partials = nullptr;
    }
    const bool stoch = rounding == FXP_ROUND_STOCHASTIC;
    const uint32_t k0 = static_cast<uint32_t>(seed), k1 = static_cast<uint32_t>(seed >> 32);
    launch_tiles_guess(jobs, grid, pa.tc, passes, stoch, k0, k1, bits, s);
    int rc = launch_status();
    if (rc) return rc;
    // the launch that verifies: an ordinary map launch that takes the workgroup maxima as block maxima
    for (int j = 0; j < 2; ++j) {
        if (jobs.j[j].blocks == 0) continue;
        jobs.j[j].partials = areas[j];
        jobs.j[j].n_partials = static_cast<int>(grid);
    }
    launch_tiles(jobs, pa.tc, passes, stoch, k0, k1, bits, s);
    return launch_status();
}

int map_launch(const MapTensor& t, uint64_t seed, int rounding, int bits, hipStream_t s) {
    const uint32_t k0 = static_cast<uint32_t>(seed), k1 = static_cast<uint32_t>(seed >> 32);
    const bool stoch = rounding == FXP_ROUND_STOCHASTIC;
    const MapPlan p = plan_map(t);
    if (p.tile_path) {
        MapJobs jobs;
        jobs.j[0] = make_job(t, p.tc, p.passes);
        jobs.j[1] = jobs.j[0];
        jobs.j[1].blocks = 0;
        launch_tiles(jobs, p.tc, p.passes, stoch, k0, k1, bits, s);
    } else {
        const uint32_t s0 = static_cast<uint32_t>(t.stream_id), s1 = static_cast<uint32_t>(t.stream_id >> 32);
        const uint32_t* xb = reinterpret_cast<const uint32_t*>(t.x);
        const uint64_t n = static_cast<uint64_t>(t.rows) * static_cast<uint64_t>(t.cols);
        uint64_t want = (n + kMapThreads - 1) / kMapThreads;
        const dim3 grid(static_cast<unsigned>(want < 1 ? 1 : (want > 16384 ? 16384 : want))), block(kMapThreads);
        if (stoch)
            hipLaunchKernelGGL(k_map_generic<true>, grid, block, 0, s, xb, t.rows, t.cols, t.e_in, t.partials, t.n_partials,
                               t.e_out, t.q, t.qT, k0, k1, s0, s1, bits);
        else
            hipLaunchKernelGGL(k_map_generic<false>, grid, block, 0, s, xb, t.rows, t.cols, t.e_in, t.partials, t.n_partials,
                               t.e_out, t.q, t.qT, k0, k1, s0, s1, bits);
    }
    return launch_status();
}

// Two tensors in one launch when both take the tiled kernel with the same tile width; the tile height is the
// one the larger tensor would pick.  Otherwise one launch each.
int map_launch2(const MapTensor& a, const MapTensor& b, uint64_t seed, int rounding, int bits, hipStream_t s) {
    const MapPlan pa = plan_map(a), pb = plan_map(b);
    if (!pa.tile_path || !pb.tile_path || pa.tc != pb.tc) {
        const int rc = map_launch(a, seed, rounding, bits, s);
        return rc ? rc : map_launch(b, seed, rounding, bits, s);
    }
    const int passes = a.rows * a.cols >= b.rows * b.cols ? pa.passes : pb.passes;
    MapJobs jobs;
    jobs.j[0] = make_job(a, pa.tc, passes);
    jobs.j[1] = make_job(b, pa.tc, passes);
    if (static_cast<uint64_t>(jobs.j[0].blocks) + jobs.j[1].blocks >= (uint64_t{1} << 31)) {
        const int rc = map_launch(a, seed, rounding, bits, s);
        return rc ? rc : map_launch(b, seed, rounding, bits, s);
    }
    launch_tiles(jobs, pa.tc, passes, rounding == FXP_ROUND_STOCHASTIC, static_cast<uint32_t>(seed),
                 static_cast<uint32_t>(seed >> 32), bits, s);
    return launch_status();
}

static int check_map_args(const float* x, int64_t rows, int64_t cols, const void* e, int8_t* q, int8_t* qT, int rounding,
                          int bits) {
    if (rows < 0 || cols < 0) return FXP_ERR_DIMS;
    if (rows > 0 && cols > 0 && rows > (int64_t{1} << 62) / cols) return FXP_ERR_DIMS;
    if (!e || (!q && !qT) || (rows * cols > 0 && !x)) return FXP_ERR_NULL;
    if (rounding != FXP_ROUND_STOCHASTIC && rounding != FXP_ROUND_NEAREST) return FXP_ERR_ROUNDING;
    if (bits < 2 || bits > 8) return FXP_ERR_BITS;
    if (!aligned(x, 4) || !aligned(e, 4)) return FXP_ERR_ALIGN;
    return FXP_OK;
}

}  // namespace fxp

extern "C" int fxp_map(const float* x, int64_t rows, int64_t cols, const int32_t* e_max, int8_t* q, int8_t* qT,
                       uint64_t seed, uint64_t stream_id, int rounding, int bits, void* stream) {
    int rc = fxp::check_map_args(x, rows, cols, e_max, q, qT, rounding, bits);
    if (rc) return rc;
    if (rows * cols == 0) return FXP_OK;
    fxp::MapTensor t{x, rows, cols, e_max, nullptr, 0, nullptr, q, qT, stream_id};
    return fxp::map_launch(t, seed, rounding, bits, static_cast<hipStream_t>(stream));
}

extern "C" int fxp_map_absmax(const float* x, int64_t rows, int64_t cols, const uint32_t* absmax, int32_t* e_max, int8_t* q,
                              int8_t* qT, uint64_t seed, uint64_t stream_id, int rounding, int bits, void* stream) {
    int rc = fxp::check_map_args(x, rows, cols, e_max, q, qT, rounding, bits);
    if (rc) return rc;
    if (!absmax) return FXP_ERR_NULL;
    if (!fxp::aligned(absmax, 4)) return FXP_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (rows * cols == 0) return fxp::scale_finish(absmax, FXP_ABSMAX_WORDS, e_max, s);     // only the scale
    // the words are a list of block maxima: the map kernel turns them into the scale and publishes it
    const fxp::MapTensor t{x, rows, cols, nullptr, absmax, FXP_ABSMAX_WORDS, e_max, q, qT, stream_id};
    return fxp::map_launch(t, seed, rounding, bits, s);
}

extern "C" int fxp_scale_map(const float* x, int64_t rows, int64_t cols, int32_t* e_max, int8_t* q, int8_t* qT,
                             uint64_t seed, uint64_t stream_id, int rounding, int bits, void* ws, size_t ws_bytes,
                             void* stream) {
    int rc = fxp::check_map_args(x, rows, cols, e_max, q, qT, rounding, bits);
    if (rc) return rc;
    if (!ws || ws_bytes < fxp::kScaleWsBytes) return FXP_ERR_WORKSPACE;
    if (!fxp::aligned(ws, 4)) return FXP_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t* partials = static_cast<uint32_t*>(ws);
    int np = 0;
    rc = fxp::scale_partials(x, static_cast<size_t>(rows * cols), partials, &np, s);
    if (rc) return rc;
    if (rows * cols == 0) return fxp::scale_finish(partials, np, e_max, s);
    fxp::MapTensor t{x, rows, cols, nullptr, partials, np, e_max, q, qT, stream_id};
    return fxp::map_launch(t, seed, rounding, bits, s);
}

static int check_desc(const fxp_map_desc* d, int rounding, int bits) {
    if (!d) return FXP_ERR_NULL;
    return fxp::check_map_args(d->x, d->rows, d->cols, d->e_max, d->q, d->qT, rounding, bits);
}

extern "C" int fxp_map2(const fxp_map_desc* a, const fxp_map_desc* b, uint64_t seed, int rounding, int bits, void* stream) {
    int rc = check_desc(a, rounding, bits);
    if (!rc) rc = check_desc(b, rounding, bits);
    if (rc) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const fxp::MapTensor ta{a->x, a->rows, a->cols, a->e_max, nullptr, 0, nullptr, a->q, a->qT, a->stream_id};
    const fxp::MapTensor tb{b->x, b->rows, b->cols, b->e_max, nullptr, 0, nullptr, b->q, b->qT, b->stream_id};
    if (a->rows * a->cols == 0 || b->rows * b->cols == 0) {     // an empty tensor has nothing to launch
        if (a->rows * a->cols && (rc = fxp::map_launch(ta, seed, rounding, bits, s))) return rc;
        if (b->rows * b->cols && (rc = fxp::map_launch(tb, seed, rounding, bits, s))) return rc;
        return FXP_OK;
    }
    return fxp::map_launch2(ta, tb, seed, rounding, bits, s);
}

extern "C" int fxp_scale_map2(const fxp_map_desc* a, const fxp_map_desc* b, uint64_t seed, int rounding, int bits, void* ws,
                              size_t ws_bytes, void* stream) {
    int rc = check_desc(a, rounding, bits);
    if (!rc) rc = check_desc(b, rounding, bits);
    if (rc) return rc;
    if (!ws || ws_bytes < 2 * fxp::kScaleWsBytes) return FXP_ERR_WORKSPACE;
    if (!fxp::aligned(ws, 4)) return FXP_ERR_ALIGN;
    uint32_t* pa = static_cast<uint32_t*>(ws);
    uint32_t* pb = pa + fxp::kMaxPartials;
    if (a->rows * a->cols == 0 || b->rows * b->cols == 0) {     // an empty tensor: the single-tensor path, twice
        rc = fxp_scale_map(a->x, a->rows, a->cols, a->e_max, a->q, a->qT, seed, a->stream_id, rounding, bits, pa,
                           fxp::kScaleWsBytes, stream);
        return rc ? rc
                  : fxp_scale_map(b->x, b->rows, b->cols, b->e_max, b->q, b->qT, seed, b->stream_id, rounding, bits, pb,
                                  fxp::kScaleWsBytes, stream);
    }
    const fxp::MapTensor ta{a->x, a->rows, a->cols, nullptr, pa, 0, a->e_max, a->q, a->qT, a->stream_id};
    const fxp::MapTensor tb{b->x, b->rows, b->cols, nullptr, pb, 0, b->e_max, b->q, b->qT, b->stream_id};
    return fxp::scale_and_map2(ta, tb, seed, rounding, bits, static_cast<hipStream_t>(stream));
}
