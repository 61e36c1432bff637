// One integer linear layer, forward and backward (paper App. A.2, Fig. 2), composed
// from the kernels of this library on one stream with no host synchronisation:
//   forward : scale+map X, scale+map W (each tensor in both orientations), then
//             Y = unmap(Xq * Wq) through the fused GEMM epilogue;
//   backward: scale+map dY once, dX = unmap(dYq * Wq^T), dW = unmap(Xq^T * dYq).
// Every GEMM takes the native operand form because the mapping wrote both copies:
//   Y  = Xq  [M,K] x WqT [N,K]^T      dX = dYq [M,N] x Wq [K,N]^T
//   dW = XqT [K,M] x dYqT[N,M]^T
#include <algorithm>
#include <atomic>
#include <mutex>
#include <vector>

#include "fxp_internal.h"

namespace fxp {

// Measurement helper (fxp_timeline_begin / _end): HIP events recorded on the caller's stream at the entry of a
// linear-layer call and after each of its launches, so that a benchmark reads the duration every kernel has
// INSIDE a step (behind the kernel that really precedes it, with what that kernel left in the caches) instead of
// timing it in a loop of its own.  Off unless a timeline has been begun; one timeline per process.
struct Timeline {
    std::vector<hipEvent_t> events;
    std::vector<int> tags;
    size_t used = 0;
    std::atomic<bool> on{false};
};
static Timeline g_timeline;
static std::mutex g_timeline_lock;

static void timeline_mark(hipStream_t s, int tag) {
    if (!g_timeline.on.load(std::memory_order_acquire)) return;     // off: no lock taken on the layer calls' path
    std::lock_guard<std::mutex> hold(g_timeline_lock);
    if (g_timeline.used >= g_timeline.events.size()) return;
    if (hipEventRecord(g_timeline.events[g_timeline.used], s) != hipSuccess) { (void)hipGetLastError(); return; }
    g_timeline.tags[g_timeline.used++] = tag;
}

// scale + map of the two operands of a forward pass: with guesses where that path applies (both in one pair of
// launches, or each tensor by itself when their tile widths differ), else two launches for both
static int scale_map_operands(const MapTensor& a, const MapTensor& b, uint32_t* area_a, uint32_t* area_b, uint64_t seed,
                              int rounding, int bits, hipStream_t s, bool guess) {
    int rc = guess ? scale_map_guess_launch(a, &b, area_a, area_b, seed, rounding, bits, s) : kNoGuessPath;
    if (rc == kNoGuessPath) return scale_and_map2(a, b, seed, rounding, bits, s);
    if (rc != kGuessOneByOne) return rc;
    const MapTensor* ts[2] = {&a, &b};
    uint32_t* areas[2] = {area_a, area_b};
    for (int j = 0; j < 2; ++j) {
        const MapTensor& t = *ts[j];
        rc = scale_map_guess_launch(t, nullptr, areas[j], nullptr, seed, rounding, bits, s);
        if (rc == kNoGuessPath)
            rc = scale_and_map(t.x, t.rows, t.cols, t.e_out, t.q, t.qT, seed, t.stream_id, rounding, bits, areas[j], s);
        if (rc) return rc;
    }
    return FXP_OK;
}

static int check_layer(int64_t M, int64_t K, int64_t N, int rounding, int bits, const void* ws, size_t ws_bytes,
                       size_t need) {
    if (M <= 0 || K <= 0 || N <= 0) return FXP_ERR_DIMS;
    if (M >= (int64_t{1} << 31) || N >= (int64_t{1} << 31) || K >= (int64_t{1} << 31)) return FXP_ERR_DIMS;
    if (rounding != FXP_ROUND_STOCHASTIC && rounding != FXP_ROUND_NEAREST) return FXP_ERR_ROUNDING;
    if (bits < 2 || bits > 8) return FXP_ERR_BITS;
    if (!ws || ws_bytes < need) return FXP_ERR_WORKSPACE;
    if (!aligned(ws, 256)) return FXP_ERR_ALIGN;
    return FXP_OK;
}

}  // namespace fxp

extern "C" const char* fxp_strerror(int status) {
    switch (status) {
        case FXP_OK: return "ok";
        case FXP_ERR_NULL: return "a required pointer is NULL";
        case FXP_ERR_DIMS: return "bad size or leading dimension";
        case FXP_ERR_ALIGN: return "pointer alignment";
        case FXP_ERR_WORKSPACE: return "workspace missing or too small";
        case FXP_ERR_ROUNDING: return "unknown rounding mode";
        case FXP_ERR_BITS: return "bits outside [2, 8]";
        case FXP_ERR_LAUNCH: return "kernel launch failed";
        case FXP_ERR_OVERFLOW: return "contraction too long for int32 accumulation";
        default: return "unknown status";
    }
}

extern "C" int fxp_version(void) { return 111; }

extern "C" size_t fxp_workspace_bytes(int op, int64_t M, int64_t N, int64_t K) {
    if (M < 0 || N < 0 || K < 0) return 0;
    switch (op) {
        case FXP_OP_SCALE: return fxp::kScaleWsBytes;
        case FXP_OP_GEMM: return fxp::gemm_ws_worst(M, N, K) + 256;
        case FXP_OP_LINEAR_FWD:
            return 2 * fxp::round_up(fxp::kScaleWsBytes, 256) + fxp::gemm_split_ws_bytes(M, N, K);
        case FXP_OP_LINEAR_BWD:   // the two gradient GEMMs run one after the other and share the slice area
            return fxp::round_up(fxp::kScaleWsBytes, 256) +
                   std::max(fxp::gemm_split_ws_bytes(M, K, N), fxp::gemm_split_ws_bytes(K, N, M));
        case FXP_OP_BMM_FWD: return 2 * fxp::round_up(fxp::kScaleWsBytes, 256);
        case FXP_OP_BMM_BWD: return fxp::round_up(fxp::kScaleWsBytes, 256);
        default: return 0;
    }
}

namespace fxp {

// argument checks of the forward call that need no workspace
static int check_linear_fwd(const float* X, const float* W, int64_t M, int64_t K, int64_t N, const float* Y,
                            const fxp_saved* saved, int rounding, int bits) {
    if (M <= 0 || K <= 0 || N <= 0) return FXP_ERR_DIMS;
    if (M >= (int64_t{1} << 31) || N >= (int64_t{1} << 31) || K >= (int64_t{1} << 31)) return FXP_ERR_DIMS;
    if (rounding != FXP_ROUND_STOCHASTIC && rounding != FXP_ROUND_NEAREST) return FXP_ERR_ROUNDING;
    if (bits < 2 || bits > 8) return FXP_ERR_BITS;
    if (!X || !W || !Y || !saved || !saved->Xq || !saved->XqT || !saved->Wq || !saved->WqT || !saved->eX || !saved->eW)
        return FXP_ERR_NULL;
    if (!aligned(X, 4) || !aligned(W, 4) || !aligned(Y, 4) || !aligned(saved->eX, 4) || !aligned(saved->eW, 4))
        return FXP_ERR_ALIGN;
    return FXP_OK;
}

// the forward pass itself: arguments validated, ws of fxp_workspace_bytes(FXP_OP_LINEAR_FWD) bytes or more
static int linear_fwd_run(const float* X, const float* W, int64_t M, int64_t K, int64_t N, float* Y, const fxp_saved* saved,
                          uint64_t seed, uint64_t step, int rounding, int bits, void* ws, size_t ws_bytes, hipStream_t s,
                          bool guess = false) {
    uint32_t* pX = static_cast<uint32_t*>(ws);
    uint32_t* pW = pX + round_up(kScaleWsBytes, 256) / sizeof(uint32_t);
    MapTensor tX{X, M, K, nullptr, pX, 0, saved->eX, saved->Xq, saved->XqT, (step << 8) | FXP_TAG_X};
    MapTensor tW{W, K, N, nullptr, pW, 0, saved->eW, saved->Wq, saved->WqT, (step << 8) | FXP_TAG_W};
    timeline_mark(s, FXP_TL_ENTRY);
    // with the scales of the last step as guesses: one pass that maps and finds the maxima, one launch that verifies
    int rc = guess ? scale_map_guess_launch(tX, &tW, pX, pW, seed, rounding, bits, s) : kNoGuessPath;
    if (rc == kGuessOneByOne) rc = scale_map_operands(tX, tW, pX, pW, seed, rounding, bits, s, true);
    if (rc == kNoGuessPath) {
        // scale + map of both operands in two launches: one reduction launch and one map launch cover both tensors
        rc = scale_partials2(X, static_cast<size_t>(M * K), pX, &tX.n_partials, W, static_cast<size_t>(K * N), pW, &tW.n_partials, s);
        if (rc) return rc;
        timeline_mark(s, FXP_TL_SCALE);
        rc = map_launch2(tX, tW, seed, rounding, bits, s);
    }
    if (rc) return rc;
    timeline_mark(s, FXP_TL_MAP);
    uint8_t* rest = static_cast<uint8_t*>(ws) + 2 * round_up(kScaleWsBytes, 256);
    rc = gemm_nt_launch(M, N, K, saved->Xq, K, saved->WqT, K, Y, N, true, saved->eX, bits, saved->eW, bits, rest,
                        ws_bytes - 2 * round_up(kScaleWsBytes, 256), s);
    timeline_mark(s, FXP_TL_GEMM_FWD);
    return rc;
}

}  // namespace fxp

extern "C" int fxp_linear_fwd(const float* X, const float* W, int64_t M, int64_t K, int64_t N, float* Y,
                              const fxp_saved* saved, uint64_t seed, uint64_t step, int rounding, int bits, void* ws,
                              size_t ws_bytes, void* stream) {
    using namespace fxp;
    int rc = check_layer(M, K, N, rounding, bits, ws, ws_bytes, fxp_workspace_bytes(FXP_OP_LINEAR_FWD, M, N, K));
    if (rc) return rc;
    if ((rc = check_linear_fwd(X, W, M, K, N, Y, saved, rounding, bits))) return rc;
    return linear_fwd_run(X, W, M, K, N, Y, saved, seed, step, rounding, bits, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

// ---- the forward pass for callers that cannot allocate -------------------------------------------------------
// The scratch of fxp_linear_fwd (two areas of block maxima, and the int32 slices of a product that is split along
// its contraction) lives in this device array instead of a caller's workspace.  Every GPU the library runs on
// holds its own copy of the array at its own address until the process ends; the array's name is only a
// host-side handle, so its device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[FXP_STATIC_SCRATCH_BYTES];

namespace fxp {

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];     // device address of `scratch` on each device, null until looked up
static std::mutex g_scratch_lock;

// the current device's copy of the array (looked up on the first call on that device), or null on failure
static void* static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

}  // namespace fxp

extern "C" size_t fxp_static_scratch_bytes(void) { return FXP_STATIC_SCRATCH_BYTES; }

extern "C" int fxp_linear_fwd_static(const float* X, const float* W, int64_t M, int64_t K, int64_t N, float* Y,
                                     const fxp_saved* saved, uint64_t seed, uint64_t step, int rounding, int bits,
                                     void* stream) {
    using namespace fxp;
    int rc = check_linear_fwd(X, W, M, K, N, Y, saved, rounding, bits);
    if (rc) return rc;
    // a layer whose scratch does not fit the array is refused before anything touches the device
    if (fxp_workspace_bytes(FXP_OP_LINEAR_FWD, M, N, K) > FXP_STATIC_SCRATCH_BYTES) return FXP_ERR_WORKSPACE;
    void* ws = static_scratch();
    if (ws == nullptr) return FXP_ERR_LAUNCH;
    // nothing in the array has to start at zero: the reduction writes every block maximum the map kernel reads,
    // and every slice element is stored by the product before the sum of the slices reads it
    return linear_fwd_run(X, W, M, K, N, Y, saved, seed, step, rounding, bits, ws, FXP_STATIC_SCRATCH_BYTES,
                          static_cast<hipStream_t>(stream));
}

namespace fxp {
static int linear_bwd_impl(const float* dY, const fxp_saved* saved, int64_t M, int64_t K, int64_t N, float* dX,
                           float* dW, int8_t* dYq, int8_t* dYqT, int32_t* e_dY, uint64_t seed, uint64_t step,
                           int rounding, int bits, void* ws, size_t ws_bytes, void* stream, bool guess) {
    int rc = check_layer(M, K, N, rounding, bits, ws, ws_bytes, fxp_workspace_bytes(FXP_OP_LINEAR_BWD, M, N, K));
    if (rc) return rc;
    if (!dY || !saved || !saved->XqT || !saved->Wq || !saved->eX || !saved->eW || !dYq || !dYqT || !e_dY)
        return FXP_ERR_NULL;
    if (!aligned(dY, 4) || !aligned(dX, 4) || !aligned(dW, 4) || !aligned(e_dY, 4)) return FXP_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    timeline_mark(s, FXP_TL_ENTRY);
    {
        MapTensor t{dY, M, N, nullptr, static_cast<uint32_t*>(ws), 0, e_dY, dYq, dYqT, (step << 8) | FXP_TAG_DY};
        rc = guess ? scale_map_guess_launch(t, nullptr, static_cast<uint32_t*>(ws), nullptr, seed, rounding, bits, s) : kNoGuessPath;
        if (rc == kNoGuessPath) {
            if ((rc = scale_partials(dY, static_cast<size_t>(M * N), static_cast<uint32_t*>(ws), &t.n_partials, s))) return rc;
            timeline_mark(s, FXP_TL_SCALE);
            rc = map_launch(t, seed, rounding, bits, s);
        }
        if (rc) return rc;
        timeline_mark(s, FXP_TL_MAP);
    }
    uint8_t* rest = static_cast<uint8_t*>(ws) + round_up(kScaleWsBytes, 256);
    const size_t rest_bytes = ws_bytes - round_up(kScaleWsBytes, 256);
    // The weight gradient first: when it is split along K, the sum of its slices does not get a launch of its own
    // but rides in the launch of the input-gradient product (whose last workgroups do it) - unless that product
    // is split too and needs the slice area for itself.
    ReduceRider pending;
    const bool rides = dX != nullptr && gemm_split_ws_bytes(M, K, N) == 0;
    if (dW && (rc = gemm_nt_launch(K, N, M, saved->XqT, M, dYqT, M, dW, N, true, saved->eX, bits, e_dY, bits, rest,
                                   rest_bytes, s, nullptr, nullptr, rides ? &pending : nullptr)))
        return rc;
    if (dW) timeline_mark(s, FXP_TL_GEMM_DW);
    if (dX && (rc = gemm_nt_launch(M, K, N, dYq, N, saved->Wq, N, dX, K, true, e_dY, bits, saved->eW, bits, rest,
                                   rest_bytes, s, nullptr, &pending, nullptr)))
        return rc;
    if (dX) timeline_mark(s, FXP_TL_GEMM_DX);
    if (pending.blocks != 0) {                                             // nobody took it along
        rc = splitk_reduce_launch(pending, s);
        timeline_mark(s, FXP_TL_REDUCE);
        return rc;
    }
    return FXP_OK;
}
}  // namespace fxp

extern "C" int fxp_linear_bwd(const float* dY, const fxp_saved* saved, int64_t M, int64_t K, int64_t N, float* dX,
                              float* dW, int8_t* dYq, int8_t* dYqT, int32_t* e_dY, uint64_t seed, uint64_t step,
                              int rounding, int bits, void* ws, size_t ws_bytes, void* stream) {
    return fxp::linear_bwd_impl(dY, saved, M, K, N, dX, dW, dYq, dYqT, e_dY, seed, step, rounding, bits, ws, ws_bytes, stream, false);
}

extern "C" int fxp_linear_fwd_guess(const float* X, const float* W, int64_t M, int64_t K, int64_t N, float* Y,
                                    const fxp_saved* saved, uint64_t seed, uint64_t step, int rounding, int bits, void* ws,
                                    size_t ws_bytes, void* stream) {
    using namespace fxp;
    int rc = check_layer(M, K, N, rounding, bits, ws, ws_bytes, fxp_workspace_bytes(FXP_OP_LINEAR_FWD, M, N, K));
    if (rc) return rc;
    if ((rc = check_linear_fwd(X, W, M, K, N, Y, saved, rounding, bits))) return rc;
    return linear_fwd_run(X, W, M, K, N, Y, saved, seed, step, rounding, bits, ws, ws_bytes, static_cast<hipStream_t>(stream), true);
}

extern "C" int fxp_linear_bwd_guess(const float* dY, const fxp_saved* saved, int64_t M, int64_t K, int64_t N, float* dX,
                                    float* dW, int8_t* dYq, int8_t* dYqT, int32_t* e_dY, uint64_t seed, uint64_t step,
                                    int rounding, int bits, void* ws, size_t ws_bytes, void* stream) {
    return fxp::linear_bwd_impl(dY, saved, M, K, N, dX, dW, dYq, dYqT, e_dY, seed, step, rounding, bits, ws, ws_bytes, stream, true);
}

extern "C" int fxp_timeline_begin(int capacity) {
    using namespace fxp;
    if (capacity <= 0 || capacity > (1 << 20)) return FXP_ERR_DIMS;
    std::lock_guard<std::mutex> hold(g_timeline_lock);
    if (g_timeline.on) return FXP_ERR_DIMS;                       // one timeline at a time
    g_timeline.events.assign(static_cast<size_t>(capacity), nullptr);
    g_timeline.tags.assign(static_cast<size_t>(capacity), 0);
    g_timeline.used = 0;
    for (auto& e : g_timeline.events)
        if (hipEventCreate(&e) != hipSuccess) {
            (void)hipGetLastError();
            for (auto& d : g_timeline.events)
                if (d) (void)hipEventDestroy(d);
            g_timeline.events.clear();
            return FXP_ERR_LAUNCH;
        }
    g_timeline.on = true;
    return FXP_OK;
}

extern "C" int fxp_timeline_end(float* microseconds, int* tags, int capacity, int* count) {
    using namespace fxp;
    std::lock_guard<std::mutex> hold(g_timeline_lock);
    if (!g_timeline.on) return FXP_ERR_DIMS;
    g_timeline.on = false;
    int rc = FXP_OK, n = 0;
    if (g_timeline.used > 0 && hipEventSynchronize(g_timeline.events[g_timeline.used - 1]) != hipSuccess) rc = FXP_ERR_LAUNCH;
    for (size_t i = 1; rc == FXP_OK && i < g_timeline.used && n < capacity; ++i) {
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, g_timeline.events[i - 1], g_timeline.events[i]) != hipSuccess) { rc = FXP_ERR_LAUNCH; break; }
        if (microseconds) microseconds[n] = ms * 1000.0f;
        if (tags) tags[n] = g_timeline.tags[i];
        ++n;
    }
    if (rc != FXP_OK) (void)hipGetLastError();
    if (count) *count = n;
    for (auto& e : g_timeline.events) (void)hipEventDestroy(e);
    g_timeline.events.clear();
    g_timeline.tags.clear();
    g_timeline.used = 0;
    return rc;
}


// Batched product layer (attention matmuls).  Every tensor is mapped once as a (batch * rows) x cols matrix in
// both orientations; matrix b of a transposed copy is a column block of it, reached by a batch stride of
// `rows` and a leading dimension of batch * rows (a per-matrix transposed layout was tried: its GEMMs read
// faster but the mapping kernel's transposed stores lose their full 128-byte lines, a net loss):
//   Y_b   = Aq_b [M,K]            x (Bq_b [N,K] | BqT cols b*K.. [N,K])^T
//   dA_b  = Gq_b [M,N]            x (BqT cols b*N.. [K,N] | Bq_b [K,N])^T          (transB | not)
//   dBm_b = AqT cols b*M.. [K,M]  x GqT cols b*M.. [N,M]^T   -> [K,N]              (operands swapped for transB)
namespace fxp {
static int check_bmm(int64_t batch, int64_t M, int64_t K, int64_t N, int rounding, int bits, const void* ws,
                     size_t ws_bytes, size_t need) {
    int rc = check_layer(M, K, N, rounding, bits, ws, ws_bytes, need);
    if (rc) return rc;
    if (batch <= 0 || batch > 65535) return FXP_ERR_DIMS;
    const int64_t lim = int64_t{1} << 31;
    if (batch * M >= lim || batch * K >= lim || batch * N >= lim) return FXP_ERR_DIMS;
    return FXP_OK;
}
}  // namespace fxp

namespace fxp {
static int bmm_fwd_impl(const float* A, const float* Bm, int64_t batch, int64_t M, int64_t K, int64_t N, int transB,
                        float* Y, const fxp_bmm_saved* saved, uint64_t seed, uint64_t step, int rounding, int bits,
                        void* ws, size_t ws_bytes, void* stream, bool guess) {
    int rc = check_bmm(batch, M, K, N, rounding, bits, ws, ws_bytes, fxp_workspace_bytes(FXP_OP_BMM_FWD, M, N, K));
    if (rc) return rc;
    if (K > kMaxContraction) return FXP_ERR_OVERFLOW;
    if (!A || !Bm || !Y || !saved || !saved->Aq || !saved->AqT || !saved->Bq || !saved->BqT || !saved->eA || !saved->eB)
        return FXP_ERR_NULL;
    if (!aligned(A, 4) || !aligned(Bm, 4) || !aligned(Y, 4) || !aligned(saved->eA, 4) || !aligned(saved->eB, 4))
        return FXP_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t* pA = static_cast<uint32_t*>(ws);
    uint32_t* pB = pA + round_up(kScaleWsBytes, 256) / sizeof(uint32_t);
    const int64_t b_rows = transB ? N : K, b_cols = transB ? K : N;
    const MapTensor tA{A, batch * M, K, nullptr, pA, 0, saved->eA, saved->Aq, saved->AqT, (step << 8) | FXP_TAG_X};
    const MapTensor tB{Bm, batch * b_rows, b_cols, nullptr, pB, 0, saved->eB, saved->Bq, saved->BqT, (step << 8) | FXP_TAG_W};
    if ((rc = scale_map_operands(tA, tB, pA, pB, seed, rounding, bits, s, guess))) return rc;
    const int8_t* Bop = transB ? saved->Bq : saved->BqT;
    const int64_t ldb = transB ? K : batch * K, strideB = transB ? N * K : K;
    return gemm_nt_batched_launch(M, N, K, saved->Aq, K, M * K, Bop, ldb, strideB, Y, N, M * N, batch, true, saved->eA, bits,
                                  saved->eB, bits, s);
}
}  // namespace fxp

extern "C" int fxp_bmm_fwd(const float* A, const float* Bm, int64_t batch, int64_t M, int64_t K, int64_t N, int transB,
                           float* Y, const fxp_bmm_saved* saved, uint64_t seed, uint64_t step, int rounding, int bits,
                           void* ws, size_t ws_bytes, void* stream) {
    return fxp::bmm_fwd_impl(A, Bm, batch, M, K, N, transB, Y, saved, seed, step, rounding, bits, ws, ws_bytes, stream, false);
}

extern "C" int fxp_bmm_fwd_guess(const float* A, const float* Bm, int64_t batch, int64_t M, int64_t K, int64_t N, int transB,
                                 float* Y, const fxp_bmm_saved* saved, uint64_t seed, uint64_t step, int rounding, int bits,
                                 void* ws, size_t ws_bytes, void* stream) {
    return fxp::bmm_fwd_impl(A, Bm, batch, M, K, N, transB, Y, saved, seed, step, rounding, bits, ws, ws_bytes, stream, true);
}

namespace fxp {
static int bmm_bwd_impl(const float* dY, const fxp_bmm_saved* saved, int64_t batch, int64_t M, int64_t K, int64_t N,
                        int transB, float* dA, float* dBm, int8_t* dYq, int8_t* dYqT, int32_t* e_dY, uint64_t seed,
                        uint64_t step, int rounding, int bits, void* ws, size_t ws_bytes, void* stream, bool guess) {
    int rc = check_bmm(batch, M, K, N, rounding, bits, ws, ws_bytes, fxp_workspace_bytes(FXP_OP_BMM_BWD, M, N, K));
    if (rc) return rc;
    if (N > kMaxContraction || M > kMaxContraction) return FXP_ERR_OVERFLOW;
    if (!dY || !saved || !saved->AqT || !saved->Bq || !saved->BqT || !saved->eA || !saved->eB || !dYq || !dYqT || !e_dY)
        return FXP_ERR_NULL;
    if (!aligned(dY, 4) || !aligned(dA, 4) || !aligned(dBm, 4) || !aligned(e_dY, 4)) return FXP_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    {
        const MapTensor t{dY, batch * M, N, nullptr, static_cast<uint32_t*>(ws), 0, e_dY, dYq, dYqT, (step << 8) | FXP_TAG_DY};
        rc = guess ? scale_map_guess_launch(t, nullptr, static_cast<uint32_t*>(ws), nullptr, seed, rounding, bits, s) : kNoGuessPath;
        if (rc == kNoGuessPath)
            rc = scale_and_map(dY, batch * M, N, e_dY, dYq, dYqT, seed, (step << 8) | FXP_TAG_DY, rounding, bits,
                               static_cast<uint32_t*>(ws), s);
        if (rc) return rc;
    }
    if (dA) {
        const int8_t* Bop = transB ? saved->BqT : saved->Bq;      // [K,N] per matrix, N contiguous
        const int64_t ldb = transB ? batch * N : N, strideB = transB ? N : K * N;
        if ((rc = gemm_nt_batched_launch(M, K, N, dYq, N, M * N, Bop, ldb, strideB, dA, K, M * K, batch, true, e_dY, bits,
                                         saved->eB, bits, s)))
            return rc;
    }
    if (dBm) {
        const int64_t ld = batch * M;                              // both operands are column blocks of a transposed copy
        if (transB)
            rc = gemm_nt_batched_launch(N, K, M, dYqT, ld, M, saved->AqT, ld, M, dBm, K, N * K, batch, true, e_dY, bits,
                                        saved->eA, bits, s);
        else
            rc = gemm_nt_batched_launch(K, N, M, saved->AqT, ld, M, dYqT, ld, M, dBm, N, K * N, batch, true, saved->eA, bits,
                                        e_dY, bits, s);
        if (rc) return rc;
    }
    return FXP_OK;
}
}  // namespace fxp

extern "C" int fxp_bmm_bwd(const float* dY, const fxp_bmm_saved* saved, int64_t batch, int64_t M, int64_t K, int64_t N,
                           int transB, float* dA, float* dBm, int8_t* dYq, int8_t* dYqT, int32_t* e_dY, uint64_t seed,
                           uint64_t step, int rounding, int bits, void* ws, size_t ws_bytes, void* stream) {
    return fxp::bmm_bwd_impl(dY, saved, batch, M, K, N, transB, dA, dBm, dYq, dYqT, e_dY, seed, step, rounding, bits, ws, ws_bytes,
                             stream, false);
}

extern "C" int fxp_bmm_bwd_guess(const float* dY, const fxp_bmm_saved* saved, int64_t batch, int64_t M, int64_t K, int64_t N,
                                 int transB, float* dA, float* dBm, int8_t* dYq, int8_t* dYqT, int32_t* e_dY, uint64_t seed,
                                 uint64_t step, int rounding, int bits, void* ws, size_t ws_bytes, void* stream) {
    return fxp::bmm_bwd_impl(dY, saved, batch, M, K, N, transB, dA, dBm, dYq, dYqT, e_dY, seed, step, rounding, bits, ws, ws_bytes,
                             stream, true);
}
