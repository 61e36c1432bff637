// One integer linear layer, forward and backward (paper App. A.2, Fig. 2), composed
// from the kernels of this library on one stream with no host synchronisation:
//   forward : scale+map X, scale+map W (each tensor in both orientations), then
//             Y = unmap(Xq * Wq) through the fused GEMM epilogue;
//   backward: scale+map dY once, dX = unmap(dYq * Wq^T), dW = unmap(Xq^T * dYq).
// Every GEMM takes the native operand form because the mapping wrote both copies:
//   Y  = Xq  [M,K] x WqT [N,K]^T      dX = dYq [M,N] x Wq [K,N]^T
//   dW = XqT [K,M] x dYqT[N,M]^T
#include <algorithm>

#include "fxp_internal.h"

namespace fxp {

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

extern "C" int fxp_version(void) { return 100; }

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
        default: return 0;
    }
}

extern "C" int fxp_linear_fwd(const float* X, const float* W, int64_t M, int64_t K, int64_t N, float* Y,
                              const fxp_saved* saved, uint64_t seed, uint64_t step, int rounding, int bits, void* ws,
                              size_t ws_bytes, void* stream) {
    using namespace fxp;
    int rc = check_layer(M, K, N, rounding, bits, ws, ws_bytes, fxp_workspace_bytes(FXP_OP_LINEAR_FWD, M, N, K));
    if (rc) return rc;
    if (K > kMaxContraction) return FXP_ERR_OVERFLOW;
    if (!X || !W || !Y || !saved || !saved->Xq || !saved->XqT || !saved->Wq || !saved->WqT || !saved->eX || !saved->eW)
        return FXP_ERR_NULL;
    if (!aligned(X, 4) || !aligned(W, 4) || !aligned(Y, 4) || !aligned(saved->eX, 4) || !aligned(saved->eW, 4))
        return FXP_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t* pX = static_cast<uint32_t*>(ws);
    uint32_t* pW = pX + round_up(kScaleWsBytes, 256) / sizeof(uint32_t);
    if ((rc = scale_and_map(X, M, K, saved->eX, saved->Xq, saved->XqT, seed, (step << 8) | FXP_TAG_X, rounding, bits, pX, s)))
        return rc;
    if ((rc = scale_and_map(W, K, N, saved->eW, saved->Wq, saved->WqT, seed, (step << 8) | FXP_TAG_W, rounding, bits, pW, s)))
        return rc;
    uint8_t* rest = static_cast<uint8_t*>(ws) + 2 * round_up(kScaleWsBytes, 256);
    return gemm_nt_launch(M, N, K, saved->Xq, K, saved->WqT, K, Y, N, true, saved->eX, bits, saved->eW, bits, rest,
                          ws_bytes - 2 * round_up(kScaleWsBytes, 256), s);
}

extern "C" int fxp_linear_bwd(const float* dY, const fxp_saved* saved, int64_t M, int64_t K, int64_t N, float* dX,
                              float* dW, int8_t* dYq, int8_t* dYqT, int32_t* e_dY, uint64_t seed, uint64_t step,
                              int rounding, int bits, void* ws, size_t ws_bytes, void* stream) {
    using namespace fxp;
    int rc = check_layer(M, K, N, rounding, bits, ws, ws_bytes, fxp_workspace_bytes(FXP_OP_LINEAR_BWD, M, N, K));
    if (rc) return rc;
    if (N > kMaxContraction || M > kMaxContraction) return FXP_ERR_OVERFLOW;
    if (!dY || !saved || !saved->XqT || !saved->Wq || !saved->eX || !saved->eW || !dYq || !dYqT || !e_dY)
        return FXP_ERR_NULL;
    if (!aligned(dY, 4) || !aligned(dX, 4) || !aligned(dW, 4) || !aligned(e_dY, 4)) return FXP_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if ((rc = scale_and_map(dY, M, N, e_dY, dYq, dYqT, seed, (step << 8) | FXP_TAG_DY, rounding, bits,
                            static_cast<uint32_t*>(ws), s)))
        return rc;
    uint8_t* rest = static_cast<uint8_t*>(ws) + round_up(kScaleWsBytes, 256);
    const size_t rest_bytes = ws_bytes - round_up(kScaleWsBytes, 256);
    if (dX && (rc = gemm_nt_launch(M, K, N, dYq, N, saved->Wq, N, dX, K, true, e_dY, bits, saved->eW, bits, rest,
                                   rest_bytes, s)))
        return rc;
    if (dW && (rc = gemm_nt_launch(K, N, M, saved->XqT, M, dYqT, M, dW, N, true, saved->eX, bits, e_dY, bits, rest,
                                   rest_bytes, s)))
        return rc;
    return FXP_OK;
}
