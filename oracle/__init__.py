"""numpy front end of the CPU oracle (oracle/fxp_ref.cpp).

TEST INFRASTRUCTURE: imported by tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py only.  It never imports the GPU package.
All arrays are host numpy arrays; every function returns new arrays.
"""
import ctypes
import os

import numpy as np

from . import build as _build

STOCHASTIC = 0
NEAREST = 1
TAG_X, TAG_W, TAG_DY = 0, 1, 2

_lib = None


def lib():
    global _lib
    if _lib is None:
        if os.environ.get("FXP_REF_SANITIZE") == "1":      # the AddressSanitizer + UBSan build (tests only)
            path = _build.build(force=False, sanitize=True)
        else:
            path = _build.LIB if os.path.exists(_build.LIB) else _build.build()
        L = ctypes.CDLL(path)
        c = ctypes
        vp, i32, i64, u64, u32 = c.c_void_p, c.c_int32, c.c_int64, c.c_uint64, c.c_uint32
        L.fxp_ref_num_threads.restype = c.c_int
        L.fxp_ref_philox4x32_10.argtypes = [vp, vp, vp]
        L.fxp_ref_philox4x32_10.restype = None
        L.fxp_ref_random_word.argtypes = [u64, u64, u64]
        L.fxp_ref_random_word.restype = u32
        L.fxp_ref_scale.argtypes = [vp, u64, vp]
        L.fxp_ref_map.argtypes = [vp, i64, i64, i32, vp, vp, u64, u64, c.c_int, c.c_int]
        L.fxp_ref_map_rows.argtypes = [vp, i64, i64, i64, i32, vp, u64, u64, c.c_int, c.c_int]
        L.fxp_ref_gemm.argtypes = [c.c_int, c.c_int, i64, i64, i64, vp, i64, vp, i64, vp, i64]
        L.fxp_ref_unmap.argtypes = [vp, u64, i32, c.c_int, i32, c.c_int, vp]
        L.fxp_ref_gemm64.argtypes = L.fxp_ref_gemm.argtypes
        L.fxp_ref_unmap64.argtypes = L.fxp_ref_unmap.argtypes
        L.fxp_ref_unmap_i8.argtypes = [vp, u64, i32, c.c_int, vp]
        L.fxp_ref_linear_fwd.argtypes = [vp, vp, i64, i64, i64, vp, vp, vp, vp, vp, u64, u64, c.c_int, c.c_int]
        L.fxp_ref_linear_bwd.argtypes = [vp, vp, vp, i32, i32, i64, i64, i64, vp, vp, vp, vp, u64, u64, c.c_int,
                                         c.c_int]
        cd = [i64] * 9       # N, H, W, C, Cout, KH, KW, stride, pad
        L.fxp_ref_gemm_batched.argtypes = [c.c_int, c.c_int, i64, i64, i64, vp, i64, i64, vp, i64, i64, vp, i64, i64, i64]
        L.fxp_ref_bmm_fwd.argtypes = [vp, vp, i64, i64, i64, i64, c.c_int, vp, vp, vp, vp, vp, u64, u64, c.c_int, c.c_int]
        L.fxp_ref_bmm_bwd.argtypes = [vp, vp, vp, i32, i32, i64, i64, i64, i64, c.c_int, vp, vp, vp, vp, u64, u64, c.c_int,
                                      c.c_int]
        L.fxp_ref_map16.argtypes = [vp, u64, i32, vp, u64, u64, c.c_int]
        L.fxp_ref_axpy16.argtypes = [vp, vp, c.c_float, u64, vp, vp, u64, u64, c.c_int]
        L.fxp_ref_sgd16_step.argtypes = [vp, vp, vp, u64, c.c_float, c.c_float, c.c_float, vp, u64, u64, c.c_int]
        L.fxp_ref_sgd16_step_multi.argtypes = [vp, vp, vp, vp, vp, u64, c.c_float, c.c_float, c.c_float, u64, u64, c.c_int]
        L.fxp_ref_conv2d_fwd_acc.argtypes = [vp, i64, i64, i64, i64, vp, i64, i64, i64, i64, i64, vp]
        L.fxp_ref_conv2d_bwd_input_acc.argtypes = [vp, vp] + cd + [vp]
        L.fxp_ref_conv2d_bwd_weight_acc.argtypes = [vp, vp] + cd + [vp]
        L.fxp_ref_conv2d_bwd_weight_acc64.argtypes = [vp, vp] + cd + [vp]
        L.fxp_ref_conv2d_fwd.argtypes = [vp, vp] + cd + [vp, vp, vp, vp, vp, u64, u64, c.c_int, c.c_int]
        L.fxp_ref_conv2d_bwd.argtypes = [vp, vp, vp, i32, i32] + cd + [vp, vp, vp, vp, u64, u64, c.c_int, c.c_int]
        _lib = L
    return _lib


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a):
    return a.ctypes.data if a is not None else None


def num_threads():
    return int(lib().fxp_ref_num_threads())


def philox4x32_10(ctr, key):
    ctr = np.ascontiguousarray(ctr, dtype=np.uint32)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    assert ctr.shape == (4,) and key.shape == (2,)
    out = np.empty(4, dtype=np.uint32)
    lib().fxp_ref_philox4x32_10(_ptr(ctr), _ptr(key), _ptr(out))
    return out


def random_word(seed, stream_id, i):
    return int(lib().fxp_ref_random_word(seed, stream_id, i))


def scale(x):
    x = _f32(x)
    e = np.zeros(1, dtype=np.int32)
    _check(lib().fxp_ref_scale(_ptr(x), x.size, _ptr(e)), "scale")
    return int(e[0])


def map(x, e_max, seed=0, stream_id=0, rounding=STOCHASTIC, bits=8, transposed=False):
    x = _f32(x)
    assert x.ndim == 2
    rows, cols = x.shape
    q = np.empty((rows, cols), dtype=np.int8)
    qT = np.empty((cols, rows), dtype=np.int8) if transposed else None
    _check(lib().fxp_ref_map(_ptr(x), rows, cols, int(e_max), _ptr(q), _ptr(qT), seed, stream_id, rounding, bits),
           "map")
    return (q, qT) if transposed else q


def map_rows(x_rows, row0, e_max, seed=0, stream_id=0, rounding=STOCHASTIC, bits=8):
    """q of rows row0 .. row0 + len(x_rows) - 1 of a larger tensor with the same number of columns."""
    x = _f32(x_rows)
    assert x.ndim == 2
    q = np.empty(x.shape, dtype=np.int8)
    _check(lib().fxp_ref_map_rows(_ptr(x), int(row0), x.shape[0], x.shape[1], int(e_max), _ptr(q), seed, stream_id,
                                  rounding, bits), "map_rows")
    return q


def gemm(A, B, transA=False, transB=False):
    A = np.ascontiguousarray(A, dtype=np.int8)
    B = np.ascontiguousarray(B, dtype=np.int8)
    M, K = (A.shape[1], A.shape[0]) if transA else A.shape
    Kb, N = (B.shape[1], B.shape[0]) if transB else B.shape
    assert K == Kb, "contraction lengths differ"
    if K > INT32_TERMS:
        return gemm64(A, B, transA, transB)
    C = np.empty((M, N), dtype=np.int32)
    _check(lib().fxp_ref_gemm(int(transA), int(transB), M, N, K, _ptr(A), A.shape[1], _ptr(B), B.shape[1], _ptr(C),
                              N), "gemm")
    return C


INT32_TERMS = 133144      # the longest contraction whose sums an int32 always holds (127^2 * 133144 < 2^31)


def gemm64(A, B, transA=False, transB=False):
    """The same product with exact int64 sums (what gemm returns for contractions beyond INT32_TERMS)."""
    A = np.ascontiguousarray(A, dtype=np.int8)
    B = np.ascontiguousarray(B, dtype=np.int8)
    M, K = (A.shape[1], A.shape[0]) if transA else A.shape
    Kb, N = (B.shape[1], B.shape[0]) if transB else B.shape
    assert K == Kb, "contraction lengths differ"
    C = np.empty((M, N), dtype=np.int64)
    _check(lib().fxp_ref_gemm64(int(transA), int(transB), M, N, K, _ptr(A), A.shape[1], _ptr(B), B.shape[1], _ptr(C),
                                N), "gemm64")
    return C


def unmap(acc, eA, eB=None, bitsA=8, bitsB=8):
    """int32 sums, or int64 sums (of a contraction beyond INT32_TERMS), to fp32."""
    acc = np.ascontiguousarray(acc)
    out = np.empty(acc.shape, dtype=np.float32)
    if acc.dtype == np.int64:
        _check(lib().fxp_ref_unmap64(_ptr(acc), acc.size, int(eA), bitsA, int(eB) if eB is not None else 0,
                                     bitsB if eB is not None else 0, _ptr(out)), "unmap64")
        return out
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    _check(lib().fxp_ref_unmap(_ptr(acc), acc.size, int(eA), bitsA, int(eB) if eB is not None else 0,
                               bitsB if eB is not None else 0, _ptr(out)), "unmap")
    return out


def unmap_i8(q, eA, bits=8):
    q = np.ascontiguousarray(q, dtype=np.int8)
    out = np.empty(q.shape, dtype=np.float32)
    _check(lib().fxp_ref_unmap_i8(_ptr(q), q.size, int(eA), bits, _ptr(out)), "unmap_i8")
    return out


def linear_fwd(X, W, seed=0, step=0, rounding=STOCHASTIC, bits=8):
    """Returns Y and the saved state dict(Xq, Wq, eX, eW)."""
    X, W = _f32(X), _f32(W)
    M, K = X.shape
    Kw, N = W.shape
    assert K == Kw
    Y = np.empty((M, N), dtype=np.float32)
    Xq = np.empty((M, K), dtype=np.int8)
    Wq = np.empty((K, N), dtype=np.int8)
    eX = np.zeros(1, dtype=np.int32)
    eW = np.zeros(1, dtype=np.int32)
    _check(lib().fxp_ref_linear_fwd(_ptr(X), _ptr(W), M, K, N, _ptr(Y), _ptr(Xq), _ptr(Wq), _ptr(eX), _ptr(eW), seed,
                                    step, rounding, bits), "linear_fwd")
    return Y, dict(Xq=Xq, Wq=Wq, eX=int(eX[0]), eW=int(eW[0]))


def linear_bwd(dY, saved, seed=0, step=0, rounding=STOCHASTIC, bits=8, need_dX=True, need_dW=True):
    """Returns dX, dW and dict(dYq, eG)."""
    dY = _f32(dY)
    M, N = dY.shape
    K = saved["Xq"].shape[1]
    dX = np.empty((M, K), dtype=np.float32) if need_dX else None
    dW = np.empty((K, N), dtype=np.float32) if need_dW else None
    dYq = np.empty((M, N), dtype=np.int8)
    eG = np.zeros(1, dtype=np.int32)
    _check(lib().fxp_ref_linear_bwd(_ptr(dY), _ptr(saved["Xq"]), _ptr(saved["Wq"]), saved["eX"], saved["eW"], M, K, N,
                                    _ptr(dX), _ptr(dW), _ptr(dYq), _ptr(eG), seed, step, rounding, bits),
           "linear_bwd")
    return dX, dW, dict(dYq=dYq, eG=int(eG[0]))


# ---- convolution, channels-last: X[N,H,W,C], W[Cout,KH,KW,C], Y / dY [N,Ho,Wo,Cout] ----------------
def conv_out_hw(H, W, KH, KW, stride, pad):
    return (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1


def _i8(a):
    return np.ascontiguousarray(a, dtype=np.int8)


def conv2d_fwd_acc(Xq, Wq, stride=1, pad=0):
    Xq, Wq = _i8(Xq), _i8(Wq)
    N, H, W, C = Xq.shape
    Cout, KH, KW, C2 = Wq.shape
    assert C == C2
    Ho, Wo = conv_out_hw(H, W, KH, KW, stride, pad)
    acc = np.empty((N, Ho, Wo, Cout), dtype=np.int32)
    _check(lib().fxp_ref_conv2d_fwd_acc(_ptr(Xq), N, H, W, C, _ptr(Wq), Cout, KH, KW, stride, pad, _ptr(acc)),
           "conv2d_fwd_acc")
    return acc


def conv2d_bwd_input_acc(Gq, Wq, x_shape, stride=1, pad=0):
    Gq, Wq = _i8(Gq), _i8(Wq)
    N, H, W, C = x_shape
    Cout, KH, KW, _ = Wq.shape
    acc = np.empty((N, H, W, C), dtype=np.int32)
    _check(lib().fxp_ref_conv2d_bwd_input_acc(_ptr(Gq), _ptr(Wq), N, H, W, C, Cout, KH, KW, stride, pad, _ptr(acc)),
           "conv2d_bwd_input_acc")
    return acc


def conv2d_bwd_weight_acc(Xq, Gq, w_shape, stride=1, pad=0):
    Xq, Gq = _i8(Xq), _i8(Gq)
    N, H, W, C = Xq.shape
    Cout, KH, KW, _ = w_shape
    Ho, Wo = conv_out_hw(H, W, KH, KW, stride, pad)
    if N * Ho * Wo > INT32_TERMS:            # more output pixels than an int32 sum is sure to hold: exact int64 sums
        acc = np.empty((Cout, KH, KW, C), dtype=np.int64)
        _check(lib().fxp_ref_conv2d_bwd_weight_acc64(_ptr(Xq), _ptr(Gq), N, H, W, C, Cout, KH, KW, stride, pad, _ptr(acc)),
               "conv2d_bwd_weight_acc64")
        return acc
    acc = np.empty((Cout, KH, KW, C), dtype=np.int32)
    _check(lib().fxp_ref_conv2d_bwd_weight_acc(_ptr(Xq), _ptr(Gq), N, H, W, C, Cout, KH, KW, stride, pad, _ptr(acc)),
           "conv2d_bwd_weight_acc")
    return acc


def conv2d_fwd(X, Wt, stride=1, pad=0, seed=0, step=0, rounding=STOCHASTIC, bits=8):
    """Returns Y[N,Ho,Wo,Cout] and the saved state dict(Xq, Wq, eX, eW, stride, pad)."""
    X, Wt = _f32(X), _f32(Wt)
    N, H, W, C = X.shape
    Cout, KH, KW, _ = Wt.shape
    Ho, Wo = conv_out_hw(H, W, KH, KW, stride, pad)
    Y = np.empty((N, Ho, Wo, Cout), dtype=np.float32)
    Xq = np.empty(X.shape, dtype=np.int8)
    Wq = np.empty(Wt.shape, dtype=np.int8)
    eX, eW = np.zeros(1, np.int32), np.zeros(1, np.int32)
    _check(lib().fxp_ref_conv2d_fwd(_ptr(X), _ptr(Wt), N, H, W, C, Cout, KH, KW, stride, pad, _ptr(Y), _ptr(Xq), _ptr(Wq),
                                    _ptr(eX), _ptr(eW), seed, step, rounding, bits), "conv2d_fwd")
    return Y, dict(Xq=Xq, Wq=Wq, eX=int(eX[0]), eW=int(eW[0]), stride=stride, pad=pad)


def conv2d_bwd(dY, saved, seed=0, step=0, rounding=STOCHASTIC, bits=8, need_dX=True, need_dW=True):
    dY = _f32(dY)
    Xq, Wq = saved["Xq"], saved["Wq"]
    N, H, W, C = Xq.shape
    Cout, KH, KW, _ = Wq.shape
    dX = np.empty(Xq.shape, dtype=np.float32) if need_dX else None
    dW = np.empty(Wq.shape, dtype=np.float32) if need_dW else None
    dYq = np.empty(dY.shape, dtype=np.int8)
    eG = np.zeros(1, np.int32)
    _check(lib().fxp_ref_conv2d_bwd(_ptr(dY), _ptr(Xq), _ptr(Wq), saved["eX"], saved["eW"], N, H, W, C, Cout, KH, KW,
                                    saved["stride"], saved["pad"], _ptr(dX), _ptr(dW), _ptr(dYq), _ptr(eG), seed, step,
                                    rounding, bits), "conv2d_bwd")
    return dX, dW, dict(dYq=dYq, eG=int(eG[0]))


# ---- batched products (attention matmuls): A[batch,M,K], Bm[batch,K,N] or [batch,N,K] with transB -------
def gemm_batched(A, B, transA=False, transB=False):
    """A[batch,.,.], B[batch,.,.] int8, dense; returns int32 C[batch,M,N] with C_b = op(A_b) op(B_b)."""
    A, B = _i8(A), _i8(B)
    batch = A.shape[0]
    assert B.shape[0] == batch
    M, K = (A.shape[2], A.shape[1]) if transA else A.shape[1:]
    Kb, N = (B.shape[2], B.shape[1]) if transB else B.shape[1:]
    assert K == Kb, "contraction lengths differ"
    C = np.empty((batch, M, N), dtype=np.int32)
    _check(lib().fxp_ref_gemm_batched(int(transA), int(transB), M, N, K, _ptr(A), A.shape[2], A.shape[1] * A.shape[2],
                                      _ptr(B), B.shape[2], B.shape[1] * B.shape[2], _ptr(C), N, M * N, batch),
           "gemm_batched")
    return C


def bmm_fwd(A, Bm, transB=False, seed=0, step=0, rounding=STOCHASTIC, bits=8):
    """Returns Y[batch,M,N] and the saved state dict(Aq, Bq, eA, eB, transB)."""
    A, Bm = _f32(A), _f32(Bm)
    batch, M, K = A.shape
    N = Bm.shape[1] if transB else Bm.shape[2]
    assert Bm.shape == ((batch, N, K) if transB else (batch, K, N))
    Y = np.empty((batch, M, N), dtype=np.float32)
    Aq = np.empty(A.shape, dtype=np.int8)
    Bq = np.empty(Bm.shape, dtype=np.int8)
    eA = np.zeros(1, dtype=np.int32)
    eB = np.zeros(1, dtype=np.int32)
    _check(lib().fxp_ref_bmm_fwd(_ptr(A), _ptr(Bm), batch, M, K, N, int(transB), _ptr(Y), _ptr(Aq), _ptr(Bq), _ptr(eA),
                                 _ptr(eB), seed, step, rounding, bits), "bmm_fwd")
    return Y, dict(Aq=Aq, Bq=Bq, eA=int(eA[0]), eB=int(eB[0]), transB=bool(transB))


def bmm_bwd(dY, saved, seed=0, step=0, rounding=STOCHASTIC, bits=8, need_dA=True, need_dB=True):
    """Returns dA, dBm (in the layouts of A, Bm) and dict(dYq, eG)."""
    dY = _f32(dY)
    batch, M, N = dY.shape
    K = saved["Aq"].shape[2]
    dA = np.empty(saved["Aq"].shape, dtype=np.float32) if need_dA else None
    dB = np.empty(saved["Bq"].shape, dtype=np.float32) if need_dB else None
    dYq = np.empty(dY.shape, dtype=np.int8)
    eG = np.zeros(1, dtype=np.int32)
    _check(lib().fxp_ref_bmm_bwd(_ptr(dY), _ptr(saved["Aq"]), _ptr(saved["Bq"]), saved["eA"], saved["eB"], batch, M, K, N,
                                 int(saved["transB"]), _ptr(dA), _ptr(dB), _ptr(dYq), _ptr(eG), seed, step, rounding,
                                 bits), "bmm_bwd")
    return dA, dB, dict(dYq=dYq, eG=int(eG[0]))


# ---- int16 weight update (Remark 5, App. A.4) ------------------------------------------------------------
TAG_AXPY_XY, TAG_AXPY_U, TAG_AXPY_A = 3, 4, 5


def map16(x, e_max, seed=0, stream_id=0, rounding=STOCHASTIC):
    x = _f32(x)
    q = np.empty(x.shape, dtype=np.int16)
    _check(lib().fxp_ref_map16(_ptr(x), x.size, int(e_max), _ptr(q), seed, stream_id, rounding), "map16")
    return q


def axpy16(x, y, a, seed=0, step=0, rounding=STOCHASTIC):
    """z = x_hat + SR(a_hat * y_hat) in 16-bit fixed point; returns z (fp32) and the scales (eX, eY, eA)."""
    x, y = _f32(x), _f32(y)
    assert x.shape == y.shape
    z = np.empty(x.shape, dtype=np.float32)
    e = np.zeros(3, dtype=np.int32)
    _check(lib().fxp_ref_axpy16(_ptr(x), _ptr(y), float(a), x.size, _ptr(z), _ptr(e), seed, step, rounding), "axpy16")
    return z, tuple(int(v) for v in e)


def sgd16_step(w, g, v=None, lr=0.1, momentum=0.0, weight_decay=0.0, seed=0, step=0, rounding=STOCHASTIC):
    """Returns (w_new, v_new); the inputs are left untouched."""
    w, g = _f32(w).copy(), _f32(g)
    v = _f32(v).copy() if v is not None else (np.zeros_like(w) if momentum != 0.0 else None)
    tmp = np.empty_like(w) if weight_decay != 0.0 else None
    _check(lib().fxp_ref_sgd16_step(_ptr(w), _ptr(g), _ptr(v), w.size, float(lr), float(momentum), float(weight_decay),
                                    _ptr(tmp), seed, step, rounding), "sgd16_step")
    return w, v


def sgd16_step_multi(ws, gs, vs=None, lr=0.1, momentum=0.0, weight_decay=0.0, seed=0, step=0, rounding=STOCHASTIC):
    """One step over a list of parameter tensors (own scales per tensor); returns (new ws, new vs), inputs untouched."""
    import ctypes as c
    ws = [_f32(w).copy() for w in ws]
    gs = [_f32(g) for g in gs]
    if momentum != 0.0:
        vs = [(_f32(v).copy() if v is not None else np.zeros_like(w)) for v, w in zip(vs or [None] * len(ws), ws)]
    else:
        vs = None
    tmps = [np.empty_like(w) for w in ws] if weight_decay != 0.0 else None
    k = len(ws)

    def ptrs(arrs):
        return (c.c_void_p * k)(*[a.ctypes.data for a in arrs]) if arrs is not None else None

    n = (c.c_uint64 * k)(*[w.size for w in ws])
    _check(lib().fxp_ref_sgd16_step_multi(ptrs(ws), ptrs(gs), ptrs(vs), ptrs(tmps), n, k, float(lr), float(momentum),
                                          float(weight_decay), seed, step, rounding), "sgd16_step_multi")
    return ws, vs
