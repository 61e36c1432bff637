"""Thin Python binding of libfxp (include/fxp.h): argument marshalling only.

Every function takes torch CUDA tensors, allocates the outputs with torch, hands raw
device pointers and the current torch stream to the C ABI and raises FxpError on a
non-zero status.  All arithmetic runs in the HIP kernels; there is no CPU or PyTorch
fallback: if libfxp.so cannot be loaded, or a tensor is not on the GPU, the call fails.
"""
import ctypes
import os

import torch

from . import build as _build

STOCHASTIC, NEAREST = 0, 1
OP_SCALE, OP_GEMM, OP_LINEAR_FWD, OP_LINEAR_BWD, OP_BMM_FWD, OP_BMM_BWD = 0, 1, 2, 3, 4, 5
TAG_X, TAG_W, TAG_DY = 0, 1, 2
ABSMAX_WORDS = 256      # uint32 words of an abs-max area (FXP_ABSMAX_WORDS)


class FxpError(RuntimeError):
    pass


class _Saved(ctypes.Structure):
    _fields_ = [("Xq", ctypes.c_void_p), ("XqT", ctypes.c_void_p), ("Wq", ctypes.c_void_p), ("WqT", ctypes.c_void_p),
                ("eX", ctypes.c_void_p), ("eW", ctypes.c_void_p)]


class _MapDesc(ctypes.Structure):
    _fields_ = [("x", ctypes.c_void_p), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64), ("e_max", ctypes.c_void_p),
                ("q", ctypes.c_void_p), ("qT", ctypes.c_void_p), ("stream_id", ctypes.c_uint64)]


class _SgdTensor(ctypes.Structure):
    _fields_ = [("w", ctypes.c_void_p), ("g", ctypes.c_void_p), ("v", ctypes.c_void_p), ("tmp", ctypes.c_void_p),
                ("n", ctypes.c_size_t)]


class _ConvShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in ("N", "H", "W", "C", "Cout", "KH", "KW", "stride", "pad")]


class _ConvSaved(ctypes.Structure):
    _fields_ = [("Xq", ctypes.c_void_p), ("Wq", ctypes.c_void_p), ("WqT", ctypes.c_void_p), ("WqF", ctypes.c_void_p),
                ("eX", ctypes.c_void_p), ("eW", ctypes.c_void_p)]


_lib = None


def lib():
    """Load libfxp.so (building it first only when no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    path = _build.LIB
    if not os.path.exists(path):
        path = _build.build()
    L = ctypes.CDLL(path)
    c = ctypes
    vp, i32, i64, u64, sz, ci = c.c_void_p, c.c_int32, c.c_int64, c.c_uint64, c.c_size_t, c.c_int
    L.fxp_strerror.restype = c.c_char_p
    L.fxp_strerror.argtypes = [ci]
    L.fxp_version.restype = ci
    L.fxp_workspace_bytes.restype = sz
    L.fxp_workspace_bytes.argtypes = [ci, i64, i64, i64]
    L.fxp_scale.argtypes = [vp, sz, vp, vp, sz, vp]
    L.fxp_map.argtypes = [vp, i64, i64, vp, vp, vp, u64, u64, ci, ci, vp]
    L.fxp_scale_map.argtypes = [vp, i64, i64, vp, vp, vp, u64, u64, ci, ci, vp, sz, vp]
    L.fxp_gemm.argtypes = [ci, ci, i64, i64, i64, vp, i64, vp, i64, vp, i64, vp, sz, vp]
    L.fxp_unmap.argtypes = [vp, sz, vp, ci, vp, ci, vp, vp]
    L.fxp_unmap_i8.argtypes = [vp, sz, vp, ci, vp, vp]
    L.fxp_gemm_unmap.argtypes = [ci, ci, i64, i64, i64, vp, i64, vp, i64, vp, ci, vp, ci, vp, i64, vp, sz, vp]
    L.fxp_gemm_unmap_absmax.argtypes = [ci, ci, i64, i64, i64, vp, i64, vp, i64, vp, ci, vp, ci, vp, i64, vp, vp, sz, vp]
    L.fxp_map_absmax.argtypes = [vp, i64, i64, vp, vp, vp, vp, u64, u64, ci, ci, vp]
    L.fxp_linear_fwd.argtypes = [vp, vp, i64, i64, i64, vp, c.POINTER(_Saved), u64, u64, ci, ci, vp, sz, vp]
    L.fxp_linear_bwd.argtypes = [vp, c.POINTER(_Saved), i64, i64, i64, vp, vp, vp, vp, vp, u64, u64, ci, ci, vp, sz, vp]
    L.fxp_linear_fwd_guess.argtypes = L.fxp_linear_fwd.argtypes
    L.fxp_linear_bwd_guess.argtypes = L.fxp_linear_bwd.argtypes
    L.fxp_linear_fwd_guess.restype = ci
    L.fxp_linear_bwd_guess.restype = ci
    L.fxp_linear_fwd_static.argtypes = [vp, vp, i64, i64, i64, vp, c.POINTER(_Saved), u64, u64, ci, ci, vp]
    L.fxp_linear_fwd_static.restype = ci
    L.fxp_static_scratch_bytes.restype = sz
    L.fxp_static_scratch_bytes.argtypes = []
    L.fxp_clock_probe.argtypes = [vp, c.c_uint32, vp]
    L.fxp_clock_probe.restype = ci
    L.fxp_timeline_begin.argtypes = [ci]
    L.fxp_timeline_begin.restype = ci
    L.fxp_timeline_end.argtypes = [vp, vp, ci, vp]
    L.fxp_timeline_end.restype = ci
    L.fxp_conv2d_workspace_bytes.restype = sz
    L.fxp_conv2d_workspace_bytes.argtypes = [c.POINTER(_ConvShape), ci]
    L.fxp_conv2d_fwd.argtypes = [vp, vp, c.POINTER(_ConvShape), vp, c.POINTER(_ConvSaved), u64, u64, ci, ci, vp, sz, vp]
    L.fxp_conv2d_bwd.argtypes = [vp, c.POINTER(_ConvSaved), c.POINTER(_ConvShape), vp, vp, vp, vp, vp, u64, u64, ci, ci,
                                 vp, sz, vp]
    L.fxp_conv2d_fwd.restype = ci
    L.fxp_conv2d_bwd.restype = ci
    L.fxp_gemm_batched.argtypes = [i64, i64, i64, vp, i64, i64, vp, i64, i64, vp, i64, i64, i64, vp]
    L.fxp_gemm_unmap_batched.argtypes = [i64, i64, i64, vp, i64, i64, vp, i64, i64, vp, ci, vp, ci, vp, i64, i64, i64, vp]
    L.fxp_bmm_fwd.argtypes = [vp, vp, i64, i64, i64, i64, ci, vp, c.POINTER(_Saved), u64, u64, ci, ci, vp, sz, vp]
    L.fxp_bmm_bwd.argtypes = [vp, c.POINTER(_Saved), i64, i64, i64, i64, ci, vp, vp, vp, vp, vp, u64, u64, ci, ci, vp, sz,
                              vp]
    L.fxp_bmm_fwd_guess.argtypes = L.fxp_bmm_fwd.argtypes
    L.fxp_bmm_bwd_guess.argtypes = L.fxp_bmm_bwd.argtypes
    L.fxp_bmm_fwd_guess.restype = ci
    L.fxp_bmm_bwd_guess.restype = ci
    L.fxp_map2.argtypes = [c.POINTER(_MapDesc), c.POINTER(_MapDesc), u64, ci, ci, vp]
    L.fxp_scale_map2.argtypes = [c.POINTER(_MapDesc), c.POINTER(_MapDesc), u64, ci, ci, vp, sz, vp]
    L.fxp_map2.restype = ci
    L.fxp_scale_map2.restype = ci
    L.fxp_sgd16_multi_workspace_bytes.restype = sz
    L.fxp_sgd16_multi_workspace_bytes.argtypes = [c.POINTER(_SgdTensor), sz]
    L.fxp_sgd16_step_multi.argtypes = [c.POINTER(_SgdTensor), sz, c.c_float, c.c_float, c.c_float, u64, u64, ci, vp, sz, vp]
    L.fxp_sgd16_step_multi.restype = ci
    L.fxp_sgd16_workspace_bytes.restype = sz
    L.fxp_sgd16_workspace_bytes.argtypes = []
    L.fxp_axpy16.argtypes = [vp, vp, c.c_float, sz, vp, vp, u64, u64, ci, vp, sz, vp]
    L.fxp_sgd16_step.argtypes = [vp, vp, vp, sz, c.c_float, c.c_float, c.c_float, vp, u64, u64, ci, vp, sz, vp]
    L.fxp_axpy16.restype = ci
    L.fxp_sgd16_step.restype = ci
    for name in ("fxp_scale", "fxp_map", "fxp_scale_map", "fxp_gemm", "fxp_unmap", "fxp_unmap_i8", "fxp_gemm_unmap",
                 "fxp_gemm_unmap_absmax", "fxp_map_absmax",
                 "fxp_linear_fwd", "fxp_linear_bwd", "fxp_gemm_batched", "fxp_gemm_unmap_batched", "fxp_bmm_fwd",
                 "fxp_bmm_bwd"):
        getattr(L, name).restype = ci
    _lib = L
    return L


def _check(rc, what):
    if rc != 0:
        raise FxpError(f"{what}: {lib().fxp_strerror(rc).decode()} ({rc})")


def _dev(t, dtype, what):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise FxpError(f"{what} must be a CUDA tensor: libfxp has no CPU path")
    if t.dtype != dtype or not t.is_contiguous():
        raise FxpError(f"{what} must be a contiguous {dtype} tensor")
    return t


def _p(t):
    return None if t is None else t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def workspace_bytes(op, M, N=0, K=0):
    return int(lib().fxp_workspace_bytes(op, M, N, K))


def _ws(op, M, N=0, K=0, device=None):
    return torch.empty(max(256, workspace_bytes(op, M, N, K)), dtype=torch.uint8, device=device)


def scale(x, ws=None):
    """e_max of a tensor as a 1-element int32 device tensor (no synchronisation)."""
    x = _dev(x, torch.float32, "x")
    e = torch.empty(1, dtype=torch.int32, device=x.device)
    ws = ws if ws is not None else _ws(OP_SCALE, x.numel(), device=x.device)
    _check(lib().fxp_scale(_p(x), x.numel(), _p(e), _p(ws), ws.numel(), _stream()), "fxp_scale")
    return e


def _map_outputs(x, want_q, want_qT):
    rows, cols = x.shape
    q = torch.empty((rows, cols), dtype=torch.int8, device=x.device) if want_q else None
    qT = torch.empty((cols, rows), dtype=torch.int8, device=x.device) if want_qT else None
    return q, qT


def map(x, e_max, seed=0, stream_id=0, rounding=STOCHASTIC, bits=8, want_q=True, want_qT=False):
    """(q, qT) int8 tensors of x[rows, cols] under the device scale e_max."""
    x = _dev(x, torch.float32, "x")
    e_max = _dev(e_max, torch.int32, "e_max")
    assert x.dim() == 2
    q, qT = _map_outputs(x, want_q, want_qT)
    _check(lib().fxp_map(_p(x), x.shape[0], x.shape[1], _p(e_max), _p(q), _p(qT), seed, stream_id, rounding, bits,
                         _stream()), "fxp_map")
    return q, qT


def scale_map(x, seed=0, stream_id=0, rounding=STOCHASTIC, bits=8, want_q=True, want_qT=False, ws=None):
    """(e_max, q, qT): scale and map in one call."""
    x = _dev(x, torch.float32, "x")
    assert x.dim() == 2
    e = torch.empty(1, dtype=torch.int32, device=x.device)
    q, qT = _map_outputs(x, want_q, want_qT)
    ws = ws if ws is not None else _ws(OP_SCALE, x.numel(), device=x.device)
    _check(lib().fxp_scale_map(_p(x), x.shape[0], x.shape[1], _p(e), _p(q), _p(qT), seed, stream_id, rounding, bits,
                               _p(ws), ws.numel(), _stream()), "fxp_scale_map")
    return e, q, qT


def _gemm_dims(A, B, transA, transB):
    M, K = (A.shape[1], A.shape[0]) if transA else A.shape
    Kb, N = (B.shape[1], B.shape[0]) if transB else B.shape
    if K != Kb:
        raise FxpError("contraction lengths differ")
    return M, N, K


def gemm(A, B, transA=False, transB=False, ws=None):
    """int32 C[M,N] = op(A) op(B) for int8 operands."""
    A, B = _dev(A, torch.int8, "A"), _dev(B, torch.int8, "B")
    M, N, K = _gemm_dims(A, B, transA, transB)
    C = torch.empty((M, N), dtype=torch.int32, device=A.device)
    ws = ws if ws is not None else _ws(OP_GEMM, M, N, K, device=A.device)
    _check(lib().fxp_gemm(int(transA), int(transB), M, N, K, _p(A), A.shape[1], _p(B), B.shape[1], _p(C), N, _p(ws),
                          ws.numel(), _stream()), "fxp_gemm")
    return C


def unmap(acc, eA, eB=None, bitsA=8, bitsB=8, out=None):
    acc = _dev(acc, torch.int32, "acc")
    out = out if out is not None else torch.empty(acc.shape, dtype=torch.float32, device=acc.device)
    _check(lib().fxp_unmap(_p(acc), acc.numel(), _p(eA), bitsA, _p(eB), bitsB, _p(out), _stream()), "fxp_unmap")
    return out


def unmap_i8(q, eA, bits=8):
    q = _dev(q, torch.int8, "q")
    out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    _check(lib().fxp_unmap_i8(_p(q), q.numel(), _p(eA), bits, _p(out), _stream()), "fxp_unmap_i8")
    return out


def gemm_unmap(A, B, eA, eB, transA=False, transB=False, bitsA=8, bitsB=8, ws=None):
    """fp32 C = unmap(op(A) op(B)) with the inverse mapping fused into the GEMM."""
    A, B = _dev(A, torch.int8, "A"), _dev(B, torch.int8, "B")
    M, N, K = _gemm_dims(A, B, transA, transB)
    C = torch.empty((M, N), dtype=torch.float32, device=A.device)
    ws = ws if ws is not None else _ws(OP_GEMM, M, N, K, device=A.device)
    _check(lib().fxp_gemm_unmap(int(transA), int(transB), M, N, K, _p(A), A.shape[1], _p(B), B.shape[1], _p(eA), bitsA,
                                _p(eB), bitsB, _p(C), N, _p(ws), ws.numel(), _stream()), "fxp_gemm_unmap")
    return C


def gemm_unmap_absmax(A, B, eA, eB, absmax, transA=False, transB=False, bitsA=8, bitsB=8, ws=None):
    """gemm_unmap that also raises the abs-max area `absmax` (ABSMAX_WORDS int32 words, bits of max |C|) for map_absmax."""
    A, B = _dev(A, torch.int8, "A"), _dev(B, torch.int8, "B")
    M, N, K = _gemm_dims(A, B, transA, transB)
    C = torch.empty((M, N), dtype=torch.float32, device=A.device)
    ws = ws if ws is not None else _ws(OP_GEMM, M, N, K, device=A.device)
    _check(lib().fxp_gemm_unmap_absmax(int(transA), int(transB), M, N, K, _p(A), A.shape[1], _p(B), B.shape[1], _p(eA), bitsA,
                                   _p(eB), bitsB, _p(C), N, _p(absmax), _p(ws), ws.numel(), _stream()),
           "fxp_gemm_unmap_absmax")
    return C


def map_absmax(x, absmax, seed=0, stream_id=0, rounding=STOCHASTIC, bits=8, want_q=True, want_qT=False):
    """(e_max, q, qT) of x with the scale taken from the abs-max area `absmax` (its maximum = bits of max |x|)."""
    x = _dev(x, torch.float32, "x")
    assert x.dim() == 2
    e = torch.empty(1, dtype=torch.int32, device=x.device)
    q, qT = _map_outputs(x, want_q, want_qT)
    _check(lib().fxp_map_absmax(_p(x), x.shape[0], x.shape[1], _p(absmax), _p(e), _p(q), _p(qT), seed, stream_id, rounding,
                            bits, _stream()), "fxp_map_absmax")
    return e, q, qT


class LayerBuffers:
    """Caller-owned device buffers of one layer shape, allocated once and reused."""

    def __init__(self, M, K, N, device="cuda"):
        i8 = dict(dtype=torch.int8, device=device)
        self.M, self.K, self.N = M, K, N
        self.Xq, self.XqT = torch.empty((M, K), **i8), torch.empty((K, M), **i8)
        self.Wq, self.WqT = torch.empty((K, N), **i8), torch.empty((N, K), **i8)
        self.dYq, self.dYqT = torch.empty((M, N), **i8), torch.empty((N, M), **i8)
        self.e = torch.zeros(3, dtype=torch.int32, device=device)       # eX, eW, e_dY
        self.Y = torch.empty((M, N), dtype=torch.float32, device=device)
        self.dX = torch.empty((M, K), dtype=torch.float32, device=device)
        self.dW = torch.empty((K, N), dtype=torch.float32, device=device)
        nbytes = max(workspace_bytes(OP_LINEAR_FWD, M, N, K), workspace_bytes(OP_LINEAR_BWD, M, N, K), 256)
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.saved = _Saved(_p(self.Xq), _p(self.XqT), _p(self.Wq), _p(self.WqT), self.e[0:1].data_ptr(),
                            self.e[1:2].data_ptr())

    @property
    def eX(self):
        return self.e[0:1]

    @property
    def eW(self):
        return self.e[1:2]

    @property
    def e_dY(self):
        return self.e[2:3]


def linear_fwd(X, W, buf, seed=0, step=0, rounding=STOCHASTIC, bits=8, guess=False):
    """Y = unmap(map(X) map(W)); fills buf.Xq/XqT/Wq/WqT/eX/eW and returns buf.Y.  guess: the scales buf.e holds
    from the previous call are taken as guesses (fxp_linear_fwd_guess)."""
    X, W = _dev(X, torch.float32, "X"), _dev(W, torch.float32, "W")
    M, K = X.shape
    if W.shape[0] != K or (M, K, W.shape[1]) != (buf.M, buf.K, buf.N):
        raise FxpError("shapes do not match the layer buffers")
    fn = lib().fxp_linear_fwd_guess if guess else lib().fxp_linear_fwd
    _check(fn(_p(X), _p(W), M, K, buf.N, _p(buf.Y), ctypes.byref(buf.saved), seed, step, rounding,
                                bits, _p(buf.ws), buf.ws.numel(), _stream()), "fxp_linear_fwd")
    return buf.Y


def linear_fwd_static(X, W, buf, seed=0, step=0, rounding=STOCHASTIC, bits=8):
    """linear_fwd through the entry point that takes no workspace (its scratch is a device array inside the library)."""
    X, W = _dev(X, torch.float32, "X"), _dev(W, torch.float32, "W")
    M, K = X.shape
    if W.shape[0] != K or (M, K, W.shape[1]) != (buf.M, buf.K, buf.N):
        raise FxpError("shapes do not match the layer buffers")
    _check(lib().fxp_linear_fwd_static(_p(X), _p(W), M, K, buf.N, _p(buf.Y), ctypes.byref(buf.saved), seed, step, rounding,
                                       bits, _stream()), "fxp_linear_fwd_static")
    return buf.Y


def linear_bwd(dY, buf, seed=0, step=0, rounding=STOCHASTIC, bits=8, need_dX=True, need_dW=True, guess=False):
    """(dX, dW) from the upstream gradient and the operands the forward call saved."""
    dY = _dev(dY, torch.float32, "dY")
    if tuple(dY.shape) != (buf.M, buf.N):
        raise FxpError("shapes do not match the layer buffers")
    dX = buf.dX if need_dX else None
    dW = buf.dW if need_dW else None
    fn = lib().fxp_linear_bwd_guess if guess else lib().fxp_linear_bwd
    _check(fn(_p(dY), ctypes.byref(buf.saved), buf.M, buf.K, buf.N, _p(dX), _p(dW), _p(buf.dYq),
                                _p(buf.dYqT), buf.e[2:3].data_ptr(), seed, step, rounding, bits, _p(buf.ws),
                                buf.ws.numel(), _stream()), "fxp_linear_bwd")
    return dX, dW


def gemm_batched(A, B, eA=None, eB=None, bitsA=8, bitsB=8):
    """C_b = A_b[M,K] B_b[N,K]^T for dense int8 A[batch,M,K], B[batch,N,K]: int32, or fp32 through the fused
    inverse mapping when the scales eA (and eB) are given."""
    A, B = _dev(A, torch.int8, "A"), _dev(B, torch.int8, "B")
    if A.dim() != 3 or B.dim() != 3 or A.shape[0] != B.shape[0] or A.shape[2] != B.shape[2]:
        raise FxpError("gemm_batched wants A[batch,M,K] and B[batch,N,K]")
    batch, M, K = A.shape
    N = B.shape[1]
    if eA is None:
        C = torch.empty((batch, M, N), dtype=torch.int32, device=A.device)
        _check(lib().fxp_gemm_batched(M, N, K, _p(A), K, M * K, _p(B), K, N * K, _p(C), N, M * N, batch, _stream()),
               "fxp_gemm_batched")
    else:
        C = torch.empty((batch, M, N), dtype=torch.float32, device=A.device)
        _check(lib().fxp_gemm_unmap_batched(M, N, K, _p(A), K, M * K, _p(B), K, N * K, _p(eA), bitsA, _p(eB), bitsB, _p(C),
                                            N, M * N, batch, _stream()), "fxp_gemm_unmap_batched")
    return C


class BmmBuffers:
    """Caller-owned device buffers of one batched product layer (attention matmul), allocated once."""

    def __init__(self, batch, M, K, N, transB=False, device="cuda"):
        i8 = dict(dtype=torch.int8, device=device)
        f32 = dict(dtype=torch.float32, device=device)
        self.batch, self.M, self.K, self.N, self.transB = batch, M, K, N, bool(transB)
        b_shape = (batch, N, K) if transB else (batch, K, N)
        self.Aq, self.AqT = torch.empty((batch, M, K), **i8), torch.empty((K, batch * M), **i8)
        self.Bq, self.BqT = torch.empty(b_shape, **i8), torch.empty((b_shape[2], batch * b_shape[1]), **i8)
        self.dYq, self.dYqT = torch.empty((batch, M, N), **i8), torch.empty((N, batch * M), **i8)
        self.e = torch.zeros(3, dtype=torch.int32, device=device)       # eA, eB, e_dY
        self.Y = torch.empty((batch, M, N), **f32)
        self.dA = torch.empty((batch, M, K), **f32)
        self.dB = torch.empty(b_shape, **f32)
        nbytes = max(workspace_bytes(OP_BMM_FWD, M, N, K), workspace_bytes(OP_BMM_BWD, M, N, K), 256)
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.saved = _Saved(_p(self.Aq), _p(self.AqT), _p(self.Bq), _p(self.BqT), self.e[0:1].data_ptr(),
                            self.e[1:2].data_ptr())


def bmm_fwd(A, Bm, buf, seed=0, step=0, rounding=STOCHASTIC, bits=8, guess=False):
    """Y_b = unmap(map(A)_b op(map(Bm)_b)); fills buf.Aq/AqT/Bq/BqT/e[0:2] and returns buf.Y."""
    A, Bm = _dev(A, torch.float32, "A"), _dev(Bm, torch.float32, "Bm")
    if tuple(A.shape) != tuple(buf.Aq.shape) or tuple(Bm.shape) != tuple(buf.Bq.shape):
        raise FxpError("shapes do not match the layer buffers")
    _check((lib().fxp_bmm_fwd_guess if guess else lib().fxp_bmm_fwd)(_p(A), _p(Bm), buf.batch, buf.M, buf.K, buf.N, int(buf.transB), _p(buf.Y),
                             ctypes.byref(buf.saved), seed, step, rounding, bits, _p(buf.ws), buf.ws.numel(), _stream()),
           "fxp_bmm_fwd")
    return buf.Y


def bmm_bwd(dY, buf, seed=0, step=0, rounding=STOCHASTIC, bits=8, need_dA=True, need_dB=True, guess=False):
    """(dA, dBm) from the upstream gradient and the operands the forward call saved."""
    dY = _dev(dY, torch.float32, "dY")
    if tuple(dY.shape) != (buf.batch, buf.M, buf.N):
        raise FxpError("shapes do not match the layer buffers")
    dA = buf.dA if need_dA else None
    dB = buf.dB if need_dB else None
    _check((lib().fxp_bmm_bwd_guess if guess else lib().fxp_bmm_bwd)(_p(dY), ctypes.byref(buf.saved), buf.batch, buf.M, buf.K, buf.N, int(buf.transB), _p(dA),
                             _p(dB), _p(buf.dYq), _p(buf.dYqT), buf.e[2:3].data_ptr(), seed, step, rounding, bits,
                             _p(buf.ws), buf.ws.numel(), _stream()), "fxp_bmm_bwd")
    return dA, dB


class ConvBuffers:
    """Caller-owned device buffers of one convolution layer (channels-last), allocated once."""

    def __init__(self, N, H, W, C, Cout, KH, KW, stride=1, pad=0, device="cuda"):
        self.shape = _ConvShape(N, H, W, C, Cout, KH, KW, stride, pad)
        self.Ho, self.Wo = (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1
        M, K = N * self.Ho * self.Wo, KH * KW * C
        i8 = dict(dtype=torch.int8, device=device)
        f32 = dict(dtype=torch.float32, device=device)
        self.Xq = torch.empty((N, H, W, C), **i8)
        self.Wq, self.WqT = torch.empty((Cout, K), **i8), torch.empty((K, Cout), **i8)
        self.WqF = torch.empty((C, KH * KW * Cout), **i8)
        self.dYq, self.dYqT = torch.empty((M, Cout), **i8), torch.empty((Cout, M), **i8)
        self.e = torch.zeros(3, dtype=torch.int32, device=device)          # eX, eW, e_dY
        self.Y = torch.empty((N, self.Ho, self.Wo, Cout), **f32)
        self.dX = torch.empty((N, H, W, C), **f32)
        self.dW = torch.empty((Cout, KH, KW, C), **f32)
        nbytes = max(int(lib().fxp_conv2d_workspace_bytes(ctypes.byref(self.shape), 0)),
                     int(lib().fxp_conv2d_workspace_bytes(ctypes.byref(self.shape), 1)), 256)
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.saved = _ConvSaved(_p(self.Xq), _p(self.Wq), _p(self.WqT), _p(self.WqF), self.e[0:1].data_ptr(),
                                self.e[1:2].data_ptr())


def conv2d_fwd(X, W, buf, seed=0, step=0, rounding=STOCHASTIC, bits=8):
    """Y[N,Ho,Wo,Cout] of the integer convolution layer; X[N,H,W,C], W[Cout,KH,KW,C] fp32."""
    X, W = _dev(X, torch.float32, "X"), _dev(W, torch.float32, "W")
    sh = buf.shape
    if tuple(X.shape) != (sh.N, sh.H, sh.W, sh.C) or tuple(W.shape) != (sh.Cout, sh.KH, sh.KW, sh.C):
        raise FxpError("shapes do not match the convolution buffers")
    _check(lib().fxp_conv2d_fwd(_p(X), _p(W), ctypes.byref(sh), _p(buf.Y), ctypes.byref(buf.saved), seed, step, rounding,
                                bits, _p(buf.ws), buf.ws.numel(), _stream()), "fxp_conv2d_fwd")
    return buf.Y


def conv2d_bwd(dY, buf, seed=0, step=0, rounding=STOCHASTIC, bits=8, need_dX=True, need_dW=True):
    dY = _dev(dY, torch.float32, "dY")
    sh = buf.shape
    if tuple(dY.shape) != (sh.N, buf.Ho, buf.Wo, sh.Cout):
        raise FxpError("shapes do not match the convolution buffers")
    dX = buf.dX if need_dX else None
    dW = buf.dW if need_dW else None
    _check(lib().fxp_conv2d_bwd(_p(dY), ctypes.byref(buf.saved), ctypes.byref(sh), _p(dX), _p(dW), _p(buf.dYq),
                                _p(buf.dYqT), buf.e[2:3].data_ptr(), seed, step, rounding, bits, _p(buf.ws),
                                buf.ws.numel(), _stream()), "fxp_conv2d_bwd")
    return dX, dW


def axpy16(x, y, a, out=None, seed=0, step=0, rounding=STOCHASTIC, ws=None):
    """z = x_hat + SR(a_hat * y_hat) in 16-bit fixed point; returns (z, e) with e = int32[3] scales of x, y, a."""
    x, y = _dev(x, torch.float32, "x"), _dev(y, torch.float32, "y")
    if x.shape != y.shape:
        raise FxpError("x and y differ in shape")
    z = out if out is not None else torch.empty_like(x)
    _dev(z, torch.float32, "out")
    e = torch.zeros(3, dtype=torch.int32, device=x.device)
    ws = ws if ws is not None else torch.empty(2 * workspace_bytes(OP_SCALE, 1), dtype=torch.uint8, device=x.device)
    _check(lib().fxp_axpy16(_p(x), _p(y), float(a), x.numel(), _p(z), _p(e), seed, step, rounding, _p(ws), ws.numel(),
                            _stream()), "fxp_axpy16")
    return z, e


class SgdBuffers:
    """Scratch of the int16 SGD step for tensors of up to n elements."""

    def __init__(self, n, device="cuda"):
        self.tmp = torch.empty(n, dtype=torch.float32, device=device)
        self.ws = torch.empty(int(lib().fxp_sgd16_workspace_bytes()), dtype=torch.uint8, device=device)


def sgd16_step(w, g, v, buf, lr, momentum=0.0, weight_decay=0.0, seed=0, step=0, rounding=STOCHASTIC):
    """In-place SGD step on w (and the momentum buffer v, which may be None when momentum == 0)."""
    w, g = _dev(w, torch.float32, "w"), _dev(g, torch.float32, "g")
    if v is not None:
        _dev(v, torch.float32, "v")
    if g.numel() != w.numel() or (v is not None and v.numel() != w.numel()) or buf.tmp.numel() < w.numel():
        raise FxpError("w, g, v and the scratch differ in size")
    _check(lib().fxp_sgd16_step(_p(w), _p(g), _p(v), w.numel(), float(lr), float(momentum), float(weight_decay),
                                _p(buf.tmp), seed, step, rounding, _p(buf.ws), buf.ws.numel(), _stream()),
           "fxp_sgd16_step")
    return w, v


def _desc(x, e, q, qT, stream_id):
    x = _dev(x, torch.float32, "x")
    if x.dim() != 2:
        raise FxpError("x must be a matrix")
    return _MapDesc(_p(x), x.shape[0], x.shape[1], _p(e), _p(q), _p(qT), stream_id)


def map2(xa, ea, xb, eb, seed=0, stream_ids=(0, 1), rounding=STOCHASTIC, bits=8):
    """fxp.map of two tensors (given scales) in one launch; returns ((qa, qaT), (qb, qbT))."""
    outs = [(torch.empty(x.shape, dtype=torch.int8, device=x.device),
             torch.empty((x.shape[1], x.shape[0]), dtype=torch.int8, device=x.device)) for x in (xa, xb)]
    da = _desc(xa, ea, outs[0][0], outs[0][1], stream_ids[0])
    db = _desc(xb, eb, outs[1][0], outs[1][1], stream_ids[1])
    _check(lib().fxp_map2(ctypes.byref(da), ctypes.byref(db), seed, rounding, bits, _stream()), "fxp_map2")
    return outs


def scale_map2(xa, xb, seed=0, stream_ids=(0, 1), rounding=STOCHASTIC, bits=8):
    """fxp.scale_map of two tensors in two launches; returns (e[2], (qa, qaT), (qb, qbT))."""
    e = torch.zeros(2, dtype=torch.int32, device=xa.device)
    outs = [(torch.empty(x.shape, dtype=torch.int8, device=x.device),
             torch.empty((x.shape[1], x.shape[0]), dtype=torch.int8, device=x.device)) for x in (xa, xb)]
    da = _desc(xa, e[0:1], outs[0][0], outs[0][1], stream_ids[0])
    db = _desc(xb, e[1:2], outs[1][0], outs[1][1], stream_ids[1])
    ws = torch.empty(2 * workspace_bytes(OP_SCALE, 1), dtype=torch.uint8, device=xa.device)
    _check(lib().fxp_scale_map2(ctypes.byref(da), ctypes.byref(db), seed, rounding, bits, _p(ws), ws.numel(), _stream()),
           "fxp_scale_map2")
    return e, outs[0], outs[1]


class SgdMultiBuffers:
    """Descriptor table and scratch for the multi-tensor int16 SGD step over fixed lists of parameter tensors."""

    def __init__(self, ws, gs, vs=None, weight_decay=True):
        k = len(ws)
        for t in list(ws) + list(gs) + [v for v in (vs or []) if v is not None]:
            _dev(t, torch.float32, "parameter tensors")
        self.tmps = [torch.empty_like(w) for w in ws] if weight_decay else [None] * k
        self.keep = (list(ws), list(gs), list(vs) if vs is not None else None)      # the table holds raw pointers
        self.table = (_SgdTensor * k)(*[
            _SgdTensor(_p(ws[t]), _p(gs[t]), _p(vs[t]) if vs is not None else None, _p(self.tmps[t]), ws[t].numel())
            for t in range(k)])
        self.count = k
        nbytes = int(lib().fxp_sgd16_multi_workspace_bytes(self.table, k))
        self.ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=ws[0].device)


def sgd16_step_multi(buf, lr, momentum=0.0, weight_decay=0.0, seed=0, step=0, rounding=STOCHASTIC):
    """In-place SGD step on every tensor of buf (own scales per tensor), a handful of launches in all."""
    _check(lib().fxp_sgd16_step_multi(buf.table, buf.count, float(lr), float(momentum), float(weight_decay), seed, step,
                                      rounding, _p(buf.ws), buf.ws.numel(), _stream()), "fxp_sgd16_step_multi")
