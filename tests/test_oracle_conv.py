"""Pins for the oracle's integer convolution (Sec. 3.4: convolution layers are the same integer
inner products as linear layers).  Channels-last tensors."""
import numpy as np
import pytest

import oracle


def rand_i8(rng, shape, lo=-127, hi=127):
    return rng.integers(lo, hi + 1, size=shape, dtype=np.int64).astype(np.int8)


def im2col_numpy(Xq, KH, KW, stride, pad):
    """Independent construction: zero-pad, gather windows with stride tricks -> [N*Ho*Wo, KH*KW*C] int64."""
    N, H, W, C = Xq.shape
    P = np.zeros((N, H + 2 * pad, W + 2 * pad, C), dtype=np.int64)
    P[:, pad:pad + H, pad:pad + W, :] = Xq
    Ho, Wo = (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1
    s = P.strides
    win = np.lib.stride_tricks.as_strided(P, shape=(N, Ho, Wo, KH, KW, C),
                                          strides=(s[0], s[1] * stride, s[2] * stride, s[1], s[2], s[3]), writeable=False)
    return np.ascontiguousarray(win).reshape(N * Ho * Wo, KH * KW * C), (N, Ho, Wo)


CASES = [  # N, H, W, C, Cout, KH, KW, stride, pad
    (2, 5, 6, 3, 4, 3, 3, 1, 1), (1, 7, 7, 2, 3, 3, 3, 2, 1), (2, 4, 4, 5, 2, 1, 1, 1, 0), (1, 8, 6, 3, 2, 3, 2, 2, 0),
    (2, 6, 6, 4, 3, 5, 5, 1, 2), (1, 9, 9, 1, 1, 3, 3, 3, 1)]


@pytest.mark.parametrize("N,H,W,C,Cout,KH,KW,stride,pad", CASES)
def test_forward_against_numpy_im2col_matmul(N, H, W, C, Cout, KH, KW, stride, pad):
    rng = np.random.default_rng(N * 100 + H)
    Xq, Wq = rand_i8(rng, (N, H, W, C)), rand_i8(rng, (Cout, KH, KW, C))
    col, (n, ho, wo) = im2col_numpy(Xq, KH, KW, stride, pad)
    want = (col @ Wq.reshape(Cout, -1).astype(np.int64).T).reshape(n, ho, wo, Cout)
    got = oracle.conv2d_fwd_acc(Xq, Wq, stride, pad)
    assert got.shape == want.shape and np.array_equal(got, want)


@pytest.mark.parametrize("N,H,W,C,Cout,KH,KW,stride,pad", CASES)
def test_gradients_are_the_exact_adjoints(N, H, W, C, Cout, KH, KW, stride, pad):
    """<conv(X, W), G> = <X, bwd_input(G, W)> = <W, bwd_weight(X, G)> exactly, in integers: pins both
    backward formulas (index pattern, stride and padding handling) to the forward definition."""
    rng = np.random.default_rng(7 + H * W)
    Xq, Wq = rand_i8(rng, (N, H, W, C), -9, 9), rand_i8(rng, (Cout, KH, KW, C), -9, 9)
    Y = oracle.conv2d_fwd_acc(Xq, Wq, stride, pad).astype(np.int64)
    Gq = rand_i8(rng, Y.shape, -9, 9)
    lhs = int((Y * Gq).sum())
    dX = oracle.conv2d_bwd_input_acc(Gq, Wq, Xq.shape, stride, pad).astype(np.int64)
    dW = oracle.conv2d_bwd_weight_acc(Xq, Gq, Wq.shape, stride, pad).astype(np.int64)
    assert int((dX * Xq).sum()) == lhs
    assert int((dW * Wq).sum()) == lhs
    # and element-wise against numpy: dW = col^T G
    col, _ = im2col_numpy(Xq, KH, KW, stride, pad)
    assert np.array_equal(dW.reshape(Cout, -1), Gq.reshape(-1, Cout).astype(np.int64).T @ col)


def col2im_numpy(dcol, x_shape, KH, KW, stride, pad):
    """Independent scatter: patch-gradient rows [N*Ho*Wo, KH*KW*C] added back onto the zero-padded image, one
    filter tap at a time with strided slices; the padding rim is cut off at the end."""
    N, H, W, C = x_shape
    Ho, Wo = (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1
    P = np.zeros((N, H + 2 * pad, W + 2 * pad, C), dtype=np.int64)
    d = dcol.reshape(N, Ho, Wo, KH, KW, C)
    for kh in range(KH):
        for kw in range(KW):
            P[:, kh:kh + stride * Ho:stride, kw:kw + stride * Wo:stride, :] += d[:, :, :, kh, kw, :]
    return P[:, pad:pad + H, pad:pad + W, :]


@pytest.mark.parametrize("N,H,W,C,Cout,KH,KW,stride,pad", CASES)
def test_input_gradient_element_by_element(N, H, W, C, Cout, KH, KW, stride, pad):
    """dX against a numpy construction that shares nothing with the oracle's loops: the patch gradient
    G[M, Cout] . W[Cout, KH*KW*C] by matmul, scattered back by col2im; and, for every input element of the
    smallest cases, against the definition dX[x] = d<conv(X, W), G>/dX[x] taken with a unit impulse."""
    rng = np.random.default_rng(11 + N + 3 * H + 5 * KH)
    Wq = rand_i8(rng, (Cout, KH, KW, C))
    Ho, Wo = (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1
    Gq = rand_i8(rng, (N, Ho, Wo, Cout))
    got = oracle.conv2d_bwd_input_acc(Gq, Wq, (N, H, W, C), stride, pad).astype(np.int64)
    dcol = Gq.reshape(-1, Cout).astype(np.int64) @ Wq.reshape(Cout, -1).astype(np.int64)
    want = col2im_numpy(dcol, (N, H, W, C), KH, KW, stride, pad)
    assert got.shape == want.shape and np.array_equal(got, want)
    if N * H * W * C <= 200:
        for idx in np.ndindex(N, H, W, C):
            impulse = np.zeros((N, H, W, C), np.int8)
            impulse[idx] = 1
            y = oracle.conv2d_fwd_acc(impulse, Wq, stride, pad).astype(np.int64)
            assert int((y * Gq).sum()) == got[idx], idx


def test_special_kernels():
    rng = np.random.default_rng(3)
    Xq = rand_i8(rng, (2, 5, 5, 3))
    # 1x1 convolution is a linear layer over the channel axis
    Wq = rand_i8(rng, (4, 1, 1, 3))
    assert np.array_equal(oracle.conv2d_fwd_acc(Xq, Wq).reshape(-1, 4),
                          oracle.gemm(Xq.reshape(-1, 3), Wq.reshape(4, 3), transB=True))
    # a centred delta kernel copies the input channel; an off-centre one shifts it (zero padding at the rim)
    Wd = np.zeros((3, 3, 3, 3), np.int8)
    for c in range(3):
        Wd[c, 1, 1, c] = 1
    assert np.array_equal(oracle.conv2d_fwd_acc(Xq, Wd, 1, 1), Xq.astype(np.int32))
    Ws = np.zeros((1, 3, 3, 3), np.int8)
    Ws[0, 0, 1, 2] = 1                       # reads the pixel one row up, channel 2
    out = oracle.conv2d_fwd_acc(Xq, Ws, 1, 1)[..., 0]
    assert np.array_equal(out[:, 1:, :], Xq[:, :-1, :, 2]) and np.all(out[:, 0, :] == 0)


def test_layer_equals_the_primitives_chained():
    rng = np.random.default_rng(5)
    X = rng.standard_normal((2, 6, 6, 4)).astype(np.float32)
    Wt = (rng.standard_normal((3, 3, 3, 4)) * 0.1).astype(np.float32)
    seed, step = 12, 3
    Y, sv = oracle.conv2d_fwd(X, Wt, 1, 1, seed, step)
    eX, eW = oracle.scale(X), oracle.scale(Wt)
    Xq = oracle.map(X.reshape(-1, 4), eX, seed=seed, stream_id=(step << 8) | 0).reshape(X.shape)
    Wq = oracle.map(Wt.reshape(3, -1), eW, seed=seed, stream_id=(step << 8) | 1).reshape(Wt.shape)
    assert (sv["eX"], sv["eW"]) == (eX, eW) and np.array_equal(sv["Xq"], Xq) and np.array_equal(sv["Wq"], Wq)
    assert np.array_equal(Y, oracle.unmap(oracle.conv2d_fwd_acc(Xq, Wq, 1, 1), eX, eW))
    dY = rng.laplace(0, 1e-3, Y.shape).astype(np.float32)
    dX, dW, aux = oracle.conv2d_bwd(dY, sv, seed, step)
    eG = oracle.scale(dY)
    Gq = oracle.map(dY.reshape(-1, 3), eG, seed=seed, stream_id=(step << 8) | 2).reshape(dY.shape)
    assert aux["eG"] == eG and np.array_equal(aux["dYq"], Gq)
    assert np.array_equal(dX, oracle.unmap(oracle.conv2d_bwd_input_acc(Gq, Wq, X.shape, 1, 1), eG, eW))
    assert np.array_equal(dW, oracle.unmap(oracle.conv2d_bwd_weight_acc(Xq, Gq, Wt.shape, 1, 1), eX, eG))
    # unbiased: mean over seeds of the integer layer output approaches the fp64 convolution
    col, shp = im2col_numpy(np.zeros((2, 6, 6, 4), np.int8), 3, 3, 1, 1)
    Ys = np.mean([oracle.conv2d_fwd(X, Wt, 1, 1, 100 + s, s)[0].astype(np.float64) for s in range(300)], axis=0)
    Pf = np.zeros((2, 8, 8, 4)); Pf[:, 1:7, 1:7, :] = X
    ref = np.zeros_like(Ys)
    for kh in range(3):
        for kw in range(3):
            ref += np.einsum("nhwc,oc->nhwo", Pf[:, kh:kh + 6, kw:kw + 6, :], Wt[:, kh, kw, :].astype(np.float64))
    assert np.abs(Ys - ref).max() < 0.02 * np.abs(ref).max()
