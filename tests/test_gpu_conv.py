"""GPU parity of the convolution layer (channels-last) against the CPU oracle: scales, every int8
tensor and all three fp32 outputs bit for bit."""
import numpy as np
import pytest

import oracle
from paper_2207_08822_amd import synth
from tests.gpu_util import dev, host, same_bits, say

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def fxp():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: there is no CPU path in libfxp")
    from paper_2207_08822_amd import fxp as binding
    binding.lib()
    return binding


def check_conv(fxp, X, Wt, dY, stride, pad, seed=3, step=1, rounding=0, bits=8, need_dX=True, need_dW=True):
    N, H, W, C = X.shape
    Cout, KH, KW, _ = Wt.shape
    buf = fxp.ConvBuffers(N, H, W, C, Cout, KH, KW, stride, pad)
    Y = host(fxp.conv2d_fwd(dev(X), dev(Wt), buf, seed, step, rounding, bits))
    Yo, sv = oracle.conv2d_fwd(X, Wt, stride, pad, seed, step, rounding, bits)
    assert host(buf.e)[:2].tolist() == [sv["eX"], sv["eW"]]
    assert np.array_equal(host(buf.Xq), sv["Xq"])
    assert np.array_equal(host(buf.Wq), sv["Wq"].reshape(Cout, -1))
    assert np.array_equal(host(buf.WqT), sv["Wq"].reshape(Cout, -1).T)
    assert same_bits(Y, Yo)
    dX, dW = fxp.conv2d_bwd(dev(dY), buf, seed, step, rounding, bits, need_dX, need_dW)
    dXo, dWo, aux = oracle.conv2d_bwd(dY, sv, seed, step, rounding, bits, need_dX, need_dW)
    assert int(host(buf.e)[2]) == aux["eG"]
    assert np.array_equal(host(buf.dYq), aux["dYq"].reshape(-1, Cout))
    if need_dX:
        assert same_bits(host(dX), dXo)
    if need_dW:
        assert same_bits(host(dW), dWo)


CASES = [  # N, H, W, C, Cout, KH, KW, stride, pad
    (2, 8, 8, 16, 16, 3, 3, 1, 1), (1, 7, 9, 3, 5, 3, 3, 2, 1), (2, 6, 6, 32, 8, 1, 1, 1, 0), (1, 12, 10, 4, 6, 3, 2, 2, 0),
    (2, 9, 9, 20, 12, 5, 5, 1, 2), (3, 14, 14, 64, 48, 3, 3, 1, 1), (2, 16, 16, 16, 64, 3, 3, 2, 1), (1, 5, 5, 1, 1, 3, 3, 3, 1),
    # channels a multiple of 128: the GEMM loader reads the patches straight from the int8 image (forward; input
    # gradient too when Cout is a multiple of 128 and the stride is 1); ragged pixel counts, paddings 0..2, strides
    (2, 9, 11, 128, 40, 3, 3, 1, 1), (1, 10, 10, 256, 128, 3, 2, 2, 0), (2, 7, 7, 128, 128, 5, 5, 1, 2),
    (3, 6, 6, 128, 16, 1, 1, 1, 0), (2, 13, 9, 128, 256, 3, 3, 1, 0), (1, 20, 20, 128, 128, 3, 3, 1, 1),
    # 64 and 192 channels: the 64-byte K step
    (2, 12, 12, 64, 64, 3, 3, 1, 1), (1, 9, 7, 192, 64, 3, 3, 2, 1), (2, 8, 8, 64, 192, 5, 3, 1, 0)]


@pytest.mark.parametrize("N,H,W,C,Cout,KH,KW,stride,pad", CASES)
def test_conv_shapes(fxp, N, H, W, C, Cout, KH, KW, stride, pad):
    say("conv", (N, H, W, C, Cout, KH, KW, stride, pad))
    rng = np.random.default_rng(N * 1000 + H * 10 + C)
    X = np.maximum(rng.standard_normal((N, H, W, C)), 0).astype(np.float32)
    Wt = (rng.standard_normal((Cout, KH, KW, C)) * 0.1).astype(np.float32)
    Ho, Wo = oracle.conv_out_hw(H, W, KH, KW, stride, pad)
    dY = rng.laplace(0, 1e-3, (N, Ho, Wo, Cout)).astype(np.float32)
    check_conv(fxp, X, Wt, dY, stride, pad)


def test_conv_modes_and_partial_gradients(fxp):
    rng = np.random.default_rng(9)
    X = rng.standard_normal((2, 10, 10, 32)).astype(np.float32)
    Wt = (rng.standard_normal((16, 3, 3, 32)) * 0.05).astype(np.float32)
    dY = rng.standard_normal((2, 10, 10, 16)).astype(np.float32) * 1e-4
    say("conv nearest, 5 bits")
    check_conv(fxp, X, Wt, dY, 1, 1, rounding=1, bits=5)
    say("conv dW only")
    check_conv(fxp, X, Wt, dY, 1, 1, need_dX=False)
    say("conv dX only")
    check_conv(fxp, X, Wt, dY, 1, 1, need_dW=False)
    # 128 channels in and out: patches read by the GEMM loader, in the forward pass and in the input gradient
    X = np.maximum(rng.standard_normal((2, 9, 9, 128)), 0).astype(np.float32)
    Wt = (rng.standard_normal((128, 3, 3, 128)) * 0.03).astype(np.float32)
    dY = rng.standard_normal((2, 9, 9, 128)).astype(np.float32) * 1e-4
    say("conv 128 channels, dX only / dW only / nearest 4 bits")
    check_conv(fxp, X, Wt, dY, 1, 1, need_dW=False)
    check_conv(fxp, X, Wt, dY, 1, 1, need_dX=False)
    check_conv(fxp, X, Wt, dY, 1, 1, rounding=1, bits=4)


def test_conv_c2_layer_reduced_and_full(fxp):
    say("conv c2 geometry, batch 4 (full oracle)")
    X, Wt, dY, g = synth.conv_tensors(N=4)
    check_conv(fxp, X, Wt, dY, g["stride"], g["pad"], seed=0, step=0)
    say("conv c2 geometry, batch 32 (full oracle, ~22 G integer MACs)")
    X, Wt, dY, g = synth.conv_tensors()
    check_conv(fxp, X, Wt, dY, g["stride"], g["pad"], seed=0, step=0)


def test_conv_random_geometries(fxp):
    """Seeded random geometries: channel counts on and off the implicit path, kernels 1..5, strides 1..2, paddings
    0..2, non-square images."""
    rng = np.random.default_rng(77)
    done = 0
    while done < 14:
        N, H, W = int(rng.integers(1, 4)), int(rng.integers(3, 15)), int(rng.integers(3, 15))
        C = int(rng.choice([3, 8, 20, 64, 128, 192]))
        Cout = int(rng.choice([1, 6, 16, 64, 128]))
        KH, KW = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        stride, pad = int(rng.integers(1, 3)), int(rng.integers(0, 3))
        if H + 2 * pad < KH or W + 2 * pad < KW:
            continue
        say("conv random", (N, H, W, C, Cout, KH, KW, stride, pad))
        X = np.maximum(rng.standard_normal((N, H, W, C)), 0).astype(np.float32)
        Wt = (rng.standard_normal((Cout, KH, KW, C)) * 0.1).astype(np.float32)
        Ho, Wo = oracle.conv_out_hw(H, W, KH, KW, stride, pad)
        dY = rng.laplace(0, 1e-3, (N, Ho, Wo, Cout)).astype(np.float32)
        check_conv(fxp, X, Wt, dY, stride, pad, seed=done, step=done % 3)
        done += 1


def test_conv_weight_gradient_over_more_pixels_than_one_int32_sum_holds(fxp):
    """3 x 212 x 212 = 134 832 output pixels: the weight gradient sums over all of them (int32 slices added in 64
    bits); channel 0 of X and of dY is at the top code everywhere, so those sums pass 2^31."""
    rng = np.random.default_rng(77)
    N, H, W, C, Cout = 3, 212, 212, 4, 8
    X = np.maximum(rng.standard_normal((N, H, W, C)), 0).astype(np.float32).clip(0, 3.9)
    Wt = (rng.standard_normal((Cout, 3, 3, C)) * 0.1).astype(np.float32)
    dY = rng.uniform(-1e-3, 1e-3, (N, H, W, Cout)).astype(np.float32)
    X[..., 0], dY[..., 0] = 127 / 32, 127 * 2.0 ** -16         # top code at every pixel (units 2^-5 and 2^-16)
    say("conv with", N * H * W, "output pixels")
    check_conv(fxp, X, Wt, dY, 1, 1)
