"""GPU parity on seeded random cases, for as long as a time budget allows: linear layers (two-pass and with scale
guesses, whatever the scale words hold and then the right ones), convolutions, batched product layers and the four
operand forms of the bare product, every output bit for bit against the oracle.  Shapes, widths, roundings, value
distributions (normal, tiny Laplace, 60 decades of magnitude, per-element binades, planted Inf / NaN, 70 % zeros)
are drawn from one seeded stream, so the k-th case is always the same; FXP_SWEEP_SECONDS (default 20) sets how many
run, FXP_SWEEP_LARGE=1 draws sizes from the upper seven eighths of the range instead of log-uniformly."""
import os
import time

import numpy as np
import pytest

import oracle
from tests.gpu_util import dev, host, same_bits, say
from tests.test_gpu_bmm import check_bmm
from tests.test_gpu_conv import check_conv
from tests.test_gpu_parity import layer_check_full, rand_i8

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def fxp():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: there is no CPU path in libfxp")
    from paper_2207_08822_amd import fxp as binding
    binding.lib()
    return binding


class Draw:
    def __init__(self, seed, large):
        self.rng = np.random.default_rng(seed)
        self.large = large

    def dim(self, hi):
        rng = self.rng
        v = int(rng.uniform(hi / 8, hi)) if self.large else int(np.exp(rng.uniform(0, np.log(hi))))
        r = rng.integers(0, 4)
        if r == 0:
            v = max(16, v // 16 * 16)        # the direct-to-LDS loaders
        elif r == 1:
            v = max(128, v // 128 * 128)     # whole K steps and tiles
        return max(1, v)

    def tensor(self, shape, kind):
        rng = self.rng
        n = int(np.prod(shape))
        if kind == 0:
            x = rng.standard_normal(shape)
        elif kind == 1:
            x = rng.laplace(0, 1e-4, shape)
        elif kind == 2:
            x = rng.standard_normal(shape) * 10.0 ** rng.uniform(-30, 30)
        else:
            x = rng.standard_normal(shape) * np.exp2(rng.integers(-40, 40, shape))
        x = x.astype(np.float32)
        if rng.integers(0, 6) == 0 and n > 3:
            x.reshape(-1)[rng.integers(0, n, 3)] = np.array([np.inf, -np.inf, np.nan], np.float32)[rng.integers(0, 3, 3)]
        if rng.integers(0, 6) == 0:
            x = np.where(rng.random(shape) < 0.3, x, np.float32(0)).astype(np.float32)
        return x


def guessed_layer(fxp, d, X, W, dY, seed, rounding, bits):
    M, K = X.shape
    N = W.shape[1]
    buf = fxp.LayerBuffers(M, K, N)
    Yo, saved = oracle.linear_fwd(X, W, seed, 3, rounding, bits)
    dXo, dWo, aux = oracle.linear_bwd(dY, saved, seed, 3, rounding, bits)
    for rep in range(2):
        if rep == 0:      # anything may stand in the scale words before the first call
            buf.e.copy_(torch.from_numpy(d.rng.integers(-5, 300, 3).astype(np.int32)))
        Y = fxp.linear_fwd(dev(X), dev(W), buf, seed, 3, rounding, bits, guess=True)
        dX, dW = fxp.linear_bwd(dev(dY), buf, seed, 3, rounding, bits, guess=True)
        assert host(buf.e).tolist() == [saved["eX"], saved["eW"], aux["eG"]]
        assert np.array_equal(host(buf.Xq), saved["Xq"]) and np.array_equal(host(buf.XqT), saved["Xq"].T)
        assert np.array_equal(host(buf.Wq), saved["Wq"]) and np.array_equal(host(buf.WqT), saved["Wq"].T)
        assert np.array_equal(host(buf.dYq), aux["dYq"]) and np.array_equal(host(buf.dYqT), aux["dYq"].T)
        assert same_bits(host(Y), Yo) and same_bits(host(dX), dXo) and same_bits(host(dW), dWo)


def test_random_cases_until_the_time_budget_is_spent(fxp):
    budget = float(os.environ.get("FXP_SWEEP_SECONDS", "20"))
    d = Draw(20220718, os.environ.get("FXP_SWEEP_LARGE", "0") == "1")
    rng = d.rng
    t_end = time.time() + budget
    it = 0
    counts = dict(layer=0, guess=0, conv=0, bmm=0, gemm=0)
    while time.time() < t_end:
        it += 1
        which = it % 5
        bits = int(rng.choice([8, 8, 8, 7, 5, 3, 2]))
        rounding = int(rng.integers(0, 2))
        if which in (0, 1):
            M, K, N = d.dim(3000), d.dim(3000), d.dim(3000)
            while M * K * N > 2.5e9:
                M, K, N = d.dim(3000), d.dim(3000), d.dim(3000)
            kinds = rng.integers(0, 4, 3)
            X, W, dY = d.tensor((M, K), kinds[0]), d.tensor((K, N), kinds[1]), d.tensor((M, N), kinds[2])
            say("sweep layer", it, (M, K, N), "bits", bits, "rounding", rounding, "kinds", kinds.tolist(), "guess", which == 1)
            if which == 0:
                layer_check_full(fxp, X, W, dY, seed=it, step=it % 7, rounding=rounding, bits=bits)
                counts["layer"] += 1
            else:
                guessed_layer(fxp, d, X, W, dY, it, rounding, bits)
                counts["guess"] += 1
        elif which == 2:
            N_, H, W_ = int(rng.integers(1, 5)), int(rng.integers(3, 30)), int(rng.integers(3, 30))
            C = int(rng.choice([1, 3, 8, 20, 64, 128, 192, 256, 100]))
            Cout = int(rng.choice([1, 6, 16, 64, 128, 256, 40]))
            KH, KW = int(rng.integers(1, 6)), int(rng.integers(1, 6))
            stride, pad = int(rng.integers(1, 4)), int(rng.integers(0, 3))
            if H + 2 * pad < KH or W_ + 2 * pad < KW:
                continue
            say("sweep conv", it, (N_, H, W_, C, Cout, KH, KW, stride, pad), "bits", bits, "rounding", rounding)
            X = np.maximum(d.tensor((N_, H, W_, C), 0), 0).astype(np.float32)
            Wt = (d.tensor((Cout, KH, KW, C), 0) * 0.1).astype(np.float32)
            Ho, Wo = oracle.conv_out_hw(H, W_, KH, KW, stride, pad)
            dY = d.tensor((N_, Ho, Wo, Cout), 1)
            check_conv(fxp, X, Wt, dY, stride, pad, seed=it, step=it % 3, rounding=rounding, bits=bits)
            counts["conv"] += 1
        elif which == 3:
            b, M, K, N = int(rng.integers(1, 20)), d.dim(300), d.dim(300), d.dim(300)
            transB = bool(rng.integers(0, 2))
            say("sweep bmm", it, (b, M, K, N), "transB", transB, "bits", bits, "rounding", rounding)
            A, Bm = d.tensor((b, M, K), 0), d.tensor((b, N, K) if transB else (b, K, N), 0)
            dY = d.tensor((b, M, N), 1)
            check_bmm(fxp, A, Bm, dY, transB, seed=it, step=2, rounding=rounding, bits=bits)
            counts["bmm"] += 1
        else:
            M, N, K = d.dim(2500), d.dim(2500), d.dim(6000)
            while M * K * N > 4e9:
                M, N, K = d.dim(2500), d.dim(2500), d.dim(6000)
            A, B = rand_i8(rng, (M, K)), rand_i8(rng, (K, N))
            want = oracle.gemm(A, np.ascontiguousarray(B.T), transB=True)
            AT, BT = np.ascontiguousarray(A.T), np.ascontiguousarray(B.T)
            for tA, tB, a, b_ in [(False, True, A, BT), (False, False, A, B), (True, False, AT, B), (True, True, AT, BT)]:
                say("sweep gemm", it, (M, N, K), "transA", tA, "transB", tB)
                assert np.array_equal(host(fxp.gemm(dev(a), dev(b_), transA=tA, transB=tB)), want)
            counts["gemm"] += 1
    say("sweep done", counts)
    assert sum(counts.values()) > 0
