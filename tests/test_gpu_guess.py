"""The layer calls that take the previous scales as guesses (fxp_linear_fwd_guess / fxp_linear_bwd_guess): bit for
bit the outputs of the oracle whatever the scale words hold on entry - the right scale (a hit: one pass over the
tensor), a scale too small or too large (a miss: the verifying launch maps again), zero, negative or huge
garbage, the scale 255 of a non-finite tensor - and for every mix of hit and miss between the two tensors of a
forward call."""
import numpy as np
import pytest

import oracle
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


def check_step(fxp, buf, X, W, dY, seed, step, what):
    Y = host(fxp.linear_fwd(dev(X), dev(W), buf, seed, step, guess=True))
    dX, dW = fxp.linear_bwd(dev(dY), buf, seed, step, guess=True)
    dX, dW = host(dX), host(dW)
    Yo, saved = oracle.linear_fwd(X, W, seed=seed, step=step)
    dXo, dWo, aux = oracle.linear_bwd(dY, saved, seed=seed, step=step)
    assert host(buf.e).tolist() == [saved["eX"], saved["eW"], aux["eG"]], what
    for got, want, nm in ((buf.Xq, saved["Xq"], "Xq"), (buf.Wq, saved["Wq"], "Wq"), (buf.dYq, aux["dYq"], "dYq")):
        assert np.array_equal(host(got), want), (what, nm)
    for got, want, nm in ((buf.XqT, saved["Xq"], "XqT"), (buf.WqT, saved["Wq"], "WqT"), (buf.dYqT, aux["dYq"], "dYqT")):
        assert np.array_equal(host(got).T, want), (what, nm)
    for got, want, nm in ((Y, Yo, "Y"), (dX, dXo, "dX"), (dW, dWo, "dW")):
        assert same_bits(got, want), (what, nm)


@pytest.mark.parametrize("M,K,N", [(4224, 1024, 1044), (2180, 2052, 2048)], ids=["activation-and-gradient-large", "all-three-large"])
def test_guessed_scales_every_case(fxp, M, K, N):
    """(4224, 1024, 1044): X and dY are above the size where the guess is used (2^22 elements), the smaller W rides
    in X's launch; ragged tiles.  (2180, 2052, 2048): all three tensors above it."""
    rng = np.random.default_rng(M)
    X = rng.standard_normal((M, K)).astype(np.float32)
    W = (rng.standard_normal((K, N)) * 0.05).astype(np.float32)
    dY = rng.laplace(0, 1e-3, (M, N)).astype(np.float32)
    buf = fxp.LayerBuffers(M, K, N)
    say("guess: first call, scale words zero", (M, K, N))
    check_step(fxp, buf, X, W, dY, 7, 0, "first call")
    say("guess: hit")
    check_step(fxp, buf, X, W, dY, 7, 1, "hit")
    say("guess: tensors grow (guess too small) / shrink (guess too large)")
    check_step(fxp, buf, X * 64, W, dY * 0.001, 7, 2, "X up, dY down")
    if K != 1024:
        return                                   # the second shape: first call, hit and miss only
    check_step(fxp, buf, X * 64, W * 8, dY * 0.001, 7, 3, "X hit, W up, dY hit")
    check_step(fxp, buf, X, W * 8, dY, 7, 4, "X down, W hit, dY up")
    say("guess: garbage in the scale words")
    for junk in ([0, -5, 100000], [255, 1, 254], [-2**31, 2**31 - 1, 256]):
        buf.e.copy_(torch.tensor(junk, dtype=torch.int64).to(torch.int32))
        check_step(fxp, buf, X, W, dY, 9, 5, junk)
    say("guess: a non-finite element (scale 255) and back")
    Xbad = X.copy()
    Xbad[M // 2, 3] = np.inf
    Xbad[5, K - 1] = np.nan
    check_step(fxp, buf, Xbad, W, dY, 9, 6, "Inf / NaN in X")
    check_step(fxp, buf, Xbad, W, dY, 9, 7, "Inf / NaN in X, guess 255 is a hit")
    check_step(fxp, buf, X, W, dY, 9, 8, "finite again")
    say("guess: an all-zero gradient (scale 1)")
    check_step(fxp, buf, X, W, np.zeros_like(dY), 9, 9, "zero dY")
    check_step(fxp, buf, X, W, np.zeros_like(dY), 9, 10, "zero dY, hit")


def test_guessed_scales_small_layer_takes_the_two_pass_path(fxp):
    rng = np.random.default_rng(3)
    X = rng.standard_normal((300, 200)).astype(np.float32)
    W = rng.standard_normal((200, 100)).astype(np.float32)
    dY = rng.standard_normal((300, 100)).astype(np.float32)
    buf = fxp.LayerBuffers(300, 200, 100)
    for step in range(2):
        check_step(fxp, buf, X, W, dY, 1, step, "small")


def test_guessed_scales_batched_products(fxp):
    """fxp_bmm_fwd_guess / _bwd_guess on attention-shaped products large enough for the guess to be used: scores
    (A and Bm of equal tile width: one pair of launches) and context (P 208 wide, V 64 wide: different tile widths,
    each tensor guesses by itself); first call, hit, and a miss in every tensor."""
    rng = np.random.default_rng(5)
    batch, S, d = 340, 208, 64                                   # 340 * 208 * 64 = 4.5 M elements per Q / K / V
    Q = rng.standard_normal((batch, S, d)).astype(np.float32)
    Kt = rng.standard_normal((batch, S, d)).astype(np.float32)
    dS = (rng.standard_normal((batch, S, S)) * 1e-3).astype(np.float32)
    P = np.abs(rng.standard_normal((batch, S, S))).astype(np.float32)
    V = rng.standard_normal((batch, S, d)).astype(np.float32)
    dO = (rng.standard_normal((batch, S, d)) * 1e-3).astype(np.float32)
    for name, A, Bm, dY, transB in (("scores", Q, Kt, dS, True), ("context", P, V, dO, False)):
        M, K = A.shape[1:]
        N = dY.shape[2]
        buf = fxp.BmmBuffers(batch, M, K, N, transB)
        for step, (fa, fb, fg) in enumerate([(1, 1, 1), (1, 1, 1), (32, 1, 1 / 64), (32, 1 / 16, 1 / 64), (1, 1, 1)]):
            say("bmm guess", name, step, (fa, fb, fg))
            a, b, g = A * np.float32(fa), Bm * np.float32(fb), dY * np.float32(fg)
            Y = host(fxp.bmm_fwd(dev(a), dev(b), buf, 2, step, guess=True))
            dA, dB = fxp.bmm_bwd(dev(g), buf, 2, step, guess=True)
            Yo, sv = oracle.bmm_fwd(a, b, transB, 2, step)
            dAo, dBo, aux = oracle.bmm_bwd(g, sv, 2, step)
            assert host(buf.e).tolist() == [sv["eA"], sv["eB"], aux["eG"]], (name, step)
            assert np.array_equal(host(buf.Aq), sv["Aq"]) and np.array_equal(host(buf.Bq), sv["Bq"]), (name, step)
            assert np.array_equal(host(buf.AqT), sv["Aq"].reshape(batch * M, K).T), (name, step)
            assert np.array_equal(host(buf.dYq), aux["dYq"]), (name, step)
            assert same_bits(Y, Yo) and same_bits(host(dA), dAo) and same_bits(host(dB), dBo), (name, step)
