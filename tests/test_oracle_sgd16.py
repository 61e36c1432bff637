"""Checks of the oracle's int16 weight update (Remark 5, App. A.4).  The paper fixes only
w_hat + alpha_hat * g_hat with stochastic rounding and its unbiasedness; the alignment and the place of the
rounding are this build's reading ("parity unpinned").  What is fixed is tested here: the operands are the
16-bit instance of the map, representable operands give the exact real result, the update is an unbiased
estimator of x + a y, and the whole step stays within a few int16 units of the floating-point optimiser."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from tests import pymodel as pm


def tensors(seed, n=96):
    rng = np.random.default_rng(seed)
    w = (rng.standard_normal(n) * 0.05).astype(np.float32)
    g = rng.laplace(0, 2e-3, n).astype(np.float32)
    v = rng.laplace(0, 1e-2, n).astype(np.float32)
    return w, g, v


def test_map16_is_the_16_bit_instance_of_the_map():
    """15 magnitude bits, the low 9 bits of the 24-bit mantissa decide the rounding: against the exact rational
    model of the format."""
    w, _, _ = tensors(1, 200)
    e = oracle.scale(w)
    q = oracle.map16(w, e, seed=7, stream_id=(2 << 8) | 3)
    for i in range(w.size):
        assert int(q[i]) == pm.map_one(float(w[i]), e, 7, (2 << 8) | 3, i, bits=16)
    assert np.abs(q.astype(np.int32)).max() >= 1 << 14        # the largest element fills the top bit
    # 15 magnitude bits reproduce the tensor to 2^-15 of its largest binade
    assert np.max(np.abs(q * 2.0 ** (e - 127 - 14) - w.astype(np.float64))) <= 2.0 ** (e - 127 - 14)


def model_map16(x, e_max, r9):
    """Exact-rational 16-bit map of a finite float with the 9-bit random number r9."""
    fl, low, cut = pm.floor_and_prob(x, e_max, 16)
    assert cut == 9
    q = min(fl + (1 if r9 < low else 0), 32767)
    return -q if (pm.f32_bits(x) >> 31) else q


def model_axpy(x, y, a, seed, step):
    """Exact-rational model of z = x_hat + SR(a_hat y_hat) from the definition of the format."""
    ex, ey, ea = oracle.scale(x), oracle.scale(y), oracle.scale(np.float32([a]))
    Ex, Ey, Ea = (pm.lsb_exponent(e, 16) for e in (ex, ey, ea))
    a_hat = model_map16(float(np.float32(a)), ea, pm.random_word(seed, (step << 8) | 5, 0) >> 23)
    out = np.empty(x.size, dtype=np.uint32)
    for i in range(x.size):
        word = pm.random_word(seed, (step << 8) | 3, i)          # one word, two 9-bit fields
        x_hat = model_map16(float(x[i]), ex, word >> 23)
        y_hat = model_map16(float(y[i]), ey, (word >> 14) & 511)
        t = Fraction(a_hat * y_hat) * pm.pow2(Ea + Ey) / pm.pow2(Ex)       # update in units of x_hat
        mag = abs(t)
        fl = mag.numerator // mag.denominator
        thr = ((mag - fl) * (1 << 32)).numerator // ((mag - fl) * (1 << 32)).denominator
        u = fl + (1 if pm.random_word(seed, (step << 8) | 4, i) < thr else 0)
        u = min(u, (1 << 23) - (1 << 15))
        r = x_hat + (-u if t < 0 else u)
        out[i] = pm.round_to_f32(Fraction(r) * pm.pow2(Ex))
    return out.view(np.float32), (ex, ey, ea)


@pytest.mark.parametrize("a", [-0.1, 0.9, 5e-4, -3.0e-6, 1024.0])
def test_axpy16_against_the_exact_rational_model(a):
    w, g, _ = tensors(3)
    z, e = oracle.axpy16(w, g, a, seed=11, step=5)
    zm, em = model_axpy(w, g, a, 11, 5)
    assert e == em
    assert np.array_equal(z.view(np.uint32), zm.view(np.uint32))


def test_representable_operands_give_the_exact_result():
    """int16-representable x, y and a power-of-two a with the product on x's grid: no rounding anywhere."""
    rng = np.random.default_rng(5)
    x = rng.integers(-2000, 2001, 64).astype(np.float32) * 2.0 ** -10
    y = rng.integers(-300, 301, 64).astype(np.float32) * 2.0 ** -6
    x[0], y[0] = 2000 * 2.0 ** -10, 300 * 2.0 ** -6
    for a in (0.5, -2.0, 0.0):
        z, _ = oracle.axpy16(x, y, a, seed=1, step=0)
        assert np.array_equal(z.astype(np.float64), x.astype(np.float64) + a * y.astype(np.float64))
    # and finer products (a = 2^-12 puts them 6 bits below x's grid) are rounded to a neighbouring grid point
    z, (ex, _, _) = oracle.axpy16(x, y, 2.0 ** -12, seed=1, step=0)
    exact = x.astype(np.float64) + 2.0 ** -12 * y.astype(np.float64)
    unit = 2.0 ** (ex - 127 - 14)
    assert np.all(np.abs(z - exact) < unit) and np.all(np.rint(z / unit) == z / unit)


def test_axpy16_is_an_unbiased_estimator():
    """E{z} = x + a y (App. A.4): the mean over independent roundings converges at the Monte-Carlo rate."""
    w, g, _ = tensors(8, 48)
    w[0], g[0] = 2.0 ** -3, 2.0 ** -7          # power-of-two maxima: nothing near the saturating top code
    w, g = np.clip(w, -2.0 ** -3, 2.0 ** -3), np.clip(g, -2.0 ** -7, 2.0 ** -7)
    a = -0.1
    S = 3000
    acc = np.zeros(w.size)
    sq = np.zeros(w.size)
    for s in range(S):
        z, (ex, _, _) = oracle.axpy16(w, g, a, seed=100 + s, step=s)
        acc += z
        sq += z.astype(np.float64) ** 2
    mean = acc / S
    exact = w.astype(np.float64) + np.float64(np.float32(a)) * g.astype(np.float64)
    std = np.sqrt(np.maximum(sq / S - mean ** 2, 0)) + 1e-30
    zscore = (mean - exact) / (std / np.sqrt(S))
    assert np.max(np.abs(zscore)) < 5.0
    unit = 2.0 ** (ex - 127 - 14)
    assert np.all(std < 1.5 * unit)            # three roundings, each below one unit of the weight grid
    # negative control: round-to-nearest everywhere is biased for these operands (same statistic fails)
    zn, _ = oracle.axpy16(w, g, a, seed=1, step=0, rounding=oracle.NEAREST)
    assert np.max(np.abs(zn - exact) / (std / np.sqrt(S))) > 5.0


def test_update_below_the_grid_still_moves_the_weights_on_average():
    """lr * g far below one unit of the weight grid: round-to-nearest would freeze the weights, the stochastic
    update moves them by the right amount on average (the point of Remark 5)."""
    n = 4096
    w = np.full(n, 0.75, np.float32)
    g = np.full(n, 1.0, np.float32)
    lr = 2.0 ** -20                             # update = 2^-20, unit of w = 2^-15
    z, _ = oracle.axpy16(w, g, -lr, seed=3, step=0)
    moved = np.mean(w.astype(np.float64) - z)
    assert abs(moved - lr) < 4 * np.sqrt(lr * 2.0 ** -15 / n)
    zn, _ = oracle.axpy16(w, g, -lr, seed=3, step=0, rounding=oracle.NEAREST)
    assert np.array_equal(zn, w)


def test_saturation_and_vanishing_updates():
    x = np.float32([1.0, -1.0, 0.5, 0.0])
    y = np.float32([1.0, -1.0, 1.0, -1.0])
    z, (ex, _, _) = oracle.axpy16(x, y, 1.0e6, seed=0, step=0)       # update >> weights: clamps, keeps the sign
    unit = 2.0 ** (ex - 127 - 14)
    sat = (2 ** 23 - 2 ** 15) * unit
    assert np.array_equal(z, np.float32([1.0 + sat, -1.0 - sat, 0.5 + sat, -sat]))
    z, _ = oracle.axpy16(x, y, 1.0e-30, seed=0, step=0)              # update 2^-85 of a unit: never rounds up
    assert np.array_equal(z, x)
    z, _ = oracle.axpy16(x, np.zeros(4, np.float32), 0.3, seed=0, step=0)
    assert np.array_equal(z, x)


def test_sgd16_step_is_three_axpys_and_tracks_the_float_optimiser():
    w, g, v = tensors(21, 500)
    lr, mu, wd = 0.1, 0.9, 5e-4
    w1, v1 = oracle.sgd16_step(w, g, v, lr, mu, wd, seed=9, step=4)
    g1, _ = oracle.axpy16(g, w, wd, seed=9, step=12)
    v_ref, _ = oracle.axpy16(g1, v, mu, seed=9, step=13)
    w_ref, _ = oracle.axpy16(w, v_ref, -lr, seed=9, step=14)
    assert np.array_equal(v1, v_ref) and np.array_equal(w1, w_ref)
    # floating-point SGD with the same hyper-parameters: every tensor agrees to a few units of its int16 grid
    g1f = g.astype(np.float64) + wd * w
    vf = g1f + mu * v
    wf = w - lr * vf
    assert np.max(np.abs(v1 - vf)) < 4 * 2.0 ** (oracle.scale(vf.astype(np.float32)) - 141)
    assert np.max(np.abs(w1 - wf)) < 4 * 2.0 ** (oracle.scale(w) - 141)
    # the optional terms drop out cleanly
    w2, v2 = oracle.sgd16_step(w, g, None, lr, 0.0, 0.0, seed=9, step=4)
    assert v2 is None and np.array_equal(w2, oracle.axpy16(w, g, -lr, seed=9, step=14)[0])
    w3, v3 = oracle.sgd16_step(w, g, v, lr, mu, 0.0, seed=9, step=4)
    v3r, _ = oracle.axpy16(g, v, mu, seed=9, step=13)
    assert np.array_equal(v3, v3r) and np.array_equal(w3, oracle.axpy16(w, v3r, -lr, seed=9, step=14)[0])


def test_multi_tensor_step_is_the_single_step_per_tensor_with_its_own_streams():
    rng = np.random.default_rng(31)
    sizes = [5, 64, 1000, 1, 333]
    ws = [(rng.standard_normal(n) * 10.0 ** -k).astype(np.float32) for k, n in enumerate(sizes)]   # very different scales
    gs = [rng.laplace(0, 2e-3, n).astype(np.float32) for n in sizes]
    vs = [rng.laplace(0, 1e-2, n).astype(np.float32) for n in sizes]
    w1, v1 = oracle.sgd16_step_multi(ws, gs, vs, 0.1, 0.9, 5e-4, seed=4, step=7)
    for t in range(len(sizes)):
        wt, vt = oracle.sgd16_step(ws[t], gs[t], vs[t], 0.1, 0.9, 5e-4, seed=4, step=(7 << 16) | t)
        assert np.array_equal(w1[t], wt) and np.array_equal(v1[t], vt)
    # own scale per tensor: the tiny tensor keeps its relative precision (a shared scale would flush it to zero)
    assert np.max(np.abs(w1[4] - ws[4])) > 0 and np.max(np.abs(w1[4])) < 1e-2
    # two tensors with identical contents do not draw identical roundings
    same, _ = oracle.sgd16_step_multi([ws[2], ws[2]], [gs[2], gs[2]], [vs[2], vs[2]], 0.1, 0.9, 5e-4, seed=4, step=7)
    assert not np.array_equal(same[0], same[1])
    w2, v2 = oracle.sgd16_step_multi(ws, gs, None, 0.05, 0.0, 0.0, seed=4, step=7)
    assert v2 is None and np.array_equal(w2[1], oracle.sgd16_step(ws[1], gs[1], None, 0.05, seed=4, step=(7 << 16) | 1)[0])
