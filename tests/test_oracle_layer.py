"""Pins for the oracle's layer composition (App. A.2; unbiasedness eq. of Sec. 3.4)."""
import numpy as np

import oracle


def small_layer(seed=0, M=12, K=48, N=10):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((M, K)).astype(np.float32)
    W = (rng.standard_normal((K, N)) * 0.05).astype(np.float32)
    dY = rng.laplace(0, 1e-3, (M, N)).astype(np.float32)
    # power-of-two maxima keep every element clear of the saturating top code
    X = np.clip(X, -4, 4); X[0, 0] = 4.0
    W = np.clip(W, -0.25, 0.25); W[0, 0] = 0.25
    dY = np.clip(dY, -2.0 ** -6, 2.0 ** -6); dY[0, 0] = 2.0 ** -6
    return X, W, dY


def test_layer_equals_the_primitives_chained():
    X, W, dY = small_layer(1, 9, 20, 7)
    seed, step = 99, 4
    Y, saved = oracle.linear_fwd(X, W, seed=seed, step=step)
    eX, eW = oracle.scale(X), oracle.scale(W)
    Xq = oracle.map(X, eX, seed=seed, stream_id=(step << 8) | oracle.TAG_X)
    Wq = oracle.map(W, eW, seed=seed, stream_id=(step << 8) | oracle.TAG_W)
    assert (saved["eX"], saved["eW"]) == (eX, eW)
    assert np.array_equal(saved["Xq"], Xq) and np.array_equal(saved["Wq"], Wq)
    assert np.array_equal(Y, oracle.unmap(oracle.gemm(Xq, Wq), eX, eW))
    dX, dW, aux = oracle.linear_bwd(dY, saved, seed=seed, step=step)
    eG = oracle.scale(dY)
    Gq = oracle.map(dY, eG, seed=seed, stream_id=(step << 8) | oracle.TAG_DY)
    assert aux["eG"] == eG and np.array_equal(aux["dYq"], Gq)
    assert np.array_equal(dX, oracle.unmap(oracle.gemm(Gq, Wq, transB=True), eG, eW))
    assert np.array_equal(dW, oracle.unmap(oracle.gemm(Xq, Gq, transA=True), eX, eG))
    # the mapped gradient is drawn once: both gradients are exact integer products of the same Gq
    assert np.array_equal(dX.astype(np.float64),
                          (Gq.astype(np.int64) @ Wq.astype(np.int64).T) * 2.0 ** (eG - 133 + eW - 133))
    only_dW = oracle.linear_bwd(dY, saved, seed=seed, step=step, need_dX=False)
    assert only_dW[0] is None and np.array_equal(only_dW[1], dW)


def test_layer_outputs_are_unbiased_and_have_the_closed_form_variance():
    """E{C_hat_ij} = C_ij (Sec. 3.4) and, for fixed operands, the per-entry variance of
    the integer product is sum_k sA_ik^2 B_kj^2 + A_ik^2 sB_kj^2 + sA_ik^2 sB_kj^2 with
    s^2 = p(1-p) LSB^2 (App. A.2 specialised to non-random X, G)."""
    X, W, dY = small_layer(2)
    S = 600
    Ys, dXs, dWs = [], [], []
    for s in range(S):
        Y, saved = oracle.linear_fwd(X, W, seed=1000 + s, step=s)
        dX, dW, _ = oracle.linear_bwd(dY, saved, seed=1000 + s, step=s)
        Ys.append(Y.astype(np.float64)); dXs.append(dX.astype(np.float64)); dWs.append(dW.astype(np.float64))
    X64, W64, G64 = X.astype(np.float64), W.astype(np.float64), dY.astype(np.float64)

    def bernoulli_var(t, e):
        lsb = 2.0 ** (e - 133)
        u = np.abs(t) / lsb
        p = u - np.floor(u)
        return p * (1 - p) * lsb * lsb

    vX, vW, vG = bernoulli_var(X64, oracle.scale(X)), bernoulli_var(W64, oracle.scale(W)), bernoulli_var(G64, oracle.scale(dY))
    cases = [
        (np.array(Ys), X64 @ W64, vX @ W64**2 + X64**2 @ vW + vX @ vW),
        (np.array(dXs), G64 @ W64.T, vG @ (W64**2).T + G64**2 @ vW.T + vG @ vW.T),
        (np.array(dWs), X64.T @ G64, vX.T @ G64**2 + (X64**2).T @ vG + vX.T @ vG),
    ]
    for samples, exact, var in cases:
        mean = samples.mean(0)
        z = (mean - exact) / np.sqrt(var / S)
        assert np.abs(z).max() < 4.8, np.abs(z).max()
        assert abs(z.mean()) < 4.0 / np.sqrt(z.size)          # no common-sign bias across entries
        ratio = samples.var(0, ddof=1) / var
        assert abs(ratio.mean() - 1.0) < 0.03, ratio.mean()
        assert ratio.min() > 0.6 and ratio.max() < 1.5


def test_steps_and_tensors_use_independent_random_streams():
    X, W, dY = small_layer(3)
    _, s0 = oracle.linear_fwd(X, W, seed=5, step=0)
    _, s1 = oracle.linear_fwd(X, W, seed=5, step=1)
    assert not np.array_equal(s0["Xq"], s1["Xq"])
    # X and W of one step do not share decisions: map W's values through X's stream and compare
    eW = oracle.scale(W)
    assert not np.array_equal(oracle.map(W, eW, seed=5, stream_id=0), s0["Wq"])
    assert np.array_equal(oracle.map(W, eW, seed=5, stream_id=1), s0["Wq"])


def test_weight_gradient_over_more_rows_than_an_int32_sum_holds():
    """A layer applied to more than 133144 rows: the weight gradient is the exact integer sum (which passes 2^31
    here: every mapped entry of one column pair is +-127) rounded once - checked against numpy's int64 product
    and numpy's own double -> float conversion."""
    M, K, N = oracle.INT32_TERMS + 5000, 3, 2
    rng = np.random.default_rng(8)
    X = rng.uniform(-1, 1, (M, K)).astype(np.float32)
    dY = rng.uniform(-1, 1, (M, N)).astype(np.float32)
    X[:, 0], dY[:, 0] = 127 / 64, -127 / 64              # mapped to +127 / -127 in every row
    W = rng.uniform(-1, 1, (K, N)).astype(np.float32)
    Y, saved = oracle.linear_fwd(X, W, seed=1, step=2, rounding=oracle.NEAREST)
    dX, dW, aux = oracle.linear_bwd(dY, saved, seed=1, step=2, rounding=oracle.NEAREST)
    acc = saved["Xq"].astype(np.int64).T @ aux["dYq"].astype(np.int64)
    assert acc[0, 0] == -16129 * M < -2**31
    E = (saved["eX"] - 133) + (aux["eG"] - 133)
    assert np.array_equal(dW, np.ldexp(acc.astype(np.float64), E).astype(np.float32))
    assert np.array_equal(dX.astype(np.float64), (aux["dYq"].astype(np.int64) @ saved["Wq"].astype(np.int64).T) * 2.0 ** (aux["eG"] - 133 + saved["eW"] - 133))
