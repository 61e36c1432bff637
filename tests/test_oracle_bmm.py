"""Pins for the oracle's batched products (attention matmuls Q K^T and A V on integer mantissas, Sec. 5)."""
import numpy as np
import pytest

import oracle


def tensors(seed, batch, M, K, N, transB):
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((batch, M, K)).astype(np.float32)
    Bm = rng.standard_normal((batch, N, K) if transB else (batch, K, N)).astype(np.float32)
    dY = rng.laplace(0, 1e-3, (batch, M, N)).astype(np.float32)
    return A, Bm, dY


@pytest.mark.parametrize("tA,tB", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_gemm_batched_equals_numpy_matmul_per_matrix(tA, tB):
    rng = np.random.default_rng(3)
    batch, M, N, K = 5, 7, 9, 13
    A = rng.integers(-127, 128, (batch, K, M) if tA else (batch, M, K), dtype=np.int8)
    B = rng.integers(-127, 128, (batch, N, K) if tB else (batch, K, N), dtype=np.int8)
    C = oracle.gemm_batched(A, B, transA=bool(tA), transB=bool(tB))
    A64 = A.astype(np.int64).transpose(0, 2, 1) if tA else A.astype(np.int64)
    B64 = B.astype(np.int64).transpose(0, 2, 1) if tB else B.astype(np.int64)
    assert np.array_equal(C, np.matmul(A64, B64))
    # every matrix of the batch is the single product of its own operands (no mixing across the batch)
    for b in range(batch):
        assert np.array_equal(C[b], oracle.gemm(A[b], B[b], transA=bool(tA), transB=bool(tB)))


def test_gemm_batched_empty_batch_and_extreme_codes():
    assert oracle.gemm_batched(np.zeros((0, 3, 4), np.int8), np.zeros((0, 4, 2), np.int8)).shape == (0, 3, 2)
    A = np.full((2, 3, 1000), -127, np.int8)
    B = np.full((2, 1000, 2), 127, np.int8)
    assert np.all(oracle.gemm_batched(A, B) == -127 * 127 * 1000)


@pytest.mark.parametrize("transB", [False, True])
def test_single_matrix_batch_is_the_linear_layer(transB):
    """batch = 1 must reproduce the (separately pinned) linear layer bit for bit: same scales, same
    random streams, same products."""
    A, Bm, dY = tensors(5, 1, 11, 24, 6, transB)
    seed, step = 17, 3
    W = Bm[0].T.copy() if transB else Bm[0]
    Y, saved = oracle.bmm_fwd(A, Bm, transB=transB, seed=seed, step=step)
    if not transB:      # with transB the element order of Bm, hence its random words, differs from W's
        Yl, sl = oracle.linear_fwd(A[0], W, seed=seed, step=step)
        assert np.array_equal(Y[0], Yl) and np.array_equal(saved["Aq"][0], sl["Xq"])
        assert np.array_equal(saved["Bq"][0], sl["Wq"]) and (saved["eA"], saved["eB"]) == (sl["eX"], sl["eW"])
        dA, dB, aux = oracle.bmm_bwd(dY, saved, seed=seed, step=step)
        dXl, dWl, auxl = oracle.linear_bwd(dY[0], sl, seed=seed, step=step)
        assert np.array_equal(dA[0], dXl) and np.array_equal(dB[0], dWl) and np.array_equal(aux["dYq"][0], auxl["dYq"])
    else:
        Bq = saved["Bq"][0]
        sl = dict(Xq=saved["Aq"][0], Wq=Bq.T.copy(), eX=saved["eA"], eW=saved["eB"])
        assert np.array_equal(Y[0], oracle.unmap(oracle.gemm(sl["Xq"], sl["Wq"]), sl["eX"], sl["eW"]))
        dA, dB, aux = oracle.bmm_bwd(dY, saved, seed=seed, step=step)
        dXl, dWl, auxl = oracle.linear_bwd(dY[0], sl, seed=seed, step=step)
        assert np.array_equal(dA[0], dXl) and np.array_equal(dB[0], dWl.T) and np.array_equal(aux["dYq"][0], auxl["dYq"])


@pytest.mark.parametrize("transB", [False, True])
def test_bmm_is_the_primitives_chained_with_one_scale_per_tensor(transB):
    batch, M, K, N = 4, 6, 10, 5
    A, Bm, dY = tensors(8, batch, M, K, N, transB)
    A[2] *= 8.0          # one loud matrix sets the scale of the whole tensor
    seed, step = 5, 9
    Y, saved = oracle.bmm_fwd(A, Bm, transB=transB, seed=seed, step=step)
    eA, eB = oracle.scale(A), oracle.scale(Bm)
    assert (saved["eA"], saved["eB"]) == (eA, eB)
    Aq = oracle.map(A.reshape(batch * M, K), eA, seed=seed, stream_id=(step << 8) | oracle.TAG_X).reshape(A.shape)
    Bq = oracle.map(Bm.reshape(-1, Bm.shape[2]), eB, seed=seed, stream_id=(step << 8) | oracle.TAG_W).reshape(Bm.shape)
    assert np.array_equal(saved["Aq"], Aq) and np.array_equal(saved["Bq"], Bq)
    B64 = Bq.astype(np.int64).transpose(0, 2, 1) if transB else Bq.astype(np.int64)
    acc = np.matmul(Aq.astype(np.int64), B64)
    assert np.array_equal(Y.astype(np.float64), acc * 2.0 ** (eA - 133 + eB - 133))
    dA, dB, aux = oracle.bmm_bwd(dY, saved, seed=seed, step=step)
    eG = oracle.scale(dY)
    Gq = oracle.map(dY.reshape(batch * M, N), eG, seed=seed, stream_id=(step << 8) | oracle.TAG_DY).reshape(dY.shape)
    assert aux["eG"] == eG and np.array_equal(aux["dYq"], Gq)
    G64 = Gq.astype(np.int64)
    accA = np.matmul(G64, B64.transpose(0, 2, 1))
    accB = np.matmul(Aq.astype(np.int64).transpose(0, 2, 1), G64)       # [batch,K,N]
    if transB:
        accB = accB.transpose(0, 2, 1)
    assert np.array_equal(dA.astype(np.float64), accA * 2.0 ** (eG - 133 + eB - 133))
    assert np.array_equal(dB.astype(np.float64), accB * 2.0 ** (eG - 133 + eA - 133))
    only_dB = oracle.bmm_bwd(dY, saved, seed=seed, step=step, need_dA=False)
    assert only_dB[0] is None and np.array_equal(only_dB[1], dB)


@pytest.mark.parametrize("transB", [False, True])
def test_bmm_gradients_are_the_exact_adjoints_of_the_forward(transB):
    """<G, A.B> = <G.B^T, A> = <A^T.G, B> holds exactly on the integer mantissas."""
    batch, M, K, N = 3, 5, 12, 7
    A, Bm, dY = tensors(11, batch, M, K, N, transB)
    Y, saved = oracle.bmm_fwd(A, Bm, transB=transB, seed=2, step=1)
    dA, dB, aux = oracle.bmm_bwd(dY, saved, seed=2, step=1)
    eA, eB, eG = saved["eA"], saved["eB"], aux["eG"]
    to_int = lambda t, E: np.rint(t.astype(np.float64) / 2.0 ** E).astype(np.int64)
    accY = to_int(Y, eA + eB - 266)
    accA = to_int(dA, eG + eB - 266)
    accB = to_int(dB, eG + eA - 266)
    lhs = int(np.sum(aux["dYq"].astype(np.int64) * accY))
    assert lhs == int(np.sum(accA * saved["Aq"].astype(np.int64)))
    assert lhs == int(np.sum(accB * saved["Bq"].astype(np.int64)))


def test_exactly_representable_operands_give_the_float_product():
    """Operands that are small integers times a power of two map without rounding, so the layer must return
    the exact real product (which fp32 holds exactly here)."""
    rng = np.random.default_rng(4)
    batch, M, K, N = 3, 4, 8, 5
    A = rng.integers(-64, 65, (batch, M, K)).astype(np.float32) * 2.0 ** -3
    Bm = rng.integers(-64, 65, (batch, K, N)).astype(np.float32) * 2.0 ** 2
    A[0, 0, 0] = 64 * 2.0 ** -3
    Bm[0, 0, 0] = 64 * 2.0 ** 2
    Y, _ = oracle.bmm_fwd(A, Bm, seed=1, step=0)
    assert np.array_equal(Y.astype(np.float64), np.matmul(A.astype(np.float64), Bm.astype(np.float64)))
    Yk, _ = oracle.bmm_fwd(A, Bm.transpose(0, 2, 1).copy(), transB=True, seed=1, step=0)
    assert np.array_equal(Yk, Y)
