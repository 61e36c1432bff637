"""GPU parity at the full sizes of the benchmark workloads, in the launch
configuration bench.py times (the layer calls): scales and all mapped int8 tensors
are compared in full with the oracle; GEMM outputs are compared exactly on sampled
rows the oracle computes one by one and through exact int64 identities that hold at
any size (C v = A (B v); sum C = colsum(A) . rowsum(B))."""
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


def exact_product_checks(out_f32, Aq, Bq_kn, E, rng, name):
    """out = unmap(A[M,K] * B[K,N]) must satisfy exact integer identities.  Entries
    are integers times 2^E below 2^24 in magnitude here, so the fp32 values convert
    back to the integer sums exactly."""
    C = np.ldexp(out_f32.astype(np.float64), -E)
    assert np.all(C == np.rint(C)) and np.abs(C).max() < 2**24, name
    C = C.astype(np.int64)
    A64, B64 = Aq.astype(np.int64), Bq_kn.astype(np.int64)
    assert int(C.sum()) == int(A64.sum(0) @ B64.sum(1)), name
    for _ in range(2):
        v = rng.integers(-3, 4, size=(B64.shape[1], 1))
        assert np.array_equal(C @ v, A64 @ (B64 @ v)), name


def sampled_rows_check(out_f32, A_rows_of, Bq_nk, eA, eB, rows, name):
    """exact comparison of sampled output rows with the oracle's GEMM + inverse map"""
    acc = oracle.gemm(A_rows_of(rows), Bq_nk, transB=True)
    assert same_bits(out_f32[rows], oracle.unmap(acc, eA, eB)), name


def run_layer_fullsize(fxp, workload, layer_index, sigma, n_rows):
    layer = synth.WORKLOADS[workload][layer_index]
    say("fullsize", workload, layer.name, "sigma", sigma, (layer.M, layer.K, layer.N))
    X, W, dY = synth.layer_tensors(workload, layer_index, sigma=sigma)
    M, K = X.shape
    N = W.shape[1]
    seed, step = 0, 0
    buf = fxp.LayerBuffers(M, K, N)
    Y = host(fxp.linear_fwd(dev(X), dev(W), buf, seed, step))
    dXd, dWd = fxp.linear_bwd(dev(dY), buf, seed, step)
    dX, dW = host(dXd), host(dWd)
    # --- scales and mapped tensors: full comparison
    eX, eW, eG = oracle.scale(X), oracle.scale(W), oracle.scale(dY)
    assert host(buf.e).tolist() == [eX, eW, eG]
    Xq = oracle.map(X, eX, seed=seed, stream_id=(step << 8) | 0)
    Wq = oracle.map(W, eW, seed=seed, stream_id=(step << 8) | 1)
    Gq = oracle.map(dY, eG, seed=seed, stream_id=(step << 8) | 2)
    for got, want, nm in [(buf.Xq, Xq, "Xq"), (buf.Wq, Wq, "Wq"), (buf.dYq, Gq, "dYq")]:
        assert np.array_equal(host(got), want), nm
    for got, want, nm in [(buf.XqT, Xq, "XqT"), (buf.WqT, Wq, "WqT"), (buf.dYqT, Gq, "dYqT")]:
        assert np.array_equal(host(got).T, want), nm
    # --- GEMM outputs
    rng = np.random.default_rng(99)
    WqT, XqT, GqT = (np.ascontiguousarray(a.T) for a in (Wq, Xq, Gq))
    rows_m = np.sort(rng.choice(M, size=min(n_rows, M), replace=False))
    rows_k = np.sort(rng.choice(K, size=min(n_rows, K), replace=False))
    sampled_rows_check(Y, lambda r: Xq[r], WqT, eX, eW, rows_m, "Y rows")
    sampled_rows_check(dX, lambda r: Gq[r], Wq, eG, eW, rows_m, "dX rows")
    sampled_rows_check(dW, lambda r: XqT[r], GqT, eX, eG, rows_k, "dW rows")
    exact_product_checks(Y, Xq, Wq, (eX - 133) + (eW - 133), rng, "Y identities")
    exact_product_checks(dX, Gq, WqT, (eG - 133) + (eW - 133), rng, "dX identities")
    exact_product_checks(dW, XqT, Gq, (eX - 133) + (eG - 133), rng, "dW identities")


def test_c2_resnet_conv_fullsize(fxp):
    run_layer_fullsize(fxp, "c2", 0, 1.0, 128)


def test_c3_vit_fc1_fullsize(fxp):
    run_layer_fullsize(fxp, "c3", 0, 1.0, 96)


@pytest.mark.parametrize("layer_index", [0, 1, 3])
def test_c4_vit_block_other_linears_fullsize(fxp, layer_index):
    run_layer_fullsize(fxp, "c4", layer_index, 1.0, 64)


@pytest.mark.parametrize("sigma", synth.C5_SIGMAS)
def test_c5_square_fullsize(fxp, sigma):
    run_layer_fullsize(fxp, "c5", 0, sigma, 32)
