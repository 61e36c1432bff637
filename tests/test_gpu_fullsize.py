"""GPU parity at the full sizes of the benchmark workloads, in the launch
configuration bench.py times (the layer calls): scales and all mapped int8 tensors
are compared in full with the oracle.  Product outputs: every element against the
oracle for the ResNet layer and the ViT layers (n_rows = None) and for the forward
product of the 8192^3 layer at sigma = 1; for its gradient products and for the other
three sigmas the oracle computes 32 rows of every 256-row band of the output (1024 rows
per product: every tile row of the launch, every 8-row group of a tile), and exact int64
identities that hold at any size cover the rest (C v = A (B v); sum C = colsum(A) .
rowsum(B))."""
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
    if n_rows is None or n_rows == "Y in full":
        # every element of every product (of the forward product only for the largest layer)
        assert same_bits(Y, oracle.unmap(oracle.gemm(Xq, WqT, transB=True), eX, eW)), "Y"
        if n_rows is None:
            assert same_bits(dX, oracle.unmap(oracle.gemm(Gq, Wq, transB=True), eG, eW)), "dX"
            assert same_bits(dW, oracle.unmap(oracle.gemm(XqT, GqT, transB=True), eX, eG)), "dW"
            return
        n_rows = "bands"
    if n_rows == "bands":
        band = lambda n: np.array([256 * t + 8 * j + (3 * j + t) % 8 for t in range((n + 255) // 256) for j in range(32)
                                   if 256 * t + 8 * j + (3 * j + t) % 8 < n])
        rows_m, rows_k = band(M), band(K)
    else:
        rows_m = np.sort(rng.choice(M, size=min(n_rows, M), replace=False))
        rows_k = np.sort(rng.choice(K, size=min(n_rows, K), replace=False))
    sampled_rows_check(Y, lambda r: Xq[r], WqT, eX, eW, rows_m, "Y rows")
    sampled_rows_check(dX, lambda r: Gq[r], Wq, eG, eW, rows_m, "dX rows")
    sampled_rows_check(dW, lambda r: XqT[r], GqT, eX, eG, rows_k, "dW rows")
    exact_product_checks(Y, Xq, Wq, (eX - 133) + (eW - 133), rng, "Y identities")
    exact_product_checks(dX, Gq, WqT, (eG - 133) + (eW - 133), rng, "dX identities")
    exact_product_checks(dW, XqT, Gq, (eX - 133) + (eG - 133), rng, "dW identities")


def test_c2_resnet_conv_fullsize(fxp):
    run_layer_fullsize(fxp, "c2", 0, 1.0, None)


def test_c3_vit_fc1_fullsize(fxp):
    run_layer_fullsize(fxp, "c3", 0, 1.0, None)


@pytest.mark.parametrize("layer_index", [0, 1, 3])
def test_c4_vit_block_other_linears_fullsize(fxp, layer_index):
    run_layer_fullsize(fxp, "c4", layer_index, 1.0, None)


@pytest.mark.parametrize("sigma", synth.C5_SIGMAS)
def test_c5_square_fullsize(fxp, sigma):
    # sigma = 1: the forward product in full (20 s of oracle time) and both gradients on 32 rows of every 256-row
    # band (all three products run the same kernel on the same shape); the other sigmas: bands for all three
    run_layer_fullsize(fxp, "c5", 0, sigma, "Y in full" if sigma == 1.0 else "bands")


# --------------------------------------------------------------------------- beyond 32-bit element counts
def _need_memory(nbytes):
    free, _ = torch.cuda.mem_get_info()
    if free < nbytes + (4 << 30):
        pytest.skip(f"needs {nbytes >> 30} GiB of device memory, {free >> 30} GiB free")


def _row_blocks(rows, cols, extra=()):
    """Row ranges to compare: both ends, the rows where the element index crosses 2^32 and 2^34, and any extra."""
    marks = [0, rows - 8] + [b // cols - 4 for b in (1 << 32, 1 << 34) if b // cols + 4 < rows] + list(extra)
    return sorted({max(0, min(rows - 8, m)) for m in marks})


@pytest.mark.parametrize("rows,cols,transposed", [((1 << 18) + 200, 16384 + 128, True), ((1 << 20) + 640, 16384, False),
                                                  (272, (1 << 22) - 4, True), (130, 1 << 22, True)],
                         ids=["2^32-elements-both-copies", "2^34-elements", "widest-rows-of-the-tiled-kernel",
                              "rows-too-wide-for-the-tiled-kernel"])
def test_scale_and_map_of_tensors_beyond_32_bit_indices(fxp, rows, cols, transposed):
    """Element counts above 2^32 (64-bit addressing, the transposed copy included) and above 2^34 (the second
    counter word of the random stream comes into use), and rows of 2^22 elements, where the tiled kernel's 32-bit
    offsets inside a tile end and the one-element-per-thread kernel takes over: the scale against a reduction by
    torch, the mapped bytes against the oracle on row blocks at both ends and around the 2^32 / 2^34 crossings."""
    n = rows * cols
    _need_memory(n * (6 if transposed else 5))
    say("huge map", rows, cols, "transposed" if transposed else "")
    gen = torch.Generator(device="cuda").manual_seed(rows)
    x = torch.empty((rows, cols), dtype=torch.float32, device="cuda")
    step = 1 << 14
    for r in range(0, rows, step):
        x[r:r + step].normal_(generator=gen)
    x[rows - 3, cols - 5] = -700.0                       # the maximum sits in the last rows
    bits = x.view(torch.int32)
    top = max(int((bits[r:r + step] & 0x7FFFFFFF).max()) for r in range(0, rows, step))
    e = fxp.scale(x)
    assert int(host(e)[0]) == top >> 23 == 136
    q, qT = fxp.map(x, e, seed=21, stream_id=(3 << 8) | 1, want_q=True, want_qT=transposed)
    torch.cuda.synchronize()
    for r0 in _row_blocks(rows, cols):
        want = oracle.map_rows(host(x[r0:r0 + 8]), r0, 136, seed=21, stream_id=(3 << 8) | 1)
        assert np.array_equal(host(q[r0:r0 + 8]), want), r0
        if transposed:
            assert np.array_equal(host(qT[:, r0:r0 + 8]).T, want), r0
    # every row block of 8 agrees between the two copies (device-side, whole tensor)
    if transposed:
        for r in range(0, rows, step):
            assert bool((q[r:r + step] == qT[:, r:r + step].T).all()), r


@pytest.mark.parametrize("M,N,K", [((1 << 22) + 300, 1152, 128), ((1 << 25) + 100, 192, 64)],
                         ids=["wide-output-4.8G", "tall-6.4G"])
def test_gemm_output_beyond_32_bit_indices(fxp, M, N, K):
    """Products whose output has more than 2^32 elements: sampled rows at both ends and around the 2^32-element
    crossing against the oracle, and an exact column-sum identity over the whole output."""
    _need_memory(M * K + M * N * 4)
    say("huge gemm", M, N, K)
    gen = torch.Generator(device="cuda").manual_seed(M)
    A = torch.randint(-127, 128, (M, K), dtype=torch.int8, device="cuda", generator=gen)
    B = torch.randint(-127, 128, (N, K), dtype=torch.int8, device="cuda", generator=gen)
    e = dev(np.array([133, 133], np.int32))               # one unit = 2^0: the output holds the integer sums
    C = fxp.gemm_unmap(A, B, e[0:1], e[1:2], transB=True)
    torch.cuda.synchronize()
    Bh = host(B)
    for r0 in _row_blocks(M, N):
        acc = oracle.gemm(host(A[r0:r0 + 8]), Bh, transB=True)
        assert same_bits(host(C[r0:r0 + 8]), acc.astype(np.float32)), r0
    # sum over all rows of C = (column sums of A) . B^T, exact in int64 / float64 (|entries| < 2^21)
    colsum = torch.zeros(K, dtype=torch.int64, device="cuda")
    total = torch.zeros(N, dtype=torch.float64, device="cuda")
    step = 1 << 18
    for r in range(0, M, step):
        colsum += A[r:r + step].sum(0, dtype=torch.int64)
        total += C[r:r + step].sum(0, dtype=torch.float64)
    want = host(colsum) @ Bh.astype(np.int64).T
    assert np.array_equal(host(total).astype(np.int64), want)
