"""GPU parity of the batched products (attention matmuls) against the CPU oracle: int32 / fp32 batched GEMM,
and the batched product layer forward + backward (scales, every int8 tensor, all fp32 outputs, bit for bit)."""
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


# batch, M, N, K: aligned (direct-to-LDS kernels, 128 and 256 tiles), K tails, unaligned (general loads), tiny,
# and the largest batch the interface accepts (through both kinds of kernel)
GEMM_CASES = [(3, 128, 128, 64), (5, 208, 208, 64), (4, 208, 64, 208), (2, 300, 260, 128), (3, 512, 512, 256),
              (40, 256, 256, 128), (7, 197, 197, 64), (6, 197, 64, 197), (9, 5, 3, 7), (1, 130, 70, 48), (2, 64, 64, 0),
              (65535, 16, 16, 16), (65535, 16, 24, 64)]


@pytest.mark.parametrize("batch,M,N,K", GEMM_CASES)
def test_gemm_batched(fxp, batch, M, N, K):
    say("gemm_batched", (batch, M, N, K))
    rng = np.random.default_rng(batch * 7 + M)
    A = rng.integers(-127, 128, (batch, M, K), dtype=np.int8)
    B = rng.integers(-127, 128, (batch, N, K), dtype=np.int8)
    ref = oracle.gemm_batched(A, B, transB=True)
    got = host(fxp.gemm_batched(dev(A), dev(B)))
    assert np.array_equal(got, ref)
    eA, eB = 120, 131
    e = torch.tensor([eA, eB], dtype=torch.int32, device="cuda")
    gotf = host(fxp.gemm_batched(dev(A), dev(B), e[0:1], e[1:2]))
    assert same_bits(gotf, oracle.unmap(ref, eA, eB))


def test_gemm_batched_rejects_bad_arguments(fxp):
    A = torch.zeros((2, 16, 16), dtype=torch.int8, device="cuda")
    with pytest.raises(fxp.FxpError):
        fxp.gemm_batched(A, torch.zeros((3, 16, 16), dtype=torch.int8, device="cuda"))
    C = torch.zeros((2, 16, 16), dtype=torch.int32, device="cuda")
    L = fxp.lib()
    p = lambda t: t.data_ptr()
    # overlapping outputs, negative stride, batch beyond the grid limit
    assert L.fxp_gemm_batched(16, 16, 16, p(A), 16, 256, p(A), 16, 256, p(C), 16, 100, 2, None) == -2
    assert L.fxp_gemm_batched(16, 16, 16, p(A), 16, -256, p(A), 16, 256, p(C), 16, 256, 2, None) == -2
    assert L.fxp_gemm_batched(16, 16, 16, p(A), 16, 0, p(A), 16, 0, p(C), 16, 256, 70000, None) == -2
    assert L.fxp_gemm_batched(16, 16, 16, None, 16, 256, p(A), 16, 256, p(C), 16, 256, 2, None) == -1


def check_bmm(fxp, A, Bm, dY, transB, seed=3, step=2, rounding=0, bits=8, need_dA=True, need_dB=True):
    batch, M, K = A.shape
    N = dY.shape[2]
    buf = fxp.BmmBuffers(batch, M, K, N, transB)
    Y = host(fxp.bmm_fwd(dev(A), dev(Bm), buf, seed, step, rounding, bits))
    Yo, sv = oracle.bmm_fwd(A, Bm, transB, seed, step, rounding, bits)
    assert host(buf.e)[:2].tolist() == [sv["eA"], sv["eB"]]
    assert np.array_equal(host(buf.Aq), sv["Aq"])
    assert np.array_equal(host(buf.AqT), sv["Aq"].reshape(batch * M, K).T)
    assert np.array_equal(host(buf.Bq), sv["Bq"])
    assert np.array_equal(host(buf.BqT), sv["Bq"].reshape(-1, Bm.shape[2]).T)
    assert same_bits(Y, Yo)
    dA, dB = fxp.bmm_bwd(dev(dY), buf, seed, step, rounding, bits, need_dA, need_dB)
    dAo, dBo, aux = oracle.bmm_bwd(dY, sv, seed, step, rounding, bits, need_dA, need_dB)
    assert int(host(buf.e)[2]) == aux["eG"]
    assert np.array_equal(host(buf.dYq), aux["dYq"])
    assert np.array_equal(host(buf.dYqT), aux["dYq"].reshape(batch * M, N).T)
    if need_dA:
        assert same_bits(host(dA), dAo)
    if need_dB:
        assert same_bits(host(dB), dBo)


BMM_CASES = [(3, 32, 64, 32), (4, 208, 64, 208), (2, 197, 64, 197), (5, 48, 80, 16), (3, 7, 5, 9), (2, 256, 128, 256),
             (1, 130, 48, 70)]


@pytest.mark.parametrize("transB", [False, True])
@pytest.mark.parametrize("batch,M,K,N", BMM_CASES)
def test_bmm_shapes(fxp, batch, M, K, N, transB):
    say("bmm", (batch, M, K, N), "transB", transB)
    rng = np.random.default_rng(batch * 100 + M + int(transB))
    A = rng.standard_normal((batch, M, K)).astype(np.float32)
    Bm = rng.standard_normal((batch, N, K) if transB else (batch, K, N)).astype(np.float32)
    dY = rng.laplace(0, 1e-3, (batch, M, N)).astype(np.float32)
    check_bmm(fxp, A, Bm, dY, transB)


def test_attention_products(fxp):
    """Q K^T (transB) and P V on a slice of the ViT-B recipe: padded sequence, softmax rows as the left operand."""
    t, g = synth.attention_tensors(seed=4, batch=6)
    say("attention", g)
    check_bmm(fxp, t["Q"], t["K"], t["dS"], True)
    check_bmm(fxp, t["P"], t["V"], t["dO"], False)
    check_bmm(fxp, t["P"], t["V"], t["dO"], False, rounding=1, bits=6, need_dA=False)


def test_bmm_full_size_sampled(fxp):
    """The bench shape (768 heads): a sample of whole matrices against the oracle's single products, the rest
    through the exact integer adjoint identity sum(G * (A B)) = sum((G B^T) * A)."""
    t, g = synth.attention_tensors(seed=1)
    say("attention full size", g)
    batch, S, d = g["batch"], g["S"], g["d"]
    buf = fxp.BmmBuffers(batch, S, d, S, True)
    Y = host(fxp.bmm_fwd(dev(t["Q"]), dev(t["K"]), buf, 1, 0))
    dA, dB = fxp.bmm_bwd(dev(t["dS"]), buf, 1, 0)
    eA, eB, eG = (int(v) for v in host(buf.e))
    assert (eA, eB, eG) == (oracle.scale(t["Q"]), oracle.scale(t["K"]), oracle.scale(t["dS"]))
    Aq, Bq, Gq = host(buf.Aq), host(buf.Bq), host(buf.dYq)
    for b in (0, 1, 383, 767):
        assert same_bits(Y[b], oracle.unmap(oracle.gemm(Aq[b], Bq[b], transB=True), eA, eB))
        assert same_bits(host(dA)[b], oracle.unmap(oracle.gemm(Gq[b], Bq[b]), eG, eB))
        assert same_bits(host(dB)[b], oracle.unmap(oracle.gemm(Gq[b], Aq[b], transA=True), eG, eA))
    # mapped operands: sampled rows against the oracle's map of the same rows is covered by the map tests; here
    # the integer identities tie every output element to the operands
    to_int = lambda x, E: np.rint(x.astype(np.float64) * 2.0 ** -E).astype(np.int64)
    lhs = int(np.sum(Gq.astype(np.int64) * to_int(Y, eA + eB - 266)))
    assert lhs == int(np.sum(to_int(host(dA), eG + eB - 266) * Aq.astype(np.int64)))
    assert lhs == int(np.sum(to_int(host(dB), eG + eA - 266) * Bq.astype(np.int64)))
