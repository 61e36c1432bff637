"""GPU parity: every entry point of the C ABI against the CPU oracle, element by
element, on the same seeded inputs.  Bar: bit-exact for scales, int8 and int32;
0 ulp for the fp32 outputs of the inverse mapping."""
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


# --------------------------------------------------------------------------- scale
@pytest.mark.parametrize("n", [0, 1, 3, 4, 5, 255, 1000, 4096 * 4 + 1, (1 << 20) + 3, 5_000_011])
def test_scale_sizes(fxp, n):
    say("scale n", n)
    rng = np.random.default_rng(n)
    x = (rng.standard_normal(n) * 10.0 ** rng.uniform(-20, 20)).astype(np.float32)
    assert int(host(fxp.scale(dev(x)))[0]) == oracle.scale(x)
    if n > 8:
        for off in (1, 2, 3):       # pointers off the 16-byte grid
            say("scale misaligned", n, off)
            assert int(host(fxp.scale(dev(x)[off:]))[0]) == oracle.scale(x[off:])


def test_scale_special_values_and_max_position(fxp):
    say("scale specials")
    cases = [np.zeros(100, np.float32), np.array([1e-45, -3e-39, 0], np.float32), np.array([np.inf, 1], np.float32),
             np.array([np.nan, 1], np.float32), np.array([-3.0e38], np.float32), np.array([2.0 ** -126], np.float32)]
    for x in cases:
        assert int(host(fxp.scale(dev(x)))[0]) == oracle.scale(x)
    base = np.random.default_rng(0).standard_normal(3_000_001).astype(np.float32)
    for pos in (0, 1, 1234567, 3_000_000):
        x = base.copy()
        x[pos] = -70000.0
        assert int(host(fxp.scale(dev(x)))[0]) == oracle.scale(x) == 127 + 16


# --------------------------------------------------------------------------- map
def check_map(fxp, x, e_max=None, seed=3, sid=(7 << 8) | 1, rounding=0, bits=8):
    e = oracle.scale(x) if e_max is None else e_max
    want = oracle.map(x, e, seed=seed, stream_id=sid, rounding=rounding, bits=bits)
    xd, ed = dev(x), dev(np.array([e], np.int32))
    q, qT = fxp.map(xd, ed, seed, sid, rounding, bits, want_q=True, want_qT=True)
    assert np.array_equal(host(q), want)
    assert np.array_equal(host(qT), want.T)
    q, _ = fxp.map(xd, ed, seed, sid, rounding, bits, want_q=True, want_qT=False)
    assert np.array_equal(host(q), want)
    _, qT = fxp.map(xd, ed, seed, sid, rounding, bits, want_q=False, want_qT=True)
    assert np.array_equal(host(qT), want.T)


@pytest.mark.parametrize("shape", [(128, 128), (256, 384), (1, 4), (5, 8), (130, 132), (16, 1000), (333, 260),
                                   (1000, 16), (48, 4096), (7, 13), (129, 3), (64, 130), (1, 1),
                                   (1100, 208), (2300, 400)])   # rows of partial lines: tiles numbered per XCD
def test_map_shapes(fxp, shape):
    say("map shape", shape)
    rng = np.random.default_rng(shape[0] * 7919 + shape[1])
    x = (rng.standard_normal(shape) * np.exp(rng.uniform(-8, 2, shape))).astype(np.float32)
    check_map(fxp, x)


@pytest.mark.parametrize("bits", [8, 7, 6, 5, 4, 2])
@pytest.mark.parametrize("rounding", [0, 1])
def test_map_bits_and_rounding(fxp, bits, rounding):
    say("map bits", bits, "rounding", rounding)
    x = np.random.default_rng(bits).standard_normal((200, 260)).astype(np.float32)
    check_map(fxp, x, rounding=rounding, bits=bits)


def test_map_edge_values(fxp):
    rng = np.random.default_rng(11)
    x = rng.standard_normal((256, 128)).astype(np.float32)
    x[0, :8] = [np.inf, -np.inf, np.nan, 0.0, -0.0, 1e-42, -1e-40, 3.0e38]
    x[5, 5] = 1.9999999
    say("map non-finite, own scale")
    check_map(fxp, x)
    say("map non-finite, scale below")
    check_map(fxp, x, e_max=120)
    say("map scale above")
    check_map(fxp, x[1:], e_max=150)
    say("map tiny scale")
    check_map(fxp, (x[1:] * np.float32(1e-38)).astype(np.float32))
    check_map(fxp, (x[1:] * np.float32(1e-38)).astype(np.float32), e_max=24)
    check_map(fxp, (x[1:] * np.float32(1e-38)).astype(np.float32), e_max=25)
    say("map top of the exponent range, scales just below the tensor's own")
    big = (x[1:] * np.float32(5e37)).astype(np.float32)
    assert oracle.scale(big) == 254
    check_map(fxp, big)
    check_map(fxp, x[1:], e_max=254)
    own = oracle.scale(x[1:])
    check_map(fxp, x[1:], e_max=own - 1)
    check_map(fxp, x[1:], e_max=own - 3)
    say("map zeros")
    check_map(fxp, np.zeros((128, 128), np.float32))
    say("map huge seed")
    check_map(fxp, x[1:], seed=2**64 - 1, sid=2**63 + 12345)


def test_map_random_magnitudes_scales_and_widths(fxp):
    """Seeded random tensors over the whole exponent range: values spread over up to 60 binades (so that shifts
    of every size occur, sub-normals and zeros included), the tensor's own scale and scales a few steps above and
    below it, every width and both roundings."""
    rng = np.random.default_rng(2024)
    for case in range(40):
        rows, cols = int(rng.integers(1, 200)), int(rng.integers(1, 70)) * 4
        centre = int(rng.integers(-125, 120))
        spread = int(rng.integers(1, 60))
        expo = rng.integers(centre - spread, centre + 1, size=(rows, cols))
        x = (rng.standard_normal((rows, cols)) * np.exp2(expo.astype(np.float64))).astype(np.float32)
        x[rng.random((rows, cols)) < 0.1] = 0.0
        own = oracle.scale(x)
        e_max = int(np.clip(own + int(rng.integers(-3, 4)), 1, 254))
        bits, rounding = int(rng.integers(2, 9)), int(rng.integers(0, 2))
        say("map random", case, (rows, cols), "own scale", own, "used", e_max, "bits", bits, "rounding", rounding)
        check_map(fxp, x, e_max=e_max, seed=case, sid=(case << 8) | 2, rounding=rounding, bits=bits)


def test_map_random_index_beyond_32_bits_is_keyed_by_element(fxp):
    """Row-major element index drives the random word, independent of the tiling."""
    say("map reshape invariance")
    x = np.random.default_rng(5).standard_normal((512, 1024)).astype(np.float32)
    e = dev(np.array([oracle.scale(x)], np.int32))
    a, _ = fxp.map(dev(x), e, 9, 4)
    b, _ = fxp.map(dev(x.reshape(2048, 256)), e, 9, 4)
    c, _ = fxp.map(dev(x.reshape(64, 8192)), e, 9, 4)
    assert np.array_equal(host(a).ravel(), host(b).ravel()) and np.array_equal(host(a).ravel(), host(c).ravel())


def test_scale_map_fused_equals_two_calls(fxp):
    for shape in [(300, 516), (64, 64), (100, 7)]:
        say("scale_map", shape)
        x = np.random.default_rng(shape[1]).standard_normal(shape).astype(np.float32) * 37
        e, q, qT = fxp.scale_map(dev(x), 5, 6, want_q=True, want_qT=True)
        eo = oracle.scale(x)
        assert int(host(e)[0]) == eo
        want = oracle.map(x, eo, seed=5, stream_id=6)
        assert np.array_equal(host(q), want) and np.array_equal(host(qT), want.T)


REUSE_SHAPES = [(256, 256), (300, 516), (1000, 64), (777, 192), (4099, 640), (25088, 128), (12608, 768), (5, 8)]


def test_scale_map_reuses_its_scratch_area(fxp):
    """fxp_scale_map with one scratch area from call to call: the block maxima a tensor with a larger scale left
    there (or any other bytes) do not leak into the next tensor's scale."""
    ws = torch.full((2 * fxp.workspace_bytes(fxp.OP_SCALE, 0),), 0xA5, dtype=torch.uint8, device="cuda")
    for i, shape in enumerate(REUSE_SHAPES):
        say("scale_map scratch reuse", shape)
        rng = np.random.default_rng(100 + i)
        x = (rng.standard_normal(shape) * 0.37).astype(np.float32)
        for scale_up in (4096.0, 1.0):
            xs = (x * np.float32(scale_up)).astype(np.float32)
            e_ref = oracle.scale(xs)
            want = oracle.map(xs, e_ref, seed=11, stream_id=3)
            e, q, qT = fxp.scale_map(dev(xs), 11, 3, want_q=True, want_qT=True, ws=ws)
            assert int(host(e)[0]) == e_ref
            assert np.array_equal(host(q), want) and np.array_equal(host(qT), want.T)


PAIRS = [((300, 516), (516, 40)), ((4000, 1152), (1152, 128)), ((64, 64), (640, 192)), ((100, 7), (64, 64)),
         ((2600, 1024), (1024, 1024)), ((33, 64), (70, 128))]


@pytest.mark.parametrize("sa,sb", PAIRS)
def test_two_tensor_calls_equal_single_calls(fxp, sa, sb):
    """fxp_map2 / fxp_scale_map2 (one launch for two tensors where their tilings agree, else two) against the
    oracle, for equal and different tile widths, and the element-wise path."""
    say("map2", sa, sb)
    rng = np.random.default_rng(sa[0] + sb[1])
    xa = (rng.standard_normal(sa) * 3).astype(np.float32)
    xb = (rng.standard_normal(sb) * 0.02).astype(np.float32)
    ea, eb = oracle.scale(xa), oracle.scale(xb)
    wa, wb = oracle.map(xa, ea, seed=5, stream_id=256), oracle.map(xb, eb, seed=5, stream_id=257)
    e, (qa, qaT), (qb, qbT) = fxp.scale_map2(dev(xa), dev(xb), seed=5, stream_ids=(256, 257))
    assert host(e).tolist() == [ea, eb]
    assert np.array_equal(host(qa), wa) and np.array_equal(host(qaT), wa.T)
    assert np.array_equal(host(qb), wb) and np.array_equal(host(qbT), wb.T)
    ed = dev(np.array([ea + 1, eb], np.int32))          # given scales (one of them above the tensor's own)
    wa1 = oracle.map(xa, ea + 1, seed=6, stream_id=1)
    wb1 = oracle.map(xb, eb, seed=6, stream_id=2, rounding=oracle.STOCHASTIC)
    (qa, qaT), (qb, qbT) = fxp.map2(dev(xa), ed[0:1], dev(xb), ed[1:2], seed=6, stream_ids=(1, 2))
    assert np.array_equal(host(qa), wa1) and np.array_equal(host(qaT), wa1.T)
    assert np.array_equal(host(qb), wb1) and np.array_equal(host(qbT), wb1.T)


# --------------------------------------------------------------------------- gemm
def rand_i8(rng, shape, lo=-127, hi=127):
    return rng.integers(lo, hi + 1, size=shape, dtype=np.int64).astype(np.int8)


GEMM_SHAPES = [(128, 128, 64), (256, 256, 128), (300, 200, 160), (1, 1, 16), (33, 65, 48), (129, 257, 80),
               (512, 768, 256), (64, 64, 0), (100, 90, 50), (17, 5, 7), (128, 128, 4096), (1152, 128, 6272),
               (1024, 2048, 512), (2100, 1800, 320),
               # ring kernel (>= 96 tiles of 256 x 256, K % 128 == 0), full and ragged edges, one and many steps
               (2560, 2560, 256), (2500, 2700, 384), (2560, 2560, 128), (3000, 2304, 1152),
               # four-stage 256 x 256 x 64 kernel: K % 128 == 64, and split along K (wide, few tiles, long K)
               (2560, 2560, 192), (1024, 1024, 4160), (768, 1536, 6336),
               # 128-tile direct-to-LDS kernels: K % 128 == 0 (8 waves) and K % 128 == 64 (4 waves), 1..5 steps
               (300, 200, 256), (300, 200, 192), (260, 130, 64), (129, 257, 640), (640, 128, 320)]


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_all_operand_forms(fxp, M, N, K):
    rng = np.random.default_rng(M * 31 + N * 17 + K)
    A, B = rand_i8(rng, (M, K)), rand_i8(rng, (K, N))
    want = oracle.gemm(A, np.ascontiguousarray(B.T), transB=True)
    AT, BT = np.ascontiguousarray(A.T), np.ascontiguousarray(B.T)
    for tA, tB, a, b in [(False, True, A, BT), (False, False, A, B), (True, False, AT, B), (True, True, AT, BT)]:
        say("gemm", (M, N, K), "transA", tA, "transB", tB)
        got = host(fxp.gemm(dev(a), dev(b), transA=tA, transB=tB))
        assert got.dtype == np.int32 and np.array_equal(got, want)


def test_gemm_extreme_values_longest_contraction(fxp):
    K = 25088
    say("gemm extremes K", K)
    A = np.full((130, K), 127, np.int8)
    B = np.full((70, K), -127, np.int8)
    A[::2] = -127
    got = host(fxp.gemm(dev(A), dev(B), transB=True))
    want = oracle.gemm(A, B, transB=True)
    assert np.array_equal(got, want) and abs(int(got[0, 0])) == 16129 * K


@pytest.mark.parametrize("K", [133144, 133136, 133120])
def test_gemm_longest_contraction_the_interface_allows(fxp, K):
    """127 * 127 * 133144 is the last sum below 2^31: extreme operands at the documented maximum of K (and at
    the nearest multiples of 16 and of 128, which take the other loaders), whole or split along K, through
    workspace slices and through atomics."""
    say("gemm extremes at the largest K", K)
    A = np.full((70, K), 127, np.int8)
    B = np.full((130, K), -127, np.int8)
    A[::2] = -127
    want = oracle.gemm(A, B, transB=True)
    assert int(np.abs(want.astype(np.int64)).max()) <= 2**31 - 1
    assert abs(int(want[0, 0])) == 16129 * K and int(want[0, 0]) == -int(want[1, 0])
    tiny = torch.empty(256, dtype=torch.uint8, device="cuda")
    for ws in (None, tiny):
        got = host(fxp.gemm(dev(A), dev(B), transB=True, ws=ws))
        assert np.array_equal(got, want)
    e = dev(np.array([140, 99], np.int32))
    assert same_bits(host(fxp.gemm_unmap(dev(A), dev(B), e[0:1], e[1:2], transB=True)), oracle.unmap(want, 140, 99))
    with pytest.raises(Exception):
        fxp.gemm(dev(np.zeros((8, 133145), np.int8)), dev(np.zeros((8, 133145), np.int8)), transB=True)


def test_gemm_split_k_both_ways_and_deterministic(fxp):
    """Long contraction, small output: slices of K go to the workspace and are summed by a
    second pass; with no room for the slices they add into the output with int32 atomics."""
    rng = np.random.default_rng(1)
    # (33, 65, 4096) and (5, 3, 2064): M * N is odd, so the slices after the first start off a 16-byte boundary
    # unless the slice stride is padded
    for (M, N, K) in [(256, 128, 8192), (512, 768, 6208), (33, 65, 4096), (5, 3, 2064)]:
        Ah, Bh = rand_i8(rng, (M, K)), rand_i8(rng, (N, K))
        want = oracle.gemm(Ah, Bh, transB=True)
        A, B = dev(Ah), dev(Bh)
        say("gemm split-K through workspace", (M, N, K))
        assert fxp.workspace_bytes(fxp.OP_GEMM, M, N, K) >= 2 * M * N * 4
        for _ in range(3):
            assert np.array_equal(host(fxp.gemm(A, B, transB=True)), want)
        say("gemm split-K through atomics", (M, N, K))
        tiny = torch.empty(256, dtype=torch.uint8, device="cuda")
        for _ in range(3):
            assert np.array_equal(host(fxp.gemm(A, B, transB=True, ws=tiny)), want)
        e = dev(np.array([120, 131], np.int32))
        got = host(fxp.gemm_unmap(A, B, e[0:1], e[1:2], transB=True, ws=tiny))
        assert same_bits(got, oracle.unmap(want, 120, 131))


# --------------------------------------------------------------------------- unmap
def test_unmap_all_exponent_ranges(fxp):
    rng = np.random.default_rng(2)
    special = np.array([0, 1, -1, (1 << 24) + 1, (1 << 24) + 3, -(1 << 24) - 1, (1 << 25) + 2, 2**31 - 1, -2**31,
                        0x00FFFFFF, 3, 5], dtype=np.int64).astype(np.int32)
    acc = np.concatenate([special, rng.integers(-2**31, 2**31, 100_003, dtype=np.int64).astype(np.int32),
                          rng.integers(-5000, 5000, 50_000, dtype=np.int64).astype(np.int32)])
    for eA, eB in [(133, 133), (1, 1), (1, 90), (1, 100), (10, 100), (60, 66), (70, 70), (254, 200), (254, 240),
                   (254, 254), (127, None), (1, None), (254, None)]:
        say("unmap", eA, eB)
        eBd = None if eB is None else dev(np.array([eB], np.int32))
        got = host(fxp.unmap(dev(acc), dev(np.array([eA], np.int32)), eBd))
        assert same_bits(got, oracle.unmap(acc, eA, eB))
    say("unmap in place, odd offset, bits")
    a = dev(acc[1:])                      # 4-byte but not 16-byte aligned
    e7 = dev(np.array([140], np.int32))
    out = fxp.unmap(a, e7, e7, bitsA=5, bitsB=7, out=a.view(torch.float32))
    assert same_bits(host(out), oracle.unmap(acc[1:], 140, 140, bitsA=5, bitsB=7))
    q = np.arange(-128, 128).astype(np.int8)
    assert same_bits(host(fxp.unmap_i8(dev(q), dev(np.array([3], np.int32)))), oracle.unmap_i8(q, 3))


@pytest.mark.parametrize("M,N,K", [(300, 200, 160), (128, 128, 4096), (512, 768, 256), (1024, 1280, 64),
                                   (2560, 2560, 256), (2560, 2600, 192), (1024, 1024, 4160), (100, 90, 50),
                                   (2500, 2570, 384), (3100, 2304, 128)])      # 160 x 128 tiles, ragged in both directions
def test_gemm_unmap_fused(fxp, M, N, K):
    rng = np.random.default_rng(M + N + K)
    A, B = rand_i8(rng, (M, K)), rand_i8(rng, (N, K))
    acc = oracle.gemm(A, B, transB=True)
    for eA, eB in [(127, 120), (3, 2), (250, 250)]:
        say("gemm_unmap", (M, N, K), eA, eB)
        got = host(fxp.gemm_unmap(dev(A), dev(B), dev(np.array([eA], np.int32)), dev(np.array([eB], np.int32)),
                                  transB=True))
        assert same_bits(got, oracle.unmap(acc, eA, eB))


# --------------------------------------------------------------------------- layer
def layer_check_full(fxp, X, W, dY, seed, step, rounding=0, bits=8):
    M, K = X.shape
    N = W.shape[1]
    buf = fxp.LayerBuffers(M, K, N)
    Y = fxp.linear_fwd(dev(X), dev(W), buf, seed, step, rounding, bits)
    dX, dW = fxp.linear_bwd(dev(dY), buf, seed, step, rounding, bits)
    Yo, saved = oracle.linear_fwd(X, W, seed, step, rounding, bits)
    dXo, dWo, aux = oracle.linear_bwd(dY, saved, seed, step, rounding, bits)
    assert host(buf.e).tolist() == [saved["eX"], saved["eW"], aux["eG"]]
    assert np.array_equal(host(buf.Xq), saved["Xq"]) and np.array_equal(host(buf.XqT), saved["Xq"].T)
    assert np.array_equal(host(buf.Wq), saved["Wq"]) and np.array_equal(host(buf.WqT), saved["Wq"].T)
    assert np.array_equal(host(buf.dYq), aux["dYq"]) and np.array_equal(host(buf.dYqT), aux["dYq"].T)
    assert same_bits(host(Y), Yo)
    assert same_bits(host(dX), dXo)
    assert same_bits(host(dW), dWo)
    return buf


@pytest.mark.parametrize("K", [140032, 140016, 140001, 300000])
def test_products_over_contractions_longer_than_one_int32_sum(fxp, K):
    """Beyond 133144 terms an int32 sum could wrap: the product then runs as int32 slices added in 64 bits and
    rounded once.  Extreme operands (sums of +-127^2 * K, past 2^31) and random ones, against the oracle's exact
    int64 sums; K a multiple of 128, of 16 only, odd (element-wise loader), and long enough for three slices."""
    say("long contraction", K)
    rng = np.random.default_rng(K)
    A, B = rand_i8(rng, (70, K)), rand_i8(rng, (130, K))
    A[0], A[1], B[0], B[1] = 127, -127, 127, -127
    want = oracle.gemm(A, B, transB=True)
    assert want.dtype == np.int64 and int(want[0, 0]) == 16129 * K > 2**31 and int(want[0, 1]) == -16129 * K
    e = dev(np.array([120, 131], np.int32))
    assert same_bits(host(fxp.gemm_unmap(dev(A), dev(B), e[0:1], e[1:2], transB=True)), oracle.unmap(want, 120, 131))
    # operands stored the other way round (transposed into the scratch area first), and the abs-max variant
    AT, Bn = dev(np.ascontiguousarray(A.T)), dev(np.ascontiguousarray(B.T))
    assert same_bits(host(fxp.gemm_unmap(AT, Bn, e[0:1], e[1:2], transA=True, transB=False)), oracle.unmap(want, 120, 131))
    area = torch.zeros(fxp.ABSMAX_WORDS, dtype=torch.int32, device="cuda")
    got = host(fxp.gemm_unmap_absmax(dev(A), dev(B), e[0:1], e[1:2], area, transB=True))
    assert same_bits(got, oracle.unmap(want, 120, 131))
    assert int(host(area).view(np.uint32).max()) == int(np.abs(got).max().view(np.uint32))
    # no 64-bit path: int32 output, or no room for the slices
    with pytest.raises(Exception):
        fxp.gemm(dev(A), dev(B), transB=True)
    with pytest.raises(Exception):
        fxp.gemm_unmap(dev(A), dev(B), e[0:1], e[1:2], transB=True, ws=torch.empty(256, dtype=torch.uint8, device="cuda"))


def test_long_contraction_forces_slices_on_a_large_output(fxp):
    """2048 x 2048 outputs are not split along K for speed; past 133144 terms they are, for exactness (two slices of
    256 x 256 tiles here).  Sampled rows against the oracle, rows of extremes included."""
    M = N = 2048
    K = 133248
    say("long contraction, large output", (M, N, K))
    gen = torch.Generator(device="cuda").manual_seed(5)
    A = torch.randint(-127, 128, (M, K), dtype=torch.int8, device="cuda", generator=gen)
    B = torch.randint(-127, 128, (N, K), dtype=torch.int8, device="cuda", generator=gen)
    A[7], B[3], B[2040] = 127, 127, -127
    e = dev(np.array([133, 133], np.int32))                      # one unit = 2^0
    assert fxp.workspace_bytes(fxp.OP_GEMM, M, N, K) >= 2 * M * N * 4
    C = host(fxp.gemm_unmap(A, B, e[0:1], e[1:2], transB=True))
    rows = [0, 7, 255, 256, 1000, 2047]
    want = oracle.gemm(host(A[rows]), host(B), transB=True)
    assert want.dtype == np.int64 and int(want[1, 3]) == 16129 * K > 2**31 and int(want[1, 2040]) == -16129 * K
    assert same_bits(C[rows], oracle.unmap(want, 133, 133))


def test_layer_over_more_rows_than_one_int32_sum_holds(fxp):
    """A linear layer applied to 140 000 rows: the weight gradient contracts over all of them (its reduction rides
    in the input-gradient launch); one column of X and of dY maps to +-127 in every row, so its sum passes 2^31."""
    M, K, N = 140000, 64, 48
    say("long-contraction layer", (M, K, N))
    rng = np.random.default_rng(12)
    X = rng.uniform(-1, 1, (M, K)).astype(np.float32)
    W = (rng.standard_normal((K, N)) * 0.05).astype(np.float32)
    dY = rng.uniform(-1e-3, 1e-3, (M, N)).astype(np.float32)
    X[:, 0], dY[:, 0] = 127 / 64, -127 * 2.0 ** -16          # top code in every row (units 2^-6 and 2^-16)
    X[:, 1], dY[:, 1] = -127 / 64, -127 * 2.0 ** -16
    for rounding in (0, 1):
        buf = layer_check_full(fxp, X, W, dY, seed=4, step=9, rounding=rounding)
    only_dW = fxp.linear_bwd(dev(dY), buf, 4, 9, 1, 8, need_dX=False)[1]
    assert same_bits(host(only_dW), oracle.linear_bwd(dY, oracle.linear_fwd(X, W, 4, 9, 1, 8)[1], 4, 9, 1, 8)[1])
    E = int(host(buf.e)[0]) - 133 + int(host(buf.e)[2]) - 133
    assert 16129 * M > 2**31 and float(host(only_dW)[0, 0]) == float(np.float32(np.ldexp(-16129.0 * M, E)))


def test_layer_with_more_input_features_than_one_int32_sum_holds(fxp):
    """The forward product's contraction (K = 140 032 input features) beyond 133144 terms; one row of X and one
    column of W at the top code, so that entry of Y passes 2^31 units."""
    M, K, N = 64, 140032, 32
    say("long-contraction forward", (M, K, N))
    rng = np.random.default_rng(13)
    X = rng.uniform(-1, 1, (M, K)).astype(np.float32)
    W = rng.uniform(-1, 1, (K, N)).astype(np.float32)
    dY = rng.uniform(-1, 1, (M, N)).astype(np.float32)
    X[5], W[:, 7] = 127 / 64, -127 / 64
    buf = layer_check_full(fxp, X, W, dY, seed=2, step=3)
    assert float(host(buf.Y)[5, 7]) == float(np.float32(-16129.0 * K * 2.0 ** -12))


ABSMAX_SHAPES = [(2560, 2560, 256), (4096, 1536, 128), (300, 200, 160), (100, 90, 50), (256, 128, 8192), (17, 5, 7)]


@pytest.mark.parametrize("M,N,K", ABSMAX_SHAPES)
def test_product_leaves_its_absmax_for_the_next_map(fxp, M, N, K):
    """fxp_gemm_unmap_absmax: same output as fxp_gemm_unmap, and the word it raises is the bit pattern of the
    largest |C|, from which fxp_map_absmax takes the scale the reduction pass would have found (every kernel
    family: 256-tiles, output-streaming tile, 128-tiles, element-wise loader, split along K with and without
    workspace)."""
    say("gemm absmax", M, N, K)
    rng = np.random.default_rng(M + N + K)
    A, B = rand_i8(rng, (M, K)), rand_i8(rng, (N, K))
    eA, eB = 128, 121
    want = oracle.unmap(oracle.gemm(A, B, transB=True), eA, eB)
    top = int(np.abs(want).max().view(np.uint32))
    e = dev(np.array([eA, eB], np.int32))
    for ws in (None, torch.empty(256, dtype=torch.uint8, device="cuda")):      # second: no room for split-K slices
        word = torch.zeros(fxp.ABSMAX_WORDS, dtype=torch.int32, device="cuda")
        C = fxp.gemm_unmap_absmax(dev(A), dev(B), e[0:1], e[1:2], word, transB=True, ws=ws)
        assert same_bits(host(C), want)
        assert int(host(word).max()) == top
        es, q, qT = fxp.map_absmax(C, word, seed=3, stream_id=515, want_q=True, want_qT=True)
        e_ref = oracle.scale(want)
        wq = oracle.map(want, e_ref, seed=3, stream_id=515)
        assert int(host(es)[0]) == e_ref
        assert np.array_equal(host(q), wq) and np.array_equal(host(qT), wq.T)
    # the word only ever rises: a larger value stays, and a second product adds its own maximum
    word = torch.full((fxp.ABSMAX_WORDS,), 0x7F000000, dtype=torch.int32, device="cuda")
    fxp.gemm_unmap_absmax(dev(A), dev(B), e[0:1], e[1:2], word, transB=True)
    assert bool((word == 0x7F000000).all())
    word = torch.full((fxp.ABSMAX_WORDS,), 5, dtype=torch.int32, device="cuda")
    fxp.gemm_unmap_absmax(dev(A), dev(B), e[0:1], e[1:2], word, transB=True)
    assert int(host(word).max()) == top and int(host(word).min()) >= 5
    # an output that overflows to Inf reports the bits of Inf: scale 255, as the reduction pass would
    big = dev(np.array([254, 254], np.int32))
    word = torch.zeros(fxp.ABSMAX_WORDS, dtype=torch.int32, device="cuda")
    C = fxp.gemm_unmap_absmax(dev(A), dev(B), big[0:1], big[1:2], word, transB=True)
    assert same_bits(host(C), oracle.unmap(oracle.gemm(A, B, transB=True), 254, 254)) and int(host(word).max()) == 0x7F800000


def test_layer_c1_full(fxp):
    say("layer c1 256^3, seed 0")
    X, W, dY = synth.layer_tensors("c1")
    layer_check_full(fxp, X, W, dY, seed=0, step=0)
    say("layer c1 nearest, 6 bits")
    layer_check_full(fxp, X, W, dY, seed=0, step=3, rounding=1, bits=6)


@pytest.mark.parametrize("workload,scale_down,sigma", [("c2", 8, 1.0), ("c3", 16, 1.0), ("c5", 16, 1e-6),
                                                        ("c5", 16, 1e3)])
def test_layer_reduced_workloads_full_check(fxp, workload, scale_down, sigma):
    say("layer reduced", workload, scale_down, sigma)
    X, W, dY = synth.layer_tensors(workload, scale_down=scale_down, sigma=sigma)
    layer_check_full(fxp, X, W, dY, seed=1, step=2)


def test_layer_ragged_shapes(fxp):
    for (M, K, N) in [(100, 48, 36), (257, 130, 66), (5, 7, 3), (1, 16, 1)]:
        say("layer ragged", (M, K, N))
        rng = np.random.default_rng(M)
        X = rng.standard_normal((M, K)).astype(np.float32)
        W = (rng.standard_normal((K, N)) * 0.1).astype(np.float32)
        dY = rng.laplace(0, 1e-3, (M, N)).astype(np.float32)
        layer_check_full(fxp, X, W, dY, seed=4, step=1)


def test_layer_random_shapes(fxp):
    """Seeded random layer shapes, half of them multiples of 16 (direct-to-LDS kernels with partial K steps in all
    three products), the rest arbitrary (element-wise loaders): the whole step against the oracle."""
    rng = np.random.default_rng(2024)
    shapes = []
    for k in range(28):
        M, K, N = (int(v) for v in rng.integers(1, 700, 3))
        if k % 2 == 0:
            M, K, N = (max(16, v // 16 * 16) for v in (M, K, N))
        shapes.append((M, K, N))
    shapes += [(1040, 208, 464), (4112, 80, 1040), (272, 4240, 144)]      # several tiles, ragged, K tails, split-K
    shapes += [(4096, 33, 65), (4112, 48, 17)]      # weight gradient split into slices of odd size, summed in the dX launch
    for (M, K, N) in shapes:
        say("layer random", (M, K, N))
        X = rng.standard_normal((M, K)).astype(np.float32)
        W = (rng.standard_normal((K, N)) * 0.1).astype(np.float32)
        dY = rng.laplace(0, 1e-3, (M, N)).astype(np.float32)
        layer_check_full(fxp, X, W, dY, seed=M, step=K % 5)


def test_layer_only_one_gradient(fxp):
    say("layer dW only / dX only")
    X, W, dY = synth.layer_tensors("c1")
    buf = fxp.LayerBuffers(256, 256, 256)
    fxp.linear_fwd(dev(X), dev(W), buf, 0, 0)
    buf.dX.fill_(7.0)
    dX, dW = fxp.linear_bwd(dev(dY), buf, 0, 0, need_dX=False)
    assert dX is None and float(buf.dX.min()) == 7.0
    _, saved = oracle.linear_fwd(X, W, 0, 0)
    _, dWo, _ = oracle.linear_bwd(dY, saved, 0, 0, need_dX=False)
    assert same_bits(host(dW), dWo)


def test_binding_refuses_cpu_tensors(fxp):
    with pytest.raises(fxp.FxpError):
        fxp.scale(torch.zeros(4))


def test_layer_step_replays_from_a_hip_graph(fxp):
    """The layer calls only launch kernels (no allocation, no memset, no host read), so a step can be captured
    into a HIP graph; every replay, with eager work of other steps in between, reproduces the eager result."""
    say("graph capture of a layer step")
    X, W, dY = synth.layer_tensors("c3", 0, scale_down=8)
    M, K = X.shape
    N = W.shape[1]
    Xd, Wd, dYd = dev(X), dev(W), dev(dY)
    buf = fxp.LayerBuffers(M, K, N)

    def step(i):
        fxp.linear_fwd(Xd, Wd, buf, seed=7, step=i)
        fxp.linear_bwd(dYd, buf, seed=7, step=i)

    step(5)
    torch.cuda.synchronize()
    want = [t.clone() for t in (buf.Y, buf.dX, buf.dW, buf.Xq, buf.dYqT, buf.e)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(5)                                    # warm-up on the side stream, as graph capture wants
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(5)
    for other in (1, 2, 3):
        step(other)                                # eager work that overwrites every buffer
        torch.cuda.synchronize()
        assert not torch.equal(buf.Xq, want[3])
        graph.replay()
        torch.cuda.synchronize()
        got = (buf.Y, buf.dX, buf.dW, buf.Xq, buf.dYqT, buf.e)
        assert all(torch.equal(a, b) for a, b in zip(got, want))


def test_empty_operands_are_no_ops(fxp):
    """Zero-sized tensors: every entry point returns FXP_OK and writes nothing."""
    say("empty operands")
    L = fxp.lib()
    p = lambda t: t.data_ptr()
    guard = torch.full((64,), 7, dtype=torch.int32, device="cuda")
    e = torch.tensor([130], dtype=torch.int32, device="cuda")
    ws = torch.empty(2 * fxp.workspace_bytes(fxp.OP_SCALE, 0), dtype=torch.uint8, device="cuda")
    x = torch.zeros(16, dtype=torch.float32, device="cuda")
    q = torch.full((16,), 5, dtype=torch.int8, device="cuda")
    assert L.fxp_map(p(x), 0, 16, p(e), p(q), None, 0, 0, 0, 8, None) == 0
    assert L.fxp_map(p(x), 16, 0, p(e), p(q), None, 0, 0, 0, 8, None) == 0
    assert L.fxp_scale_map(p(x), 0, 16, p(e), p(q), None, 0, 0, 0, 8, p(ws), ws.numel(), None) == 0
    torch.cuda.synchronize()
    assert int(e[0]) == 1 and bool((q == 5).all())              # the scale of an empty tensor is 1; q untouched
    A = torch.ones((16, 16), dtype=torch.int8, device="cuda")
    assert L.fxp_gemm(0, 1, 0, 16, 16, p(A), 16, p(A), 16, p(guard), 16, None, 0, None) == 0
    assert L.fxp_gemm(0, 1, 16, 0, 16, p(A), 16, p(A), 16, p(guard), 16, None, 0, None) == 0
    assert L.fxp_gemm_batched(16, 16, 16, p(A), 16, 0, p(A), 16, 0, p(guard), 16, 256, 0, None) == 0
    assert L.fxp_unmap(p(guard), 0, p(e), 8, p(e), 8, p(x), None) == 0
    assert L.fxp_axpy16(p(x), p(x), 0.5, 0, p(x), None, 0, 0, 0, p(ws), ws.numel(), None) == 0
    torch.cuda.synchronize()
    assert bool((guard == 7).all()) and bool((x == 0).all())


def test_timeline_and_clock_probe_measure_without_changing_results(fxp):
    """The measurement helpers: the events recorded inside the layer calls come back as one interval per launch,
    in launch order, and the outputs are the ones an undisturbed call gives; the clock probe reports a plausible
    core clock."""
    import ctypes
    say("timeline / clock probe")
    L = fxp.lib()
    X, W, dY = synth.layer_tensors("c2", scale_down=8)
    M, K = X.shape
    N = W.shape[1]
    buf0, buf1 = fxp.LayerBuffers(M, K, N), fxp.LayerBuffers(M, K, N)
    Xd, Wd, Gd = dev(X), dev(W), dev(dY)
    fxp.linear_fwd(Xd, Wd, buf0, 5, 2)
    fxp.linear_bwd(Gd, buf0, 5, 2)
    torch.cuda.synchronize()
    assert L.fxp_timeline_begin(64) == 0
    assert L.fxp_timeline_begin(64) == -2                      # one timeline at a time
    for _ in range(2):
        fxp.linear_fwd(Xd, Wd, buf1, 5, 2)
        fxp.linear_bwd(Gd, buf1, 5, 2)
    us, tags, n = (ctypes.c_float * 64)(), (ctypes.c_int * 64)(), ctypes.c_int(0)
    assert L.fxp_timeline_end(us, tags, 64, ctypes.byref(n)) == 0
    got = [tags[i] for i in range(n.value)]
    one = [1, 2, 3, 0, 1, 2, 4, 5]                             # scale, map, product; entry, scale, map, dW, dX
    assert got in (one + [0] + one, one + [6, 0] + one + [6]), got     # (a stand-alone slice sum would add a 6)
    assert all(us[i] > 0.0 for i in range(n.value)) and sum(us[i] for i in range(n.value)) < 1e6
    assert L.fxp_timeline_end(us, tags, 64, ctypes.byref(n)) == -2
    for a, b in ((buf0.Y, buf1.Y), (buf0.dX, buf1.dX), (buf0.dW, buf1.dW)):
        assert same_bits(host(a), host(b))
    out = torch.zeros(2, dtype=torch.int64, device="cuda")
    assert L.fxp_clock_probe(out.data_ptr(), 300, torch.cuda.current_stream().cuda_stream) == 0
    torch.cuda.synchronize()
    ticks, cycles = host(out).tolist()
    assert 30000 <= ticks < 60000 and 300.0 < 100.0 * cycles / ticks < 3500.0, (ticks, cycles)
