"""GPU parity of the int16 weight update (axpy16, SGD step with weight decay and momentum) against the CPU
oracle: every output bit for bit (0 ulp), scales exact."""
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


def tensors(seed, n):
    rng = np.random.default_rng(seed)
    w = (rng.standard_normal(n) * 0.05).astype(np.float32)
    g = rng.laplace(0, 2e-3, n).astype(np.float32)
    v = rng.laplace(0, 1e-2, n).astype(np.float32)
    return w, g, v


@pytest.mark.parametrize("n", [1, 3, 4, 5, 1023, 4096, 262147, 3_000_001])
@pytest.mark.parametrize("a", [-0.1, 0.9, 5e-4, 1024.0, -3.0e-6])
def test_axpy16(fxp, n, a):
    say("axpy16", n, a)
    w, g, _ = tensors(n % 97, n)
    z, e = fxp.axpy16(dev(w), dev(g), a, seed=5, step=7)
    zo, eo = oracle.axpy16(w, g, a, seed=5, step=7)
    assert tuple(host(e).tolist()) == eo
    assert same_bits(host(z), zo)


@pytest.mark.parametrize("rounding", [0, 1])
def test_axpy16_special_values_in_place_and_unaligned(fxp, rounding):
    say("axpy16 special", rounding)
    rng = np.random.default_rng(2)
    n = 5000
    x = rng.standard_normal(n).astype(np.float32)
    y = rng.standard_normal(n).astype(np.float32)
    x[:8] = [0.0, -0.0, 1e-41, -1e-41, np.inf, -np.inf, np.nan, 3.0e38]
    y[3:9] = [np.inf, np.nan, -1e-45, 0.0, 1.0, -3.0e38]
    zo, eo = oracle.axpy16(x, y, 0.25, seed=1, step=2, rounding=rounding)
    xd, yd = dev(x), dev(y)
    z, e = fxp.axpy16(xd, yd, 0.25, seed=1, step=2, rounding=rounding)
    assert tuple(host(e).tolist()) == eo and same_bits(host(z), zo)
    # finite tensors: in place on x, and through views that are only 4-byte aligned
    x[:8] = 0.5
    y[3:9] = -0.25
    zo, _ = oracle.axpy16(x[1:], y[1:], -2.0, seed=1, step=2, rounding=rounding)
    xd, yd = dev(x), dev(y)
    z, _ = fxp.axpy16(xd[1:], yd[1:], -2.0, out=xd[1:], seed=1, step=2, rounding=rounding)
    assert same_bits(host(xd[1:]), zo) and host(xd)[0] == x[0]
    # tiny and huge scalars: vanishing update, saturating update
    for a in (1e-30, 1e30, 0.0):
        zo, eo = oracle.axpy16(x, y, a, seed=4, step=1, rounding=rounding)
        z, e = fxp.axpy16(dev(x), dev(y), a, seed=4, step=1, rounding=rounding)
        assert tuple(host(e).tolist()) == eo and same_bits(host(z), zo)


@pytest.mark.parametrize("lr,mu,wd", [(0.1, 0.9, 5e-4), (0.1, 0.0, 0.0), (0.01, 0.9, 0.0), (0.05, 0.0, 1e-5)])
@pytest.mark.parametrize("n", [7, 1000, 1_200_003])
def test_sgd16_step(fxp, n, lr, mu, wd):
    say("sgd16", n, lr, mu, wd)
    w, g, v = tensors(n % 89 + 1, n)
    buf = fxp.SgdBuffers(n)
    wd_, gd, vd = dev(w), dev(g), (dev(v) if mu != 0.0 else None)
    wo, vo = w, (v if mu != 0.0 else None)
    for step in range(3):                                  # a few steps: the state feeds back
        fxp.sgd16_step(wd_, gd, vd, buf, lr, mu, wd, seed=8, step=step)
        wo, vo = oracle.sgd16_step(wo, g, vo, lr, mu, wd, seed=8, step=step)
        assert same_bits(host(wd_), wo)
        if mu != 0.0:
            assert same_bits(host(vd), vo)
    assert np.array_equal(host(gd), g)


def test_sgd16_bench_size_full_oracle(fxp):
    """The vector bench.py times (ResNet-18's parameter count, its recipe and hyper-parameters): every element of
    w and v against the oracle over two consecutive steps."""
    from paper_2207_08822_amd import synth
    n = synth.RESNET18_PARAMS
    say("sgd16 full size", n)
    w, g, v = synth.sgd_tensors(n)
    buf = fxp.SgdBuffers(n)
    wd_, gd, vd = dev(w), dev(g), dev(v)
    wo, vo = w, v
    for step in range(2):
        fxp.sgd16_step(wd_, gd, vd, buf, 0.1, 0.9, 5e-4, seed=0, step=step)
        wo, vo = oracle.sgd16_step(wo, g, vo, 0.1, 0.9, 5e-4, seed=0, step=step)
        assert same_bits(host(wd_), wo) and same_bits(host(vd), vo)


def test_sgd16_rejects_bad_arguments(fxp):
    w = torch.zeros(16, device="cuda")
    buf = fxp.SgdBuffers(16)
    L = fxp.lib()
    p = lambda t: t.data_ptr()
    assert L.fxp_sgd16_step(p(w), p(w), None, 16, 0.1, 0.9, 0.0, None, 0, 0, 0, p(buf.ws), buf.ws.numel(), None) == -1
    assert L.fxp_sgd16_step(p(w), p(w), None, 16, 0.1, 0.0, 1e-4, None, 0, 0, 0, p(buf.ws), buf.ws.numel(), None) == -1
    assert L.fxp_sgd16_step(p(w), p(w), None, 16, 0.1, 0.0, 0.0, None, 0, 0, 0, p(buf.ws), 16, None) == -4
    assert L.fxp_sgd16_step(p(w), p(w), None, 16, 0.1, 0.0, 0.0, None, 0, 0, 7, p(buf.ws), buf.ws.numel(), None) == -5
    assert L.fxp_axpy16(p(w), None, 0.1, 16, p(w), None, 0, 0, 0, p(buf.ws), buf.ws.numel(), None) == -1


@pytest.mark.parametrize("lr,mu,wd", [(0.1, 0.9, 5e-4), (0.05, 0.0, 0.0), (0.01, 0.9, 0.0), (0.05, 0.0, 1e-4)])
def test_sgd16_step_multi(fxp, lr, mu, wd):
    """Lists of tensors of very different sizes and scales (more than one launch group: 70 tensors), odd lengths and
    4-byte-aligned views: every tensor equals the oracle's single-tensor step with its own stream."""
    say("sgd16 multi", lr, mu, wd)
    rng = np.random.default_rng(17)
    sizes = [5, 64, 1000, 1, 333, 70000, 4096, 3_000_001] + [int(s) for s in rng.integers(1, 5000, 62)]
    ws = [(rng.standard_normal(n) * 10.0 ** -(k % 5)).astype(np.float32) for k, n in enumerate(sizes)]
    gs = [rng.laplace(0, 2e-3, n).astype(np.float32) * np.float32(10.0 ** -(k % 3)) for k, n in enumerate(sizes)]
    vs = [rng.laplace(0, 1e-2, n).astype(np.float32) for n in sizes] if mu != 0.0 else None
    # one flat device buffer per kind with odd offsets: most views are only 4-byte aligned
    def views(arrs):
        flat = torch.empty(sum(a.size + 1 for a in arrs), dtype=torch.float32, device="cuda")
        out, off = [], 0
        for a in arrs:
            v = flat[off:off + a.size]
            v.copy_(torch.from_numpy(a))
            out.append(v)
            off += a.size + 1
        return out
    wd_, gd = views(ws), views(gs)
    vd = views(vs) if vs is not None else None
    buf = fxp.SgdMultiBuffers(wd_, gd, vd, weight_decay=(wd != 0.0))
    wo, vo = ws, vs
    for step in range(2):
        fxp.sgd16_step_multi(buf, lr, mu, wd, seed=3, step=step)
        wo, vo = oracle.sgd16_step_multi(wo, gs, vo, lr, mu, wd, seed=3, step=step)
        for t in range(len(sizes)):
            assert same_bits(host(wd_[t]), wo[t]), (step, t, sizes[t])
            if mu != 0.0:
                assert same_bits(host(vd[t]), vo[t]), (step, t, sizes[t])


def test_sgd16_step_multi_resnet18_list(fxp):
    """The bench's list (62 tensors of ResNet-18's sizes): every tensor against the oracle."""
    from paper_2207_08822_amd import synth
    say("sgd16 multi resnet18")
    ws, gs, vs = synth.sgd_tensor_list()
    wd_, gd, vd = [dev(a) for a in ws], [dev(a) for a in gs], [dev(a) for a in vs]
    buf = fxp.SgdMultiBuffers(wd_, gd, vd)
    fxp.sgd16_step_multi(buf, 0.1, 0.9, 5e-4, seed=0, step=0)
    wo, vo = oracle.sgd16_step_multi(ws, gs, vs, 0.1, 0.9, 5e-4, seed=0, step=0)
    for t in range(len(ws)):
        assert same_bits(host(wd_[t]), wo[t]) and same_bits(host(vd[t]), vo[t]), t


@pytest.mark.parametrize("rounding", [0, 1])
def test_axpy16_smallest_scales(fxp, rounding):
    """Tensors whose scale is at the bottom of the exponent range (all zero: scale 1; sub-normal only; around
    1e-38): the fast path scales by up to 2^149 and must agree with the oracle bit for bit."""
    say("axpy16 smallest scales", rounding)
    rng = np.random.default_rng(17)
    n = 4096 + 7
    base = rng.standard_normal(n).astype(np.float32)
    cases = [(base * np.float32(1e-38), np.zeros(n, np.float32), 0.5),
             ((base * np.float32(1e-42)).astype(np.float32), (base[::-1] * np.float32(3e-39)).astype(np.float32), -1.5),
             (np.zeros(n, np.float32), (base * np.float32(1e-30)).astype(np.float32), 1e-8),
             ((base * np.float32(2e-31)).astype(np.float32), (base[::-1] * np.float32(1e-36)).astype(np.float32), 3.0e5)]
    for x, y, a in cases:
        x, y = np.ascontiguousarray(x), np.ascontiguousarray(y)
        zo, eo = oracle.axpy16(x, y, a, seed=6, step=9, rounding=rounding)
        z, e = fxp.axpy16(dev(x), dev(y), a, seed=6, step=9, rounding=rounding)
        assert tuple(host(e).tolist()) == eo and same_bits(host(z), zo), (eo, a)
