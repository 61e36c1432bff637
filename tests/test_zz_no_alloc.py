"""The forward entry point that takes no workspace (its scratch is a device array inside the library) against
fxp_linear_fwd, through the C ABI: every output bit for bit, on two calls in a row, the second on a smaller
layer (the array then still holds the first call's block maxima and product slices), and against the oracle."""
import ctypes

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


def layer_inputs(M, K, N, seed):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((M, K)).astype(np.float32)
    W = (rng.standard_normal((K, N)) * 0.05).astype(np.float32)
    return X, W


def forward_both_ways(fxp, M, K, N, seed, step):
    """(outputs of fxp_linear_fwd, outputs of fxp_linear_fwd_static) as host arrays, raw C-ABI calls."""
    L = fxp.lib()
    X, W = layer_inputs(M, K, N, seed)
    Xd, Wd = dev(X), dev(W)
    st = torch.cuda.current_stream().cuda_stream
    outs = []
    for static in (False, True):
        buf = fxp.LayerBuffers(M, K, N)
        for t in (buf.Xq, buf.XqT, buf.Wq, buf.WqT):
            t.fill_(77)
        buf.Y.fill_(-5.0)
        if static:
            rc = L.fxp_linear_fwd_static(Xd.data_ptr(), Wd.data_ptr(), M, K, N, buf.Y.data_ptr(), ctypes.byref(buf.saved),
                                         seed, step, 0, 8, st)
        else:
            rc = L.fxp_linear_fwd(Xd.data_ptr(), Wd.data_ptr(), M, K, N, buf.Y.data_ptr(), ctypes.byref(buf.saved), seed,
                                  step, 0, 8, buf.ws.data_ptr(), buf.ws.numel(), st)
        assert rc == 0, (static, rc)
        torch.cuda.synchronize()
        outs.append(dict(Y=host(buf.Y), Xq=host(buf.Xq), XqT=host(buf.XqT), Wq=host(buf.Wq), WqT=host(buf.WqT),
                         e=host(buf.e)[:2].tolist()))
    return (X, W), outs[0], outs[1]


def test_static_scratch_forward_equals_the_workspace_forward_twice_in_a_row(fxp):
    L = fxp.lib()
    assert L.fxp_static_scratch_bytes() >= 1 << 20
    # first a layer whose product is split along its contraction (slices go through the scratch), then a smaller
    # one (also split), then one that is not split at all
    for (M, K, N) in [(384, 4224, 256), (130, 2064, 48), (200, 96, 72)]:
        say("no-alloc forward", (M, K, N))
        if K >= 2048:
            assert L.fxp_workspace_bytes(fxp.OP_LINEAR_FWD, M, N, K) >= 8192 + 2 * M * N * 4      # it does use slices
        (X, W), ref, got = forward_both_ways(fxp, M, K, N, seed=11, step=3)
        assert got["e"] == ref["e"]
        for name in ("Xq", "XqT", "Wq", "WqT"):
            assert np.array_equal(got[name], ref[name]), name
        assert same_bits(got["Y"], ref["Y"])
        Yo, saved = oracle.linear_fwd(X, W, seed=11, step=3)
        assert got["e"] == [saved["eX"], saved["eW"]] and np.array_equal(got["Xq"], saved["Xq"])
        assert same_bits(got["Y"], Yo)


def test_static_scratch_forward_refuses_what_does_not_fit(fxp):
    L = fxp.lib()
    M, K, N = 2048, 1 << 16, 1024            # 64 tiles of 128 x 256, split four ways: 32 MiB of slices + the maxima
    assert L.fxp_workspace_bytes(fxp.OP_LINEAR_FWD, M, N, K) > L.fxp_static_scratch_bytes()
    fake = ctypes.c_void_p(1 << 20)          # never dereferenced: the size test comes before any device work
    saved = fxp._Saved(*([1 << 20] * 6))
    assert L.fxp_linear_fwd_static(fake, fake, M, K, N, fake, ctypes.byref(saved), 0, 0, 0, 8, None) == -4
