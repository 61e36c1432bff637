"""Seeded synthetic inputs for the integer linear-layer step.

Shared by the tests, the benchmark and the smoke check; it holds no arithmetic
of the method (no scale, mapping, GEMM or inverse mapping) — only random fp32
tensors with the shapes and value distributions of the five benchmark
workloads, which stand in for the ResNet / ViT layers the paper trains
(Sec. 5, App. A.5): the paper's datasets and weights are not used.

All draws come from numpy.random.Generator(PCG64(seed)) in a fixed order
(X, then W, then dY), so a (workload, seed) pair names one set of tensors.
"""
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Layer:
    name: str
    M: int  # rows of X and dY (batch x tokens, or batch x output pixels)
    K: int  # input features (contraction length of the forward GEMM)
    N: int  # output features


# ViT-B/16 at batch 64 x 197 tokens
_VIT_M = 64 * 197

WORKLOADS = {
    # single small linear layer
    "c1": [Layer("linear256", 256, 256, 256)],
    # ResNet-18 stage-2 3x3 conv as an im2col GEMM: batch 32, 128->128 channels, 28x28
    "c2": [Layer("resnet18_conv3x3_128", 32 * 28 * 28, 128 * 9, 128)],
    # ViT-B/16 MLP fc1
    "c3": [Layer("vit_fc1", _VIT_M, 768, 3072)],
    # ViT-B/16 encoder block: every linear layer
    "c4": [Layer("vit_qkv", _VIT_M, 768, 2304), Layer("vit_proj", _VIT_M, 768, 768),
           Layer("vit_fc1", _VIT_M, 768, 3072), Layer("vit_fc2", _VIT_M, 3072, 768)],
    # large square stress GEMM; sigma is a parameter
    "c5": [Layer("square8192", 8192, 8192, 8192)],
}
C5_SIGMAS = (1e-6, 1e-2, 1.0, 1e3)
DEFAULT_SEED = {"c1": 0, "c2": 1, "c3": 2, "c4": 3, "c5": 4}


def _normal(rng, shape, sigma):
    return (rng.standard_normal(shape, dtype=np.float32) * np.float32(sigma)).astype(np.float32)


def _laplace(rng, shape, b):
    return rng.laplace(0.0, b, size=shape).astype(np.float32)


def im2col_3x3(act):
    """[B,C,H,W] -> [B*H*W, C*9] patches of a 3x3, stride 1, zero-padded-by-1
    convolution; column order (c, kh, kw).  Input construction only."""
    B, C, H, W = act.shape
    p = np.zeros((B, C, H + 2, W + 2), dtype=act.dtype)
    p[:, :, 1:-1, 1:-1] = act
    s = p.strides
    win = np.lib.stride_tricks.as_strided(p, shape=(B, H, W, C, 3, 3), strides=(s[0], s[2], s[3], s[1], s[2], s[3]),
                                          writeable=False)
    return np.ascontiguousarray(win).reshape(B * H * W, C * 9)


def layer_tensors(workload, layer_index=0, seed=None, sigma=1.0, scale_down=1):
    """fp32 (X[M,K], W[K,N], dY[M,N]) of one layer of a workload.

    scale_down > 1 divides M (and, for c5, K and N) for reduced-size parity
    cases; distributions are unchanged.
    """
    layer = WORKLOADS[workload][layer_index]
    if seed is None:
        seed = DEFAULT_SEED[workload]
    rng = np.random.Generator(np.random.PCG64([seed, layer_index]))
    M, K, N = layer.M, layer.K, layer.N
    if workload == "c1":
        X = _normal(rng, (M, K), 1.0)
        W = _normal(rng, (K, N), 1.0)
        dY = _laplace(rng, (M, N), 1e-4)
    elif workload == "c2":
        batch = max(1, 32 // scale_down)
        act = np.maximum(_normal(rng, (batch, 128, 28, 28), 1.0), 0.0)  # ReLU'd N(0,1)
        X = im2col_3x3(act)
        M = X.shape[0]
        W = _normal(rng, (K, N), np.sqrt(2.0 / K))                      # N(0, 2/fan_in) as a variance
        dY = _normal(rng, (M, N), 1e-3)
    elif workload in ("c3", "c4"):
        M = max(1, M // scale_down)
        X = _normal(rng, (M, K), 1.0)
        W = _normal(rng, (K, N), 0.02)
        dY = _laplace(rng, (M, N), 1e-5)
        outlier = rng.random((M, N), dtype=np.float32) < np.float32(1e-3)  # 0.1 % of entries x1000
        dY = np.where(outlier, dY * np.float32(1000.0), dY).astype(np.float32)
    elif workload == "c5":
        M, K, N = (max(1, v // scale_down) for v in (M, K, N))
        X = _normal(rng, (M, K), sigma)
        W = _normal(rng, (K, N), sigma)
        dY = _normal(rng, (M, N), sigma)
    else:
        raise KeyError(workload)
    return X, W, dY


def ops_per_layer(layer):
    """Integer operations (multiply and add counted separately) of the three
    GEMMs of one forward + backward layer step."""
    return 3 * 2 * layer.M * layer.K * layer.N


def mapped_elements(layer):
    """fp32 elements that go through scale + map in one layer step (X, W, dY)."""
    return layer.M * layer.K + layer.K * layer.N + layer.M * layer.N


# The convolution of workload c2 given as a convolution (channels-last) instead of its patch matrix.
C2_CONV = dict(N=32, H=28, W=28, C=128, Cout=128, KH=3, KW=3, stride=1, pad=1)


def conv_tensors(seed=1, N=None, H=None, W=None, C=None, Cout=None, KH=3, KW=3, stride=1, pad=1):
    """fp32 (X[N,H,W,C], Wt[Cout,KH,KW,C], dY[N,Ho,Wo,Cout]): ReLU'd N(0,1) activations, N(0, 2/fan_in)
    weights, N(0, 1e-3) gradients; defaults are the c2 layer."""
    g = dict(C2_CONV)
    for k, v in dict(N=N, H=H, W=W, C=C, Cout=Cout).items():
        if v is not None:
            g[k] = v
    g.update(KH=KH, KW=KW, stride=stride, pad=pad)
    rng = np.random.Generator(np.random.PCG64([seed, 77]))
    X = np.maximum(_normal(rng, (g["N"], g["H"], g["W"], g["C"]), 1.0), 0.0)
    fan_in = KH * KW * g["C"]
    Wt = _normal(rng, (g["Cout"], KH, KW, g["C"]), np.sqrt(2.0 / fan_in))
    Ho, Wo = (g["H"] + 2 * pad - KH) // stride + 1, (g["W"] + 2 * pad - KW) // stride + 1
    dY = _normal(rng, (g["N"], Ho, Wo, g["Cout"]), 1e-3)
    return X, Wt, dY, g


# The two attention products of one ViT-B/16 encoder block at batch 64: 64 x 12 heads, 197 tokens padded to
# 208 (a multiple of 16; the padding rows are zero), head width 64.
VITB_ATTN = dict(batch=768, S=208, S_real=197, d=64)


def attention_tensors(seed=1, batch=None, S=None, S_real=None, d=None):
    """fp32 inputs of the attention products: Q, K, V [batch,S,d] ~ N(0,1) with rows >= S_real zero,
    P [batch,S,S] = row softmax of Q K^T / sqrt(d) over the real tokens (zero elsewhere), and N(0, 1e-3)
    upstream gradients dS [batch,S,S] (of the scores) and dO [batch,S,d] (of the context)."""
    g = dict(VITB_ATTN)
    for k, v in dict(batch=batch, S=S, S_real=S_real, d=d).items():
        if v is not None:
            g[k] = v
    b, s, r, dd = g["batch"], g["S"], g["S_real"], g["d"]
    rng = np.random.Generator(np.random.PCG64([seed, 78]))
    Q, K, V = (_normal(rng, (b, s, dd), 1.0) for _ in range(3))
    for t in (Q, K, V):
        t[:, r:, :] = 0.0
    z = np.matmul(Q[:, :r], K[:, :r].transpose(0, 2, 1)) / np.float32(np.sqrt(dd))
    z = np.exp(z - z.max(axis=2, keepdims=True))
    P = np.zeros((b, s, s), dtype=np.float32)
    P[:, :r, :r] = z / z.sum(axis=2, keepdims=True)
    dS = _normal(rng, (b, s, s), 1e-3)
    dO = _normal(rng, (b, s, dd), 1e-3)
    return dict(Q=Q, K=K, V=V, P=P, dS=dS, dO=dO), g


# Parameter count of torchvision's ResNet-18 (the smallest model of the paper's classification table), used as
# one flat vector for the optimiser step.
RESNET18_PARAMS = 11_689_512


def sgd_tensors(n=RESNET18_PARAMS, seed=1):
    """fp32 (w, g, v): N(0, 0.05) weights, N(0, 2e-3) gradients, N(0, 1e-2) momentum buffer."""
    rng = np.random.Generator(np.random.PCG64([seed, 79]))
    return _normal(rng, (n,), 0.05), _normal(rng, (n,), 2e-3), _normal(rng, (n,), 1e-2)


def resnet18_parameter_sizes():
    """Element counts of the 62 parameter tensors of a ResNet-18 classifier (7x7 stem, four stages of two basic
    blocks at 64/128/256/512 channels with 1x1 projection shortcuts where the shape changes, 1000-way head),
    in definition order: every convolution is followed by the scale and shift of its batch-norm."""
    sizes = [64 * 3 * 7 * 7, 64, 64]
    cin = 64
    for stage, cout in enumerate((64, 128, 256, 512)):
        for block in range(2):
            c_in = cin if block == 0 else cout
            sizes += [cout * c_in * 9, cout, cout, cout * cout * 9, cout, cout]
            if block == 0 and c_in != cout:
                sizes += [cout * c_in, cout, cout]
        cin = cout
    sizes += [1000 * 512, 1000]
    assert sum(sizes) == RESNET18_PARAMS and len(sizes) == 62
    return sizes


def sgd_tensor_list(sizes=None, seed=1):
    """Per-tensor fp32 (w, g, v) lists: weights N(0, 2/n-ish scale differing per tensor), gradients and momentum
    three and one orders of magnitude below, so that every tensor has its own scale."""
    sizes = sizes if sizes is not None else resnet18_parameter_sizes()
    rng = np.random.Generator(np.random.PCG64([seed, 80]))
    ws, gs, vs = [], [], []
    for n in sizes:
        sigma = float(np.sqrt(2.0 / max(n, 64)) * 8.0)
        ws.append(_normal(rng, (n,), sigma))
        gs.append(_normal(rng, (n,), sigma * 2e-2))
        vs.append(_normal(rng, (n,), sigma * 1e-1))
    return ws, gs, vs
