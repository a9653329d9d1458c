"""Workload recipes: the five multi-tenant low-batch inference mixes.

Each recipe returns a list of `Problem` descriptions (shape, dtype, deadline and
the distributions its operands are drawn from).  `draw_host` turns one
description into fp32 numpy arrays; `draw_device` does the same on the GPU for
sizes that are too large to draw on the host in reasonable time.  The draws are
fp32; rounding to the problem dtype is done by whoever consumes them.

The mixes stand in for the paper's workloads (replicas of ResNet-style and
other DNN models sharing one GPU at small batch, Sections 3-5): the paper's
own model corpus and traces are not available, so shapes follow the public
ResNet-50 / BERT-base layer dimensions and random low-batch GEMM shapes.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import List, Tuple

import numpy as np

ELEM_SIZE = {"f32": 4, "bf16": 2, "f16": 2}


@dataclass(frozen=True)
class Problem:
    """One independent operator from one model stream.

    GEMM:  C[M,N] = A[M,K] . B^T  with B stored K-contiguous as [N,K].
    CONV:  Y[Nb,Ho,Wo,Cout] = X[Nb,H,W,Cin] (*) W[Cout,R,S,Cin], NHWC,
           stride `stride` in both directions, dilation 1, zero padding (pad_h, pad_w),
           cross-correlation.
    CONV_NCHW: the same operator on channel-major arrays: Y[Nb,Cout,Ho,Wo] = X[Nb,Cin,H,W] (*) W[Cout,Cin,R,S].
    """

    op: str  # "gemm" | "conv" | "conv_nchw"
    dtype: str  # "f32" | "bf16" | "f16"
    M: int = 0
    N: int = 0
    K: int = 0
    Nb: int = 0
    H: int = 0
    W: int = 0
    Cin: int = 0
    Cout: int = 0
    R: int = 0
    S: int = 0
    pad_h: int = 0
    pad_w: int = 0
    stride: int = 1
    deadline_ms: float = math.inf
    a_dist: Tuple = ("normal", 1.0)
    b_dist: Tuple = ("normal", 1.0)
    tag: str = ""

    @property
    def a_shape(self):
        if self.op == "conv_nchw":
            return (self.Nb, self.Cin, self.H, self.W)
        return (self.M, self.K) if self.op == "gemm" else (self.Nb, self.H, self.W, self.Cin)

    @property
    def b_shape(self):
        if self.op == "conv_nchw":
            return (self.Cout, self.Cin, self.R, self.S)
        return (self.N, self.K) if self.op == "gemm" else (self.Cout, self.R, self.S, self.Cin)

    @property
    def c_shape(self):
        if self.op == "gemm":
            return (self.M, self.N)
        ho = (self.H + 2 * self.pad_h - self.R) // self.stride + 1
        wo = (self.W + 2 * self.pad_w - self.S) // self.stride + 1
        return (self.Nb, self.Cout, ho, wo) if self.op == "conv_nchw" else (self.Nb, ho, wo, self.Cout)


def canonical_dims(p: Problem):
    """(Mg, Ng, Kg) of the GEMM an operator is counted as (for flop/byte accounting)."""
    if p.op == "gemm":
        return p.M, p.N, p.K
    ho = (p.H + 2 * p.pad_h - p.R) // p.stride + 1
    wo = (p.W + 2 * p.pad_w - p.S) // p.stride + 1
    return p.Nb * ho * wo, p.Cout, p.R * p.S * p.Cin


def flops(p: Problem) -> int:
    """2*Mg*Ng*Kg; for convolutions this counts the zero-padding taps too."""
    mg, ng, kg = canonical_dims(p)
    return 2 * mg * ng * kg


def algorithmic_bytes(p: Problem) -> int:
    """Bytes the operator must move once: activations + weights read, output written."""
    es = ELEM_SIZE[p.dtype]
    return es * (int(np.prod(p.a_shape)) + int(np.prod(p.b_shape)) + int(np.prod(p.c_shape)))


# ----------------------------------------------------------------------------
# recipes
# ----------------------------------------------------------------------------

def _gemm(dtype, m, n, k, a_dist, b_dist, deadline=math.inf, tag=""):
    return Problem(op="gemm", dtype=dtype, M=m, N=n, K=k, a_dist=a_dist, b_dist=b_dist,
                   deadline_ms=deadline, tag=tag)


def _conv(dtype, hw, cin, cout, r, deadline=math.inf, tag=""):
    pad = (r - 1) // 2
    he_std = math.sqrt(2.0 / (r * r * cin))
    return Problem(op="conv", dtype=dtype, Nb=1, H=hw, W=hw, Cin=cin, Cout=cout, R=r, S=r,
                   pad_h=pad, pad_w=pad, a_dist=("uniform", 0.0, 1.0), b_dist=("normal", he_std),
                   deadline_ms=deadline, tag=tag)


def _rng(seed: int, *stream) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), *map(int, stream)])))


def _cfg1(seed):
    u = ("uniform", -1.0, 1.0)
    shapes = [(1, 256, 256), (4, 256, 512), (8, 512, 256), (2, 128, 384)]
    return [_gemm("f32", m, n, k, u, u, tag="fp32-gemm") for (m, n, k) in shapes]


def _cfg2(seed):
    g = _rng(seed, 2)
    out = []
    for _ in range(16):
        m = int(g.choice([1, 2, 4, 8, 16, 32]))
        n = int(g.choice([512, 1024, 2048, 4096]))
        k = int(g.choice([512, 1024, 2048, 4096]))
        out.append(_gemm("bf16", m, n, k, ("normal", 1.0), ("normal", 1.0 / math.sqrt(k)), tag="lowbatch-gemm"))
    return out


def _cfg3(seed):
    layers = [(56, 64, 256, 1), (56, 64, 64, 3), (28, 128, 512, 1), (28, 128, 128, 3),
              (14, 256, 1024, 1), (14, 256, 256, 3), (7, 512, 2048, 1), (7, 512, 512, 3)]
    return [_conv("bf16", hw, ci, co, r, tag="resnet50-conv") for (hw, ci, co, r) in layers]


def _cfg4(seed):
    g = _rng(seed, 4)
    # (K, N): three 768x768 projections, FFN-up 768->3072, FFN-down 3072->768
    kinds = [(768, 768), (768, 768), (768, 768), (768, 3072), (3072, 768)]
    out = []
    for _ in range(32):
        L = int(g.integers(1, 129))
        k, n = kinds[int(g.integers(0, 5))]
        out.append(_gemm("bf16", L, n, k, ("normal", 1.0), ("normal", 0.02), tag="bert-linear"))
    return out


def _cfg5(seed):
    g = _rng(seed, 5)
    dims = list(range(256, 8192 + 1, 256))
    out = []
    for _ in range(256):
        is_gemm = g.random() < 0.6
        deadline = float(g.uniform(0.5, 5.0))
        if is_gemm:
            m = int(math.floor(math.exp(g.random() * math.log(64.0)) + 0.5))
            m = max(1, min(64, m))
            n = int(g.choice(dims))
            k = int(g.choice(dims))
            out.append(_gemm("bf16", m, n, k, ("normal", 1.0), ("normal", 1.0 / math.sqrt(k)),
                             deadline=deadline, tag="lowbatch-gemm"))
        else:
            hw = int(g.choice([7, 14, 28, 56]))
            ci = int(g.choice([64, 128, 256, 512]))
            co = int(g.choice([64, 128, 256, 512]))
            r = 3 if g.random() < 0.5 else 1
            out.append(_conv("bf16", hw, ci, co, r, deadline=deadline, tag="conv"))
    return out


def _cfg6(seed):
    # LSTM-cell-shaped matrix-vector products at batch 1 (the second workload the paper's
    # Section 5.3 evaluates): one operator = the four gates of one cell, [x_t ; h_{t-1}] (K = 2h)
    # against the stacked gate weights (N = 4h), fp16.
    g = _rng(seed, 6)
    out = []
    for _ in range(64):
        h = int(g.choice([256, 512, 1024, 2048]))
        out.append(_gemm("f16", 1, 4 * h, 2 * h, ("normal", 1.0), ("normal", 1.0 / math.sqrt(2 * h)), tag="lstm-matvec"))
    return out


def _cfg7(seed):
    # The down-sampling layers of a 50-layer residual network at batch 1 (the paper's Section 5.3
    # serves ResNet-50): the stride-2 7x7 stem on a 224x224 RGB image, and at each of the three stage
    # transitions the stride-2 3x3 convolution of the first block and its stride-2 1x1 projection.
    def strided(hw, cin, cout, r, pad):
        he_std = math.sqrt(2.0 / (r * r * cin))
        return Problem(op="conv", dtype="bf16", Nb=1, H=hw, W=hw, Cin=cin, Cout=cout, R=r, S=r, pad_h=pad, pad_w=pad,
                       stride=2, a_dist=("uniform", 0.0, 1.0), b_dist=("normal", he_std), tag="resnet50-stride2")
    return [strided(224, 3, 64, 7, 3),
            strided(56, 128, 128, 3, 1), strided(56, 256, 512, 1, 0),
            strided(28, 256, 256, 3, 1), strided(28, 512, 1024, 1, 0),
            strided(14, 512, 512, 3, 1), strided(14, 1024, 2048, 1, 0)]


def _cfg8(seed):
    # The experiment behind the paper's headline figures (Section 5.3): the second convolution of the
    # first residual stage of an 18-layer network (3x3, 64 -> 64 channels on a 56x56 image, batch 1),
    # one instance per tenant, every tenant with weights and activations of its own.
    return [_conv("bf16", 56, 64, 64, 3, tag=f"resnet18-conv2_2-tenant{i}") for i in range(32)]


def _cfg9(seed):
    # Not a workload of the paper (its regime is small batches): sixteen square GEMMs far above the ridge
    # of the roofline, the probe for what the LDS-tile class reaches when it is bound by the matrix cores.
    return [_gemm("bf16", 2048, 2048, 2048, ("normal", 1.0), ("normal", 1.0 / math.sqrt(2048.0)), tag="square-gemm")
            for _ in range(16)]


def _cfg10(seed):
    # The one layer of the residual-network mix whose arithmetic intensity lies above the ridge
    # (3x3, 128 -> 128 channels on 28x28), one instance for each of 64 tenants.
    return [_conv("bf16", 28, 128, 128, 3, tag=f"resnet50-conv3x3-28-tenant{i}") for i in range(64)]


_RECIPES = {
    "cfg1_fp32_gemm4": _cfg1,
    "cfg2_bf16_gemm16": _cfg2,
    "cfg3_resnet_conv8": _cfg3,
    "cfg4_bert_linear32": _cfg4,
    "cfg5_mixed256_edf": _cfg5,
    "cfg6_lstm_matvec64": _cfg6,
    "cfg7_resnet_stride2_conv7": _cfg7,
    "cfg8_conv2_2_tenants32": _cfg8,
    "cfg9_square_gemm16": _cfg9,
    "cfg10_conv3x3_28_tenants64": _cfg10,
}


def config_names() -> List[str]:
    return list(_RECIPES)


def config(name_or_index, seed: int = 0, dtype: str | None = None) -> List[Problem]:
    """Problem list for one of the mixes (by name or 1-based index)."""
    if isinstance(name_or_index, int):
        name = config_names()[name_or_index - 1]
    else:
        name = name_or_index
    probs = _RECIPES[name](seed)
    if dtype is not None:
        probs = [replace(p, dtype=dtype) for p in probs]
    return probs


# ----------------------------------------------------------------------------
# draws
# ----------------------------------------------------------------------------

def _draw_np(g: np.random.Generator, dist, shape) -> np.ndarray:
    if dist[0] == "uniform":
        lo, hi = dist[1], dist[2]
        x = g.random(size=shape, dtype=np.float32)
        return (np.float32(lo) + np.float32(hi - lo) * x).astype(np.float32)
    if dist[0] == "normal":
        return (np.float32(dist[1]) * g.standard_normal(size=shape, dtype=np.float32)).astype(np.float32)
    raise ValueError(dist)


def draw_host(p: Problem, seed: int, index: int):
    """fp32 numpy arrays (A_or_X, B_or_W) for problem `index` of a mix."""
    ga = _rng(seed, 1000, index, 0)
    gb = _rng(seed, 1000, index, 1)
    return _draw_np(ga, p.a_dist, p.a_shape), _draw_np(gb, p.b_dist, p.b_shape)


def draw_device(p: Problem, seed: int, index: int, device="cuda"):
    """fp32 torch tensors on `device`, drawn there (for mixes of several GB)."""
    import torch

    def one(dist, shape, which):
        gen = torch.Generator(device=device)
        gen.manual_seed((int(seed) * 1000003 + index) * 2 + which)
        if dist[0] == "uniform":
            x = torch.rand(shape, generator=gen, device=device, dtype=torch.float32)
            return x * (dist[2] - dist[1]) + dist[1]
        if dist[0] == "normal":
            return torch.randn(shape, generator=gen, device=device, dtype=torch.float32) * dist[1]
        raise ValueError(dist)

    return one(p.a_dist, p.a_shape, 0), one(p.b_dist, p.b_shape, 1)
