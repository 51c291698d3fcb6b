"""Seeded synthetic inputs for the operator workloads.

This module holds shapes and random draws only: none of the operators'
arithmetic.  It is the one module that both the tests of the CPU oracle and
the callers of the HIP path use, so that both see identical fp32 values.

The workloads stand in for the single-operator and subgraph benchmarks of
arXiv 2006.06762 (Sec. 7.1, Sec. 7.2, shape lists in Appendix C): dense fp32
tensors with i.i.d. entries, no sparsity, batch 16 (or 1).  Values are drawn in
float64 from numpy's PCG64 generator and rounded to float32 once.
"""
from dataclasses import dataclass, field
from typing import Dict, Tuple

import numpy as np

SEED_BASE = 2006067620


@dataclass(frozen=True)
class ConvShape:
    N: int
    C: int
    H: int
    W: int
    K: int          # output channels (== C for depthwise)
    R: int
    S: int
    stride: Tuple[int, int] = (1, 1)
    pad: Tuple[int, int] = (0, 0)
    dil: Tuple[int, int] = (1, 1)
    groups: int = 1

    @property
    def OH(self) -> int:
        return (self.H + 2 * self.pad[0] - self.dil[0] * (self.R - 1) - 1) // self.stride[0] + 1

    @property
    def OW(self) -> int:
        return (self.W + 2 * self.pad[1] - self.dil[1] * (self.S - 1) - 1) // self.stride[1] + 1


@dataclass(frozen=True)
class GemmShape:
    M: int
    N: int
    K: int
    batch: int = 1


@dataclass(frozen=True)
class TbgShape:
    B: int
    S: int
    H: int
    D: int


# The six calls of one benchmark step, in order.  Names follow the paper's
# operator abbreviations; "C2D_S2" is the stride-2 convolution that follows DEP.
GMM = GemmShape(512, 512, 512)
C2D = ConvShape(16, 64, 56, 56, 64, 3, 3, (1, 1), (1, 1))
CONVLAYER = ConvShape(16, 128, 28, 28, 128, 3, 3, (1, 1), (1, 1))
TBG = TbgShape(16, 128, 12, 64)
DEP = ConvShape(16, 256, 28, 28, 256, 3, 3, (1, 1), (1, 1))
C2D_S2 = ConvShape(16, 256, 28, 28, 512, 3, 3, (2, 2), (1, 1))

BN_EPS = 1e-5

# Shape lists of the single-operator and subgraph benchmarks (Appendix C), each run at
# batch 1 and 16 (Sec. 7.1).  Field order as in the appendix:
#   C2D, ConvLayer: height, width, in_channels, out_channels, kernel, stride, padding
#   GMM: N, M, K        DEP: height, width, channels, kernel, stride, padding
#   TBS: sequence_length, heads, hidden_dimension (per head)
#   GRP: as C2D plus groups        DIL: as C2D plus dilation        NRM: N, M
# The first GRP record has 3 input channels and 4 groups; it is kept as printed and skipped
# wherever shapes are built (the channel count is not a multiple of the group count).
APPENDIX_C = {
    "C2D": [(224, 224, 3, 64, 7, 2, 3), (56, 56, 64, 64, 1, 1, 0), (14, 14, 256, 256, 3, 1, 1),
            (7, 7, 512, 512, 3, 1, 1)],
    "GMM": [(128, 128, 128), (512, 32, 512), (512, 512, 512), (1024, 1024, 1024)],
    "DEP": [(112, 112, 32, 3, 1, 1), (112, 112, 64, 3, 2, 1), (14, 14, 512, 3, 2, 1),
            (7, 7, 1024, 3, 1, 1)],
    "ConvLayer": [(224, 224, 3, 64, 7, 2, 3), (56, 56, 64, 64, 3, 2, 1), (28, 28, 128, 256, 1, 2, 0),
                  (7, 7, 512, 512, 3, 1, 1)],
    "TBS": [(128, 12, 64), (128, 16, 64), (64, 12, 128), (128, 12, 128)],
    "GRP": [(224, 224, 3, 64, 7, 2, 3, 4), (56, 56, 64, 64, 1, 1, 0, 4), (14, 14, 256, 256, 3, 1, 1, 4),
            (7, 7, 512, 512, 3, 1, 1, 4)],
    "NRM": [(256, 256), (512, 512), (1024, 1024), (4096, 4096)],
    "DIL": [(224, 224, 3, 64, 7, 2, 3, 2), (56, 56, 64, 64, 1, 1, 0, 2), (14, 14, 256, 256, 3, 1, 1, 2),
            (7, 7, 512, 512, 3, 1, 1, 2)],
}
BATCHES = (1, 16)


def appendix_shape(op: str, fields, batch: int):
    """The shape object of one Appendix C record at the given batch size (None for a record that
    cannot be built: channels not a multiple of the group count)."""
    if op in ("C2D", "ConvLayer"):
        h, w, ci, co, ks, st, pd = fields
        return ConvShape(batch, ci, h, w, co, ks, ks, (st, st), (pd, pd))
    if op == "GRP":
        h, w, ci, co, ks, st, pd, groups = fields
        if ci % groups or co % groups:
            return None
        return ConvShape(batch, ci, h, w, co, ks, ks, (st, st), (pd, pd), (1, 1), groups)
    if op == "DIL":
        h, w, ci, co, ks, st, pd, dil = fields
        return ConvShape(batch, ci, h, w, co, ks, ks, (st, st), (pd, pd), (dil, dil), 1)
    if op == "DEP":
        h, w, c, ks, st, pd = fields
        return ConvShape(batch, c, h, w, c, ks, ks, (st, st), (pd, pd))
    if op == "GMM":
        n, m, k = fields
        return GemmShape(m, n, k, batch)
    if op == "TBS":
        s, h, d = fields
        return TbgShape(batch, s, h, d)
    raise KeyError(op)

CONFIG_SEEDS: Dict[str, int] = {
    "GMM": SEED_BASE + 1,
    "C2D": SEED_BASE + 2,
    "ConvLayer": SEED_BASE + 3,
    "TBG": SEED_BASE + 4,
    "DEP": SEED_BASE + 5,
    "C2D_S2": SEED_BASE + 6,
}


def _rng(seed) -> np.random.Generator:
    """A fresh PCG64 generator for an int seed; an existing generator is passed through
    (so that one config can draw all its tensors from one stream, in a fixed order)."""
    if isinstance(seed, np.random.Generator):
        return seed
    return np.random.Generator(np.random.PCG64(seed))


def uniform(rng, shape, lo=-1.0, hi=1.0) -> np.ndarray:
    return rng.uniform(lo, hi, size=shape).astype(np.float32)


def normal(rng, shape, sigma=1.0, mu=0.0) -> np.ndarray:
    return (mu + sigma * rng.standard_normal(size=shape)).astype(np.float32)


def small_ints(rng, shape, lo=-3, hi=3) -> np.ndarray:
    """Integer-valued fp32 in [lo, hi]: every partial sum of products stays
    exactly representable in fp32, so any summation order gives the same bits."""
    return rng.integers(lo, hi + 1, size=shape).astype(np.float32)


def gemm_inputs(shape: GemmShape, seed, ints: bool = False):
    """A [batch,M,K], B [batch,K,N] ~ U[-1,1] (batch axis dropped when batch == 1)."""
    rng = _rng(seed)
    draw = small_ints if ints else uniform
    a_shape = (shape.batch, shape.M, shape.K) if shape.batch > 1 else (shape.M, shape.K)
    b_shape = (shape.batch, shape.K, shape.N) if shape.batch > 1 else (shape.K, shape.N)
    A = draw(rng, a_shape)
    B = draw(rng, b_shape)
    return A, B


def conv_inputs(shape: ConvShape, seed, ints: bool = False):
    """x [N,C,H,W] ~ U[-1,1]; w [K,C/groups,R,S] ~ N(0, 0.05^2)."""
    rng = _rng(seed)
    cg = shape.C // shape.groups
    if ints:
        x = small_ints(rng, (shape.N, shape.C, shape.H, shape.W))
        w = small_ints(rng, (shape.K, cg, shape.R, shape.S))
    else:
        x = uniform(rng, (shape.N, shape.C, shape.H, shape.W))
        w = normal(rng, (shape.K, cg, shape.R, shape.S), 0.05)
    return x, w


def bn_inputs(K: int, seed):
    """gamma ~ U[0.5,1.5], beta ~ U[-0.1,0.1], mean ~ N(0,0.1^2), var ~ U[0.5,2]."""
    rng = _rng(seed)
    gamma = uniform(rng, (K,), 0.5, 1.5)
    beta = uniform(rng, (K,), -0.1, 0.1)
    mean = normal(rng, (K,), 0.1)
    var = uniform(rng, (K,), 0.5, 2.0)
    return gamma, beta, mean, var


def dwconv_inputs(shape: ConvShape, seed, ints: bool = False):
    """x [N,C,H,W] ~ U[-1,1]; w [C,1,R,S] ~ N(0, 0.05^2)."""
    rng = _rng(seed)
    if ints:
        x = small_ints(rng, (shape.N, shape.C, shape.H, shape.W))
        w = small_ints(rng, (shape.C, 1, shape.R, shape.S))
    else:
        x = uniform(rng, (shape.N, shape.C, shape.H, shape.W))
        w = normal(rng, (shape.C, 1, shape.R, shape.S), 0.05)
    return x, w


def tbg_inputs(shape: TbgShape, seed, ints: bool = False):
    """q, k [B,S,H,D] ~ N(0,1)."""
    rng = _rng(seed)
    dims = (shape.B, shape.S, shape.H, shape.D)
    if ints:
        return small_ints(rng, dims), small_ints(rng, dims)
    return normal(rng, dims), normal(rng, dims)


def config_inputs(name: str):
    """The seeded tensors of one named benchmark config, as a dict."""
    seed = CONFIG_SEEDS[name]
    if name == "GMM":
        A, B = gemm_inputs(GMM, seed)
        return {"shape": GMM, "A": A, "B": B}
    if name == "C2D":
        x, w = conv_inputs(C2D, seed)
        return {"shape": C2D, "x": x, "w": w}
    if name == "ConvLayer":
        rng = _rng(seed)        # one stream: x, w, gamma, beta, mean, var in this order
        x, w = conv_inputs(CONVLAYER, rng)
        gamma, beta, mean, var = bn_inputs(CONVLAYER.K, rng)
        return {"shape": CONVLAYER, "x": x, "w": w, "gamma": gamma, "beta": beta,
                "mean": mean, "var": var, "eps": BN_EPS}
    if name == "TBG":
        q, k = tbg_inputs(TBG, seed)
        return {"shape": TBG, "q": q, "k": k}
    if name == "DEP":
        x, w = dwconv_inputs(DEP, seed)
        return {"shape": DEP, "x": x, "w": w}
    if name == "C2D_S2":
        x, w = conv_inputs(C2D_S2, seed)
        return {"shape": C2D_S2, "x": x, "w": w}
    raise KeyError(name)


CONFIG_NAMES = ("GMM", "C2D", "ConvLayer", "TBG", "DEP", "C2D_S2")
