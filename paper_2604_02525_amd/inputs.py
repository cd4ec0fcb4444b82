"""Seeded synthetic inputs shaped like the paper's LLM training tensors.

This module only draws random numbers and lays them out; it holds none of the method's arithmetic
(no transform, no quantisation, no selection) so that the CPU oracle and the GPU library can both be
fed from it without sharing anything else.

The paper's tensors come from C4-trained models and are not available; these stand in for them with
the structure the paper reports (Sec. 3.1, App. D): activations carry a few large input channels
(column-wise outliers), output gradients carry a few large token rows (row-wise outliers), weights
are featureless Gaussians.  Values are drawn in fp32 with torch's CPU generator, scaled, and rounded
to bf16 (round-to-nearest-even); the bf16 bit patterns are what both sides consume.

A GEMM operand is described the way the library's boundary does: a logical [outer, K] matrix plus a
flag saying whether K is the contiguous axis of the stored array (Eq. 1-3 of the paper give all
three combinations).
"""
from dataclasses import dataclass
import math

import numpy as np
import torch

NONE, IHT, IHT_OE_ROW, IHT_OE_COL, IHT_OE_K, OHT = range(6)
STRATEGY_NAMES = {NONE: "none", IHT: "iht", IHT_OE_ROW: "iht+oe-row", IHT_OE_COL: "iht+oe-col", IHT_OE_K: "iht+oe-k",
                  OHT: "oht"}


@dataclass
class Operand:
    bits: np.ndarray      # uint16 bf16 bit patterns, [outer, K] if k_contig else [K, outer]
    k_contig: bool

    @property
    def outer(self):
        return self.bits.shape[0] if self.k_contig else self.bits.shape[1]

    @property
    def K(self):
        return self.bits.shape[1] if self.k_contig else self.bits.shape[0]


@dataclass
class Gemm:
    name: str
    A: Operand            # logical [M, K]
    B: Operand            # logical [N, K]  (C = A B^T in this notation, C = A*B in the paper's)
    strategy: int
    iht_block: int
    k: int

    @property
    def shape(self):
        return self.A.outer, self.B.outer, self.A.K


def matrix(rows, cols, std, seed, row_outliers=None, col_outliers=None):
    """[rows, cols] bf16 bits of N(0, std^2) with optional amplified rows / columns.

    row_outliers / col_outliers = (count, lo, hi): `count` distinct indices chosen by a seeded
    permutation, each multiplied by one factor drawn uniformly from [lo, hi] (lo == hi: fixed).
    Scaling is applied in fp32 before the rounding to bf16.
    """
    g = torch.Generator().manual_seed(int(seed))
    x = torch.randn(rows, cols, generator=g, dtype=torch.float32)
    if std != 1.0:
        x.mul_(std)
    for spec, n, axis in ((row_outliers, rows, 0), (col_outliers, cols, 1)):
        if not spec:
            continue
        count, lo, hi = spec
        idx = torch.randperm(n, generator=g)[:count]
        fac = lo + (hi - lo) * torch.rand(count, generator=g, dtype=torch.float32)
        if axis == 0:
            x[idx, :] *= fac[:, None]
        else:
            x[:, idx] *= fac[None, :]
    return x.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def pct(p, dim):
    """k = ceil(p % of dim)."""
    return int(math.ceil(p * dim / 100.0 - 1e-9))


def config0():
    """M=N=K=256, seed 0: A ~ N(0,1) with 4 K-channels x50, B ~ N(0,0.02); IHT block 32; OE off."""
    A = Operand(matrix(256, 256, 1.0, 0, col_outliers=(4, 50.0, 50.0)), True)
    B = Operand(matrix(256, 256, 0.02, 1), True)
    return [Gemm("cfg0", A, B, IHT, 32, 0)]


def config1(strategy=IHT, k=0):
    """Forward MLP up-projection Y = X W^T: X 8192x2048 with 8 channels x U(20,100), W 8192x2048."""
    X = Operand(matrix(8192, 2048, 1.0, 1000, col_outliers=(8, 20.0, 100.0)), True)
    W = Operand(matrix(8192, 2048, 0.02, 1001), True)
    return [Gemm("cfg1.fwd", X, W, strategy, 128, k)]


def config2():
    """A 8192x4096 with 1% rows x100; B stored [K=4096, N=4096] with 1% N-columns x30; OE-row k=82."""
    A = Operand(matrix(8192, 4096, 1.0, 2000, row_outliers=(pct(1, 8192), 100.0, 100.0)), True)
    B = Operand(matrix(4096, 4096, 0.02, 2001, col_outliers=(pct(1, 4096), 30.0, 30.0)), False)
    return [Gemm("cfg2", A, B, IHT_OE_ROW, 128, pct(1, 8192))]


def linear_layer_gemms(prefix, T, d_in, d_out, seed, iht_block, strategies, k_pct, n_channels=16):
    """fwd / dgrad / wgrad of one linear layer (Eq. 1-3) on shared X [T,d_in], W [d_out,d_in], G_Y [T,d_out].

    X: N(0,1) with n_channels input channels x50; G_Y: N(0,1)*1e-3 with ceil(0.5% T) token rows
    x100; W: N(0, 0.02).  strategies = (fwd, dgrad, wgrad); k = ceil(k_pct % of the extracted dim).
    """
    X = matrix(T, d_in, 1.0, seed, col_outliers=(n_channels, 50.0, 50.0))
    W = matrix(d_out, d_in, 0.02, seed + 1)
    G = matrix(T, d_out, 1e-3, seed + 2, row_outliers=(pct(0.5, T), 100.0, 100.0))
    triples = (
        ("fwd", Operand(X, True), Operand(W, True)),          # Y   = X W^T     : M=T,     N=d_out, K=d_in
        ("dgrad", Operand(G, True), Operand(W, False)),       # G_X = G_Y W     : M=T,     N=d_in,  K=d_out
        ("wgrad", Operand(G, False), Operand(X, False)),      # G_W = G_Y^T X   : M=d_out, N=d_in,  K=T
    )
    out = []
    for (kind, A, B), s in zip(triples, strategies):
        dim = {IHT_OE_ROW: A.outer, IHT_OE_COL: B.outer, IHT_OE_K: A.K}.get(s, 0)
        out.append(Gemm(f"{prefix}.{kind}", A, B, s, iht_block, pct(k_pct, dim) if dim else 0))
    return out


# LLaMA-7B-shaped decoder layer, 8192 tokens: (name, d_in, d_out)
CFG3_LINEARS = (("qkv", 4096, 12288), ("o", 4096, 4096), ("gate", 4096, 11008), ("up", 4096, 11008),
                ("down", 11008, 4096))


def config3_strategy_table():
    """The fixed seeded per-GEMM strategy table: 5 linears x (fwd, dgrad, wgrad)."""
    rng = np.random.default_rng(3000)
    return rng.integers(IHT, IHT_OE_K + 1, size=(len(CFG3_LINEARS), 3))


def config3(linears=None, T=8192):
    table = config3_strategy_table()
    out = []
    for li, (name, d_in, d_out) in enumerate(CFG3_LINEARS):
        if linears is not None and name not in linears:
            continue
        out += linear_layer_gemms(f"cfg3.{name}", T, d_in, d_out, 3000 + 10 * li, 128,
                                  tuple(int(s) for s in table[li]), 1.0)
    return out


def config4(which=("up", "down"), strategies=(IHT, IHT, IHT), k_pct=0.0, T=16384, hidden=8192, ffn=28672):
    """Stress shapes: up 8192->28672 and down 28672->8192 at 16384 tokens, IHT block 256."""
    out = []
    if "up" in which:
        out += linear_layer_gemms("cfg4.up", T, hidden, ffn, 4000, 256, strategies, k_pct)
    if "down" in which:
        out += linear_layer_gemms("cfg4.down", T, ffn, hidden, 4010, 256, strategies, k_pct)
    return out


def paper_latency_shapes(which=("mlp", "attn"), T=32768, iht_block=32, k=64):
    """The two GEMMs of the paper's kernel latency table (Table 3, right; App. F): (m, n, k) =
    (14336, 4096, 32768) "MLP projection" and (4096, 4096, 32768) "attention projection" of Llama3.1-8B at
    8 x 4096 tokens, i.e. the weight-gradient products G_W = G_Y^T X (Eq. 3) with the tokens as the
    contraction axis, both operands stored token-major.  Same stand-in tensors as the configs: G_Y with
    0.5 % token rows x100, X with 16 channels x50.  The paper's settings: IHT block 32, extraction rank 64;
    the amplified channels of X are columns of B, which the paper's table routes to OE-Right (OE-col).
    """
    out = []
    for name, d_out, seed in (("mlp", 14336, 5000), ("attn", 4096, 5010)):
        if name not in which:
            continue
        X = matrix(T, 4096, 1.0, seed, col_outliers=(16, 50.0, 50.0))
        G = matrix(T, d_out, 1e-3, seed + 2, row_outliers=(pct(0.5, T), 100.0, 100.0))
        out.append(Gemm(f"table3.{name}.wgrad", Operand(G, False), Operand(X, False), IHT_OE_COL, iht_block, k))
    return out


# ---- the paper's synthetic error studies (Sec. 3.2 / Fig. 2 left, App. D; App. G right) ----------------------------
QUALITY_SEEDS = (42, 256, 1925, 2048, 7777)
# The paper amplifies "random columns" by 25 (Column-wise) or 5 (Row-wise) and reports the resulting mean kurtosis,
# 208.30 and 9.08, but not how many columns.  For a 4096-wide Gaussian tensor with n of its columns scaled by f the
# kurtosis is 3 (1 + p (f^4 - 1)) / (1 + p (f^2 - 1))^2 with p = n / 4096: n = 45 gives 208.7 for f = 25 and n = 18
# gives 9.1 for f = 5, so these counts reproduce the statistics the paper states.
QUALITY_COUNT = {"C": 45, "R": 18}
QUALITY_FACTOR = {"C": 25.0, "R": 5.0}


def pattern_operand(kind, outer, K, seed, as_b):
    """Logical [outer, K] bf16 bits of a tensor with the paper's pattern letter (App. D).
    A (m x k, passed as [m, k]):  R = amplified rows,                 C = amplified columns = K-channels.
    B (k x n, passed as [n, k]):  R = amplified rows  = K-channels,   C = amplified columns = outer rows.
    Row-wise tensors are Column-wise tensors transposed (App. G): x5 on 18 lines; Column-wise: x25 on 45 lines."""
    if kind == "N":
        return matrix(outer, K, 1.0, seed)
    spec = (QUALITY_COUNT[kind], QUALITY_FACTOR[kind], QUALITY_FACTOR[kind])
    rows_amplified = (kind == "R") != as_b
    return matrix(outer, K, 1.0, seed, row_outliers=spec) if rows_amplified else matrix(outer, K, 1.0, seed, col_outliers=spec)
