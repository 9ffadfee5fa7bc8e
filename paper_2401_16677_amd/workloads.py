"""Seeded synthetic inputs for the fused GEMM + reduce-scatter path.

Shapes follow the transformer tensor-parallel sub-layers the T3 paper evaluates
(output projection and FC-2, Sec. 6.1 and Table 2): M tokens, hidden size N,
K = slice width of the row-parallel weight, TP degree P, rank r.  This module
only draws numbers and rounds them to the storage types; it contains none of
the method's arithmetic and is the one module the GPU tests hand to both the
library and the CPU oracle.
"""
from dataclasses import dataclass

import numpy as np

SEED_BASE = 0x54330000


@dataclass(frozen=True)
class Workload:
    name: str
    M: int
    N: int
    K: int
    tp: int
    rank: int
    tile_m: int
    tile_n: int
    a_dist: str = "normal"      # "normal" | "halfnormal" (ReLU-like: half exact zeros)
    index: int = 0

    @property
    def W(self):
        return self.N // self.tp

    @property
    def flop(self):
        return 2.0 * self.M * self.N * self.K

    @property
    def seed(self):
        return SEED_BASE + self.index


# The five configurations, smallest first.
WORKLOADS = {
    "tiny_outproj": Workload("tiny_outproj", 256, 1024, 256, 4, 0, 128, 128, index=0),
    "gpt3_outproj": Workload("gpt3_outproj", 4096, 12288, 1536, 8, 3, 256, 256, index=1),
    "gpt3_fc2": Workload("gpt3_fc2", 4096, 12288, 6144, 8, 5, 256, 256, a_dist="halfnormal",
                         index=2),
    "wide_fc2": Workload("wide_fc2", 2048, 20480, 10240, 8, 7, 128, 256, index=3),
    "hightp_outproj": Workload("hightp_outproj", 8192, 18432, 1152, 16, 9, 256, 256, index=4),
}


# Further shapes: row-parallel sub-layers of the models the paper evaluates (its Table 2: hidden
# size H, tokens = sequence length x batch, TP degree), K = H/TP for the output projection and
# 4H/TP for FC-2.  tile 0 x 0 = the library's default tile for the shape.
PAPER_SHAPES = {
    "megagpt2_fc2_tp8": Workload("megagpt2_fc2_tp8", 16384, 3072, 1536, 8, 2, 0, 0, index=10),
    "megagpt2_outproj_tp16": Workload("megagpt2_outproj_tp16", 16384, 3072, 192, 16, 11, 0, 0, index=11),
    "tnlg_fc2_tp8": Workload("tnlg_fc2_tp8", 8192, 4256, 2128, 8, 6, 0, 0, a_dist="halfnormal", index=12),
    "gpt3_fc2_tp32": Workload("gpt3_fc2_tp32", 2048, 12288, 1536, 32, 17, 0, 0, index=13),
    "palm_outproj_tp32": Workload("palm_outproj_tp32", 2048, 18432, 576, 32, 30, 0, 0, index=14),
    "mtnlg_fc2_tp32": Workload("mtnlg_fc2_tp32", 2048, 20480, 2560, 32, 5, 0, 0, index=15),
}
WORKLOADS.update(PAPER_SHAPES)


def f32_to_bf16_bits(x):
    """Round fp32 to bf16 (round to nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(bits):
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(
        np.float32)


def _rng(seed, stream):
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def std_c(w):
    """Analytic standard deviation of one element of C = A.B for the drawn distributions."""
    return float(np.sqrt(0.5)) if w.a_dist == "halfnormal" else 1.0


def make_inputs(w, seed=None, rows_chunk=1024):
    """Draw A (M,K) and B (N,K) as bf16 bit patterns and incoming (M,N) fp32.

    A, B ~ N(0, sigma^2) with sigma = K^(-1/4), so Var(C) is 1 (1/2 for the
    half-normal A).  incoming ~ N(0, (P-1) Var(C)): the partial a rank receives
    has up to P-1 upstream contributions in it.
    """
    seed = w.seed if seed is None else seed
    sigma = float(w.K) ** -0.25
    a = _rng(seed, 1).standard_normal((w.M, w.K), dtype=np.float32) * np.float32(sigma)
    if w.a_dist == "halfnormal":
        a = np.maximum(a, np.float32(0.0))
    b = _rng(seed, 2).standard_normal((w.N, w.K), dtype=np.float32) * np.float32(sigma)
    inc = np.empty((w.M, w.N), dtype=np.float32)
    g = _rng(seed, 3)
    scale = np.float32(np.sqrt(max(w.tp - 1, 1)) * std_c(w))
    for m0 in range(0, w.M, rows_chunk):
        m1 = min(m0 + rows_chunk, w.M)
        inc[m0:m1] = g.standard_normal((m1 - m0, w.N), dtype=np.float32) * scale
    return f32_to_bf16_bits(a), f32_to_bf16_bits(b), inc


def make_integer_inputs(M, N, K, seed, amax=2, incmax=1000):
    """Small-integer inputs: every partial sum stays below 2^24, so fp32 accumulation in any
    order is exact and the GPU result must equal the fp64 oracle bit for bit."""
    assert K * amax * amax + incmax < (1 << 24)
    a = _rng(seed, 11).integers(-amax, amax + 1, size=(M, K)).astype(np.float32)
    b = _rng(seed, 12).integers(-amax, amax + 1, size=(N, K)).astype(np.float32)
    inc = _rng(seed, 13).integers(-incmax, incmax + 1, size=(M, N)).astype(np.float32)
    return f32_to_bf16_bits(a), f32_to_bf16_bits(b), inc


def make_shape(name, M, N, K, tp, rank, tile_m, tile_n, a_dist="normal", index=99):
    return Workload(name, M, N, K, tp, rank, tile_m, tile_n, a_dist, index)
