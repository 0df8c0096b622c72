"""Seeded synthetic inputs for the QTIP decode + multiply path.

This module holds none of the method's arithmetic: it only names the workload
shapes and draws random buffers.  Both the tests' oracle side and the GPU side
get their inputs from here.

The inputs stand in for RHT-processed Llama layers (weights that the paper
argues are close to i.i.d. Gaussian, hence code streams close to uniformly
random bits); no model weights or datasets are used.

Recipe: numpy.random.Generator(PCG64(240611235 + 1000*config + subcase)),
drawn in this order: code words (uniform uint32), signs_n, signs_m (+1/-1 int8,
P = 1/2), row scale (fp16 of U(0.5, 1.5), only where the workload has one),
LUT (fp16 of N(0,1), shape 512x2 for HYB, 2^14 values for the lookup-only code, 64 for the V = 1
hash code), X (fp16 of N(0,1),
shape B x n).
"""
from dataclasses import dataclass, replace

import numpy as np

CODE_1MAD, CODE_3INST, CODE_HYB, CODE_HYB2, CODE_LUT, CODE_HYB1 = 0, 1, 2, 3, 4, 5
CODE_NAMES = {CODE_1MAD: "1MAD", CODE_3INST: "3INST", CODE_HYB: "HYB", CODE_HYB2: "HYB2", CODE_LUT: "LUT14",
              CODE_HYB1: "HYB1"}
BASE_SEED = 240611235


@dataclass(frozen=True)
class Workload:
    name: str
    config: int      # index into the benchmark's config list (0 = the metric shape)
    subcase: int
    m: int           # outputs
    n: int           # inputs
    code_id: int
    k: int
    V: int
    block_n: int     # Hadamard block on the input side
    block_m: int     # Hadamard block on the output side
    B: int = 1
    row_scale: bool = False
    L: int = 16
    Q: int = 9

    @property
    def seed(self):
        return BASE_SEED + 1000 * self.config + self.subcase

    @property
    def tile(self):
        """(T_x, T_y): the block of the matrix that is one sequence."""
        return (32, 8) if self.code_id == CODE_LUT else (16, 16)

    @property
    def tiles(self):
        return (self.m // self.tile[0]) * (self.n // self.tile[1])

    @property
    def words_per_tile(self):
        return 8 * self.k

    @property
    def code_bytes(self):
        return self.m * self.n * self.k // 8


def _w(name, config, subcase, m, n, code_id, k, V, bn, bm, **kw):
    return Workload(name, config, subcase, m, n, code_id, k, V, bn, bm, **kw)


WORKLOADS = {w.name: w for w in [
    _w("metric_3inst_k2_8192x28672", 0, 0, 8192, 28672, CODE_3INST, 2, 1, 4096, 4096),
    _w("cfg1_3inst_k2_1024x1024", 1, 0, 1024, 1024, CODE_3INST, 2, 1, 1024, 1024,
       row_scale=True),
    _w("cfg2_3inst_k2_4096x4096", 2, 0, 4096, 4096, CODE_3INST, 2, 1, 4096, 4096),
    _w("cfg3_1mad_k2_14336x4096", 3, 0, 14336, 4096, CODE_1MAD, 2, 1, 2048, 2048),
    _w("cfg3_1mad_k3_14336x4096", 3, 1, 14336, 4096, CODE_1MAD, 3, 1, 2048, 2048),
    _w("cfg3_1mad_k4_14336x4096", 3, 2, 14336, 4096, CODE_1MAD, 4, 1, 2048, 2048),
    _w("cfg3_1mad_k2_4096x14336", 3, 3, 4096, 14336, CODE_1MAD, 2, 1, 2048, 2048),
    _w("cfg3_1mad_k3_4096x14336", 3, 4, 4096, 14336, CODE_1MAD, 3, 1, 2048, 2048),
    _w("cfg3_1mad_k4_4096x14336", 3, 5, 4096, 14336, CODE_1MAD, 4, 1, 2048, 2048),
    _w("cfg4_hyb_k2_8192x28672", 4, 0, 8192, 28672, CODE_HYB, 2, 2, 4096, 4096),
    _w("next_hyb2_k2_8192x28672", 6, 0, 8192, 28672, CODE_HYB2, 2, 2, 4096, 4096),
    _w("next_lut14_k2_8192x28672", 7, 0, 8192, 28672, CODE_LUT, 2, 1, 4096, 4096, L=14),
    _w("next_hyb1_k2_8192x28672", 8, 0, 8192, 28672, CODE_HYB1, 2, 1, 4096, 4096, Q=6),
    _w("cfg5_hyb_k4_8192x8192_b1", 5, 0, 8192, 8192, CODE_HYB, 4, 2, 4096, 4096, B=1),
    _w("cfg5_hyb_k4_8192x8192_b4", 5, 1, 8192, 8192, CODE_HYB, 4, 2, 4096, 4096, B=4),
    _w("cfg5_hyb_k4_8192x8192_b16", 5, 2, 8192, 8192, CODE_HYB, 4, 2, 4096, 4096, B=16),
    _w("cfg5_hyb_k4_8192x8192_b64", 5, 3, 8192, 8192, CODE_HYB, 4, 2, 4096, 4096, B=64),
]}


def small(w, m, n, block_n=None, block_m=None, subcase_offset=100):
    """A reduced-size copy of a workload (for parity cases the oracle finishes fast)."""
    bn = block_n or min(w.block_n, n)
    bm = block_m or min(w.block_m, m)
    return replace(w, name=f"{w.name}_small_{m}x{n}", m=m, n=n, block_n=bn, block_m=bm,
                   subcase=w.subcase + subcase_offset)


@dataclass
class Inputs:
    codes: np.ndarray       # uint32, (tiles, 8k)
    signs_n: np.ndarray     # int8 +1/-1, (n,)
    signs_m: np.ndarray     # int8 +1/-1, (m,)
    row_scale: np.ndarray   # float16 (m,) or None
    lut: np.ndarray         # float16 (512, 2), (2^14,), (64,) or None
    X: np.ndarray           # float16 (B, n)


def make_inputs(w, seed=None):
    rng = np.random.Generator(np.random.PCG64(w.seed if seed is None else seed))
    codes = rng.integers(0, 1 << 32, size=(w.tiles, w.words_per_tile), dtype=np.uint64)
    codes = codes.astype(np.uint32)
    signs_n = (rng.integers(0, 2, size=w.n, dtype=np.int8) * 2 - 1).astype(np.int8)
    signs_m = (rng.integers(0, 2, size=w.m, dtype=np.int8) * 2 - 1).astype(np.int8)
    row_scale = None
    if w.row_scale:
        row_scale = rng.uniform(0.5, 1.5, size=w.m).astype(np.float16)
    lut = None
    if w.code_id in (CODE_HYB, CODE_HYB2):
        lut = rng.standard_normal(size=(1 << w.Q, 2)).astype(np.float16)
    elif w.code_id == CODE_LUT:
        lut = rng.standard_normal(size=1 << w.L).astype(np.float16)
    elif w.code_id == CODE_HYB1:
        lut = rng.standard_normal(size=64).astype(np.float16)
    X = rng.standard_normal(size=(w.B, w.n)).astype(np.float16)
    return Inputs(codes, signs_n, signs_m, row_scale, lut, X)
