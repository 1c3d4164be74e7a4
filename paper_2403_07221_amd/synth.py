"""Seeded synthetic inputs for the LookupFFN forward pass.

This module only draws random numbers and rounds them to storage formats; it
holds none of the method's arithmetic.  Both the CPU oracle's tests and the
GPU tests/bench take their inputs from here so that they see identical arrays.

The paper's workload is post-attention RoBERTa activations with trained
tables (Sec. 4, "Evaluation Task"); neither the corpus nor trained weights are
available, so every input is a synthetic stand-in of the same shape:
``x ~ N(0,1)``, ``tables ~ N(0, 0.02^2)``, sign diagonals i.i.d. Rademacher.
With a random rotation of Gaussian input the codes are uniform over the
``2^tau`` rows, i.e. no hot rows -- the worst case for cache reuse.

bf16 arrays are returned as ``uint16`` raw bit patterns (round-to-nearest-even
of the fp32 draw).
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

SEED_BASE = 240307221


@dataclass(frozen=True)
class Workload:
    """Shape of one LookupFFN layer workload (k = number of tables, the paper's h)."""
    name: str
    index: int          # 1..5: which benchmark configuration the seeds belong to
    n_tokens: int
    d: int
    n_rounds: int
    k: int
    tau: int
    d_out: int
    x_dtype: str = "f32"       # "f32" | "bf16" | "f16"
    table_dtype: str = "f32"   # "f32" | "bf16" | "f16"
    n_layers: int = 1
    seed_index: int | None = None  # reuse another configuration's signs/tables seeds

    @property
    def d_pad(self) -> int:
        p = 1
        while p < self.d:
            p <<= 1
        return p

    @property
    def n_proj(self) -> int:
        return -(-self.k * self.tau // self.d_pad)

    @property
    def rows(self) -> int:
        return 1 << self.tau

    def with_tokens(self, n: int) -> "Workload":
        return replace(self, n_tokens=n)


# The five benchmark configurations.
C1 = Workload("C1-tiny-f32", 1, 64, 64, 2, 8, 8, 64)
C2 = Workload("C2-roberta-base-f32", 2, 16384, 768, 3, 96, 8, 768)
C3 = Workload("C3-roberta-base-bf16", 3, 65536, 768, 3, 96, 8, 768, "bf16", "bf16", seed_index=2)
C4 = Workload("C4-roberta-large-f32", 4, 16384, 1024, 3, 128, 10, 1024)
C5 = Workload("C5-latency-12-layers-f32", 5, 8, 768, 3, 96, 8, 768, n_layers=12)
CONFIGS = {1: C1, 2: C2, 3: C3, 4: C4, 5: C5}

# The paper's own layer shapes (Sec. 4): 4-layer RoBERTa with d = 512 and h = 256 / 128 tables of
# 2^8 rows (Tab. "baselines"), and RoBERTa-base with h = 170, tau = 9 (the scaling experiment), each
# at the 32768-token effective batch of the latency study (Sec. 4.3: batch 64 x sequence 512),
# hashed with the three-round sign-diagonal projection of Sec. 3.2, eq. "hadamard".
P6 = Workload("P6-paper-small-h256-f32", 6, 32768, 512, 3, 256, 8, 512)
P7 = Workload("P7-paper-small-h128-f32", 7, 32768, 512, 3, 128, 8, 512)
P8 = Workload("P8-paper-base-h170-tau9-f32", 8, 32768, 768, 3, 170, 9, 768)
CONFIGS.update({6: P6, 7: P7, 8: P8})


def seed_for(config: int, layer: int, what: int) -> int:
    """what: 0 = sign diagonals, 1 = x, 2 = tables, 3 = block-diagonal factors of the BH4 hash, 4 = skewed codes."""
    return SEED_BASE + 1000 * config + 10 * layer + what


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round finite fp32 values to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of raw bf16 bit patterns to fp32."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def make_signs(seed: int, n_proj: int, n_rounds: int, d_pad: int) -> np.ndarray:
    """[P][R][d_pad] int8 Rademacher (+1/-1)."""
    r = _rng(seed).integers(0, 2, size=(n_proj, n_rounds, d_pad), dtype=np.int8)
    return (2 * r - 1).astype(np.int8)


def make_bmats(seed: int, n_proj: int, n_factors: int, d_pad: int, block: int) -> np.ndarray:
    """[P][m][d_pad/block][block][block] float32 block-diagonal factors, entries N(0, 1/block)."""
    b = _rng(seed).standard_normal((n_proj, n_factors, d_pad // block, block, block), dtype=np.float32)
    b *= np.float32(1.0 / np.sqrt(block))
    return b


def make_x(seed: int, n: int, d: int, dtype: str = "f32") -> np.ndarray:
    x = _rng(seed).standard_normal((n, d), dtype=np.float32)
    return to_bf16_bits(x) if dtype == "bf16" else x.astype(np.float16) if dtype == "f16" else x


def make_tables(seed: int, k: int, rows: int, d_out: int, dtype: str = "f32",
                sigma: float = 0.02) -> np.ndarray:
    t = _rng(seed).standard_normal((k, rows, d_out), dtype=np.float32)
    t *= np.float32(sigma)
    return to_bf16_bits(t) if dtype == "bf16" else t.astype(np.float16) if dtype == "f16" else t


def make_zipf_codes(seed: int, n: int, k: int, tau: int, s: float = 1.0) -> np.ndarray:
    """codes[n, k] uint16 with skewed buckets: in every table the rows are ranked by a random permutation
    and drawn with probability proportional to 1 / rank^s (trained hashes fill their buckets unevenly,
    Sec. 3.1; the rotation of Gaussian inputs fills them evenly)."""
    rng = _rng(seed)
    rows = 1 << tau
    p = 1.0 / np.arange(1, rows + 1, dtype=np.float64) ** s
    p /= p.sum()
    codes = np.empty((n, k), dtype=np.uint16)
    for j in range(k):
        perm = rng.permutation(rows).astype(np.uint16)
        codes[:, j] = perm[rng.choice(rows, size=n, p=p)]
    return codes


def make_layer(w: Workload, layer: int = 0, n_tokens: int | None = None, with_x: bool = True,
               with_tables: bool = True):
    """(x, signs, tables) numpy arrays for one layer of workload `w`.

    `n_tokens` overrides the token count (the first n rows of the full draw are
    NOT guaranteed; a shorter draw is simply a shorter stream from the same seed).
    """
    cs = w.seed_index or w.index
    signs = make_signs(seed_for(cs, layer, 0), w.n_proj, w.n_rounds, w.d_pad)
    tables = None
    if with_tables:
        tables = make_tables(seed_for(cs, layer, 2), w.k, w.rows, w.d_out, w.table_dtype)
    x = None
    if with_x:
        n = w.n_tokens if n_tokens is None else n_tokens
        x = make_x(seed_for(w.index, layer, 1), n, w.d, w.x_dtype)
    return x, signs, tables
