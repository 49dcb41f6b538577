"""Seeded synthetic SpQR inputs (logical form) for tests and the benchmark.

This module only draws random numbers and arranges them into the logical parts
of the SpQR representation (Sec. 4.2 of the paper): code matrix, first-level
statistic codes, second-level fp16 statistics and a CSR outlier set.  It holds
none of the method's arithmetic: no dequantisation, no products, no packing.
Both the CPU oracle and the HIP path consume what it returns.

Geometry (notation of App. B of the paper: b_w, beta1, beta2):

  group_axis = 0   a first-level group is beta1 consecutive input columns of
                   one output row (Alg. 1: column blocks of width beta1);
                   a tile is beta2 rows x beta1 columns.
  group_axis = 1   a first-level group is beta1 consecutive output rows of one
                   input column; a tile is beta1 rows x beta2 columns.

  Q    uint8   [m, n]                      codes in [0, 2^b_w)
  s_q  uint8   [m, n/beta1] (axis 0)  or  [m/beta1, n] (axis 1)   3-bit codes
  z_q  uint8   same shape as s_q
  s_s, z_s, s_z, z_z  float16 [tile_rows_count, tile_cols_count]  one per tile
  row_ptr int32 [m+1] exclusive prefix; col_idx uint16 [nnz]; val float16 [nnz]

Variants of the statistics (Sec. 5, ablations), selected by `stat_layout`:
  "bilevel"     as above (the method's own format);
  "round_zero"  the zero-point code z_q is the zero-point itself (an integer):
                there is no s_z, z_z (both None);
  "stats16"     first-level statistics kept in 16 bit: s16, z16 float16 arrays of
                the shape of s_q, no codes and no second level (all None).

Recipe (all draws in float64, rounded to float16 where the format stores
float16; the rounded values are the ground truth for both sides):
  codes iid uniform over [0, 2^b_w); s_q, z_q iid uniform over [0, 8);
  s_s, s_z ~ U[0.01, 0.05), z_s, z_z ~ U[2, 5); outlier values ~ N(0, 0.2^2);
  x ~ N(0, 1).  Draw order: codes, s_q, z_q, s_s, z_s, s_z, z_z, outlier
  positions, outlier values.  x is drawn from its own stream.
  "round_zero" makes the same draws and drops s_z, z_z.  "stats16" draws, in
  place of the six statistic arrays, s16 ~ U[0.02, 0.2) and z16 ~ U[0, 2^b_w - 1).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

__all__ = [
    "SpQRLogical", "tile_shape", "make_matrix", "make_x", "outlier_positions",
    "LayerSpec", "CONFIGS", "config_layers", "make_config_layer", "make_quantizer_problem",
]


@dataclass
class SpQRLogical:
    """Logical (unpacked) SpQR representation of one weight matrix W[m, n]."""
    m: int
    n: int
    w_bits: int
    s_bits: int
    z_bits: int
    beta1: int
    beta2: int
    group_axis: int
    Q: np.ndarray
    s_q: np.ndarray
    z_q: np.ndarray
    s_s: np.ndarray
    z_s: np.ndarray
    s_z: np.ndarray
    z_z: np.ndarray
    row_ptr: np.ndarray
    col_idx: np.ndarray
    val: np.ndarray
    perm: Optional[np.ndarray] = None   # optional input permutation (int32[n])
    stat_layout: str = "bilevel"
    s16: Optional[np.ndarray] = None    # "stats16" only
    z16: Optional[np.ndarray] = None

    @property
    def nnz(self) -> int:
        return int(self.col_idx.shape[0])


def tile_shape(beta1: int, beta2: int, group_axis: int) -> Tuple[int, int]:
    """(rows, cols) of one second-level tile."""
    return (beta2, beta1) if group_axis == 0 else (beta1, beta2)


def _rng(*key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(list(key))))


def _uniform_distinct(rng: np.random.Generator, universe: int, k: int) -> np.ndarray:
    """k distinct integers in [0, universe), uniform, in draw order."""
    if k <= 0:
        return np.zeros(0, dtype=np.int64)
    if k > universe:
        raise ValueError("more outliers than positions")
    if universe <= 4 * k or universe < 4096:
        return rng.permutation(universe)[:k].astype(np.int64)
    got = np.zeros(0, dtype=np.int64)
    while got.shape[0] < k:
        need = k - got.shape[0]
        draw = rng.integers(0, universe, size=int(need * 1.1) + 64, dtype=np.int64)
        allv = np.concatenate([got, draw])
        _, first = np.unique(allv, return_index=True)
        got = allv[np.sort(first)]
    return got[:k]


def outlier_positions(rng: np.random.Generator, m: int, n: int, rate: float,
                      structure: str) -> np.ndarray:
    """Sorted flat positions (row*n + col) of the outliers.

    structure:
      "uniform"        uniform without replacement over all positions
      "rows8cols4"     8 random full rows + 4 random full columns, the rest of
                       the budget uniform over the complement
      "cols64"         64 random full columns + uniform remainder
      "zipf"           per-row counts follow Zipf(s=1.2) over a random row
                       order, each capped at n with the excess handed down to
                       the following rows; columns uniform inside a row
      "none"           no outliers
    """
    total = int(round(rate * m * n))
    if structure == "none" or total == 0:
        return np.zeros(0, dtype=np.int64)
    if structure == "uniform":
        return np.sort(_uniform_distinct(rng, m * n, total))
    if structure in ("rows8cols4", "cols64"):
        n_rows, n_cols = (8, 4) if structure == "rows8cols4" else (0, 64)
        n_rows, n_cols = min(n_rows, m), min(n_cols, n)
        rows = np.sort(rng.permutation(m)[:n_rows]) if n_rows else np.zeros(0, np.int64)
        cols = np.sort(rng.permutation(n)[:n_cols]) if n_cols else np.zeros(0, np.int64)
        mask_r = np.zeros(m, dtype=bool); mask_r[rows] = True
        mask_c = np.zeros(n, dtype=bool); mask_c[cols] = True
        parts = []
        if n_rows:
            parts.append((rows[:, None] * n + np.arange(n)[None, :]).ravel())
        if n_cols:
            free_rows = np.nonzero(~mask_r)[0]
            parts.append((free_rows[:, None] * n + cols[None, :]).ravel())
        structured = np.concatenate(parts).astype(np.int64)
        rest = total - structured.shape[0]
        if rest > 0:
            # uniform over the complement: rejection on the structured lines
            got = np.zeros(0, dtype=np.int64)
            while got.shape[0] < rest:
                need = rest - got.shape[0]
                draw = rng.integers(0, m * n, size=int(need * 1.15) + 64, dtype=np.int64)
                keep = ~(mask_r[draw // n] | mask_c[draw % n])
                allv = np.concatenate([got, draw[keep]])
                _, first = np.unique(allv, return_index=True)
                got = allv[np.sort(first)]
            structured = np.concatenate([structured, got[:rest]])
        return np.sort(structured)
    if structure == "zipf":
        order = rng.permutation(m)
        weights = np.arange(1, m + 1, dtype=np.float64) ** -1.2
        tail = np.cumsum(weights[::-1])[::-1]          # sum_{j>=k} j^-s
        counts = np.zeros(m, dtype=np.int64)
        remaining = total
        for k in range(m):
            c = int(round(remaining * weights[k] / tail[k])) if remaining > 0 else 0
            c = max(0, min(n, c, remaining))
            counts[k] = c
            remaining -= c
        parts = []
        for k in range(m):
            c = int(counts[k])
            if c == 0:
                continue
            r = int(order[k])
            if c == n:
                cols = np.arange(n, dtype=np.int64)
            else:
                cols = _uniform_distinct(rng, n, c)
            parts.append(r * n + cols)
        if not parts:
            return np.zeros(0, dtype=np.int64)
        return np.sort(np.concatenate(parts))
    raise ValueError(f"unknown outlier structure {structure!r}")


def make_matrix(m: int, n: int, *, w_bits: int = 3, beta1: int = 16, beta2: int = 16,
                group_axis: int = 1, outlier_rate: float = 0.01,
                outlier_structure: str = "uniform", seed=(0,),
                s_bits: int = 3, z_bits: int = 3, stat_layout: str = "bilevel") -> SpQRLogical:
    """Draw one logical SpQR matrix following the recipe in the module header."""
    tr, tc = tile_shape(beta1, beta2, group_axis)
    if m % tr or n % tc:
        raise ValueError(f"shape {m}x{n} is not a multiple of the {tr}x{tc} tile")
    if n > 65536:
        raise ValueError("16-bit column indices need n <= 65536")
    key = tuple(int(s) for s in (seed if isinstance(seed, (tuple, list)) else (seed,)))
    rng = _rng(*key)
    Q = rng.integers(0, 1 << w_bits, size=(m, n), dtype=np.uint8)
    gshape = (m, n // beta1) if group_axis == 0 else (m // beta1, n)
    if stat_layout not in ("bilevel", "round_zero", "stats16"):
        raise ValueError(f"unknown statistic layout {stat_layout!r}")
    s16 = z16 = None
    if stat_layout == "stats16":
        s_q = z_q = s_s = z_s = s_z = z_z = None
        s16 = rng.uniform(0.02, 0.2, size=gshape).astype(np.float16)
        z16 = rng.uniform(0.0, (1 << w_bits) - 1, size=gshape).astype(np.float16)
        s_bits = z_bits = 16
    else:
        s_q = rng.integers(0, 1 << s_bits, size=gshape, dtype=np.uint8)
        z_q = rng.integers(0, 1 << z_bits, size=gshape, dtype=np.uint8)
        tshape = (m // tr, n // tc)
        s_s = rng.uniform(0.01, 0.05, size=tshape).astype(np.float16)
        z_s = rng.uniform(2.0, 5.0, size=tshape).astype(np.float16)
        s_z = rng.uniform(0.01, 0.05, size=tshape).astype(np.float16)
        z_z = rng.uniform(2.0, 5.0, size=tshape).astype(np.float16)
        if stat_layout == "round_zero":
            s_z = z_z = None
    pos = outlier_positions(rng, m, n, outlier_rate, outlier_structure)
    rows = pos // n
    col_idx = (pos % n).astype(np.uint16)
    row_ptr = np.zeros(m + 1, dtype=np.int64)
    np.add.at(row_ptr, rows + 1, 1)
    row_ptr = np.cumsum(row_ptr).astype(np.int32)
    val = (0.2 * rng.standard_normal(pos.shape[0])).astype(np.float16)
    return SpQRLogical(m, n, w_bits, s_bits, z_bits, beta1, beta2, group_axis,
                       Q, s_q, z_q, s_s, z_s, s_z, z_z, row_ptr, col_idx, val,
                       stat_layout=stat_layout, s16=s16, z16=z16)


def make_x(n: int, batch: int = 1, seed=(0,)) -> np.ndarray:
    """Activations X[batch, n], N(0,1) rounded to float16."""
    key = tuple(int(s) for s in (seed if isinstance(seed, (tuple, list)) else (seed,)))
    rng = _rng(*key, 0x78)
    return rng.standard_normal((batch, n)).astype(np.float16)


# ----------------------------------------------------------------------------
# The five benchmark configurations (LLaMA-shaped layers; shapes are public
# architecture facts: hidden/MLP = 4096/11008, 6656/17920, 8192/22016).
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class LayerSpec:
    name: str
    m: int
    n: int
    w_bits: int
    beta1: int
    beta2: int
    outlier_rate: float
    outlier_structure: str
    batches: Tuple[int, ...] = (1,)


def _block(h: int, f: int, **kw) -> List[LayerSpec]:
    return ([LayerSpec(nm, h, h, **kw) for nm in ("q", "k", "v", "o")]
            + [LayerSpec("gate", f, h, **kw), LayerSpec("up", f, h, **kw),
               LayerSpec("down", h, f, **kw)])


CONFIGS: Dict[int, List[LayerSpec]] = {
    0: [LayerSpec("linear4096", 4096, 4096, 3, 16, 16, 0.01, "uniform")],
    1: [LayerSpec("mlp_up", 11008, 4096, 3, 16, 16, 0.005, "rows8cols4"),
        LayerSpec("mlp_down", 4096, 11008, 3, 16, 16, 0.005, "rows8cols4")],
    2: _block(4096, 11008, w_bits=3, beta1=16, beta2=16, outlier_rate=0.01,
              outlier_structure="rows8cols4"),
    3: _block(6656, 17920, w_bits=4, beta1=16, beta2=16, outlier_rate=0.01,
              outlier_structure="zipf", batches=(1, 2, 4, 8, 16)),
    4: _block(8192, 22016, w_bits=3, beta1=8, beta2=32, outlier_rate=0.02,
              outlier_structure="cols64", batches=(1, 16)),
}


def config_layers(cfg: int) -> List[LayerSpec]:
    return list(CONFIGS[cfg])


def make_config_layer(cfg: int, layer: int, group_axis: int = 1, stat_layout: str = "bilevel") -> SpQRLogical:
    """Logical matrix of layer `layer` of configuration `cfg`.

    Seed key is (cfg, layer); configuration 0 therefore uses seed (0, 0).
    """
    sp = CONFIGS[cfg][layer]
    return make_matrix(sp.m, sp.n, w_bits=sp.w_bits, beta1=sp.beta1, beta2=sp.beta2,
                       group_axis=group_axis, outlier_rate=sp.outlier_rate,
                       outlier_structure=sp.outlier_structure, seed=(cfg, layer), stat_layout=stat_layout)


def make_quantizer_problem(seed: int, m: int, n: int, d: Optional[int] = None, corr: float = 0.3,
                           heavy: float = 0.02) -> Tuple[np.ndarray, np.ndarray]:
    """Seeded inputs of the quantiser (Alg. 1): a weight matrix W[m, n] and calibration inputs X[n, d].

    W ~ N(0, 0.05^2) with a fraction `heavy` of the entries scaled by 6 (the isolated sensitive weights of
    Sec. 3.2); X = A G with G ~ N(0, 1)[n, d] and A = I + corr / sqrt(n) * N(0, 1)[n, n] (spectral norm of the mixing about 2 corr
    whatever the width, so the Hessian's condition number stays in the hundreds), so that the Hessian 2 X X^T has
    the correlated inputs the error feedback exploits.  d defaults to 4 n.  These stand in for a trained layer and
    its calibration activations, which are not available here.
    """
    rng = _rng(9000 + seed, m, n)
    W = rng.normal(0.0, 0.05, (m, n))
    W[rng.random((m, n)) < heavy] *= 6.0
    A = rng.normal(size=(n, n)) * (corr / np.sqrt(n)) + np.eye(n)
    X = A @ rng.normal(size=(n, d or 4 * n))
    return W, X
