"""Seeded synthetic inputs: flattened question+table token structures and Q/K/V/dO tensors.

This module only *draws inputs*.  It holds none of the attention arithmetic, no mask
logic and no sorting: both the CPU oracle's tests and the HIP path's tests/bench feed
from it, so that the two sides see identical bytes without sharing any method code.

The token layout follows the paper's input description (Section 3, first paragraph):
a prefix of question tokens (the set Q, flagged GLOBAL here), then the table flattened
row-major cell by cell, then padding.  Each table token carries the row and column
number of its cell (header row = 0, data rows 1.., columns 1..C).

The five named configurations stand in for the paper's table-QA datasets (short cells,
many rows), which are not available; sizes are those of the benchmark configurations.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

TOK_LOCAL = 0   # table token: attends to globals and to its own row / column
TOK_GLOBAL = 1  # question token (member of the set Q): attends to / from everything
TOK_PAD = 2     # padding: no weight as key, zero output as query

HEAD_ROW = 0
HEAD_COL = 1

BASE_SEED = 210904312


@dataclass
class Structure:
    """Integer description of a batch of sequences."""
    row_ids: np.ndarray   # [B,N] int32
    col_ids: np.ndarray   # [B,N] int32
    flags: np.ndarray     # [B,N] uint8 (TOK_*)

    @property
    def B(self) -> int:
        return self.row_ids.shape[0]

    @property
    def N(self) -> int:
        return self.row_ids.shape[1]


@dataclass
class Workload:
    name: str
    dtype: str                 # "f32" or "bf16"
    structure: Structure
    head_kind: np.ndarray      # [H] uint8 (HEAD_*)
    q: np.ndarray              # [B,H,N,D] float32 holding dtype-representable values
    k: np.ndarray
    v: np.ndarray
    do: Optional[np.ndarray]   # None for forward-only workloads
    scale: float
    meta: dict = field(default_factory=dict)

    @property
    def shape(self):
        return self.q.shape


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result kept as float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint32)
    return (r << np.uint32(16)).view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def geometric_lengths(rng: np.random.Generator, mean: float, cap: int, size: int) -> np.ndarray:
    return np.minimum(rng.geometric(1.0 / mean, size=size), cap).astype(np.int64)


def flatten_table(N: int, n_global: int, n_rows: int, n_cols: int, cell_len: np.ndarray):
    """One sequence: `n_global` question tokens, then cells row-major, cut / padded to N."""
    row = np.zeros(N, np.int32)
    col = np.zeros(N, np.int32)
    flag = np.full(N, TOK_PAD, np.uint8)
    g = min(n_global, N)
    flag[:g] = TOK_GLOBAL
    cell_len = np.asarray(cell_len, np.int64).reshape(n_rows, n_cols)
    rr = np.repeat(np.repeat(np.arange(n_rows), n_cols), cell_len.ravel())
    cc = np.repeat(np.tile(np.arange(n_cols) + 1, n_rows), cell_len.ravel())
    m = min(len(rr), N - g)
    row[g:g + m] = rr[:m]
    col[g:g + m] = cc[:m]
    flag[g:g + m] = TOK_LOCAL
    return row, col, flag


def _stack(seqs) -> Structure:
    r, c, f = zip(*seqs)
    return Structure(np.stack(r), np.stack(c), np.stack(f))


def half_row_half_col(H: int) -> np.ndarray:
    """First half of the heads are row heads, the rest column heads (the paper's 1:1 ratio)."""
    hk = np.full(H, HEAD_COL, np.uint8)
    hk[: H // 2] = HEAD_ROW
    return hk


def draw_tensors(rng: np.random.Generator, B, H, N, D, dtype: str, n: int, data_scale: float = 1.0):
    out = []
    for _ in range(n):
        x = rng.standard_normal((B, H, N, D), dtype=np.float32)
        if data_scale != 1.0:
            x = x * np.float32(data_scale)
        if dtype == "bf16":
            x = round_to_bf16(x)
        out.append(x)
    return out


def draw_wide_range_tensors(rng: np.random.Generator, st: "Structure", H: int, D: int, dtype: str,
                            sigma_raw: float = 60.0, outliers=(150.0, 200.0, 250.0, 300.0, 350.0),
                            quantiles=(0.45, 0.6, 0.75, 0.9, 0.97)):
    """Q, K, V, dO whose raw scores q.k span a wide range (an input recipe only; no attention
    arithmetic): Q and K are N(0,1) scaled so that q.k has standard deviation `sigma_raw`; the
    key norms grow with the token's rank among the non-pad positions (factor 0.3 .. 1.7); and a
    few table tokens, at the given quantiles of the table tokens of each sequence, carry a key
    that scores about `outliers[i]` more than the rest against every query (all queries share a
    component of 10 along one random unit direction u, the outlier keys get outliers[i] / 10
    along u).  V and dO are plain N(0,1).  Returns q, k, v, do as float32 holding dtype-
    representable values, [B,H,N,D]."""
    B, N = st.flags.shape
    c = float(np.sqrt(sigma_raw / np.sqrt(D)))
    q, k, v, do = (rng.standard_normal((B, H, N, D), dtype=np.float32) for _ in range(4))
    q *= np.float32(c)
    k *= np.float32(c)
    u = rng.standard_normal(D)
    u = (u / np.linalg.norm(u)).astype(np.float32)
    q += np.float32(10.0) * u
    for b in range(B):
        nonpad = np.flatnonzero(st.flags[b] != TOK_PAD)
        if len(nonpad):
            growth = np.ones(N, np.float32)
            growth[nonpad] = 0.3 + 1.4 * np.arange(len(nonpad), dtype=np.float32) / max(1, len(nonpad) - 1)
            k[b] *= growth[None, :, None]
        table = np.flatnonzero(st.flags[b] == TOK_LOCAL)
        for amount, qt in zip(outliers, quantiles):
            if len(table):
                pos = table[min(len(table) - 1, int(qt * len(table)))]
                k[b, :, pos, :] += np.float32(amount / 10.0) * u
    out = [q, k, v, do]
    if dtype == "bf16":
        out = [round_to_bf16(x) for x in out]
    return out


CONFIG_NAMES = {
    1: "cfg1_tiny_f32_B1_N128_H4",
    2: "cfg2_B32_N512_H12",
    3: "cfg3_B8_N2048_H16",
    4: "cfg4_B2_N8192_H16",
    5: "cfg5_ragged_B16_N4096_H16",
    6: "cfg6_longcells_B8_N2048_H16",
}


def config_structure(idx: int, rng: np.random.Generator):
    """Structure + (B,N,H,D,dtype,backward?) of benchmark configuration `idx` (1..6)."""
    D = 64
    if idx == 1:
        B, N, H, dtype, bwd = 1, 128, 4, "f32", False
        seqs = [flatten_table(N, 16, 8, 4, rng.integers(1, 5, size=32))]
    elif idx == 2:
        B, N, H, dtype, bwd = 32, 512, 12, "bf16", True
        seqs = []
        for _ in range(B):
            R = int(rng.integers(8, 33))
            C = int(rng.integers(3, 9))
            seqs.append(flatten_table(N, 32, R, C, geometric_lengths(rng, 2.0, 8, R * C)))
    elif idx == 3:
        B, N, H, dtype, bwd = 8, 2048, 16, "bf16", True
        seqs = [flatten_table(N, 64, 100, 6, geometric_lengths(rng, 2.0, 8, 600)) for _ in range(B)]
    elif idx == 4:
        B, N, H, dtype, bwd = 2, 8192, 16, "bf16", True
        seqs = [flatten_table(N, 64, 400, 8, geometric_lengths(rng, 2.0, 8, 3200)) for _ in range(B)]
    elif idx == 5:
        B, N, H, dtype, bwd = 16, 4096, 16, "bf16", True
        seqs = []
        for b in range(B):
            G = int(rng.integers(16, 129))
            R = int(rng.integers(1, 401))
            C = int(rng.integers(1, 21))
            if b == 0:
                R = 1      # degenerate one-row table
            if b == 1:
                C = 1      # degenerate one-column table
            seqs.append(flatten_table(N, G, R, C, geometric_lengths(rng, 3.0, 16, R * C)))
    elif idx == 6:
        # Long expanded cells (the shape of the paper's HybridQA inputs, Section 4 and the
        # appendix on hyper-parameters: about 70 cells, most of them with tens of tokens of
        # entity text, sequence length 2048): rows AND columns are segments of hundreds of tokens.
        B, N, H, dtype, bwd = 8, 2048, 16, "bf16", True
        seqs = []
        for _ in range(B):
            R, C = 14, 5
            long_cell = rng.random(R * C) < 0.63
            lens = np.where(long_cell, geometric_lengths(rng, 40.0, 120, R * C),
                            geometric_lengths(rng, 2.0, 8, R * C))
            seqs.append(flatten_table(N, 64, R, C, lens))
    else:
        raise ValueError(f"unknown config {idx}")
    return _stack(seqs), (B, N, H, D, dtype, bwd)


def make_config(idx: int, seed: Optional[int] = None, tensors: bool = True) -> Workload:
    """Benchmark configuration `idx` (1..6); seed defaults to BASE_SEED + idx."""
    rng = np.random.default_rng(BASE_SEED + idx if seed is None else seed)
    st, (B, N, H, D, dtype, bwd) = config_structure(idx, rng)
    hk = half_row_half_col(H)
    if tensors:
        ds = (1.0 / np.sqrt(D)) if idx == 1 else 1.0
        ts = draw_tensors(rng, B, H, N, D, dtype, 4 if bwd else 3, ds)
        q, k, v = ts[:3]
        do = ts[3] if bwd else None
    else:
        q = k = v = np.zeros((B, H, N, D), np.float32)[:0]
        do = None
    return Workload(CONFIG_NAMES[idx], dtype, st, hk, q, k, v, do, 1.0 / float(np.sqrt(D)),
                    meta=dict(config=idx, B=B, N=N, H=H, D=D, backward=bwd))


def random_structure(rng: np.random.Generator, B: int, N: int, *, max_rows=6, max_cols=5,
                     max_global=6, max_cell=3, scatter=False, sparse_ids=False) -> Structure:
    """Small adversarial structures for tests.

    scatter=True shuffles token positions inside each sequence, so that globals, pads and
    table tokens interleave arbitrarily (the attention pattern is defined per token, not by
    position).  sparse_ids=True relabels row/column numbers by a random strictly increasing
    map with large gaps, and lets the header row keep id 0 (shared with question tokens).
    """
    seqs = []
    for _ in range(B):
        G = int(rng.integers(0, max_global + 1))
        R = int(rng.integers(1, max_rows + 1))
        C = int(rng.integers(1, max_cols + 1))
        row, col, flag = flatten_table(N, G, R, C, rng.integers(1, max_cell + 1, size=R * C))
        if sparse_ids:
            rmap = np.concatenate([[0], np.cumsum(rng.integers(1, 1 << 20, size=R))]).astype(np.int64)
            cmap = np.concatenate([[0], np.cumsum(rng.integers(1, 1 << 20, size=C + 1))]).astype(np.int64)
            loc = flag == TOK_LOCAL
            row = np.where(loc, rmap[row], row).astype(np.int32)
            col = np.where(loc, cmap[col], col).astype(np.int32)
        if scatter:
            p = rng.permutation(N)
            row, col, flag = row[p], col[p], flag[p]
        seqs.append((row, col, flag))
    return _stack(seqs)
