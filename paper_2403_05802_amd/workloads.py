"""Seeded synthetic sparse matrices shaped like the paper's evaluation matrices.

The paper evaluates on public collections (its dataset table: few-diagonal PDE
matrices, power-law graphs, FEM-like blocked band matrices).  None of those is
reproduced here; each generator below draws a matrix with the same *structure*
from a seeded numpy generator.  This module holds no arithmetic of the method
itself (no index maps, no sorting into a format, no kernels): it only produces
unsorted COO triplets and dense operands, and it is the one module that both
the CPU oracle's tests and the HIP path's tests/bench are allowed to share.

All matrices are returned as unsorted COO with int32 indices, fp32 values in
U(-1, 1) with exact zeros redrawn, coordinates unique, and one final global
random permutation of the entry list.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SEED0 = 20240305


@dataclass
class Coo:
    nrows: int
    ncols: int
    row: np.ndarray  # int32 [nnz]
    col: np.ndarray  # int32 [nnz]
    val: np.ndarray  # float32 [nnz]
    name: str = ""

    @property
    def nnz(self) -> int:
        return int(self.row.shape[0])


def rng_for(config_index: int, salt: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(SEED0 + config_index + 1000 * salt))


def _values(rng: np.random.Generator, n: int) -> np.ndarray:
    v = rng.uniform(-1.0, 1.0, n).astype(np.float32)
    while True:
        z = np.flatnonzero(v == 0.0)
        if z.size == 0:
            return v
        v[z] = rng.uniform(-1.0, 1.0, z.size).astype(np.float32)


def dense_operand(config_index: int, shape, salt: int = 7) -> np.ndarray:
    """Dense x (1-D) or X (2-D, row-major) with entries U(-1,1), fp32."""
    rng = rng_for(config_index, salt)
    return rng.uniform(-1.0, 1.0, shape).astype(np.float32)


def _finish(rng, nrows, ncols, row, col, name) -> Coo:
    nnz = row.shape[0]
    perm = rng.permutation(nnz)
    row = np.ascontiguousarray(row[perm]).astype(np.int32)
    col = np.ascontiguousarray(col[perm]).astype(np.int32)
    val = _values(rng, nnz)
    return Coo(int(nrows), int(ncols), row, col, val, name)


def _make_distinct(row: np.ndarray, col: np.ndarray, ncols: int, redraw) -> None:
    """Redraw `col` in place (via redraw(indices) -> new cols) until all (row, col) are unique."""
    key = row.astype(np.int64) * np.int64(ncols) + col.astype(np.int64)
    order = np.argsort(key, kind="stable")
    ks = key[order]
    pending = order[np.flatnonzero(ks[1:] == ks[:-1]) + 1]
    extra = np.empty(0, dtype=np.int64)  # sorted keys accepted after the first pass
    while pending.size:
        newc = redraw(pending).astype(np.int64)
        nk = row[pending].astype(np.int64) * np.int64(ncols) + newc
        pos = np.searchsorted(ks, nk)
        pos[pos == ks.size] = ks.size - 1
        clash = ks[pos] == nk
        if extra.size:
            pe = np.searchsorted(extra, nk)
            pe[pe == extra.size] = extra.size - 1
            clash |= extra[pe] == nk
        _, first = np.unique(nk, return_index=True)
        uniq = np.zeros(nk.size, dtype=bool)
        uniq[first] = True
        ok = uniq & ~clash
        col[pending[ok]] = newc[ok]
        extra = np.sort(np.concatenate([extra, nk[ok]]))
        pending = pending[~ok]


def zipf_lengths(rng, n: int, s: float, max_len: int, target_nnz: int) -> np.ndarray:
    """Row lengths: Zipf(s) truncated to [1, max_len] by inverse CDF, rescaled to hit target_nnz."""
    k = np.arange(1, max_len + 1, dtype=np.float64)
    cdf = np.cumsum(k ** (-s))
    cdf /= cdf[-1]
    z = np.searchsorted(cdf, rng.random(n), side="left").astype(np.int64) + 1
    u = rng.random(n)
    # the scale that makes the lengths add up to target_nnz AFTER the clipping to [1, max_len] (bisection: the
    # clipped sum grows with the scale)
    lo, hi = 0.0, 4.0 * float(target_nnz) / float(z.sum()) + 1.0
    for _ in range(60):
        c = 0.5 * (lo + hi)
        total = int(np.clip(np.floor(c * z + u).astype(np.int64), 1, max_len).sum())
        if total < target_nnz:
            lo = c
        else:
            hi = c
    return np.clip(np.floor(hi * z + u).astype(np.int64), 1, max_len)


# --------------------------------------------------------------------------- config 1
def cfg1_uniform(n: int = 4096, nnz: int = 40960, index: int = 1) -> Coo:
    """n x n, nnz distinct uniformly random positions."""
    rng = rng_for(index)
    lin = rng.choice(n * n, size=nnz, replace=False)
    row, col = lin // n, lin % n
    return _finish(rng, n, n, row, col, "cfg1_uniform")


# --------------------------------------------------------------------------- config 2
def cfg2_powerlaw(n: int = 1 << 20, target_nnz: int = 1 << 24, s: float = 1.8,
                  max_len: int = 20000, empty_frac: float = 0.0, index: int = 2) -> Coo:
    """Power-law row lengths (Zipf s, min 1, max max_len), uniform distinct columns.

    empty_frac > 0 empties that fraction of rows (so that doubly compressed layouts
    have something to compress)."""
    rng = rng_for(index)
    lens = zipf_lengths(rng, n, s, min(max_len, n), target_nnz)
    if empty_frac > 0.0:
        lens[rng.random(n) < empty_frac] = 0
    row = np.repeat(np.arange(n, dtype=np.int64), lens)
    col = rng.integers(0, n, row.shape[0], dtype=np.int64)
    _make_distinct(row, col, n, lambda idx: rng.integers(0, n, idx.shape[0], dtype=np.int64))
    return _finish(rng, n, n, row, col, "cfg2_powerlaw")


# --------------------------------------------------------------------------- config 3
CFG3_OFFSETS = (-2048, -1024, -1, 0, 1, 1024, 2048)


def cfg3_banded(n: int = 1 << 21, offsets=CFG3_OFFSETS, extra_frac: float = 0.01,
                index: int = 3) -> Coo:
    """Full diagonals at `offsets` plus extra_frac more entries scattered uniformly off them."""
    rng = rng_for(index)
    rows, cols = [], []
    for off in offsets:
        i = np.arange(max(0, -off), min(n, n - off), dtype=np.int64)
        rows.append(i)
        cols.append(i + off)
    row = np.concatenate(rows)
    col = np.concatenate(cols)
    n_extra = int(round(extra_frac * row.shape[0]))
    offs = np.asarray(offsets, dtype=np.int64)

    def draw(m):
        r = rng.integers(0, n, m, dtype=np.int64)
        c = rng.integers(0, n, m, dtype=np.int64)
        while True:
            bad = np.flatnonzero(np.isin(c - r, offs))
            if bad.size == 0:
                return r, c
            r[bad] = rng.integers(0, n, bad.size, dtype=np.int64)
            c[bad] = rng.integers(0, n, bad.size, dtype=np.int64)

    er, ec = draw(n_extra)
    while True:  # distinct among the extras (they cannot collide with the diagonals)
        key = er * n + ec
        _, first = np.unique(key, return_index=True)
        if first.size == key.size:
            break
        dup = np.setdiff1d(np.arange(key.size), first)
        er[dup], ec[dup] = draw(dup.size)
    row = np.concatenate([row, er])
    col = np.concatenate([col, ec])
    return _finish(rng, n, n, row, col, "cfg3_banded")


# --------------------------------------------------------------------------- config 4
def cfg4_blockfem(n: int = 1 << 19, b: int = 4, blocks_per_row: int = 24,
                  band_blocks: int = 1024, index: int = 4) -> Coo:
    """FEM-like: dense b x b blocks, blocks_per_row block columns per block row, chosen
    uniformly (distinct) within +-band_blocks block columns of the diagonal block."""
    rng = rng_for(index)
    nb = n // b
    assert nb * b == n
    brow = np.repeat(np.arange(nb, dtype=np.int64), blocks_per_row)
    lo = np.maximum(brow - band_blocks, 0)
    hi = np.minimum(brow + band_blocks, nb - 1)
    assert int((hi - lo + 1).min()) >= blocks_per_row

    def draw(idx):
        return lo[idx] + np.floor(rng.random(idx.shape[0]) * (hi[idx] - lo[idx] + 1)).astype(np.int64)

    bcol = draw(np.arange(brow.shape[0]))
    _make_distinct(brow, bcol, nb, draw)
    inner = np.arange(b * b, dtype=np.int64)
    row = (brow[:, None] * b + inner[None, :] // b).reshape(-1)
    col = (bcol[:, None] * b + inner[None, :] % b).reshape(-1)
    return _finish(rng, n, n, row, col, "cfg4_blockfem")


# --------------------------------------------------------------------------- config 5
def cfg5_powerlaw_local(n: int = 2_000_000, target_nnz: int = 40_000_000, s: float = 2.0,
                        max_len: int = 20000, window: int = 512, local_frac: float = 0.7,
                        index: int = 5) -> Coo:
    """Power-law row lengths; each entry is 'local' (column within +-window of the row) with
    probability local_frac (at most `window` local entries per row), else uniform."""
    rng = rng_for(index)
    lens = zipf_lengths(rng, n, s, min(max_len, n), target_nnz)
    i = np.arange(n, dtype=np.int64)
    wlo = np.maximum(i - window, 0)
    whi = np.minimum(i + window, n - 1)
    wsize = whi - wlo + 1
    nloc = np.minimum(np.minimum(rng.binomial(lens, local_frac), window), wsize)
    row = np.repeat(i, lens)
    start = np.cumsum(lens) - lens
    within = np.arange(row.shape[0], dtype=np.int64) - np.repeat(start, lens)
    is_local = within < np.repeat(nloc, lens)
    col = np.empty(row.shape[0], dtype=np.int64)

    def draw(idx):
        r = row[idx]
        u = rng.random(idx.shape[0])
        loc = wlo[r] + np.floor(u * wsize[r]).astype(np.int64)
        uni = np.floor(u * n).astype(np.int64)
        return np.where(is_local[idx], loc, uni)

    col[:] = draw(np.arange(row.shape[0]))
    # rows with many local entries: sample the window without replacement exactly
    dense_rows = np.flatnonzero(nloc > 32)
    chunk = 4096
    for c0 in range(0, dense_rows.size, chunk):
        rr = dense_rows[c0:c0 + chunk]
        wmax = 2 * window + 1
        keys = rng.random((rr.size, wmax), dtype=np.float32)
        keys[np.arange(wmax)[None, :] >= wsize[rr][:, None]] = 2.0
        order = np.argsort(keys, axis=1)
        for j, r in enumerate(rr):
            m = int(nloc[r])
            col[start[r]:start[r] + m] = wlo[r] + order[j, :m]
    _make_distinct(row, col, n, draw)
    return _finish(rng, n, n, row, col, "cfg5_powerlaw_local")
