"""CPU oracle for sparse-format customization (test infrastructure, not a product path).

A plain, slow, generic numpy implementation of what the paper's format abstraction
*defines*: given an unsorted COO matrix and a format encoding (index map + trim/merge,
Section 4.1; Figure 7 lists the encodings), produce the level-wise arrays that the
data-structure inference rules of Section 5.1 prescribe; split a matrix by a `sum`
query (Section 4.1.2, the decompose op of Section 6); and evaluate SpMV / SpMM over a
formatted matrix the way the generated kernel of Figure 9 does (walk the levels,
invert the index map, guard the bounds), in float64.

It interprets the descriptor level by level; nothing in here is specialised per format,
blocked, fused or tuned, so that it can be checked against the paper by eye.  It shares
no code with the HIP library and must never be imported by it.  Only tests, the smoke
check and the CPU-baseline leg of the benchmark may import this module.

Readings of the paper where it is silent or its figures are unavailable (each is also
listed in the design notes of the repository):
  * the output is always sorted by the full target tuple (Section 5.2: a Sort orders the
    indices as the target format specifies), whatever the input order;
  * coordinates must be unique; duplicates are an error;
  * every stored COO entry is structural: values are never tested against zero;
  * `/` is floor division and `%` the non-negative remainder; a level `d/b` has extent
    ceil(D/b), a level `d%b` extent b; leaves that map outside the matrix are padding;
  * a `ptr` array has parents+1 entries and starts at 0 (Figure 9, loop bounds);
  * dense trailing levels are laid out node-major, inner index minor (Figure 9, the
    value access);
  * a trimmed level that sits directly above a dense level is fused like a merged one
    (its dense children are addressed by position, so equal paths cannot stay apart):
    this is what makes BDIA's middle level one node per (block, diagonal) although its
    encoding lists merge(0) only (Figure 3c; Figure 9 addresses val[node*size_2 + id2]);
  * ELL: the indirect level is the rank of an entry in its row by ascending column
    (the enum query of Figure 7), exposed as a size K (K = longest row unless a width is
    fixed); the column level that follows holds one index per (slot,row) with pad = -1
    and pad value +0.0;
  * blocked ELL (the BELL of Section 7.2.2, whose encoding is in a figure that is not available): ELL's
    map over block rows and block columns with the two in-block indices below it,
    (indirect(d1/bw), d0/bh, d1/bw, d0%bh, d1%bw), merge(0), trim(0,0); the enum query numbers the
    blocks of a block row (entries of one block share a number);
  * CISR-plus (Section 7.2.4, its printed encoding): the indirect level is built from three
    queries -- sum (entries per row), reorder (rows with the most entries first; equal rows in
    ascending row order) and schedule into N partitions; the text asks only that the assignment be balanced,
    and that is read here as dealing: the k-th row of that order goes to
    partition k mod N.  The level is untouched by trim(1,2), hence a size N; rows and columns
    below it are compressed levels (a row level with a ptr over the N partitions);
  * parity unpinned by the paper: the pad column (-1), percentile-based ELL width, the
    "fraction of the in-bounds diagonal length" predicate, the dealing rule of schedule and the
    blocked ELL encoding are this repository's readings, pinned only by hand-derived layouts and
    brute-force tests.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

# --------------------------------------------------------------------------- descriptors

AFFINE, DIV, MOD, ENUM, SCHED = "affine", "div", "mod", "enum", "sched"


@dataclass(frozen=True)
class Expr:
    """One destination index expression of an index map (Figure 5a).

    affine: c0*d0 + c1*d1 + c
    div   : (c0*d0 + c1*d1 + c) / factor       (floor)
    mod   : (c0*d0 + c1*d1 + c) % factor       (non-negative)
    enum  : indirect level: rank of the entry inside its group (group key = the affine
            part / factor, e.g. d0, or d0/bh for blocked ELL) when the group is traversed by
            ascending `traverse` dim / traverse_factor; entries that agree in that key share
            a rank (the blocks of a block row are numbered, not their entries)
    sched : indirect level: the partition (0..factor-1) that the entry's group (key = the
            affine part, e.g. d0) is scheduled to: groups ordered by size, largest first
            (sum + reorder queries), then dealt to `factor` partitions (schedule query)
    """
    kind: str
    c0: int = 0
    c1: int = 0
    c: int = 0
    factor: int = 1
    traverse: int = 1  # for ENUM: logical dim that orders the group (1 = d1)
    traverse_factor: int = 1  # for ENUM: the group is traversed by (traverse dim) / traverse_factor


def d0() -> Expr: return Expr(AFFINE, 1, 0)
def d1() -> Expr: return Expr(AFFINE, 0, 1)
def diag() -> Expr: return Expr(AFFINE, -1, 1)          # d1 - d0
def div(dim: int, f: int) -> Expr: return Expr(DIV, 1 - dim, dim, 0, f)
def mod(dim: int, f: int) -> Expr: return Expr(MOD, 1 - dim, dim, 0, f)
def enum_by_row() -> Expr: return Expr(ENUM, 1, 0, 0, 1, traverse=1)
def sched_rows(n: int) -> Expr: return Expr(SCHED, 1, 0, 0, n)


@dataclass(frozen=True)
class FormatDesc:
    levels: Tuple[Expr, ...]
    trim: Optional[Tuple[int, int]]      # trim(S, E), None = no trim
    merge: Tuple[int, ...] = ()          # merge(L, ...)
    ell_width: int = 0                   # ENUM level: 0 = longest group, >0 = fixed


# the encodings of Figure 7 (and the swapped / DIA-variant maps of Section 4.1.1)
def COO() -> FormatDesc: return FormatDesc((d0(), d1()), (0, 1))
def CSR() -> FormatDesc: return FormatDesc((d0(), d1()), (1, 1), (0,))
def DCSR() -> FormatDesc: return FormatDesc((d0(), d1()), (0, 1), (0,))
def CSC() -> FormatDesc: return FormatDesc((d1(), d0()), (1, 1), (0,))
def DCSC() -> FormatDesc: return FormatDesc((d1(), d0()), (0, 1), (0,))
def DIA() -> FormatDesc: return FormatDesc((diag(), d0()), (0, 0), (0,))
def DIA_VARIANT() -> FormatDesc: return FormatDesc((diag(), d1()), (0, 0), (0,))
def BCSR(bh: int, bw: Optional[int] = None) -> FormatDesc:
    bw = bh if bw is None else bw
    return FormatDesc((div(0, bh), div(1, bw), mod(0, bh), mod(1, bw)), (1, 1), (0, 1))
def CSB(bh: int, bw: Optional[int] = None) -> FormatDesc:
    bw = bh if bw is None else bw
    return FormatDesc((div(0, bh), div(1, bw), mod(0, bh), mod(1, bw)), (2, 3), (1,))
def BDIA(b: int) -> FormatDesc:
    return FormatDesc((div(0, b), diag(), mod(0, b)), (1, 1), (0,))
def ELL(width: int = 0) -> FormatDesc:
    return FormatDesc((enum_by_row(), d0(), d1()), (0, 0), (0,), ell_width=width)
def BELL(bh: int, bw: Optional[int] = None, width: int = 0) -> FormatDesc:
    """Blocked ELL (the BELL of Section 7.2.2; its encoding sits in a figure that is not available, so this is a
    reading): ELL's map with rows and columns replaced by block rows and block columns, and the two in-block
    indices below -- (indirect(d1/bw), d0/bh, d1/bw, d0%bh, d1%bw), merge(0), trim(0,0).  The indirect level
    numbers the blocks of a block row by ascending block column."""
    bw = bh if bw is None else bw
    return FormatDesc((Expr(ENUM, 1, 0, 0, bh, traverse=1, traverse_factor=bw), div(0, bh), div(1, bw), mod(0, bh), mod(1, bw)),
                      (0, 0), (0,), ell_width=width)
def CISR_PLUS(n: int) -> FormatDesc:
    """Section 7.2.4: (indirect(d0), d0, d1), merge(0,1), trim(1,2), n partitions."""
    return FormatDesc((sched_rows(n), d0(), d1()), (1, 2), (0, 1))


class OracleError(Exception):
    def __init__(self, code: str, msg: str = ""):
        super().__init__(f"{code}: {msg}")
        self.code = code


@dataclass
class Level:
    kind: str                             # 'dense' | 'compressed' | 'coordinate' | 'payload'
    size: Optional[int] = None            # dense: extent; ENUM level: K
    lo: int = 0                           # dense: smallest index value (0 except skewed dense levels)
    ptr: Optional[np.ndarray] = None      # int32 [parents+1]
    idx: Optional[np.ndarray] = None      # int32


@dataclass
class Formatted:
    desc: FormatDesc
    nrows: int
    ncols: int
    nnz: int
    levels: List[Level] = field(default_factory=list)
    val: np.ndarray = None                # float32, one slot per leaf


# --------------------------------------------------------------------------- index map

def _affine(e: Expr, r: np.ndarray, c: np.ndarray) -> np.ndarray:
    return e.c0 * r + e.c1 * c + e.c


def _affine_range(e: Expr, nrows: int, ncols: int) -> Tuple[int, int]:
    corners = [e.c0 * a + e.c1 * b + e.c for a in (0, nrows - 1) for b in (0, ncols - 1)]
    return min(corners), max(corners)


def _group_rank(group: np.ndarray, order_key: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """enum query: rank of every entry inside its group when the group is traversed by
    ascending order_key, entries with equal order_key sharing a rank (with unique (group, order_key)
    pairs, as in ELL, that is the position in the group); also returns, aligned with the entries,
    the number of distinct order_key values of their group."""
    n = group.shape[0]
    order = np.lexsort((order_key, group))
    g, k = group[order], order_key[order]
    new_group = np.concatenate(([True], g[1:] != g[:-1])) if n else np.empty(0, bool)
    new_key = (new_group | np.concatenate(([True], k[1:] != k[:-1]))) if n else np.empty(0, bool)
    distinct_before = np.cumsum(new_key) - 1                       # running count of distinct (group, key) pairs
    group_start = np.flatnonzero(new_group)
    lens = np.diff(np.concatenate((group_start, [n])))
    rank_sorted = distinct_before - np.repeat(distinct_before[group_start], lens) if n else np.empty(0, np.int64)
    size_sorted = np.repeat(np.add.reduceat(new_key.astype(np.int64), group_start), lens) if n else np.empty(0, np.int64)
    rank = np.empty(n, dtype=np.int64)
    rank[order] = rank_sorted
    size = np.empty(n, dtype=np.int64)
    size[order] = size_sorted
    return rank, size


def _scheduled_partition(group: np.ndarray, nparts: int) -> np.ndarray:
    """The three queries behind the indirect level of CISR-plus, one after the other.
    sum:      entries per group (only groups that hold an entry exist);
    reorder:  groups by descending size, equal sizes by ascending group index;
    schedule: the k-th group of that order is dealt to partition k mod nparts.
    Returns the partition of every entry."""
    if nparts < 1:
        raise OracleError("US_ERR_UNSUPPORTED_DESC", "number of partitions")
    ids, inv, size = np.unique(group, return_inverse=True, return_counts=True)   # sum
    order = np.lexsort((ids, -size))                                             # reorder
    part_of_group = np.empty(ids.shape[0], dtype=np.int64)
    part_of_group[order] = np.arange(ids.shape[0], dtype=np.int64) % nparts      # schedule
    return part_of_group[inv.reshape(-1)]


def eval_index_map(desc: FormatDesc, nrows: int, ncols: int, row: np.ndarray, col: np.ndarray
                   ) -> List[np.ndarray]:
    """Target tuple e = M(d0, d1) of every entry (Section 4.1.1), one int64 array per level."""
    r = row.astype(np.int64)
    c = col.astype(np.int64)
    out = []
    for e in desc.levels:
        a = _affine(e, r, c)
        if e.kind == AFFINE:
            out.append(a)
        elif e.kind == DIV:
            out.append(np.floor_divide(a, e.factor))
        elif e.kind == MOD:
            out.append(np.mod(a, e.factor))
        elif e.kind == ENUM:
            rank, _ = _group_rank(np.floor_divide(a, e.factor),
                                  np.floor_divide(c if e.traverse == 1 else r, e.traverse_factor))
            out.append(rank)
        elif e.kind == SCHED:
            out.append(_scheduled_partition(a, e.factor))
        else:
            raise OracleError("US_ERR_UNSUPPORTED_DESC", e.kind)
    return out


def _level_extent(desc: FormatDesc, L: int, nrows: int, ncols: int, eL: np.ndarray) -> Tuple[int, int]:
    """(lo, extent) of the index values a dense level L can take."""
    e = desc.levels[L]
    if e.kind == ENUM:
        if desc.ell_width > 0:
            return 0, int(desc.ell_width)
        return 0, int(eL.max()) + 1 if eL.size else 0
    if e.kind == SCHED:
        return 0, int(e.factor)
    lo, hi = _affine_range(e, nrows, ncols)
    if e.kind == AFFINE:
        return lo, hi - lo + 1
    if e.kind == DIV:
        return lo // e.factor, hi // e.factor - lo // e.factor + 1
    return 0, e.factor  # MOD


def infer_level_kinds(desc: FormatDesc) -> List[str]:
    """Section 5.1: untouched level -> size (dense); trimmed level -> explicit idx, with a
    ptr when its parent level is merged; after an indirect enum level and the level
    holding its group dimension, the traversed dimension is determined by its parents and
    is kept as one explicit index per parent ('payload')."""
    kinds = []
    S, E = desc.trim if desc.trim is not None else (1, 0)
    enum_traverse = None
    enum_factor = 1
    deepest_merge = max(desc.merge) if desc.merge else -1   # merge(L) fuses whole paths root..L
    for L, e in enumerate(desc.levels):
        if e.kind == ENUM:
            kinds.append("dense")  # slots 0..K-1 are contiguous from 0: a size, not an idx
            enum_traverse, enum_factor = e.traverse, e.traverse_factor
            continue
        # the level that holds the key the groups were traversed by: d1 (ELL) or d1/bw (blocked ELL)
        is_traversed_dim = (enum_traverse is not None and e.c == 0 and
                            (e.c0, e.c1) == ((0, 1) if enum_traverse == 1 else (1, 0)) and
                            ((e.kind == AFFINE and enum_factor == 1) or (e.kind == DIV and e.factor == enum_factor)))
        if is_traversed_dim:
            kinds.append("payload")
        elif S <= L <= E:
            parent_merged = (L == 0) or (L - 1 <= deepest_merge) or (kinds[L - 1] == "dense")
            kinds.append("compressed" if (L <= deepest_merge or parent_merged) else "coordinate")
        else:
            kinds.append("dense")
    return kinds


# --------------------------------------------------------------------------- conversion

def validate_coo(nrows: int, ncols: int, row, col, val) -> None:
    if nrows <= 0 or ncols <= 0:
        raise OracleError("US_ERR_SHAPE")
    if not (row.shape == col.shape == val.shape) or row.ndim != 1:
        raise OracleError("US_ERR_SHAPE")
    if row.size:
        if row.min() < 0 or row.max() >= nrows or col.min() < 0 or col.max() >= ncols:
            raise OracleError("US_ERR_INDEX_RANGE")
        key = row.astype(np.int64) * ncols + col.astype(np.int64)
        if np.unique(key).size != key.size:
            raise OracleError("US_ERR_DUPLICATE")


def convert(nrows: int, ncols: int, row, col, val, desc: FormatDesc) -> Formatted:
    """COO -> target format: evaluate the index map, sort by the target tuple, then emit
    the arrays level by level (Figure 8, steps 1-2, and the rules of Section 5.1)."""
    row = np.asarray(row)
    col = np.asarray(col)
    val = np.asarray(val, dtype=np.float32)
    validate_coo(nrows, ncols, row, col, val)
    nnz = row.shape[0]
    e = eval_index_map(desc, nrows, ncols, row, col)
    order = np.lexsort(tuple(reversed(e))) if nnz else np.empty(0, np.int64)
    e = [x[order] for x in e]
    v = val[order]

    kinds = infer_level_kinds(desc)
    out = Formatted(desc, nrows, ncols, nnz)
    node = np.zeros(nnz, dtype=np.int64)   # node id (storage order) of each entry at the previous level
    nnodes = 1                             # the root
    for L, kind in enumerate(kinds):
        eL = e[L]
        if kind == "dense":
            lo, D = _level_extent(desc, L, nrows, ncols, eL)
            if nnz and (eL.min() < lo or eL.max() >= lo + D):
                raise OracleError("US_ERR_SHAPE", "entry outside a fixed-width level")
            node = node * D + (eL - lo)
            nnodes = nnodes * D
            out.levels.append(Level("dense", size=int(D), lo=int(lo)))
        elif kind == "payload":
            idx = np.full(nnodes, -1, dtype=np.int32)
            idx[node] = eL
            out.levels.append(Level("payload", idx=idx))
        else:
            # merge(L') fuses whole paths root..L'; a level whose children are a dense level is
            # fused as well, since dense children are addressed by position under one parent
            merged = (bool(desc.merge) and L <= max(desc.merge)) or \
                (L + 1 < len(kinds) and kinds[L + 1] == "dense")
            if merged:   # equal (parent, index) paths are one node
                head = np.ones(nnz, dtype=bool)
                if nnz:
                    head[1:] = (node[1:] != node[:-1]) | (eL[1:] != eL[:-1])
            else:        # every entry keeps a node of its own
                head = np.ones(nnz, dtype=bool)
            new_node = np.cumsum(head) - 1
            first = np.flatnonzero(head)
            lvl = Level(kind, idx=eL[first].astype(np.int32))
            if kind == "compressed" and L >= 1:
                children = np.bincount(node[first], minlength=nnodes)
                ptr = np.zeros(nnodes + 1, dtype=np.int64)
                np.cumsum(children, out=ptr[1:])
                lvl.ptr = ptr.astype(np.int32)
            out.levels.append(lvl)
            node = new_node
            nnodes = int(first.size)
        if nnodes >= 2 ** 31:
            raise OracleError("US_ERR_OVERFLOW")
    out.val = np.zeros(nnodes, dtype=np.float32)
    out.val[node] = v
    return out


# --------------------------------------------------------------------------- reading a layout back

def _invert_map(desc: FormatDesc, e: List[np.ndarray]) -> Tuple[np.ndarray, np.ndarray]:
    """M^-1 (Section 4.1.1; Figure 9 restores d0 = e0*3+e2, d1 = e1+d0 for BDIA):
    re-join every (d/f, d%f) pair, then solve the remaining affine equations exactly."""
    eqs = []  # (c0, c1, rhs array) meaning c0*d0 + c1*d1 = rhs
    used = set()
    for i, a in enumerate(desc.levels):
        if a.kind == DIV:
            for j, b in enumerate(desc.levels):
                if b.kind == MOD and (b.c0, b.c1, b.c, b.factor) == (a.c0, a.c1, a.c, a.factor):
                    eqs.append((a.c0, a.c1, e[i] * a.factor + e[j] - a.c))
                    used.update((i, j))
    for i, a in enumerate(desc.levels):
        if a.kind == AFFINE and i not in used:
            eqs.append((a.c0, a.c1, e[i] - a.c))
    for i in range(len(eqs)):
        for j in range(i + 1, len(eqs)):
            a0, a1, ra = eqs[i]
            b0, b1, rb = eqs[j]
            det = a0 * b1 - a1 * b0
            if det != 0:
                n0 = ra * b1 - a1 * rb
                n1 = a0 * rb - ra * b0
                assert np.all(n0 % det == 0) and np.all(n1 % det == 0)
                return n0 // det, n1 // det
    raise OracleError("US_ERR_UNSUPPORTED_DESC", "index map is not invertible")


def leaves(f: Formatted) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Walk the stored levels top-down using only the arrays (size / ptr / idx), rebuild
    the target tuple of every leaf, invert the index map and keep the leaves that fall
    inside the matrix (the guard of Figure 9).  Returns (d0, d1, leaf id)."""
    tuples: List[np.ndarray] = []
    n = 1
    alive = np.ones(1, dtype=bool)
    for L, lvl in enumerate(f.levels):
        if lvl.kind == "dense":
            D = lvl.size
            tuples = [np.repeat(t, D) for t in tuples]
            alive = np.repeat(alive, D)
            tuples.append(np.tile(np.arange(D, dtype=np.int64) + lvl.lo, n))
            n *= D
        elif lvl.kind == "payload":
            assert lvl.idx.shape[0] == n
            tuples.append(lvl.idx.astype(np.int64))
            alive = alive & (lvl.idx >= 0)
        else:
            if lvl.ptr is not None:
                assert lvl.ptr.shape[0] == n + 1 and lvl.ptr[0] == 0
                cnt = np.diff(lvl.ptr.astype(np.int64))
                assert np.all(cnt >= 0) and lvl.ptr[-1] == lvl.idx.shape[0]
                tuples = [np.repeat(t, cnt) for t in tuples]
                alive = np.repeat(alive, cnt)
            else:
                assert L == 0 or lvl.idx.shape[0] == n
            tuples.append(lvl.idx.astype(np.int64))
            n = lvl.idx.shape[0]
            if L == 0:
                alive = np.ones(n, dtype=bool)
    assert f.val.shape[0] == n
    leaf = np.flatnonzero(alive)
    e = [t[leaf] for t in tuples]
    r, c = _invert_map(f.desc, e)
    ok = (r >= 0) & (r < f.nrows) & (c >= 0) & (c < f.ncols)
    return r[ok], c[ok], leaf[ok]


def to_coo(f: Formatted, drop_zero_slots: bool = True):
    """Formatted -> COO sorted by (row, col).  Slots of dense levels that hold +0.0/-0.0 are
    indistinguishable from padding and are dropped (inputs never contain exact zeros)."""
    r, c, leaf = leaves(f)
    v = f.val[leaf]
    has_dense_slots = f.levels[-1].kind in ("dense", "payload")
    if drop_zero_slots and has_dense_slots:
        keep = v != 0
        r, c, v = r[keep], c[keep], v[keep]
    order = np.lexsort((c, r))
    return r[order].astype(np.int32), c[order].astype(np.int32), v[order]


def to_dense(f: Formatted) -> np.ndarray:
    r, c, leaf = leaves(f)
    A = np.zeros((f.nrows, f.ncols), dtype=np.float64)
    np.add.at(A, (r, c), f.val[leaf].astype(np.float64))
    return A


# --------------------------------------------------------------------------- decompose

SUM_GE_ABS, SUM_GE_FRAC_OF_CAPACITY, RANK_LT_ABS, RANK_LT_PERCENTILE = (
    "sum_ge_abs", "sum_ge_frac_of_capacity", "rank_lt_abs", "rank_lt_percentile")


@dataclass(frozen=True)
class Predicate:
    """Which entries go to part A of a hybrid.  `group` is the groupBy index map of the
    sum query (Section 4.1.2); the predicate compares the per-group count of stored
    entries with a threshold, or the entry's rank inside its group with a width."""
    group: Tuple[Expr, ...]
    kind: str
    num: int = 0
    den: int = 1
    abs: int = 0


def group_capacity(group: Sequence[Expr], nrows: int, ncols: int, key: List[np.ndarray]) -> np.ndarray:
    """Number of in-bounds matrix positions that fall in the group of each given key."""
    if len(group) == 1 and group[0].kind == AFFINE and group[0].c == 0:
        g = group[0]
        k = key[0]
        if (g.c0, g.c1) == (-1, 1):   # diagonal col-row = k: rows max(0,-k) .. min(nrows, ncols-k)-1
            return np.maximum(np.minimum(nrows, ncols - k) - np.maximum(0, -k), 0)
        if (g.c0, g.c1) == (1, 0):
            return np.full(k.shape, ncols, dtype=np.int64)
        if (g.c0, g.c1) == (0, 1):
            return np.full(k.shape, nrows, dtype=np.int64)
    raise OracleError("US_ERR_UNSUPPORTED_DESC", "capacity of this group map")


def percentile_width(lengths_all_groups: np.ndarray, num: int, den: int) -> int:
    """Nearest-rank percentile over all groups (empty ones included)."""
    s = np.sort(lengths_all_groups)
    n = s.shape[0]
    k = -(-(num * n) // den)  # ceil(num*n/den)
    return int(s[max(k, 1) - 1])


def predicate_mask(nrows: int, ncols: int, row, col, pred: Predicate) -> np.ndarray:
    r = np.asarray(row).astype(np.int64)
    c = np.asarray(col).astype(np.int64)
    gdesc = FormatDesc(tuple(pred.group), None)
    key = eval_index_map(gdesc, nrows, ncols, r, c)
    # sum query: count of stored entries per group (value map: stored -> 1)
    if len(key) == 1:
        _, inv, cnt = np.unique(key[0], return_inverse=True, return_counts=True)
    else:
        stacked = np.stack(key, axis=1) if r.size else np.zeros((0, len(key)), np.int64)
        _, inv, cnt = np.unique(stacked, axis=0, return_inverse=True, return_counts=True)
    inv = inv.reshape(-1)
    count = cnt[inv] if r.size else np.zeros(0, np.int64)
    if pred.kind == SUM_GE_ABS:
        return count >= pred.abs
    if pred.kind == SUM_GE_FRAC_OF_CAPACITY:
        cap = group_capacity(pred.group, nrows, ncols, key)
        return pred.den * count >= pred.num * cap
    if pred.kind in (RANK_LT_ABS, RANK_LT_PERCENTILE):
        if not (len(pred.group) == 1 and pred.group[0].kind == AFFINE and
                (pred.group[0].c0, pred.group[0].c1, pred.group[0].c) == (1, 0, 0)):
            raise OracleError("US_ERR_UNSUPPORTED_DESC", "rank predicates group by row")
        rank, _ = _group_rank(r, c)
        if pred.kind == RANK_LT_ABS:
            K = pred.abs
        else:
            K = percentile_width(np.bincount(r, minlength=nrows), pred.num, pred.den)
        return rank < K
    raise OracleError("US_ERR_UNSUPPORTED_DESC", pred.kind)


def decompose(nrows, ncols, row, col, val, desc_a: FormatDesc, desc_b: FormatDesc, pred: Predicate):
    """Split into two COO lists by the predicate (stable), then convert each part.  Both
    parts keep the shape of the whole matrix."""
    row = np.asarray(row); col = np.asarray(col); val = np.asarray(val, dtype=np.float32)
    validate_coo(nrows, ncols, row, col, val)
    m = predicate_mask(nrows, ncols, row, col, pred)
    a = convert(nrows, ncols, row[m], col[m], val[m], desc_a)
    b = convert(nrows, ncols, row[~m], col[~m], val[~m], desc_b)
    return a, b, m


# --------------------------------------------------------------------------- SpMV / SpMM (float64)

def spmv_coo(nrows, ncols, row, col, val, x) -> np.ndarray:
    """y_i = sum_j A_ij x_j straight from the COO list."""
    w = np.asarray(val, dtype=np.float64) * np.asarray(x, dtype=np.float64)[np.asarray(col)]
    return np.bincount(np.asarray(row), weights=w, minlength=nrows).astype(np.float64)


def spmm_coo(nrows, ncols, row, col, val, X) -> np.ndarray:
    """Y_i: = sum_j A_ij X_j: straight from the COO list."""
    X = np.asarray(X, dtype=np.float64)
    Y = np.zeros((nrows, X.shape[1]), dtype=np.float64)
    np.add.at(Y, np.asarray(row), np.asarray(val, dtype=np.float64)[:, None] * X[np.asarray(col)])
    return Y


def spmv(f: Formatted, x, y0=None) -> np.ndarray:
    """y (+)= A x over the stored layout: every leaf, inverse map, bounds guard (Figure 9)."""
    r, c, leaf = leaves(f)
    w = f.val[leaf].astype(np.float64) * np.asarray(x, dtype=np.float64)[c]
    y = np.bincount(r, weights=w, minlength=f.nrows).astype(np.float64)
    return y if y0 is None else y + np.asarray(y0, dtype=np.float64)


def spmm(f: Formatted, X, Y0=None) -> np.ndarray:
    r, c, leaf = leaves(f)
    Y = spmm_coo(f.nrows, f.ncols, r, c, f.val[leaf], X)
    return Y if Y0 is None else Y + np.asarray(Y0, dtype=np.float64)


def abs_row_sums(nrows, row, col, val, x) -> np.ndarray:
    """sum_j |a_ij x_j| per row: the scale that bounds fp32 summation error."""
    w = np.abs(np.asarray(val, dtype=np.float64) * np.asarray(x, dtype=np.float64)[np.asarray(col)])
    return np.bincount(np.asarray(row), weights=w, minlength=nrows)
