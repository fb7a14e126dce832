"""Pins for the CPU oracle: the paper's worked example, library routines that special
cases reduce to (scipy CSR/CSC/BSR/DIA), brute force on tiny inputs, invariants."""
import itertools

import numpy as np
import pytest
import scipy.sparse as sp

from oracle import unisparse_oracle as O

ALL_FORMATS = [
    ("COO", O.COO()), ("CSR", O.CSR()), ("DCSR", O.DCSR()), ("CSC", O.CSC()), ("DCSC", O.DCSC()),
    ("DIA", O.DIA()), ("DIAv", O.DIA_VARIANT()), ("BCSR2", O.BCSR(2)), ("BCSR4", O.BCSR(4)),
    ("BCSR2x3", O.BCSR(2, 3)), ("CSB2", O.CSB(2)), ("ELL", O.ELL()), ("BDIA3", O.BDIA(3)),
    ("CISRplus3", O.CISR_PLUS(3)),
]


def random_coo(rng, nrows, ncols, nnz):
    lin = rng.choice(nrows * ncols, size=min(nnz, nrows * ncols), replace=False)
    row, col = (lin // ncols).astype(np.int32), (lin % ncols).astype(np.int32)
    val = rng.uniform(-1, 1, row.shape[0]).astype(np.float32)
    val[val == 0] = 0.5
    return row, col, val


def dense_of(nrows, ncols, row, col, val):
    A = np.zeros((nrows, ncols))
    A[row, col] = val
    return A


# ------------------------------------------------------------------ the paper's example (Section 4.2)

def shuffled_A(example_A, seed=0):
    r = np.array(example_A["d0"], np.int32)
    c = np.array(example_A["d1"], np.int32)
    v = np.array(example_A["val"], np.float32)
    p = np.random.default_rng(seed).permutation(r.size)
    return example_A["nrows"][0], example_A["ncols"][0], r[p], c[p], v[p]


def test_example_coo_is_the_printed_traversal(example_A):
    nr, nc, r, c, v = shuffled_A(example_A)
    f = O.convert(nr, nc, r, c, v, O.COO())
    assert f.levels[0].idx.tolist() == example_A["d0"]
    assert f.levels[1].idx.tolist() == example_A["d1"]
    assert f.val.tolist() == example_A["val"]
    assert f.levels[0].ptr is None and f.levels[1].ptr is None
    # the DOK (packed) form printed in the paper is the same triples zipped
    trip = list(zip(f.levels[0].idx.tolist(), f.levels[1].idx.tolist(), f.val.astype(int).tolist()))
    assert list(trip[0]) == example_A["dok_first"]
    assert list(trip[1]) == example_A["dok_second"]
    assert list(trip[-1]) == example_A["dok_last"]


def test_example_trim_keeps_or_removes_the_empty_row(example_A):
    # trim(1,1) leaves the dangling row-3 node, trim(0,1) removes it (Section 4.1.3)
    nr, nc, r, c, v = shuffled_A(example_A, 1)
    csr = O.convert(nr, nc, r, c, v, O.CSR())
    assert csr.levels[0].kind == "dense" and csr.levels[0].size == 5
    assert csr.levels[1].ptr.tolist() == [0, 1, 2, 5, 5, 6]      # hand-derived: row 3 repeats
    assert csr.levels[1].idx.tolist() == [0, 1, 1, 2, 3, 3]
    dcsr = O.convert(nr, nc, r, c, v, O.DCSR())
    assert dcsr.levels[0].idx.tolist() == [0, 1, 2, 4] and dcsr.levels[0].ptr is None
    assert dcsr.levels[1].ptr.tolist() == [0, 1, 2, 5, 6]
    assert dcsr.levels[1].idx.tolist() == [0, 1, 1, 2, 3, 3]
    assert csr.val.tolist() == dcsr.val.tolist() == [1, 2, 3, 4, 5, 6]


def test_example_dia_padding_sizes(example_A):
    # arrays hand-derived from the Section 5.1 rules applied to the printed COO
    nr, nc, r, c, v = shuffled_A(example_A, 2)
    dia = O.convert(nr, nc, r, c, v, O.DIA())
    assert dia.levels[0].idx.tolist() == [-1, 0, 1]
    assert dia.levels[1].size == example_A["dia_slots_per_diagonal"][0]
    assert dia.val.reshape(3, 5).tolist() == [[0, 0, 3, 0, 6], [1, 2, 4, 0, 0], [0, 0, 5, 0, 0]]
    diav = O.convert(nr, nc, r, c, v, O.DIA_VARIANT())
    assert diav.levels[1].size == example_A["dia_variant_slots_per_diagonal"][0]
    assert diav.val.reshape(3, 4).tolist() == [[0, 3, 0, 6], [1, 2, 4, 0], [0, 0, 0, 5]]


def test_example_blocked_and_ell(example_A):
    nr, nc, r, c, v = shuffled_A(example_A, 3)
    b = O.convert(nr, nc, r, c, v, O.BCSR(2))
    assert [l.kind for l in b.levels] == ["dense", "compressed", "dense", "dense"]
    assert b.levels[0].size == 3                              # 5 rows, b=2: ceil
    assert b.levels[1].ptr.tolist() == [0, 1, 3, 4]
    assert b.levels[1].idx.tolist() == [0, 0, 1, 1]
    assert b.val.reshape(4, 4).tolist() == [[1, 0, 0, 2], [0, 3, 0, 0], [4, 5, 0, 0], [0, 6, 0, 0]]
    e = O.convert(nr, nc, r, c, v, O.ELL())
    assert e.levels[0].size == 3 and e.levels[1].size == 5
    P = -1
    assert e.levels[2].idx.reshape(3, 5).tolist() == [[0, 1, 1, P, 3], [P, P, 2, P, P], [P, P, 3, P, P]]
    assert e.val.reshape(3, 5).tolist() == [[1, 2, 3, 0, 6], [0, 0, 4, 0, 0], [0, 0, 5, 0, 0]]
    # BDIA with block 3 (the program of Figure 3c; Figure 9 reads val[node*size_2 + id2])
    d = O.convert(nr, nc, r, c, v, O.BDIA(3))
    assert d.levels[0].size == 2 and d.levels[2].size == 3
    assert d.levels[1].ptr.tolist() == [0, 3, 4] and d.levels[1].idx.tolist() == [-1, 0, 1, -1]
    assert d.val.reshape(4, 3).tolist() == [[0, 0, 3], [1, 2, 4], [0, 0, 5], [0, 6, 0]]


def test_example_spmv_all_formats(example_A):
    nr, nc, r, c, v = shuffled_A(example_A, 4)
    for name, d in ALL_FORMATS:
        f = O.convert(nr, nc, r, c, v, d)
        assert O.spmv(f, np.ones(4)).tolist() == [1, 2, 12, 0, 6], name


# ------------------------------------------------------------------ library special cases

@pytest.mark.parametrize("shape", [(7, 5), (16, 16), (33, 50), (1, 9), (9, 1)])
def test_csr_csc_equal_scipy(shape):
    rng = np.random.default_rng(10)
    nr, nc = shape
    r, c, v = random_coo(rng, nr, nc, nr * nc // 3 + 1)
    S = sp.coo_matrix((v, (r, c)), shape=shape)
    csr = S.tocsr(); csr.sort_indices()
    f = O.convert(nr, nc, r, c, v, O.CSR())
    assert np.array_equal(f.levels[1].ptr, csr.indptr) and np.array_equal(f.levels[1].idx, csr.indices)
    assert np.array_equal(f.val, csr.data)
    csc = S.tocsc(); csc.sort_indices()
    g = O.convert(nr, nc, r, c, v, O.CSC())
    assert g.levels[0].size == nc
    assert np.array_equal(g.levels[1].ptr, csc.indptr) and np.array_equal(g.levels[1].idx, csc.indices)
    assert np.array_equal(g.val, csc.data)


@pytest.mark.parametrize("shape,blk", [((8, 8), (2, 2)), ((16, 12), (4, 4)), ((12, 18), (2, 3)), ((24, 24), (8, 8))])
def test_bcsr_equals_scipy_bsr(shape, blk):
    rng = np.random.default_rng(11)
    nr, nc = shape
    r, c, v = random_coo(rng, nr, nc, nr * nc // 4)
    bsr = sp.coo_matrix((v, (r, c)), shape=shape).tocsr().tobsr(blocksize=blk)
    bsr.sort_indices()
    f = O.convert(nr, nc, r, c, v, O.BCSR(*blk))
    assert np.array_equal(f.levels[1].ptr, bsr.indptr)
    assert np.array_equal(f.levels[1].idx, bsr.indices)
    assert np.array_equal(f.val, bsr.data.reshape(-1))   # (nblk, bh, bw) row-major


@pytest.mark.parametrize("shape", [(9, 6), (6, 9), (12, 12)])
def test_dia_variant_equals_scipy_dia_and_dia_is_its_transpose(shape):
    rng = np.random.default_rng(12)
    nr, nc = shape
    r, c, v = random_coo(rng, nr, nc, nr * nc // 3)
    S = sp.coo_matrix((v, (r, c)), shape=shape)
    dia = S.todia()                                  # data[k, j] = A[j - off_k, j]: column-indexed
    order = np.argsort(dia.offsets)
    f = O.convert(nr, nc, r, c, v, O.DIA_VARIANT())
    assert np.array_equal(f.levels[0].idx, dia.offsets[order])
    assert np.array_equal(f.val.reshape(-1, nc), dia.data[order][:, :nc].astype(np.float32))
    # row-indexed DIA of A = column-indexed DIA of A^T with negated offsets
    diaT = S.T.todia()
    orderT = np.argsort(-diaT.offsets)
    g = O.convert(nr, nc, r, c, v, O.DIA())
    assert np.array_equal(g.levels[0].idx, -diaT.offsets[orderT])
    assert np.array_equal(g.val.reshape(-1, nr), diaT.data[orderT][:, :nr].astype(np.float32))


# ------------------------------------------------------------------ brute force / invariants

def brute_ell(nr, nc, A):
    rows = [[j for j in range(nc) if A[i, j] != 0] for i in range(nr)]
    K = max((len(x) for x in rows), default=0)
    col = -np.ones((K, nr), np.int64); val = np.zeros((K, nr))
    for i, js in enumerate(rows):
        for k, j in enumerate(js):
            col[k, i] = j; val[k, i] = A[i, j]
    return K, col, val


@pytest.mark.parametrize("seed", range(4))
def test_ell_brute_force(seed):
    rng = np.random.default_rng(20 + seed)
    nr, nc = int(rng.integers(1, 12)), int(rng.integers(1, 12))
    r, c, v = random_coo(rng, nr, nc, int(rng.integers(1, nr * nc + 1)))
    A = dense_of(nr, nc, r, c, v)
    K, col, val = brute_ell(nr, nc, A)
    f = O.convert(nr, nc, r, c, v, O.ELL())
    assert f.levels[0].size == K and f.levels[1].size == nr
    assert np.array_equal(f.levels[2].idx.reshape(K, nr), col)
    assert np.array_equal(f.val.reshape(K, nr), val.astype(np.float32))
    # fixed width wider than needed pads; narrower is an error
    g = O.convert(nr, nc, r, c, v, O.ELL(K + 2))
    assert g.levels[0].size == K + 2 and np.all(g.levels[2].idx.reshape(K + 2, nr)[K:] == -1)
    if K > 1:
        with pytest.raises(O.OracleError):
            O.convert(nr, nc, r, c, v, O.ELL(K - 1))


@pytest.mark.parametrize("seed", range(6))
def test_roundtrip_dense_and_matvec(seed):
    rng = np.random.default_rng(30 + seed)
    nr, nc = int(rng.integers(1, 20)), int(rng.integers(1, 20))
    r, c, v = random_coo(rng, nr, nc, int(rng.integers(0, nr * nc + 1)))
    A = dense_of(nr, nc, r, c, v)
    x = rng.uniform(-1, 1, nc)
    X = rng.uniform(-1, 1, (nc, 3))
    order = np.lexsort((c, r))
    for name, d in ALL_FORMATS:
        f = O.convert(nr, nc, r, c, v, d)
        assert f.nnz == r.size
        rr, cc, vv = O.to_coo(f)
        assert np.array_equal(rr, r[order]) and np.array_equal(cc, c[order]) and np.array_equal(vv, v[order]), name
        assert np.array_equal(O.to_dense(f), A.astype(np.float32).astype(np.float64)), name
        np.testing.assert_allclose(O.spmv(f, x), A @ x, rtol=0, atol=1e-12, err_msg=name)
        np.testing.assert_allclose(O.spmm(f, X), A @ X, rtol=0, atol=1e-12, err_msg=name)
    np.testing.assert_allclose(O.spmv_coo(nr, nc, r, c, v, x), A @ x, rtol=0, atol=1e-12)
    np.testing.assert_allclose(O.spmm_coo(nr, nc, r, c, v, X), A @ X, rtol=0, atol=1e-12)
    np.testing.assert_allclose(O.spmv_coo(nr, nc, r, c, v, np.ones(nc)), A.sum(1), rtol=0, atol=1e-12)


def test_structural_invariants_medium():
    rng = np.random.default_rng(40)
    nr, nc = 300, 257
    r, c, v = random_coo(rng, nr, nc, 5000)
    counts = np.bincount(r, minlength=nr)
    csr = O.convert(nr, nc, r, c, v, O.CSR())
    ptr, idx = csr.levels[1].ptr, csr.levels[1].idx
    assert ptr[0] == 0 and ptr[-1] == r.size and np.all(np.diff(ptr) == counts)
    for i in range(nr):
        assert np.all(np.diff(idx[ptr[i]:ptr[i + 1]]) > 0)
    dcsr = O.convert(nr, nc, r, c, v, O.DCSR())
    assert np.array_equal(dcsr.levels[0].idx, np.flatnonzero(counts))
    assert np.array_equal(np.diff(dcsr.levels[1].ptr), counts[counts > 0])
    b = O.convert(nr, nc, r, c, v, O.BCSR(4))
    assert b.levels[0].size == 75 and b.levels[1].ptr.shape[0] == 76
    assert np.count_nonzero(b.val) == r.size
    e = O.convert(nr, nc, r, c, v, O.ELL())
    assert e.levels[0].size == counts.max()
    assert np.count_nonzero(e.levels[2].idx >= 0) == r.size
    assert np.all(e.val[e.levels[2].idx < 0] == 0)


def test_errors():
    r = np.array([0, 1, 1], np.int32); c = np.array([0, 2, 2], np.int32); v = np.ones(3, np.float32)
    with pytest.raises(O.OracleError) as ei:
        O.convert(3, 3, r, c, v, O.CSR())
    assert ei.value.code == "US_ERR_DUPLICATE"
    with pytest.raises(O.OracleError) as ei:
        O.convert(3, 2, r[:2], c[:2], v[:2], O.CSR())
    assert ei.value.code == "US_ERR_INDEX_RANGE"
    with pytest.raises(O.OracleError):
        O.convert(0, 2, r[:0], c[:0], v[:0], O.CSR())
    f = O.convert(3, 3, r[:0], c[:0], v[:0], O.CSR())           # empty matrix is fine
    assert f.levels[1].ptr.tolist() == [0, 0, 0, 0] and f.val.size == 0
    d = O.convert(3, 3, r[:0], c[:0], v[:0], O.DIA())
    assert d.levels[0].idx.size == 0 and d.val.size == 0


# ------------------------------------------------------------------ decompose

def test_capacity_brute_force():
    for nr, nc in [(5, 4), (4, 7), (6, 6), (1, 3)]:
        ks = np.arange(-(nr - 1), nc)
        cap = O.group_capacity((O.diag(),), nr, nc, [ks])
        brute = [sum(1 for i in range(nr) if 0 <= i + k < nc) for k in ks]
        assert cap.tolist() == brute


def test_percentile_width_closed_forms():
    L = np.array([5, 1, 3, 2, 4, 0, 9, 7, 8, 6])
    assert O.percentile_width(L, 9, 10) == 8       # nearest rank: ceil(.9*10)=9th smallest
    assert O.percentile_width(L, 1, 2) == 4
    assert O.percentile_width(L, 1, 1) == 9
    assert O.percentile_width(np.array([3]), 9, 10) == 3
    assert O.percentile_width(np.array([0, 0, 0, 7]), 3, 4) == 0


@pytest.mark.parametrize("seed", range(4))
def test_decompose_dia_csr_brute_force(seed):
    rng = np.random.default_rng(50 + seed)
    n = 24
    rows, cols = [], []
    for off in (-3, 0, 2):
        i = np.arange(max(0, -off), min(n, n - off))
        keep = rng.random(i.size) < 0.95
        rows.append(i[keep]); cols.append(i[keep] + off)
    er, ec, _ = random_coo(rng, n, n, 30)
    key = set(zip(np.concatenate(rows).tolist(), np.concatenate(cols).tolist()))
    extra = [(a, b) for a, b in zip(er.tolist(), ec.tolist()) if (a, b) not in key]
    r = np.concatenate(rows + [np.array([a for a, _ in extra], int)]).astype(np.int32)
    c = np.concatenate(cols + [np.array([b for _, b in extra], int)]).astype(np.int32)
    p = rng.permutation(r.size); r, c = r[p], c[p]
    v = rng.uniform(0.1, 1, r.size).astype(np.float32)
    pred = O.Predicate((O.diag(),), O.SUM_GE_FRAC_OF_CAPACITY, num=9, den=10)
    a, b, m = O.decompose(n, n, r, c, v, O.DIA(), O.CSR(), pred)
    # brute force predicate
    for t in range(r.size):
        k = int(c[t]) - int(r[t])
        cnt = sum(1 for u in range(r.size) if int(c[u]) - int(r[u]) == k)
        cap = sum(1 for i in range(n) if 0 <= i + k < n)
        assert bool(m[t]) == (10 * cnt >= 9 * cap)
    assert a.nnz + b.nnz == r.size
    A = dense_of(n, n, r, c, v).astype(np.float32).astype(np.float64)
    assert np.array_equal(O.to_dense(a) + O.to_dense(b), A)
    assert np.count_nonzero(O.to_dense(a) * O.to_dense(b)) == 0
    x = rng.uniform(-1, 1, n)
    np.testing.assert_allclose(O.spmv(b, x, O.spmv(a, x)), A @ x, atol=1e-12)


@pytest.mark.parametrize("seed", range(4))
def test_decompose_ell_coo_brute_force(seed):
    rng = np.random.default_rng(60 + seed)
    nr, nc = 40, 30
    r, c, v = random_coo(rng, nr, nc, 200)
    heavy = rng.integers(0, nr, 3)
    extra = [(int(h), j) for h in heavy for j in range(nc)]
    have = set(zip(r.tolist(), c.tolist()))
    extra = [e for e in dict.fromkeys(extra) if e not in have]
    r = np.concatenate([r, np.array([a for a, _ in extra], np.int32)])
    c = np.concatenate([c, np.array([b for _, b in extra], np.int32)])
    v = np.concatenate([v, rng.uniform(0.1, 1, len(extra)).astype(np.float32)])
    p = rng.permutation(r.size); r, c, v = r[p], c[p], v[p]
    lens = np.bincount(r, minlength=nr)
    K = int(np.sort(lens)[int(np.ceil(0.9 * nr)) - 1])
    pred = O.Predicate((O.d0(),), O.RANK_LT_PERCENTILE, num=9, den=10)
    a, b, m = O.decompose(nr, nc, r, c, v, O.ELL(), O.COO(), pred)
    for t in range(r.size):   # brute-force rank: entries of the same row with a smaller column
        rank = sum(1 for u in range(r.size) if r[u] == r[t] and c[u] < c[t])
        assert bool(m[t]) == (rank < K)
    assert a.levels[0].size == min(K, lens.max())
    assert a.nnz == int(np.minimum(lens, K).sum()) and b.nnz == r.size - a.nnz
    A = dense_of(nr, nc, r, c, v).astype(np.float32).astype(np.float64)
    assert np.array_equal(O.to_dense(a) + O.to_dense(b), A)
    X = rng.uniform(-1, 1, (nc, 4))
    np.testing.assert_allclose(O.spmm(b, X, O.spmm(a, X)), A @ X, atol=1e-12)
    # absolute-threshold variants
    m2 = O.predicate_mask(nr, nc, r, c, O.Predicate((O.d0(),), O.RANK_LT_ABS, abs=2))
    assert m2.sum() == np.minimum(lens, 2).sum()
    m3 = O.predicate_mask(nr, nc, r, c, O.Predicate((O.d0(),), O.SUM_GE_ABS, abs=10))
    assert np.array_equal(m3, lens[r] >= 10)


@pytest.mark.parametrize("seed", range(4))
def test_decompose_blocked_groups_brute_force(seed):
    """#sum over (d0/b, d1-d0) (the BDIA/CSR program of Figure 3c) and over blocks (d0/bh, d1/bw) (the per-block
    threshold of the BELL/COO case study): per-entry group counts recomputed with plain loops; BDIA slots
    addressed as Figure 9 does (val[node*b + d0%b], d0 = e0*b + e2, d1 = e1 + d0)."""
    rng = np.random.default_rng(70 + seed)
    nr, nc = 29, 31
    r, c, v = random_coo(rng, nr, nc, 260)
    b = [2, 3, 4, 5][seed]
    thld = [2, 3, 2, 4][seed]
    pred = O.Predicate((O.div(0, b), O.diag()), O.SUM_GE_ABS, abs=thld)
    pa, pb, m = O.decompose(nr, nc, r, c, v, O.BDIA(b), O.CSR(), pred)
    for t in range(r.size):
        cnt = sum(1 for u in range(r.size) if r[u] // b == r[t] // b and c[u] - r[u] == c[t] - r[t])
        assert bool(m[t]) == (cnt >= thld)
    A = dense_of(nr, nc, r, c, v).astype(np.float32).astype(np.float64)
    assert np.array_equal(O.to_dense(pa) + O.to_dense(pb), A)
    # walk the BDIA arrays by hand
    size0, ptr, idx, size2 = pa.levels[0].size, pa.levels[1].ptr, pa.levels[1].idx, pa.levels[2].size
    assert size0 == -(-nr // b) and size2 == b and ptr[0] == 0 and ptr[-1] == idx.size and pa.val.size == idx.size * b
    D = np.zeros((nr, nc))
    for e0 in range(size0):
        offs = idx[ptr[e0]:ptr[e0 + 1]]
        assert np.all(np.diff(offs) > 0)                      # diagonals of a block row ascend, no repeats
        for node in range(ptr[e0], ptr[e0 + 1]):
            seen = 0
            for e2 in range(b):
                d0 = e0 * b + e2
                d1 = int(idx[node]) + d0
                x = pa.val[node * b + e2]
                if 0 <= d0 < nr and 0 <= d1 < nc:
                    D[d0, d1] = x
                    seen += x != 0
                else:
                    assert x == 0                              # slots outside the matrix are padding
            assert seen >= thld                                # only groups that met the threshold are stored
    assert np.array_equal(D, O.to_dense(pa))
    # blocks
    bh, bw = [2, 3, 4, 2][seed], [2, 2, 4, 5][seed]
    pred = O.Predicate((O.div(0, bh), O.div(1, bw)), O.SUM_GE_ABS, abs=thld)
    qa, qb, m = O.decompose(nr, nc, r, c, v, O.BCSR(bh, bw), O.COO(), pred)
    for t in range(r.size):
        cnt = sum(1 for u in range(r.size) if r[u] // bh == r[t] // bh and c[u] // bw == c[t] // bw)
        assert bool(m[t]) == (cnt >= thld)
    assert np.array_equal(O.to_dense(qa) + O.to_dense(qb), A)
    assert qa.val.size % (bh * bw) == 0 and qa.nnz + qb.nnz == r.size


# ------------------------------------------------------------------ CISR-plus (Section 7.2.4): sum, reorder, schedule
def brute_cisr_plus(nr, A, nparts):
    """Plain loops: rows with entries, most entries first (ties: lower row first), dealt to the partitions
    in turn; inside a partition rows ascending, inside a row columns ascending."""
    lens = [(int(np.count_nonzero(A[i])), i) for i in range(nr)]
    order = sorted([t for t in lens if t[0] > 0], key=lambda t: (-t[0], t[1]))
    parts = [[] for _ in range(nparts)]
    for k, (_, i) in enumerate(order):
        parts[k % nparts].append(i)
    ptr1, rows, ptr2, cols, vals = [0], [], [0], [], []
    for p in parts:
        for i in sorted(p):
            rows.append(i)
            for j in np.flatnonzero(A[i]):
                cols.append(int(j)); vals.append(A[i, j])
            ptr2.append(len(cols))
        ptr1.append(len(rows))
    return ptr1, rows, ptr2, cols, vals, parts


@pytest.mark.parametrize("seed", range(6))
def test_cisr_plus_brute_force(seed):
    rng = np.random.default_rng(100 + seed)
    nr, nc = int(rng.integers(1, 40)), int(rng.integers(1, 30))
    row, col, val = random_coo(rng, nr, nc, int(rng.integers(0, nr * nc // 2 + 1)))
    if seed % 2 == 0 and row.size:   # skew: pile extra entries into two rows
        extra = [(int(r0), j) for r0 in rng.choice(nr, size=min(2, nr), replace=False) for j in range(nc)]
        have = set(zip(row.tolist(), col.tolist()))
        extra = [e for e in extra if e not in have]
        row = np.concatenate([row, np.array([e[0] for e in extra], np.int32)])
        col = np.concatenate([col, np.array([e[1] for e in extra], np.int32)])
        val = np.concatenate([val, rng.uniform(0.5, 1, len(extra)).astype(np.float32)])
    A = dense_of(nr, nc, row, col, val)
    for nparts in (1, 2, 3, 7, 64):
        f = O.convert(nr, nc, row, col, val, O.CISR_PLUS(nparts))
        ptr1, rows, ptr2, cols, vals, parts = brute_cisr_plus(nr, A, nparts)
        assert [l.kind for l in f.levels] == ["dense", "compressed", "compressed"]
        assert f.levels[0].size == nparts
        assert f.levels[1].ptr.tolist() == ptr1 and f.levels[1].idx.tolist() == rows
        assert f.levels[2].ptr.tolist() == ptr2 and f.levels[2].idx.tolist() == cols
        assert np.array_equal(f.val, np.array(vals, np.float32))
        # what dealing a descending order guarantees: partition sizes differ by at most one row, and an
        # earlier partition never holds fewer entries than a later one
        nrows_p = [len(p) for p in parts]
        loads = [sum(int(np.count_nonzero(A[i])) for i in p) for p in parts]
        assert max(nrows_p) - min(nrows_p) <= 1
        assert all(loads[j] >= loads[j + 1] for j in range(nparts - 1))
        assert np.allclose(O.to_dense(f), A)
        x = rng.uniform(-1, 1, nc)
        assert np.allclose(O.spmv(f, x), A @ x)


def test_cisr_plus_with_one_partition_is_dcsr_under_a_root():
    rng = np.random.default_rng(5)
    row, col, val = random_coo(rng, 30, 20, 90)
    f = O.convert(30, 20, row, col, val, O.CISR_PLUS(1))
    d = O.convert(30, 20, row, col, val, O.DCSR())
    assert f.levels[1].ptr.tolist() == [0, d.levels[0].idx.size]
    assert np.array_equal(f.levels[1].idx, d.levels[0].idx)
    assert np.array_equal(f.levels[2].ptr, d.levels[1].ptr) and np.array_equal(f.levels[2].idx, d.levels[1].idx)
    assert np.array_equal(f.val, d.val)


def test_cisr_plus_on_the_example(example_A):
    """Matrix A with two partitions, by hand: rows by entries 2 (3 entries), then 0, 1, 4 (one each) ->
    partitions {2, 1} and {0, 4}; stored by ascending row inside a partition."""
    nr, nc, r, c, v = shuffled_A(example_A, 3)
    f = O.convert(nr, nc, r, c, v, O.CISR_PLUS(2))
    assert f.levels[0].size == 2
    assert f.levels[1].ptr.tolist() == [0, 2, 4] and f.levels[1].idx.tolist() == [1, 2, 0, 4]
    assert f.levels[2].ptr.tolist() == [0, 1, 4, 5, 6] and f.levels[2].idx.tolist() == [1, 1, 2, 3, 0, 3]
    assert f.val.tolist() == [2, 3, 4, 5, 1, 6]
