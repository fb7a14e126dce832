"""More pins for the CPU oracle, each with planted mistakes that the pin has to catch: the scale of the product
tolerance (abs_row_sums), the CSB arrays of the paper's example, the capacity of row / column / diagonal groups,
and SpMM straight from the COO list."""
import numpy as np
import pytest

from oracle import unisparse_oracle as O


def random_coo(rng, nrows, ncols, nnz):
    lin = rng.choice(nrows * ncols, size=min(nnz, nrows * ncols), replace=False)
    row, col = (lin // ncols).astype(np.int32), (lin % ncols).astype(np.int32)
    val = rng.uniform(-1, 1, row.shape[0]).astype(np.float32)
    val[val == 0] = 0.5
    return row, col, val


# ------------------------------------------------------------------ abs_row_sums: S_i = sum_j |a_ij x_j|
def pin_abs_row_sums(fn):
    rng = np.random.default_rng(21)
    for nr, nc, nnz in ((1, 1, 1), (6, 5, 14), (9, 4, 30), (5, 7, 0)):
        r, c, v = random_coo(rng, nr, nc, nnz)
        x = rng.uniform(-2, 2, nc).astype(np.float32)
        want = [0.0] * nr
        for k in range(r.size):                      # one entry at a time, plain Python floats
            want[int(r[k])] += abs(float(v[k]) * float(x[int(c[k])]))
        got = fn(nr, r, c, v, x)
        assert got.shape == (nr,)
        np.testing.assert_allclose(got, want, rtol=1e-13, atol=0)


def test_abs_row_sums_brute_force():
    pin_abs_row_sums(O.abs_row_sums)


ABS_ROW_SUM_MUTANTS = {
    "no abs of x": lambda nr, r, c, v, x: np.bincount(r, weights=np.abs(v.astype(np.float64)) * x.astype(np.float64)[c], minlength=nr),
    "summed by column": lambda nr, r, c, v, x: np.bincount(c, weights=np.abs(v.astype(np.float64) * x.astype(np.float64)[c]), minlength=nr)[:nr],
    "x taken at the row": lambda nr, r, c, v, x: np.bincount(r, weights=np.abs(v.astype(np.float64) * np.resize(x.astype(np.float64), max(nr, x.size))[r]), minlength=nr),
    "scaled by the row count": lambda nr, r, c, v, x: O.abs_row_sums(nr, r, c, v, x) * nr,
    "last entry dropped": lambda nr, r, c, v, x: O.abs_row_sums(nr, r[:-1], c[:-1], v[:-1], x),
    "abs of the sum": lambda nr, r, c, v, x: np.abs(np.bincount(r, weights=v.astype(np.float64) * x.astype(np.float64)[c], minlength=nr)),
}


@pytest.mark.parametrize("name", sorted(ABS_ROW_SUM_MUTANTS))
def test_abs_row_sums_pin_catches(name):
    with pytest.raises(AssertionError):
        pin_abs_row_sums(ABS_ROW_SUM_MUTANTS[name])


# ------------------------------------------------------------------ CSB of the paper's example, by hand
# Matrix A (Section 4.2): entries (d0, d1, val) = (0,0,1) (1,1,2) (2,1,3) (2,2,4) (2,3,5) (4,3,6), 5 x 4.
# CSB with 2 x 2 blocks (Figure 7): index map (d0/2, d1/2, d0%2, d1%2), merge(1), trim(2,3).  Target tuples:
#   (0,0,0,0)=1  (0,0,1,1)=2  (1,0,0,1)=3  (1,1,0,0)=4  (1,1,0,1)=5  (2,1,0,1)=6      (already in sorted order)
# Section 5.1: levels 0 and 1 are not trimmed -> two sizes, ceil(5/2) = 3 and ceil(4/2) = 2, a dense grid of
# 6 blocks numbered e0*2 + e1; level 2 is trimmed and its parent level is merged -> ptr over the 6 blocks
# (7 entries, starting at 0) + idx (d0%2); level 3 is trimmed, its parent is not merged -> one idx (d1%2) per
# entry and no ptr.  Blocks 0..5 hold 2, 0, 1, 2, 0, 1 entries.
CSB_EXAMPLE = dict(size0=3, size1=2, ptr2=[0, 2, 2, 3, 5, 5, 6], idx2=[0, 1, 0, 0, 0, 0], idx3=[0, 1, 1, 0, 1, 1],
                   val=[1, 2, 3, 4, 5, 6])


def pin_csb_example(convert, example_A):
    r = np.array(example_A["d0"], np.int32); c = np.array(example_A["d1"], np.int32)
    v = np.array(example_A["val"], np.float32)
    for seed in range(3):
        p = np.random.default_rng(seed).permutation(r.size)
        f = convert(5, 4, r[p], c[p], v[p], O.CSB(2))
        assert [l.kind for l in f.levels] == ["dense", "dense", "compressed", "coordinate"]
        assert (f.levels[0].size, f.levels[1].size) == (CSB_EXAMPLE["size0"], CSB_EXAMPLE["size1"])
        assert f.levels[0].ptr is None and f.levels[0].idx is None and f.levels[1].ptr is None and f.levels[1].idx is None
        assert f.levels[2].ptr.tolist() == CSB_EXAMPLE["ptr2"]
        assert f.levels[2].idx.tolist() == CSB_EXAMPLE["idx2"]
        assert f.levels[3].ptr is None and f.levels[3].idx.tolist() == CSB_EXAMPLE["idx3"]
        assert f.val.tolist() == CSB_EXAMPLE["val"]


def test_csb_example_by_hand(example_A):
    pin_csb_example(O.convert, example_A)


def _mutated_convert(change):
    def convert(nr, nc, r, c, v, d):
        f = O.convert(nr, nc, r, c, v, d)
        change(f)
        return f
    return convert


def _swap_inner(f): f.levels[2].idx, f.levels[3].idx = f.levels[3].idx, f.levels[2].idx
def _ptr_over_stored_blocks(f): f.levels[2].ptr = np.concatenate(([0], np.unique(f.levels[2].ptr)[1:])).astype(np.int32)
def _ptr_without_origin(f): f.levels[2].ptr = f.levels[2].ptr[1:]
def _column_major_grid(f):   # blocks numbered e1*3 + e0 instead of e0*2 + e1
    cnt = np.diff(f.levels[2].ptr).reshape(3, 2).T.reshape(-1)
    f.levels[2].ptr = np.concatenate(([0], np.cumsum(cnt))).astype(np.int32)
def _sizes_swapped(f): f.levels[0].size, f.levels[1].size = f.levels[1].size, f.levels[0].size
def _ptr_on_level3(f): f.levels[3].ptr = np.arange(7, dtype=np.int32)


CSB_MUTANTS = {"in-block indices swapped": _swap_inner, "ptr over the stored blocks only": _ptr_over_stored_blocks,
               "ptr without its leading 0": _ptr_without_origin, "grid numbered column-major": _column_major_grid,
               "sizes swapped": _sizes_swapped, "a ptr on the last level": _ptr_on_level3}


@pytest.mark.parametrize("name", sorted(CSB_MUTANTS))
def test_csb_pin_catches(name, example_A):
    with pytest.raises(AssertionError):
        pin_csb_example(_mutated_convert(CSB_MUTANTS[name]), example_A)


def test_csb_spmv_and_dense_reconstruction_of_the_example(example_A):
    r = np.array(example_A["d0"], np.int32); c = np.array(example_A["d1"], np.int32)
    v = np.array(example_A["val"], np.float32)
    f = O.convert(5, 4, r, c, v, O.CSB(2))
    A = np.zeros((5, 4)); A[r, c] = v
    assert np.array_equal(O.to_dense(f), A)
    assert O.spmv(f, np.array([1, 10, 100, 1000.0])).tolist() == [1, 20, 5430, 0, 6000]


# ------------------------------------------------------------------ capacity of a group: rows, columns, diagonals
def pin_group_capacity(fn):
    for nr, nc in ((5, 4), (3, 8), (1, 6), (7, 1), (6, 6)):
        inside = [(i, j) for i in range(nr) for j in range(nc)]
        for group, key_of, keys in ((O.d0(), lambda i, j: i, range(nr)), (O.d1(), lambda i, j: j, range(nc)),
                                    (O.diag(), lambda i, j: j - i, range(-(nr - 1), nc))):
            ks = np.array(list(keys), dtype=np.int64)
            want = [sum(1 for (i, j) in inside if key_of(i, j) == k) for k in ks]   # count the positions one by one
            assert fn((group,), nr, nc, [ks]).tolist() == want, (nr, nc, group)


def test_group_capacity_all_branches_brute_force():
    pin_group_capacity(O.group_capacity)
    with pytest.raises(O.OracleError):
        O.group_capacity((O.Expr(O.AFFINE, 1, 1),), 4, 4, [np.arange(3)])


def _cap_rows_cols_swapped(group, nr, nc, key):
    g = group[0]
    if (g.c0, g.c1) == (1, 0): return np.full(key[0].shape, nr, dtype=np.int64)
    if (g.c0, g.c1) == (0, 1): return np.full(key[0].shape, nc, dtype=np.int64)
    return O.group_capacity(group, nr, nc, key)


def _cap_diag_full_length(group, nr, nc, key):
    g = group[0]
    if (g.c0, g.c1) == (-1, 1): return np.full(key[0].shape, min(nr, nc), dtype=np.int64)
    return O.group_capacity(group, nr, nc, key)


def _cap_diag_sign(group, nr, nc, key):
    g = group[0]
    if (g.c0, g.c1) == (-1, 1): return O.group_capacity(group, nr, nc, [-key[0]])
    return O.group_capacity(group, nr, nc, key)


@pytest.mark.parametrize("mutant", [_cap_rows_cols_swapped, _cap_diag_full_length, _cap_diag_sign],
                         ids=["rows and columns swapped", "diagonals never clipped", "diagonal sign"])
def test_group_capacity_pin_catches(mutant):
    with pytest.raises(AssertionError):
        pin_group_capacity(mutant)


# ------------------------------------------------------------------ SpMM from the COO list = dense matmul
def pin_spmm_coo(fn):
    rng = np.random.default_rng(22)
    for nr, nc, nnz, N in ((1, 1, 1, 1), (6, 5, 14, 3), (9, 4, 30, 7), (5, 7, 0, 2)):
        r, c, v = random_coo(rng, nr, nc, nnz)
        X = rng.uniform(-2, 2, (nc, N)).astype(np.float32)
        A = np.zeros((nr, nc)); A[r, c] = v
        want = [[sum(A[i, j] * float(X[j, k]) for j in range(nc)) for k in range(N)] for i in range(nr)]
        np.testing.assert_allclose(fn(nr, nc, r, c, v, X), np.array(want).reshape(nr, N), rtol=1e-12, atol=1e-15)


def test_spmm_coo_brute_force():
    pin_spmm_coo(O.spmm_coo)


SPMM_MUTANTS = {
    "X row taken at the matrix row": lambda nr, nc, r, c, v, X: O.spmm_coo(nr, nc, r, np.minimum(r, nc - 1), v, X),
    "transposed": lambda nr, nc, r, c, v, X: O.spmm_coo(nr, nc, np.minimum(c, nr - 1), np.minimum(r, nc - 1), v, X),
    "in fp32": lambda nr, nc, r, c, v, X: (O.spmm_coo(nr, nc, r, c, v, X).astype(np.float32) * np.float32(1 + 1e-6)).astype(np.float64),
    "a repeated row index counted once": lambda nr, nc, r, c, v, X: _last_write_wins(nr, r, c, v, X),
}


def _last_write_wins(nr, r, c, v, X):
    Y = np.zeros((nr, X.shape[1]))
    Y[r] += v.astype(np.float64)[:, None] * X.astype(np.float64)[c]    # fancy-index += drops repeated rows
    return Y


@pytest.mark.parametrize("name", sorted(SPMM_MUTANTS))
def test_spmm_coo_pin_catches(name):
    with pytest.raises(AssertionError):
        pin_spmm_coo(SPMM_MUTANTS[name])


# ------------------------------------------------------------------ blocked ELL (BELL), by hand and by plain loops
# Matrix A with 2 x 2 blocks.  Block rows: 0 = rows 0-1 holds block column 0 {(0,0)=1, (1,1)=2}; 1 = rows 2-3 holds
# block columns 0 {(2,1)=3} and 1 {(2,2)=4, (2,3)=5}; 2 = rows 4-5 holds block column 1 {(4,3)=6}.  The indirect level
# numbers the blocks of a block row by ascending block column, so K = 2 slots; levels (slot, block row) are sizes 2 and
# 3, the block-column level holds one index per (slot, block row), slot-major, -1 where a block row has no such block;
# values node-major, row-major inside a block (Section 5.1 and the value access of Figure 9).
BELL_EXAMPLE = dict(K=2, nbr=3, bcol=[0, 0, 1, -1, 1, -1],
                    val=[1, 0, 0, 2,  0, 3, 0, 0,  0, 6, 0, 0,  0, 0, 0, 0,  4, 5, 0, 0,  0, 0, 0, 0])


def pin_bell_example(convert, example_A):
    r = np.array(example_A["d0"], np.int32); c = np.array(example_A["d1"], np.int32)
    v = np.array(example_A["val"], np.float32)
    for seed in range(3):
        p = np.random.default_rng(seed).permutation(r.size)
        f = convert(5, 4, r[p], c[p], v[p], O.BELL(2))
        assert [l.kind for l in f.levels] == ["dense", "dense", "payload", "dense", "dense"]
        assert [f.levels[L].size for L in (0, 1, 3, 4)] == [BELL_EXAMPLE["K"], BELL_EXAMPLE["nbr"], 2, 2]
        assert f.levels[2].idx.tolist() == BELL_EXAMPLE["bcol"] and f.levels[2].ptr is None
        assert f.val.tolist() == BELL_EXAMPLE["val"]


def test_bell_example_by_hand(example_A):
    pin_bell_example(O.convert, example_A)
    r = np.array(example_A["d0"], np.int32); c = np.array(example_A["d1"], np.int32)
    v = np.array(example_A["val"], np.float32)
    f = O.convert(5, 4, r, c, v, O.BELL(2))
    A = np.zeros((5, 4)); A[r, c] = v
    assert np.array_equal(O.to_dense(f), A)
    assert O.spmv(f, np.array([1, 10, 100, 1000.0])).tolist() == [1, 20, 5430, 0, 6000]
    rr, cc, vv = O.to_coo(f)
    assert (rr.tolist(), cc.tolist(), vv.tolist()) == (example_A["d0"], example_A["d1"], example_A["val"])
    assert O.convert(5, 4, r, c, v, O.BELL(2, width=3)).levels[0].size == 3      # a fixed width pads further
    with pytest.raises(O.OracleError):
        O.convert(5, 4, r, c, v, O.BELL(2, width=1))                             # block row 1 holds two blocks


def _bell_slab_major_swapped(f):   # block-row-major instead of slot-major
    K, nbr = f.levels[0].size, f.levels[1].size
    f.levels[2].idx = f.levels[2].idx.reshape(K, nbr).T.reshape(-1).copy()
def _bell_rank_per_entry(f):       # slots numbered by entries instead of blocks: K grows to the longest row's entries
    f.levels[0].size = 3
def _bell_pad_zero(f): f.levels[2].idx = np.where(f.levels[2].idx < 0, 0, f.levels[2].idx)
def _bell_block_transposed(f): f.val = f.val.reshape(-1, 2, 2).transpose(0, 2, 1).reshape(-1).copy()


BELL_MUTANTS = {"block-row-major slab": _bell_slab_major_swapped, "one slot per entry": _bell_rank_per_entry,
                "pad block column 0": _bell_pad_zero, "blocks stored column-major": _bell_block_transposed}


@pytest.mark.parametrize("name", sorted(BELL_MUTANTS))
def test_bell_pin_catches(name, example_A):
    with pytest.raises(AssertionError):
        pin_bell_example(_mutated_convert(BELL_MUTANTS[name]), example_A)


@pytest.mark.parametrize("seed", range(6))
def test_bell_brute_force(seed):
    rng = np.random.default_rng(100 + seed)
    nr, nc = int(rng.integers(1, 30)), int(rng.integers(1, 30))
    bh, bw = int(rng.integers(1, 5)), int(rng.integers(1, 5))
    r, c, v = random_coo(rng, nr, nc, int(rng.integers(0, nr * nc // 2 + 1)))
    f = O.convert(nr, nc, r, c, v, O.BELL(bh, bw))
    nbr = -(-nr // bh)
    blocks = [sorted({int(cc) // bw for rr, cc in zip(r, c) if int(rr) // bh == br}) for br in range(nbr)]
    K = max((len(b) for b in blocks), default=0)
    assert [f.levels[L].size for L in (0, 1, 3, 4)] == [K, nbr, bh, bw]
    bcol = [[-1] * nbr for _ in range(K)]
    val = np.zeros((K, nbr, bh, bw), np.float32)
    for br in range(nbr):
        for k, bc in enumerate(blocks[br]):
            bcol[k][br] = bc
    for rr, cc, vv in zip(r, c, v):
        br, bc = int(rr) // bh, int(cc) // bw
        val[blocks[br].index(bc), br, int(rr) % bh, int(cc) % bw] = vv
    assert f.levels[2].idx.tolist() == [x for row in bcol for x in row]
    assert np.array_equal(f.val, val.reshape(-1))
    A = np.zeros((nr, nc)); A[r, c] = v
    assert np.array_equal(O.to_dense(f), A)
    x = rng.uniform(-1, 1, nc)
    np.testing.assert_allclose(O.spmv(f, x), A @ x, atol=1e-12)
