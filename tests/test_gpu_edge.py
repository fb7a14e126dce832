"""HIP library vs oracle: degenerate shapes of the method, determinism, empty parts."""
import numpy as np
import pytest
import torch

from oracle import unisparse_oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2403_05802_amd import binding as B
    return B.Context("cuda:0")


def roundtrip(ctx, nr, nc, r, c, v, descs):
    from paper_2403_05802_amd import binding as B
    from helpers import assert_same_layout, dev, us_desc_of
    for d in descs:
        o = O.convert(nr, nc, r, c, v, d)
        g = B.us_convert(ctx, nr, nc, dev(r), dev(c), dev(v), us_desc_of(d))
        assert_same_layout(g, o, str(d.levels))
        g.free()


def test_all_entries_in_one_row_and_one_column(ctx):
    """A row (column) longer than several sort tiles and SpMV tiles."""
    rng = np.random.default_rng(1)
    n = 70_000
    cols = rng.permutation(n)[:50_000].astype(np.int32)
    rows = np.full(cols.size, 12345, np.int32)
    v = rng.uniform(0.5, 1, cols.size).astype(np.float32)
    roundtrip(ctx, n, n, rows, cols, v, [O.CSR(), O.DCSR(), O.COO(), O.CSC(), O.BCSR(4)])
    roundtrip(ctx, n, n, cols, rows, v, [O.CSR(), O.DCSR(), O.CSC(), O.DCSC()])
    from paper_2403_05802_amd import binding as B
    from helpers import assert_product, dev, host, row_terms, us_desc_of
    x = rng.uniform(-1, 1, n).astype(np.float32)
    for d in (O.CSR(), O.DCSR(), O.COO()):
        g = B.us_convert(ctx, n, n, dev(rows), dev(cols), dev(v), us_desc_of(d))
        y = torch.empty(n, device="cuda")
        B.us_spmv(ctx, g, dev(x), y)
        assert_product(host(y), O.spmv_coo(n, n, rows, cols, v, x), O.abs_row_sums(n, rows, cols, v, x), row_terms(n, rows),
                       f"one row of {cols.size} entries, spmv {d}")
        X = rng.uniform(-1, 1, (n, 128)).astype(np.float32)
        Y = torch.empty(n, 128, device="cuda")
        B.us_spmm(ctx, g, dev(X), Y)
        ref = v.astype(np.float64) @ X[cols].astype(np.float64)
        got = host(Y[12345])
        assert_product(got, ref, np.abs(v).astype(np.float64) @ np.abs(X[cols]).astype(np.float64), float(cols.size),
                       f"one row of {cols.size} entries, spmm {d}")
        assert float(Y.abs().sum()) == pytest.approx(float(np.abs(got).sum()), rel=1e-5)   # other rows are zero
        g.free()


def test_single_full_diagonal_and_far_corners(ctx):
    n = 5000
    i = np.arange(n, dtype=np.int32)
    v = np.linspace(0.1, 1, n).astype(np.float32)
    roundtrip(ctx, n, n, i, i, v, [O.DIA(), O.DIA_VARIANT(), O.CSR(), O.ELL(), O.BCSR(8)])
    # two entries in opposite corners: offsets -(n-1) and +(n-1), almost all rows empty
    r = np.array([0, n - 1], np.int32); c = np.array([n - 1, 0], np.int32); w = np.array([2, 3], np.float32)
    roundtrip(ctx, n, n, r, c, w, [O.DIA(), O.DIA_VARIANT(), O.CSR(), O.DCSR(), O.ELL(), O.BCSR(2)])
    # non-square
    roundtrip(ctx, 40, 3000, np.array([0, 39, 7], np.int32), np.array([2999, 0, 7], np.int32),
              np.array([1, 2, 3], np.float32), [O.DIA(), O.DIA_VARIANT(), O.CSR(), O.CSC(), O.BCSR(4, 2)])


def test_duplicates_on_the_sort_free_dia_path(ctx):
    from paper_2403_05802_amd import binding as B
    from helpers import dev, us_desc_of, us_pred_of
    n = 3000
    i = np.arange(n, dtype=np.int32)
    r = np.concatenate([i, i[100:101]]); c = np.concatenate([i, i[100:101]])
    v = np.ones(r.size, np.float32)                       # identical duplicate: same slot, same value
    with pytest.raises(B.UnisparseError) as ei:
        B.us_convert(ctx, n, n, dev(r), dev(c), dev(v), us_desc_of(O.DIA()))
    assert ei.value.code == "US_ERR_DUPLICATE"
    pred = O.Predicate((O.diag(),), O.SUM_GE_FRAC_OF_CAPACITY, num=9, den=10)
    with pytest.raises(B.UnisparseError) as ei:
        B.us_decompose(ctx, n, n, dev(r), dev(c), dev(v), us_desc_of(O.DIA()), us_desc_of(O.CSR()), us_pred_of(pred))
    assert ei.value.code == "US_ERR_DUPLICATE"


def test_decompose_with_an_empty_part(ctx):
    from paper_2403_05802_amd import binding as B
    from helpers import assert_same_layout, dev, us_desc_of, us_pred_of
    rng = np.random.default_rng(3)
    n = 400
    lin = rng.choice(n * n, 3000, replace=False)
    r, c = (lin // n).astype(np.int32), (lin % n).astype(np.int32)
    v = rng.uniform(0.1, 1, r.size).astype(np.float32)
    cases = [
        (O.DIA(), O.CSR(), O.Predicate((O.diag(),), O.SUM_GE_ABS, abs=10 ** 6)),     # nothing goes to A
        (O.CSR(), O.COO(), O.Predicate((O.d0(),), O.SUM_GE_ABS, abs=0)),             # everything goes to A
        (O.ELL(), O.COO(), O.Predicate((O.d0(),), O.RANK_LT_ABS, abs=0)),            # K = 0
        (O.ELL(), O.CSR(), O.Predicate((O.d0(),), O.RANK_LT_PERCENTILE, num=1, den=1)),  # K = longest row
        (O.CSC(), O.DCSR(), O.Predicate((O.d1(),), O.SUM_GE_ABS, abs=9)),            # column groups
    ]
    for da, db, pred in cases:
        oa, ob, _ = O.decompose(n, n, r, c, v, da, db, pred)
        ga, gb = B.us_decompose(ctx, n, n, dev(r), dev(c), dev(v), us_desc_of(da), us_desc_of(db), us_pred_of(pred))
        assert_same_layout(ga, oa, f"A {pred.kind}")
        assert_same_layout(gb, ob, f"B {pred.kind}")


def test_results_are_reproducible_bit_for_bit(ctx):
    """Two runs of every path give identical bytes: the row-major layouts never add floats
    with atomics (only the column-major scatter forms do), integer atomics only count."""
    from paper_2403_05802_amd import binding as B
    from paper_2403_05802_amd import workloads as W
    from helpers import coo_to_dev, dev, us_desc_of, us_pred_of
    m = W.cfg5_powerlaw_local(n=40_000, target_nnz=800_000, max_len=6000)
    d = coo_to_dev(m)
    x = dev(W.dense_operand(5, m.ncols)); X = dev(W.dense_operand(5, (m.ncols, 128)))
    pred = us_pred_of(O.Predicate((O.d0(),), O.RANK_LT_PERCENTILE, num=9, den=10))

    def run():
        out = []
        for desc in (O.CSR(), O.DCSR(), O.BCSR(4), O.ELL(), O.COO()):
            g = B.us_convert(ctx, m.nrows, m.ncols, *d, us_desc_of(desc))
            y = torch.empty(m.nrows, device="cuda"); Y = torch.empty(m.nrows, 128, device="cuda")
            B.us_spmv(ctx, g, x, y); B.us_spmm(ctx, g, X, Y)
            out += [g.val().clone(), y, Y] + [t.clone() for L in range(g.desc.nlevels)
                                              for t in (g.ptr(L), g.idx(L)) if t is not None]
        ga, gb = B.us_decompose(ctx, m.nrows, m.ncols, *d, us_desc_of(O.ELL()), us_desc_of(O.COO()), pred)
        Y = torch.empty(m.nrows, 128, device="cuda")
        B.us_spmm(ctx, ga, X, Y); B.us_spmm(ctx, gb, X, Y, accumulate=True)
        out += [ga.val().clone(), gb.val().clone(), Y]
        return out

    a, b = run(), run()
    assert len(a) == len(b)
    for s, t in zip(a, b):
        assert s.dtype == t.dtype and torch.equal(s.view(torch.int32), t.view(torch.int32))


def test_dia_large_slab(ctx):
    """A slab larger than the L2s (5 diagonals of a 2^20 matrix): same arrays as the oracle, and
    the duplicate check of the sort-free path still fires."""
    from paper_2403_05802_amd import binding as B
    from paper_2403_05802_amd import workloads as W
    from helpers import assert_same_layout, coo_to_dev, dev, us_desc_of, us_pred_of
    m = W.cfg3_banded(n=1 << 20, offsets=(-300, -1, 0, 1, 70000), extra_frac=0.002, index=7)
    pred = O.Predicate((O.diag(),), O.SUM_GE_FRAC_OF_CAPACITY, num=9, den=10)
    oa, ob, _ = O.decompose(m.nrows, m.ncols, m.row, m.col, m.val, O.DIA(), O.DCSR(), pred)
    ga, gb = B.us_decompose(ctx, m.nrows, m.ncols, *coo_to_dev(m), us_desc_of(O.DIA()), us_desc_of(O.DCSR()),
                            us_pred_of(pred))
    assert_same_layout(ga, oa, "large DIA part")
    assert_same_layout(gb, ob, "DCSR remainder")
    r = np.concatenate([m.row, m.row[:1]]); c = np.concatenate([m.col, m.col[:1]]); v = np.concatenate([m.val, m.val[:1]])
    on_diag = np.isin(m.col[:1].astype(np.int64) - m.row[:1], (-300, -1, 0, 1, 70000))[0]
    with pytest.raises(B.UnisparseError) as ei:
        B.us_decompose(ctx, m.nrows, m.ncols, dev(r), dev(c), dev(v), us_desc_of(O.DIA()), us_desc_of(O.DCSR()),
                       us_pred_of(pred))
    assert ei.value.code == "US_ERR_DUPLICATE", on_diag


def test_dia_value_equal_to_the_empty_slot_pattern(ctx):
    """The sort-free DIA path tells occupied slots from empty ones by a NaN fill pattern; an input value
    that carries this very pattern makes the call fall back to its byte-map form: same arrays, bit for bit."""
    from paper_2403_05802_amd import binding as B
    from helpers import assert_same_layout, dev, us_desc_of, us_pred_of
    rng = np.random.default_rng(21)
    n = 3000
    rows, cols = [], []
    for off in (-5, 0, 2, 700):
        i = np.arange(max(0, -off), min(n, n - off))
        keep = rng.random(i.size) < 0.95
        rows.append(i[keep]); cols.append(i[keep] + off)
    r = np.concatenate(rows).astype(np.int32); c = np.concatenate(cols).astype(np.int32)
    p = rng.permutation(r.size); r, c = r[p], c[p]
    v = rng.uniform(0.1, 1, r.size).astype(np.float32)
    v[17] = np.array([0x7FC5A5A5], dtype=np.uint32).view(np.float32)[0]
    for desc in (O.DIA(), O.DIA_VARIANT()):
        g = B.us_convert(ctx, n, n, dev(r), dev(c), dev(v), us_desc_of(desc))
        assert_same_layout(g, O.convert(n, n, r, c, v, desc), "DIA with the pattern as a value")
    pred = O.Predicate((O.diag(),), O.SUM_GE_FRAC_OF_CAPACITY, num=9, den=10)
    oa, ob, _ = O.decompose(n, n, r, c, v, O.DIA(), O.CSR(), pred)
    ga, gb = B.us_decompose(ctx, n, n, dev(r), dev(c), dev(v), us_desc_of(O.DIA()), us_desc_of(O.CSR()), us_pred_of(pred))
    assert_same_layout(ga, oa, "A"); assert_same_layout(gb, ob, "B")
    # and a duplicate is still a duplicate on both forms
    r2 = np.append(r, r[3]); c2 = np.append(c, c[3])
    for vv in (np.append(v, np.float32(2)), np.append(np.where(np.isnan(v), np.float32(1), v), np.float32(2))):
        with pytest.raises(B.UnisparseError) as ei:
            B.us_convert(ctx, n, n, dev(r2), dev(c2), dev(vv), us_desc_of(O.DIA()))
        assert ei.value.code == "US_ERR_DUPLICATE"


def test_duplicate_cut_in_two_by_a_rank_split(ctx):
    """The two copies of a coordinate get ranks K-1 and K: each part alone looks clean."""
    from paper_2403_05802_amd import binding as B
    from helpers import dev, us_desc_of, us_pred_of
    rng = np.random.default_rng(5)
    n = 500
    lin = rng.choice(n * n, 4000, replace=False)
    r, c = (lin // n).astype(np.int32), (lin % n).astype(np.int32)
    keep = r != 5
    r = np.concatenate([r[keep], np.array([5, 5, 5, 5], np.int32)])
    c = np.concatenate([c[keep], np.array([1, 2, 3, 3], np.int32)])
    p = rng.permutation(r.size); r, c = r[p], c[p]
    v = rng.uniform(0.1, 1, r.size).astype(np.float32)
    pred = us_pred_of(O.Predicate((O.d0(),), O.RANK_LT_ABS, abs=3))
    for da, db in ((O.ELL(), O.COO()), (O.CSR(), O.DCSR()), (O.BCSR(4), O.CSC()), (O.COO(), O.BDIA(3))):
        with pytest.raises(B.UnisparseError) as ei:
            B.us_decompose(ctx, n, n, dev(r), dev(c), dev(v), us_desc_of(da), us_desc_of(db), pred)
        assert ei.value.code == "US_ERR_DUPLICATE", (da, db)


def test_row_pointers_over_runs_of_empty_rows(ctx):
    """The pointer pass walks the sorted entries and fills ptr wherever the row index steps: steps of every
    length (inside one thread, listed for the workgroup, more of them than the list holds) and the tail
    behind the last entry, with entries >= rows (one pass) and entries < rows (binary search per row)."""
    from paper_2403_05802_amd import binding as B
    from helpers import dev, us_desc_of
    rng = np.random.default_rng(11)
    # (a) 1024 consecutive entries each in a row of its own, 40 rows apart: > 256 long steps in one workgroup
    far = np.arange(1500, dtype=np.int64) * 40 + 7
    # (b) a dense head so that entries >= rows, with steps of 1..17 rows around the in-thread limit
    steps = np.concatenate([np.arange(1, 18), rng.integers(1, 18, 300)])
    mid = far[-1] + 1 + np.cumsum(steps)
    nrows = int(mid[-1]) + 5000                      # a long tail of empty rows behind the last entry
    head_r = np.repeat(np.arange(3, dtype=np.int64), nrows // 3 + 2)[: nrows + 10]
    head_c = np.concatenate([rng.permutation(nrows)[: (head_r == k).sum()] for k in range(3)])
    r = np.concatenate([head_r, far, mid]).astype(np.int32)
    c = np.concatenate([head_c, rng.integers(0, nrows, far.size + mid.size)]).astype(np.int32)
    keep = np.unique(r.astype(np.int64) * nrows + c, return_index=True)[1]
    r, c = r[keep], c[keep]
    p = rng.permutation(r.size); r, c = r[p], c[p]
    v = rng.uniform(0.5, 1, r.size).astype(np.float32)
    assert r.size >= nrows
    roundtrip(ctx, nrows, nrows, r, c, v, [O.CSR(), O.DCSR(), O.ELL(), O.CSC()])
    # the same rows with few entries: fewer entries than rows
    sel = r >= 3
    roundtrip(ctx, nrows, nrows, r[sel], c[sel], v[sel], [O.CSR(), O.DCSR(), O.CSC(), O.DCSC()])
    # equal neighbours that fall into different threads / workgroups of the pass
    for cut in (4, 1024, 4096 + 3):
        order = np.lexsort((c, r))
        a, b = order[cut - 1], order[cut]             # neighbours in sorted order: make them equal
        rr2, cc2 = r.copy(), c.copy()
        rr2[b], cc2[b] = rr2[a], cc2[a]
        with pytest.raises(B.UnisparseError) as ei:
            B.us_convert(ctx, nrows, nrows, dev(rr2), dev(cc2), dev(v), us_desc_of(O.CSR()))
        assert ei.value.code == "US_ERR_DUPLICATE"


def test_hypersparse_dcsr_array_counts(ctx):
    """Stored-row arrays are allocated before their count is known; what the handle reports is the count."""
    from paper_2403_05802_amd import binding as B
    from helpers import dev, us_desc_of
    n = 3_000_000
    r = np.array([5, 5, 2_999_999, 17, 17, 17], np.int32)
    c = np.array([1, 0, 2_999_999, 9, 3, 4], np.int32)
    v = np.arange(1, 7, dtype=np.float32)
    g = B.us_convert(ctx, n, n, dev(r), dev(c), dev(v), us_desc_of(O.DCSR()))
    assert g.idx(0).cpu().tolist() == [5, 17, 2_999_999]
    assert g.ptr(1).cpu().tolist() == [0, 2, 5, 6]
    assert g.idx(1).cpu().tolist() == [0, 1, 3, 4, 9, 2_999_999]
    x = torch.ones(n, device="cuda"); y = torch.empty(n, device="cuda")
    B.us_spmv(ctx, g, x, y)
    assert float(y[5]) == 3.0 and float(y[17]) == 15.0 and float(y[2_999_999]) == 3.0 and float(y.sum()) == 21.0
    g.free()
    roundtrip(ctx, n, n, r, c, v, [O.DCSR(), O.CSR(), O.DCSC()])


@pytest.mark.parametrize("shift", [(1, 0, 0), (0, 2, 0), (0, 0, 3), (1, 2, 3)], ids=["row", "col", "val", "all"])
def test_coordinate_arrays_that_are_not_16_byte_aligned(ctx, shift):
    """The first pass of the sort reads four entries per load when the caller's arrays are 16-byte aligned; arrays
    that start 4, 8 or 12 bytes into an allocation take the one-entry loads and must give the same layouts."""
    from paper_2403_05802_amd import binding as B
    from helpers import assert_same_layout, dev, us_desc_of
    rng = np.random.default_rng(11)
    nr, nc, n = 3000, 2500, 4096 * 3 + 517        # several full tiles and a ragged one
    lin = rng.choice(nr * nc, size=n, replace=False)
    r, c = (lin // nc).astype(np.int32), (lin % nc).astype(np.int32)
    v = rng.uniform(0.1, 1, n).astype(np.float32)
    pad = lambda a, k: dev(np.concatenate([np.zeros(k, a.dtype), a]))[k:]
    rd, cd, vd = pad(r, shift[0]), pad(c, shift[1]), pad(v, shift[2])
    assert rd.data_ptr() % 16 == 4 * shift[0] and cd.data_ptr() % 16 == 4 * shift[1] and vd.data_ptr() % 16 == 4 * shift[2]
    for d in (O.CSR(), O.CSC(), O.BCSR(4), O.BDIA(4), O.ELL()):
        g = B.us_convert(ctx, nr, nc, rd, cd, vd, us_desc_of(d))
        assert_same_layout(g, O.convert(nr, nc, r, c, v, d), f"{d} shift {shift}")
        g.free()


def test_percentile_cut_over_many_length_distributions(ctx):
    """The nearest-rank percentile of the row lengths is picked on the device digit by digit: lengths that need one,
    two and three digits, many equal lengths, empty rows, more rows than one sweep of the counting grid covers, and
    ranks at both ends."""
    from paper_2403_05802_amd import binding as B
    from helpers import assert_same_layout, dev, us_desc_of, us_pred_of
    rng = np.random.default_rng(21)

    def matrix(lens, ncols):
        r = np.repeat(np.arange(lens.size, dtype=np.int64), lens)
        c = np.concatenate([rng.choice(ncols, size=l, replace=False) for l in lens if l > 0]) if r.size else r
        p = rng.permutation(r.size)
        return r[p].astype(np.int32), c[p].astype(np.int32), rng.uniform(0.1, 1, r.size).astype(np.float32)

    cases = [
        (rng.integers(0, 9, 700), 40),                                             # one digit, ties everywhere
        (np.where(rng.random(3000) < 0.9, 3, 300).astype(np.int64), 1000),         # two values far apart
        (np.minimum(rng.zipf(1.6, 5000), 2_000).astype(np.int64), 70_000),         # three digits (17-bit lengths), long tail
        (np.concatenate([np.zeros(66_000, np.int64), np.array([5, 1, 2])]), 8),    # nearly all rows empty, > 256*256 rows
        (np.full(513, 7, np.int64), 7),                                            # all equal, full rows
    ]
    for lens, ncols in cases:
        nrows = int(lens.size)
        r, c, v = matrix(lens, ncols)
        for num, den in ((9, 10), (1, 2), (1, 1), (1, 1000), (999, 1000)):
            pred = O.Predicate((O.d0(),), O.RANK_LT_PERCENTILE, num=num, den=den)
            oa, ob, _ = O.decompose(nrows, ncols, r, c, v, O.ELL(), O.COO(), pred)
            ga, gb = B.us_decompose(ctx, nrows, ncols, dev(r), dev(c), dev(v), us_desc_of(O.ELL()), us_desc_of(O.COO()),
                                    us_pred_of(pred))
            assert_same_layout(ga, oa, f"ELL part, {nrows} rows, {num}/{den}")
            assert_same_layout(gb, ob, f"COO part, {nrows} rows, {num}/{den}")
            ga.free(); gb.free()


def test_spmm_with_row_strides(ctx):
    """X and Y as column slices of wider arrays (ldx > N, ldy > N): every layout, with and without accumulation;
    the columns of Y beyond N are the caller's and must come back untouched."""
    from paper_2403_05802_amd import binding as B
    from helpers import assert_product, dev, host, row_terms, us_desc_of
    rng = np.random.default_rng(31)
    nr, nc, N, ldx, ldy = 300, 260, 70, 96, 80
    lin = rng.choice(nr * nc, size=6000, replace=False)
    r, c = (lin // nc).astype(np.int32), (lin % nc).astype(np.int32)
    v = rng.uniform(-1, 1, r.size).astype(np.float32); v[v == 0] = 0.5
    Xw = rng.uniform(-1, 1, (nc, ldx)).astype(np.float32)
    Yw0 = rng.uniform(-1, 1, (nr, ldy)).astype(np.float32)
    ref = O.spmm_coo(nr, nc, r, c, v, Xw[:, :N])
    S = O.spmm_coo(nr, nc, r, c, np.abs(v), np.abs(Xw[:, :N]))
    nt = row_terms(nr, r)[:, None]
    for d in (O.CSR(), O.DCSR(), O.COO(), O.CSC(), O.ELL(), O.BCSR(4), O.BCSR(2, 3), O.BDIA(3), O.CSB(16), O.CISR_PLUS(5),
              O.BELL(4), O.BELL(3, 2)):
        g = B.us_convert(ctx, nr, nc, dev(r), dev(c), dev(v), us_desc_of(d))
        for acc in (False, True):
            Xd, Yd = dev(Xw), dev(Yw0)
            B.us_spmm(ctx, g, Xd[:, :N], Yd[:, :N], accumulate=acc)
            got = host(Yd)
            assert np.array_equal(got[:, N:], Yw0[:, N:]), (d, acc)
            if acc:
                assert_product(got[:, :N], ref + Yw0[:, :N], S + np.abs(Yw0[:, :N]), nt + 1, f"strided spmm {d} accumulate")
            else:
                assert_product(got[:, :N], ref, S, nt, f"strided spmm {d}")
        g.free()
