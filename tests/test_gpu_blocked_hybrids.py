"""Hybrids cut by the nodes of a blocked layout: the BDIA/CSR program of Figure 3c (#sum over (d0/b, d1-d0),
part A as blocked DIA, Figure 9 addressing val[node*b + d0%b]) and the per-block threshold of the BELL/COO case
study (Section 7.2.2); HIP vs oracle."""
import numpy as np
import pytest
import torch

from oracle import unisparse_oracle as O
from paper_2403_05802_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2403_05802_amd import binding as B
    return B.Context("cuda:0")


def block_pred(b, thld):
    return O.Predicate((O.div(0, b), O.diag()), O.SUM_GE_ABS, abs=thld)


def broken_bands(n, ncols, seed, keep=0.85, extra=0.02):
    """A few diagonals with holes plus scattered entries, shuffled."""
    rng = np.random.default_rng(seed)
    have = {}
    for off in (-n // 3, -2, 0, 1, 5, ncols // 2):
        i = np.arange(max(0, -off), min(n, ncols - off))
        i = i[rng.random(i.size) < keep]
        for a in i.tolist():
            have[(a, a + off)] = 1
    for e in rng.choice(n * ncols, int(extra * n) + 1, replace=False).tolist():
        have[(e // ncols, e % ncols)] = 1
    rc = np.array(list(have.keys()), dtype=np.int32)
    rc = rc[rng.permutation(rc.shape[0])]
    v = rng.uniform(0.1, 1, rc.shape[0]).astype(np.float32)
    return rc[:, 0].copy(), rc[:, 1].copy(), v


@pytest.mark.parametrize("shape", [(1000, 1000), (3001, 1777), (50, 4000)], ids=lambda s: f"{s[0]}x{s[1]}")
@pytest.mark.parametrize("b,thld", [(3, 3), (3, 2), (4, 4), (16, 12), (1, 1)])
def test_bdia_csr_hybrid(ctx, shape, b, thld):
    from paper_2403_05802_amd import binding as B
    from helpers import assert_product, row_terms, assert_same_layout, dev, host, us_desc_of, us_pred_of
    nr, nc = shape
    r, c, v = broken_bands(nr, nc, seed=b * 100 + thld)
    pred = block_pred(b, thld)
    oa, ob, mask = O.decompose(nr, nc, r, c, v, O.BDIA(b), O.CSR(), pred)
    assert mask.sum() > 0 and (b == 1 or mask.sum() < mask.size)
    ga, gb = B.us_decompose(ctx, nr, nc, dev(r), dev(c), dev(v), us_desc_of(O.BDIA(b)), us_desc_of(O.CSR()),
                            us_pred_of(pred))
    assert_same_layout(ga, oa, "A BDIA")
    assert_same_layout(gb, ob, "B CSR")
    rng = np.random.default_rng(1)
    x = rng.uniform(-1, 1, nc).astype(np.float32)
    y = torch.full((nr,), 3.0, device="cuda")
    B.us_spmv(ctx, ga, dev(x), y)
    B.us_spmv(ctx, gb, dev(x), y, accumulate=True)
    assert_product(host(y), O.spmv_coo(nr, nc, r, c, v, x), O.abs_row_sums(nr, r, c, v, x), row_terms(nr, r), "hybrid spmv")
    X = rng.uniform(-1, 1, (nc, 70)).astype(np.float32)
    Y = torch.full((nr, 70), 3.0, device="cuda")
    B.us_spmm(ctx, ga, dev(X), Y)
    B.us_spmm(ctx, gb, dev(X), Y, accumulate=True)
    S = O.spmm_coo(nr, nc, r, c, np.abs(v), np.abs(X))
    assert_product(host(Y), O.spmm_coo(nr, nc, r, c, v, X), S, row_terms(nr, r)[:, None], "hybrid spmm")
    ga.free(); gb.free()


def test_block_diagonal_groups_with_other_part_formats(ctx):
    """The grouping is independent of how the parts are stored afterwards."""
    from paper_2403_05802_amd import binding as B
    from helpers import assert_same_layout, dev, us_desc_of, us_pred_of
    nr, nc = 700, 900
    r, c, v = broken_bands(nr, nc, seed=9)
    for da, db, b, thld in [(O.BDIA(4), O.COO(), 2, 2), (O.DIA(), O.DCSR(), 8, 7), (O.CSR(), O.BDIA(3), 3, 3),
                            (O.BDIA(3), O.CSR(), 3, 10 ** 9), (O.BDIA(3), O.CSR(), 3, 0)]:
        pred = block_pred(b, thld)
        oa, ob, _ = O.decompose(nr, nc, r, c, v, da, db, pred)
        ga, gb = B.us_decompose(ctx, nr, nc, dev(r), dev(c), dev(v), us_desc_of(da), us_desc_of(db), us_pred_of(pred))
        assert_same_layout(ga, oa, f"A b={b} thld={thld}")
        assert_same_layout(gb, ob, f"B b={b} thld={thld}")
        ga.free(); gb.free()


def test_bdia_hybrid_errors_and_empty(ctx):
    from paper_2403_05802_amd import binding as B
    from helpers import assert_same_layout, dev, us_desc_of, us_pred_of
    pred = block_pred(3, 3)
    e = np.zeros(0, np.int32); ev = np.zeros(0, np.float32)
    oa, ob, _ = O.decompose(7, 9, e, e, ev, O.BDIA(3), O.CSR(), pred)
    ga, gb = B.us_decompose(ctx, 7, 9, dev(e), dev(e), dev(ev), us_desc_of(O.BDIA(3)), us_desc_of(O.CSR()), us_pred_of(pred))
    assert_same_layout(ga, oa, "empty A"); assert_same_layout(gb, ob, "empty B")
    r = np.array([0, 1, 1], np.int32); c = np.array([0, 2, 2], np.int32); v = np.ones(3, np.float32)
    with pytest.raises(B.UnisparseError) as ei:
        B.us_decompose(ctx, 3, 3, dev(r), dev(c), dev(v), us_desc_of(O.BDIA(3)), us_desc_of(O.CSR()), us_pred_of(pred))
    assert ei.value.code == "US_ERR_DUPLICATE"
    with pytest.raises(B.UnisparseError) as ei:
        B.us_decompose(ctx, 3, 2, dev(r[:2]), dev(c[:2]), dev(v[:2]), us_desc_of(O.BDIA(3)), us_desc_of(O.CSR()),
                       us_pred_of(pred))
    assert ei.value.code == "US_ERR_INDEX_RANGE"
    bad = O.Predicate((O.div(0, 3), O.diag()), O.SUM_GE_FRAC_OF_CAPACITY, num=1, den=2)
    with pytest.raises(B.UnisparseError) as ei:
        B.us_decompose(ctx, 3, 3, dev(r[:2]), dev(c[:2]), dev(v[:2]), us_desc_of(O.BDIA(3)), us_desc_of(O.CSR()),
                       us_pred_of(bad))
    assert ei.value.code == "US_ERR_UNSUPPORTED_DESC"


def test_bdia_hybrid_on_scaled_banded_workload(ctx):
    """Config-3-like matrix (7 diagonals + 1 % scattered) at 2^17 rows with the Figure 3c program."""
    from paper_2403_05802_amd import binding as B
    from helpers import assert_product, row_terms, assert_same_layout, coo_to_dev, dev, host, us_desc_of, us_pred_of
    m = W.cfg3_banded(n=1 << 17)
    pred = block_pred(4, 4)
    oa, ob, mask = O.decompose(m.nrows, m.ncols, m.row, m.col, m.val, O.BDIA(4), O.CSR(), pred)
    ga, gb = B.us_decompose(ctx, m.nrows, m.ncols, *coo_to_dev(m), us_desc_of(O.BDIA(4)), us_desc_of(O.CSR()),
                            us_pred_of(pred))
    assert_same_layout(ga, oa, "A"); assert_same_layout(gb, ob, "B")
    x = W.dense_operand(3, m.ncols)
    y = torch.empty(m.nrows, device="cuda")
    B.us_spmv(ctx, ga, dev(x), y); B.us_spmv(ctx, gb, dev(x), y, accumulate=True)
    yref = O.spmv(oa, x) + O.spmv(ob, x)
    np.testing.assert_allclose(yref, O.spmv_coo(m.nrows, m.ncols, m.row, m.col, m.val, x), atol=1e-9)
    assert_product(host(y), yref, O.abs_row_sums(m.nrows, m.row, m.col, m.val, x), row_terms(m.nrows, m.row), "hybrid spmv")


def clustered_blocks(nr, nc, seed, bh, bw, dense_blocks, fill, extra):
    """`dense_blocks` random bh x bw blocks filled to `fill`, plus `extra` scattered entries, shuffled."""
    rng = np.random.default_rng(seed)
    nbr, nbc = -(-nr // bh), -(-nc // bw)
    blk = rng.choice(nbr * nbc, dense_blocks, replace=False)
    rows, cols = [], []
    for b in blk.tolist():
        br, bc = divmod(b, nbc)
        ii, jj = np.meshgrid(np.arange(bh), np.arange(bw), indexing="ij")
        keep = rng.random((bh, bw)) < fill
        rows.append(br * bh + ii[keep]); cols.append(bc * bw + jj[keep])
    r = np.concatenate(rows + [rng.integers(0, nr, extra)]); c = np.concatenate(cols + [rng.integers(0, nc, extra)])
    ok = (r < nr) & (c < nc)
    lin = np.unique(r[ok].astype(np.int64) * nc + c[ok])
    lin = lin[rng.permutation(lin.size)]
    v = rng.uniform(0.1, 1, lin.size).astype(np.float32)
    return (lin // nc).astype(np.int32), (lin % nc).astype(np.int32), v


@pytest.mark.parametrize("bh,bw,thld", [(4, 4, 8), (2, 3, 4), (8, 8, 1), (16, 2, 33), (4, 4, 0)])
def test_block_threshold_hybrid(ctx, bh, bw, thld):
    """Decomposition of the BELL/COO case study (Section 7.2.2): blocks holding at least `thld` entries go to
    the blocked part (stored as BCSR, as two other formats, and as blocked ELL), the rest stays COO; SpMM over the hybrid."""
    from paper_2403_05802_amd import binding as B
    from helpers import assert_product, row_terms, assert_same_layout, dev, host, us_desc_of, us_pred_of
    nr, nc = 1003, 2050
    r, c, v = clustered_blocks(nr, nc, seed=bh * 10 + bw, bh=bh, bw=bw, dense_blocks=1500, fill=0.8, extra=20_000)
    pred = O.Predicate((O.div(0, bh), O.div(1, bw)), O.SUM_GE_ABS, abs=thld)
    for da, db in ((O.BCSR(bh, bw), O.COO()), (O.CSR(), O.DCSR()), (O.BELL(bh, bw), O.COO())):
        oa, ob, mask = O.decompose(nr, nc, r, c, v, da, db, pred)
        ga, gb = B.us_decompose(ctx, nr, nc, dev(r), dev(c), dev(v), us_desc_of(da), us_desc_of(db), us_pred_of(pred))
        assert_same_layout(ga, oa, "A"); assert_same_layout(gb, ob, "B")
        if thld == 8:
            assert 0 < mask.sum() < mask.size
        rng = np.random.default_rng(2)
        X = rng.uniform(-1, 1, (nc, 33)).astype(np.float32)
        Y = torch.full((nr, 33), 9.0, device="cuda")
        B.us_spmm(ctx, ga, dev(X), Y); B.us_spmm(ctx, gb, dev(X), Y, accumulate=True)
        S = O.spmm_coo(nr, nc, r, c, np.abs(v), np.abs(X))
        assert_product(host(Y), O.spmm_coo(nr, nc, r, c, v, X), S, row_terms(nr, r)[:, None], "hybrid spmm")
        ga.free(); gb.free()
