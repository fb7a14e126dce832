"""HIP library vs oracle on the five benchmark workloads: scaled-down versions compared
array by array, and the full sizes (the launch configuration the benchmark times)."""
import numpy as np
import pytest
import torch

from oracle import unisparse_oracle as O
from paper_2403_05802_amd import workloads as W
import helpers as H

pytestmark = pytest.mark.gpu

DIAG_PRED = O.Predicate((O.diag(),), O.SUM_GE_FRAC_OF_CAPACITY, num=9, den=10)
P90_PRED = O.Predicate((O.d0(),), O.RANK_LT_PERCENTILE, num=9, den=10)


@pytest.fixture(scope="module")
def ctx():
    from paper_2403_05802_amd import binding as B
    return B.Context("cuda:0")


def check_spmv(ctx, parts, m, x, what="spmv"):
    """y = sum of parts * x on the GPU vs fp64 product from the original COO, every row."""
    from paper_2403_05802_amd import binding as B
    from helpers import assert_product, dev, host, row_terms
    y = torch.full((m.nrows,), 123.0, device="cuda")
    xd = dev(x)
    for k, g in enumerate(parts):
        B.us_spmv(ctx, g, xd, y, accumulate=k > 0)
    yref = O.spmv_coo(m.nrows, m.ncols, m.row, m.col, m.val, x)
    assert_product(host(y), yref, O.abs_row_sums(m.nrows, m.row, m.col, m.val, x), row_terms(m.nrows, m.row), what)
    return y


# ------------------------------------------------------------------ scaled-down versions, full comparison
def test_cfg2_small_csr_dcsr(ctx):
    from paper_2403_05802_amd import binding as B
    from helpers import assert_same_layout, coo_to_dev, us_desc_of
    for empty in (0.0, 0.5):
        m = W.cfg2_powerlaw(n=1 << 14, target_nnz=1 << 18, max_len=3000, empty_frac=empty)
        d = coo_to_dev(m)
        x = W.dense_operand(2, m.ncols)
        for desc in (O.CSR(), O.DCSR(), O.CISR_PLUS(64)):
            o = O.convert(m.nrows, m.ncols, m.row, m.col, m.val, desc)
            g = B.us_convert(ctx, m.nrows, m.ncols, *d, us_desc_of(desc))
            assert_same_layout(g, o, f"cfg2s empty={empty}")
            check_spmv(ctx, [g], m, x)
            g.free()


def test_cfg3_small_dia_csr(ctx):
    from paper_2403_05802_amd import binding as B
    from helpers import assert_same_layout, coo_to_dev, us_desc_of, us_pred_of
    m = W.cfg3_banded(n=1 << 14)
    oa, ob, _ = O.decompose(m.nrows, m.ncols, m.row, m.col, m.val, O.DIA(), O.CSR(), DIAG_PRED)
    assert oa.levels[0].idx.tolist() == list(W.CFG3_OFFSETS)
    ga, gb = B.us_decompose(ctx, m.nrows, m.ncols, *coo_to_dev(m), us_desc_of(O.DIA()), us_desc_of(O.CSR()),
                            us_pred_of(DIAG_PRED))
    assert_same_layout(ga, oa, "cfg3s DIA part")
    assert_same_layout(gb, ob, "cfg3s CSR part")
    check_spmv(ctx, [ga, gb], m, W.dense_operand(3, m.ncols))
    # the same split into other pairs of formats
    for da, db in ((O.DIA_VARIANT(), O.DCSR()), (O.CSR(), O.COO()), (O.ELL(), O.BCSR(2))):
        oa, ob, _ = O.decompose(m.nrows, m.ncols, m.row, m.col, m.val, da, db, DIAG_PRED)
        ga, gb = B.us_decompose(ctx, m.nrows, m.ncols, *coo_to_dev(m), us_desc_of(da), us_desc_of(db),
                                us_pred_of(DIAG_PRED))
        assert_same_layout(ga, oa, "cfg3s A")
        assert_same_layout(gb, ob, "cfg3s B")
        check_spmv(ctx, [ga, gb], m, W.dense_operand(3, m.ncols))
    # absolute threshold (the paper's %thld) on rows
    pred = O.Predicate((O.d0(),), O.SUM_GE_ABS, abs=8)
    oa, ob, _ = O.decompose(m.nrows, m.ncols, m.row, m.col, m.val, O.ELL(), O.COO(), pred)
    ga, gb = B.us_decompose(ctx, m.nrows, m.ncols, *coo_to_dev(m), us_desc_of(O.ELL()), us_desc_of(O.COO()),
                            us_pred_of(pred))
    assert_same_layout(ga, oa, "rows>=8 ELL")
    assert_same_layout(gb, ob, "rows<8 COO")


def test_cfg4_small_bcsr_spmm(ctx):
    from paper_2403_05802_amd import binding as B
    from helpers import assert_same_layout, coo_to_dev, us_desc_of
    m = W.cfg4_blockfem(n=1 << 13, band_blocks=64)
    o = O.convert(m.nrows, m.ncols, m.row, m.col, m.val, O.BCSR(4))
    g = B.us_convert(ctx, m.nrows, m.ncols, *coo_to_dev(m), us_desc_of(O.BCSR(4)))
    assert_same_layout(g, o, "cfg4s BCSR")
    assert np.array_equal(o.levels[1].ptr, 24 * np.arange(m.nrows // 4 + 1))   # closed form
    X = W.dense_operand(4, (m.ncols, 64))
    H.check_spmm_all_rows(ctx, [g], m, X, "cfg4 small spmm", slab=1000)
    check_spmv(ctx, [g], m, W.dense_operand(4, m.ncols))


def test_cfg5_small_ell_coo_spmm(ctx):
    from paper_2403_05802_amd import binding as B
    from helpers import assert_same_layout, coo_to_dev, us_desc_of, us_pred_of
    m = W.cfg5_powerlaw_local(n=50_000, target_nnz=1_000_000, max_len=5000)
    oa, ob, _ = O.decompose(m.nrows, m.ncols, m.row, m.col, m.val, O.ELL(), O.COO(), P90_PRED)
    ga, gb = B.us_decompose(ctx, m.nrows, m.ncols, *coo_to_dev(m), us_desc_of(O.ELL()), us_desc_of(O.COO()),
                            us_pred_of(P90_PRED))
    assert_same_layout(ga, oa, "cfg5s ELL part")
    assert_same_layout(gb, ob, "cfg5s COO part")
    X = W.dense_operand(5, (m.ncols, 128))
    H.check_spmm_all_rows(ctx, [ga, gb], m, X, "cfg5 small spmm", slab=7001)
    check_spmv(ctx, [ga, gb], m, W.dense_operand(5, m.ncols))
    # rank split into other format pairs, and with a fixed width
    for da, db, pred in ((O.ELL(), O.CSR(), P90_PRED), (O.CSR(), O.DCSR(), P90_PRED),
                         (O.ELL(), O.BCSR(4), O.Predicate((O.d0(),), O.RANK_LT_ABS, abs=5))):
        oa, ob, _ = O.decompose(m.nrows, m.ncols, m.row, m.col, m.val, da, db, pred)
        ga, gb = B.us_decompose(ctx, m.nrows, m.ncols, *coo_to_dev(m), us_desc_of(da), us_desc_of(db), us_pred_of(pred))
        assert_same_layout(ga, oa, "cfg5s A")
        assert_same_layout(gb, ob, "cfg5s B")


# ------------------------------------------------------------------ full sizes
def test_cfg2_full(ctx):
    from paper_2403_05802_amd import binding as B
    from helpers import assert_same_layout, coo_to_dev, us_desc_of
    m = W.cfg2_powerlaw()
    d = coo_to_dev(m)
    x = W.dense_operand(2, m.ncols)
    o = O.convert(m.nrows, m.ncols, m.row, m.col, m.val, O.CSR())
    g = B.us_convert(ctx, m.nrows, m.ncols, *d, us_desc_of(O.CSR()))
    assert_same_layout(g, o, "cfg2 CSR")
    y1 = check_spmv(ctx, [g], m, x)
    g2 = B.us_convert(ctx, m.nrows, m.ncols, *d, us_desc_of(O.DCSR()))
    # min row length is 1, so DCSR keeps every row: arrays follow from the CSR ones
    assert np.array_equal(g2.idx(0).cpu().numpy(), np.arange(m.nrows))
    assert torch.equal(g2.ptr(1), g.ptr(1)) and torch.equal(g2.idx(1), g.idx(1)) and torch.equal(g2.val(), g.val())
    y2 = check_spmv(ctx, [g2], m, x)
    assert torch.equal(y1.view(torch.int32), y2.view(torch.int32))
    # the other Sort path at full size: forced in-LDS finish (its heavy rows end in the fall-back) gives the same bytes
    ctx.set_sort_lds_finish(True)
    try:
        g3 = B.us_convert(ctx, m.nrows, m.ncols, *d, us_desc_of(O.CSR()))
    finally:
        ctx.set_sort_lds_finish(None)
    assert torch.equal(g3.ptr(1), g.ptr(1)) and torch.equal(g3.idx(1), g.idx(1))
    assert torch.equal(g3.val().view(torch.int32), g.val().view(torch.int32))
    # CISR-plus with 1024 partitions (the core count of Section 7.2.4) against the full oracle output
    o4 = O.convert(m.nrows, m.ncols, m.row, m.col, m.val, O.CISR_PLUS(1024))
    g4 = B.us_convert(ctx, m.nrows, m.ncols, *d, us_desc_of(O.CISR_PLUS(1024)))
    assert_same_layout(g4, o4, "cfg2 CISR-plus")
    rows_per_part = np.diff(o4.levels[1].ptr)
    assert rows_per_part.max() - rows_per_part.min() <= 1
    check_spmv(ctx, [g4], m, x)


def test_cfg3_full(ctx):
    from paper_2403_05802_amd import binding as B
    from helpers import assert_same_layout, coo_to_dev, us_desc_of, us_pred_of
    m = W.cfg3_banded()
    oa, ob, _ = O.decompose(m.nrows, m.ncols, m.row, m.col, m.val, O.DIA(), O.CSR(), DIAG_PRED)
    assert oa.levels[0].idx.tolist() == list(W.CFG3_OFFSETS)           # closed form: the 7 diagonals
    assert oa.nnz == 7 * m.nrows - 6146 and ob.nnz == m.nnz - oa.nnz    # closed form: 7n - 2(1+1024+2048)
    ga, gb = B.us_decompose(ctx, m.nrows, m.ncols, *coo_to_dev(m), us_desc_of(O.DIA()), us_desc_of(O.CSR()),
                            us_pred_of(DIAG_PRED))
    assert_same_layout(ga, oa, "cfg3 DIA part")
    assert_same_layout(gb, ob, "cfg3 CSR part")
    check_spmv(ctx, [ga, gb], m, W.dense_operand(3, m.ncols))


from progress import say  # noqa: E402


def test_cfg4_full(ctx):
    from paper_2403_05802_amd import binding as B
    from helpers import assert_same_layout, coo_to_dev, us_desc_of
    m = W.cfg4_blockfem()
    say("cfg4 generated")
    g = B.us_convert(ctx, m.nrows, m.ncols, *coo_to_dev(m), us_desc_of(O.BCSR(4)))
    say("cfg4 converted on the GPU")
    o = O.convert(m.nrows, m.ncols, m.row, m.col, m.val, O.BCSR(4))
    say("cfg4 oracle done")
    nbr = m.nrows // 4
    assert np.array_equal(o.levels[1].ptr, 24 * np.arange(nbr + 1))    # closed form: 24 blocks per block row
    assert o.val.shape[0] == m.nnz and np.count_nonzero(o.val) == m.nnz  # blocks are dense: no padding
    assert_same_layout(g, o, "cfg4 BCSR")
    # the other Sort path at full size (blocked tuples finish inside LDS by default): whole-array passes only
    ctx.set_sort_lds_finish(False)
    try:
        g2 = B.us_convert(ctx, m.nrows, m.ncols, *coo_to_dev(m), us_desc_of(O.BCSR(4)))
    finally:
        ctx.set_sort_lds_finish(None)
    assert torch.equal(g2.ptr(1), g.ptr(1)) and torch.equal(g2.idx(1), g.idx(1))
    assert torch.equal(g2.val().view(torch.int32), g.val().view(torch.int32))
    g2.free()
    del o
    H.check_spmm_all_rows(ctx, [g], m, W.dense_operand(4, (m.ncols, 64)), "cfg4 spmm N=64")


def test_cfg5_full(ctx):
    from paper_2403_05802_amd import binding as B
    from helpers import assert_same_layout, coo_to_dev, us_desc_of, us_pred_of
    m = W.cfg5_powerlaw_local()
    say("cfg5 generated")
    ga, gb = B.us_decompose(ctx, m.nrows, m.ncols, *coo_to_dev(m), us_desc_of(O.ELL()), us_desc_of(O.COO()),
                            us_pred_of(P90_PRED))
    say("cfg5 decomposed on the GPU")
    oa, ob, _ = O.decompose(m.nrows, m.ncols, m.row, m.col, m.val, O.ELL(), O.COO(), P90_PRED)
    say("cfg5 oracle done")
    lens = np.bincount(m.row, minlength=m.nrows)
    K = int(np.sort(lens)[int(np.ceil(0.9 * m.nrows)) - 1])
    assert oa.levels[0].size == K and oa.nnz == int(np.minimum(lens, K).sum()) and ob.nnz == m.nnz - oa.nnz
    assert_same_layout(ga, oa, "cfg5 ELL part")
    assert_same_layout(gb, ob, "cfg5 COO part")
    del oa, ob
    H.check_spmm_all_rows(ctx, [ga, gb], m, W.dense_operand(5, (m.ncols, 128)), "cfg5 spmm N=128")
    # SpMV over the same hybrid (the extra data point the benchmark times), every row
    check_spmv(ctx, [ga, gb], m, W.dense_operand(5, m.ncols), "cfg5 hybrid spmv")


def test_label_propagation_small(ctx):
    """A few iterations Y <- A_hat Y (row-normalised graph, Section 7.2.5) over CSR and over the
    ELL+COO hybrid against the fp64 iteration from the COO list."""
    from paper_2403_05802_amd import binding as B
    from helpers import assert_product, coo_to_dev, dev, host, row_terms, us_desc_of, us_pred_of
    m = W.cfg5_powerlaw_local(n=3000, target_nnz=40_000, max_len=800, index=6)
    deg = np.bincount(m.row, minlength=m.nrows)
    m.val = (1.0 / deg[m.row]).astype(np.float32)
    N, iters = 40, 5
    Y0 = W.dense_operand(6, (m.ncols, N))
    # fp64 iteration, and beside it the same iteration over absolute values: S_t = |A| S_{t-1} bounds what every
    # element has summed so far, so the rounding error of t fp32 products in a row is judged against it
    ref, S = Y0.astype(np.float64), np.abs(Y0).astype(np.float64)
    for _ in range(iters):
        ref = O.spmm_coo(m.nrows, m.ncols, m.row, m.col, m.val, ref)
        S = O.spmm_coo(m.nrows, m.ncols, m.row, m.col, np.abs(m.val), S)
    # error of iterate t: what the rows it gathers already carry (at most that of the longest row), plus its own
    # sum; over `iters` products that is at most iters * C * sqrt(longest row) * 2^-24 * S, written as a term count
    nt = float(row_terms(m.nrows, m.row).max()) * iters ** 2
    d = coo_to_dev(m)
    csr = [B.us_convert(ctx, m.nrows, m.ncols, *d, us_desc_of(O.CSR()))]
    hyb = list(B.us_decompose(ctx, m.nrows, m.ncols, *d, us_desc_of(O.ELL()), us_desc_of(O.COO()), us_pred_of(P90_PRED)))
    for parts in (csr, hyb):
        bufs = [dev(Y0), torch.empty(m.nrows, N, device="cuda")]
        for t in range(iters):
            for k, p in enumerate(parts):
                B.us_spmm(ctx, p, bufs[t & 1], bufs[(t + 1) & 1], accumulate=k > 0)
        assert_product(host(bufs[iters & 1]), ref, S, nt, f"label propagation, {len(parts)} part(s)")
