"""Format -> format conversion through the COO hub (the reversibility / reachability argument
of Section 5.2, the CSR->CSC, DCSC->BCSR, CSB->DIA-variant, COO->ELL, COO->DIA cases of Table 5) vs the oracle."""
import numpy as np
import pytest

from oracle import unisparse_oracle as O
from paper_2403_05802_amd import workloads as W

pytestmark = pytest.mark.gpu

FORMATS = [("COO", O.COO()), ("CSR", O.CSR()), ("DCSR", O.DCSR()), ("CSC", O.CSC()), ("DCSC", O.DCSC()),
           ("DIA", O.DIA()), ("DIAv", O.DIA_VARIANT()), ("BCSR4", O.BCSR(4)), ("BCSR2x3", O.BCSR(2, 3)), ("ELL", O.ELL()),
           ("BDIA3", O.BDIA(3)), ("CSB8x4", O.CSB(8, 4)), ("CISRplus5", O.CISR_PLUS(5)), ("BELL4x2", O.BELL(4, 2))]


@pytest.fixture(scope="module")
def ctx():
    from paper_2403_05802_amd import binding as B
    return B.Context("cuda:0")


@pytest.mark.parametrize("sname,sdesc", FORMATS, ids=[f[0] for f in FORMATS])
def test_every_pair_small(ctx, sname, sdesc):
    from paper_2403_05802_amd import binding as B
    from helpers import assert_same_layout, dev, us_desc_of
    rng = np.random.default_rng(5)
    nr, nc = 203, 117
    # a few diagonals + scattered entries, so that DIA slabs stay small
    rows, cols = [], []
    for off in (-7, 0, 3, 40):
        i = np.arange(max(0, -off), min(nr, nc - off))
        keep = rng.random(i.size) < 0.8
        rows.append(i[keep]); cols.append(i[keep] + off)
    r = np.concatenate(rows).astype(np.int32); c = np.concatenate(cols).astype(np.int32)
    extra = rng.choice(nr * nc, 60, replace=False)
    have = set(zip(r.tolist(), c.tolist()))
    ex = [(int(e // nc), int(e % nc)) for e in extra if (int(e // nc), int(e % nc)) not in have]
    r = np.concatenate([r, np.array([a for a, _ in ex], np.int32)]); c = np.concatenate([c, np.array([b for _, b in ex], np.int32)])
    p = rng.permutation(r.size); r, c = r[p], c[p]
    v = rng.uniform(0.1, 1, r.size).astype(np.float32)
    osrc = O.convert(nr, nc, r, c, v, sdesc)
    gsrc = B.us_convert(ctx, nr, nc, dev(r), dev(c), dev(v), us_desc_of(sdesc))
    rr, cc, vv = O.to_coo(osrc)
    for tname, tdesc in FORMATS:
        o = O.convert(nr, nc, rr, cc, vv, tdesc)
        g = B.us_convert_formatted(ctx, gsrc, us_desc_of(tdesc))
        assert_same_layout(g, o, f"{sname}->{tname}")
        g.free()
    assert_same_layout(gsrc, osrc, "source untouched")


def test_table5_cases_on_scaled_workloads(ctx):
    from paper_2403_05802_amd import binding as B
    from helpers import assert_same_layout, coo_to_dev, us_desc_of
    m = W.cfg2_powerlaw(n=1 << 14, target_nnz=1 << 18, max_len=3000, empty_frac=0.3)
    d = coo_to_dev(m)
    csr = B.us_convert(ctx, m.nrows, m.ncols, *d, us_desc_of(O.CSR()))
    csc = B.us_convert_formatted(ctx, csr, us_desc_of(O.CSC()))                 # CSR -> CSC
    assert_same_layout(csc, O.convert(m.nrows, m.ncols, m.row, m.col, m.val, O.CSC()), "CSR->CSC")
    dcsc = B.us_convert_formatted(ctx, csc, us_desc_of(O.DCSC()))
    bcsr = B.us_convert_formatted(ctx, dcsc, us_desc_of(O.BCSR(4)))             # DCSC -> BCSR
    assert_same_layout(bcsr, O.convert(m.nrows, m.ncols, m.row, m.col, m.val, O.BCSR(4)), "DCSC->BCSR")
    back = B.us_convert_formatted(ctx, bcsr, us_desc_of(O.COO()))               # and back to the hub
    assert_same_layout(back, O.convert(m.nrows, m.ncols, m.row, m.col, m.val, O.COO()), "BCSR->COO")
    ell = B.us_convert_formatted(ctx, back, us_desc_of(O.ELL()))                # COO -> ELL
    assert_same_layout(ell, O.convert(m.nrows, m.ncols, m.row, m.col, m.val, O.ELL()), "COO->ELL")
    b = W.cfg3_banded(n=1 << 13, extra_frac=0.0)
    coo = B.us_convert(ctx, b.nrows, b.ncols, *coo_to_dev(b), us_desc_of(O.COO()))
    dia = B.us_convert_formatted(ctx, coo, us_desc_of(O.DIA()))                 # COO -> DIA
    assert_same_layout(dia, O.convert(b.nrows, b.ncols, b.row, b.col, b.val, O.DIA()), "COO->DIA")
    diav = B.us_convert_formatted(ctx, dia, us_desc_of(O.DIA_VARIANT()))
    assert_same_layout(diav, O.convert(b.nrows, b.ncols, b.row, b.col, b.val, O.DIA_VARIANT()), "DIA->DIA variant")
    csb = B.us_convert(ctx, b.nrows, b.ncols, *coo_to_dev(b), us_desc_of(O.CSB(512, 256)))
    assert_same_layout(csb, O.convert(b.nrows, b.ncols, b.row, b.col, b.val, O.CSB(512, 256)), "COO->CSB")
    diav2 = B.us_convert_formatted(ctx, csb, us_desc_of(O.DIA_VARIANT()))       # CSB -> DIA variant
    assert_same_layout(diav2, O.convert(b.nrows, b.ncols, b.row, b.col, b.val, O.DIA_VARIANT()), "CSB->DIA variant")
