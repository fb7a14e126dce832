"""HIP library vs oracle on small inputs: every format, edge cases, error paths."""
import zlib

import numpy as np
import pytest
import torch

from oracle import unisparse_oracle as O
from paper_2403_05802_amd import workloads as W

pytestmark = pytest.mark.gpu

FORMATS = [
    ("COO", O.COO()), ("CSR", O.CSR()), ("DCSR", O.DCSR()), ("CSC", O.CSC()), ("DCSC", O.DCSC()),
    ("DIA", O.DIA()), ("DIAv", O.DIA_VARIANT()), ("BCSR2", O.BCSR(2)), ("BCSR4", O.BCSR(4)),
    ("BCSR2x3", O.BCSR(2, 3)), ("BCSR8", O.BCSR(8)), ("ELL", O.ELL()), ("BDIA3", O.BDIA(3)), ("BDIA16", O.BDIA(16)),
    ("CSB2", O.CSB(2)), ("CSB5x3", O.CSB(5, 3)), ("CSB64x128", O.CSB(64, 128)),
    ("CISRplus1", O.CISR_PLUS(1)), ("CISRplus3", O.CISR_PLUS(3)), ("CISRplus256", O.CISR_PLUS(256)),
    ("BELL4", O.BELL(4)), ("BELL2x3", O.BELL(2, 3)), ("BELL16x1", O.BELL(16, 1)),
]


@pytest.fixture(scope="module")
def ctx():
    from paper_2403_05802_amd import binding as B
    return B.Context("cuda:0")


def random_coo(rng, nrows, ncols, nnz):
    lin = rng.choice(nrows * ncols, size=min(nnz, nrows * ncols), replace=False)
    row, col = (lin // ncols).astype(np.int32), (lin % ncols).astype(np.int32)
    val = rng.uniform(-1, 1, row.shape[0]).astype(np.float32)
    val[val == 0] = 0.5
    return row, col, val


SHAPES = [(5, 4, 6), (1, 1, 1), (1, 300, 120), (300, 1, 77), (64, 64, 0), (257, 129, 3000),
          (1000, 1000, 20000), (4099, 37, 9000), (33, 5000, 9000)]


@pytest.mark.parametrize("name,desc", FORMATS, ids=[f[0] for f in FORMATS])
@pytest.mark.parametrize("shape", SHAPES, ids=[f"{a}x{b}n{c}" for a, b, c in SHAPES])
def test_convert_matches_oracle(ctx, name, desc, shape):
    from paper_2403_05802_amd import binding as B
    from helpers import assert_same_layout, dev, us_desc_of
    nr, nc, nnz = shape
    if name in ("DIA", "DIAv") and nnz > 5000:
        pytest.skip("dense diagonal slab too large for a scattered matrix")
    seed = zlib.crc32(repr((name, shape)).encode())   # the same input in every run of the suite
    rng = np.random.default_rng(seed)
    r, c, v = random_coo(rng, nr, nc, nnz)
    o = O.convert(nr, nc, r, c, v, desc)
    g = B.us_convert(ctx, nr, nc, dev(r), dev(c), dev(v), us_desc_of(desc))
    assert_same_layout(g, o, f"{name} {shape} seed {seed}")
    g.free()


@pytest.mark.parametrize("name,desc", FORMATS, ids=[f[0] for f in FORMATS])
def test_spmv_spmm_all_formats(ctx, name, desc):
    from paper_2403_05802_amd import binding as B
    from helpers import assert_product, dev, host, row_terms, us_desc_of
    rng = np.random.default_rng(7)
    nr, nc = 777, 530
    r, c, v = random_coo(rng, nr, nc, 1500 if name.startswith("DIA") else 30000)
    g = B.us_convert(ctx, nr, nc, dev(r), dev(c), dev(v), us_desc_of(desc))
    x = rng.uniform(-1, 1, nc).astype(np.float32)
    yref = O.spmv_coo(nr, nc, r, c, v, x)
    scale = O.abs_row_sums(nr, r, c, v, x)
    nt = row_terms(nr, r)
    y = torch.full((nr,), 7.0, device="cuda")
    B.us_spmv(ctx, g, dev(x), y)
    assert_product(host(y), yref, scale, nt, f"{name} spmv")
    y0 = rng.uniform(-1, 1, nr).astype(np.float32)
    y = dev(y0)
    B.us_spmv(ctx, g, dev(x), y, accumulate=True)
    assert_product(host(y), yref + y0, scale + np.abs(y0), nt + 1, f"{name} spmv accumulate")
    for N in (1, 5, 64, 130, 260):
        X = rng.uniform(-1, 1, (nc, N)).astype(np.float32)
        Yref = O.spmm_coo(nr, nc, r, c, v, X)
        S = O.spmm_coo(nr, nc, r, c, np.abs(v), np.abs(X))
        Y = torch.full((nr, N), -3.0, device="cuda")
        B.us_spmm(ctx, g, dev(X), Y)
        assert_product(host(Y), Yref, S, nt[:, None], f"{name} spmm N={N}")
        Y0 = rng.uniform(-1, 1, (nr, N)).astype(np.float32)
        Y = dev(Y0)
        B.us_spmm(ctx, g, dev(X), Y, accumulate=True)
        assert_product(host(Y), Yref + Y0, S + np.abs(Y0), nt[:, None] + 1, f"{name} spmm N={N} accumulate")
    g.free()


def test_config1_csr_spmv(ctx):
    """4096 x 4096, 40,960 uniformly placed entries: COO -> CSR bit-exact, then SpMV."""
    from paper_2403_05802_amd import binding as B
    from helpers import assert_product, assert_same_layout, coo_to_dev, dev, host, row_terms, us_desc_of
    m = W.cfg1_uniform()
    o = O.convert(m.nrows, m.ncols, m.row, m.col, m.val, O.CSR())
    g = B.us_convert(ctx, m.nrows, m.ncols, *coo_to_dev(m), us_desc_of(O.CSR()))
    assert_same_layout(g, o, "cfg1 CSR")
    x = W.dense_operand(1, m.ncols)
    y = torch.empty(m.nrows, device="cuda")
    B.us_spmv(ctx, g, dev(x), y)
    yref = O.spmv(o, x)
    np.testing.assert_allclose(yref, O.spmv_coo(m.nrows, m.ncols, m.row, m.col, m.val, x), atol=1e-12)
    assert_product(host(y), yref, O.abs_row_sums(m.nrows, m.row, m.col, m.val, x), row_terms(m.nrows, m.row), "cfg1 spmv")
    # determinism: a second conversion and product give identical bytes
    g2 = B.us_convert(ctx, m.nrows, m.ncols, *coo_to_dev(m), us_desc_of(O.CSR()))
    y2 = torch.empty(m.nrows, device="cuda")
    B.us_spmv(ctx, g2, dev(x), y2)
    assert torch.equal(y.view(torch.int32), y2.view(torch.int32))
    assert torch.equal(g.idx(1), g2.idx(1)) and torch.equal(g.ptr(1), g2.ptr(1))


def test_free_without_waiting(ctx):
    """us_free_async right after products were enqueued: the next conversion takes the freed memory over while
    they may still run, and the stream order keeps their results intact."""
    from paper_2403_05802_amd import binding as B
    from helpers import assert_product, assert_same_layout, dev, host, row_terms, us_desc_of
    m = W.cfg2_powerlaw(n=1 << 15, target_nnz=1 << 20, max_len=4000)
    r, c, v = dev(m.row), dev(m.col), dev(m.val)
    rng = np.random.default_rng(3)
    x = rng.uniform(-1, 1, m.ncols).astype(np.float32)
    yref = O.spmv_coo(m.nrows, m.ncols, m.row, m.col, m.val, x)
    scale = O.abs_row_sums(m.nrows, m.row, m.col, m.val, x)
    xd = dev(x)
    before = ctx.live_bytes()
    ys = []
    for d in (O.CSR(), O.DCSR(), O.CSC(), O.CSR()):
        g = B.us_convert(ctx, m.nrows, m.ncols, r, c, v, us_desc_of(d))
        y = torch.empty(m.nrows, device="cuda")
        for _ in range(3):
            B.us_spmv(ctx, g, xd, y)
        g.free(wait=False)
        ys.append(y)
    g = B.us_convert(ctx, m.nrows, m.ncols, r, c, v, us_desc_of(O.CSR()))
    assert_same_layout(g, O.convert(m.nrows, m.ncols, m.row, m.col, m.val, O.CSR()), "after async frees")
    g.free()
    for y in ys:
        assert_product(host(y), yref, scale, row_terms(m.nrows, m.row), "after async frees")
    assert ctx.live_bytes() == before


def test_error_paths(ctx):
    from paper_2403_05802_amd import binding as B
    from helpers import dev, us_desc_of
    r = np.array([0, 1, 1], np.int32); c = np.array([0, 2, 2], np.int32); v = np.ones(3, np.float32)
    for d in (O.CSR(), O.COO(), O.DCSR(), O.BCSR(2), O.ELL(), O.DIA(), O.BDIA(3), O.CSB(2), O.BELL(2)):
        with pytest.raises(B.UnisparseError) as ei:
            B.us_convert(ctx, 3, 3, dev(r), dev(c), dev(v), us_desc_of(d))
        assert ei.value.code == "US_ERR_DUPLICATE", d
        with pytest.raises(B.UnisparseError) as ei:
            B.us_convert(ctx, 3, 2, dev(r[:2]), dev(c[:2]), dev(v[:2]), us_desc_of(d))
        assert ei.value.code == "US_ERR_INDEX_RANGE", d
    with pytest.raises(B.UnisparseError) as ei:
        B.us_convert(ctx, 0, 3, dev(r), dev(c), dev(v), us_desc_of(O.CSR()))
    assert ei.value.code == "US_ERR_SHAPE"
    bad = B.make_desc([B.expr(B.US_E_AFFINE, 1, 1), B.expr(B.US_E_AFFINE, 0, 1)], (1, 1), (0,))
    with pytest.raises(B.UnisparseError) as ei:
        B.us_convert(ctx, 3, 3, dev(r[:2]), dev(c[:2]), dev(v[:2]), bad)
    assert ei.value.code == "US_ERR_UNSUPPORTED_DESC"
    with pytest.raises(B.UnisparseError) as ei:   # a row longer than the fixed ELL width
        B.us_convert(ctx, 3, 3, dev(np.array([1, 1], np.int32)), dev(np.array([0, 2], np.int32)), dev(v[:2]),
                     us_desc_of(O.ELL(1)))
    assert ei.value.code == "US_ERR_SHAPE"
    with pytest.raises(B.UnisparseError) as ei:   # a block row with more blocks than the fixed blocked-ELL width
        B.us_convert(ctx, 3, 3, dev(np.array([1, 1], np.int32)), dev(np.array([0, 2], np.int32)), dev(v[:2]),
                     us_desc_of(O.BELL(2, width=1)))
    assert ei.value.code == "US_ERR_SHAPE"
    # allocator failure leaves nothing behind, whichever of a call's allocations is the first to fail
    before = ctx.live_bytes()
    for d in (O.CSR(), O.COO(), O.DCSR(), O.DCSC(), O.ELL(), O.BCSR(2), O.DIA(), O.CISR_PLUS(2), O.BELL(2)):
        failed = 0
        for k in range(12):
            ctx.fail_alloc_after = ctx._nalloc + k
            try:
                g = B.us_convert(ctx, 3, 3, dev(r[:2]), dev(c[:2]), dev(v[:2]), us_desc_of(d))
                ctx.fail_alloc_after = None
                g.free()
            except B.UnisparseError as e:
                ctx.fail_alloc_after = None
                assert e.code == "US_ERR_ALLOC", (d, k)
                failed += 1
            assert ctx.live_bytes() == before, (d, k)
        assert failed >= 1, d   # (k = 0: the very first allocation fails)
    g = B.us_convert(ctx, 3, 3, dev(r[:2]), dev(c[:2]), dev(v[:2]), us_desc_of(O.CSR()))
    X = torch.zeros(3, 4, device="cuda")
    with pytest.raises(B.UnisparseError) as ei:   # N = 0
        B._check(B.lib().us_spmm(B.C.byref(ctx.c), g.handle, X.data_ptr(), 0, 4, X.data_ptr(), 4, 0), "us_spmm")
    assert ei.value.code == "US_ERR_SHAPE"


@pytest.mark.parametrize("nc", [512, 530])
@pytest.mark.parametrize("N", [3, 64, 70, 200])
def test_bcsr44_spmm_fast_and_guarded_groups(ctx, nc, N):
    """4x4 blocks on the matrix cores: block rows with 0..70 blocks (full groups of eight, leftovers, more than
    64 blocks), a block grid that divides the matrix (nc = 512) or sticks out of it (530), ragged N."""
    from paper_2403_05802_amd import binding as B
    from helpers import assert_product, dev, host, row_terms, us_desc_of
    rng = np.random.default_rng(nc + N)
    nr = 301
    rows, cols = [], []
    for br in range((nr + 3) // 4):
        nb = int(rng.integers(0, 71)) if br % 5 else 0
        for bc in rng.choice((nc + 3) // 4, size=min(nb, (nc + 3) // 4), replace=False):
            k = int(rng.integers(1, 17))
            e = rng.choice(16, size=k, replace=False)
            rows.append(br * 4 + e // 4); cols.append(bc * 4 + e % 4)
    r = np.concatenate(rows).astype(np.int32); c = np.concatenate(cols).astype(np.int32)
    keep = (r < nr) & (c < nc)
    r, c = r[keep], c[keep]
    p = rng.permutation(r.size); r, c = r[p], c[p]
    v = rng.uniform(-1, 1, r.size).astype(np.float32); v[v == 0] = 0.5
    g = B.us_convert(ctx, nr, nc, dev(r), dev(c), dev(v), us_desc_of(O.BCSR(4)))
    X = rng.uniform(-1, 1, (nc, N)).astype(np.float32)
    S = O.spmm_coo(nr, nc, r, c, np.abs(v), np.abs(X))
    Y = torch.full((nr, N), -3.0, device="cuda")
    B.us_spmm(ctx, g, dev(X), Y)
    nt = row_terms(nr, r)[:, None]
    assert_product(host(Y), O.spmm_coo(nr, nc, r, c, v, X), S, nt, f"bcsr44 nc={nc} N={N}")
    Y0 = rng.uniform(-1, 1, (nr, N)).astype(np.float32)
    Y = dev(Y0)
    B.us_spmm(ctx, g, dev(X), Y, accumulate=True)
    assert_product(host(Y), O.spmm_coo(nr, nc, r, c, v, X) + Y0, S + np.abs(Y0), nt + 1, f"bcsr44 nc={nc} N={N} accumulate")
    g.free()
