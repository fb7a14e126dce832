"""The optional in-LDS finish of the Sort step gives the same arrays as the whole-array digit
passes: small buckets, buckets that need the extra split, and inputs that make the call fall
back (retry) -- all against the oracle."""
import contextlib

import numpy as np
import pytest

from oracle import unisparse_oracle as O
from paper_2403_05802_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2403_05802_amd import binding as B
    return B.Context("cuda:0")


@contextlib.contextmanager
def lds_finish(ctx):
    ctx.set_sort_lds_finish(True)
    try:
        yield
    finally:
        ctx.set_sort_lds_finish(None)


def distinct(nr, nc, r, c):
    lin = np.unique(r.astype(np.int64) * nc + c)
    return (lin // nc).astype(np.int32), (lin % nc).astype(np.int32)


def shuffled(rng, r, c):
    p = rng.permutation(r.size)
    v = rng.uniform(0.1, 1, r.size).astype(np.float32)
    return r[p], c[p], v


def scatter_passes(ctx, nr, nc, r, c, v, desc):
    """Whole-array digit passes one conversion runs (launches of the scatter kernel), with the option on."""
    from paper_2403_05802_amd import binding as B
    from helpers import dev, us_desc_of
    ctx.enable_profile(); ctx.profile_reset()
    try:
        with lds_finish(ctx):
            B.us_convert(ctx, nr, nc, dev(r), dev(c), dev(v), us_desc_of(desc)).free()
        return {e["kernel"]: e["launches"] for e in ctx.profile_report()}.get("radix_scatter", 0)
    finally:
        ctx.disable_profile()


def check(ctx, nr, nc, r, c, v, descs):
    from paper_2403_05802_amd import binding as B
    from helpers import assert_same_layout, dev, us_desc_of
    for d in descs:
        o = O.convert(nr, nc, r, c, v, d)
        with lds_finish(ctx):
            g = B.us_convert(ctx, nr, nc, dev(r), dev(c), dev(v), us_desc_of(d))
        assert_same_layout(g, o, str(d))
        g.free()


def test_uniform_entries_every_sorted_format(ctx):
    rng = np.random.default_rng(11)
    nr, nc, n = 50_000, 70_001, 300_000
    r, c = distinct(nr, nc, rng.integers(0, nr, n), rng.integers(0, nc, n))
    r, c, v = shuffled(rng, r, c)
    check(ctx, nr, nc, r, c, v, [O.CSR(), O.CSC(), O.DCSR(), O.COO(), O.BCSR(4), O.BCSR(2, 3), O.ELL(), O.BDIA(3)])


def test_heavy_row_goes_through_the_extra_split(ctx):
    """16 rows share the top key bits; one of them holds 24,000 entries: a bucket of ~26,000 that
    the 8-bit split cuts into pieces of ~1,500."""
    rng = np.random.default_rng(12)
    nr, nc = 1024, 1 << 20
    r = np.concatenate([rng.integers(0, nr, 100_000), np.full(24_000, 5)])
    c = np.concatenate([rng.integers(0, nc, 100_000), rng.integers(0, nc, 24_000)])
    r, c = distinct(nr, nc, r, c)
    r, c, v = shuffled(rng, r, c)
    check(ctx, nr, nc, r, c, v, [O.CSR(), O.DCSR(), O.BCSR(4)])
    # 30 key bits, 6 of them sorted by one whole-array pass: no second attempt happened
    assert scatter_passes(ctx, nr, nc, r, c, v, O.CSR()) == 1


def test_inputs_the_finish_cannot_take_are_sorted_again(ctx):
    rng = np.random.default_rng(13)
    nr = nc = 1 << 20
    # (a) a 10,000-entry row among 4,096 rows of equal top bits: one piece of the split stays too large
    r = np.concatenate([rng.integers(0, nr, 200_000), np.full(10_000, 77)])
    c = np.concatenate([rng.integers(0, nc, 200_000), rng.integers(0, nc, 10_000)])
    r, c = distinct(nr, nc, r, c)
    r, c, v = shuffled(rng, r, c)
    check(ctx, nr, nc, r, c, v, [O.CSR(), O.COO()])
    assert scatter_passes(ctx, nr, nc, r, c, v, O.CSR()) == 1 + 5      # one pass of the attempt, then 40 bits / 8
    # (b) 300,000 entries in four rows: more than 64 tiles share their top bits
    r, c = distinct(nr, nc, rng.integers(0, 4, 300_000), rng.integers(0, nc, 300_000))
    r, c, v = shuffled(rng, r, c)
    check(ctx, nr, nc, r, c, v, [O.CSR(), O.CSC()])
    assert scatter_passes(ctx, nr, nc, r, c, v, O.CSR()) == 1 + 5


def test_errors_are_reported_on_this_path_too(ctx):
    from paper_2403_05802_amd import binding as B
    from helpers import dev, us_desc_of
    rng = np.random.default_rng(14)
    nr, nc = 1024, 1 << 20
    r = np.concatenate([rng.integers(0, nr, 100_000), np.full(24_000, 5)])
    c = np.concatenate([rng.integers(0, nc, 100_000), rng.integers(0, nc, 24_000)])
    r, c = distinct(nr, nc, r, c)
    r, c, v = shuffled(rng, r, c)
    for at in (3, r.size - 1, int(np.flatnonzero(r == 5)[7])):       # duplicate in a small and in a split bucket
        r2 = np.append(r, r[at]); c2 = np.append(c, c[at]); v2 = np.append(v, np.float32(1))
        for d in (O.CSR(), O.BCSR(4)):
            with lds_finish(ctx), pytest.raises(B.UnisparseError) as ei:
                B.us_convert(ctx, nr, nc, dev(r2), dev(c2), dev(v2), us_desc_of(d))
            assert ei.value.code == "US_ERR_DUPLICATE"
    for bad_r, bad_c in ((nr, 0), (0, nc), (-1, 3), (2**31 - 1, 2**31 - 1)):
        r2 = np.append(r, np.int32(bad_r)); c2 = np.append(c, np.int32(bad_c)); v2 = np.append(v, np.float32(1))
        for d in (O.CSR(), O.BCSR(4), O.CSC()):
            with lds_finish(ctx), pytest.raises(B.UnisparseError) as ei:
                B.us_convert(ctx, nr, nc, dev(r2), dev(c2), dev(v2), us_desc_of(d))
            assert ei.value.code == "US_ERR_INDEX_RANGE"


def test_scaled_workloads_and_hybrids(ctx):
    from paper_2403_05802_amd import binding as B
    from helpers import assert_same_layout, coo_to_dev, us_desc_of, us_pred_of
    m = W.cfg2_powerlaw(n=1 << 16, target_nnz=1 << 20, max_len=20000)
    check(ctx, m.nrows, m.ncols, m.row, m.col, m.val, [O.CSR(), O.DCSR()])
    m = W.cfg4_blockfem(n=1 << 15)
    check(ctx, m.nrows, m.ncols, m.row, m.col, m.val, [O.BCSR(4)])
    m = W.cfg5_powerlaw_local(n=100_000, target_nnz=2_000_000, max_len=20000)
    pred = O.Predicate((O.d0(),), O.RANK_LT_PERCENTILE, num=9, den=10)
    oa, ob, _ = O.decompose(m.nrows, m.ncols, m.row, m.col, m.val, O.ELL(), O.COO(), pred)
    with lds_finish(ctx):
        ga, gb = B.us_decompose(ctx, m.nrows, m.ncols, *coo_to_dev(m), us_desc_of(O.ELL()), us_desc_of(O.COO()),
                                us_pred_of(pred))
    assert_same_layout(ga, oa, "ELL part"); assert_same_layout(gb, ob, "COO part")


def blocks_matrix(rng, nr, nc, bh, bw, nblocks, fill):
    """`nblocks` distinct bh x bw blocks at random places, `fill` entries in each (at random in-block positions)."""
    nbr, nbc = -(-nr // bh), -(-nc // bw)
    blk = rng.choice(nbr * nbc, size=nblocks, replace=False)
    rows, cols = [], []
    for b in blk:
        at = rng.choice(bh * bw, size=min(fill, bh * bw), replace=False)
        rows.append((b // nbc) * bh + at // bw)
        cols.append((b % nbc) * bw + at % bw)
    r, c = np.concatenate(rows), np.concatenate(cols)
    keep = (r < nr) & (c < nc)
    return distinct(nr, nc, r[keep], c[keep])


# (bh, bw, entries per block, blocks): few nodes per bucket (counted ranks), hundreds (sorted ranks), more than the
# table takes or a bit map that does not fit (the bucket's entries are sorted instead), multi-word bit maps (8x8, 16x16),
# block shapes that are no powers of two, a block height of one
RANK_CASES = [(4, 4, 16, 12_000), (4, 4, 5, 40_000), (4, 4, 2, 90_000), (4, 4, 1, 150_000), (4, 4, 1, 260_000), (2, 2, 3, 60_000),
              (8, 8, 40, 5_000), (8, 8, 3, 60_000), (16, 16, 200, 1_000), (16, 16, 2, 90_000), (3, 5, 9, 20_000),
              (5, 3, 2, 80_000), (1, 4, 3, 60_000), (16, 1, 7, 25_000)]


@pytest.mark.parametrize("bh,bw,fill,nblocks", RANK_CASES)
def test_blocked_tuples_placed_by_node_rank(ctx, bh, bw, fill, nblocks):
    rng = np.random.default_rng(1000 + 37 * bh + 5 * bw + fill)
    nr, nc = 30_011, 41_003
    r, c = blocks_matrix(rng, nr, nc, bh, bw, nblocks, fill)
    r, c, v = shuffled(rng, r, c)
    descs = [O.BCSR(bh, bw)] + ([O.BELL(bh, bw)] if bh * bw <= 64 else []) + ([O.BDIA(bh)] if bw == 1 or bh == bw else [])
    check(ctx, nr, nc, r, c, v, descs)


@pytest.mark.parametrize("bh,bw,fill,nblocks", [(4, 4, 16, 12_000), (4, 4, 2, 90_000), (4, 4, 1, 260_000), (8, 8, 40, 5_000),
                                                (16, 16, 2, 90_000)])
def test_duplicates_are_found_whichever_way_a_bucket_is_finished(ctx, bh, bw, fill, nblocks):
    from paper_2403_05802_amd import binding as B
    from helpers import dev, us_desc_of
    rng = np.random.default_rng(2000 + 37 * bh + fill)
    nr, nc = 30_011, 41_003
    r, c = blocks_matrix(rng, nr, nc, bh, bw, nblocks, fill)
    r, c, v = shuffled(rng, r, c)
    for at in (0, r.size // 2, r.size - 1):
        r2 = np.append(r, r[at]); c2 = np.append(c, c[at]); v2 = np.append(v, np.float32(1))
        p = rng.permutation(r2.size)
        for d in (O.BCSR(bh, bw), O.BDIA(bh)):
            with lds_finish(ctx), pytest.raises(B.UnisparseError) as ei:
                B.us_convert(ctx, nr, nc, dev(r2[p]), dev(c2[p]), dev(v2[p]), us_desc_of(d))
            assert ei.value.code == "US_ERR_DUPLICATE"


def test_pieces_between_half_and_full_capacity_are_groups_of_their_own(ctx):
    """8 rows share the top key bits; one of them holds 100,000 entries: the 8-bit split of that bucket leaves pieces
    of ~3,100 entries (row, 32,768 columns), more than pieces may have to be bundled and still small enough for one
    workgroup: no second attempt."""
    rng = np.random.default_rng(15)
    nr, nc = 1024, 1 << 20
    r = np.concatenate([rng.integers(0, nr, 60_000), np.full(100_000, 5)])
    c = np.concatenate([rng.integers(0, nc, 60_000), rng.choice(nc, 100_000, replace=False)])
    r, c = distinct(nr, nc, r, c)
    per_piece = np.bincount(c[r == 5] >> 15)
    assert 2048 < per_piece.max() <= 4096
    r, c, v = shuffled(rng, r, c)
    check(ctx, nr, nc, r, c, v, [O.CSR(), O.DCSR(), O.COO(), O.BCSR(4), O.BDIA(2)])
    assert scatter_passes(ctx, nr, nc, r, c, v, O.CSR()) == 1
