"""Seeded sweep over shapes, densities, formats, block sizes and both Sort paths: conversion bit-exact
against the oracle, SpMV / SpMM within tolerance.  Small cases, many of them, one process."""
import numpy as np
import pytest
import torch

from oracle import unisparse_oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2403_05802_amd import binding as B
    return B.Context("cuda:0")


def draw_case(seed):
    rng = np.random.default_rng(1000 + seed)
    shape_kind = rng.integers(0, 5)
    if shape_kind == 0:
        nr, nc = int(rng.integers(1, 40)), int(rng.integers(1, 40))
    elif shape_kind == 1:
        nr, nc = int(rng.integers(1, 8)), int(rng.integers(2000, 60000))
    elif shape_kind == 2:
        nr, nc = int(rng.integers(2000, 60000)), int(rng.integers(1, 8))
    else:
        nr, nc = int(rng.integers(50, 5000)), int(rng.integers(50, 5000))
    cap = nr * nc
    nnz = int(min(cap, rng.choice([0, 1, 7, 300, 5000, 12000, 40000])))
    fmt_kind = int(rng.integers(0, 11))
    if fmt_kind in (5, 6) and nnz > 3000:     # dense diagonal slabs: keep the slab small by banding the entries
        offs = rng.choice(np.arange(-(nr - 1), nc), size=min(6, nr + nc - 1), replace=False)
        rows, cols = [], []
        for off in offs:
            i = np.arange(max(0, -off), min(nr, nc - off))
            i = i[rng.random(i.size) < 0.7]
            rows.append(i); cols.append(i + off)
        r = np.concatenate(rows).astype(np.int32); c = np.concatenate(cols).astype(np.int32)
    else:
        lin = rng.choice(cap, size=nnz, replace=False) if cap < 2 ** 31 else np.unique(rng.integers(0, cap, nnz))
        r, c = (lin // nc).astype(np.int32), (lin % nc).astype(np.int32)
    if rng.random() < 0.3 and r.size > 50:    # a heavy row / column
        k = int(min(nc, r.size // 3))
        hr = np.full(k, int(rng.integers(0, nr)), np.int32); hc = rng.choice(nc, k, replace=False).astype(np.int32)
        lin = np.unique(np.concatenate([r.astype(np.int64) * nc + c, hr.astype(np.int64) * nc + hc]))
        r, c = (lin // nc).astype(np.int32), (lin % nc).astype(np.int32)
    p = rng.permutation(r.size); r, c = r[p], c[p]
    v = rng.uniform(-1, 1, r.size).astype(np.float32); v[v == 0] = 0.25
    desc = [O.COO(), O.CSR(), O.DCSR(), O.CSC(), O.DCSC(), O.DIA(), O.DIA_VARIANT(),
            O.BCSR(int(rng.integers(1, 17)), int(rng.integers(1, 17))), O.BDIA(int(rng.integers(1, 17))),
            O.CSB(int(rng.integers(1, 300)), int(rng.integers(1, 300))),
            O.CISR_PLUS(int(rng.choice([1, 2, 7, 64, 1000, 65536])))][fmt_kind]
    if fmt_kind == 8 and r.size > 3000 and nr * 1.0 * r.size > 2 ** 27:
        desc = O.CSR()                         # a scattered matrix in BDIA: nodes x block would be huge
    mode = [None, True, False][seed % 3]
    return nr, nc, r, c, v, desc, mode


@pytest.mark.parametrize("chunk", range(6))
def test_random_cases(ctx, chunk):
    from paper_2403_05802_amd import binding as B
    from helpers import assert_product, row_terms, assert_same_layout, dev, host, us_desc_of
    try:
        for seed in range(chunk * 20, chunk * 20 + 20):
            nr, nc, r, c, v, desc, mode = draw_case(seed)
            what = f"seed {seed}: {nr}x{nc} nnz={r.size} {desc} mode={mode}"
            ctx.set_sort_lds_finish(mode)
            o = O.convert(nr, nc, r, c, v, desc)
            g = B.us_convert(ctx, nr, nc, dev(r), dev(c), dev(v), us_desc_of(desc))
            assert_same_layout(g, o, what)
            rng = np.random.default_rng(seed)
            x = rng.uniform(-1, 1, nc).astype(np.float32)
            y = torch.full((nr,), 5.0, device="cuda")
            B.us_spmv(ctx, g, dev(x), y)
            assert_product(host(y), O.spmv_coo(nr, nc, r, c, v, x), O.abs_row_sums(nr, r, c, v, x), row_terms(nr, r), what)
            N = int(rng.choice([1, 3, 64, 128, 200]))
            if nr * N <= 2_000_000 and nc * N <= 8_000_000:
                X = rng.uniform(-1, 1, (nc, N)).astype(np.float32)
                Y = torch.full((nr, N), 5.0, device="cuda")
                B.us_spmm(ctx, g, dev(X), Y)
                S = O.spmm_coo(nr, nc, r, c, np.abs(v), np.abs(X))
                assert_product(host(Y), O.spmm_coo(nr, nc, r, c, v, X), S, row_terms(nr, r)[:, None], what)
            g.free()
    finally:
        ctx.set_sort_lds_finish(None)


def draw_decomposition(seed):
    rng = np.random.default_rng(5000 + seed)
    nr, nc = int(rng.integers(20, 3000)), int(rng.integers(20, 3000))
    # a few broken diagonals, a few dense blocks, scattered entries and one long row: every predicate finds both kinds
    have = set()
    for off in rng.choice(np.arange(-(nr - 1), nc), size=3, replace=False):
        i = np.arange(max(0, -off), min(nr, nc - off))
        i = i[rng.random(i.size) < 0.9]
        have.update(zip(i.tolist(), (i + off).tolist()))
    for _ in range(30):
        br, bc = int(rng.integers(0, nr)), int(rng.integers(0, nc))
        for a in range(br, min(nr, br + 4)):
            for b in range(bc, min(nc, bc + 4)):
                if rng.random() < 0.8:
                    have.add((a, b))
    for e in rng.integers(0, nr * nc, int(rng.choice([50, 2000, 9000]))).tolist():
        have.add((e // nc, e % nc))
    long_row = int(rng.integers(0, nr))
    for b in rng.choice(nc, size=min(nc, 400), replace=False).tolist():
        have.add((long_row, b))
    rc = np.array(sorted(have), dtype=np.int32)
    rc = rc[rng.permutation(rc.shape[0])]
    r, c = rc[:, 0].copy(), rc[:, 1].copy()
    v = rng.uniform(-1, 1, r.size).astype(np.float32); v[v == 0] = 0.25
    kind = int(rng.integers(0, 8))
    b1, b2 = int(rng.integers(1, 9)), int(rng.integers(1, 9))
    sparse_fmts = [O.COO(), O.CSR(), O.DCSR(), O.CSC(), O.DCSC(), O.BCSR(b1, b2), O.ELL()]
    pick = lambda: sparse_fmts[int(rng.integers(0, len(sparse_fmts)))]
    if kind == 0:
        pred, da, db = O.Predicate((O.diag(),), O.SUM_GE_FRAC_OF_CAPACITY, num=int(rng.integers(1, 10)), den=10), O.DIA(), pick()
    elif kind == 1:
        pred, da, db = O.Predicate((O.diag(),), O.SUM_GE_ABS, abs=int(rng.integers(2, 200))), O.DIA_VARIANT(), pick()
    elif kind == 2:
        pred, da, db = O.Predicate((O.d0(),), O.SUM_GE_ABS, abs=int(rng.integers(1, 60))), pick(), pick()
    elif kind == 3:
        pred, da, db = O.Predicate((O.d1(),), O.SUM_GE_ABS, abs=int(rng.integers(1, 20))), pick(), pick()
    elif kind == 4:
        pred, da, db = O.Predicate((O.d0(),), O.RANK_LT_ABS, abs=int(rng.integers(0, 12))), pick(), pick()
    elif kind == 5:
        pred, da, db = O.Predicate((O.d0(),), O.RANK_LT_PERCENTILE, num=int(rng.integers(1, 11)), den=10), O.ELL(), pick()
    elif kind == 6:
        pred, da, db = O.Predicate((O.div(0, b1), O.diag()), O.SUM_GE_ABS, abs=int(rng.integers(1, b1 + 2))), O.BDIA(b1), pick()
    else:
        pred = O.Predicate((O.div(0, b1), O.div(1, b2)), O.SUM_GE_ABS, abs=int(rng.integers(1, b1 * b2 + 2)))
        da, db = (O.BELL(b1, b2) if seed % 2 else O.BCSR(b1, b2)), pick()   # blocked ELL for every other seed
    return nr, nc, r, c, v, da, db, pred, [None, True, False][seed % 3]


@pytest.mark.parametrize("chunk", range(4))
def test_random_decompositions(ctx, chunk):
    from paper_2403_05802_amd import binding as B
    from helpers import assert_product, row_terms, assert_same_layout, dev, host, us_desc_of, us_pred_of
    try:
        for seed in range(chunk * 12, chunk * 12 + 12):
            nr, nc, r, c, v, da, db, pred, mode = draw_decomposition(seed)
            what = f"seed {seed}: {nr}x{nc} nnz={r.size} {pred.kind} {pred.group} mode={mode}"
            ctx.set_sort_lds_finish(mode)
            oa, ob, mask = O.decompose(nr, nc, r, c, v, da, db, pred)
            ga, gb = B.us_decompose(ctx, nr, nc, dev(r), dev(c), dev(v), us_desc_of(da), us_desc_of(db), us_pred_of(pred))
            assert_same_layout(ga, oa, what + " part A")
            assert_same_layout(gb, ob, what + " part B")
            x = np.random.default_rng(seed).uniform(-1, 1, nc).astype(np.float32)
            y = torch.full((nr,), 5.0, device="cuda")
            B.us_spmv(ctx, ga, dev(x), y); B.us_spmv(ctx, gb, dev(x), y, accumulate=True)
            assert_product(host(y), O.spmv_coo(nr, nc, r, c, v, x), O.abs_row_sums(nr, r, c, v, x), row_terms(nr, r), what)
            ga.free(); gb.free()
    finally:
        ctx.set_sort_lds_finish(None)


def spoil(rng, nr, nc, r, c, v):
    """A repeated coordinate, a coordinate outside the matrix, or both, somewhere in the list."""
    kind = int(rng.integers(0, 3))
    r, c, v = r.copy(), c.copy(), v.copy()
    if kind in (0, 2):
        a, b = rng.choice(r.size, 2, replace=False)
        r[b], c[b] = r[a], c[a]
    if kind in (1, 2):
        k = int(rng.integers(0, r.size))
        which = int(rng.integers(0, 4))
        if which == 0: r[k] = nr + int(rng.integers(0, 5))
        elif which == 1: c[k] = nc + int(rng.integers(0, 5))
        elif which == 2: r[k] = -1 - int(rng.integers(0, 3))
        else: c[k] = np.int32(2 ** 31 - 1)
    return r, c, v


def test_random_invalid_inputs(ctx):
    """Every conversion and decomposition path names the same error as the oracle (a coordinate out of range
    before a repeated one) and leaves no memory behind; 10,000 more seeds of this ran clean once."""
    from paper_2403_05802_amd import binding as B
    from helpers import dev, us_desc_of, us_pred_of
    before = ctx.live_bytes()
    try:
        for seed in range(240):
            rng = np.random.default_rng(77000 + seed)
            if seed % 2 == 0:
                nr, nc, r, c, v, desc, mode = draw_case(seed)
                if r.size < 2:
                    continue
                r, c, v = spoil(rng, nr, nc, r, c, v)
                call_o = lambda: O.convert(nr, nc, r, c, v, desc)
                call_g = lambda: (B.us_convert(ctx, nr, nc, dev(r), dev(c), dev(v), us_desc_of(desc)),)
            else:
                nr, nc, r, c, v, da, db, pred, mode = draw_decomposition(seed)
                r, c, v = spoil(rng, nr, nc, r, c, v)
                call_o = lambda: O.decompose(nr, nc, r, c, v, da, db, pred)
                call_g = lambda: B.us_decompose(ctx, nr, nc, dev(r), dev(c), dev(v), us_desc_of(da), us_desc_of(db),
                                                us_pred_of(pred))
            ctx.set_sort_lds_finish(mode)
            try:
                call_o(); want = "US_OK"
            except O.OracleError as e:
                want = e.code
            try:
                for g in call_g():
                    g.free()
                got = "US_OK"
            except B.UnisparseError as e:
                got = e.code
            assert got == want, f"seed {seed}"
            assert want in ("US_ERR_INDEX_RANGE", "US_ERR_DUPLICATE")
    finally:
        ctx.set_sort_lds_finish(None)
    assert ctx.live_bytes() == before
