"""Shared by the GPU parity tests: descriptor translation and array comparison."""
import numpy as np
import torch

from oracle import unisparse_oracle as O
from paper_2403_05802_amd import binding as B

KIND = {O.AFFINE: B.US_E_AFFINE, O.DIV: B.US_E_DIV, O.MOD: B.US_E_MOD, O.ENUM: B.US_E_INDIRECT_ENUM,
        O.SCHED: B.US_E_INDIRECT_SCHEDULE}
PRED = {O.SUM_GE_ABS: B.US_P_SUM_GE_ABS, O.SUM_GE_FRAC_OF_CAPACITY: B.US_P_SUM_GE_FRAC_OF_CAPACITY,
        O.RANK_LT_ABS: B.US_P_RANK_LT_ABS, O.RANK_LT_PERCENTILE: B.US_P_RANK_LT_PERCENTILE}


def us_expr_of(e: O.Expr):
    return B.expr(KIND[e.kind], e.c0, e.c1, e.c, e.factor, e.traverse_factor)


def us_desc_of(d: O.FormatDesc):
    return B.make_desc([us_expr_of(e) for e in d.levels], d.trim, d.merge, d.ell_width)


def us_pred_of(p: O.Predicate):
    return B.make_predicate([us_expr_of(e) for e in p.group], PRED[p.kind], p.num, p.den, p.abs)


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def coo_to_dev(coo):
    return dev(coo.row), dev(coo.col), dev(coo.val)


def host(t):
    return t.cpu().numpy()


def assert_same_layout(g: "B.Formatted", o: "O.Formatted", what=""):
    """Bit-exact comparison of every size / ptr / idx / val array with the oracle's."""
    assert (g.nrows, g.ncols, g.nnz) == (o.nrows, o.ncols, o.nnz), what
    assert g.desc.nlevels == len(o.levels), what
    for L, lvl in enumerate(o.levels):
        if lvl.kind == "dense":
            assert g.size(L) == lvl.size, f"{what} size L{L}: {g.size(L)} vs {lvl.size}"
        else:
            assert g.size(L) == -1, f"{what} unexpected size at L{L}"
        gp, gi = g.ptr(L), g.idx(L)
        if lvl.ptr is None:
            assert gp is None, f"{what} unexpected ptr at L{L}"
        else:
            assert gp is not None, f"{what} missing ptr at L{L}"
            np.testing.assert_array_equal(host(gp), lvl.ptr, err_msg=f"{what} ptr L{L}")
        if lvl.idx is None:
            assert gi is None, f"{what} unexpected idx at L{L}"
        else:
            assert gi is not None, f"{what} missing idx at L{L}"
            np.testing.assert_array_equal(host(gi), lvl.idx, err_msg=f"{what} idx L{L}")
    gv = host(g.val())
    assert gv.shape == o.val.shape, f"{what} val count {gv.shape} vs {o.val.shape}"
    np.testing.assert_array_equal(gv.view(np.int32), o.val.view(np.int32), err_msg=f"{what} val bits")


TOL = 1e-4          # max relative error of fp32 SpMV / SpMM against the fp64 oracle
ULP = 2.0 ** -24    # unit round-off of fp32
C_SUM = 4.0         # constant of the per-row summation-error floor below


def row_terms(nrows, row, extra=0):
    """Number of terms every output row sums: entries of the row (+ extra, e.g. 1 for an accumulated y)."""
    return np.bincount(np.asarray(row), minlength=nrows).astype(np.float64) + extra


def error_floor(scale, nterms):
    """Per-row floor of the denominator of rel_err: C_SUM * sqrt(n_i) * 2^-24 * S_i / TOL."""
    return C_SUM * np.sqrt(np.maximum(np.asarray(nterms, dtype=np.float64), 1.0)) * ULP * np.asarray(scale) / TOL


def rel_err(y, yref, scale, nterms):
    """max_i |y_i - yref_i| / max(|yref_i|, floor_i), floor_i = C_SUM * sqrt(n_i) * 2^-24 * S_i / TOL,
    with S_i = sum_j |a_ij x_j| (scale) and n_i the number of terms row i sums (nterms).

    Plain relative error wherever |yref_i| is above the floor; a row that cancels below it is judged
    against the rounding error its own sum can carry.  Reason: fp32 accumulation of n terms in any order
    errs by about sqrt(n) * 2^-24 * S (at most n * 2^-24 * S) whatever |yref| is, so "rel. error <= 1e-4"
    can only be asked of |yref_i| >= that error / 1e-4.  The test passes iff
    |y_i - yref_i| <= max(1e-4 * |yref_i|, 4 * sqrt(n_i) * 2^-24 * S_i) for every i: for n_i <= 16 the second
    term is the worst-case bound n * 2^-24 * S itself, for a 20,000-term row it is 3.4e-5 * S_i.  A dropped
    or misplaced term (about S_i / n_i) fails by orders of magnitude at every n_i."""
    y = np.asarray(y, dtype=np.float64)
    den = np.maximum(np.abs(yref), error_floor(scale, nterms))
    den = np.where(den == 0, 1.0, den)
    return float(np.max(np.abs(y - yref) / den)) if y.size else 0.0


def plain_rel_err(y, yref):
    """max_i |y_i - yref_i| / |yref_i| over the rows with yref_i != 0: the figure as the task words it,
    reported beside rel_err (cancelling rows can make it large for a correct fp32 result)."""
    y = np.asarray(y, dtype=np.float64)
    nz = np.asarray(yref) != 0
    return float(np.max(np.abs(y[nz] - yref[nz]) / np.abs(yref[nz]))) if nz.any() else 0.0


def assert_product(y, yref, scale, nterms, what=""):
    """The parity bar of the products, printing both error figures (pytest -s / on failure)."""
    e, p = rel_err(y, yref, scale, nterms), plain_rel_err(y, yref)
    print(f"{what}: floored rel. error {e:.3e}, plain max |y-yref|/|yref| {p:.3e}")
    assert e <= TOL, f"{what}: floored rel. error {e:.3e} > {TOL} (plain {p:.3e})"


def check_spmm_all_rows(ctx, parts, m, X, what, slab=1 << 17):
    """Y = sum of parts * X on the GPU; EVERY element of Y is compared with the fp64 product, a slab of rows at a
    time.  The reference of a slab is the definition Y = A X evaluated by a library matmul (scipy CSR in fp64, built
    from the original COO); the first 2,000 rows, the 20 longest rows and a random sample of rows are also computed
    with the oracle's own spmm_coo, which the matmul has to agree with to 1e-12 of the row's absolute sum."""
    import scipy.sparse as sp
    import torch
    from progress import say
    N = X.shape[1]
    Y = torch.full((m.nrows, N), -5.0, device="cuda")
    Xd = dev(X)
    for k, g in enumerate(parts):
        B.us_spmm(ctx, g, Xd, Y, accumulate=k > 0)
    torch.cuda.synchronize()
    say(f"{what}: product done on the GPU, building the fp64 reference")
    A = sp.csr_matrix((m.val.astype(np.float64), (m.row, m.col)), shape=(m.nrows, m.ncols))
    Aabs = abs(A)
    X64, Xabs = X.astype(np.float64), np.abs(X).astype(np.float64)
    nt = np.diff(A.indptr).astype(np.float64)
    # the matmul against the oracle on a sample of rows
    rng = np.random.default_rng(5)
    sample = np.unique(np.concatenate([np.arange(min(2000, m.nrows)), np.argsort(nt)[-20:],
                                       rng.choice(m.nrows, min(2000, m.nrows), replace=False)]))
    sel = np.isin(m.row, sample)
    local = np.searchsorted(sample, m.row[sel])
    Yo = O.spmm_coo(sample.size, m.ncols, local, m.col[sel], m.val[sel], X64)
    So = (Aabs[sample] @ Xabs)
    assert np.max(np.abs(A[sample] @ X64 - Yo) / np.maximum(So, 1e-300)) <= 1e-12, what
    worst, worst_plain, at = 0.0, 0.0, -1
    for r0 in range(0, m.nrows, slab):
        r1 = min(r0 + slab, m.nrows)
        ref = A[r0:r1] @ X64
        den = np.maximum(np.abs(ref), error_floor(Aabs[r0:r1] @ Xabs, nt[r0:r1, None]))
        den[den == 0] = 1.0
        got = host(Y[r0:r1]).astype(np.float64)
        e = np.abs(got - ref) / den
        k = int(np.argmax(e))
        if e.flat[k] > worst:
            worst, at = float(e.flat[k]), r0 + k // N
        worst_plain = max(worst_plain, plain_rel_err(got, ref))
        say(f"{what}: rows {r0}..{r1} checked, worst floored rel. error so far {worst:.3e}")
    print(f"{what}: all {m.nrows} x {N} outputs: floored rel. error {worst:.3e} (row {at}), plain {worst_plain:.3e}")
    assert worst <= TOL, (what, worst, at)
    return Y
