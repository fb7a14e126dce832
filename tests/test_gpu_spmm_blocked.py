"""SpMM over BCSR with blocks of every shape (the 4 x 4 matrix-core kernel, the block-row kernel for up to 64 values a
block, the plain loop beyond) and over BDIA with every block height: every output element against the fp64
definition, for the three vector widths (1 / 2 / 4 columns per lane), ragged N, shapes that are no multiples of the
block, strided X and Y, accumulation."""
import numpy as np
import pytest
import scipy.sparse as sp

from oracle import unisparse_oracle as O
import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2403_05802_amd import binding as B
    return B.Context("cuda:0")


def scattered_blocks(rng, nr, nc, n):
    """n distinct entries: clusters around random places (so that blocks hold several entries) plus a band."""
    cr = rng.integers(0, nr, n // 8); cc = rng.integers(0, nc, n // 8)
    r = np.clip(np.repeat(cr, 8) + rng.integers(-3, 4, cr.size * 8), 0, nr - 1)
    c = np.clip(np.repeat(cc, 8) + rng.integers(-3, 4, cc.size * 8), 0, nc - 1)
    i = rng.integers(0, min(nr, nc), n // 4)
    r = np.concatenate([r, i]); c = np.concatenate([c, np.clip(i + rng.integers(-2, 3, i.size), 0, nc - 1)])
    lin = np.unique(r.astype(np.int64) * nc + c)
    p = rng.permutation(lin.size)
    v = rng.uniform(-1, 1, lin.size).astype(np.float32); v[v == 0] = 0.5
    return (lin[p] // nc).astype(np.int32), (lin[p] % nc).astype(np.int32), v


def reference(nr, nc, r, c, v, X, Y0=None):
    A = sp.csr_matrix((v.astype(np.float64), (r, c)), shape=(nr, nc))
    ref = A @ X.astype(np.float64)
    S = abs(A) @ np.abs(X).astype(np.float64)
    if Y0 is not None:
        ref = ref + Y0; S = S + np.abs(Y0)
    return ref, S, H.row_terms(nr, r, 0 if Y0 is None else 1)[:, None]


BLOCKS = [(1, 4), (2, 2), (2, 1), (3, 5), (5, 3), (4, 4), (4, 8), (8, 8), (7, 9), (2, 16), (16, 2), (16, 4), (16, 16), (9, 8)]


@pytest.mark.parametrize("bh,bw", BLOCKS)
@pytest.mark.parametrize("N", [7, 64, 130, 256])
def test_bcsr_spmm_every_output(ctx, bh, bw, N):
    from paper_2403_05802_amd import binding as B
    rng = np.random.default_rng(8000 + 17 * bh + bw + N)
    nr, nc = 3001, 2203
    r, c, v = scattered_blocks(rng, nr, nc, 24_000)
    X = rng.uniform(-1, 1, (nc, N)).astype(np.float32)
    ref, S, nt = reference(nr, nc, r, c, v, X)
    g = B.us_convert(ctx, nr, nc, H.dev(r), H.dev(c), H.dev(v), H.us_desc_of(O.BCSR(bh, bw)))
    Y = H.dev(np.full((nr, N), 3.0, np.float32))
    B.us_spmm(ctx, g, H.dev(X), Y)
    H.assert_product(H.host(Y), ref, S, nt, f"BCSR {bh}x{bw} N={N}")
    g.free()


@pytest.mark.parametrize("bh", [1, 2, 3, 4, 7, 8, 13, 16])
@pytest.mark.parametrize("N", [7, 64, 130, 256])
def test_bdia_spmm_every_output(ctx, bh, N):
    from paper_2403_05802_amd import binding as B
    rng = np.random.default_rng(8100 + 17 * bh + N)
    nr, nc = 3001, 2203
    r, c, v = scattered_blocks(rng, nr, nc, 24_000)
    X = rng.uniform(-1, 1, (nc, N)).astype(np.float32)
    ref, S, nt = reference(nr, nc, r, c, v, X)
    g = B.us_convert(ctx, nr, nc, H.dev(r), H.dev(c), H.dev(v), H.us_desc_of(O.BDIA(bh)))
    Y = H.dev(np.full((nr, N), 3.0, np.float32))
    B.us_spmm(ctx, g, H.dev(X), Y)
    H.assert_product(H.host(Y), ref, S, nt, f"BDIA {bh} N={N}")
    g.free()


@pytest.mark.parametrize("desc", [O.BCSR(8, 8), O.BCSR(3, 5), O.BCSR(16, 16), O.BDIA(4), O.BDIA(13)], ids=str)
@pytest.mark.parametrize("N,ldx,ldy", [(130, 136, 160), (256, 260, 264), (33, 40, 35)])
def test_blocked_spmm_accumulate_and_strides(ctx, desc, N, ldx, ldy):
    from paper_2403_05802_amd import binding as B
    rng = np.random.default_rng(8200 + N)
    nr, nc = 3001, 2203
    r, c, v = scattered_blocks(rng, nr, nc, 24_000)
    Xw = rng.uniform(-1, 1, (nc, ldx)).astype(np.float32)
    Yw0 = rng.uniform(-1, 1, (nr, ldy)).astype(np.float32)
    ref, S, nt = reference(nr, nc, r, c, v, Xw[:, :N], Yw0[:, :N].astype(np.float64))
    g = B.us_convert(ctx, nr, nc, H.dev(r), H.dev(c), H.dev(v), H.us_desc_of(desc))
    Xd, Yd = H.dev(Xw), H.dev(Yw0)
    B.us_spmm(ctx, g, Xd[:, :N], Yd[:, :N], accumulate=True)
    got = H.host(Yd)
    assert np.array_equal(got[:, N:], Yw0[:, N:])
    H.assert_product(got[:, :N], ref, S, nt, f"strided accumulate N={N}")
    g.free()


@pytest.mark.parametrize("bh,bw", [(64, 48), (300, 700), (1, 1), (4000, 4000)])
@pytest.mark.parametrize("N", [0, 7, 64, 130, 256])
def test_csb_products_every_output(ctx, bh, bw, N):
    """CSB: runs of one row inside a block are summed before they reach y / Y (N = 0: SpMV)."""
    from paper_2403_05802_amd import binding as B
    rng = np.random.default_rng(8300 + bh + N)
    nr, nc = 3001, 2203
    r, c, v = scattered_blocks(rng, nr, nc, 60_000)
    g = B.us_convert(ctx, nr, nc, H.dev(r), H.dev(c), H.dev(v), H.us_desc_of(O.CSB(bh, bw)))
    if N == 0:
        x = rng.uniform(-1, 1, nc).astype(np.float32)
        ref, S, nt = reference(nr, nc, r, c, v, x[:, None])
        y = H.dev(np.full(nr, 3.0, np.float32))
        B.us_spmv(ctx, g, H.dev(x), y)
        H.assert_product(H.host(y), ref[:, 0], S[:, 0], nt[:, 0], f"CSB {bh}x{bw} SpMV")
        y0 = rng.uniform(-1, 1, nr).astype(np.float32)
        ref, S, nt = reference(nr, nc, r, c, v, x[:, None], y0[:, None].astype(np.float64))
        y = H.dev(y0)
        B.us_spmv(ctx, g, H.dev(x), y, accumulate=True)
        H.assert_product(H.host(y), ref[:, 0], S[:, 0], nt[:, 0], f"CSB {bh}x{bw} SpMV accumulate")
    else:
        X = rng.uniform(-1, 1, (nc, N)).astype(np.float32)
        ref, S, nt = reference(nr, nc, r, c, v, X)
        Y = H.dev(np.full((nr, N), 3.0, np.float32))
        B.us_spmm(ctx, g, H.dev(X), Y)
        H.assert_product(H.host(Y), ref, S, nt, f"CSB {bh}x{bw} N={N}")
    g.free()
