"""SpMM over the entry-balanced layouts (CSR, COO, DCSR) on a power-law matrix of a few million entries with rows of
thousands of entries and an X larger than the L2s: every output element against the fp64 definition, for the
vector widths 1 / 2 / 4 columns per lane, ragged N, strided X and Y, accumulation, bit-for-bit reproducibility."""
import numpy as np
import pytest
import torch

from oracle import unisparse_oracle as O
from paper_2403_05802_amd import workloads as W
import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2403_05802_amd import binding as B
    return B.Context("cuda:0")


@pytest.fixture(scope="module")
def matrix():
    # 300,000 rows, ~3 M entries, rows of up to 20,000 entries: ~40 % of the entries sit in rows of 256 and more
    return W.cfg2_powerlaw(n=300_000, target_nnz=3_000_000, s=1.6, max_len=20000, index=8)


@pytest.mark.parametrize("N", [40, 130, 260])
def test_powerlaw_spmm_every_output(ctx, matrix, N):
    from paper_2403_05802_amd import binding as B
    m = matrix
    lens = np.bincount(m.row, minlength=m.nrows)
    assert lens.max() > 2048 and lens[lens >= 256].sum() >= m.nnz // 2      # rows cut by many chunk boundaries
    d = H.coo_to_dev(m)
    X = W.dense_operand(8, (m.ncols, N))
    for desc in (O.CSR(), O.COO(), O.DCSR()):
        g = B.us_convert(ctx, m.nrows, m.ncols, *d, H.us_desc_of(desc))
        Y1 = H.check_spmm_all_rows(ctx, [g], m, X, f"power-law {desc.trim} N={N}", slab=1 << 16)
        Y2 = torch.full_like(Y1, 9.0)
        B.us_spmm(ctx, g, H.dev(X), Y2)
        assert torch.equal(Y1.view(torch.int32), Y2.view(torch.int32))
        g.free()


def test_powerlaw_spmm_accumulate_and_strides(ctx, matrix):
    from paper_2403_05802_amd import binding as B
    m = matrix
    N, ldx, ldy = 130, 136, 160
    rng = np.random.default_rng(41)
    Xw = rng.uniform(-1, 1, (m.ncols, ldx)).astype(np.float32)
    Yw0 = rng.uniform(-1, 1, (m.nrows, ldy)).astype(np.float32)
    import scipy.sparse as sp
    A = sp.csr_matrix((m.val.astype(np.float64), (m.row, m.col)), shape=(m.nrows, m.ncols))
    ref = A @ Xw[:, :N].astype(np.float64) + Yw0[:, :N]
    S = abs(A) @ np.abs(Xw[:, :N]).astype(np.float64) + np.abs(Yw0[:, :N])
    nt = H.row_terms(m.nrows, m.row, 1)[:, None]
    g = B.us_convert(ctx, m.nrows, m.ncols, *H.coo_to_dev(m), H.us_desc_of(O.CSR()))
    Xd, Yd = H.dev(Xw), H.dev(Yw0)
    B.us_spmm(ctx, g, Xd[:, :N], Yd[:, :N], accumulate=True)
    got = H.host(Yd)
    assert np.array_equal(got[:, N:], Yw0[:, N:])
    H.assert_product(got[:, :N], ref, S, nt, "power-law, strided, accumulate")
    g.free()
