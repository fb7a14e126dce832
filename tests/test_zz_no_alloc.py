"""us_spmv_noalloc, the product for callers that cannot allocate: same bits as us_spmv, no call into the
allocator, on two calls in a row (the second over a smaller tensor: the shared scratch then still holds what the
first left), and a clear error beyond the scratch limit."""
import numpy as np
import pytest
import torch

from paper_2403_05802_amd import workloads as W

pytestmark = pytest.mark.gpu


def bits(t):
    return t.view(torch.int32)


def test_noalloc_spmv_matches_spmv_and_never_allocates():
    from paper_2403_05802_amd import binding as B
    from helpers import dev
    ctx = B.Context("cuda:0")
    P = B.us_desc_preset
    big = W.cfg2_powerlaw(n=1 << 16, target_nnz=1 << 21, max_len=20000, empty_frac=0.3)
    small = W.cfg2_powerlaw(n=3000, target_nnz=20000, max_len=900, empty_frac=0.3, index=7)
    formats = [B.US_F_CSR, B.US_F_DCSR, B.US_F_COO, (B.US_F_CISR_PLUS, 64), B.US_F_CSC, (B.US_F_BCSR, 4, 4), B.US_F_ELL]
    for fmt in formats:
        desc = P(*fmt) if isinstance(fmt, tuple) else P(fmt)
        tensors = []
        for m in (big, small):        # the larger tensor first: the second call finds its leftovers in the scratch
            if fmt == B.US_F_ELL and m is big:
                m = W.cfg4_blockfem(n=1 << 14, band_blocks=64)   # (an ELL slab of a 20,000-entry row would be huge)
            g = B.us_convert(ctx, m.nrows, m.ncols, dev(m.row), dev(m.col), dev(m.val), desc)
            x = dev(W.dense_operand(2, m.ncols))
            y0 = dev(W.dense_operand(3, m.nrows))
            tensors.append((m, g, x, y0))
        for acc in (False, True):
            want = []
            for m, g, x, y0 in tensors:
                y = y0.clone()
                B.us_spmv(ctx, g, x, y, accumulate=acc)
                want.append(y)
            torch.cuda.synchronize()
            outs = [y0.clone() for _, _, _, y0 in tensors]
            torch.cuda.synchronize()
            n_before, live_before = ctx._nalloc, ctx.live_bytes()
            for (m, g, x, y0), y in zip(tensors, outs):        # two calls in a row, nothing in between
                B.us_spmv_noalloc(ctx, g, x, y, accumulate=acc)
            torch.cuda.synchronize()
            assert ctx._nalloc == n_before and ctx.live_bytes() == live_before, fmt
            atomic = fmt in (B.US_F_CSC,)      # scatter form: fp32 atomics, the order of the adds is not fixed
            for (m, g, x, y0), y, w in zip(tensors, outs, want):
                if atomic:
                    assert torch.allclose(y, w, rtol=1e-4, atol=1e-4), (fmt, acc)
                else:
                    assert torch.equal(bits(y), bits(w)), (fmt, acc, m.nrows)
        for _, g, _, _ in tensors:
            g.free()


def test_noalloc_spmv_rejects_what_does_not_fit():
    """Compressed rows take 8 bytes of scratch per 2048 rows + entries: 2^31 - 1 entries in 2^20 rows need
    8,392,704 bytes, the array holds 8 MiB = 8,388,608; 2^29 entries fit."""
    from paper_2403_05802_amd import binding as B
    from test_gpu_large import generate
    ctx = B.Context("cuda:0")
    dim, n, row, col, val, _ = generate((1 << 31) - 1)
    g = B.us_convert(ctx, dim, dim, row, col, val, B.us_desc_preset(B.US_F_CSR))
    del row, col, val
    x = torch.ones(dim, device="cuda")
    y = torch.full((dim,), 3.0, device="cuda")
    n_before = ctx._nalloc
    with pytest.raises(B.UnisparseError) as ei:
        B.us_spmv_noalloc(ctx, g, x, y)
    assert ei.value.code == "US_ERR_SCRATCH_LIMIT" and ctx._nalloc == n_before
    torch.cuda.synchronize()
    assert bool((y == 3.0).all())          # nothing was enqueued
    g.free()
    dim, n, row, col, val, _ = generate(1 << 29)
    g = B.us_convert(ctx, dim, dim, row, col, val, B.us_desc_preset(B.US_F_CSR))
    del row, col, val
    y2 = torch.empty(dim, device="cuda")
    B.us_spmv(ctx, g, x, y)
    B.us_spmv_noalloc(ctx, g, x, y2)
    assert torch.equal(bits(y2), bits(y))
    g.free()
