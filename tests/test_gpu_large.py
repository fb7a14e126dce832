"""Beyond the benchmark sizes: 2^29 entries (record and index arrays of more than 2^32 bytes) and the largest
count the interface takes, 2^31 - 1, checked by properties that hold at any size -- the oracle cannot get
there in minutes.

The input is generated on the device: entry i sits at linear position L_i = (i * A) mod 2^40 of a
2^20 x 2^20 matrix (A odd, so positions are distinct and arrive in scrambled order) and carries the small
integer f(L_i), so that the value that ends up beside a coordinate can be recomputed from the coordinate,
and every sum of values in a row is an integer below 2^24: fp32 adds them exactly in any order."""
import pytest
import torch

pytestmark = pytest.mark.gpu

LOG_DIM = 20
A = 0x9E3779B97F4A7C15 & ((1 << 40) - 1) | 1


def f_of(lin: torch.Tensor) -> torch.Tensor:
    return ((lin * 40503 + 12345) % 4093 + 1).to(torch.float32)


def generate(n):
    dim = 1 << LOG_DIM
    i = torch.arange(n, dtype=torch.int64, device="cuda")
    lin = (i * A) & ((1 << 40) - 1)            # wraps mod 2^64 first, which keeps the map a bijection mod 2^40
    del i
    row = (lin >> LOG_DIM).to(torch.int32)
    col = (lin & (dim - 1)).to(torch.int32)
    val = f_of(lin)
    sums = (int(lin.sum()), int((lin * lin).sum()))   # mod 2^64
    del lin
    return dim, n, row, col, val, sums


@pytest.mark.parametrize("n,finish", [(1 << 29, None), (1 << 29, True), ((1 << 31) - 1, None)],
                         ids=["2^29_whole_array_passes", "2^29_lds_finish", "2^31-1_whole_array_passes"])
def test_csr_beyond_the_benchmark_sizes(n, finish):
    from paper_2403_05802_amd import binding as B
    dim, n, row, col, val, sums = generate(n)
    ctx = B.Context("cuda:0")
    ctx.set_sort_lds_finish(finish)
    try:
        g = B.us_convert(ctx, dim, dim, row, col, val, B.us_desc_preset(B.US_F_CSR))
    finally:
        ctx.set_sort_lds_finish(None)
    ptr, idx, v = g.ptr(1), g.idx(1), g.val()
    assert ptr.numel() == dim + 1 and idx.numel() == n and v.numel() == n
    assert int(ptr[0]) == 0 and int(ptr[-1]) == n
    counts = (ptr[1:] - ptr[:-1]).to(torch.int64)
    assert int(counts.min()) >= 0
    rows = torch.repeat_interleave(torch.arange(dim, dtype=torch.int64, device="cuda"), counts)
    lin = (rows << LOG_DIM) | idx.to(torch.int64)
    del rows
    assert bool((lin[1:] > lin[:-1]).all())                              # sorted by (row, col), no coordinate twice
    assert (int(lin.sum()), int((lin * lin).sum())) == sums              # the same multiset of coordinates
    assert bool((v == f_of(lin)).all())                                  # every value stayed with its coordinate
    del lin
    # SpMV with x = 1: row sums, exact in fp32
    x = torch.ones(dim, device="cuda"); y = torch.empty(dim, device="cuda")
    B.us_spmv(ctx, g, x, y)
    ref = torch.zeros(dim, dtype=torch.float64, device="cuda").index_add_(0, row.to(torch.int64), val.to(torch.float64))
    assert float(ref.max()) < 2 ** 24
    assert bool((y.to(torch.float64) == ref).all())
    g.free()
    del row, col, val, ref, x, y, ptr, idx, v, counts
    torch.cuda.empty_cache()


def test_every_layout_and_back_at_2_to_27():
    """2^27 entries: every layout that can hold a scattered matrix of this size, converted back to CSR through the
    COO hub, gives the bytes of the direct COO -> CSR conversion (two different code paths that must agree), and the
    rank decomposition into ELL + COO keeps every entry: its two products add up to the exact row sums."""
    from paper_2403_05802_amd import binding as B
    dim, n, row, col, val, _ = generate(1 << 27)
    ctx = B.Context("cuda:0")
    P = B.us_desc_preset
    csr = B.us_convert(ctx, dim, dim, row, col, val, P(B.US_F_CSR))
    ref_ptr, ref_idx, ref_val = csr.ptr(1), csr.idx(1), csr.val()
    for name, desc in (("DCSR", P(B.US_F_DCSR)), ("CSC", P(B.US_F_CSC)), ("COO", P(B.US_F_COO)),
                       ("BCSR2", P(B.US_F_BCSR, 2, 2)), ("CSB1024", P(B.US_F_CSB, 1024, 1024)),
                       ("CISR-plus1024", P(B.US_F_CISR_PLUS, 1024)), ("ELL", P(B.US_F_ELL))):
        g = B.us_convert(ctx, dim, dim, row, col, val, desc)
        back = B.us_convert_formatted(ctx, g, P(B.US_F_CSR))
        assert torch.equal(back.ptr(1), ref_ptr) and torch.equal(back.idx(1), ref_idx), name
        assert torch.equal(back.val().view(torch.int32), ref_val.view(torch.int32)), name
        back.free(); g.free()
        torch.cuda.empty_cache()
    # scattered entries in 4x4 blocks: nearly one block per entry, 16 value slots each = 2^31 slots: reported, not built
    import pytest as _pytest
    with _pytest.raises(B.UnisparseError) as ei:
        B.us_convert(ctx, dim, dim, row, col, val, P(B.US_F_BCSR, 4, 4))
    assert ei.value.code == "US_ERR_OVERFLOW"
    x = torch.ones(dim, device="cuda"); y = torch.empty(dim, device="cuda")
    ref = torch.zeros(dim, dtype=torch.float64, device="cuda").index_add_(0, row.to(torch.int64), val.to(torch.float64))
    pred = B.make_predicate([B.expr(B.US_E_AFFINE, 1, 0)], B.US_P_RANK_LT_PERCENTILE, 9, 10)
    ga, gb = B.us_decompose(ctx, dim, dim, row, col, val, P(B.US_F_ELL), P(B.US_F_COO), pred)
    assert ga.nnz + gb.nnz == n and gb.nnz > 0
    counts = (ref_ptr[1:] - ref_ptr[:-1])
    K = ga.size(0)
    assert K == int(torch.sort(counts).values[-(-9 * dim // 10) - 1])        # nearest-rank 90th percentile of the row lengths
    assert ga.nnz == int(torch.clamp(counts, max=K).sum())
    B.us_spmv(ctx, ga, x, y); B.us_spmv(ctx, gb, x, y, accumulate=True)
    assert bool((y.to(torch.float64) == ref).all())
    ga.free(); gb.free(); csr.free()
