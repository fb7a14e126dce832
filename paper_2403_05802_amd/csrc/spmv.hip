// y (+)= A x over a formatted tensor: the SpMV of Figure 3c specialised per storage layout
// (what the two-step kernel generator of Section 5.3 would emit for each: walk the levels,
// recover (d0,d1) with the inverse index map, guard the bounds, multiply-accumulate).
#include "common.h"
#include "device.h"

#include <atomic>

namespace us {

// ------------------------------------------------------------------ compressed rows (CSR / DCSR / CSC-transposed use)
// Work is split evenly over the merged sequence {row ends} U {non-zeros}, so a 20,000-entry
// row and 20,000 one-entry rows cost the same.  Each workgroup takes MP_TILE consecutive steps of
// that sequence, stages the products in LDS, every thread walks MP_IPT steps, and partial row
// sums are stitched together with a segmented scan (fixed order: bitwise reproducible).
constexpr int MP_T = 256, MP_IPT = 8;
static_assert(MP_TILE == MP_T * MP_IPT, "tile of the merge path = threads x steps per thread");

// number of row ends consumed before step `diag`: largest r with ptr_end[r-1] <= diag - r ...
__device__ __forceinline__ int64_t merge_path_rows(const int32_t *row_end, int64_t nrows, int64_t nnz, int64_t diag) {
  int64_t lo = diag > nnz ? diag - nnz : 0, hi = diag < nrows ? diag : nrows;
  while (lo < hi) {
    int64_t mid = (lo + hi) >> 1;
    if ((int64_t)row_end[mid] <= diag - mid - 1) lo = mid + 1; else hi = mid;
  }
  return lo;
}

struct SegPair { int32_t key; float val; };

// split[t] = row ends consumed before merge step t * MP_TILE (t = 0..ntiles)
// nrows_dev != null: the row count is *nrows_dev (at most nrows) and the tile count follows from it
__global__ __launch_bounds__(256) void merge_path_split_kernel(const int32_t *ptr, int64_t nrows, int64_t nnz,
                                                              int64_t ntiles, const int32_t *nrows_dev,
                                                              int32_t *split) {
  int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (nrows_dev) {
    const int64_t r = *nrows_dev;
    nrows = r >= 0 && r < nrows ? r : nrows;
    ntiles = (nrows + nnz + MP_TILE - 1) / MP_TILE;
  }
  if (t > ntiles) return;
  int64_t d = t * MP_TILE;
  if (d > nrows + nnz) d = nrows + nnz;
  split[t] = (int32_t)merge_path_rows(ptr + 1, nrows, nnz, d);
}

template <bool INDIRECT_ROWS>
__global__ __launch_bounds__(MP_T) void csr_spmv_kernel(const int32_t *ptr, const int32_t *idx, const float *val,
                                                       const int32_t *row_ids, const int32_t *split, int64_t nrows,
                                                       int64_t nnz, const float *x, float *y, int accumulate,
                                                       int32_t *carry_row, float *carry_val) {
  __shared__ float s_prod[MP_TILE];
  __shared__ int32_t s_end[MP_TILE + 1];
  __shared__ int32_t s_wkey[MP_T / 64];
  __shared__ float s_wval[MP_T / 64];
  const int32_t *row_end = ptr + 1;
  const int64_t total = nrows + nnz;
  const int64_t diag0 = (int64_t)blockIdx.x * MP_TILE;
  const int64_t diag1 = min(diag0 + MP_TILE, total);
  const int64_t r0 = split[blockIdx.x], r1 = split[blockIdx.x + 1];
  const int64_t z0 = diag0 - r0, z1 = diag1 - r1;
  const int nr = (int)(r1 - r0), nz = (int)(z1 - z0);
  {  // all index/value loads first, then all gathers of x: two round trips instead of sixteen.
     // (Non-temporal loads of the streamed arrays were measured: 7 % faster right after a conversion, 16 %
     // slower when the product is repeated and the matrix would otherwise stay in the memory-side cache.)
    int32_t ci[MP_IPT];
    float vv[MP_IPT], xv[MP_IPT];
    int32_t re[MP_IPT];
#pragma unroll
    for (int k = 0; k < MP_IPT; ++k) {
      const int i = k * MP_T + threadIdx.x;
      ci[k] = i < nz ? idx[z0 + i] : 0;
      vv[k] = i < nz ? val[z0 + i] : 0.f;
      re[k] = i < nr ? row_end[r0 + i] : 0;
    }
#pragma unroll
    for (int k = 0; k < MP_IPT; ++k) xv[k] = (k * MP_T + (int)threadIdx.x) < nz ? x[ci[k]] : 0.f;
#pragma unroll
    for (int k = 0; k < MP_IPT; ++k) {
      const int i = k * MP_T + threadIdx.x;
      if (i < nz) s_prod[i] = vv[k] * xv[k];
      if (i < nr) s_end[i] = (int32_t)(re[k] - z0);
    }
  }
  __syncthreads();

  // this thread's slice of the tile's merge sequence
  const int steps = (int)(diag1 - diag0);
  int d = min((int)threadIdx.x * MP_IPT, steps);
  int lo = d > nz ? d - nz : 0, hi = d < nr ? d : nr;
  while (lo < hi) {
    int mid = (lo + hi) >> 1;
    if (s_end[mid] <= d - mid - 1) lo = mid + 1; else hi = mid;
  }
  int ri = lo, zi = d - lo;
  const int dend = min(d + MP_IPT, steps);
  float sum = 0.f, first_sum = 0.f;
  int first_row = -1;  // first row that ends inside this thread's slice
  for (int s = d; s < dend; ++s) {
    bool take_nz = zi < nz && (ri >= nr || zi < s_end[ri]);
    if (take_nz) {
      sum += s_prod[zi++];
    } else {
      if (first_row < 0) { first_row = ri; first_sum = sum; }
      else {
        int64_t row = r0 + ri;
        int64_t out = INDIRECT_ROWS ? row_ids[row] : row;
        y[out] = (accumulate ? y[out] : 0.f) + sum;
      }
      sum = 0.f;
      ++ri;
    }
  }
  // Inclusive segmented scan over the workgroup of (row the thread stopped in, unfinished sum).
  // Rows only grow from thread to thread, so equal keys are contiguous.
  SegPair p{ri, sum};
  const int lane = lane_id(), w = wave_id();
#pragma unroll
  for (int dd = 1; dd < 64; dd <<= 1) {
    int32_t k = __shfl_up(p.key, dd);
    float v = __shfl_up(p.val, dd);
    if (lane >= dd && k == p.key) p.val += v;
  }
  if (lane == 63) { s_wkey[w] = p.key; s_wval[w] = p.val; }
  __syncthreads();
  // state of the scan at the end of the previous wave (fixed left-to-right order)
  int32_t head_key = -2;
  float wave_carry = 0.f;
  for (int ww = 0; ww < w; ++ww) {
    if (s_wkey[ww] == head_key) wave_carry += s_wval[ww];
    else { head_key = s_wkey[ww]; wave_carry = s_wval[ww]; }
  }
  const float incl = p.val + (p.key == head_key ? wave_carry : 0.f);
  // what the previous thread hands over: it stopped in the row this thread starts in
  int32_t prev_key = __shfl_up(p.key, 1);
  float prev_val = __shfl_up(incl, 1);
  if (lane == 0) { prev_key = head_key; prev_val = wave_carry; }
  if (first_row >= 0) {
    float inherit = (prev_key == first_row) ? prev_val : 0.f;
    int64_t row = r0 + first_row;
    int64_t out = INDIRECT_ROWS ? row_ids[row] : row;
    y[out] = (accumulate ? y[out] : 0.f) + (first_sum + inherit);
  }
  if (threadIdx.x == MP_T - 1) {
    carry_row[blockIdx.x] = (int32_t)min(r0 + (int64_t)p.key, nrows);
    carry_val[blockIdx.x] = incl;
  }
}

// rows that span several workgroups: add the unfinished sums of the earlier workgroups
template <bool INDIRECT_ROWS>
__global__ __launch_bounds__(256) void csr_spmv_fixup_kernel(const int32_t *carry_row, const float *carry_val,
                                                            int64_t nblocks, int64_t nrows,
                                                            const int32_t *row_ids, float *y) {
  int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (b >= nblocks) return;
  int32_t row = carry_row[b];
  if (row >= nrows) return;
  if (b > 0 && carry_row[b - 1] == row) return;  // not the first workgroup of this run
  float s = 0.f;
  for (int64_t j = b; j < nblocks && carry_row[j] == row; ++j) s += carry_val[j];
  int64_t out = INDIRECT_ROWS ? row_ids[row] : row;
  y[out] += s;
}

static void spmv_compressed(Env &env, const us_formatted &A, const int32_t *ptr, const int32_t *idx, const float *val,
                            const int32_t *row_ids, int64_t nrows_stored, int64_t nnz, const float *x, float *y,
                            bool accumulate) {
  const int64_t total = nrows_stored + nnz;
  if (total == 0) return;
  const int64_t nb = ceil_div<int64_t>(total, MP_TILE);
  if (!A.mp_split || A.mp_tiles != nb) { env.fail(US_ERR_FORMAT_MISMATCH); return; }
  const size_t half = ((size_t)nb * 4 + 255) / 256 * 256;
  char *ws = (char *)ensure_workspace(env, A, 2 * half);
  if (!env.ok()) return;
  int32_t *carry_row = (int32_t *)ws;
  float *carry_val = (float *)(ws + half);
  // (x counted once, as its length: what the gathers re-read is traffic, not algorithmic bytes)
  const double bytes = 8.0 * nnz + 4.0 * (nrows_stored + 1) + 4.0 * (A.swapped ? A.nrows : A.ncols) + 4.0 * nrows_stored;
  if (row_ids) {
    US_LAUNCH(env, "spmv_csr", bytes, (csr_spmv_kernel<true>), nb, MP_T, ptr, idx, val, row_ids,
              (const int32_t *)A.mp_split, nrows_stored, nnz,
              x, y, accumulate ? 1 : 0, carry_row, carry_val);
    US_LAUNCH(env, "spmv_csr_fixup", 8.0 * nb, (csr_spmv_fixup_kernel<true>), ceil_div<int64_t>(nb, 256), 256,
              (const int32_t *)carry_row, (const float *)carry_val, nb, nrows_stored, row_ids, y);
  } else {
    US_LAUNCH(env, "spmv_csr", bytes, (csr_spmv_kernel<false>), nb, MP_T, ptr, idx, val, row_ids,
              (const int32_t *)A.mp_split, nrows_stored, nnz,
              x, y, accumulate ? 1 : 0, carry_row, carry_val);
    US_LAUNCH(env, "spmv_csr_fixup", 8.0 * nb, (csr_spmv_fixup_kernel<false>), ceil_div<int64_t>(nb, 256), 256,
              (const int32_t *)carry_row, (const float *)carry_val, nb, nrows_stored, row_ids, y);
  }
}

// ------------------------------------------------------------------ row-major COO: y[row] += sum of val * x[col] over the row's run
// The list is sorted by (row, col), so a row is a run of consecutive entries.  A workgroup takes COO_TILE consecutive
// entries: coalesced loads, products into LDS, then every thread walks COO_IPT consecutive entries and closes the
// runs that end inside its slice; the run still open at the end of a slice goes through the same segmented scan as
// the merge-path kernel above, and a run that a tile boundary cuts leaves its partial sum in the tile's carry slot
// for the fix-up kernel (fixed order everywhere: two calls give the same bits).  y must hold what the sums are
// added to (zeros for a plain product): rows without entries are not visited.
constexpr int COO_T = 256, COO_IPT = 8, COO_TILE = COO_T * COO_IPT;

__global__ __launch_bounds__(COO_T) void coo_spmv_kernel(const int32_t *row, const int32_t *col, const float *val,
                                                        int64_t nnz, int64_t nrows, const float *x, float *y,
                                                        int32_t *carry_row, float *carry_val) {
  __shared__ float s_prod[COO_TILE];
  __shared__ int32_t s_row[COO_TILE + 1];
  __shared__ int32_t s_wkey[COO_T / 64];
  __shared__ float s_wval[COO_T / 64];
  const int64_t base = (int64_t)blockIdx.x * COO_TILE;
  const int cnt = (int)min((int64_t)COO_TILE, nnz - base);
  {
    int32_t ri[COO_IPT], ci[COO_IPT];
    float vv[COO_IPT], xv[COO_IPT];
#pragma unroll
    for (int k = 0; k < COO_IPT; ++k) {   // all loads of the lists first, then all gathers of x
      const int i = k * COO_T + threadIdx.x;
      ri[k] = i < cnt ? row[base + i] : -1;
      ci[k] = i < cnt ? col[base + i] : 0;
      vv[k] = i < cnt ? val[base + i] : 0.f;
    }
#pragma unroll
    for (int k = 0; k < COO_IPT; ++k) xv[k] = (k * COO_T + (int)threadIdx.x) < cnt ? x[ci[k]] : 0.f;
#pragma unroll
    for (int k = 0; k < COO_IPT; ++k) {
      const int i = k * COO_T + threadIdx.x;
      s_prod[i] = vv[k] * xv[k];
      s_row[i] = ri[k];
    }
    // the row of the entry behind the tile (-1: none), which tells whether the tile's last run goes on
    if (threadIdx.x == 0) s_row[COO_TILE] = base + COO_TILE < nnz ? row[base + COO_TILE] : -1;
  }
  __syncthreads();

  const int d = (int)threadIdx.x * COO_IPT;
  // runs that end inside this thread's slice: the first one may have begun in an earlier thread (it takes what the
  // scan hands over), the others lie wholly inside the slice and are added to y at once
  int32_t first_row = -1, open_row = -3;   // open_row: the row whose run goes on behind the slice, or none
  float sum = 0.f, first_sum = 0.f;
  bool seen_end = false;
#pragma unroll
  for (int k = 0; k < COO_IPT; ++k) {
    const int i = d + k;
    if (i < cnt) {
      const int32_t r = s_row[i];
      sum += s_prod[i];
      const int32_t next = s_row[i + 1 < cnt ? i + 1 : COO_TILE];   // behind the last tile: -1
      if (next != r) {   // the run of row r ends with entry i
        if (!seen_end) { first_row = r; first_sum = sum; seen_end = true; }
        else y[r] += sum;
        sum = 0.f;
        open_row = -3;
      } else {
        open_row = r;
      }
    }
  }
  SegPair p{open_row, sum};
  const int lane = lane_id(), w = wave_id();
#pragma unroll
  for (int dd = 1; dd < 64; dd <<= 1) {
    int32_t k = __shfl_up(p.key, dd);
    float v = __shfl_up(p.val, dd);
    if (lane >= dd && k == p.key) p.val += v;
  }
  if (lane == 63) { s_wkey[w] = p.key; s_wval[w] = p.val; }
  __syncthreads();
  int32_t head_key = -2;
  float wave_carry = 0.f;
  for (int ww = 0; ww < w; ++ww) {
    if (s_wkey[ww] == head_key) wave_carry += s_wval[ww];
    else { head_key = s_wkey[ww]; wave_carry = s_wval[ww]; }
  }
  const float incl = p.val + (p.key == head_key ? wave_carry : 0.f);
  int32_t prev_key = __shfl_up(p.key, 1);
  float prev_val = __shfl_up(incl, 1);
  if (lane == 0) { prev_key = head_key; prev_val = wave_carry; }
  if (first_row >= 0) y[first_row] += first_sum + (prev_key == first_row ? prev_val : 0.f);
  if (threadIdx.x == COO_T - 1) {   // a run still open here goes on in the next tile: its sum so far is the tile's carry
    carry_row[blockIdx.x] = p.key >= 0 ? p.key : (int32_t)nrows;
    carry_val[blockIdx.x] = p.key >= 0 ? incl : 0.f;
  }
}

// ------------------------------------------------------------------ DIA: y[i] (+)= sum_k val[k*nrows+i] * x[i+off_k]
// (the DIA variant keeps the slab indexed by column: val[k*ncols + j], j = i + off_k)
__global__ __launch_bounds__(256) void dia_spmv_kernel(const int32_t *off, const float *val, int64_t ndiag,
                                                      int64_t nrows, int64_t ncols, int by_col, const float *x,
                                                      float *y, int accumulate) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= nrows) return;
  float s = accumulate ? y[i] : 0.f;
  const int64_t L = by_col ? ncols : nrows;
  for (int64_t k = 0; k < ndiag; ++k) {
    int64_t j = i + off[k];
    if (j >= 0 && j < ncols) s += val[k * L + (by_col ? j : i)] * x[j];
  }
  y[i] = s;
}

// Row-indexed slab, nrows a multiple of 4: four rows per thread, the slab read as 16-byte vectors (the summation
// order per row is the same as above: diagonals in ascending order of offset)
__global__ __launch_bounds__(256) void dia_spmv4_kernel(const int32_t *off, const float *val, int64_t ndiag, int64_t nrows,
                                                       int64_t ncols, const float *x, float *y, int accumulate) {
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= nrows) return;
  float4 s = accumulate ? *reinterpret_cast<const float4 *>(y + i) : make_float4(0.f, 0.f, 0.f, 0.f);
  for (int64_t k = 0; k < ndiag; ++k) {
    const int64_t j = i + off[k];
    if (j + 3 < 0 || j >= ncols) continue;
    const float4 v = *reinterpret_cast<const float4 *>(val + k * nrows + i);
    if (j >= 0 && j + 3 < ncols) {
      s.x += v.x * x[j]; s.y += v.y * x[j + 1]; s.z += v.z * x[j + 2]; s.w += v.w * x[j + 3];
    } else {
      if (j >= 0 && j < ncols) s.x += v.x * x[j];
      if (j + 1 >= 0 && j + 1 < ncols) s.y += v.y * x[j + 1];
      if (j + 2 >= 0 && j + 2 < ncols) s.z += v.z * x[j + 2];
      if (j + 3 >= 0 && j + 3 < ncols) s.w += v.w * x[j + 3];
    }
  }
  *reinterpret_cast<float4 *>(y + i) = s;
}

// column-major compressed layouts (CSC / DCSC): scatter form, one thread per stored column
__global__ __launch_bounds__(256) void csc_spmv_atomic_kernel(const int32_t *ptr, const int32_t *idx, const float *val,
                                                             const int32_t *col_ids, int64_t ncols_stored,
                                                             const float *x, float *y) {
  int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (j >= ncols_stored) return;
  const float xj = x[col_ids ? col_ids[j] : j];
  for (int e = ptr[j]; e < ptr[j + 1]; ++e) atomicAdd(&y[idx[e]], val[e] * xj);
}

// generic scatter form used by the layouts whose leaves are not grouped by output row
// (COO, CSC/DCSC, DIA variant, ELL): y[d0] += val * x[d1] with float atomics.
__global__ __launch_bounds__(256) void coo_spmv_atomic_kernel(const int32_t *r, const int32_t *c, const float *val,
                                                             int64_t n, const float *x, float *y) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) atomicAdd(&y[r[i]], val[i] * x[c[i]]);
}

__global__ __launch_bounds__(256) void ell_spmv_kernel(const int32_t *ecol, const float *ev, int64_t K, int64_t nrows,
                                                      const float *x, float *y, int accumulate) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= nrows) return;
  float s = accumulate ? y[i] : 0.f;
  for (int64_t k = 0; k < K; ++k) {
    int32_t c = ecol[k * nrows + i];
    if (c >= 0) s += ev[k * nrows + i] * x[c];
  }
  y[i] = s;
}

// BCSR: one wavefront per block row, lanes over the entries of the blocks
__global__ __launch_bounds__(256) void bcsr_spmv_kernel(const int32_t *ptr, const int32_t *idx, const float *val,
                                                       int64_t nbr, int bh, int bw, int64_t nrows, int64_t ncols,
                                                       const float *x, float *y, int accumulate) {
  int64_t br = (int64_t)blockIdx.x * 4 + wave_id();
  if (br >= nbr) return;
  const int bsz = bh * bw, lane = lane_id();
  for (int r = 0; r < bh; ++r) {
    float s = 0.f;
    for (int64_t e = (int64_t)ptr[br] * bw + lane; e < (int64_t)ptr[br + 1] * bw; e += 64) {
      int64_t blk = e / bw; int c = (int)(e - blk * bw);
      int64_t col = (int64_t)idx[blk] * bw + c;
      if (col < ncols) s += val[blk * bsz + r * bw + c] * x[col];
    }
    s = wave_sum(s);
    int64_t row = br * bh + r;
    if (lane == 0 && row < nrows) y[row] = (accumulate ? y[row] : 0.f) + s;
  }
}

// BDIA (Figure 3c, Figure 9): node n of block row br holds the bh entries (br*bh + ri, br*bh + ri + off_n);
// one thread per row walks the nodes of its block row, so x is read along the diagonal (unit stride
// across threads) and val in runs of bh.
__global__ __launch_bounds__(256) void bdia_spmv_kernel(const int32_t *ptr, const int32_t *off, const float *val,
                                                       int bh, int64_t nrows, int64_t ncols, const float *x, float *y,
                                                       int accumulate) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= nrows) return;
  const int64_t br = i / bh;
  const int ri = (int)(i - br * bh);
  float s = accumulate ? y[i] : 0.f;
  for (int64_t n = ptr[br]; n < ptr[br + 1]; ++n) {
    const int64_t j = i + off[n];
    if (j >= 0 && j < ncols) s += val[n * bh + ri] * x[j];
  }
  y[i] = s;
}

// Blocked ELL: a thread per row walks the slots of its block row (they fill from the front); the values of a slot are
// contiguous over (block row, row in block, column in block), so neighbouring threads read neighbouring runs of bw.
__global__ __launch_bounds__(256) void bell_spmv_kernel(const int32_t *ecol, const float *val, int64_t K, int64_t nbr,
                                                       int bh, int bw, int64_t nrows, int64_t ncols, const float *x,
                                                       float *y, int accumulate) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= nrows) return;
  const int64_t br = i / bh;
  const int ri = (int)(i - br * bh);
  float s = accumulate ? y[i] : 0.f;
  for (int64_t k = 0; k < K; ++k) {
    const int64_t bc = ecol[k * nbr + br];
    if (bc < 0) break;
    const float *v = val + ((k * nbr + br) * bh + ri) * bw;
    for (int c = 0; c < bw; ++c) {
      const int64_t j = bc * bw + c;
      if (j < ncols) s += v[c] * x[j];
    }
  }
  y[i] = s;
}

// CSB: a lane per entry, 64 consecutive entries at a time, a wavefront per chunk of consecutive entries.  The blocks
// of the chunk's first and last entries are found by bisection over all blocks (the same search for every lane), a
// lane's own block between those two.  Entries of a block are sorted by row, so the lanes of one row are neighbours: their products are summed by a
// segmented scan and the last lane of every run adds the sum to y.  Other blocks of the block row add to the same
// rows, so that add is an fp32 atomic (not bit-reproducible); one per run instead of one per entry.
constexpr int CSB_CHUNK = 512;   // entries per wavefront: the two bisections over all blocks are paid once per chunk
__global__ __launch_bounds__(256) void csb_spmv_kernel(const int32_t *ptr, const int32_t *in_row, const int32_t *in_col,
                                                      const float *val, int64_t n, int64_t nblocks, int64_t nbc, int64_t bh,
                                                      int64_t bw, const float *x, float *y) {
  const int lane = lane_id();
  const int64_t e0 = ((int64_t)blockIdx.x * 4 + wave_id()) * CSB_CHUNK;
  if (e0 >= n) return;
  const int64_t e1 = min(e0 + CSB_CHUNK, n);
  const int64_t blk_first = parent_of(ptr, nblocks, e0), blk_last = parent_of(ptr, nblocks, e1 - 1);
  for (int64_t base = e0; base < e1; base += 64) {
    const int64_t e = base + lane;
    const bool live = e < e1;
    int64_t lo = blk_first, hi = blk_last;
    if (live) {
      while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)ptr[mid + 1] <= e) lo = mid + 1; else hi = mid;
      }
    }
    const int64_t row = live ? (lo / nbc) * bh + in_row[e] : -1;
    float p = live ? val[e] * x[(lo % nbc) * bw + in_col[e]] : 0.f;
    // runs of one row: head = first lane of a run; a lane's run = number of heads up to it
    const int64_t prev = __shfl_up(row, 1);
    const uint64_t heads = __ballot(lane == 0 || prev != row);
    const int run = __popcll(heads & (lanes_below() | (1ull << lane)));
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const float t = __shfl_up(p, d);
      const int tr = __shfl_up(run, d);
      if (lane >= d && tr == run) p += t;
    }
    const bool tail = lane == 63 || ((heads >> (lane + 1)) & 1ull);
    if (live && tail) atomicAdd(&y[row], p);
  }
}

static void spmv_coo_rows(Env &env, const us_formatted &A, const float *x, float *y, bool accumulate) {
  const int64_t nb = ceil_div<int64_t>(A.nnz, COO_TILE);
  const size_t half = Env::granule((size_t)(nb > 0 ? nb : 1) * 4);
  char *ws = (char *)ensure_workspace(env, A, 2 * half);   // (asked for before anything is enqueued)
  if (!env.ok()) return;
  if (!accumulate) fill_u32(env, (uint32_t *)y, A.nrows, 0u);
  if (A.nnz == 0) return;
  int32_t *carry_row = (int32_t *)ws;
  float *carry_val = (float *)(ws + half);
  US_LAUNCH(env, "spmv_coo", 12.0 * A.nnz + 4.0 * A.ncols + 4.0 * A.nrows, coo_spmv_kernel, nb, COO_T,
            (const int32_t *)A.level[0].idx, (const int32_t *)A.level[1].idx, (const float *)A.val, A.nnz, A.nrows, x, y,
            carry_row, carry_val);
  US_LAUNCH(env, "spmv_coo_fixup", 8.0 * nb, (csr_spmv_fixup_kernel<false>), ceil_div<int64_t>(nb, 256), 256,
            (const int32_t *)carry_row, (const float *)carry_val, nb, A.nrows, (const int32_t *)nullptr, y);
}

int64_t spmv_tiles(int64_t nmajor, int64_t nnz) { return ceil_div<int64_t>(nmajor + nnz, MP_TILE); }

void spmv_prepare(Env &env, us_formatted *f, const int32_t *nmajor_dev, int64_t nmajor_cap) {
  // (column-major CSC / DCSC get the tile starts too: their products scatter and do not use them, but the way
  // back to COO does)
  if (f->pattern != P_CSR && f->pattern != P_DCSR && f->pattern != P_CISR) return;
  const int64_t nmajor = nmajor_dev ? nmajor_cap : f->nmajor;
  const int64_t total = nmajor + f->nnz;
  if (total == 0) return;
  const int64_t nb = spmv_tiles(nmajor, f->nnz);
  f->mp_split = env.owned<int32_t>(nb + 1);
  f->mp_tiles = nb;
  if (!env.ok()) return;
  US_LAUNCH(env, "spmv_split", 4.0 * (nb + 1), merge_path_split_kernel, ceil_div<int64_t>(nb + 1, 256), 256,
            stored_rows(*f).ptr, nmajor, f->nnz, nb, nmajor_dev, f->mp_split);
}

us_status spmv_impl(Env &env, const us_formatted &A, const float *x, float *y, bool accumulate) {
  switch (A.pattern) {
    case P_CSR:
    case P_DCSR:
    case P_CISR: {
      const StoredRows sr = stored_rows(A);
      if (A.swapped) {
        if (!accumulate) fill_u32(env, (uint32_t *)y, A.nrows, 0u);
        if (A.nmajor > 0)
          US_LAUNCH(env, "spmv_csc", 16.0 * A.nnz, csc_spmv_atomic_kernel, ceil_div<int64_t>(A.nmajor, 256), 256,
                    sr.ptr, sr.idx, (const float *)A.val, sr.row_ids, A.nmajor, x, y);
        return env.status;
      }
      if (sr.row_ids) {   // a list of stored rows: the others are zero (unless every row is stored)
        const bool every_row = A.nmajor == A.nrows;
        if (!accumulate && !every_row) fill_u32(env, (uint32_t *)y, A.nrows, 0u);
        spmv_compressed(env, A, sr.ptr, sr.idx, A.val, sr.row_ids, A.nmajor, A.nnz, x, y, accumulate || !every_row);
        return env.status;
      }
      spmv_compressed(env, A, sr.ptr, sr.idx, A.val, nullptr, A.nrows, A.nnz, x, y, accumulate);
      return env.status;
    }
    case P_DIA:
      if (!A.swapped && A.nrows % 4 == 0 && (((uintptr_t)A.val | (uintptr_t)y) & 15) == 0)
        US_LAUNCH(env, "spmv_dia", 4.0 * A.nval + 8.0 * A.nrows + 4.0 * A.ncols, dia_spmv4_kernel,
                  ceil_div<int64_t>(A.nrows / 4, 256), 256, (const int32_t *)A.level[0].idx, (const float *)A.val,
                  A.nmajor, A.nrows, A.ncols, x, y, accumulate ? 1 : 0);
      else
        US_LAUNCH(env, "spmv_dia", 4.0 * A.nval + 8.0 * A.nrows + 4.0 * A.ncols, dia_spmv_kernel,
                  ceil_div<int64_t>(A.nrows, 256), 256, (const int32_t *)A.level[0].idx, (const float *)A.val,
                  A.nmajor, A.nrows, A.ncols, A.swapped ? 1 : 0, x, y, accumulate ? 1 : 0);
      return env.status;
    case P_ELL:
      US_LAUNCH(env, "spmv_ell", 8.0 * A.nval + 8.0 * A.nrows, ell_spmv_kernel, ceil_div<int64_t>(A.nrows, 256), 256,
                (const int32_t *)A.level[2].idx, (const float *)A.val, A.nmajor, A.nrows, x, y, accumulate ? 1 : 0);
      return env.status;
    case P_BCSR:
      US_LAUNCH(env, "spmv_bcsr", 4.0 * A.nval + 4.0 * A.nblk + 8.0 * A.nrows, bcsr_spmv_kernel,
                ceil_div<int64_t>(A.nmajor, 4), 256, (const int32_t *)A.level[1].ptr, (const int32_t *)A.level[1].idx,
                (const float *)A.val, A.nmajor, (int)A.bh, (int)A.bw, A.nrows, A.ncols, x, y, accumulate ? 1 : 0);
      return env.status;
    case P_BELL:
      US_LAUNCH(env, "spmv_bell", 4.0 * A.nval + 4.0 * A.level[2].nidx + 8.0 * A.nrows + 4.0 * A.ncols, bell_spmv_kernel,
                ceil_div<int64_t>(A.nrows, 256), 256, (const int32_t *)A.level[2].idx, (const float *)A.val, A.nmajor, A.nblk,
                (int)A.bh, (int)A.bw, A.nrows, A.ncols, x, y, accumulate ? 1 : 0);
      return env.status;
    case P_CSB:
      if (!accumulate) fill_u32(env, (uint32_t *)y, A.nrows, 0u);
      if (A.nnz > 0)
        US_LAUNCH(env, "spmv_csb_atomic", 20.0 * A.nnz, csb_spmv_kernel, ceil_div<int64_t>(A.nnz, 4 * CSB_CHUNK), 256,
                  (const int32_t *)A.level[2].ptr, (const int32_t *)A.level[2].idx, (const int32_t *)A.level[3].idx,
                  (const float *)A.val, A.nnz, A.nmajor, A.level[1].size, A.bh, A.bw, x, y);
      return env.status;
    case P_BDIA:
      US_LAUNCH(env, "spmv_bdia", 4.0 * A.nval + 4.0 * A.nblk + 8.0 * A.nrows + 4.0 * A.ncols, bdia_spmv_kernel,
                ceil_div<int64_t>(A.nrows, 256), 256, (const int32_t *)A.level[1].ptr, (const int32_t *)A.level[1].idx,
                (const float *)A.val, (int)A.bh, A.nrows, A.ncols, x, y, accumulate ? 1 : 0);
      return env.status;
    case P_COO:
      // row-major COO: runs of equal rows summed in a fixed order; column-major COO scatters with float atomics
      if (!A.swapped) { spmv_coo_rows(env, A, x, y, accumulate); return env.status; }
      if (!accumulate) fill_u32(env, (uint32_t *)y, A.nrows, 0u);
      if (A.nnz > 0)
        US_LAUNCH(env, "spmv_coo_atomic", 16.0 * A.nnz, coo_spmv_atomic_kernel, ceil_div<int64_t>(A.nnz, 256), 256,
                  (const int32_t *)A.level[1].idx, (const int32_t *)A.level[0].idx, (const float *)A.val, A.nnz, x, y);
      return env.status;
    default: break;
  }
  return US_ERR_FORMAT_MISMATCH;
}

// ------------------------------------------------------------------ the product for callers that cannot allocate
// The partial-sum scratch of the kernels above comes from this array instead of the tensor's own (allocated) one.
// Every GPU holds its own copy of the array at its own address; the name below is only a handle for
// hipGetSymbolAddress, which is asked once per device (with that device current), and the kernels get the
// address it returns as an ordinary argument.
static __device__ __align__(256) unsigned char scratch[US_NOALLOC_SCRATCH_BYTES];
constexpr int NOALLOC_MAX_DEVICES = 64;
static std::atomic<void *> g_scratch_ptr[NOALLOC_MAX_DEVICES];

static void *scratch_of_current_device(Env &env) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= NOALLOC_MAX_DEVICES) { env.fail(US_ERR_HIP); return nullptr; }
  void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p) return p;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { env.fail(US_ERR_HIP); return nullptr; }
  g_scratch_ptr[dev].store(p, std::memory_order_release);   // (two first calls at once store the same address)
  return p;
}

us_status spmv_noalloc_impl(Env &env, const us_formatted &A, const float *x, float *y, bool accumulate) {
  env.prof = nullptr;   // timing a launch creates events, which allocates
  env.fixed_ws = (char *)scratch_of_current_device(env);
  env.fixed_ws_bytes = US_NOALLOC_SCRATCH_BYTES;
  if (!env.ok()) return env.status;
  // Nothing of the array has to start at zero: the kernels write every carry slot they later read (one pair per
  // tile or chunk of THIS call), so what an earlier, larger call left behind is never looked at.
  // what the product will ask ensure_workspace for, checked before anything (a clearing of y, say) is enqueued
  size_t need = 0;
  if ((A.pattern == P_CSR || A.pattern == P_DCSR || A.pattern == P_CISR) && !A.swapped)
    need = 2 * Env::granule(4 * (size_t)spmv_tiles(A.nmajor, A.nnz));
  else if (A.pattern == P_COO && !A.swapped)
    need = 2 * Env::granule(4 * (size_t)ceil_div<int64_t>(A.nnz > 0 ? A.nnz : 1, COO_TILE));
  if (need > US_NOALLOC_SCRATCH_BYTES) return US_ERR_SCRATCH_LIMIT;
  return spmv_impl(env, A, x, y, accumulate);
}

}  // namespace us
