// CISR-plus (Section 7.2.4): rows reordered by their number of entries and scheduled to partitions.
#include "convert_internal.h"
#include "device.h"

namespace us {

// ------------------------------------------------------------------ CISR-plus (Section 7.2.4)
// The indirect level of its encoding is three queries over the rows: sum (entries per row), reorder (most
// entries first, equal rows by ascending index) and schedule (the paper asks only that the assignment be balanced; read
// here as dealing: the k-th row of that order goes to partition k mod P).  After the (row, col) sort these are row-level steps: the stored rows are compacted in row order,
// one stable key sort by (longest possible - length) gives the order, a second one by partition (from row order
// again, so rows stay ascending inside a partition) gives the storage order; then the entries of every row move
// as a block.
__global__ __launch_bounds__(256) void cisr_rows_kernel(const int32_t *ptr, const int32_t *pos, int64_t nrows,
                                                       int64_t cap, uint32_t longest, int32_t *row_of,
                                                       uint32_t *len_key, uint32_t *iota) {
  int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (g >= nrows) return;
  const int32_t len = ptr[g + 1] - ptr[g];
  const int64_t k = pos[g];
  if (len > 0 && k >= 0 && k < cap) {
    row_of[k] = (int32_t)g;
    len_key[k] = longest - min((uint32_t)len, longest);   // ascending key = descending length
    iota[k] = (uint32_t)k;
  }
}
__global__ __launch_bounds__(256) void cisr_deal_kernel(const uint32_t *order, int64_t nnr, uint32_t nparts,
                                                       uint32_t *part_of) {
  int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (k < nnr) { const uint32_t q = order[k]; if (q < nnr) part_of[q] = (uint32_t)(k % nparts); }
}
// ptr over the partitions (closed form of dealing), the stored rows in storage order and their lengths
__global__ __launch_bounds__(256) void cisr_place_kernel(const uint32_t *perm, const int32_t *row_of, const int32_t *ptr,
                                                        int64_t nnr, int64_t nparts, int32_t *part_ptr,
                                                        int32_t *row_idx, int32_t *len) {
  int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (p <= nparts) {
    const int64_t q = nnr / nparts, rem = nnr % nparts;
    part_ptr[p] = (int32_t)(p * q + (p < rem ? p : rem));
  }
  if (p < nnr) {
    const uint32_t k = perm[p];
    const int32_t row = k < nnr ? row_of[k] : 0;
    row_idx[p] = row;
    len[p] = ptr[row + 1] - ptr[row];
  }
}
// Entries move row by row into storage order.  A workgroup writes CM_TILE consecutive output entries: it finds
// the stored row of its first entry once, stages the row boundaries that can fall into the tile (rows hold at
// least one entry, so at most CM_TILE + 1 of them) and where each of those rows starts in the sorted list, and
// every entry then finds its row by a search in LDS.
constexpr int CM_T = 256, CM_IPT = 4, CM_TILE = CM_T * CM_IPT;
// the stored row that holds the first entry of every tile (a search of ~20 dependent loads: all tiles at once
// here, not one lane at the start of every workgroup)
__global__ __launch_bounds__(256) void cisr_tile_rows_kernel(const int32_t *ptr_new, int64_t nnr, int64_t ntiles,
                                                            int32_t *tile_row) {
  int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t < ntiles) tile_row[t] = (int32_t)parent_of(ptr_new, nnr, t * CM_TILE);
}
__global__ __launch_bounds__(CM_T) void cisr_move_kernel(const int32_t *ptr_new, const int32_t *row_idx, const int32_t *ptr,
                                                        const int32_t *minor, const float *val, const int32_t *tile_row,
                                                        int64_t nnr, int64_t n, int32_t *col_out, float *val_out) {
  __shared__ int32_t s_ptr[CM_TILE + 1], s_src[CM_TILE + 1];
  const int64_t e0 = (int64_t)blockIdx.x * CM_TILE;
  int64_t p0 = tile_row[blockIdx.x];
  p0 = p0 < 0 ? 0 : (p0 > nnr - 1 ? nnr - 1 : p0);
  const int cnt = (int)min<int64_t>(CM_TILE + 1, nnr + 1 - p0);   // boundaries p0 .. p0 + cnt - 1
  for (int i = threadIdx.x; i < cnt; i += CM_T) {
    s_ptr[i] = ptr_new[p0 + i];
    s_src[i] = p0 + i < nnr ? ptr[row_idx[p0 + i]] : 0;
  }
  __syncthreads();
  // where every entry comes from first, then all loads, then all stores: one trip to memory, not CM_IPT
  int64_t src[CM_IPT];
#pragma unroll
  for (int k = 0; k < CM_IPT; ++k) {
    const int64_t e = e0 + k * CM_T + threadIdx.x;
    src[k] = -1;
    if (e >= n) continue;
    int lo = 0, hi = cnt - 1;   // s_ptr[lo] <= e < s_ptr[hi] throughout
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (s_ptr[mid] <= e) lo = mid; else hi = mid;
    }
    const int64_t from = (int64_t)s_src[lo] + (e - s_ptr[lo]);
    src[k] = from < 0 ? 0 : (from >= n ? n - 1 : from);
  }
  int32_t c[CM_IPT];
  float v[CM_IPT];
#pragma unroll
  for (int k = 0; k < CM_IPT; ++k) {
    c[k] = src[k] >= 0 ? minor[src[k]] : 0;
    v[k] = src[k] >= 0 ? val[src[k]] : 0.f;
  }
#pragma unroll
  for (int k = 0; k < CM_IPT; ++k) {
    const int64_t e = e0 + k * CM_T + threadIdx.x;
    if (src[k] >= 0) { col_out[e] = c[k]; val_out[e] = v[k]; }
  }
}

us_status convert_cisr(Env &env, const us_coo &coo, const Plan &plan, const us_format_desc &desc, Flags *flags,
                       us_formatted **out) {
  const int64_t n = coo.nnz, nrows = coo.nrows, nparts = plan.bh;
  int32_t *major = env.temp<int32_t>(n), *minor = env.temp<int32_t>(n);
  float *val = env.temp<float>(n);
  int32_t *ptr = env.temp<int32_t>(nrows + 1), *flag = env.temp<int32_t>(nrows), *pos = env.temp<int32_t>(nrows);
  if (!env.ok()) return env.status;
  SortOut so{};
  so.major = major; so.minor = minor; so.val = val;
  const bool checked = sort_coo(env, coo.row, coo.col, coo.val, n, rowcol_keyspec(coo, false), so, flags);
  sorted_ptr(env, major, minor, n, nrows, ptr, !checked, flags);
  nonempty_flags(env, ptr, nrows, flag);
  exclusive_scan_i32(env, flag, pos, nrows, &flags->scalar[0]);
  Flags h{};
  if (!read_flags(env, flags, &h)) return env.status;
  if (flag_status(h) != US_OK) return flag_status(h);
  const int64_t nnr = h.scalar[0];   // rows that hold entries (the sum query, value ne 0)

  us_formatted *f = new us_formatted();
  f->desc = desc; f->pattern = P_CISR; f->swapped = false;
  f->nrows = nrows; f->ncols = coo.ncols; f->nnz = n; f->nmajor = nnr;
  f->nlevels = 3;
  f->level[0].size = nparts;
  f->level[1].ptr = env.owned<int32_t>(nparts + 1); f->level[1].nptr = nparts + 1;
  f->level[1].idx = env.owned<int32_t>(nnr); f->level[1].nidx = nnr;
  f->level[2].ptr = env.owned<int32_t>(nnr + 1); f->level[2].nptr = nnr + 1;
  f->level[2].idx = env.owned<int32_t>(n); f->level[2].nidx = n;
  f->val = env.owned<float>(n); f->nval = n;
  int32_t *row_of = env.temp<int32_t>(nnr), *len = env.temp<int32_t>(nnr + 1);
  uint32_t *key = env.temp<uint32_t>(nnr), *iota = env.temp<uint32_t>(nnr), *order = env.temp<uint32_t>(nnr);
  uint32_t *part_of = env.temp<uint32_t>(nnr), *perm = env.temp<uint32_t>(nnr), *key_out = env.temp<uint32_t>(nnr);
  if (!env.ok()) { free_formatted(env, f); return env.status; }
  const uint32_t longest = (uint32_t)(n < coo.ncols ? n : coo.ncols);
  US_LAUNCH(env, "cisr_rows", 12.0 * nrows + 12.0 * nnr, cisr_rows_kernel, ceil_div<int64_t>(nrows, 256), 256,
            (const int32_t *)ptr, (const int32_t *)pos, nrows, nnr, longest, row_of, key, iota);
  // reorder: rows by descending length, equal ones in ascending row order (the sort is stable)
  sort_u32_payload(env, key, iota, nnr, bits_for(longest), key_out, order, flags);
  // schedule: deal them to the partitions
  if (nnr > 0)
    US_LAUNCH(env, "cisr_deal", 8.0 * nnr, cisr_deal_kernel, ceil_div<int64_t>(nnr, 256), 256, (const uint32_t *)order,
              nnr, (uint32_t)nparts, part_of);
  // storage order = (partition, row): stable sort by partition of the rows taken in row order
  sort_u32_payload(env, part_of, iota, nnr, bits_for((uint64_t)nparts - 1) > 0 ? bits_for((uint64_t)nparts - 1) : 1,
                   key_out, perm, flags);
  const int64_t m = nnr > nparts + 1 ? nnr : nparts + 1;
  US_LAUNCH(env, "cisr_place", 16.0 * nnr + 4.0 * nparts, cisr_place_kernel, ceil_div<int64_t>(m, 256), 256,
            (const uint32_t *)perm, (const int32_t *)row_of, (const int32_t *)ptr, nnr, nparts, f->level[1].ptr,
            f->level[1].idx, len);
  exclusive_scan_i32(env, len, f->level[2].ptr, nnr, &flags->scalar[1]);
  fill_u32(env, (uint32_t *)f->level[2].ptr + nnr, 1, (uint32_t)n);
  if (n > 0) {
    const int64_t ntiles = ceil_div<int64_t>(n, CM_TILE);
    int32_t *tile_row = env.temp<int32_t>(ntiles);
    if (!env.ok()) { free_formatted(env, f); return env.status; }
    US_LAUNCH(env, "cisr_tile_rows", 4.0 * ntiles, cisr_tile_rows_kernel, ceil_div<int64_t>(ntiles, 256), 256,
              (const int32_t *)f->level[2].ptr, nnr, ntiles, tile_row);
    US_LAUNCH(env, "cisr_move", 16.0 * n, cisr_move_kernel, ntiles, CM_T, (const int32_t *)f->level[2].ptr,
              (const int32_t *)f->level[1].idx, (const int32_t *)ptr, (const int32_t *)minor, (const float *)val,
              (const int32_t *)tile_row, nnr, n, f->level[2].idx, f->val);
  }
  spmv_prepare(env, f);
  if (!read_flags(env, flags, &h)) { free_formatted(env, f); return env.status; }
  if (flag_status(h) != US_OK) { free_formatted(env, f); return flag_status(h); }
  *out = f;
  return US_OK;
}

}  // namespace us
