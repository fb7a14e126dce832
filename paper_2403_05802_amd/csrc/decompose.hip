// The decompose op (Section 6): rank-in-row splits (ELL + COO hybrids), splits by the nodes of a blocked layout
// (the #sum queries of Figure 3c and of the BELL/COO case study), and the dispatch over predicates.
#include "convert_internal.h"
#include "device.h"

namespace us {

// ------------------------------------------------------------------ decompose
// The row length of a given rank (the nearest-rank percentile) without sorting the lengths: digit by digit from
// the top, one kernel counts the values of the next digit among the rows whose length agrees with the digits
// picked so far, the next one picks the digit that holds the rank.  Every workgroup of the count leaves its 256
// counts in a row of its own and the pick adds the rows up: the lengths of a matrix crowd into a few values, and
// adds from a thousand workgroups to the same few device counters took their turns at ~20 ns each (63 us a pass
// on 2 M rows); a single kernel per pass, whose last workgroup picks, was slower too (37 us: every workgroup
// then needs a device-wide fence, which writes its L2 back).
constexpr int SEL_GRID = 256, SEL_IPT = 8, SEL_TILE = 256 * SEL_IPT;
struct SelectState { uint32_t prefix, rank, pad[2]; uint32_t hist[SEL_GRID][256]; };

__global__ void select_init_kernel(SelectState *s, uint32_t rank) { s->prefix = 0; s->rank = rank; }

__global__ __launch_bounds__(256) void select_count_kernel(const int32_t *ptr, int64_t nrows, int shift, int bits,
                                                          SelectState *s) {
  __shared__ uint32_t s_hist[256];
  s_hist[threadIdx.x] = 0;
  __syncthreads();
  const uint32_t prefix = s->prefix;   // left by the previous pick
  const int hi = shift + bits;
  const uint32_t mask = (1u << bits) - 1u;
  for (int64_t base = (int64_t)blockIdx.x * SEL_TILE; base < nrows; base += (int64_t)gridDim.x * SEL_TILE) {
    uint32_t v[SEL_IPT];
#pragma unroll
    for (int k = 0; k < SEL_IPT; ++k) {   // all loads first
      const int64_t g = base + k * 256 + threadIdx.x;
      v[k] = g < nrows ? (uint32_t)(ptr[g + 1] - ptr[g]) : 0xFFFFFFFFu;
    }
#pragma unroll
    for (int k = 0; k < SEL_IPT; ++k) {
      const int64_t g = base + k * 256 + threadIdx.x;
      if (g < nrows && (hi >= 32 ? 0u : v[k] >> hi) == prefix) atomicAdd(&s_hist[(v[k] >> shift) & mask], 1u);
    }
  }
  __syncthreads();
  s->hist[blockIdx.x][threadIdx.x] = s_hist[threadIdx.x];
}
__global__ __launch_bounds__(256) void select_pick_kernel(SelectState *s, int nrows_hist, int bits, int32_t *out) {   // out: last pass only
  __shared__ uint32_t s_wave[256 / 64 + 1];
  const uint32_t prefix = s->prefix, rank = s->rank;
  uint32_t cnt = 0;
  for (int w0 = 0; w0 < nrows_hist; w0 += 32) {   // 32 loads in flight
    uint32_t part[32];
#pragma unroll
    for (int k = 0; k < 32; ++k) part[k] = w0 + k < nrows_hist ? s->hist[w0 + k][threadIdx.x] : 0u;
#pragma unroll
    for (int k = 0; k < 32; ++k) cnt += part[k];
  }
  uint32_t total;
  const uint32_t before = block_exclusive_sum<256>(cnt, s_wave, &total);
  if (cnt > 0 && before <= rank && rank < before + cnt) {   // one thread, unless the lengths are garbage
    const uint32_t picked = (prefix << bits) | threadIdx.x;
    s->prefix = picked;
    s->rank = rank - before;
    if (out) *out = (int32_t)picked;
  }
}

// K_dev != null: the cut is still on the device (the percentile picked just before)
__global__ __launch_bounds__(256) void clipped_len_kernel(const int32_t *ptr, int64_t n, int64_t K, const int32_t *K_dev,
                                                         int32_t *out) {
  int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (K_dev) K = *K_dev;
  if (g < n) { int64_t l = ptr[g + 1] - ptr[g]; out[g] = (int32_t)(l < K ? l : K); }
}

// stable split of the sorted list by rank-in-row: rank < K -> part A, else part B.  (Equal neighbours have
// been looked for before: the two copies of a coordinate may end up in different parts.)
// ar == null: part A is not written as a list (an ELL part A is built from the rows of the sorted list itself).
constexpr int RSP_IPT = 4;
__global__ __launch_bounds__(256) void rank_split_kernel(const int32_t *major, const int32_t *minor, const float *val,
                                                        const int32_t *ptr, const int32_t *ptr_a, int64_t n,
                                                        int64_t K, int32_t *ar, int32_t *ac, float *av, int32_t *br,
                                                        int32_t *bc, float *bv) {
  // RSP_IPT entries per thread, each step for all of them before the next: the entry, then the two pointers of its
  // row, then the stores
  const int64_t base = (int64_t)blockIdx.x * (256 * RSP_IPT) + threadIdx.x;
  int32_t r[RSP_IPT], c[RSP_IPT], p0[RSP_IPT], pa[RSP_IPT];
  float v[RSP_IPT];
#pragma unroll
  for (int k = 0; k < RSP_IPT; ++k) {
    const int64_t i = base + k * 256;
    r[k] = i < n ? major[i] : 0; c[k] = i < n ? minor[i] : 0; v[k] = i < n ? val[i] : 0.f;
  }
#pragma unroll
  for (int k = 0; k < RSP_IPT; ++k) {
    const bool in = base + k * 256 < n;
    p0[k] = in ? ptr[r[k]] : 0; pa[k] = in ? ptr_a[r[k]] : 0;
  }
#pragma unroll
  for (int k = 0; k < RSP_IPT; ++k) {
    const int64_t i = base + k * 256;
    if (i >= n) continue;
    const int64_t rank = i - p0[k];
    if (rank < K) {
      if (ar) {
        const int64_t p = pa[k] + rank;
        ar[p] = r[k]; ac[p] = c[k]; av[p] = v[k];
      }
    } else {
      const int64_t p = (int64_t)(p0[k] - pa[k]) + (rank - K);
      br[p] = r[k]; bc[p] = c[k]; bv[p] = v[k];
    }
  }
}

static bool row_major_family(const Plan &p) {
  return !p.swapped && (p.pattern == P_COO || p.pattern == P_CSR || p.pattern == P_DCSR || p.pattern == P_ELL);
}

static us_status decompose_rank(Env &env, const us_coo &coo, const Plan &pa, const us_format_desc &da, const Plan &pb,
                                const us_format_desc &db, const us_predicate &pred, us_formatted **oa,
                                us_formatted **ob) {
  const int64_t n = coo.nnz, nrows = coo.nrows;
  {  // every temporary of the call in one allocation
    auto g = [](size_t count) { return Env::granule(4 * count); };
    env.reserve(sort_temp_bytes(n) + 3 * g(n) + 3 * g(nrows + 1) + g(nrows) + g(nrows / 1024 + 64) +
                Env::granule(sizeof(SelectState)) + 4 * Env::granule(sizeof(Flags)));
  }
  Flags *flags = new_flags(env);
  int32_t *major = env.temp<int32_t>(n), *minor = env.temp<int32_t>(n);
  float *val = env.temp<float>(n);
  int32_t *ptr = env.temp<int32_t>(nrows + 1), *ptr_a = env.temp<int32_t>(nrows + 1), *clip = env.temp<int32_t>(nrows + 1);
  if (!env.ok()) return env.status;
  SortOut so{};
  so.major = major; so.minor = minor; so.val = val;
  const bool checked = sort_coo(env, coo.row, coo.col, coo.val, n, rowcol_keyspec(coo, false), so, flags);
  sorted_ptr(env, major, minor, n, nrows, ptr, !checked, flags);
  Flags h{};
  int64_t K = pred.abs;
  if (pred.kind == US_P_RANK_LT_PERCENTILE) {
    // nearest-rank percentile of the row lengths over all rows: the length of rank k - 1 in ascending order
    SelectState *sel = env.temp<SelectState>(1);
    if (!env.ok()) return env.status;
    const int64_t maxlen = n < coo.ncols ? n : coo.ncols;
    int64_t k = (pred.num * nrows + pred.den - 1) / pred.den;
    if (k < 1) k = 1;
    if (k > nrows) k = nrows;
    US_LAUNCH(env, "select_init", 8.0, select_init_kernel, 1, 1, sel, (uint32_t)(k - 1));
    const int total_bits = bits_for((uint64_t)maxlen) > 0 ? bits_for((uint64_t)maxlen) : 1;
    const int npass = ceil_div(total_bits, 8);
    const int64_t grid = ceil_div<int64_t>(nrows, SEL_TILE) < SEL_GRID ? ceil_div<int64_t>(nrows, SEL_TILE) : SEL_GRID;
    for (int p = 0, left = total_bits; p < npass; ++p) {
      const int w = total_bits / npass + (p < total_bits % npass ? 1 : 0);
      left -= w;
      US_LAUNCH(env, "select_count", 4.0 * nrows, select_count_kernel, grid, 256, (const int32_t *)ptr, nrows, left, w, sel);
      US_LAUNCH(env, "select_pick", 1024.0 * grid, select_pick_kernel, 1, 256, sel, (int)grid, w,
                p == npass - 1 ? &flags->scalar[2] : (int32_t *)nullptr);
    }
  }
  // the cut K (if picked above), the size of part A and the longest row all come back in one read of the flags
  const bool by_percentile = pred.kind == US_P_RANK_LT_PERCENTILE;
  US_LAUNCH(env, "clipped_len", 8.0 * nrows, clipped_len_kernel, ceil_div<int64_t>(nrows, 256), 256,
            (const int32_t *)ptr, nrows, K, (const int32_t *)(by_percentile ? &flags->scalar[2] : nullptr), clip);
  exclusive_scan_i32(env, clip, ptr_a, nrows, &flags->scalar[1]);
  max_group_len(env, ptr, nrows, &flags->scalar[3]);
  if (!read_flags(env, flags, &h)) return env.status;
  if (flag_status(h) != US_OK) return flag_status(h);
  if (by_percentile) K = h.scalar[2];
  const int64_t longest = h.scalar[3];
  const int64_t na = h.scalar[1], nb = n - na;
  // part A as row-major ELL: its slab is built from the first min(length, K) entries of every row of the sorted
  // list (which gives the automatic width), 64 rows at a time through LDS; only part B is split off as a list.
  // Any other format of part A gets a sorted list first.
  us_formatted *ell = nullptr;
  if (pa.pattern == P_ELL && !pa.swapped) {
    const int64_t ell_width = pa.ell_width > 0 ? pa.ell_width : (longest < K ? longest : K);
    if (ell_width * nrows >= (1ll << 31)) return US_ERR_OVERFLOW;
    ell = new_ell_of_rows(env, da, nrows, coo.ncols, na, ell_width, K, minor, val, ptr, flags);
    if (!ell) return env.status;
  }
  CooLists la = ell ? CooLists() : alloc_lists(env, na), lb = alloc_lists(env, nb);
  us_status st = env.status;
  if (st == US_OK && n > 0 && (nb > 0 || !ell)) {
    US_LAUNCH(env, "rank_split", 16.0 * n + 12.0 * (ell ? nb : n), rank_split_kernel, ceil_div<int64_t>(n, 256 * RSP_IPT), 256,
              (const int32_t *)major, (const int32_t *)minor, (const float *)val, (const int32_t *)ptr,
              (const int32_t *)ptr_a, n, K, la.r, la.c, la.v, lb.r, lb.c, lb.v);
    st = env.status;
  }
  auto finish_part = [&](const Plan &p, const us_format_desc &d, CooLists &l, int64_t cnt, us_formatted **o) {
    if (row_major_family(p)) {   // the list is already in (row, col) order: no second sort
      // the same flag block goes on (its duplicate flag may have been set by the split); sizes start from zero
      fill_u32(env, (uint32_t *)&flags->scalar[0], 4, 0u);
      if (!env.ok()) return env.status;
      Plan q = p;
      // part A as ELL of automatic width: its rows hold min(length, K) entries, so the width is known here
      if (&l == &la && q.pattern == P_ELL && q.ell_width == 0) q.ell_width = longest < K ? longest : K;
      us_status s = build_from_sorted(env, q, d, coo.nrows, coo.ncols, cnt, l.r, l.c, l.v, flags, false, o, true);
      l = CooLists();  // ownership moved
      return s;
    }
    Flags hh{};
    if (!read_flags(env, flags, &hh)) return env.status;
    if (flag_status(hh) != US_OK) return flag_status(hh);
    us_coo c{coo.nrows, coo.ncols, cnt, l.r, l.c, l.v};
    return convert_with_plan(env, c, p, d, o);
  };
  if (st == US_OK && !ell) st = finish_part(pa, da, la, na, oa);
  if (st == US_OK) st = finish_part(pb, db, lb, nb, ob);   // ends with a read of the flags: covers the slab's overflow flag too
  if (ell) {
    if (st == US_OK) *oa = ell; else free_formatted(env, ell);
  }
  env.sync();
  free_lists(env, la);
  free_lists(env, lb);
  return st;
}

// ------------------------------------------------------------------ decompose by the nodes of a blocked layout
// The #sum query of the BDIA/CSR hybrid (Figure 3c) groups by (d0/b, d1-d0), the one of the BELL/COO case
// study (Section 7.2.2) by blocks (d0/bh, d1/bw).  Such groups are exactly the nodes of the BDIA / BCSR tree, so the entries are sorted by the BDIA tuple first: a group is then a run
// of the sorted list, its count is the run length, and the entries that stay (part A) are already
// in BDIA order -- no second sort for them.
__global__ __launch_bounds__(256) void node_head_kernel(const uint64_t *key, int64_t n, int ih_bits, int32_t *head,
                                                       Flags *flags) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const uint64_t cur = key[i], prev = i > 0 ? key[i - 1] : ~0ull;
  if (i > 0 && cur == prev) flags->duplicate = 1;
  head[i] = (i == 0) | ((cur >> ih_bits) != (prev >> ih_bits));
}

// start[g] = first entry of run g; the slot after the last run gets n
__global__ __launch_bounds__(256) void node_start_kernel(const int32_t *head, const int32_t *pos, int64_t n,
                                                        int32_t *start) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  if (head[i]) start[pos[i]] = (int32_t)i;
  if (i == n - 1) start[pos[i] + head[i]] = (int32_t)n;
}

__global__ __launch_bounds__(256) void node_keep_kernel(const int32_t *head, const int32_t *pos, const int32_t *start,
                                                       int64_t n, int64_t thld, int32_t *keep) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const int32_t g = pos[i] + head[i] - 1;
  keep[i] = (int64_t)(start[g + 1] - start[g]) >= thld ? 1 : 0;
}

// The same decision without the run tables when a node cannot hold more than `width` entries (a blocked
// diagonal piece holds at most b, a bh x bw block bh*bw): every entry counts its run by looking at most
// width - 1 neighbours to either side (cached reads), and equal neighbours are flagged on the way.
constexpr int NK_T = 256, NK_IPT = 4, NK_TILE = NK_T * NK_IPT, NK_HALO = 15;
__global__ __launch_bounds__(NK_T) void node_keep_window_kernel(const uint64_t *key, int64_t n, int ih_bits, int width,
                                                               int64_t thld, int32_t *keep, Flags *flags) {
  __shared__ uint64_t s_key[NK_TILE + 2 * NK_HALO];   // the tile's keys with width - 1 <= NK_HALO neighbours either side
  const int64_t i0 = (int64_t)blockIdx.x * NK_TILE - NK_HALO;
  for (int t = threadIdx.x; t < NK_TILE + 2 * NK_HALO; t += NK_T) {
    const int64_t i = i0 + t;
    s_key[t] = (i >= 0 && i < n) ? key[i] : 0ull;
  }
  __syncthreads();
  bool dup = false;
#pragma unroll
  for (int k = 0; k < NK_IPT; ++k) {
    const int t = NK_HALO + k * NK_T + threadIdx.x;
    const int64_t i = i0 + t;
    if (i >= n) continue;
    const uint64_t cur = s_key[t], node = cur >> ih_bits;
    dup |= i > 0 && s_key[t - 1] == cur;
    int count = 1;
    for (int d = 1; d < width && i - d >= 0 && (s_key[t - d] >> ih_bits) == node; ++d) ++count;
    for (int d = 1; d < width && i + d < n && (s_key[t + d] >> ih_bits) == node; ++d) ++count;
    keep[i] = count >= thld ? 1 : 0;
  }
  if (dup) flags->duplicate = 1;
}

__global__ __launch_bounds__(256) void node_split_kernel(const uint64_t *key, const float *val, const int32_t *keep,
                                                        const int32_t *pos_a, int64_t n, KeySpec ks, uint64_t *key_a,
                                                        float *val_a, CooLists la, CooLists lb) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const uint64_t k = key[i];
  const bool a = keep[i] != 0;
  const int64_t at = a ? pos_a[i] : i - pos_a[i];
  if (a && key_a) { key_a[at] = k; val_a[at] = val[i]; return; }
  const int inner = ks.ih_bits + ks.iw_bits;
  const uint64_t bk = k >> inner;
  const int32_t row = (int32_t)((bk >> ks.b_bits) * ks.bh + ((k >> ks.iw_bits) & ((1ull << ks.ih_bits) - 1)));
  const int32_t second = (int32_t)(bk & ((1ull << ks.b_bits) - 1));
  // blocked diagonal: the second component is d1 - d0 biased by nrows - 1; blocks: d1 / bw, with d1 % bw below
  const int32_t col = ks.mode == 2 ? row + second - (int32_t)(ks.a_extent - 1)
                                   : second * (int32_t)ks.bw + (int32_t)(k & ((1ull << ks.iw_bits) - 1));
  const CooLists &l = a ? la : lb;
  l.r[at] = row; l.c[at] = col; l.v[at] = val[i];
}

static us_status decompose_blocked(Env &env, const us_coo &coo, const Plan &pa, const us_format_desc &da,
                                   const Plan &pb, const us_format_desc &db, const Plan &pg, int64_t thld,
                                   us_formatted **oa, us_formatted **ob) {
  Flags *flags = new_flags(env);
  const int64_t n = coo.nnz;
  const KeySpec ks = blocked_keyspec(pg, coo.nrows, coo.ncols);
  const int inner_bits = ks.ih_bits + ks.iw_bits;
  // part A keeps the sorted order when it is stored by the very tuple the groups were cut by
  const bool direct = (pa.pattern == pg.pattern || (pa.pattern == P_BELL && pg.pattern == P_BCSR)) && pa.bh == pg.bh && pa.bw == pg.bw;
  uint64_t *skey = env.temp<uint64_t>(n);
  float *sval = env.temp<float>(n);
  int32_t *keep = env.temp<int32_t>(n), *pos_a = env.temp<int32_t>(n);
  if (!env.ok()) return env.status;
  int64_t na = 0;
  if (n > 0) {
    SortOut so{};
    so.key64 = skey; so.val = sval;
    sort_coo(env, coo.row, coo.col, coo.val, n, ks, so, flags);
    const int64_t g = ceil_div<int64_t>(n, 256);
    const int64_t width = pg.bh * pg.bw;   // the most entries a node can hold
    if (width <= 16) {
      US_LAUNCH(env, "node_keep", 12.0 * n, node_keep_window_kernel, ceil_div<int64_t>(n, NK_TILE), NK_T,
                (const uint64_t *)skey, n, inner_bits, (int)width, thld, keep, flags);
    } else {
      int32_t *head = env.temp<int32_t>(n), *pos = env.temp<int32_t>(n), *start = env.temp<int32_t>(n + 1);
      if (!env.ok()) return env.status;
      US_LAUNCH(env, "node_head", 12.0 * n, node_head_kernel, g, 256, (const uint64_t *)skey, n, inner_bits, head, flags);
      exclusive_scan_i32(env, head, pos, n, &flags->scalar[0]);
      US_LAUNCH(env, "node_start", 12.0 * n, node_start_kernel, g, 256, (const int32_t *)head, (const int32_t *)pos, n,
                start);
      US_LAUNCH(env, "node_keep", 16.0 * n, node_keep_kernel, g, 256, (const int32_t *)head, (const int32_t *)pos,
                (const int32_t *)start, n, thld, keep);
    }
    exclusive_scan_i32(env, keep, pos_a, n, &flags->scalar[1]);
    Flags h{};
    if (!read_flags(env, flags, &h)) return env.status;
    if (flag_status(h) != US_OK) return flag_status(h);
    na = h.scalar[1];
  }
  const int64_t nb = n - na;
  uint64_t *key_a = direct ? env.temp<uint64_t>(na) : nullptr;
  float *val_a = direct ? env.temp<float>(na) : nullptr;
  CooLists la = direct ? CooLists() : alloc_lists(env, na), lb = alloc_lists(env, nb);
  us_status st = env.status;
  if (st == US_OK && n > 0) {
    US_LAUNCH(env, "node_split", 20.0 * n + 12.0 * n, node_split_kernel, ceil_div<int64_t>(n, 256), 256,
              (const uint64_t *)skey, (const float *)sval, (const int32_t *)keep, (const int32_t *)pos_a, n, ks, key_a,
              val_a, la, lb);
    st = env.status;
  }
  if (st == US_OK) {
    if (direct) {
      st = emit_blocked(env, pa, da, coo.nrows, coo.ncols, ks, key_a, val_a, na, flags, oa);
    } else {
      us_coo ca{coo.nrows, coo.ncols, na, la.r, la.c, la.v};
      st = convert_with_plan(env, ca, pa, da, oa);
    }
  }
  if (st == US_OK) {
    us_coo cb{coo.nrows, coo.ncols, nb, lb.r, lb.c, lb.v};
    st = convert_with_plan(env, cb, pb, db, ob);
  }
  env.sync();
  free_lists(env, la);
  free_lists(env, lb);
  return st;
}

us_status decompose_impl(Env &env, const us_coo &coo, const us_format_desc &da, const us_format_desc &db,
                         const us_predicate &pred, us_formatted **oa, us_formatted **ob) {
  *oa = *ob = nullptr;
  us_status s = validate_coo(coo);
  if (s != US_OK) return s;
  Plan pa, pb;
  if (!match_desc(da, &pa) || !match_desc(db, &pb)) return US_ERR_UNSUPPORTED_DESC;
  if ((pa.pattern == P_ELL && pa.swapped) || (pb.pattern == P_ELL && pb.swapped)) return US_ERR_UNSUPPORTED_DESC;
  if (pred.ngroup == 2) {
    // groups that are the nodes of a blocked layout: (d0/b, d1-d0) of Figure 3c, or the blocks (d0/bh, d1/bw)
    // of the BELL/COO case study (Section 7.2.2: a threshold on the entries of each block)
    Plan pg;
    int64_t bh, bw;
    if (pred.kind != US_P_SUM_GE_ABS || !tile(pred.group[0], US_E_DIV, 0, &bh)) return US_ERR_UNSUPPORTED_DESC;
    if (aff(pred.group[1], -1, 1)) { pg.pattern = P_BDIA; pg.bh = bh; pg.bw = 1; }
    else if (tile(pred.group[1], US_E_DIV, 1, &bw)) { pg.pattern = P_BCSR; pg.bh = bh; pg.bw = bw; }
    else return US_ERR_UNSUPPORTED_DESC;
    s = decompose_blocked(env, coo, pa, da, pb, db, pg, pred.abs, oa, ob);
    if (s == US_OK && !env.ok()) s = env.status;
    if (s != US_OK) {
      if (*oa) { free_formatted(env, *oa); *oa = nullptr; }
      if (*ob) { free_formatted(env, *ob); *ob = nullptr; }
    }
    return s;
  }
  if (pred.ngroup != 1) return US_ERR_UNSUPPORTED_DESC;
  const us_expr &ge = pred.group[0];
  int gkind = aff(ge, -1, 1) ? G_DIAG : aff(ge, 1, 0) ? G_ROW : aff(ge, 0, 1) ? G_COL : -1;
  if (gkind < 0) return US_ERR_UNSUPPORTED_DESC;
  if (pred.kind == US_P_SUM_GE_ABS || pred.kind == US_P_SUM_GE_FRAC_OF_CAPACITY) {
    if (pred.kind == US_P_SUM_GE_FRAC_OF_CAPACITY && (pred.den <= 0 || pred.num < 0)) return US_ERR_SHAPE;
    s = decompose_sum(env, coo, pa, da, pb, db, pred, gkind, oa, ob);
  } else if (pred.kind == US_P_RANK_LT_ABS || pred.kind == US_P_RANK_LT_PERCENTILE) {
    if (gkind != G_ROW) return US_ERR_UNSUPPORTED_DESC;
    if (pred.kind == US_P_RANK_LT_PERCENTILE && (pred.den <= 0 || pred.num < 0 || pred.num > pred.den)) return US_ERR_SHAPE;
    if (pred.kind == US_P_RANK_LT_ABS && pred.abs < 0) return US_ERR_SHAPE;
    s = decompose_rank(env, coo, pa, da, pb, db, pred, oa, ob);
  } else {
    return US_ERR_UNSUPPORTED_DESC;
  }
  if (s == US_OK && !env.ok()) s = env.status;
  if (s != US_OK) {
    if (*oa) { free_formatted(env, *oa); *oa = nullptr; }
    if (*ob) { free_formatted(env, *ob); *ob = nullptr; }
  }
  return s;
}

}  // namespace us
