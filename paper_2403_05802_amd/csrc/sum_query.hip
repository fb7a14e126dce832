// The sum query (Section 4.1.2) over diagonals, rows or columns as a histogram, what it selects, the DIA layout
// (Devectorize/Fill/Vectorize: entries scattered into a pre-filled slab, no sort), and the decomposition
// driven by that query (Section 6, the decompose op).
#include "convert_internal.h"
#include "device.h"

namespace us {

// ------------------------------------------------------------------ Sum query (group histogram) and DIA
// Groups supported by the groupBy map of the sum query: diagonals (d1-d0), rows (d0), columns (d1).

__device__ __forceinline__ uint32_t group_bin(int gkind, uint32_t r, uint32_t c, uint32_t nrows) {
  return gkind == G_DIAG ? c - r + (nrows - 1) : (gkind == G_ROW ? r : c);
}

// One counter per group.  A matrix whose entries sit on a handful of diagonals would send
// almost every update to the same few counters, and same-address HBM atomics cost ~20 ns apiece
// on this part, so updates are combined in a small LDS hash table first (LDS takes 64 lanes
// hitting one slot in about as many cycles; electing one lane per bin with ballots beforehand was
// slower).  A workgroup walks several tiles; after each it flushes and frees the slots that stayed
// cold and keeps the hot ones, so a hot counter gets one HBM atomic per workgroup (at most
// ONE_COUNTER_GRID of them), not one per tile.  Freeing a slot may cut a probe chain; the bin then
// simply takes a second slot, and counts add up all the same.
constexpr int GH_T = 256, GH_IPT = 16, GH_TILE = GH_T * GH_IPT, GH_SLOTS = 1024, GH_PROBES = 8;
constexpr uint32_t GH_HOT = 64;

__global__ __launch_bounds__(GH_T) void group_hist_kernel(const int32_t *row, const int32_t *col, int64_t n,
                                                         int gkind, uint32_t nrows, uint32_t ncols, uint32_t *count,
                                                         Flags *flags) {
  __shared__ uint32_t s_key[GH_SLOTS];
  __shared__ uint32_t s_cnt[GH_SLOTS];
  for (int i = threadIdx.x; i < GH_SLOTS; i += GH_T) { s_key[i] = 0xFFFFFFFFu; s_cnt[i] = 0; }
  __syncthreads();
  bool bad = false;
  for (int64_t base = (int64_t)blockIdx.x * GH_TILE; base < n; base += (int64_t)gridDim.x * GH_TILE) {
    uint32_t bin[GH_IPT];
#pragma unroll
    for (int k = 0; k < GH_IPT; ++k) {
      int64_t i = base + k * GH_T + threadIdx.x;
      bin[k] = 0xFFFFFFFFu;
      if (i < n) {
        uint32_t r = (uint32_t)row[i], c = (uint32_t)col[i];
        if (r >= nrows || c >= ncols) bad = true;
        else bin[k] = group_bin(gkind, r, c, nrows);
      }
    }
#pragma unroll 1
    for (int k = 0; k < GH_IPT; ++k) {
      const uint32_t b = bin[k];
      if (b == 0xFFFFFFFFu) continue;
      uint32_t h = (b * 2654435761u) >> 22;
      bool done = false;
      for (int probe = 0; probe < GH_PROBES && !done; ++probe) {
        uint32_t old = s_key[h];   // a bin that is already in the table (the hot ones, soon) needs no CAS
        if (old == 0xFFFFFFFFu) old = atomicCAS(&s_key[h], 0xFFFFFFFFu, b);
        if (old == 0xFFFFFFFFu || old == b) { atomicAdd(&s_cnt[h], 1u); done = true; }
        h = (h + 1) & (GH_SLOTS - 1);
      }
      if (!done) atomicAdd(&count[b], 1u);
    }
    __syncthreads();
    const bool last = base + (int64_t)gridDim.x * GH_TILE >= n;
    for (int i = threadIdx.x; i < GH_SLOTS; i += GH_T) {
      const uint32_t c = s_cnt[i];
      if (s_key[i] != 0xFFFFFFFFu && (last || c < GH_HOT)) {
        if (c) atomicAdd(&count[s_key[i]], c);
        s_key[i] = 0xFFFFFFFFu; s_cnt[i] = 0;
      }
    }
    __syncthreads();
  }
  if (bad) flags->index_range = 1;
}

// flag[g] = group g goes to part A.  pkind < 0: every non-empty group (plain conversion).
// Adds the number of entries in flagged groups to *nnz_a.
__global__ __launch_bounds__(256) void group_flag_kernel(const uint32_t *count, int64_t nbins, int gkind, int pkind,
                                                        int64_t num, int64_t den, int64_t thr, int64_t nrows,
                                                        int64_t ncols, int32_t *flag, int32_t *nnz_a) {
  __shared__ uint32_t s_wave[256 / 64 + 1];
  uint32_t mine = 0;
  for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < nbins; g += (int64_t)gridDim.x * 256) {
    const uint32_t cnt = count[g];
    bool f = false;
    if (cnt > 0) {
      if (pkind < 0) f = true;
      else if (pkind == US_P_SUM_GE_ABS) f = (int64_t)cnt >= thr;
      else {
        int64_t cap;
        if (gkind == G_DIAG) {
          int64_t off = g - (nrows - 1);
          int64_t hi = nrows < ncols - off ? nrows : ncols - off, lo = off < 0 ? -off : 0;
          cap = hi > lo ? hi - lo : 0;
        } else cap = gkind == G_ROW ? ncols : nrows;
        f = den * (int64_t)cnt >= num * cap;
      }
    }
    flag[g] = f ? 1 : 0;
    if (f) mine += cnt;
  }
  uint32_t total;
  block_exclusive_sum<256>(mine, s_wave, &total);
  if (threadIdx.x == 0 && total) atomicAdd(nnz_a, (int32_t)total);
}

// gmap[g] = position of group g among the flagged groups, or -1; offsets of the flagged diagonals
__global__ __launch_bounds__(256) void group_map_kernel(const int32_t *flag, const int32_t *pos, int64_t nbins,
                                                       int32_t *gmap) {
  int64_t d = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (d < nbins) gmap[d] = flag[d] ? pos[d] : -1;
}
__global__ __launch_bounds__(256) void diag_offsets_kernel(const int32_t *gmap, int64_t nbins, int32_t nrows,
                                                          int32_t *off) {
  int64_t d = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (d < nbins && gmap[d] >= 0) off[gmap[d]] = (int32_t)(d - (nrows - 1));
}


// One pass over the COO list that sends every entry to its part of a decomposition.
//   TO_SLAB: entries of flagged diagonals go straight into the DIA slab val[k*L + i]
//            (Devectorize/Fill/Vectorize).  A duplicate coordinate shows as fewer occupied slots
//            than entries, counted afterwards.  Occupied = not the fill pattern: the slab starts
//            out filled with DIA_EMPTY (a NaN bit pattern no computation produces) and a finishing
//            pass counts and zeroes what is left of it, which costs two streaming passes over the
//            slab instead of one more scattered byte store per entry (a byte map of marked slots,
//            the form used when an input value happens to carry that very bit pattern);
//   otherwise they are appended to list A.  Entries of unflagged groups are appended to list B.
// Appends reserve space once per workgroup (one atomic per list), so order inside a list is
// arbitrary; each part is put into canonical order by its conversion.
// (Ordering the entries by the top bits of their slot first, so that slab writes stay inside an
// L2-sized window, was measured and dropped: the extra pass cost more than the ~110 G
// scattered store transactions per second the direct form already sustains.)
constexpr int SP_T = 512, SP_IPT = 16, SP_TILE = SP_T * SP_IPT;
constexpr uint32_t DIA_EMPTY = 0x7FC5A5A5u;

template <bool TO_SLAB>
__global__ __launch_bounds__(SP_T) void split_kernel(const int32_t *row, const int32_t *col, const float *val,
                                                    int64_t n, int gkind, uint32_t nrows, const int32_t *gmap,
                                                    int64_t L, int by_col, float *slab, uint8_t *slotmap,
                                                    CooLists la, CooLists lb, int32_t *cursors, Flags *flags) {
  __shared__ uint32_t s_wave[SP_T / 64 + 1];
  __shared__ int32_t s_base[2];
  const int64_t base = (int64_t)blockIdx.x * SP_TILE;
  uint32_t r[SP_IPT], c[SP_IPT];
  float v[SP_IPT];
  int32_t g[SP_IPT];
#pragma unroll
  for (int k = 0; k < SP_IPT; ++k) {
    int64_t i = base + k * SP_T + threadIdx.x;
    r[k] = c[k] = 0; v[k] = 0.f;
    if (i < n) { r[k] = (uint32_t)row[i]; c[k] = (uint32_t)col[i]; v[k] = val[i]; }
  }
  uint32_t na = 0, nb = 0;
#pragma unroll
  for (int k = 0; k < SP_IPT; ++k) {
    int64_t i = base + k * SP_T + threadIdx.x;
    g[k] = -2;  // no entry
    if (i < n) {
      g[k] = gmap[group_bin(gkind, r[k], c[k], nrows)];
      if (g[k] >= 0) ++na; else ++nb;
    }
  }
  uint32_t ta, tb;
  uint32_t pa = (!TO_SLAB && la.r) ? block_exclusive_sum<SP_T>(na, s_wave, &ta) : 0u;
  uint32_t pb = lb.r ? block_exclusive_sum<SP_T>(nb, s_wave, &tb) : 0u;
  if (threadIdx.x == 0) {
    s_base[0] = (!TO_SLAB && la.r && ta) ? atomicAdd(&cursors[0], (int32_t)ta) : 0;
    s_base[1] = (lb.r && tb) ? atomicAdd(&cursors[1], (int32_t)tb) : 0;
  }
  __syncthreads();
  pa += s_base[0]; pb += s_base[1];
#pragma unroll
  for (int k = 0; k < SP_IPT; ++k) {
    if (g[k] >= 0) {
      if (TO_SLAB) {
        int64_t slot = (int64_t)g[k] * L + (by_col ? c[k] : r[k]);
        slab[slot] = v[k];
        if (slotmap) slotmap[slot] = 1;
        else if (__float_as_uint(v[k]) == DIA_EMPTY) flags->retry = RETRY_DIA_MARKS;
      } else if (la.r) {
        la.r[pa] = (int32_t)r[k]; la.c[pa] = (int32_t)c[k]; la.v[pa] = v[k]; ++pa;
      }
    } else if (g[k] == -1 && lb.r) {
      lb.r[pb] = (int32_t)r[k]; lb.c[pb] = (int32_t)c[k]; lb.v[pb] = v[k]; ++pb;
    }
  }
}

// occupied slots of a slab that started out as DIA_EMPTY; what is still empty becomes +0.0
__global__ __launch_bounds__(256) void dia_finish_kernel(uint4 *slab4, int64_t nvec, int64_t nslots, int32_t *out) {
  __shared__ uint32_t s_wave[256 / 64 + 1];
  uint32_t cnt = 0;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * 256) {
    uint4 w = slab4[i];
    uint32_t *e = reinterpret_cast<uint32_t *>(&w);
    bool changed = false;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (i * 4 + k >= nslots) continue;   // the allocation is padded to whole vectors
      if (e[k] == DIA_EMPTY) { e[k] = 0u; changed = true; } else ++cnt;
    }
    if (changed) slab4[i] = w;
  }
  uint32_t total;
  block_exclusive_sum<256>(cnt, s_wave, &total);
  if (threadIdx.x == 0 && total) atomicAdd(out, (int32_t)total);
}

// number of marked slots (bytes are 0 or 1; the map is padded with zeros to a multiple of 16)
__global__ __launch_bounds__(256) void count_marks_kernel(const uint4 *m, int64_t nvec, int32_t *out) {
  __shared__ uint32_t s_wave[256 / 64 + 1];
  uint32_t cnt = 0;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * 256) {
    uint4 w = m[i];
    cnt += __popc(w.x) + __popc(w.y) + __popc(w.z) + __popc(w.w);
  }
  uint32_t total;
  block_exclusive_sum<256>(cnt, s_wave, &total);
  if (threadIdx.x == 0 && total) atomicAdd(out, (int32_t)total);
}

CooLists alloc_lists(Env &env, int64_t n) {
  CooLists l;
  l.r = env.owned<int32_t>(n); l.c = env.owned<int32_t>(n); l.v = env.owned<float>(n);
  return l;
}
void free_lists(Env &env, CooLists &l) {
  env.free_raw(l.r); env.free_raw(l.c); env.free_raw(l.v);
  l = CooLists();
}

// DIA from per-diagonal flags (flags->scalar[1] already holds the number of flagged entries).
// If `rest` is given, the entries of the unflagged diagonals are collected into it in the same
// pass (its arrays are allocated here; the caller owns them afterwards) and *nrest is their number.
// verify_later != null: the last read of the flags (coordinates in range, no value carrying the empty pattern, as
// many occupied slots as entries) is left to the caller, who enqueues more work first and then calls
// dia_verify with *verify_later: the host then waits once for both instead of twice.
struct DiaPending { Flags *flags = nullptr; int64_t na = 0; };

static us_status dia_verify(Env &env, const DiaPending &p) {
  Flags h{};
  if (!read_flags(env, p.flags, &h)) return env.status;
  if (flag_status(h) != US_OK) return flag_status(h);
  return h.scalar[3] != p.na ? US_ERR_DUPLICATE : US_OK;
}

static us_status dia_from_flags(Env &env, const us_coo &coo, const Plan &plan, const us_format_desc &desc,
                                Flags *flags, const int32_t *flag, us_formatted **out, CooLists *rest,
                                int64_t *nrest, DiaPending *verify_later = nullptr) {
  const int64_t nbins = coo.nrows + coo.ncols - 1, n = coo.nnz;
  const int64_t L = plan.swapped ? coo.ncols : coo.nrows;
  int32_t *pos = env.temp<int32_t>(nbins), *gmap = env.temp<int32_t>(nbins);
  int32_t *cursors = env.temp<int32_t>(2);
  if (!env.ok()) return env.status;
  exclusive_scan_i32(env, flag, pos, nbins, &flags->scalar[0]);
  US_LAUNCH(env, "group_map", 12.0 * nbins, group_map_kernel, ceil_div<int64_t>(nbins, 256), 256, flag,
            (const int32_t *)pos, nbins, gmap);
  Flags h{};
  if (!read_flags(env, flags, &h)) return env.status;
  if (flag_status(h) != US_OK) return flag_status(h);
  const int64_t ndiag = h.scalar[0], na = h.scalar[1];
  if (ndiag * L >= (1ll << 31)) return US_ERR_OVERFLOW;
  us_formatted *f = new us_formatted();
  f->desc = desc; f->pattern = P_DIA; f->swapped = plan.swapped;
  f->nrows = coo.nrows; f->ncols = coo.ncols; f->nnz = na;
  f->nlevels = 2;
  f->level[0].idx = env.owned<int32_t>(ndiag); f->level[0].nidx = ndiag;
  f->level[1].size = L;
  const int64_t nslab4 = ceil_div<int64_t>(ndiag * L, 4);
  f->val = env.owned<float>(nslab4 * 4); f->nval = ndiag * L; f->nmajor = ndiag;   // whole 16-byte vectors
  const bool marks = env.dia_marks;
  const int64_t nvec = ceil_div<int64_t>(ndiag * L, 16) + 1;
  uint8_t *slotmap = marks ? (uint8_t *)env.temp<uint4>(nvec) : nullptr;
  CooLists lb;
  if (rest) { *nrest = n - na; lb = alloc_lists(env, n - na); *rest = lb; }
  if (!env.ok()) { free_formatted(env, f); return env.status; }
  fill_u32(env, (uint32_t *)f->val, ndiag * L, marks ? 0u : DIA_EMPTY);
  if (marks) fill_u32(env, (uint32_t *)slotmap, nvec * 4, 0u);
  fill_u32(env, (uint32_t *)cursors, 2, 0u);
  US_LAUNCH(env, "diag_offsets", 8.0 * nbins, diag_offsets_kernel, ceil_div<int64_t>(nbins, 256), 256,
            (const int32_t *)gmap, nbins, (int32_t)coo.nrows, f->level[0].idx);
  if (n > 0)
    US_LAUNCH(env, "dia_split_scatter", 12.0 * n + 5.0 * na + 12.0 * (rest ? n - na : 0), (split_kernel<true>),
              ceil_div<int64_t>(n, SP_TILE), SP_T, coo.row, coo.col, coo.val, n, (int)G_DIAG, (uint32_t)coo.nrows,
              (const int32_t *)gmap, L, plan.swapped ? 1 : 0, f->val, slotmap, CooLists(), lb, cursors, flags);
  if (marks)
    US_LAUNCH(env, "count_marks", 1.0 * ndiag * L, count_marks_kernel, one_counter_grid(nvec, 256), 256, (const uint4 *)slotmap, nvec, &flags->scalar[3]);
  else if (nslab4 > 0)
    US_LAUNCH(env, "dia_finish", 4.0 * ndiag * L, dia_finish_kernel, one_counter_grid(nslab4, 256), 256, (uint4 *)f->val, nslab4, ndiag * L, &flags->scalar[3]);
  if (verify_later) {
    verify_later->flags = flags; verify_later->na = na;
    if (!env.ok()) { free_formatted(env, f); return env.status; }
    *out = f;
    return US_OK;
  }
  const us_status st = dia_verify(env, DiaPending{flags, na});
  if (st != US_OK) { free_formatted(env, f); return st; }
  *out = f;
  return US_OK;
}


// histogram of the groups + predicate flags; pkind < 0 flags every non-empty group
struct GroupCounts { uint32_t *count; int32_t *flag; int64_t nbins; };

static GroupCounts group_flags(Env &env, const us_coo &coo, int gkind, int pkind, int64_t num, int64_t den,
                               int64_t thr, Flags *flags) {
  GroupCounts g{};
  g.nbins = gkind == G_DIAG ? coo.nrows + coo.ncols - 1 : (gkind == G_ROW ? coo.nrows : coo.ncols);
  g.count = env.temp<uint32_t>(g.nbins);
  g.flag = env.temp<int32_t>(g.nbins);
  if (!env.ok()) return g;
  fill_u32(env, g.count, g.nbins, 0);
  if (coo.nnz > 0)
    US_LAUNCH(env, "group_hist", 8.0 * coo.nnz, group_hist_kernel, one_counter_grid(coo.nnz, GH_TILE), GH_T, coo.row,
              coo.col, coo.nnz, gkind, (uint32_t)coo.nrows, (uint32_t)coo.ncols, g.count, flags);
  US_LAUNCH(env, "group_flag", 8.0 * g.nbins, group_flag_kernel, one_counter_grid(g.nbins, 256), 256,
            (const uint32_t *)g.count, g.nbins, gkind, pkind, num, den, thr, coo.nrows, coo.ncols, g.flag,
            &flags->scalar[1]);
  return g;
}

// what the histogram, the flags and (for DIA) the positions and slab indices of the groups take from Env::temp
static size_t group_temp_bytes(int64_t nbins) {
  return 4 * Env::granule(4 * (size_t)nbins) + Env::granule(4 * ((size_t)nbins / 1024 + 64)) + 8 * Env::granule(256);
}

us_status convert_dia(Env &env, const us_coo &coo, const Plan &plan, const us_format_desc &desc,
                      Flags *flags, us_formatted **out) {
  GroupCounts g = group_flags(env, coo, G_DIAG, -1, 0, 1, 0, flags);
  if (!env.ok()) return env.status;
  return dia_from_flags(env, coo, plan, desc, flags, g.flag, out, nullptr, nullptr);
}

us_status decompose_sum(Env &env, const us_coo &coo, const Plan &pa, const us_format_desc &da, const Plan &pb,
                        const us_format_desc &db, const us_predicate &pred, int gkind, us_formatted **oa,
                        us_formatted **ob) {
  env.reserve(group_temp_bytes(gkind == G_DIAG ? coo.nrows + coo.ncols - 1 : (gkind == G_ROW ? coo.nrows : coo.ncols)));
  Flags *flags = new_flags(env);
  if (!env.ok()) return env.status;
  GroupCounts g = group_flags(env, coo, gkind, pred.kind, pred.num, pred.den, pred.abs, flags);
  if (!env.ok()) return env.status;
  const int64_t n = coo.nnz;
  CooLists la, lb;
  int64_t na = 0, nb = 0;
  us_status st;
  DiaPending pending;
  if (gkind == G_DIAG && pa.pattern == P_DIA) {
    // part A goes straight into the slab while part B is collected, in one pass over the input; its flags are read
    // after part B's conversion has been enqueued (and has read its own): an input that fails them (a coordinate
    // out of range reaches no slab slot and no list; a duplicate is a slot written twice) is reported then
    st = dia_from_flags(env, coo, pa, da, flags, g.flag, oa, &lb, &nb, &pending);
  } else {
    Flags h{};
    if (!read_flags(env, flags, &h)) return env.status;
    if (flag_status(h) != US_OK) return flag_status(h);
    na = h.scalar[1]; nb = n - na;
    la = alloc_lists(env, na); lb = alloc_lists(env, nb);
    int32_t *gmap = env.temp<int32_t>(g.nbins), *cursors = env.temp<int32_t>(2);
    st = env.status;
    if (st == US_OK) {
      fill_u32(env, (uint32_t *)cursors, 2, 0u);
      US_LAUNCH(env, "group_map", 12.0 * g.nbins, group_map_kernel, ceil_div<int64_t>(g.nbins, 256), 256,
                (const int32_t *)g.flag, (const int32_t *)g.flag, g.nbins, gmap);
      if (n > 0)
        US_LAUNCH(env, "split", 24.0 * n, (split_kernel<false>), ceil_div<int64_t>(n, SP_TILE), SP_T, coo.row, coo.col,
                  coo.val, n, gkind, (uint32_t)coo.nrows, (const int32_t *)gmap, (int64_t)0, 0, (float *)nullptr,
                  (uint8_t *)nullptr, la, lb, cursors, flags);
      st = env.status;
    }
    if (st == US_OK) {
      us_coo ca{coo.nrows, coo.ncols, na, la.r, la.c, la.v};
      st = convert_with_plan(env, ca, pa, da, oa);
    }
  }
  if (st == US_OK) {
    us_coo cb{coo.nrows, coo.ncols, nb, lb.r, lb.c, lb.v};
    st = convert_with_plan(env, cb, pb, db, ob);
  }
  if (pending.flags) {   // part A's own verdict comes first: part B may have failed only because of what it reports
    const us_status sa = dia_verify(env, pending);
    if (sa != US_OK) st = sa;
  }
  env.sync();
  free_lists(env, la);
  free_lists(env, lb);
  return st;
}

}  // namespace us
