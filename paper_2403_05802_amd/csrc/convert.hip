// COO -> target format, and the decompose op.  Host side: match the format encoding against
// the supported patterns and infer which size/ptr/idx/val arrays exist (Section 5.1); device
// side: the runtime effect of the conversion operators of Table 2 -- index-map evaluation
// (Swap / Skew / TileSplit) inside the sort-key build, Sort, Sum (histograms), Merge (head
// flags + scan -> ptr), Fill / Trim of the major level, Enumerate (rank in row), and
// Devectorize/Fill/Vectorize (zero-filled dense inner levels that entries are scattered into).
#include "common.h"
#include "device.h"

namespace us {

// ------------------------------------------------------------------ descriptor matching (host)
struct Plan {
  Pattern pattern;
  bool swapped = false;  // major dimension is d1
  int64_t bh = 1, bw = 1;
  int64_t ell_width = 0;
};

static bool aff(const us_expr &e, int c0, int c1) {
  return e.kind == US_E_AFFINE && e.c0 == c0 && e.c1 == c1 && e.c == 0;
}
static bool tile(const us_expr &e, int kind, int dim, int64_t *f, int64_t max_factor = 16) {
  if (e.kind != kind || e.c != 0 || e.factor < 1 || e.factor > max_factor) return false;
  if (!(e.c0 == (dim == 0) && e.c1 == (dim == 1))) return false;
  *f = e.factor;
  return true;
}

static bool match_desc(const us_format_desc &d, Plan *p) {
  const int S = d.trim_s, E = d.trim_e;
  const uint32_t m = d.merge_mask;
  if (d.nlevels == 2) {
    const us_expr &a = d.level[0], &b = d.level[1];
    bool ident = aff(a, 1, 0) && aff(b, 0, 1), swap = aff(a, 0, 1) && aff(b, 1, 0);
    if (ident || swap) {
      p->swapped = swap;
      if (S == 0 && E == 1 && m == 0) { p->pattern = P_COO; return true; }
      if (S == 1 && E == 1 && m == 1) { p->pattern = P_CSR; return true; }
      if (S == 0 && E == 1 && m == 1) { p->pattern = P_DCSR; return true; }
      return false;
    }
    if (aff(a, -1, 1) && S == 0 && E == 0 && m == 1) {
      if (aff(b, 1, 0)) { p->pattern = P_DIA; p->swapped = false; return true; }
      if (aff(b, 0, 1)) { p->pattern = P_DIA; p->swapped = true; return true; }
    }
    return false;
  }
  if (d.nlevels == 4) {
    int64_t f0, f1, f2, f3;
    if (tile(d.level[0], US_E_DIV, 0, &f0) && tile(d.level[1], US_E_DIV, 1, &f1) &&
        tile(d.level[2], US_E_MOD, 0, &f2) && tile(d.level[3], US_E_MOD, 1, &f3) && f0 == f2 && f1 == f3 &&
        S == 1 && E == 1 && (m == 3 || m == 2)) {
      p->pattern = P_BCSR; p->bh = f0; p->bw = f1;
      return true;
    }
    if (tile(d.level[0], US_E_DIV, 0, &f0, 65536) && tile(d.level[1], US_E_DIV, 1, &f1, 65536) &&
        tile(d.level[2], US_E_MOD, 0, &f2, 65536) && tile(d.level[3], US_E_MOD, 1, &f3, 65536) && f0 == f2 &&
        f1 == f3 && S == 2 && E == 3 && m == 2) {
      p->pattern = P_CSB; p->bh = f0; p->bw = f1;
      return true;
    }
    return false;
  }
  if (d.nlevels == 3) {
    const us_expr &e = d.level[0];
    if (e.kind == US_E_INDIRECT_ENUM && e.c0 == 1 && e.c1 == 0 && e.c == 0 && aff(d.level[1], 1, 0) &&
        aff(d.level[2], 0, 1) && S == 0 && E == 0 && m == 1 && d.ell_width >= 0) {
      p->pattern = P_ELL; p->ell_width = d.ell_width;
      return true;
    }
    if (e.kind == US_E_INDIRECT_SCHEDULE && e.c0 == 1 && e.c1 == 0 && e.c == 0 && e.factor >= 1 && e.factor <= 65536 &&
        aff(d.level[1], 1, 0) && aff(d.level[2], 0, 1) && S == 1 && E == 2 && m == 3) {
      p->pattern = P_CISR; p->bh = e.factor;   // bh: number of partitions
      return true;
    }
    int64_t f0, f2;
    if (tile(d.level[0], US_E_DIV, 0, &f0) && aff(d.level[1], -1, 1) && tile(d.level[2], US_E_MOD, 0, &f2) &&
        f0 == f2 && S == 1 && E == 1 && m == 1) {
      p->pattern = P_BDIA; p->bh = f0; p->bw = 1;
      return true;
    }
  }
  return false;
}

// ------------------------------------------------------------------ small kernels
__global__ __launch_bounds__(256) void check_unique_unpacked_kernel(const int32_t *major, const int32_t *minor,
                                                                   int64_t n, Flags *flags) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x + 1;
  if (i < n && major[i] == major[i - 1] && minor[i] == minor[i - 1]) flags->duplicate = 1;
}

__global__ __launch_bounds__(256) void nonempty_flag_kernel(const int32_t *ptr, int64_t n, int32_t *flag) {
  int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (g < n) flag[g] = ptr[g + 1] > ptr[g] ? 1 : 0;
}

// *nnr_dev = number of non-empty groups (the total of the scan that made pos); the arrays hold `cap` of
// them, which a valid input never exceeds
__global__ __launch_bounds__(256) void dcsr_compact_kernel(const int32_t *ptr, const int32_t *pos, int64_t n,
                                                          const int32_t *nnr_dev, int64_t cap, int32_t nnz,
                                                          int32_t *idx0, int32_t *ptr1) {
  int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (g == 0) {
    const int64_t nnr = *nnr_dev;
    ptr1[nnr >= 0 && nnr < cap ? nnr : cap] = nnz;
  }
  if (g < n && ptr[g + 1] > ptr[g]) {
    int32_t k = pos[g];
    if (k >= 0 && k < cap) {
      idx0[k] = (int32_t)g;
      ptr1[k] = ptr[g];
    }
  }
}

// Kernels that end with one atomic per workgroup on a single counter run on at most ONE_COUNTER_GRID
// workgroups (grid-stride loops): same-address device atomics cost ~20 ns apiece on this part, so
// thousands of them would outlast the kernel's real work.
constexpr int ONE_COUNTER_GRID = 768;
static inline int64_t one_counter_grid(int64_t items, int per_block) {
  const int64_t g = ceil_div<int64_t>(items, per_block);
  return g < ONE_COUNTER_GRID ? (g > 0 ? g : 1) : ONE_COUNTER_GRID;
}

__global__ __launch_bounds__(256) void max_len_kernel(const int32_t *ptr, int64_t n, int32_t *out_max) {
  __shared__ int32_t s_max[4];
  int32_t len = 0;
  for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < n; g += (int64_t)gridDim.x * 256)
    len = max(len, ptr[g + 1] - ptr[g]);
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) len = max(len, __shfl_xor(len, d));
  if (lane_id() == 0) s_max[wave_id()] = len;
  __syncthreads();
  if (threadIdx.x == 0) {
    int32_t m = max(max(s_max[0], s_max[1]), max(s_max[2], s_max[3]));
    if (m > 0) atomicMax(out_max, m);
  }
}

// ELL: entry i of the sorted list sits in slot rank = i - ptr[row] of its row (the enum query)
__global__ __launch_bounds__(256) void ell_scatter_kernel(const int32_t *major, const int32_t *minor,
                                                         const float *val, const int32_t *ptr, int64_t n,
                                                         int64_t nrows, int64_t K, int32_t *ecol, float *eval,
                                                         Flags *flags) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  int32_t r = major[i];
  int64_t rank = i - ptr[r];
  if (rank >= K) { flags->ell_overflow = 1; return; }
  int64_t slot = rank * nrows + r;
  ecol[slot] = minor[i];
  eval[slot] = val[i];
}

// ------------------------------------------------------------------ helpers (host)
static bool read_flags(Env &env, Flags *dev, Flags *host) {
  env.check(hipMemcpyAsync(host, dev, sizeof(Flags), hipMemcpyDeviceToHost, env.stream));
  env.sync();
  return env.ok();
}

static us_status flag_status(const Flags &h) {
  if (h.retry) return US_SORT_RETRY;
  if (h.index_range) return US_ERR_INDEX_RANGE;
  if (h.duplicate) return US_ERR_DUPLICATE;
  if (h.ell_overflow) return US_ERR_SHAPE;
  return US_OK;
}

void free_formatted(Env &env, us_formatted *f) {
  if (!f) return;
  for (int l = 0; l < 4; ++l) {
    env.free_raw(f->level[l].ptr);
    env.free_raw(f->level[l].idx);
  }
  env.free_raw(f->val);
  env.free_raw(f->ws);
  env.free_raw(f->mp_split);
  delete f;
}

void *ensure_workspace(Env &env, const us_formatted &A, size_t bytes) {
  if (A.ws_bytes >= bytes && A.ws) return A.ws;
  if (A.ws) {
    env.sync();  // an earlier compute call may still use the old scratch
    env.free_raw(A.ws);
    A.ws = nullptr; A.ws_bytes = 0;
  }
  A.ws = env.alloc_raw(bytes < 256 ? 256 : bytes);
  if (!A.ws) { env.fail(US_ERR_ALLOC); return nullptr; }
  A.ws_bytes = bytes;
  return A.ws;
}

static KeySpec rowcol_keyspec(const us_coo &coo, bool swapped) {
  KeySpec ks{};
  ks.mode = 0; ks.swap = swapped ? 1 : 0;
  ks.a_extent = (uint32_t)(swapped ? coo.ncols : coo.nrows);
  ks.b_extent = (uint32_t)(swapped ? coo.nrows : coo.ncols);
  ks.b_bits = bits_for(ks.b_extent - 1);
  ks.total_bits = ks.b_bits + bits_for(ks.a_extent - 1);
  ks.bh = ks.bw = 1;
  return ks;
}

// Gives f (shape already set) the levels of an ELL tensor of width K with every slot empty: column -1, value 0.
static bool ell_shell(Env &env, us_formatted *f, int64_t K) {
  const int64_t slots = K * f->nrows;
  int32_t *ecol = env.owned<int32_t>(slots);
  float *ev = env.owned<float>(slots);
  f->nlevels = 3;
  f->level[0].size = K; f->level[1].size = f->nrows;
  f->level[2].idx = ecol; f->level[2].nidx = slots;
  f->val = ev; f->nval = slots; f->nmajor = K;
  if (!env.ok()) return false;
  fill_u32(env, (uint32_t *)ecol, slots, 0xFFFFFFFFu);
  fill_u32(env, (uint32_t *)ev, slots, 0u);
  return true;
}

static us_formatted *new_empty_ell(Env &env, const us_format_desc &desc, int64_t nrows, int64_t ncols, int64_t nnz,
                                   int64_t K) {
  us_formatted *f = new us_formatted();
  f->desc = desc; f->pattern = P_ELL; f->swapped = false;
  f->nrows = nrows; f->ncols = ncols; f->nnz = nnz;
  if (!ell_shell(env, f, K)) { free_formatted(env, f); return nullptr; }
  return f;
}

// Build COO / CSR / DCSR / ELL from entries already sorted by (major, minor).  `major` is a
// temporary unless the format keeps it (COO); `minor` and `val` are owned arrays of nnz entries
// that move into the result (or are released when the format re-lays them out: ELL).
static us_status build_from_sorted(Env &env, const Plan &plan, const us_format_desc &desc, int64_t nrows,
                                   int64_t ncols, int64_t nnz, int32_t *major, int32_t *minor, float *val,
                                   Flags *flags, bool check_dups, us_formatted **out, bool validated = false) {
  // Takes ownership of major, minor and val (arrays of nnz entries from Env::owned).
  // validated: the caller has already read the flags after the sort (indices are in range).
  us_formatted *f = new us_formatted();
  f->desc = desc; f->pattern = plan.pattern; f->swapped = plan.swapped;
  f->nrows = nrows; f->ncols = ncols; f->nnz = nnz;
  const int64_t nmaj = plan.swapped ? ncols : nrows;
  bool major_loose = true, minor_loose = true, val_loose = true;  // not yet attached to f
  auto finish = [&](us_status s) {
    if (major_loose) env.free_raw(major);
    if (minor_loose) env.free_raw(minor);
    if (val_loose) env.free_raw(val);
    if (s != US_OK) free_formatted(env, f); else *out = f;
    return s;
  };
  auto flags_ok = [&](Flags *h) {
    if (!read_flags(env, flags, h)) return env.status;
    return flag_status(*h);
  };
  Flags h{};

  if (plan.pattern == P_COO) {
    if (check_dups && nnz > 1)
      US_LAUNCH(env, "check_unique", 8.0 * nnz, check_unique_unpacked_kernel, ceil_div<int64_t>(nnz, 256), 256,
                (const int32_t *)major, (const int32_t *)minor, nnz, flags);
    f->nlevels = 2;
    f->level[0].idx = major; f->level[0].nidx = nnz;
    f->level[1].idx = minor; f->level[1].nidx = nnz;
    f->val = val; f->nval = nnz; f->nmajor = nnz;
    major_loose = minor_loose = val_loose = false;
    return finish(flags_ok(&h));
  }

  // pointers over every major index (Fill(0) + Merge(0))
  int32_t *ptr;
  if (plan.pattern == P_CSR) {
    ptr = env.owned<int32_t>(nmaj + 1);
    f->level[1].ptr = ptr; f->level[1].nptr = nmaj + 1;
  } else {
    ptr = env.temp<int32_t>(nmaj + 1);
  }
  if (!env.ok()) return finish(env.status);
  // one pass over the entries gives both ptr and the duplicate check; with fewer entries than groups the
  // runs of empty groups are long and a binary search per group is the quicker way to ptr
  if (nnz >= nmaj) {
    group_ptr_unique(env, major, minor, nnz, nmaj, ptr, check_dups, flags);
  } else {
    if (check_dups && nnz > 1)
      US_LAUNCH(env, "check_unique", 8.0 * nnz, check_unique_unpacked_kernel, ceil_div<int64_t>(nnz, 256), 256,
                (const int32_t *)major, (const int32_t *)minor, nnz, flags);
    lower_bound_ptr(env, major, nnz, nmaj, ptr);
  }

  if (plan.pattern == P_CSR) {
    f->nlevels = 2;
    f->level[0].size = nmaj;
    f->level[1].idx = minor; f->level[1].nidx = nnz;
    f->val = val; f->nval = nnz; f->nmajor = nmaj;
    minor_loose = val_loose = false;
    spmv_prepare(env, f);
    return finish(flags_ok(&h));
  }

  if (plan.pattern == P_DCSR) {
    // Trim(0): keep only the major indices that have children.  How many there are (nnr) stays on the
    // device until the one read of the flags that ends the call: idx and ptr are allocated for the most
    // there can be, min(nmaj, nnz), and the kernels in between take nnr from device memory.
    const int64_t cap = nmaj < nnz ? nmaj : nnz;
    int32_t *flag = env.temp<int32_t>(nmaj), *pos = env.temp<int32_t>(nmaj);
    int32_t *idx0 = env.owned<int32_t>(cap), *ptr1 = env.owned<int32_t>(cap + 1);
    f->nlevels = 2;
    f->level[0].idx = idx0; f->level[0].nidx = 0;
    f->level[1].ptr = ptr1; f->level[1].nptr = 1;
    f->level[1].idx = minor; f->level[1].nidx = nnz;
    f->val = val; f->nval = nnz; f->nmajor = 0;
    minor_loose = val_loose = false;
    if (!env.ok()) return finish(env.status);
    US_LAUNCH(env, "nonempty_flag", 8.0 * nmaj, nonempty_flag_kernel, ceil_div<int64_t>(nmaj, 256), 256,
              (const int32_t *)ptr, nmaj, flag);
    exclusive_scan_i32(env, flag, pos, nmaj, &flags->scalar[0]);
    US_LAUNCH(env, "dcsr_compact", 12.0 * nmaj + 8.0 * cap, dcsr_compact_kernel, ceil_div<int64_t>(nmaj, 256), 256,
              (const int32_t *)ptr, (const int32_t *)pos, nmaj, (const int32_t *)&flags->scalar[0], cap,
              (int32_t)nnz, idx0, ptr1);
    spmv_prepare(env, f, &flags->scalar[0], cap);
    us_status s = flags_ok(&h);
    if (s != US_OK) return finish(s);
    const int64_t nnr = h.scalar[0];
    f->level[0].nidx = nnr; f->level[1].nptr = nnr + 1; f->nmajor = nnr;
    f->mp_tiles = f->mp_split ? spmv_tiles(nnr, nnz) : 0;
    return finish(US_OK);
  }

  if (plan.pattern == P_ELL) {
    int64_t K = plan.ell_width;
    if (K == 0)
      US_LAUNCH(env, "max_row_len", 4.0 * nmaj, max_len_kernel, one_counter_grid(nmaj, 256), 256,
                (const int32_t *)ptr, nmaj, &flags->scalar[0]);
    if (K == 0 || !validated) {   // the scatter below indexes by the major index: it must be known to be in range
      us_status s = flags_ok(&h);
      if (s != US_OK) return finish(s);
      if (K == 0) K = h.scalar[0];
    }
    if (K * nrows >= (1ll << 31)) return finish(US_ERR_OVERFLOW);
    if (!ell_shell(env, f, K)) return finish(env.status);
    int32_t *ecol = f->level[2].idx;
    float *ev = f->val;
    if (nnz > 0)
      US_LAUNCH(env, "ell_scatter", 16.0 * nnz + 8.0 * nnz, ell_scatter_kernel, ceil_div<int64_t>(nnz, 256), 256,
                (const int32_t *)major, (const int32_t *)minor, (const float *)val, (const int32_t *)ptr, nnz,
                nrows, K, ecol, ev, flags);
    return finish(flags_ok(&h));
  }
  return finish(US_ERR_UNSUPPORTED_DESC);
}

// ------------------------------------------------------------------ Sum query (group histogram) and DIA
// Groups supported by the groupBy map of the sum query: diagonals (d1-d0), rows (d0), columns (d1).
enum { G_DIAG = 0, G_ROW = 1, G_COL = 2 };

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

struct CooLists { int32_t *r = nullptr, *c = nullptr; float *v = nullptr; };

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

static CooLists alloc_lists(Env &env, int64_t n) {
  CooLists l;
  l.r = env.owned<int32_t>(n); l.c = env.owned<int32_t>(n); l.v = env.owned<float>(n);
  return l;
}
static void free_lists(Env &env, CooLists &l) {
  env.free_raw(l.r); env.free_raw(l.c); env.free_raw(l.v);
  l = CooLists();
}

// DIA from per-diagonal flags (flags->scalar[1] already holds the number of flagged entries).
// If `rest` is given, the entries of the unflagged diagonals are collected into it in the same
// pass (its arrays are allocated here; the caller owns them afterwards) and *nrest is their number.
static us_status dia_from_flags(Env &env, const us_coo &coo, const Plan &plan, const us_format_desc &desc,
                                Flags *flags, const int32_t *flag, us_formatted **out, CooLists *rest,
                                int64_t *nrest) {
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
  if (!read_flags(env, flags, &h)) { free_formatted(env, f); return env.status; }
  if (flag_status(h) != US_OK) { free_formatted(env, f); return flag_status(h); }
  if (h.scalar[3] != na) { free_formatted(env, f); return US_ERR_DUPLICATE; }
  *out = f;
  return US_OK;
}

struct GroupCounts { uint32_t *count; int32_t *flag; int64_t nbins; };

// histogram of the groups + predicate flags; pkind < 0 flags every non-empty group
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

static us_status convert_dia(Env &env, const us_coo &coo, const Plan &plan, const us_format_desc &desc,
                             Flags *flags, us_formatted **out) {
  GroupCounts g = group_flags(env, coo, G_DIAG, -1, 0, 1, 0, flags);
  if (!env.ok()) return env.status;
  return dia_from_flags(env, coo, plan, desc, flags, g.flag, out, nullptr, nullptr);
}

// ------------------------------------------------------------------ BCSR
// After sorting by (d0/bh, d1/bw, d0%bh, d1%bw) the entries of a block are contiguous.
// Merge(0,1): head flag where the block prefix changes, scan -> block id.
constexpr int BE_T = 256, BE_IPT = 8, BE_TILE = BE_T * BE_IPT;

__global__ __launch_bounds__(BE_T) void bcsr_count_kernel(const uint64_t *key, int64_t n, int inner_bits,
                                                         uint32_t *partial, Flags *flags) {
  __shared__ uint32_t s_wave[BE_T / 64 + 1];
  int64_t base = (int64_t)blockIdx.x * BE_TILE;
  uint32_t heads = 0;
  bool dup = false;
#pragma unroll
  for (int k = 0; k < BE_IPT; ++k) {
    int64_t i = base + k * BE_T + threadIdx.x;
    if (i < n) {
      uint64_t cur = key[i], prev = i > 0 ? key[i - 1] : ~0ull;
      dup |= (i > 0) & (cur == prev);
      heads += (i == 0) | ((cur >> inner_bits) != (prev >> inner_bits));
    }
  }
  if (dup) flags->duplicate = 1;
  uint32_t total;
  block_exclusive_sum<BE_T>(heads, s_wave, &total);
  if (threadIdx.x == 0) partial[blockIdx.x] = total;
}

__global__ __launch_bounds__(BE_T) void bcsr_emit_kernel(const uint64_t *key, const float *val, int64_t n,
                                                        KeySpec ks, int32_t col_bias, const uint32_t *partial,
                                                        int32_t *blk_row, int32_t *blk_col, float *bval) {
  __shared__ uint32_t s_wave[BE_T / 64 + 1];
  const int inner_bits = ks.ih_bits + ks.iw_bits;
  const int lane = lane_id();
  // a wavefront owns 64*BE_IPT consecutive entries, lanes striped (coalesced loads); block ids
  // come from ballots of the head flags, so no per-thread serial run is needed
  const int64_t wbase = (int64_t)blockIdx.x * BE_TILE + (int64_t)wave_id() * (64 * BE_IPT);
  uint64_t k[BE_IPT];
  uint64_t hb[BE_IPT];   // ballot of head flags of item j
  uint32_t wave_total = 0;
  uint64_t last_prev = (wbase > 0 && wbase <= n) ? key[wbase - 1] : ~0ull;  // key before the wave's slice
#pragma unroll
  for (int j = 0; j < BE_IPT; ++j) {
    const int64_t i = wbase + j * 64 + lane;
    k[j] = i < n ? key[i] : ~0ull;
  }
#pragma unroll
  for (int j = 0; j < BE_IPT; ++j) {
    const int64_t i = wbase + j * 64 + lane;
    uint64_t prev = __shfl_up(k[j], 1);
    if (lane == 0) prev = last_prev;
    const bool head = (i < n) && ((i == 0) | ((k[j] >> inner_bits) != (prev >> inner_bits)));
    hb[j] = __ballot(head);
    wave_total += (uint32_t)__popcll(hb[j]);
    last_prev = __shfl(k[j], 63);
  }
  uint32_t total;
  uint32_t wave_base = block_exclusive_sum<BE_T>(lane == 0 ? wave_total : 0u, s_wave, &total);
  uint32_t run = __shfl(wave_base, 0) + partial[blockIdx.x];  // blocks before this wave's slice
  const uint32_t bsz = ks.bh * ks.bw;
#pragma unroll
  for (int j = 0; j < BE_IPT; ++j) {
    const int64_t i = wbase + j * 64 + lane;
    if (i < n) {
      const bool head = (hb[j] >> lane) & 1ull;
      const uint32_t blk = run + (uint32_t)__popcll(hb[j] & (lanes_below() | (1ull << lane))) - 1;
      const uint32_t bi = (uint32_t)(k[j] & ((1ull << ks.iw_bits) - 1));
      const uint32_t ai = (uint32_t)((k[j] >> ks.iw_bits) & ((1ull << ks.ih_bits) - 1));
      const uint64_t bk = k[j] >> inner_bits;
      if (head) {
        blk_col[blk] = (int32_t)(bk & ((1ull << ks.b_bits) - 1)) - col_bias;
        blk_row[blk] = (int32_t)(bk >> ks.b_bits);
      }
      bval[(size_t)blk * bsz + ai * ks.bw + bi] = val[i];
    }
    run += (uint32_t)__popcll(hb[j]);
  }
}

// Key layout of the two blocked families: BCSR (d0/bh, d1/bw, d0%bh, d1%bw) and BDIA
// (d0/bh, d1-d0 biased by nrows-1, d0%bh).
static KeySpec blocked_keyspec(const Plan &plan, int64_t nrows, int64_t ncols) {
  const int64_t nbr = ceil_div<int64_t>(nrows, plan.bh);
  KeySpec ks{};
  ks.swap = 0; ks.bh = (uint32_t)plan.bh; ks.bw = (uint32_t)plan.bw;
  ks.a_extent = (uint32_t)nrows; ks.b_extent = (uint32_t)ncols;
  ks.ih_bits = bits_for(plan.bh - 1);
  if (plan.pattern == P_BDIA) {
    ks.mode = 2; ks.b_bits = bits_for(nrows + ncols - 2); ks.iw_bits = 0;
  } else {
    ks.mode = 1; ks.b_bits = bits_for(ceil_div<int64_t>(ncols, plan.bw) - 1); ks.iw_bits = bits_for(plan.bw - 1);
  }
  ks.total_bits = bits_for(nbr - 1) + ks.b_bits + ks.ih_bits + ks.iw_bits;
  return ks;
}

// Sorted keys -> ptr/idx of the merged node level and the zero-filled dense inner levels.
static us_status emit_blocked(Env &env, const Plan &plan, const us_format_desc &desc, int64_t nrows, int64_t ncols,
                              const KeySpec &ks, const uint64_t *skey, const float *sval, int64_t n, Flags *flags,
                              us_formatted **out) {
  const int64_t nbr = ceil_div<int64_t>(nrows, plan.bh);
  const int64_t nb = ceil_div<int64_t>(n > 0 ? n : 1, BE_TILE);
  uint32_t *partial = env.temp<uint32_t>(nb);
  if (!env.ok()) return env.status;
  US_LAUNCH(env, "bcsr_count", 8.0 * n, bcsr_count_kernel, nb, BE_T, skey, n, ks.ih_bits + ks.iw_bits, partial, flags);
  scan_partials_launch(env, partial, nb, &flags->scalar[0]);
  Flags h{};
  if (!read_flags(env, flags, &h)) return env.status;
  if (flag_status(h) != US_OK) return flag_status(h);
  const int64_t nblk = h.scalar[0], bsz = plan.bh * plan.bw;
  if (nblk * bsz >= (1ll << 31)) return US_ERR_OVERFLOW;
  const bool bdia = plan.pattern == P_BDIA;
  us_formatted *f = new us_formatted();
  f->desc = desc; f->pattern = plan.pattern;
  f->nrows = nrows; f->ncols = ncols; f->nnz = n;
  f->nlevels = bdia ? 3 : 4;
  f->level[0].size = nbr;
  f->level[1].ptr = env.owned<int32_t>(nbr + 1); f->level[1].nptr = nbr + 1;
  f->level[1].idx = env.owned<int32_t>(nblk); f->level[1].nidx = nblk;
  f->level[2].size = plan.bh;
  if (!bdia) f->level[3].size = plan.bw;
  f->val = env.owned<float>(nblk * bsz); f->nval = nblk * bsz;
  f->nmajor = nbr; f->bh = plan.bh; f->bw = plan.bw; f->nblk = nblk;
  int32_t *blk_row = env.temp<int32_t>(nblk);
  if (!env.ok()) { free_formatted(env, f); return env.status; }
  fill_u32(env, (uint32_t *)f->val, nblk * bsz, 0u);
  if (n > 0)
    US_LAUNCH(env, "bcsr_emit", 12.0 * n + 4.0 * n, bcsr_emit_kernel, nb, BE_T, skey, sval, n, ks,
              (int32_t)(bdia ? nrows - 1 : 0), (const uint32_t *)partial, blk_row, f->level[1].idx, f->val);
  lower_bound_ptr(env, blk_row, nblk, nbr, f->level[1].ptr);
  env.sync();
  if (!env.ok()) { free_formatted(env, f); return env.status; }
  *out = f;
  return US_OK;
}

static us_status convert_blocked(Env &env, const us_coo &coo, const Plan &plan, const us_format_desc &desc,
                                 Flags *flags, us_formatted **out) {
  const int64_t n = coo.nnz;
  const KeySpec ks = blocked_keyspec(plan, coo.nrows, coo.ncols);
  if (ks.total_bits > 64) return US_ERR_OVERFLOW;
  uint64_t *skey = env.temp<uint64_t>(n);
  float *sval = env.temp<float>(n);
  if (!env.ok()) return env.status;
  SortOut so{};
  so.key64 = skey; so.val = sval;
  sort_coo(env, coo.row, coo.col, coo.val, n, ks, so, flags);
  return emit_blocked(env, plan, desc, coo.nrows, coo.ncols, ks, skey, sval, n, flags, out);
}

// CSB (Section 2.1: a dense collection of blocks stored compressed): the entries in BCSR tuple order, a ptr
// over all blocks of the dense grid, and the two in-block indices of every entry.
__global__ __launch_bounds__(256) void csb_unpack_kernel(const uint64_t *key, int64_t n, KeySpec ks, int64_t nbc,
                                                        int32_t *blk, int32_t *in_row, int32_t *in_col, Flags *flags) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const uint64_t k = key[i];
  if (i > 0 && key[i - 1] == k) flags->duplicate = 1;
  const uint64_t bk = k >> (ks.ih_bits + ks.iw_bits);
  blk[i] = (int32_t)((int64_t)(bk >> ks.b_bits) * nbc + (int64_t)(bk & ((1ull << ks.b_bits) - 1)));
  in_row[i] = (int32_t)((k >> ks.iw_bits) & ((1ull << ks.ih_bits) - 1));
  in_col[i] = (int32_t)(k & ((1ull << ks.iw_bits) - 1));
}

static us_status convert_csb(Env &env, const us_coo &coo, const Plan &plan, const us_format_desc &desc, Flags *flags,
                             us_formatted **out) {
  const int64_t n = coo.nnz;
  const int64_t nbr = ceil_div<int64_t>(coo.nrows, plan.bh), nbc = ceil_div<int64_t>(coo.ncols, plan.bw);
  if (nbr * nbc + 1 >= (1ll << 31)) return US_ERR_OVERFLOW;
  Plan pk = plan; pk.pattern = P_BCSR;   // same target tuple as BCSR
  const KeySpec ks = blocked_keyspec(pk, coo.nrows, coo.ncols);
  uint64_t *skey = env.temp<uint64_t>(n);
  int32_t *blk = env.temp<int32_t>(n);
  us_formatted *f = new us_formatted();
  f->desc = desc; f->pattern = P_CSB;
  f->nrows = coo.nrows; f->ncols = coo.ncols; f->nnz = n;
  f->nlevels = 4;
  f->level[0].size = nbr; f->level[1].size = nbc;
  f->level[2].ptr = env.owned<int32_t>(nbr * nbc + 1); f->level[2].nptr = nbr * nbc + 1;
  f->level[2].idx = env.owned<int32_t>(n); f->level[2].nidx = n;
  f->level[3].idx = env.owned<int32_t>(n); f->level[3].nidx = n;
  f->val = env.owned<float>(n); f->nval = n;
  f->nmajor = nbr * nbc; f->bh = plan.bh; f->bw = plan.bw; f->nblk = nbr * nbc;
  if (!env.ok()) { free_formatted(env, f); return env.status; }
  SortOut so{};
  so.key64 = skey; so.val = f->val;
  sort_coo(env, coo.row, coo.col, coo.val, n, ks, so, flags);
  if (n > 0)
    US_LAUNCH(env, "csb_unpack", 20.0 * n, csb_unpack_kernel, ceil_div<int64_t>(n, 256), 256, (const uint64_t *)skey, n, ks,
              nbc, blk, f->level[2].idx, f->level[3].idx, flags);
  lower_bound_ptr(env, blk, n, nbr * nbc, f->level[2].ptr);
  Flags h{};
  if (!read_flags(env, flags, &h)) { free_formatted(env, f); return env.status; }
  if (flag_status(h) != US_OK) { free_formatted(env, f); return flag_status(h); }
  *out = f;
  return US_OK;
}

// ------------------------------------------------------------------ CISR-plus (Section 7.2.4)
// The indirect level of its encoding is three queries over the rows: sum (entries per row), reorder (most
// entries first, equal rows by ascending index) and schedule (the k-th row of that order is dealt to partition
// k mod P).  After the (row, col) sort these are row-level steps: the stored rows are compacted in row order,
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
#pragma unroll
  for (int k = 0; k < CM_IPT; ++k) {
    const int64_t e = e0 + k * CM_T + threadIdx.x;
    if (e >= n) continue;
    int lo = 0, hi = cnt - 1;   // s_ptr[lo] <= e < s_ptr[hi] throughout
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (s_ptr[mid] <= e) lo = mid; else hi = mid;
    }
    int64_t src = (int64_t)s_src[lo] + (e - s_ptr[lo]);
    src = src < 0 ? 0 : (src >= n ? n - 1 : src);
    col_out[e] = minor[src];
    val_out[e] = val[src];
  }
}

static us_status convert_cisr(Env &env, const us_coo &coo, const Plan &plan, const us_format_desc &desc, Flags *flags,
                              us_formatted **out) {
  const int64_t n = coo.nnz, nrows = coo.nrows, nparts = plan.bh;
  int32_t *major = env.temp<int32_t>(n), *minor = env.temp<int32_t>(n);
  float *val = env.temp<float>(n);
  int32_t *ptr = env.temp<int32_t>(nrows + 1), *flag = env.temp<int32_t>(nrows), *pos = env.temp<int32_t>(nrows);
  if (!env.ok()) return env.status;
  SortOut so{};
  so.major = major; so.minor = minor; so.val = val;
  const bool checked = sort_coo(env, coo.row, coo.col, coo.val, n, rowcol_keyspec(coo, false), so, flags);
  if (n >= nrows) {
    group_ptr_unique(env, major, minor, n, nrows, ptr, !checked, flags);
  } else {
    if (!checked && n > 1)
      US_LAUNCH(env, "check_unique", 8.0 * n, check_unique_unpacked_kernel, ceil_div<int64_t>(n, 256), 256,
                (const int32_t *)major, (const int32_t *)minor, n, flags);
    lower_bound_ptr(env, major, n, nrows, ptr);
  }
  US_LAUNCH(env, "nonempty_flag", 8.0 * nrows, nonempty_flag_kernel, ceil_div<int64_t>(nrows, 256), 256,
            (const int32_t *)ptr, nrows, flag);
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

// ------------------------------------------------------------------ convert
static us_status validate_coo(const us_coo &coo) {
  if (coo.nrows <= 0 || coo.ncols <= 0 || coo.nnz < 0) return US_ERR_SHAPE;
  if (coo.nrows >= (1ll << 31) || coo.ncols >= (1ll << 31) || coo.nnz >= (1ll << 31)) return US_ERR_OVERFLOW;
  if (coo.nnz > 0 && (!coo.row || !coo.col || !coo.val)) return US_ERR_NULL;
  return US_OK;
}

static Flags *new_flags(Env &env) {
  Flags *flags = env.temp<Flags>(1);
  fill_u32(env, (uint32_t *)flags, sizeof(Flags) / 4, 0u);
  return flags;
}

static us_status convert_with_plan(Env &env, const us_coo &coo, const Plan &plan, const us_format_desc &desc,
                                   us_formatted **out) {
  const bool by_sort = plan.pattern == P_COO || plan.pattern == P_CSR || plan.pattern == P_DCSR ||
                       plan.pattern == P_ELL || plan.pattern == P_CISR;
  if (by_sort) env.reserve(sort_temp_bytes(coo.nnz) + 4 * Env::granule(sizeof(Flags)));   // flags and the sort's buffers together
  Flags *flags = new_flags(env);
  if (!env.ok()) return env.status;
  if (plan.pattern == P_DIA) return convert_dia(env, coo, plan, desc, flags, out);
  if (plan.pattern == P_BCSR || plan.pattern == P_BDIA) return convert_blocked(env, coo, plan, desc, flags, out);
  if (plan.pattern == P_CSB) return convert_csb(env, coo, plan, desc, flags, out);
  if (plan.pattern == P_CISR) return convert_cisr(env, coo, plan, desc, flags, out);
  // COO / CSR / DCSR / ELL: sort by (major, minor), then build
  const int64_t n = coo.nnz;
  int32_t *major = env.owned<int32_t>(n), *minor = env.owned<int32_t>(n);
  float *val = env.owned<float>(n);
  if (!env.ok()) { env.free_raw(major); env.free_raw(minor); env.free_raw(val); return env.status; }
  SortOut so{};
  so.major = major; so.minor = minor; so.val = val;
  const bool checked = sort_coo(env, coo.row, coo.col, coo.val, n, rowcol_keyspec(coo, plan.swapped), so, flags);
  return build_from_sorted(env, plan, desc, coo.nrows, coo.ncols, n, major, minor, val, flags, !checked, out);
}

us_status convert_impl(Env &env, const us_coo &coo, const us_format_desc &desc, us_formatted **out) {
  *out = nullptr;
  us_status s = validate_coo(coo);
  if (s != US_OK) return s;
  Plan plan;
  if (!match_desc(desc, &plan)) return US_ERR_UNSUPPORTED_DESC;
  if (plan.pattern == P_ELL && plan.swapped) return US_ERR_UNSUPPORTED_DESC;
  s = convert_with_plan(env, coo, plan, desc, out);
  if (s == US_OK && !env.ok()) s = env.status;
  if (s != US_OK && *out) { free_formatted(env, *out); *out = nullptr; }
  return s;
}

// ------------------------------------------------------------------ formatted -> COO (the hub of Section 5.2)
// Every format whose encoding uses only direct index maps and mutation primitives converts
// back to COO (reversibility, Section 5.2): Split re-expands a ptr level into one parent index
// per child, Trim drops the padding of dense inner levels, TileUnion re-joins (d/b, d%b), and
// the inverse index map restores (d0, d1).  ELL is read back as well (its column level stores
// d1).  Slots of dense levels that hold +-0.0 are padding and are dropped.
// Step 1 flags the slots that carry an entry, a scan gives their positions, step 2 writes.
struct SrcView {
  int pattern, swapped;
  int64_t nrows, ncols, nslots, nmajor, bh, bw;
  const int32_t *ptr, *idx, *idx0;  // ptr/idx of the compressed level; idx0: stored rows (DCSR) / offsets (DIA)
  const float *val;
};

__device__ __forceinline__ bool slot_entry(const SrcView &v, int64_t s, int32_t *r, int32_t *c, float *x) {
  int64_t a, b;  // major, minor logical indices before undoing a swap
  float val = v.val[s];
  switch (v.pattern) {
    case P_COO: a = v.idx0[s]; b = v.idx[s]; break;
    case P_CSR: a = parent_of(v.ptr, v.nmajor, s); b = v.idx[s]; break;
    case P_DCSR: a = v.idx0[parent_of(v.ptr, v.nmajor, s)]; b = v.idx[s]; break;
    case P_DIA: {
      const int64_t L = v.swapped ? v.ncols : v.nrows, k = s / L, i = s - k * L, off = v.idx0[k];
      const int64_t row = v.swapped ? i - off : i, col = v.swapped ? i : i + off;
      if (val == 0.f || row < 0 || row >= v.nrows || col < 0 || col >= v.ncols) return false;
      *r = (int32_t)row; *c = (int32_t)col; *x = val;
      return true;
    }
    case P_BCSR: {
      const int64_t bsz = v.bh * v.bw, blk = s / bsz, in = s - blk * bsz, ri = in / v.bw, ci = in - ri * v.bw;
      const int64_t row = parent_of(v.ptr, v.nmajor, blk) * v.bh + ri, col = (int64_t)v.idx[blk] * v.bw + ci;
      if (val == 0.f || row >= v.nrows || col >= v.ncols) return false;
      *r = (int32_t)row; *c = (int32_t)col; *x = val;
      return true;
    }
    case P_CSB: {    // TileUnion: d0 = e0*bh + e2, d1 = e1*bw + e3 with (e0, e1) = block id / and % blocks per block row
      const int64_t blk = parent_of(v.ptr, v.nmajor, s), nbc = (v.ncols + v.bw - 1) / v.bw;
      a = (blk / nbc) * v.bh + v.idx0[s]; b = (blk % nbc) * v.bw + v.idx[s];
      break;
    }
    case P_BDIA: {   // inverse map of Figure 9: d0 = e0*b + e2, d1 = e1 + d0
      const int64_t node = s / v.bh, ri = s - node * v.bh;
      const int64_t row = parent_of(v.ptr, v.nmajor, node) * v.bh + ri, col = row + v.idx[node];
      if (val == 0.f || row >= v.nrows || col < 0 || col >= v.ncols) return false;
      *r = (int32_t)row; *c = (int32_t)col; *x = val;
      return true;
    }
    case P_ELL: {
      const int64_t k = s / v.nrows, i = s - k * v.nrows;
      if (v.idx[s] < 0 || val == 0.f) return false;
      *r = (int32_t)i; *c = v.idx[s]; *x = val;
      return true;
    }
    default: return false;
  }
  *r = (int32_t)(v.swapped ? b : a); *c = (int32_t)(v.swapped ? a : b); *x = val;
  return true;
}

__global__ __launch_bounds__(256) void expand_flag_kernel(SrcView v, int32_t *flag) {
  int64_t s = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (s >= v.nslots) return;
  int32_t r, c; float x;
  flag[s] = slot_entry(v, s, &r, &c, &x) ? 1 : 0;
}
__global__ __launch_bounds__(256) void expand_write_kernel(SrcView v, const int32_t *flag, const int32_t *pos,
                                                          int32_t *row, int32_t *col, float *val) {
  int64_t s = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (s >= v.nslots || !flag[s]) return;
  int32_t r, c; float x;
  slot_entry(v, s, &r, &c, &x);
  row[pos[s]] = r; col[pos[s]] = c; val[pos[s]] = x;
}

us_status convert_formatted_impl(Env &env, const us_formatted &src, const us_format_desc &desc, us_formatted **out) {
  *out = nullptr;
  Plan plan;
  if (!match_desc(desc, &plan)) return US_ERR_UNSUPPORTED_DESC;
  if (plan.pattern == P_ELL && plan.swapped) return US_ERR_UNSUPPORTED_DESC;
  SrcView v{};
  v.pattern = src.pattern; v.swapped = src.swapped ? 1 : 0;
  v.nrows = src.nrows; v.ncols = src.ncols; v.nslots = src.nval; v.nmajor = src.nmajor;
  v.bh = src.bh; v.bw = src.bw; v.val = src.val;
  switch (src.pattern) {
    case P_COO: v.idx0 = src.level[0].idx; v.idx = src.level[1].idx; break;
    case P_CSR: v.ptr = src.level[1].ptr; v.idx = src.level[1].idx; break;
    case P_DCSR: v.idx0 = src.level[0].idx; v.ptr = src.level[1].ptr; v.idx = src.level[1].idx; break;
    case P_DIA: v.idx0 = src.level[0].idx; break;
    case P_BCSR:
    case P_BDIA: v.ptr = src.level[1].ptr; v.idx = src.level[1].idx; break;
    case P_ELL: v.idx = src.level[2].idx; break;
    case P_CSB: v.ptr = src.level[2].ptr; v.idx0 = src.level[2].idx; v.idx = src.level[3].idx; break;
    case P_CISR:   // below the partition level it reads like DCSR: stored rows, ptr over them, columns
      v.pattern = P_DCSR; v.idx0 = src.level[1].idx; v.ptr = src.level[2].ptr; v.idx = src.level[2].idx; break;
    default: return US_ERR_FORMAT_MISMATCH;
  }
  const int64_t ns = v.nslots;
  Flags *flags = new_flags(env);
  int32_t *flag = env.temp<int32_t>(ns), *pos = env.temp<int32_t>(ns);
  if (!env.ok()) return env.status;
  if (ns > 0)
    US_LAUNCH(env, "expand_flag", 8.0 * ns, expand_flag_kernel, ceil_div<int64_t>(ns, 256), 256, v, flag);
  exclusive_scan_i32(env, flag, pos, ns, &flags->scalar[0]);
  Flags h{};
  if (!read_flags(env, flags, &h)) return env.status;
  const int64_t n = ns > 0 ? h.scalar[0] : 0;
  CooLists l = alloc_lists(env, n);
  us_status st = env.status;
  if (st == US_OK && ns > 0)
    US_LAUNCH(env, "expand_write", 12.0 * ns + 12.0 * n, expand_write_kernel, ceil_div<int64_t>(ns, 256), 256, v,
              (const int32_t *)flag, (const int32_t *)pos, l.r, l.c, l.v);
  if (st == US_OK) st = env.status;
  if (st == US_OK) {
    us_coo coo{src.nrows, src.ncols, n, l.r, l.c, l.v};
    st = convert_with_plan(env, coo, plan, desc, out);
  }
  env.sync();
  free_lists(env, l);
  if (st == US_OK && !env.ok()) st = env.status;
  if (st != US_OK && *out) { free_formatted(env, *out); *out = nullptr; }
  return st;
}

// ------------------------------------------------------------------ decompose
__global__ __launch_bounds__(256) void row_len_kernel(const int32_t *ptr, int64_t n, uint32_t *len) {
  int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (g < n) len[g] = (uint32_t)(ptr[g + 1] - ptr[g]);
}
__global__ void pick_kernel(const uint32_t *sorted, int64_t at, int32_t *out) { *out = (int32_t)sorted[at]; }

// K_dev != null: the cut is still on the device (the percentile picked just before)
__global__ __launch_bounds__(256) void clipped_len_kernel(const int32_t *ptr, int64_t n, int64_t K, const int32_t *K_dev,
                                                         int32_t *out) {
  int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (K_dev) K = *K_dev;
  if (g < n) { int64_t l = ptr[g + 1] - ptr[g]; out[g] = (int32_t)(l < K ? l : K); }
}

// stable split of the sorted list by rank-in-row: rank < K -> part A, else part B.  (Equal neighbours have
// been looked for before: the two copies of a coordinate may end up in different parts.)
// ell_col != null: part A is an ELL slab of width ell_width over nrows rows and takes its entries directly
// (slot rank * nrows + row) instead of the list (ar, ac, av).
__global__ __launch_bounds__(256) void rank_split_kernel(const int32_t *major, const int32_t *minor, const float *val,
                                                        const int32_t *ptr, const int32_t *ptr_a, int64_t n,
                                                        int64_t K, int32_t *ar, int32_t *ac, float *av, int32_t *br,
                                                        int32_t *bc, float *bv, int32_t *ell_col, float *ell_val,
                                                        int64_t ell_width, int64_t nrows, Flags *flags) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const int32_t r = major[i], c = minor[i];
  int64_t rank = i - ptr[r];
  if (rank < K) {
    if (ell_col) {
      if (rank >= ell_width) { flags->ell_overflow = 1; return; }
      const int64_t slot = rank * nrows + r;
      ell_col[slot] = c; ell_val[slot] = val[i];
    } else {
      int64_t p = ptr_a[r] + rank;
      ar[p] = r; ac[p] = c; av[p] = val[i];
    }
  } else {
    int64_t p = (int64_t)(ptr[r] - ptr_a[r]) + (rank - K);
    br[p] = r; bc[p] = c; bv[p] = val[i];
  }
}

static bool row_major_family(const Plan &p) {
  return !p.swapped && (p.pattern == P_COO || p.pattern == P_CSR || p.pattern == P_DCSR || p.pattern == P_ELL);
}

static us_status decompose_sum(Env &env, const us_coo &coo, const Plan &pa, const us_format_desc &da, const Plan &pb,
                               const us_format_desc &db, const us_predicate &pred, int gkind, us_formatted **oa,
                               us_formatted **ob) {
  Flags *flags = new_flags(env);
  if (!env.ok()) return env.status;
  GroupCounts g = group_flags(env, coo, gkind, pred.kind, pred.num, pred.den, pred.abs, flags);
  if (!env.ok()) return env.status;
  const int64_t n = coo.nnz;
  CooLists la, lb;
  int64_t na = 0, nb = 0;
  us_status st;
  if (gkind == G_DIAG && pa.pattern == P_DIA) {
    // part A goes straight into the slab while part B is collected, in one pass over the input
    st = dia_from_flags(env, coo, pa, da, flags, g.flag, oa, &lb, &nb);
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
  env.sync();
  free_lists(env, la);
  free_lists(env, lb);
  return st;
}

static us_status decompose_rank(Env &env, const us_coo &coo, const Plan &pa, const us_format_desc &da, const Plan &pb,
                                const us_format_desc &db, const us_predicate &pred, us_formatted **oa,
                                us_formatted **ob) {
  Flags *flags = new_flags(env);
  const int64_t n = coo.nnz, nrows = coo.nrows;
  int32_t *major = env.temp<int32_t>(n), *minor = env.temp<int32_t>(n);
  float *val = env.temp<float>(n);
  int32_t *ptr = env.temp<int32_t>(nrows + 1), *ptr_a = env.temp<int32_t>(nrows + 1), *clip = env.temp<int32_t>(nrows + 1);
  if (!env.ok()) return env.status;
  SortOut so{};
  so.major = major; so.minor = minor; so.val = val;
  const bool checked = sort_coo(env, coo.row, coo.col, coo.val, n, rowcol_keyspec(coo, false), so, flags);
  if (n >= nrows) {
    group_ptr_unique(env, major, minor, n, nrows, ptr, !checked, flags);
  } else {
    if (!checked && n > 1)
      US_LAUNCH(env, "check_unique", 8.0 * n, check_unique_unpacked_kernel, ceil_div<int64_t>(n, 256), 256,
                (const int32_t *)major, (const int32_t *)minor, n, flags);
    lower_bound_ptr(env, major, n, nrows, ptr);
  }
  Flags h{};
  int64_t K = pred.abs;
  if (pred.kind == US_P_RANK_LT_PERCENTILE) {
    // nearest-rank percentile of the row lengths over all rows: sort the lengths, pick one
    uint32_t *len = env.temp<uint32_t>(nrows), *slen = env.temp<uint32_t>(nrows);
    if (!env.ok()) return env.status;
    US_LAUNCH(env, "row_len", 8.0 * nrows, row_len_kernel, ceil_div<int64_t>(nrows, 256), 256, (const int32_t *)ptr,
              nrows, len);
    const int64_t maxlen = n < coo.ncols ? n : coo.ncols;
    sort_u32(env, len, nrows, bits_for((uint64_t)maxlen), slen, flags);
    int64_t k = (pred.num * nrows + pred.den - 1) / pred.den;
    if (k < 1) k = 1;
    if (k > nrows) k = nrows;
    US_LAUNCH(env, "pick", 8.0, pick_kernel, 1, 1, (const uint32_t *)slen, k - 1, &flags->scalar[2]);
  }
  // the cut K (if picked above), the size of part A and the longest row all come back in one read of the flags
  const bool by_percentile = pred.kind == US_P_RANK_LT_PERCENTILE;
  US_LAUNCH(env, "clipped_len", 8.0 * nrows, clipped_len_kernel, ceil_div<int64_t>(nrows, 256), 256,
            (const int32_t *)ptr, nrows, K, (const int32_t *)(by_percentile ? &flags->scalar[2] : nullptr), clip);
  exclusive_scan_i32(env, clip, ptr_a, nrows, &flags->scalar[1]);
  US_LAUNCH(env, "max_row_len", 4.0 * nrows, max_len_kernel, one_counter_grid(nrows, 256), 256, (const int32_t *)ptr,
            nrows, &flags->scalar[3]);
  if (!read_flags(env, flags, &h)) return env.status;
  if (flag_status(h) != US_OK) return flag_status(h);
  if (by_percentile) K = h.scalar[2];
  const int64_t longest = h.scalar[3];
  const int64_t na = h.scalar[1], nb = n - na;
  // part A as row-major ELL: the split writes its slab directly (its rows hold min(length, K) entries, which
  // gives the automatic width); any other format gets a sorted list first
  us_formatted *ell = nullptr;
  int64_t ell_width = 0;
  if (pa.pattern == P_ELL && !pa.swapped) {
    ell_width = pa.ell_width > 0 ? pa.ell_width : (longest < K ? longest : K);
    if (ell_width * nrows >= (1ll << 31)) return US_ERR_OVERFLOW;
    ell = new_empty_ell(env, da, nrows, coo.ncols, na, ell_width);
    if (!ell) return env.status;
  }
  CooLists la = ell ? CooLists() : alloc_lists(env, na), lb = alloc_lists(env, nb);
  us_status st = env.status;
  if (st == US_OK && n > 0) {
    US_LAUNCH(env, "rank_split", 16.0 * n + 12.0 * n, rank_split_kernel, ceil_div<int64_t>(n, 256), 256,
              (const int32_t *)major, (const int32_t *)minor, (const float *)val, (const int32_t *)ptr,
              (const int32_t *)ptr_a, n, K, la.r, la.c, la.v, lb.r, lb.c, lb.v,
              ell ? ell->level[2].idx : (int32_t *)nullptr, ell ? ell->val : (float *)nullptr, ell_width, nrows, flags);
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
  const bool direct = pa.pattern == pg.pattern && pa.bh == pg.bh && pa.bw == pg.bw;
  uint64_t *skey = env.temp<uint64_t>(n);
  float *sval = env.temp<float>(n);
  int32_t *head = env.temp<int32_t>(n), *pos = env.temp<int32_t>(n), *start = env.temp<int32_t>(n + 1);
  int32_t *keep = env.temp<int32_t>(n), *pos_a = env.temp<int32_t>(n);
  if (!env.ok()) return env.status;
  int64_t na = 0;
  if (n > 0) {
    SortOut so{};
    so.key64 = skey; so.val = sval;
    sort_coo(env, coo.row, coo.col, coo.val, n, ks, so, flags);
    const int64_t g = ceil_div<int64_t>(n, 256);
    US_LAUNCH(env, "node_head", 12.0 * n, node_head_kernel, g, 256, (const uint64_t *)skey, n, inner_bits, head, flags);
    exclusive_scan_i32(env, head, pos, n, &flags->scalar[0]);
    US_LAUNCH(env, "node_start", 12.0 * n, node_start_kernel, g, 256, (const int32_t *)head, (const int32_t *)pos, n,
              start);
    US_LAUNCH(env, "node_keep", 16.0 * n, node_keep_kernel, g, 256, (const int32_t *)head, (const int32_t *)pos,
              (const int32_t *)start, n, thld, keep);
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
    // of the BELL/COO case study (Section 7.2.2: "non-zero threshold within each block")
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
