// COO -> target format.  Host side: match the format encoding against the supported patterns and infer which
// size/ptr/idx/val arrays exist (Section 5.1); device side: the runtime effect of the conversion operators of
// Table 2 for the layouts that follow from a (major, minor) sort -- Merge (head flags + scan -> ptr), Fill / Trim
// of the major level, Enumerate (rank in row) -- and the way back from any layout to COO (Section 5.2).
// The other families of layouts live in sum_query.hip (DIA), blocked.hip (BCSR, BDIA, CSB) and cisr.hip.
#include "convert_internal.h"
#include "device.h"

#include <atomic>
#include <mutex>

namespace us {

// ------------------------------------------------------------------ descriptor matching (host)

bool aff(const us_expr &e, int c0, int c1) {
  return e.kind == US_E_AFFINE && e.c0 == c0 && e.c1 == c1 && e.c == 0;
}
bool tile(const us_expr &e, int kind, int dim, int64_t *f, int64_t max_factor) {
  if (e.kind != kind || e.c != 0 || e.factor < 1 || e.factor > max_factor) return false;
  if (!(e.c0 == (dim == 0) && e.c1 == (dim == 1))) return false;
  *f = e.factor;
  return true;
}

bool match_desc(const us_format_desc &d, Plan *p) {
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
  if (d.nlevels == 5) {
    const us_expr &e = d.level[0];
    int64_t f1, f2, f3, f4;
    if (e.kind == US_E_INDIRECT_ENUM && e.c0 == 1 && e.c1 == 0 && e.c == 0 && tile(d.level[1], US_E_DIV, 0, &f1) &&
        tile(d.level[2], US_E_DIV, 1, &f2) && tile(d.level[3], US_E_MOD, 0, &f3) && tile(d.level[4], US_E_MOD, 1, &f4) &&
        f1 == f3 && f2 == f4 && e.factor == f1 && e.factor2 == f2 && S == 0 && E == 0 && m == 1 && d.ell_width >= 0) {
      p->pattern = P_BELL; p->bh = f1; p->bw = f2; p->ell_width = d.ell_width;
      return true;
    }
    return false;
  }
  if (d.nlevels == 3) {
    const us_expr &e = d.level[0];
    if (e.kind == US_E_INDIRECT_ENUM && e.c0 == 1 && e.c1 == 0 && e.c == 0 && e.factor <= 1 && e.factor2 <= 1 &&
        aff(d.level[1], 1, 0) && aff(d.level[2], 0, 1) && S == 0 && E == 0 && m == 1 && d.ell_width >= 0) {
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

// Trim of the major level (DCSR): the groups that have children, in order, with where their children start.
// Counted per tile, the tile counts scanned by one workgroup (scan_partials_launch, which leaves the total, nnr, in
// device memory), then every tile numbers its own groups and writes them: no flag or position arrays in between.
// The arrays hold `cap` groups, which a valid input never exceeds.
constexpr int NE_T = 256, NE_IPT = 8, NE_TILE = NE_T * NE_IPT;
__global__ __launch_bounds__(NE_T) void nonempty_count_kernel(const int32_t *ptr, int64_t n, uint32_t *partial) {
  __shared__ uint32_t s_wave[NE_T / 64 + 1];
  const int64_t base = (int64_t)blockIdx.x * NE_TILE;
  uint32_t s = 0;
#pragma unroll
  for (int k = 0; k < NE_IPT; ++k) {
    const int64_t g = base + k * NE_T + threadIdx.x;
    if (g < n) s += ptr[g + 1] > ptr[g] ? 1u : 0u;
  }
  uint32_t total;
  block_exclusive_sum<NE_T>(s, s_wave, &total);
  if (threadIdx.x == 0) partial[blockIdx.x] = total;
}
__global__ __launch_bounds__(NE_T) void nonempty_compact_kernel(const int32_t *ptr, int64_t n, const uint32_t *partial,
                                                               const int32_t *nnr_dev, int64_t cap, int32_t nnz,
                                                               int32_t *idx0, int32_t *ptr1) {
  __shared__ uint32_t s_wave[NE_T / 64 + 1];
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    const int64_t nnr = *nnr_dev;
    ptr1[nnr >= 0 && nnr < cap ? nnr : cap] = nnz;
  }
  // a thread owns NE_IPT consecutive groups, so its numbers are consecutive too
  const int64_t g0 = (int64_t)blockIdx.x * NE_TILE + (int64_t)threadIdx.x * NE_IPT;
  int32_t p[NE_IPT + 1];
#pragma unroll
  for (int k = 0; k <= NE_IPT; ++k) p[k] = g0 + k <= n ? ptr[g0 + k] : 0;
  uint32_t s = 0;
#pragma unroll
  for (int k = 0; k < NE_IPT; ++k) s += (g0 + k < n && p[k + 1] > p[k]) ? 1u : 0u;
  uint32_t total;
  int64_t at = (int64_t)block_exclusive_sum<NE_T>(s, s_wave, &total) + partial[blockIdx.x];
#pragma unroll
  for (int k = 0; k < NE_IPT; ++k)
    if (g0 + k < n && p[k + 1] > p[k]) {
      if (at < cap) { idx0[at] = (int32_t)(g0 + k); ptr1[at] = p[k]; }
      ++at;
    }
}

// Kernels that end with one atomic per workgroup on a single counter run on at most ONE_COUNTER_GRID
// workgroups (grid-stride loops): same-address device atomics cost ~20 ns apiece on this part, so
// thousands of them would outlast the kernel's real work.

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

// ELL: entry i of the sorted list sits in slot rank = i - ptr[row] of its row (the enum query).  The slab is
// slot-major (col/val[slot * nrows + row]) while the list is row-major: a wavefront takes 64 rows and moves them
// EF_SLOTS slots at a time through LDS -- in, EF_RPL rows per load instruction (EF_SLOTS consecutive entries of a
// row each); out, a lane per row, 256 contiguous bytes per slot and array, pads included (no separate fill).
constexpr int EF_ROWS = 64, EF_SLOTS = 16, EF_PITCH = EF_SLOTS + 1, EF_RPL = 64 / EF_SLOTS;   // rows per load instruction
// clip >= 0: only the first `clip` entries of a row belong to this layout (the rank split of a decomposition).
__global__ __launch_bounds__(64) void ell_fill_kernel(const int32_t *minor, const float *val, const int32_t *ptr,
                                                     int64_t nrows, int64_t K, int64_t clip, int32_t *ecol, float *eval,
                                                     Flags *flags) {
  __shared__ int32_t s_col[EF_ROWS * EF_PITCH];
  __shared__ float s_val[EF_ROWS * EF_PITCH];
  const int lane = threadIdx.x;
  const int64_t r = (int64_t)blockIdx.x * EF_ROWS + lane;
  const int32_t start = r < nrows ? ptr[r] : 0;
  int32_t len = r < nrows ? ptr[r + 1] - start : 0;
  if (clip >= 0 && len > clip) len = (int32_t)clip;
  if (len > K) flags->ell_overflow = 1;
  for (int64_t k0 = 0; k0 < K; k0 += EF_SLOTS) {
    // all loads of the chunk first (32 in flight), then the LDS writes: one trip to memory per chunk
    int32_t cv[EF_ROWS / EF_RPL];
    float vv[EF_ROWS / EF_RPL];
#pragma unroll
    for (int j = 0; j < EF_ROWS; j += EF_RPL) {
      const int row = j + lane / EF_SLOTS, kk = lane % EF_SLOTS;
      const int32_t st = __shfl(start, row), ln = __shfl(len, row);
      const bool has = k0 + kk < ln;
      cv[j / EF_RPL] = has ? minor[(int64_t)st + k0 + kk] : -1;
      vv[j / EF_RPL] = has ? val[(int64_t)st + k0 + kk] : 0.f;
    }
#pragma unroll
    for (int j = 0; j < EF_ROWS; j += EF_RPL) {
      const int row = j + lane / EF_SLOTS, kk = lane % EF_SLOTS;
      s_col[row * EF_PITCH + kk] = cv[j / EF_RPL];
      s_val[row * EF_PITCH + kk] = vv[j / EF_RPL];
    }
    __syncthreads();
    if (r < nrows) {
      const int nk = (int)min<int64_t>(EF_SLOTS, K - k0);
      for (int kk = 0; kk < nk; ++kk) {
        ecol[(k0 + kk) * nrows + r] = s_col[lane * EF_PITCH + kk];
        eval[(k0 + kk) * nrows + r] = s_val[lane * EF_PITCH + kk];
      }
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------ launches shared with the other conversion files
void check_unique(Env &env, const int32_t *major, const int32_t *minor, int64_t n, Flags *flags) {
  if (n > 1)
    US_LAUNCH(env, "check_unique", 8.0 * n, check_unique_unpacked_kernel, ceil_div<int64_t>(n, 256), 256, major, minor, n,
              flags);
}
void nonempty_flags(Env &env, const int32_t *ptr, int64_t n, int32_t *flag) {
  US_LAUNCH(env, "nonempty_flag", 8.0 * n, nonempty_flag_kernel, ceil_div<int64_t>(n, 256), 256, ptr, n, flag);
}
void max_group_len(Env &env, const int32_t *ptr, int64_t n, int32_t *out_max) {
  US_LAUNCH(env, "max_row_len", 4.0 * n, max_len_kernel, one_counter_grid(n, 256), 256, ptr, n, out_max);
}
// ptr over the groups of a list sorted by (major, minor), with the duplicate check if asked for: one pass over
// the entries gives both; with fewer entries than groups the runs of empty groups are long and a binary
// search per group is the quicker way to ptr
void sorted_ptr(Env &env, const int32_t *major, const int32_t *minor, int64_t n, int64_t ngroups, int32_t *ptr,
                bool check_dups, Flags *flags) {
  if (n >= ngroups) {
    group_ptr_unique(env, major, minor, n, ngroups, ptr, check_dups, flags);
  } else {
    if (check_dups) check_unique(env, major, minor, n, flags);
    lower_bound_ptr(env, major, n, ngroups, ptr);
  }
}

// ------------------------------------------------------------------ helpers (host)
// Read-backs land in pinned host memory: a copy into pageable memory kept the GPU waiting ~6 us longer (24 against
// 18 us from the end of the last kernel to the start of the next launch).  One page of slots for the process,
// allocated on first use and kept; a call that finds none free (or no pinned memory) copies to its own variable.
namespace {
constexpr int RB_SLOTS = 32;
Flags *g_rb_page = nullptr;
std::once_flag g_rb_once;
std::atomic<uint32_t> g_rb_busy{0};

Flags *readback_slot(int *slot) {
  std::call_once(g_rb_once, [] {
    void *p = nullptr;
    if (hipHostMalloc(&p, RB_SLOTS * sizeof(Flags), hipHostMallocPortable) == hipSuccess) g_rb_page = static_cast<Flags *>(p);
    else (void)hipGetLastError();   // not an error of the call: it falls back to pageable memory
  });
  if (!g_rb_page) return nullptr;
  uint32_t busy = g_rb_busy.load(std::memory_order_relaxed);
  while (busy != 0xFFFFFFFFu) {
    const int s = __builtin_ctz(~busy);
    if (g_rb_busy.compare_exchange_weak(busy, busy | (1u << s), std::memory_order_acquire)) {
      *slot = s;
      return g_rb_page + s;
    }
  }
  return nullptr;
}
}  // namespace

bool read_flags(Env &env, Flags *dev, Flags *host) {
  int slot = -1;
  Flags *pinned = readback_slot(&slot);
  env.check(hipMemcpyAsync(pinned ? pinned : host, dev, sizeof(Flags), hipMemcpyDeviceToHost, env.stream));
  env.sync();   // (also when the copy failed: nothing may still write the slot once it is free again)
  if (pinned) {
    *host = *pinned;
    g_rb_busy.fetch_and(~(1u << slot), std::memory_order_release);
  }
  return env.ok();
}

us_status flag_status(const Flags &h) {
  if (h.retry) return US_SORT_RETRY;
  if (h.index_range) return US_ERR_INDEX_RANGE;
  if (h.duplicate) return US_ERR_DUPLICATE;
  if (h.ell_overflow) return US_ERR_SHAPE;
  return US_OK;
}

void free_formatted(Env &env, us_formatted *f) {
  if (!f) return;
  const char *s0 = (const char *)f->slab, *s1 = s0 + f->slab_bytes;
  auto drop = [&](void *p) {   // arrays inside the result's own block go with the block
    if (p && !(s0 && (const char *)p >= s0 && (const char *)p < s1)) env.free_raw(p);
  };
  for (int l = 0; l < 5; ++l) {
    drop(f->level[l].ptr);
    drop(f->level[l].idx);
  }
  drop(f->val);
  drop(f->ws);
  drop(f->mp_split);
  env.free_raw(f->slab);
  delete f;
}

void *ensure_workspace(Env &env, const us_formatted &A, size_t bytes) {
  if (env.fixed_ws) {
    if (bytes > env.fixed_ws_bytes) { env.fail(US_ERR_SCRATCH_LIMIT); return nullptr; }
    return env.fixed_ws;
  }
  if (A.ws_bytes >= bytes && A.ws) return A.ws;
  if (A.ws) {
    env.sync();  // an earlier compute call may still use the old scratch
    const char *s0 = (const char *)A.slab, *w = (const char *)A.ws;
    if (!(s0 && w >= s0 && w < s0 + A.slab_bytes)) env.free_raw(A.ws);   // (scratch set aside inside the result's own block stays there)
    A.ws = nullptr; A.ws_bytes = 0;
  }
  A.ws = env.alloc_raw(bytes < 256 ? 256 : bytes);
  if (!A.ws) { env.fail(US_ERR_ALLOC); return nullptr; }
  A.ws_bytes = bytes;
  return A.ws;
}

KeySpec rowcol_keyspec(const us_coo &coo, bool swapped) {
  KeySpec ks{};
  ks.mode = 0; ks.swap = swapped ? 1 : 0;
  ks.a_extent = (uint32_t)(swapped ? coo.ncols : coo.nrows);
  ks.b_extent = (uint32_t)(swapped ? coo.nrows : coo.ncols);
  ks.b_bits = bits_for(ks.b_extent - 1);
  ks.total_bits = ks.b_bits + bits_for(ks.a_extent - 1);
  ks.bh = ks.bw = 1;
  return ks;
}

// Gives f (shape already set) the levels of an ELL tensor of width K, every slot empty (column -1, value 0) if `fill`.
static bool ell_shell(Env &env, us_formatted *f, int64_t K, bool fill = true) {
  const int64_t slots = K * f->nrows;
  int32_t *ecol = env.owned<int32_t>(slots);
  float *ev = env.owned<float>(slots);
  f->nlevels = 3;
  f->level[0].size = K; f->level[1].size = f->nrows;
  f->level[2].idx = ecol; f->level[2].nidx = slots;
  f->val = ev; f->nval = slots; f->nmajor = K;
  if (!env.ok()) return false;
  if (fill) {
    fill_u32(env, (uint32_t *)ecol, slots, 0xFFFFFFFFu);
    fill_u32(env, (uint32_t *)ev, slots, 0u);
  }
  return true;
}

static void ell_fill(Env &env, const int32_t *minor, const float *val, const int32_t *ptr, int64_t nrows, int64_t nnz,
                     int64_t K, int64_t clip, us_formatted *f, Flags *flags) {
  if (K > 0)
    US_LAUNCH(env, "ell_fill", 8.0 * nnz + 8.0 * K * nrows, ell_fill_kernel, ceil_div<int64_t>(nrows, EF_ROWS), EF_ROWS, minor,
              val, ptr, nrows, K, clip, f->level[2].idx, f->val, flags);
}

// ELL of width K over the first min(length, clip) entries of every row of a list sorted by (row, col), ptr over its
// rows; nnz = how many entries that is.  The list must be known to be in range (the slab is indexed by row).
us_formatted *new_ell_of_rows(Env &env, const us_format_desc &desc, int64_t nrows, int64_t ncols, int64_t nnz, int64_t K,
                              int64_t clip, const int32_t *minor, const float *val, const int32_t *ptr, Flags *flags) {
  us_formatted *f = new us_formatted();
  f->desc = desc; f->pattern = P_ELL; f->swapped = false;
  f->nrows = nrows; f->ncols = ncols; f->nnz = nnz;
  if (!ell_shell(env, f, K, false)) { free_formatted(env, f); return nullptr; }
  ell_fill(env, minor, val, ptr, nrows, nnz, K, clip, f, flags);
  return f;
}

// The scratch of the merge-path product (two words per tile) comes out of the result's own block when that has
// room for it (convert_with_plan sizes it so); otherwise the first product allocates it.
static void product_scratch(Env &env, us_formatted *f) {
  if (!f->mp_split || f->mp_tiles <= 0 || f->swapped) return;
  const size_t bytes = 2 * Env::granule(4 * (size_t)f->mp_tiles);
  if (env.out_left < bytes) return;
  f->ws = env.owned<char>(bytes);
  f->ws_bytes = bytes;
}

// Build COO / CSR / DCSR / ELL from entries already sorted by (major, minor).  `major` is a
// temporary unless the format keeps it (COO); `minor` and `val` are owned arrays of nnz entries
// that move into the result (or are released when the format re-lays them out: ELL).
us_status build_from_sorted(Env &env, const Plan &plan, const us_format_desc &desc, int64_t nrows,
                            int64_t ncols, int64_t nnz, int32_t *major, int32_t *minor, float *val,
                            Flags *flags, bool check_dups, us_formatted **out, bool validated, bool major_is_temp) {
  // Takes ownership of major, minor and val (arrays of nnz entries from Env::owned; major from Env::temp if
  // major_is_temp, which the COO layout, the one that keeps it, does not allow).
  // validated: the caller has already read the flags after the sort (indices are in range).
  if (major_is_temp && plan.pattern == P_COO) return US_ERR_UNSUPPORTED_DESC;
  us_formatted *f = new us_formatted();
  f->desc = desc; f->pattern = plan.pattern; f->swapped = plan.swapped;
  f->nrows = nrows; f->ncols = ncols; f->nnz = nnz;
  const int64_t nmaj = plan.swapped ? ncols : nrows;
  bool major_loose = !major_is_temp, minor_loose = true, val_loose = true;  // not yet attached to f
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
    if (check_dups) check_unique(env, major, minor, nnz, flags);
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
  sorted_ptr(env, major, minor, nnz, nmaj, ptr, check_dups, flags);

  if (plan.pattern == P_CSR) {
    f->nlevels = 2;
    f->level[0].size = nmaj;
    f->level[1].idx = minor; f->level[1].nidx = nnz;
    f->val = val; f->nval = nnz; f->nmajor = nmaj;
    minor_loose = val_loose = false;
    spmv_prepare(env, f);
    product_scratch(env, f);
    return finish(flags_ok(&h));
  }

  if (plan.pattern == P_DCSR) {
    // Trim(0): keep only the major indices that have children.  How many there are (nnr) stays on the
    // device until the one read of the flags that ends the call: idx and ptr are allocated for the most
    // there can be, min(nmaj, nnz), and the kernels in between take nnr from device memory.
    const int64_t cap = nmaj < nnz ? nmaj : nnz;
    const int64_t ntile = ceil_div<int64_t>(nmaj, NE_TILE);
    uint32_t *partial = env.temp<uint32_t>(ntile);
    int32_t *idx0 = env.owned<int32_t>(cap), *ptr1 = env.owned<int32_t>(cap + 1);
    f->nlevels = 2;
    f->level[0].idx = idx0; f->level[0].nidx = 0;
    f->level[1].ptr = ptr1; f->level[1].nptr = 1;
    f->level[1].idx = minor; f->level[1].nidx = nnz;
    f->val = val; f->nval = nnz; f->nmajor = 0;
    minor_loose = val_loose = false;
    if (!env.ok()) return finish(env.status);
    US_LAUNCH(env, "nonempty_count", 4.0 * nmaj, nonempty_count_kernel, ntile, NE_T, (const int32_t *)ptr, nmaj, partial);
    scan_partials_launch(env, partial, ntile, &flags->scalar[0]);
    US_LAUNCH(env, "nonempty_compact", 4.0 * nmaj + 8.0 * cap, nonempty_compact_kernel, ntile, NE_T, (const int32_t *)ptr,
              nmaj, (const uint32_t *)partial, (const int32_t *)&flags->scalar[0], cap, (int32_t)nnz, idx0, ptr1);
    spmv_prepare(env, f, &flags->scalar[0], cap);
    product_scratch(env, f);
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
      max_group_len(env, ptr, nmaj, &flags->scalar[0]);
    if (K == 0 || !validated) {   // the scatter below indexes by the major index: it must be known to be in range
      us_status s = flags_ok(&h);
      if (s != US_OK) return finish(s);
      if (K == 0) K = h.scalar[0];
    }
    if (K * nrows >= (1ll << 31)) return finish(US_ERR_OVERFLOW);
    if (!ell_shell(env, f, K, false)) return finish(env.status);
    ell_fill(env, minor, val, ptr, nrows, nnz, K, -1, f, flags);
    return finish(flags_ok(&h));
  }
  return finish(US_ERR_UNSUPPORTED_DESC);
}

// ------------------------------------------------------------------ convert
us_status validate_coo(const us_coo &coo) {
  if (coo.nrows <= 0 || coo.ncols <= 0 || coo.nnz < 0) return US_ERR_SHAPE;
  if (coo.nrows >= (1ll << 31) || coo.ncols >= (1ll << 31) || coo.nnz >= (1ll << 31)) return US_ERR_OVERFLOW;
  if (coo.nnz > 0 && (!coo.row || !coo.col || !coo.val)) return US_ERR_NULL;
  return US_OK;
}

Flags *new_flags(Env &env) {
  Flags *flags = env.temp<Flags>(1);
  fill_u32(env, (uint32_t *)flags, sizeof(Flags) / 4, 0u);
  return flags;
}

us_status convert_with_plan(Env &env, const us_coo &coo, const Plan &plan, const us_format_desc &desc,
                            us_formatted **out) {
  const bool by_sort = plan.pattern == P_COO || plan.pattern == P_CSR || plan.pattern == P_DCSR ||
                       plan.pattern == P_ELL || plan.pattern == P_CISR;
  const bool rowcol = by_sort && plan.pattern != P_CISR;   // built below from the (major, minor) order
  const int64_t n = coo.nnz;
  size_t late_res = 0;
  if (by_sort) {
    // two calls into the caller's allocator for the whole conversion: the flags, the sort's buffers and the other
    // temporaries in one block, the arrays of the result in another (each call costs microseconds of an idle GPU)
    auto g = [](size_t count) { return Env::granule(4 * count); };
    const size_t nmaj = (size_t)(plan.swapped ? coo.ncols : coo.nrows), cap = nmaj < (size_t)n ? nmaj : (size_t)n;
    size_t tmp = sort_temp_bytes(n) + 4 * Env::granule(sizeof(Flags)), res = 0;
    if (rowcol && plan.pattern != P_COO) tmp += g(n);   // the major indices: only the COO layout keeps them
    if (plan.pattern == P_COO) res = 3 * g(n);
    // (with the tile starts of the product goes its scratch, two words per tile: the first product then allocates nothing)
    if (plan.pattern == P_CSR) res = 2 * g(n) + g(nmaj + 1) + g(spmv_tiles(nmaj, n) + 1) + 2 * g(spmv_tiles(nmaj, n));
    if (plan.pattern == P_DCSR) {
      res = 2 * g(n) + g(cap) + g(cap + 1) + g(spmv_tiles(cap, n) + 1) + 2 * g(spmv_tiles(cap, n));
      tmp += g(nmaj + 1) + g(nmaj / 1024 + 64);   // pointers over all rows, counts of the stored rows per tile
    }
    if (plan.pattern == P_ELL) tmp += g(nmaj + 1);
    env.reserve(tmp);
    late_res = env.one_result && rowcol ? res : 0;   // the block of the result is allocated while the sort runs
    if (env.one_result && !rowcol) env.reserve_out(res);
  } else if (plan.pattern == P_DIA) {   // counters, flags, positions and slab indices of the diagonals, scan sums
    const size_t nbins = (size_t)(coo.nrows + coo.ncols);
    env.reserve(4 * Env::granule(4 * nbins) + Env::granule(4 * (nbins / 1024 + 64)) + 8 * Env::granule(256));
  } else if (plan.pattern == P_BCSR || plan.pattern == P_BDIA || plan.pattern == P_BELL) {   // sorted keys and values, block counts per tile
    env.reserve(Env::granule(8 * (size_t)n) + Env::granule(4 * (size_t)n) + Env::granule(4 * ((size_t)n / 1024 + 64)) +
                8 * Env::granule(256));
  }
  Flags *flags = new_flags(env);
  if (!env.ok()) return env.status;
  if (plan.pattern == P_DIA) return convert_dia(env, coo, plan, desc, flags, out);
  if (plan.pattern == P_BCSR || plan.pattern == P_BDIA || plan.pattern == P_BELL) return convert_blocked(env, coo, plan, desc, flags, out);
  if (plan.pattern == P_CSB) return convert_csb(env, coo, plan, desc, flags, out);
  if (plan.pattern == P_CISR) return convert_cisr(env, coo, plan, desc, flags, out);
  // COO / CSR / DCSR / ELL: sort by (major, minor), then build
  const bool keep_major = plan.pattern == P_COO;
  int32_t *major = nullptr, *minor = nullptr;
  float *val = nullptr;
  SortOut so{};
  so.late = [&](SortOut &o) {
    if (late_res) env.reserve_out(late_res);
    major = keep_major ? env.owned<int32_t>(n) : env.temp<int32_t>(n);
    minor = env.owned<int32_t>(n);
    val = env.owned<float>(n);
    o.major = major; o.minor = minor; o.val = val;
  };
  const bool checked = sort_coo(env, coo.row, coo.col, coo.val, n, rowcol_keyspec(coo, plan.swapped), so, flags);
  if (!env.ok()) { if (keep_major) env.free_raw(major); env.free_raw(minor); env.free_raw(val); return env.status; }
  return build_from_sorted(env, plan, desc, coo.nrows, coo.ncols, n, major, minor, val, flags, !checked, out, false,
                           !keep_major);
}

us_status convert_impl(Env &env, const us_coo &coo, const us_format_desc &desc, us_formatted **out) {
  *out = nullptr;
  us_status s = validate_coo(coo);
  if (s != US_OK) return s;
  Plan plan;
  if (!match_desc(desc, &plan)) return US_ERR_UNSUPPORTED_DESC;
  if (plan.pattern == P_ELL && plan.swapped) return US_ERR_UNSUPPORTED_DESC;
  env.one_result = true;
  s = convert_with_plan(env, coo, plan, desc, out);
  if (s == US_OK && !env.ok()) s = env.status;
  if (s != US_OK && *out) { free_formatted(env, *out); *out = nullptr; }
  if (s == US_OK) env.adopt_out(*out);
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
    case P_BELL: {   // slot node = (slot, block row); TileUnion: d0 = br*bh + r, d1 = bc*bw + c
      const int64_t bsz = v.bh * v.bw, node = s / bsz, in = s - node * bsz, ri = in / v.bw, ci = in - ri * v.bw;
      const int64_t nbr = (v.nrows + v.bh - 1) / v.bh, br = node % nbr, bc = v.idx[node];
      const int64_t row = br * v.bh + ri, col = bc * v.bw + ci;
      if (bc < 0 || val == 0.f || row >= v.nrows || col >= v.ncols) return false;
      *r = (int32_t)row; *c = (int32_t)col; *x = val;
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

// Compressed layouts (CSR, DCSR, CISR-plus, and CSC / DCSC with columns in the role of rows): Split(ptr) = one
// major index per entry, found with the
// tile starts on the merge path that the conversion left for the product kernels: a workgroup stages the row ends
// that fall into its tile and every entry searches them in LDS.  Columns and values are used where they are.
__global__ __launch_bounds__(256) void expand_rows_kernel(const int32_t *ptr, const int32_t *row_ids, const int32_t *split,
                                                         int64_t nrows, int64_t nnz, int32_t *row_out) {
  __shared__ int32_t s_end[MP_TILE];
  const int32_t *row_end = ptr + 1;
  const int64_t total = nrows + nnz;
  const int64_t diag0 = (int64_t)blockIdx.x * MP_TILE, diag1 = min(diag0 + (int64_t)MP_TILE, total);
  const int64_t r0 = split[blockIdx.x], r1 = split[blockIdx.x + 1];
  const int64_t z0 = diag0 - r0, z1 = diag1 - r1;
  const int nr = (int)(r1 - r0), nz = (int)(z1 - z0);
  for (int i = threadIdx.x; i < nr; i += 256) s_end[i] = (int32_t)(row_end[r0 + i] - z0);
  __syncthreads();
  for (int i = threadIdx.x; i < nz; i += 256) {
    int lo = 0, hi = nr;   // first staged row whose end lies behind entry i; none: the row that runs on past the tile
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (s_end[mid] <= i) lo = mid + 1; else hi = mid;
    }
    int64_t row = r0 + lo;
    if (row > nrows - 1) row = nrows - 1;
    row_out[z0 + i] = row_ids ? row_ids[row] : (int32_t)row;
  }
}

// layouts without padding: every slot is an entry, so only its coordinates have to be rebuilt
__global__ __launch_bounds__(256) void expand_coords_kernel(SrcView v, int32_t *row, int32_t *col) {
  int64_t s = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (s >= v.nslots) return;
  int32_t r, c; float x;
  slot_entry(v, s, &r, &c, &x);
  row[s] = r; col[s] = c;
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
    case P_ELL:
    case P_BELL: v.idx = src.level[2].idx; break;
    case P_CSB: v.ptr = src.level[2].ptr; v.idx0 = src.level[2].idx; v.idx = src.level[3].idx; break;
    case P_CISR:   // below the partition level it reads like DCSR: stored rows, ptr over them, columns
      v.pattern = P_DCSR; v.idx0 = src.level[1].idx; v.ptr = src.level[2].ptr; v.idx = src.level[2].idx; break;
    default: return US_ERR_FORMAT_MISMATCH;
  }
  const int64_t ns = v.nslots;
  if ((src.pattern == P_CSR || src.pattern == P_DCSR || src.pattern == P_CISR) && src.mp_split && ns > 0 &&
      src.mp_tiles == ceil_div<int64_t>(src.nmajor + ns, MP_TILE)) {
    const StoredRows sr = stored_rows(src);
    int32_t *r = env.temp<int32_t>(ns);
    if (!env.ok()) return env.status;
    US_LAUNCH(env, "expand_rows", 4.0 * ns + 4.0 * src.nmajor, expand_rows_kernel, src.mp_tiles, 256, sr.ptr, sr.row_ids,
              (const int32_t *)src.mp_split, src.nmajor, ns, r);
    us_coo coo{src.nrows, src.ncols, ns, src.swapped ? sr.idx : r, src.swapped ? r : sr.idx, src.val};   // CSC: the major index is d1
    us_status st = env.status;
    if (st == US_OK) st = convert_with_plan(env, coo, plan, desc, out);
    env.sync();
    if (st == US_OK && !env.ok()) st = env.status;
    if (st != US_OK && *out) { free_formatted(env, *out); *out = nullptr; }
    return st;
  }
  if (src.pattern == P_COO || src.pattern == P_CSR || src.pattern == P_DCSR || src.pattern == P_CSB ||
      src.pattern == P_CISR) {
    // no padding anywhere: the values are used where they are, the coordinates are written out once
    int32_t *r = env.temp<int32_t>(ns), *c = env.temp<int32_t>(ns);
    if (!env.ok()) return env.status;
    if (ns > 0)
      US_LAUNCH(env, "expand_coords", 12.0 * ns, expand_coords_kernel, ceil_div<int64_t>(ns, 256), 256, v, r, c);
    us_coo coo{src.nrows, src.ncols, ns, r, c, src.val};
    us_status st = env.status;
    if (st == US_OK) st = convert_with_plan(env, coo, plan, desc, out);
    env.sync();
    if (st == US_OK && !env.ok()) st = env.status;
    if (st != US_OK && *out) { free_formatted(env, *out); *out = nullptr; }
    return st;
  }
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

}  // namespace us
