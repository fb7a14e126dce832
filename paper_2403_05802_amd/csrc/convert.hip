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
static bool tile(const us_expr &e, int kind, int dim, int64_t *f) {
  if (e.kind != kind || e.c != 0 || e.factor < 1 || e.factor > 16) return false;
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
    return false;
  }
  if (d.nlevels == 3) {
    const us_expr &e = d.level[0];
    if (e.kind == US_E_INDIRECT_ENUM && e.c0 == 1 && e.c1 == 0 && e.c == 0 && aff(d.level[1], 1, 0) &&
        aff(d.level[2], 0, 1) && S == 0 && E == 0 && m == 1 && d.ell_width >= 0) {
      p->pattern = P_ELL; p->ell_width = d.ell_width;
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

__global__ __launch_bounds__(256) void dcsr_compact_kernel(const int32_t *ptr, const int32_t *pos, int64_t n,
                                                          int64_t nnr, int32_t nnz, int32_t *idx0, int32_t *ptr1) {
  int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (g == 0) ptr1[nnr] = nnz;
  if (g < n && ptr[g + 1] > ptr[g]) {
    int32_t k = pos[g];
    idx0[k] = (int32_t)g;
    ptr1[k] = ptr[g];
  }
}

__global__ __launch_bounds__(256) void max_len_kernel(const int32_t *ptr, int64_t n, int32_t *out_max) {
  __shared__ int32_t s_max[4];
  int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  int32_t len = g < n ? ptr[g + 1] - ptr[g] : 0;
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

// Build COO / CSR / DCSR / ELL from entries already sorted by (major, minor).  `major` is a
// temporary unless the format keeps it (COO); `minor` and `val` are owned arrays of nnz entries
// that move into the result (or are released when the format re-lays them out: ELL).
static us_status build_from_sorted(Env &env, const Plan &plan, const us_format_desc &desc, int64_t nrows,
                                   int64_t ncols, int64_t nnz, int32_t *major, int32_t *minor, float *val,
                                   Flags *flags, us_formatted **out) {
  // Takes ownership of major, minor and val (arrays of nnz entries from Env::owned).
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
  if (nnz > 1)
    US_LAUNCH(env, "check_unique", 8.0 * nnz, check_unique_unpacked_kernel, ceil_div<int64_t>(nnz, 256), 256,
              (const int32_t *)major, (const int32_t *)minor, nnz, flags);

  if (plan.pattern == P_COO) {
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
  lower_bound_ptr(env, major, nnz, nmaj, ptr);

  if (plan.pattern == P_CSR) {
    f->nlevels = 2;
    f->level[0].size = nmaj;
    f->level[1].idx = minor; f->level[1].nidx = nnz;
    f->val = val; f->nval = nnz; f->nmajor = nmaj;
    minor_loose = val_loose = false;
    return finish(flags_ok(&h));
  }

  if (plan.pattern == P_DCSR) {
    // Trim(0): keep only the major indices that have children
    int32_t *flag = env.temp<int32_t>(nmaj), *pos = env.temp<int32_t>(nmaj);
    if (!env.ok()) return finish(env.status);
    US_LAUNCH(env, "nonempty_flag", 8.0 * nmaj, nonempty_flag_kernel, ceil_div<int64_t>(nmaj, 256), 256,
              (const int32_t *)ptr, nmaj, flag);
    exclusive_scan_i32(env, flag, pos, nmaj, &flags->scalar[0]);
    us_status s = flags_ok(&h);
    if (s != US_OK) return finish(s);
    const int64_t nnr = h.scalar[0];
    int32_t *idx0 = env.owned<int32_t>(nnr), *ptr1 = env.owned<int32_t>(nnr + 1);
    f->nlevels = 2;
    f->level[0].idx = idx0; f->level[0].nidx = nnr;
    f->level[1].ptr = ptr1; f->level[1].nptr = nnr + 1;
    f->level[1].idx = minor; f->level[1].nidx = nnz;
    f->val = val; f->nval = nnz; f->nmajor = nnr;
    minor_loose = val_loose = false;
    if (!env.ok()) return finish(env.status);
    US_LAUNCH(env, "dcsr_compact", 12.0 * nmaj + 8.0 * nnr, dcsr_compact_kernel, ceil_div<int64_t>(nmaj, 256), 256,
              (const int32_t *)ptr, (const int32_t *)pos, nmaj, nnr, (int32_t)nnz, idx0, ptr1);
    env.sync();
    return finish(env.status);
  }

  if (plan.pattern == P_ELL) {
    int64_t K = plan.ell_width;
    if (K == 0)
      US_LAUNCH(env, "max_row_len", 4.0 * nmaj, max_len_kernel, ceil_div<int64_t>(nmaj, 256), 256,
                (const int32_t *)ptr, nmaj, &flags->scalar[0]);
    us_status s = flags_ok(&h);
    if (s != US_OK) return finish(s);
    if (K == 0) K = h.scalar[0];
    if (K * nrows >= (1ll << 31)) return finish(US_ERR_OVERFLOW);
    const int64_t slots = K * nrows;
    int32_t *ecol = env.owned<int32_t>(slots);
    float *ev = env.owned<float>(slots);
    f->nlevels = 3;
    f->level[0].size = K; f->level[1].size = nrows;
    f->level[2].idx = ecol; f->level[2].nidx = slots;
    f->val = ev; f->nval = slots; f->nmajor = K;
    if (!env.ok()) return finish(env.status);
    fill_u32(env, (uint32_t *)ecol, slots, 0xFFFFFFFFu);
    fill_u32(env, (uint32_t *)ev, slots, 0u);
    if (nnz > 0)
      US_LAUNCH(env, "ell_scatter", 16.0 * nnz + 8.0 * nnz, ell_scatter_kernel, ceil_div<int64_t>(nnz, 256), 256,
                (const int32_t *)major, (const int32_t *)minor, (const float *)val, (const int32_t *)ptr, nnz,
                nrows, K, ecol, ev, flags);
    return finish(flags_ok(&h));
  }
  return finish(US_ERR_UNSUPPORTED_DESC);
}

// ------------------------------------------------------------------ DIA
// Sum query grouped by d1-d0: one counter per diagonal, bin = d1 - d0 + (nrows-1).
// Entries of a wavefront that hit the same bin are combined before the atomic.
__global__ __launch_bounds__(256) void diag_hist_kernel(const int32_t *row, const int32_t *col, int64_t n,
                                                       uint32_t nrows, uint32_t ncols, uint32_t *count,
                                                       Flags *flags) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  bool valid = i < n;
  uint32_t r = valid ? (uint32_t)row[i] : 0u, c = valid ? (uint32_t)col[i] : 0u;
  if (valid && (r >= nrows || c >= ncols)) { flags->index_range = 1; valid = false; }
  uint32_t bin = c - r + (nrows - 1);
  uint64_t todo = __ballot(valid);
  while (todo) {
    int leader = __ffsll((unsigned long long)todo) - 1;
    uint32_t lb = __shfl(bin, leader);
    uint64_t same = __ballot(valid && bin == lb) & todo;
    if (lane_id() == leader) atomicAdd(&count[lb], (uint32_t)__popcll(same));
    todo &= ~same;
  }
}

// flag of a diagonal: stored (count > 0) for a plain conversion
__global__ __launch_bounds__(256) void diag_flag_nonempty_kernel(const uint32_t *count, int64_t nbins, int32_t *flag) {
  int64_t d = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (d < nbins) flag[d] = count[d] > 0 ? 1 : 0;
}

__global__ __launch_bounds__(256) void diag_offsets_kernel(const int32_t *flag, const int32_t *pos, int64_t nbins,
                                                          int32_t nrows, int32_t *off) {
  int64_t d = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (d < nbins && flag[d]) off[pos[d]] = (int32_t)(d - (nrows - 1));
}

// scatter into the zero-filled slab val[k*L + i]; a bitmap with one bit per slot detects duplicates
__global__ __launch_bounds__(256) void dia_scatter_kernel(const int32_t *row, const int32_t *col, const float *val,
                                                         int64_t n, uint32_t nrows, const int32_t *flag,
                                                         const int32_t *pos, int64_t L, int by_col, float *slab,
                                                         uint32_t *bitmap, Flags *flags) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  uint32_t r = (uint32_t)row[i], c = (uint32_t)col[i];
  uint32_t bin = c - r + (nrows - 1);
  if (!flag[bin]) return;
  int64_t slot = (int64_t)pos[bin] * L + (by_col ? c : r);
  uint32_t bit = 1u << (slot & 31);
  uint32_t old = atomicOr(&bitmap[slot >> 5], bit);
  if (old & bit) flags->duplicate = 1;
  slab[slot] = val[i];
}

static us_status convert_dia(Env &env, const us_coo &coo, const Plan &plan, const us_format_desc &desc,
                             Flags *flags, us_formatted **out) {
  const int64_t nbins = coo.nrows + coo.ncols - 1, n = coo.nnz;
  const int64_t L = plan.swapped ? coo.ncols : coo.nrows;
  uint32_t *count = env.temp<uint32_t>(nbins);
  int32_t *flag = env.temp<int32_t>(nbins), *pos = env.temp<int32_t>(nbins);
  if (!env.ok()) return env.status;
  fill_u32(env, count, nbins, 0);
  if (n > 0)
    US_LAUNCH(env, "diag_hist", 8.0 * n, diag_hist_kernel, ceil_div<int64_t>(n, 256), 256, coo.row, coo.col, n,
              (uint32_t)coo.nrows, (uint32_t)coo.ncols, count, flags);
  US_LAUNCH(env, "diag_flag", 8.0 * nbins, diag_flag_nonempty_kernel, ceil_div<int64_t>(nbins, 256), 256,
            (const uint32_t *)count, nbins, flag);
  exclusive_scan_i32(env, flag, pos, nbins, &flags->scalar[0]);
  Flags h{};
  if (!read_flags(env, flags, &h)) return env.status;
  if (flag_status(h) != US_OK) return flag_status(h);
  const int64_t ndiag = h.scalar[0];
  if (ndiag * L >= (1ll << 31)) return US_ERR_OVERFLOW;
  us_formatted *f = new us_formatted();
  f->desc = desc; f->pattern = P_DIA; f->swapped = plan.swapped;
  f->nrows = coo.nrows; f->ncols = coo.ncols; f->nnz = n;
  f->nlevels = 2;
  f->level[0].idx = env.owned<int32_t>(ndiag); f->level[0].nidx = ndiag;
  f->level[1].size = L;
  f->val = env.owned<float>(ndiag * L); f->nval = ndiag * L; f->nmajor = ndiag;
  uint32_t *bitmap = env.temp<uint32_t>(ceil_div<int64_t>(ndiag * L, 32) + 1);
  if (!env.ok()) { free_formatted(env, f); return env.status; }
  fill_u32(env, (uint32_t *)f->val, ndiag * L, 0u);
  fill_u32(env, bitmap, ceil_div<int64_t>(ndiag * L, 32) + 1, 0u);
  US_LAUNCH(env, "diag_offsets", 8.0 * nbins, diag_offsets_kernel, ceil_div<int64_t>(nbins, 256), 256,
            (const int32_t *)flag, (const int32_t *)pos, nbins, (int32_t)coo.nrows, f->level[0].idx);
  if (n > 0)
    US_LAUNCH(env, "dia_scatter", 16.0 * n, dia_scatter_kernel, ceil_div<int64_t>(n, 256), 256, coo.row, coo.col,
              coo.val, n, (uint32_t)coo.nrows, (const int32_t *)flag, (const int32_t *)pos, L,
              plan.swapped ? 1 : 0, f->val, bitmap, flags);
  if (!read_flags(env, flags, &h)) { free_formatted(env, f); return env.status; }
  if (flag_status(h) != US_OK) { free_formatted(env, f); return flag_status(h); }
  *out = f;
  return US_OK;
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
                                                        KeySpec ks, const uint32_t *partial, int32_t *blk_row,
                                                        int32_t *blk_col, float *bval) {
  __shared__ uint32_t s_wave[BE_T / 64 + 1];
  const int inner_bits = ks.ih_bits + ks.iw_bits;
  int64_t base = (int64_t)blockIdx.x * BE_TILE + (int64_t)threadIdx.x * BE_IPT;
  uint64_t k[BE_IPT];
  uint32_t head[BE_IPT], heads = 0;
  uint64_t prev = (base > 0 && base <= n) ? key[base - 1] : ~0ull;
#pragma unroll
  for (int j = 0; j < BE_IPT; ++j) {
    int64_t i = base + j;
    k[j] = i < n ? key[i] : ~0ull;
    head[j] = (i < n) && ((i == 0) | ((k[j] >> inner_bits) != (prev >> inner_bits)));
    heads += head[j];
    prev = k[j];
  }
  uint32_t total;
  uint32_t id = block_exclusive_sum<BE_T>(heads, s_wave, &total) + partial[blockIdx.x];  // blocks before
  const uint32_t bsz = ks.bh * ks.bw;
#pragma unroll
  for (int j = 0; j < BE_IPT; ++j) {
    int64_t i = base + j;
    if (i >= n) break;
    id += head[j];
    uint32_t blk = id - 1;
    uint32_t bi = (uint32_t)(k[j] & ((1ull << ks.iw_bits) - 1));
    uint32_t ai = (uint32_t)((k[j] >> ks.iw_bits) & ((1ull << ks.ih_bits) - 1));
    uint64_t bk = k[j] >> inner_bits;
    if (head[j]) {
      blk_col[blk] = (int32_t)(bk & ((1ull << ks.b_bits) - 1));
      blk_row[blk] = (int32_t)(bk >> ks.b_bits);
    }
    bval[(size_t)blk * bsz + ai * ks.bw + bi] = val[i];
  }
}

static us_status convert_bcsr(Env &env, const us_coo &coo, const Plan &plan, const us_format_desc &desc,
                              Flags *flags, us_formatted **out) {
  const int64_t n = coo.nnz;
  const int64_t nbr = ceil_div<int64_t>(coo.nrows, plan.bh), nbc = ceil_div<int64_t>(coo.ncols, plan.bw);
  KeySpec ks{};
  ks.mode = 1; ks.swap = 0; ks.bh = (uint32_t)plan.bh; ks.bw = (uint32_t)plan.bw;
  ks.a_extent = (uint32_t)coo.nrows; ks.b_extent = (uint32_t)coo.ncols;
  ks.b_bits = bits_for(nbc - 1);
  ks.ih_bits = bits_for(plan.bh - 1); ks.iw_bits = bits_for(plan.bw - 1);
  ks.total_bits = bits_for(nbr - 1) + ks.b_bits + ks.ih_bits + ks.iw_bits;
  uint64_t *skey = env.temp<uint64_t>(n);
  float *sval = env.temp<float>(n);
  const int64_t nb = ceil_div<int64_t>(n > 0 ? n : 1, BE_TILE);
  uint32_t *partial = env.temp<uint32_t>(nb);
  if (!env.ok()) return env.status;
  SortOut so{};
  so.key64 = skey; so.val = sval;
  sort_coo(env, coo.row, coo.col, coo.val, n, ks, so, flags);
  US_LAUNCH(env, "bcsr_count", 8.0 * n, bcsr_count_kernel, nb, BE_T, (const uint64_t *)skey, n,
            ks.ih_bits + ks.iw_bits, partial, flags);
  scan_partials_launch(env, partial, nb, &flags->scalar[0]);
  Flags h{};
  if (!read_flags(env, flags, &h)) return env.status;
  if (flag_status(h) != US_OK) return flag_status(h);
  const int64_t nblk = h.scalar[0], bsz = plan.bh * plan.bw;
  if (nblk * bsz >= (1ll << 31)) return US_ERR_OVERFLOW;
  us_formatted *f = new us_formatted();
  f->desc = desc; f->pattern = P_BCSR;
  f->nrows = coo.nrows; f->ncols = coo.ncols; f->nnz = n;
  f->nlevels = 4;
  f->level[0].size = nbr;
  f->level[1].ptr = env.owned<int32_t>(nbr + 1); f->level[1].nptr = nbr + 1;
  f->level[1].idx = env.owned<int32_t>(nblk); f->level[1].nidx = nblk;
  f->level[2].size = plan.bh; f->level[3].size = plan.bw;
  f->val = env.owned<float>(nblk * bsz); f->nval = nblk * bsz;
  f->nmajor = nbr; f->bh = plan.bh; f->bw = plan.bw; f->nblk = nblk;
  int32_t *blk_row = env.temp<int32_t>(nblk);
  if (!env.ok()) { free_formatted(env, f); return env.status; }
  fill_u32(env, (uint32_t *)f->val, nblk * bsz, 0u);
  if (n > 0)
    US_LAUNCH(env, "bcsr_emit", 12.0 * n + 4.0 * n, bcsr_emit_kernel, nb, BE_T, (const uint64_t *)skey,
              (const float *)sval, n, ks, (const uint32_t *)partial, blk_row, f->level[1].idx, f->val);
  lower_bound_ptr(env, blk_row, nblk, nbr, f->level[1].ptr);
  env.sync();
  if (!env.ok()) { free_formatted(env, f); return env.status; }
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
  Flags *flags = new_flags(env);
  if (!env.ok()) return env.status;
  if (plan.pattern == P_DIA) return convert_dia(env, coo, plan, desc, flags, out);
  if (plan.pattern == P_BCSR) return convert_bcsr(env, coo, plan, desc, flags, out);
  // COO / CSR / DCSR / ELL: sort by (major, minor), then build
  const int64_t n = coo.nnz;
  int32_t *major = env.owned<int32_t>(n), *minor = env.owned<int32_t>(n);
  float *val = env.owned<float>(n);
  if (!env.ok()) { env.free_raw(major); env.free_raw(minor); env.free_raw(val); return env.status; }
  SortOut so{};
  so.major = major; so.minor = minor; so.val = val;
  sort_coo(env, coo.row, coo.col, coo.val, n, rowcol_keyspec(coo, plan.swapped), so, flags);
  return build_from_sorted(env, plan, desc, coo.nrows, coo.ncols, n, major, minor, val, flags, out);
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

us_status decompose_impl(Env &env, const us_coo &coo, const us_format_desc &da, const us_format_desc &db,
                         const us_predicate &pred, us_formatted **oa, us_formatted **ob) {
  *oa = *ob = nullptr;
  return US_ERR_UNSUPPORTED_DESC;
}

}  // namespace us
