// Device-wide building blocks: fill, exclusive scan, group pointers by binary search, and the
// LSD radix sort that realises the Sort operator of the conversion algorithm (Figure 8:
// "apply Sort to T_format"; Section 7.2.1 reports it as 65 % of COO->BDIA conversion time).
#include "common.h"
#include "device.h"

namespace us {

// ------------------------------------------------------------------ Env / Profile (host)
void *Env::alloc_raw(size_t bytes) {
  if (ctx && ctx->alloc) return ctx->alloc(bytes, ctx->user);
  void *p = nullptr;
  if (hipMalloc(&p, bytes) != hipSuccess) return nullptr;
  return p;
}
void Env::free_raw(void *p) {
  if (!p) return;
  if (ctx && ctx->alloc) { if (ctx->free) ctx->free(p, ctx->user); }
  else (void)hipFree(p);
}
void Env::release_temps() {
  if (temps.empty()) return;
  (void)hipStreamSynchronize(stream);  // kernels may still read the temporaries
  for (void *p : temps) free_raw(p);
  temps.clear();
}

int Profile::intern(const char *name) {
  for (size_t i = 0; i < entries.size(); ++i)
    if (entries[i].name == name || strcmp(entries[i].name, name) == 0) return (int)i;
  entries.push_back({name, 0, 0.0, 0.0});
  return (int)entries.size() - 1;
}
hipEvent_t Profile::get_event() {
  if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  (void)hipEventCreate(&e);
  return e;
}

LaunchScope::LaunchScope(Env &e, const char *name, double alg_bytes) : env(e), bytes(alg_bytes) {
  if (!env.prof) return;
  idx = env.prof->intern(name);
  a = env.prof->get_event();
  b = env.prof->get_event();
  env.check(hipEventRecord(a, env.stream));
}
LaunchScope::~LaunchScope() {
  if (!env.prof || idx < 0) return;
  env.check(hipEventRecord(b, env.stream));
  env.prof->pending.push_back({idx, a, b, bytes});
}

// ------------------------------------------------------------------ fill
__global__ __launch_bounds__(256) void fill_u32_kernel(uint32_t *p, uint64_t n, uint32_t v) {
  uint64_t i = (uint64_t)blockIdx.x * 1024 + threadIdx.x;
#pragma unroll
  for (int k = 0; k < 4; ++k, i += 256)
    if (i < n) p[i] = v;
}
void fill_u32(Env &env, uint32_t *p, uint64_t n, uint32_t v) {
  if (n == 0) return;
  US_LAUNCH(env, "fill_u32", 4.0 * n, fill_u32_kernel, ceil_div<uint64_t>(n, 1024), 256, p, n, v);
}

// ------------------------------------------------------------------ exclusive scan (int32), three phases
constexpr int SCAN_T = 256, SCAN_IPT = 8, SCAN_TILE = SCAN_T * SCAN_IPT;

__global__ __launch_bounds__(SCAN_T) void scan_reduce_kernel(const int32_t *in, int64_t n, uint32_t *partial) {
  __shared__ uint32_t s_wave[SCAN_T / 64 + 1];
  int64_t base = (int64_t)blockIdx.x * SCAN_TILE;
  uint32_t s = 0;
#pragma unroll
  for (int k = 0; k < SCAN_IPT; ++k) {
    int64_t i = base + k * SCAN_T + threadIdx.x;
    if (i < n) s += (uint32_t)in[i];
  }
  uint32_t total;
  block_exclusive_sum<SCAN_T>(s, s_wave, &total);
  if (threadIdx.x == 0) partial[blockIdx.x] = total;
}

// single workgroup: exclusive scan of the per-tile sums in place, grand total to *total_dev
__global__ __launch_bounds__(1024) void scan_partials_kernel(uint32_t *partial, int64_t nb, int32_t *total_dev) {
  __shared__ uint32_t s_wave[1024 / 64 + 1];
  uint32_t carry = 0;
  for (int64_t base = 0; base < nb; base += 1024) {
    int64_t i = base + threadIdx.x;
    uint32_t v = i < nb ? partial[i] : 0u, total;
    uint32_t ex = block_exclusive_sum<1024>(v, s_wave, &total);
    if (i < nb) partial[i] = ex + carry;
    carry += total;
  }
  if (threadIdx.x == 0 && total_dev) *total_dev = (int32_t)carry;
}

__global__ __launch_bounds__(SCAN_T) void scan_apply_kernel(const int32_t *in, int32_t *out, int64_t n,
                                                           const uint32_t *partial) {
  __shared__ uint32_t s_wave[SCAN_T / 64 + 1];
  // blocked arrangement: thread t owns SCAN_IPT consecutive elements
  int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_IPT;
  uint32_t v[SCAN_IPT], s = 0;
#pragma unroll
  for (int k = 0; k < SCAN_IPT; ++k) {
    v[k] = (base + k < n) ? (uint32_t)in[base + k] : 0u;
    s += v[k];
  }
  uint32_t total;
  uint32_t ex = block_exclusive_sum<SCAN_T>(s, s_wave, &total) + partial[blockIdx.x];
#pragma unroll
  for (int k = 0; k < SCAN_IPT; ++k) {
    if (base + k < n) out[base + k] = (int32_t)ex;
    ex += v[k];
  }
}

void scan_partials_launch(Env &env, uint32_t *partial, int64_t nb, int32_t *total_dev) {
  US_LAUNCH(env, "scan_partials", 8.0 * nb, scan_partials_kernel, 1, 1024, partial, nb, total_dev);
}

void exclusive_scan_i32(Env &env, const int32_t *in, int32_t *out, int64_t n, int32_t *total_dev) {
  int64_t nb = ceil_div<int64_t>(n > 0 ? n : 1, SCAN_TILE);
  uint32_t *partial = env.temp<uint32_t>(nb);
  if (!env.ok()) return;
  US_LAUNCH(env, "scan_reduce", 4.0 * n, scan_reduce_kernel, nb, SCAN_T, in, n, partial);
  scan_partials_launch(env, partial, nb, total_dev);
  US_LAUNCH(env, "scan_apply", 8.0 * n, scan_apply_kernel, nb, SCAN_T, in, out, n, (const uint32_t *)partial);
}

// ------------------------------------------------------------------ ptr[g] = first position whose major >= g
__global__ __launch_bounds__(256) void lower_bound_ptr_kernel(const int32_t *major, int64_t n, int64_t ngroups,
                                                              int32_t *ptr) {
  int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (g > ngroups) return;
  int64_t lo = 0, hi = n;
  while (lo < hi) {
    int64_t mid = (lo + hi) >> 1;
    if ((int64_t)major[mid] < g) lo = mid + 1; else hi = mid;
  }
  ptr[g] = (int32_t)lo;
}
void lower_bound_ptr(Env &env, const int32_t *sorted_major, int64_t n, int64_t ngroups, int32_t *ptr) {
  US_LAUNCH(env, "ptr_lower_bound", 4.0 * n + 4.0 * (ngroups + 1), lower_bound_ptr_kernel,
            ceil_div<int64_t>(ngroups + 1, 256), 256, sorted_major, n, ngroups, ptr);
}

// ------------------------------------------------------------------ radix sort
// One pass = per-tile digit histogram, per-digit scan over tiles, stable tile scatter.
constexpr int RS_T = 512, RS_IPT = 8, RS_TILE = RS_T * RS_IPT, RS_NW = RS_T / 64, RS_MAXBITS = 8, RS_BINS = 1 << RS_MAXBITS;

template <typename K>
__device__ __forceinline__ K build_key(const KeySpec &ks, uint32_t r, uint32_t c) {
  uint32_t a = ks.swap ? c : r, b = ks.swap ? r : c;
  if (ks.mode == 0) return ((K)a << ks.b_bits) | (K)b;
  uint32_t ab = a / ks.bh, ai = a - ab * ks.bh, bb = b / ks.bw, bi = b - bb * ks.bw;
  return (((((K)ab << ks.b_bits) | (K)bb) << ks.ih_bits | (K)ai) << ks.iw_bits) | (K)bi;
}

template <typename K>
struct PassArgs {
  const int32_t *row, *col;      // COO input (first pass) or null
  const K *key_in;               // packed input otherwise
  const uint32_t *val_in;
  K *key_out; uint32_t *val_out; // packed output, or
  int32_t *major_out, *minor_out;  // unpacked output (last pass, mode 0)
  uint32_t n; int shift; uint32_t mask; uint32_t nblocks;
  uint32_t *hist;                // [bins][nblocks]
  uint32_t *totals;              // [bins]
  KeySpec ks;
  Flags *flags;
};

template <typename K, bool FROM_COO>
__device__ __forceinline__ K load_key(const PassArgs<K> &a, uint32_t i) {
  if (FROM_COO) return build_key<K>(a.ks, (uint32_t)a.row[i], (uint32_t)a.col[i]);
  return a.key_in[i];
}

template <typename K, bool FROM_COO>
__global__ __launch_bounds__(RS_T) void radix_hist_kernel(PassArgs<K> a) {
  __shared__ uint32_t s_hist[RS_BINS];
  for (int i = threadIdx.x; i < RS_BINS; i += RS_T) s_hist[i] = 0;
  __syncthreads();
  const uint32_t base = blockIdx.x * RS_TILE;
  bool bad = false;
#pragma unroll
  for (int k = 0; k < RS_IPT; ++k) {
    uint32_t i = base + k * RS_T + threadIdx.x;
    if (i < a.n) {
      K key;
      if (FROM_COO) {
        uint32_t r = (uint32_t)a.row[i], c = (uint32_t)a.col[i];
        uint32_t ra = a.ks.swap ? c : r, cb = a.ks.swap ? r : c;
        bad |= (ra >= a.ks.a_extent) | (cb >= a.ks.b_extent);
        key = build_key<K>(a.ks, r, c);
      } else {
        key = a.key_in[i];
      }
      atomicAdd(&s_hist[(uint32_t)(key >> a.shift) & a.mask], 1u);
    }
  }
  if (FROM_COO && bad) a.flags->index_range = 1;
  __syncthreads();
  for (uint32_t d = threadIdx.x; d <= a.mask; d += RS_T) {
    uint32_t c = s_hist[d];
    a.hist[(size_t)d * a.nblocks + blockIdx.x] = c;
    if (c) atomicAdd(&a.totals[d], c);
  }
}

// one workgroup per digit: global start of the digit + exclusive scan over the tiles
__global__ __launch_bounds__(256) void radix_scan_kernel(uint32_t *hist, const uint32_t *totals, uint32_t nblocks) {
  __shared__ uint32_t s_wave[256 / 64 + 1];
  const uint32_t d = blockIdx.x;
  uint32_t part = 0;
  for (uint32_t i = threadIdx.x; i < d; i += 256) part += totals[i];
  uint32_t start;
  block_exclusive_sum<256>(part, s_wave, &start);
  uint32_t *h = hist + (size_t)d * nblocks;
  uint32_t carry = start;
  for (uint32_t base = 0; base < nblocks; base += 256) {
    uint32_t i = base + threadIdx.x;
    uint32_t v = i < nblocks ? h[i] : 0u, total;
    uint32_t ex = block_exclusive_sum<256>(v, s_wave, &total);
    if (i < nblocks) h[i] = ex + carry;
    carry += total;
  }
}

template <typename K, bool FROM_COO, bool UNPACK>
__global__ __launch_bounds__(RS_T) void radix_scatter_kernel(PassArgs<K> a) {
  __shared__ uint32_t s_cnt[RS_NW][RS_BINS];  // per-wave digit counts, then per-wave bases
  __shared__ uint32_t s_start[RS_BINS];       // first in-tile position of each digit
  __shared__ uint32_t s_goff[RS_BINS];        // global position of the digit's run minus s_start
  __shared__ uint32_t s_wave[RS_T / 64 + 1];
  __shared__ K s_key[RS_TILE];
  uint32_t *s_val = reinterpret_cast<uint32_t *>(s_key);

  const int lane = lane_id(), w = wave_id();
  const uint32_t nbins = a.mask + 1;
  for (uint32_t i = threadIdx.x; i < RS_NW * RS_BINS; i += RS_T) (&s_cnt[0][0])[i] = 0;

  const uint32_t base = blockIdx.x * RS_TILE;
  const uint32_t in_tile = min((uint32_t)RS_TILE, a.n - base);
  K key[RS_IPT];
  uint32_t val[RS_IPT], pos[RS_IPT];
  // wave w owns the contiguous slice [w*64*IPT, (w+1)*64*IPT) of the tile, lanes striped
#pragma unroll
  for (int j = 0; j < RS_IPT; ++j) {
    uint32_t t = w * (64 * RS_IPT) + j * 64 + lane;
    if (t < in_tile) {
      key[j] = load_key<K, FROM_COO>(a, base + t);
      val[j] = FROM_COO ? ((const uint32_t *)a.val_in)[base + t] : a.val_in[base + t];
    } else {
      key[j] = 0; val[j] = 0;
    }
  }
  __syncthreads();

  // stable rank of every item among the items of its wave with the same digit
#pragma unroll
  for (int j = 0; j < RS_IPT; ++j) {
    uint32_t t = w * (64 * RS_IPT) + j * 64 + lane;
    bool valid = t < in_tile;
    uint32_t d = (uint32_t)(key[j] >> a.shift) & a.mask;
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < RS_MAXBITS; ++b) {
      uint64_t bal = __ballot((d >> b) & 1u);
      peers &= ((d >> b) & 1u) ? bal : ~bal;
    }
    uint32_t before = __popcll(peers & lanes_below());
    int leader = __ffsll((unsigned long long)peers) - 1;
    uint32_t old = 0;
    if (valid && lane == leader) {
      old = s_cnt[w][d];
      s_cnt[w][d] = old + (uint32_t)__popcll(peers);
    }
    old = __shfl(old, leader < 0 ? 0 : leader);
    pos[j] = old + before;
    __builtin_amdgcn_wave_barrier();
  }
  __syncthreads();

  // per digit: bases of the waves, tile total
  uint32_t tile_total = 0;
  if (threadIdx.x < nbins) {
#pragma unroll
    for (int ww = 0; ww < RS_NW; ++ww) {
      uint32_t c = s_cnt[ww][threadIdx.x];
      s_cnt[ww][threadIdx.x] = tile_total;
      tile_total += c;
    }
  }
  uint32_t dummy;
  uint32_t start = block_exclusive_sum<RS_T>(tile_total, s_wave, &dummy);
  if (threadIdx.x < nbins) {
    s_start[threadIdx.x] = start;
    s_goff[threadIdx.x] = a.hist[(size_t)threadIdx.x * a.nblocks + blockIdx.x] - start;
  }
  __syncthreads();

#pragma unroll
  for (int j = 0; j < RS_IPT; ++j) {
    uint32_t t = w * (64 * RS_IPT) + j * 64 + lane;
    if (t < in_tile) {
      uint32_t d = (uint32_t)(key[j] >> a.shift) & a.mask;
      pos[j] += s_start[d] + s_cnt[w][d];
      s_key[pos[j]] = key[j];
    }
  }
  __syncthreads();
  uint32_t gpos[RS_IPT];
#pragma unroll
  for (int k = 0; k < RS_IPT; ++k) {
    uint32_t i = k * RS_T + threadIdx.x;
    if (i < in_tile) {
      K kk = s_key[i];
      uint32_t g = s_goff[(uint32_t)(kk >> a.shift) & a.mask] + i;
      gpos[k] = g;
      if (UNPACK) {
        a.major_out[g] = (int32_t)(kk >> a.ks.b_bits);
        a.minor_out[g] = (int32_t)(kk & (((K)1 << a.ks.b_bits) - 1));
      } else {
        a.key_out[g] = kk;
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < RS_IPT; ++j) {
    uint32_t t = w * (64 * RS_IPT) + j * 64 + lane;
    if (t < in_tile) s_val[pos[j]] = val[j];
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < RS_IPT; ++k) {
    uint32_t i = k * RS_T + threadIdx.x;
    if (i < in_tile) a.val_out[gpos[k]] = s_val[i];
  }
}

template <typename K>
static void sort_generic(Env &env, const int32_t *row, const int32_t *col, const K *key_in, const float *val,
                         int64_t nnz, const KeySpec &ks, const SortOut &out, Flags *flags) {
  if (nnz <= 0 || !env.ok()) return;
  const bool unpack = out.major != nullptr;
  const int total_bits = ks.total_bits > 0 ? ks.total_bits : 1;
  const int npass = ceil_div(total_bits, RS_MAXBITS);
  const uint32_t nblocks = (uint32_t)ceil_div<int64_t>(nnz, RS_TILE);
  K *kbuf[2] = {nullptr, nullptr};
  uint32_t *vbuf[2] = {nullptr, nullptr};
  for (int i = 0; i < 2 && i < npass - 1; ++i) {
    kbuf[i] = env.temp<K>(nnz);
    vbuf[i] = env.temp<uint32_t>(nnz);
  }
  uint32_t *hist = env.temp<uint32_t>((size_t)RS_BINS * nblocks);
  uint32_t *totals = env.temp<uint32_t>((size_t)RS_BINS * npass);
  if (!env.ok()) return;
  fill_u32(env, totals, (uint64_t)RS_BINS * npass, 0);

  K *packed_out = sizeof(K) == 8 ? (K *)out.key64 : (K *)out.key32;
  int shift = 0;
  for (int p = 0; p < npass; ++p) {
    const int width = total_bits / npass + (p < total_bits % npass ? 1 : 0);
    const bool first = p == 0, last = p == npass - 1;
    PassArgs<K> a{};
    const bool from_coo = first && row != nullptr;
    a.row = from_coo ? row : nullptr;
    a.col = from_coo ? col : nullptr;
    a.key_in = first ? key_in : kbuf[(p - 1) & 1];
    a.val_in = first ? (const uint32_t *)val : vbuf[(p - 1) & 1];
    a.key_out = last ? (unpack ? nullptr : packed_out) : kbuf[p & 1];
    a.val_out = last ? (uint32_t *)out.val : vbuf[p & 1];
    a.major_out = last ? out.major : nullptr;
    a.minor_out = last ? out.minor : nullptr;
    a.n = (uint32_t)nnz; a.shift = shift; a.mask = (1u << width) - 1u; a.nblocks = nblocks;
    a.hist = hist; a.totals = totals + (size_t)p * RS_BINS; a.ks = ks; a.flags = flags;
    const double kb = sizeof(K);
    if (from_coo) US_LAUNCH(env, "radix_hist", 8.0 * nnz, (radix_hist_kernel<K, true>), nblocks, RS_T, a);
    else US_LAUNCH(env, "radix_hist", kb * nnz, (radix_hist_kernel<K, false>), nblocks, RS_T, a);
    US_LAUNCH(env, "radix_scan", 8.0 * (a.mask + 1.0) * nblocks, radix_scan_kernel, a.mask + 1, 256, hist,
              (const uint32_t *)a.totals, nblocks);
    const double rd = (from_coo ? 12.0 : kb + 4.0) * nnz, wr = ((last && unpack) ? 12.0 : kb + 4.0) * nnz;
    if (from_coo && last && unpack) US_LAUNCH(env, "radix_scatter", rd + wr, (radix_scatter_kernel<K, true, true>), nblocks, RS_T, a);
    else if (from_coo && last) US_LAUNCH(env, "radix_scatter", rd + wr, (radix_scatter_kernel<K, true, false>), nblocks, RS_T, a);
    else if (from_coo) US_LAUNCH(env, "radix_scatter", rd + wr, (radix_scatter_kernel<K, true, false>), nblocks, RS_T, a);
    else if (last && unpack) US_LAUNCH(env, "radix_scatter", rd + wr, (radix_scatter_kernel<K, false, true>), nblocks, RS_T, a);
    else US_LAUNCH(env, "radix_scatter", rd + wr, (radix_scatter_kernel<K, false, false>), nblocks, RS_T, a);
    shift += width;
  }
}

void sort_coo(Env &env, const int32_t *row, const int32_t *col, const float *val, int64_t nnz,
              const KeySpec &ks, const SortOut &out, Flags *flags_dev) {
  const bool k32 = ks.total_bits <= 32 && out.key64 == nullptr;
  if (k32) sort_generic<uint32_t>(env, row, col, nullptr, val, nnz, ks, out, flags_dev);
  else sort_generic<uint64_t>(env, row, col, nullptr, val, nnz, ks, out, flags_dev);
}

// ascending sort of 32-bit keys (no payload of interest)
void sort_u32(Env &env, const uint32_t *key, int64_t n, int bits, uint32_t *out) {
  if (n <= 0) return;
  KeySpec ks{};
  ks.total_bits = bits;
  float *dummy_in = env.temp<float>(n), *dummy_out = env.temp<float>(n);
  if (!env.ok()) return;
  SortOut so{};
  so.key32 = out; so.val = dummy_out;
  sort_generic<uint32_t>(env, nullptr, nullptr, key, dummy_in, n, ks, so, nullptr);
}

void sort_keys(Env &env, const uint64_t *key, const float *val, int64_t nnz, const KeySpec &ks,
               const SortOut &out, Flags *flags_dev) {
  sort_generic<uint64_t>(env, nullptr, nullptr, key, val, nnz, ks, out, flags_dev);
}

}  // namespace us
