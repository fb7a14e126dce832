// Device-wide building blocks: per-call environment, fill, exclusive scan, group pointers by
// binary search.
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
  if (!p || in_out(p)) return;
  if (ctx && ctx->alloc) { if (ctx->free) ctx->free(p, ctx->user); }
  else (void)hipFree(p);
}

void Env::reserve(size_t bytes) {
  if (arena_left >= bytes || bytes == 0) return;
  void *p = alloc_raw(granule(bytes));
  if (!p) return;   // temp() falls back to one allocation per array
  temps.push_back(p);
  arena = (char *)p; arena_left = granule(bytes);
}

void Env::reserve_out(size_t bytes) {
  if (out_base || bytes == 0) return;
  void *p = alloc_raw(granule(bytes));
  if (!p) return;
  out_base = out_next = (char *)p; out_bytes = out_left = granule(bytes);
}
void Env::adopt_out(us_formatted *f) {
  if (!out_base || !f) return;
  f->slab = out_base; f->slab_bytes = out_bytes;
  out_base = out_next = nullptr; out_bytes = out_left = 0;
}
void Env::drop_out() {
  if (!out_base) return;
  (void)hipStreamSynchronize(stream);  // kernels of a failed call may still write its arrays
  void *p = out_base;
  out_base = out_next = nullptr; out_bytes = out_left = 0;
  free_raw(p);
}

void Env::release_temps() {
  arena = nullptr; arena_left = 0;
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

LaunchScope::LaunchScope(Env &e, const char *name, double alg_bytes, bool in_dispatch_)
    : env(e), bytes(alg_bytes), in_dispatch(in_dispatch_) {
  if (!env.prof || alg_bytes < env.prof->min_bytes) return;
  // With every launch timed (no byte threshold) the events are recorded around the launches: in-dispatch pairs on
  // runs of short back-to-back kernels came out several times too long (a 5 us kernel reported with the duration
  // of the 180 us one that followed it), while on the few large launches that a threshold selects they agree
  // with rocprofv3's kernel trace to a few tenths of a microsecond.
  if (env.prof->min_bytes <= 0.0) in_dispatch = false;
  idx = env.prof->intern(name);
  a = env.prof->get_event();
  b = env.prof->get_event();
  if (!a || !b) { idx = -1; env.fail(US_ERR_HIP); return; }
  if (!in_dispatch) env.check(hipEventRecord(a, env.stream));
}
LaunchScope::~LaunchScope() {
  if (!env.prof || idx < 0) return;
  if (!in_dispatch) env.check(hipEventRecord(b, env.stream));
  env.prof->pending.push_back({idx, a, b, bytes});
}

// ------------------------------------------------------------------ fill
__global__ __launch_bounds__(256) void fill_u32_kernel(uint32_t *p, uint64_t n, uint32_t v) {
  uint64_t i = (uint64_t)blockIdx.x * 1024 + threadIdx.x;
#pragma unroll
  // MITIGATION ON A GUESS, NOT A FIX.  Once, in some thirty runs of the GPU tests, the last few elements of a
  // product whose output is cleared here and then added into came out short; which test, layout and kernel it was
  // is not known, reading every such path found no second writer and no ordering hole, and the case never showed
  // again.  Launches on one stream already order this kernel's write-back before the next kernel, so these
  // device-scope (write-through) stores and the wait for their acknowledgement change nothing unless that
  // guarantee failed.  They cost nothing measurable (the fill runs at the same rate) and stay until a cause is known.
  for (int k = 0; k < 4; ++k, i += 256)
    if (i < n) __hip_atomic_store(p + i, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
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

// single workgroup: exclusive scan of the per-tile sums in place, grand total to *total_dev.
// Every thread takes IPT consecutive sums per round (all its loads in flight together), so 24,000 of them are
// one round of 1024 x 32 instead of three of 1024 x 8: the kernel is one workgroup waiting on memory.
template <int IPT>
__global__ __launch_bounds__(1024) void scan_partials_kernel(uint32_t *partial, int64_t nb, int32_t *total_dev) {
  __shared__ uint32_t s_wave[1024 / 64 + 1];
  uint32_t carry = 0;
  for (int64_t base = 0; base < nb; base += 1024 * IPT) {
    const int64_t i0 = base + (int64_t)threadIdx.x * IPT;
    uint32_t v[IPT], s = 0, total;
#pragma unroll
    for (int k = 0; k < IPT; ++k) {
      v[k] = i0 + k < nb ? partial[i0 + k] : 0u;
      s += v[k];
    }
    uint32_t ex = block_exclusive_sum<1024>(s, s_wave, &total) + carry;
#pragma unroll
    for (int k = 0; k < IPT; ++k) {
      if (i0 + k < nb) partial[i0 + k] = ex;
      ex += v[k];
    }
    carry += total;
  }
  if (threadIdx.x == 0 && total_dev) *total_dev = (int32_t)carry;
}

__global__ __launch_bounds__(SCAN_T) void scan_apply_kernel(const int32_t *in, int32_t *out, int64_t n,
                                                           const uint32_t *partial) {
  __shared__ uint32_t s_wave[SCAN_T / 64 + 1];
  // blocked arrangement: thread t owns SCAN_IPT consecutive elements, moved as 16-byte vectors where the
  // arrays allow it (two load and two store instructions per thread instead of eight each)
  static_assert(SCAN_IPT == 8, "two int4 per thread");
  int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_IPT;
  const bool vec = base + SCAN_IPT <= n && (((uintptr_t)in | (uintptr_t)out) & 15) == 0;
  uint32_t v[SCAN_IPT], s = 0;
  if (vec) {
    const int4 a = *reinterpret_cast<const int4 *>(in + base), b = *reinterpret_cast<const int4 *>(in + base + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  } else {
#pragma unroll
    for (int k = 0; k < SCAN_IPT; ++k) v[k] = (base + k < n) ? (uint32_t)in[base + k] : 0u;
  }
#pragma unroll
  for (int k = 0; k < SCAN_IPT; ++k) s += v[k];
  uint32_t total;
  uint32_t ex = block_exclusive_sum<SCAN_T>(s, s_wave, &total) + partial[blockIdx.x];
  uint32_t o[SCAN_IPT];
#pragma unroll
  for (int k = 0; k < SCAN_IPT; ++k) {
    o[k] = ex;
    ex += v[k];
  }
  if (vec) {
    *reinterpret_cast<int4 *>(out + base) = make_int4((int)o[0], (int)o[1], (int)o[2], (int)o[3]);
    *reinterpret_cast<int4 *>(out + base + 4) = make_int4((int)o[4], (int)o[5], (int)o[6], (int)o[7]);
  } else {
#pragma unroll
    for (int k = 0; k < SCAN_IPT; ++k)
      if (base + k < n) out[base + k] = (int32_t)o[k];
  }
}

void scan_partials_launch(Env &env, uint32_t *partial, int64_t nb, int32_t *total_dev) {
  if (nb > 1024 * 8) US_LAUNCH(env, "scan_partials", 8.0 * nb, scan_partials_kernel<32>, 1, 1024, partial, nb, total_dev);
  else US_LAUNCH(env, "scan_partials", 8.0 * nb, scan_partials_kernel<8>, 1, 1024, partial, nb, total_dev);
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

// ------------------------------------------------------------------ the same pointers from one pass over the entries
// Entries sorted by (major, minor): wherever the major index steps from p to r, ptr[p+1..r] is that
// position; behind the last entry everything is n.  The same pass compares neighbours (check != 0:
// Flags::duplicate).  Short steps are written by the thread that finds them, long ones (runs of empty
// groups) by the whole workgroup afterwards.  Index arrays that failed validation may hold anything:
// every write stays inside ptr[0..ngroups], whatever they hold (entries of ptr may then stay unwritten;
// the call ends in US_ERR_INDEX_RANGE and ptr is only ever read as numbers before that).
constexpr int GP_IPT = 4, GP_SHORT = 16, GP_LIST = 256;

__global__ __launch_bounds__(256) void group_ptr_unique_kernel(const int32_t *major, const int32_t *minor, int64_t n,
                                                               int64_t ngroups, int32_t *ptr, int check,
                                                               Flags *flags) {
  __shared__ int32_t s_lo[GP_LIST], s_hi[GP_LIST], s_v[GP_LIST];
  __shared__ uint32_t s_n;
  // The list is not sorted when an earlier kernel of the call has already given up (a coordinate out of range, or a
  // sort that will be run again the plain way): every entry would then "step" over a random range of groups, and
  // what is a 30 us pass over sorted rows took 3.5 ms over 16.8 M unsorted ones.  The call's result is discarded.
  if (flags && (flags->index_range | flags->retry)) return;
  if (threadIdx.x == 0) s_n = 0;
  __syncthreads();
  auto emit = [&](int64_t lo, int64_t hi, int64_t v) {   // ptr[lo..hi] = v
    if (hi - lo < GP_SHORT) {
      for (int64_t q = lo; q <= hi; ++q) ptr[q] = (int32_t)v;
      return;
    }
    const uint32_t k = atomicAdd(&s_n, 1u);
    if (k < GP_LIST) {
      s_lo[k] = (int32_t)lo; s_hi[k] = (int32_t)hi; s_v[k] = (int32_t)v;
    } else {
      for (int64_t q = lo; q <= hi; ++q) ptr[q] = (int32_t)v;
    }
  };
  auto clampg = [&](int32_t m) { return (int64_t)((uint32_t)m < (uint64_t)ngroups ? m : ngroups - 1); };
  const int64_t i0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * GP_IPT;
  if (i0 < n) {
    int32_t m[GP_IPT], c[GP_IPT];
    const bool vec = i0 + GP_IPT <= n && (((uintptr_t)major | (uintptr_t)minor) & 15) == 0;
    if (vec) {
      const int4 mv = *reinterpret_cast<const int4 *>(major + i0);
      m[0] = mv.x; m[1] = mv.y; m[2] = mv.z; m[3] = mv.w;
      if (check) {
        const int4 cv = *reinterpret_cast<const int4 *>(minor + i0);
        c[0] = cv.x; c[1] = cv.y; c[2] = cv.z; c[3] = cv.w;
      } else {
        c[0] = c[1] = c[2] = c[3] = 0;
      }
    } else {
#pragma unroll
      for (int k = 0; k < GP_IPT; ++k) {
        const int64_t i = i0 + k < n ? i0 + k : n - 1;
        m[k] = major[i];
        c[k] = check ? minor[i] : 0;
      }
    }
    int64_t pm = i0 > 0 ? clampg(major[i0 - 1]) : -1;
    int32_t pm_raw = i0 > 0 ? major[i0 - 1] : -1, pc = i0 > 0 && check ? minor[i0 - 1] : -1;
    bool dup = false;
#pragma unroll
    for (int k = 0; k < GP_IPT; ++k) {
      if (i0 + k < n) {
        const int64_t r = clampg(m[k]);
        if (r > pm) emit(pm + 1, r, i0 + k);
        if (check && i0 + k > 0 && m[k] == pm_raw && c[k] == pc) dup = true;
        if (r > pm) pm = r;
        pm_raw = m[k]; pc = c[k];
      }
    }
    if (i0 + GP_IPT >= n) emit(pm + 1, ngroups, n);
    if (dup) flags->duplicate = 1;
  }
  __syncthreads();
  const uint32_t cnt = s_n < (uint32_t)GP_LIST ? s_n : (uint32_t)GP_LIST;
  for (uint32_t k = 0; k < cnt; ++k)
    for (int64_t q = (int64_t)s_lo[k] + threadIdx.x; q <= (int64_t)s_hi[k]; q += 256) ptr[q] = s_v[k];
}

void group_ptr_unique(Env &env, const int32_t *sorted_major, const int32_t *sorted_minor, int64_t n, int64_t ngroups,
                      int32_t *ptr, bool check, Flags *flags) {
  if (n <= 0) {
    fill_u32(env, (uint32_t *)ptr, (uint64_t)ngroups + 1, 0u);
    return;
  }
  US_LAUNCH(env, "ptr_unique", (check ? 8.0 : 4.0) * n + 4.0 * (ngroups + 1), group_ptr_unique_kernel,
            ceil_div<int64_t>(n, 256 * GP_IPT), 256, sorted_major, sorted_minor, n, ngroups, ptr, check ? 1 : 0, flags);
}

}  // namespace us
