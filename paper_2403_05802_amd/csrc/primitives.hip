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
  if (!p) return;
  if (ctx && ctx->alloc) { if (ctx->free) ctx->free(p, ctx->user); }
  else (void)hipFree(p);
}
int g_lds_finish = -1;

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
  if (!env.prof || alg_bytes < env.prof->min_bytes) return;
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

}  // namespace us
