// Internal host/device helpers shared by the translation units of the library.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <string.h>

#include <functional>
#include <string>
#include <vector>

#include "unisparse.h"

namespace us {

constexpr int WAVE = 64;

template <typename T>
__host__ __device__ inline T ceil_div(T a, T b) { return (a + b - 1) / b; }

inline int bits_for(uint64_t max_value) {  // bits needed to hold values 0..max_value
  int b = 0;
  while (max_value) { ++b; max_value >>= 1; }
  return b;
}

// ------------------------------------------------------------------ profiling
struct Profile {
  struct Pending { int name; hipEvent_t a, b; double bytes; };
  struct Entry { const char *name; int64_t launches; double ms; double bytes; };
  std::vector<Pending> pending;
  std::vector<hipEvent_t> pool;
  std::vector<Entry> entries;
  double min_bytes = 0.0;
  int intern(const char *name);
  hipEvent_t get_event();
};

// ------------------------------------------------------------------ per-call environment
struct Env {
  const us_ctx *ctx;
  hipStream_t stream;
  Profile *prof;
  us_status status = US_OK;
  std::vector<void *> temps;  // temporaries, released by release_temps() after the stream is idle
  int lds_finish;             // sort: finish buckets inside LDS: 1 always, 0 never (also the retry after Flags::retry),
                              // -1 by key layout (blocked tuples yes, (row, col) tuples no)
  bool dia_marks = false;     // DIA slab: find occupied slots with a byte map instead of the fill pattern (set for the retry)
  // set by the entry point that must not allocate: ensure_workspace hands out this memory instead of the tensor's
  // own scratch and fails with US_ERR_SCRATCH_LIMIT when a product needs more
  char *fixed_ws = nullptr; size_t fixed_ws_bytes = 0;

  explicit Env(const us_ctx *c)
      : ctx(c), stream(c ? (hipStream_t)c->hip_stream : nullptr), prof(c ? (Profile *)c->profile : nullptr),
        lds_finish(!c || c->sort_finish == US_SORT_FINISH_AUTO ? -1 : (c->sort_finish == US_SORT_FINISH_LDS ? 1 : 0)) {}
  ~Env() { release_temps(); drop_out(); }

  void *alloc_raw(size_t bytes);
  void free_raw(void *p);
  // Temporaries are carved out of a reserved block while it lasts (256-byte granules): a call into the
  // caller's allocator costs microseconds of host time during which the GPU may sit idle.
  char *arena = nullptr; size_t arena_left = 0;
  static size_t granule(size_t bytes) { return bytes < 256 ? 256 : (bytes + 255) & ~(size_t)255; }
  void reserve(size_t bytes);   // one allocation for the temp() calls that follow (no error if it fails)
  template <typename T>
  T *temp(size_t count) {  // never returns NULL for count == 0 callers: allocates at least 256 B
    const size_t need = granule(count * sizeof(T));
    if (arena_left >= need) {
      void *p = arena;
      arena += need; arena_left -= need;
      return (T *)p;
    }
    void *p = alloc_raw(need);
    if (!p) { fail(US_ERR_ALLOC); return nullptr; }
    temps.push_back(p);
    return (T *)p;
  }
  // The arrays of a result can come out of one block as well (reserve_out, for layouts whose array sizes are
  // known, or bounded, before the first kernel): the result then owns the block (us_formatted::slab, handed over
  // by adopt_out) and not its arrays one by one; free_raw leaves pointers into the block alone.  A block that no
  // result adopted is released with the temporaries.
  char *out_base = nullptr, *out_next = nullptr; size_t out_bytes = 0, out_left = 0;
  bool one_result = false;          // set by the entry point whose call produces exactly one result, which adopts the block
  void reserve_out(size_t bytes);   // (no error if it fails: owned() then allocates per array)
  bool in_out(const void *p) const {
    return out_base && (const char *)p >= out_base && (const char *)p < out_base + out_bytes;
  }
  void adopt_out(us_formatted *f);
  void drop_out();
  template <typename T>
  T *owned(size_t count) {  // for arrays that end up in a us_formatted
    const size_t need = granule(count * sizeof(T));
    if (out_left >= need) {
      void *p = out_next;
      out_next += need; out_left -= need;
      return (T *)p;
    }
    void *p = alloc_raw(need);
    if (!p) fail(US_ERR_ALLOC);
    return (T *)p;
  }
  void release_temps();
  bool ok() const { return status == US_OK; }
  void fail(us_status s) { if (status == US_OK) status = s; }
  void check(hipError_t e) { if (e != hipSuccess) fail(US_ERR_HIP); }
  void sync() { check(hipStreamSynchronize(stream)); }
};

// Times one kernel launch with a pair of events when profiling is on.  in_dispatch: the launch itself carries the
// events (hipExtLaunchKernelGGL: they take the start and end of that dispatch, no marker packets before and
// after it, which cost the queue ~5 us a pair); otherwise the events are recorded around whatever the scope holds.
struct LaunchScope {
  Env &env; int idx = -1; hipEvent_t a{}, b{}; double bytes; bool in_dispatch;
  LaunchScope(Env &e, const char *name, double alg_bytes, bool in_dispatch = false);
  ~LaunchScope();
  bool active() const { return idx >= 0; }
};

// US_LAUNCH(env, "name", algorithmic_bytes, kernel<...>, grid, block, args...)
#define US_LAUNCH(env, name, algbytes, kern, grid, block, ...)                         \
  do {                                                                                 \
    if ((env).ok()) {                                                                  \
      ::us::LaunchScope _ls((env), (name), (double)(algbytes), true);                  \
      if (_ls.active() && _ls.in_dispatch)                                             \
        hipExtLaunchKernelGGL(kern, dim3((unsigned)(grid)), dim3((unsigned)(block)), 0, \
                              (env).stream, _ls.a, _ls.b, 0, __VA_ARGS__);             \
      else                                                                             \
        hipLaunchKernelGGL(kern, dim3((unsigned)(grid)), dim3((unsigned)(block)), 0,   \
                           (env).stream, __VA_ARGS__);                                 \
      (env).check(hipGetLastError());                                                  \
    }                                                                                  \
  } while (0)

// ------------------------------------------------------------------ formatted tensor
enum Pattern { P_COO = 0, P_CSR, P_DCSR, P_DIA, P_BCSR, P_ELL, P_BDIA, P_CSB, P_CISR, P_BELL };

struct LevelStore {
  int64_t size = -1;      // extent of a dense level, -1 if none
  int32_t *ptr = nullptr; int64_t nptr = -1;
  int32_t *idx = nullptr; int64_t nidx = -1;
};

}  // namespace us

struct us_formatted {
  us_format_desc desc{};
  int pattern = 0;       // us::Pattern
  bool swapped = false;  // map (d1,d0): CSC / DCSC; DIA: slab indexed by d1 (DIA variant)
  int64_t nrows = 0, ncols = 0, nnz = 0;
  int nlevels = 0;
  us::LevelStore level[5];
  float *val = nullptr; int64_t nval = 0;
  // derived sizes
  int64_t nmajor = 0;   // CSR: rows (cols if swapped); DCSR, CISR-plus: stored rows; DIA: ndiag; BCSR/BDIA: block rows; ELL: K
  int64_t bh = 1, bw = 1, nblk = 0;   // BDIA: bh = block height, bw = 1, nblk = (block row, diagonal) nodes;
                                      // CSB: nblk = nmajor = blocks of the dense grid, level[1].size = blocks per block row;
                                      // BELL: nmajor = K slots, nblk = block rows
  // CSR / DCSR / CISR-plus (and CSC / DCSC by columns): where every tile starts on the merge path of row ends and non-zeros
  // (rows consumed before step t * tile), computed once at conversion
  int32_t *mp_split = nullptr; int64_t mp_tiles = 0;
  // scratch for the compute kernels (partial sums of rows cut by a tile boundary); grown on
  // demand by ensure_workspace and released by us_free.  One compute call at a time per tensor.
  mutable void *ws = nullptr; mutable size_t ws_bytes = 0;
  // one allocation that holds some or all of the arrays above (they are then not freed one by one), or null
  void *slab = nullptr; size_t slab_bytes = 0;
};

namespace us {

// Steps of the merged sequence {row ends} U {non-zeros} per workgroup of the compressed-row kernels
// (us_formatted::mp_split holds where every such tile starts)
constexpr int MP_TILE = 2048;

// Compressed rows as the product kernels see them: CSR (every row), DCSR and CISR-plus (a list of stored rows).
struct StoredRows { const int32_t *ptr, *idx, *row_ids; };
inline StoredRows stored_rows(const us_formatted &A) {
  if (A.pattern == P_CISR) return {A.level[2].ptr, A.level[2].idx, A.level[1].idx};
  if (A.pattern == P_DCSR) return {A.level[1].ptr, A.level[1].idx, A.level[0].idx};
  return {A.level[1].ptr, A.level[1].idx, nullptr};
}

// internal status: a fast path met an input it cannot take (Flags::retry): a bucket too large for the
// in-LDS finish of the sort, or a value carrying the bit pattern that marks empty DIA slots.  The entry
// point runs the call again with Env::lds_finish cleared and Env::dia_marks set.  Never returned to the caller.
constexpr us_status US_SORT_RETRY = -100;
enum { RETRY_SORT_LDS = 1, RETRY_DIA_MARKS = 2 };

// device-side status flags written by kernels, read back once per call
struct Flags {
  int32_t index_range;  // != 0: some coordinate out of range
  int32_t duplicate;    // != 0: two equal keys
  int32_t ell_overflow; // != 0: an entry's rank >= fixed ELL width
  int32_t retry;        // != 0: a fast path met an input it cannot take (RETRY_*); the entry point runs the call again without them
  int32_t scalar[4];    // data-dependent sizes (nnr, ndiag, nblk, K, nnz_a ...)
};

// primitives.hip / sort.hip
void fill_u32(Env &env, uint32_t *p, uint64_t n, uint32_t v);
void exclusive_scan_i32(Env &env, const int32_t *in, int32_t *out, int64_t n, int32_t *total_dev);
// in-place exclusive scan of nb per-tile sums by one workgroup; grand total to *total_dev
void scan_partials_launch(Env &env, uint32_t *partial, int64_t nb, int32_t *total_dev);
void lower_bound_ptr(Env &env, const int32_t *sorted_major, int64_t n, int64_t ngroups, int32_t *ptr);
// the same ptr from one pass over sorted entries, which also flags equal neighbours if `check`
void group_ptr_unique(Env &env, const int32_t *sorted_major, const int32_t *sorted_minor, int64_t n, int64_t ngroups,
                      int32_t *ptr, bool check, Flags *flags);

// how the 64/32-bit sort key is built from a COO entry
struct KeySpec {
  int mode;        // 0: (a,b) with a = row (or col if swap), b = the other; 1: block (a/bh, b/bw, a%bh, b%bw);
                   // 2: blocked diagonal (a/bh, b-a+a_extent-1, a%bh)
  int swap;        // 1: a = col, b = row
  int b_bits;      // bits of b (mode 0) / of b/bw (mode 1)
  int ih_bits, iw_bits;
  uint32_t bh, bw;
  uint32_t a_extent, b_extent;  // for range validation: row < a_extent ... (after swap)
  int total_bits;
};

// Sort COO entries by key.  Output either unpacked (major, minor, val) or (key, val).
// Returns true when the sort itself has looked for equal keys (Flags::duplicate).
struct SortOut {
  int32_t *major = nullptr, *minor = nullptr;  // unpacked output (mode 0 only)
  uint64_t *key64 = nullptr; uint32_t *key32 = nullptr;  // packed output
  float *val = nullptr;
  // Unpacked output whose arrays are not there yet: `late` sets major, minor and val and is called once all but
  // the last step of the sort are enqueued (an allocation made then costs no idle time on the GPU).  After a
  // failure inside it (Env::status) nothing more is launched.
  std::function<void(SortOut &)> late;
  // Blocked tuples, packed output: node_count[t] (zeroed by the sort) receives the number of entries of output tile
  // t (NODE_TILE consecutive entries) whose node key -- the key without its in-block bits -- differs from their
  // predecessor's, i.e. the nodes that start in the tile.  Only the finish inside LDS counts them (it has the sorted
  // keys at hand): *node_counted says whether it did.
  uint32_t *node_count = nullptr; bool *node_counted = nullptr;
};
constexpr int NODE_TILE_SHIFT = 11, NODE_TILE = 1 << NODE_TILE_SHIFT;
bool sort_coo(Env &env, const int32_t *row, const int32_t *col, const float *val, int64_t nnz,
              const KeySpec &ks, const SortOut &out, Flags *flags_dev);
// what a whole-array sort of nnz entries takes from Env::temp (for Env::reserve by a caller with temporaries of its own)
size_t sort_temp_bytes(int64_t nnz);
// stable ascending sort of 32-bit keys with a 32-bit payload that travels with its key
void sort_u32_payload(Env &env, const uint32_t *key, const uint32_t *payload, int64_t n, int bits, uint32_t *key_out,
                      uint32_t *payload_out, Flags *flags_dev);
// convert.hip
us_status convert_impl(Env &env, const us_coo &coo, const us_format_desc &desc, us_formatted **out);
us_status decompose_impl(Env &env, const us_coo &coo, const us_format_desc &da, const us_format_desc &db,
                         const us_predicate &pred, us_formatted **oa, us_formatted **ob);
void free_formatted(Env &env, us_formatted *f);
us_status convert_formatted_impl(Env &env, const us_formatted &src, const us_format_desc &desc, us_formatted **out);

// device scratch attached to a formatted tensor, at least `bytes` large (contents undefined)
void *ensure_workspace(Env &env, const us_formatted &A, size_t bytes);

// spmv.hip / spmm.hip
// fills mp_split for row-major CSR / DCSR.  With nmajor_dev the number of stored rows is still on the device
// (at most nmajor_cap): mp_split is sized for the cap and the caller sets nmajor and mp_tiles once it knows.
void spmv_prepare(Env &env, us_formatted *f, const int32_t *nmajor_dev = nullptr, int64_t nmajor_cap = 0);
int64_t spmv_tiles(int64_t nmajor, int64_t nnz);
us_status spmv_impl(Env &env, const us_formatted &A, const float *x, float *y, bool accumulate);
us_status spmv_noalloc_impl(Env &env, const us_formatted &A, const float *x, float *y, bool accumulate);
us_status spmm_impl(Env &env, const us_formatted &A, const float *X, int64_t N, int64_t ldx, float *Y,
                    int64_t ldy, bool accumulate);
// scratch the entry-balanced product (row-major COO, CSR, DCSR) takes from ensure_workspace; vec = columns per lane
size_t entry_balanced_scratch_bytes(int64_t nnz, int64_t N, int vec);

}  // namespace us
