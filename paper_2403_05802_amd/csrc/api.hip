// extern "C" entry points: argument checks, then the implementations in convert / spmv / spmm.
#include "common.h"

using namespace us;

extern "C" {

const char *us_status_str(us_status s) {
  switch (s) {
    case US_OK: return "US_OK";
    case US_ERR_NULL: return "US_ERR_NULL";
    case US_ERR_SHAPE: return "US_ERR_SHAPE";
    case US_ERR_INDEX_RANGE: return "US_ERR_INDEX_RANGE";
    case US_ERR_UNSUPPORTED_DESC: return "US_ERR_UNSUPPORTED_DESC";
    case US_ERR_DUPLICATE: return "US_ERR_DUPLICATE";
    case US_ERR_ALLOC: return "US_ERR_ALLOC";
    case US_ERR_OVERFLOW: return "US_ERR_OVERFLOW";
    case US_ERR_HIP: return "US_ERR_HIP";
    case US_ERR_FORMAT_MISMATCH: return "US_ERR_FORMAT_MISMATCH";
    case US_ERR_SCRATCH_LIMIT: return "US_ERR_SCRATCH_LIMIT";
    default: return "US_ERR_UNKNOWN";
  }
}

static us_expr mk(int kind, int c0, int c1, int factor) {
  us_expr e{};
  e.kind = kind; e.c0 = c0; e.c1 = c1; e.c = 0; e.factor = factor; e.factor2 = 1;
  return e;
}

us_status us_desc_preset(int32_t format, int64_t b0, int64_t b1, us_format_desc *out) {
  if (!out) return US_ERR_NULL;
  us_format_desc d{};
  d.trim_s = d.trim_e = -1;
  const us_expr r = mk(US_E_AFFINE, 1, 0, 1), c = mk(US_E_AFFINE, 0, 1, 1), dg = mk(US_E_AFFINE, -1, 1, 1);
  switch (format) {
    case US_F_COO: d.nlevels = 2; d.level[0] = r; d.level[1] = c; d.trim_s = 0; d.trim_e = 1; break;
    case US_F_CSR: d.nlevels = 2; d.level[0] = r; d.level[1] = c; d.trim_s = 1; d.trim_e = 1; d.merge_mask = 1; break;
    case US_F_DCSR: d.nlevels = 2; d.level[0] = r; d.level[1] = c; d.trim_s = 0; d.trim_e = 1; d.merge_mask = 1; break;
    case US_F_CSC: d.nlevels = 2; d.level[0] = c; d.level[1] = r; d.trim_s = 1; d.trim_e = 1; d.merge_mask = 1; break;
    case US_F_DCSC: d.nlevels = 2; d.level[0] = c; d.level[1] = r; d.trim_s = 0; d.trim_e = 1; d.merge_mask = 1; break;
    case US_F_DIA: d.nlevels = 2; d.level[0] = dg; d.level[1] = r; d.trim_s = 0; d.trim_e = 0; d.merge_mask = 1; break;
    case US_F_DIA_VARIANT: d.nlevels = 2; d.level[0] = dg; d.level[1] = c; d.trim_s = 0; d.trim_e = 0; d.merge_mask = 1; break;
    case US_F_BCSR:
      if (b0 < 1 || b1 < 1 || b0 > 16 || b1 > 16) return US_ERR_UNSUPPORTED_DESC;
      d.nlevels = 4;
      d.level[0] = mk(US_E_DIV, 1, 0, (int)b0); d.level[1] = mk(US_E_DIV, 0, 1, (int)b1);
      d.level[2] = mk(US_E_MOD, 1, 0, (int)b0); d.level[3] = mk(US_E_MOD, 0, 1, (int)b1);
      d.trim_s = 1; d.trim_e = 1; d.merge_mask = 3;
      break;
    case US_F_CSB:
      if (b0 < 1 || b1 < 1 || b0 > 65536 || b1 > 65536) return US_ERR_UNSUPPORTED_DESC;
      d.nlevels = 4;
      d.level[0] = mk(US_E_DIV, 1, 0, (int)b0); d.level[1] = mk(US_E_DIV, 0, 1, (int)b1);
      d.level[2] = mk(US_E_MOD, 1, 0, (int)b0); d.level[3] = mk(US_E_MOD, 0, 1, (int)b1);
      d.trim_s = 2; d.trim_e = 3; d.merge_mask = 2;
      break;
    case US_F_BDIA:
      if (b0 < 1 || b0 > 16) return US_ERR_UNSUPPORTED_DESC;
      d.nlevels = 3;
      d.level[0] = mk(US_E_DIV, 1, 0, (int)b0); d.level[1] = dg; d.level[2] = mk(US_E_MOD, 1, 0, (int)b0);
      d.trim_s = 1; d.trim_e = 1; d.merge_mask = 1;
      break;
    case US_F_ELL:
      if (b0 < 0) return US_ERR_UNSUPPORTED_DESC;
      d.nlevels = 3;
      d.level[0] = mk(US_E_INDIRECT_ENUM, 1, 0, 1); d.level[1] = r; d.level[2] = c;
      d.trim_s = 0; d.trim_e = 0; d.merge_mask = 1; d.ell_width = b0;
      break;
    case US_F_BELL:
      if (b0 < 1 || b1 < 1 || b0 > 16 || b1 > 16) return US_ERR_UNSUPPORTED_DESC;
      d.nlevels = 5;
      d.level[0] = mk(US_E_INDIRECT_ENUM, 1, 0, (int)b0); d.level[0].factor2 = (int)b1;
      d.level[1] = mk(US_E_DIV, 1, 0, (int)b0); d.level[2] = mk(US_E_DIV, 0, 1, (int)b1);
      d.level[3] = mk(US_E_MOD, 1, 0, (int)b0); d.level[4] = mk(US_E_MOD, 0, 1, (int)b1);
      d.trim_s = 0; d.trim_e = 0; d.merge_mask = 1; d.ell_width = 0;
      break;
    case US_F_CISR_PLUS:
      if (b0 < 1 || b0 > 65536) return US_ERR_UNSUPPORTED_DESC;
      d.nlevels = 3;
      d.level[0] = mk(US_E_INDIRECT_SCHEDULE, 1, 0, (int)b0); d.level[1] = r; d.level[2] = c;
      d.trim_s = 1; d.trim_e = 2; d.merge_mask = 3;
      break;
    default: return US_ERR_UNSUPPORTED_DESC;
  }
  *out = d;
  return US_OK;
}

us_status us_convert(const us_ctx *ctx, const us_coo *coo, const us_format_desc *target, us_formatted **out) {
  if (out) *out = nullptr;
  if (!ctx || !coo || !target || !out) return US_ERR_NULL;
  us_status s;
  { Env env(ctx); s = convert_impl(env, *coo, *target, out); }
  if (s == US_SORT_RETRY) { Env env(ctx); env.lds_finish = 0; env.dia_marks = true; s = convert_impl(env, *coo, *target, out); }
  return s;
}

us_status us_convert_formatted(const us_ctx *ctx, const us_formatted *src, const us_format_desc *target,
                               us_formatted **out) {
  if (out) *out = nullptr;
  if (!ctx || !src || !target || !out) return US_ERR_NULL;
  us_status s;
  { Env env(ctx); s = convert_formatted_impl(env, *src, *target, out); }
  if (s == US_SORT_RETRY) { Env env(ctx); env.lds_finish = 0; env.dia_marks = true; s = convert_formatted_impl(env, *src, *target, out); }
  return s;
}

us_status us_decompose(const us_ctx *ctx, const us_coo *coo, const us_format_desc *desc_a,
                       const us_format_desc *desc_b, const us_predicate *pred, us_formatted **out_a,
                       us_formatted **out_b) {
  if (out_a) *out_a = nullptr;
  if (out_b) *out_b = nullptr;
  if (!ctx || !coo || !desc_a || !desc_b || !pred || !out_a || !out_b) return US_ERR_NULL;
  us_status s;
  { Env env(ctx); s = decompose_impl(env, *coo, *desc_a, *desc_b, *pred, out_a, out_b); }
  if (s == US_SORT_RETRY) {
    Env env(ctx); env.lds_finish = 0; env.dia_marks = true;
    s = decompose_impl(env, *coo, *desc_a, *desc_b, *pred, out_a, out_b);
  }
  return s;
}

us_status us_spmv(const us_ctx *ctx, const us_formatted *A, const float *x, float *y, int32_t accumulate) {
  if (!ctx || !A || !x || !y) return US_ERR_NULL;
  Env env(ctx);
  return spmv_impl(env, *A, x, y, accumulate != 0);
}

us_status us_spmv_noalloc(const us_ctx *ctx, const us_formatted *A, const float *x, float *y, int32_t accumulate) {
  if (!ctx || !A || !x || !y) return US_ERR_NULL;
  Env env(ctx);
  return spmv_noalloc_impl(env, *A, x, y, accumulate != 0);
}

us_status us_spmm(const us_ctx *ctx, const us_formatted *A, const float *X, int64_t N, int64_t ldx, float *Y,
                  int64_t ldy, int32_t accumulate) {
  if (!ctx || !A || !X || !Y) return US_ERR_NULL;
  if (N <= 0 || ldx < N || ldy < N) return US_ERR_SHAPE;
  Env env(ctx);
  return spmm_impl(env, *A, X, N, ldx, Y, ldy, accumulate != 0);
}

us_status us_formatted_array(const us_formatted *f, int32_t level, int32_t which, const void **dev_ptr,
                             int64_t *count, int32_t *dtype) {
  if (!f || !dev_ptr || !count) return US_ERR_NULL;
  *dev_ptr = nullptr; *count = -1;
  if (dtype) *dtype = US_T_NONE;
  if (which == US_A_VAL) { *dev_ptr = f->val; *count = f->nval; if (dtype) *dtype = US_T_FLOAT32; return US_OK; }
  if (level < 0 || level >= f->nlevels) return US_ERR_SHAPE;
  const LevelStore &l = f->level[level];
  if (which == US_A_SIZE) { *count = l.size; return US_OK; }
  if (which == US_A_PTR) { if (l.ptr) { *dev_ptr = l.ptr; *count = l.nptr; if (dtype) *dtype = US_T_INT32; } return US_OK; }
  if (which == US_A_IDX) { if (l.idx) { *dev_ptr = l.idx; *count = l.nidx; if (dtype) *dtype = US_T_INT32; } return US_OK; }
  return US_ERR_SHAPE;
}

us_status us_formatted_info(const us_formatted *f, int64_t *nrows, int64_t *ncols, int64_t *nnz,
                            us_format_desc *desc) {
  if (!f) return US_ERR_NULL;
  if (nrows) *nrows = f->nrows;
  if (ncols) *ncols = f->ncols;
  if (nnz) *nnz = f->nnz;
  if (desc) *desc = f->desc;
  return US_OK;
}

void us_free(const us_ctx *ctx, us_formatted *f) {
  if (!f) return;
  Env env(ctx);
  env.sync();  // compute kernels may still read the arrays
  free_formatted(env, f);
}

void us_free_async(const us_ctx *ctx, us_formatted *f) {
  if (!f) return;
  Env env(ctx);
  free_formatted(env, f);   // the caller vouches that its free is ordered with the stream
}

// ------------------------------------------------------------------ profiling
struct us_profile { Profile p; };

us_status us_profile_create(us_profile **out) {
  if (!out) return US_ERR_NULL;
  *out = new us_profile();
  return US_OK;
}
void us_profile_destroy(us_profile *p) {
  if (!p) return;
  for (auto &q : p->p.pending) { (void)hipEventDestroy(q.a); (void)hipEventDestroy(q.b); }
  for (auto e : p->p.pool) (void)hipEventDestroy(e);
  delete p;
}
us_status us_profile_collect(us_profile *p, int32_t *n) {
  if (!p) return US_ERR_NULL;
  us_status st = US_OK;
  for (auto &q : p->p.pending) {
    float ms = 0.f;
    if (hipEventSynchronize(q.b) != hipSuccess || hipEventElapsedTime(&ms, q.a, q.b) != hipSuccess) st = US_ERR_HIP;
    auto &e = p->p.entries[q.name];
    e.launches += 1; e.ms += ms; e.bytes += q.bytes;
    p->p.pool.push_back(q.a);
    p->p.pool.push_back(q.b);
  }
  p->p.pending.clear();
  if (n) *n = (int32_t)p->p.entries.size();
  return st;
}
us_status us_profile_reset(us_profile *p) {
  if (!p) return US_ERR_NULL;
  us_status st = us_profile_collect(p, nullptr);
  for (auto &e : p->p.entries) { e.launches = 0; e.ms = 0.0; e.bytes = 0.0; }
  return st;
}
us_status us_profile_set_min_bytes(us_profile *p, double min_bytes) {
  if (!p) return US_ERR_NULL;
  p->p.min_bytes = min_bytes;
  return US_OK;
}
us_status us_profile_entry(const us_profile *p, int32_t i, const char **name, int64_t *launches, double *total_ms,
                           double *alg_bytes) {
  if (!p) return US_ERR_NULL;
  if (i < 0 || i >= (int32_t)p->p.entries.size()) return US_ERR_SHAPE;
  const auto &e = p->p.entries[i];
  if (name) *name = e.name;
  if (launches) *launches = e.launches;
  if (total_ms) *total_ms = e.ms;
  if (alg_bytes) *alg_bytes = e.bytes;
  return US_OK;
}

}  // extern "C"
