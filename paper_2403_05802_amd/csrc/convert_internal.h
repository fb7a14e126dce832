// Shared by the conversion files (convert.hip, sum_query.hip, blocked.hip, cisr.hip, decompose.hip): the result of
// matching a format encoding, status flags, and the entry points of each family of layouts.
#pragma once
#include "common.h"

namespace us {

// what a format encoding was recognised as (Section 4.1 encodings restricted to the supported ones)
struct Plan {
  Pattern pattern;
  bool swapped = false;  // major dimension is d1
  int64_t bh = 1, bw = 1;
  int64_t ell_width = 0;
};

bool aff(const us_expr &e, int c0, int c1);                                   // e == c0*d0 + c1*d1
bool tile(const us_expr &e, int kind, int dim, int64_t *f, int64_t max_factor = 16);   // e == d_dim / f or d_dim % f
bool match_desc(const us_format_desc &d, Plan *p);
us_status validate_coo(const us_coo &coo);

// Kernels that end with one atomic per workgroup on a single counter run on at most ONE_COUNTER_GRID
// workgroups (grid-stride loops): same-address device atomics cost ~20 ns apiece on this part, so
// thousands of them would outlast the kernel's real work.
constexpr int ONE_COUNTER_GRID = 768;
inline int64_t one_counter_grid(int64_t items, int per_block) {
  const int64_t g = ceil_div<int64_t>(items, per_block);
  return g < ONE_COUNTER_GRID ? (g > 0 ? g : 1) : ONE_COUNTER_GRID;
}

// status flags of a call (device block, zeroed) and their one read-back
Flags *new_flags(Env &env);
bool read_flags(Env &env, Flags *dev, Flags *host);
us_status flag_status(const Flags &h);

// convert.hip: formats built from a (major, minor) sort
KeySpec rowcol_keyspec(const us_coo &coo, bool swapped);
void check_unique(Env &env, const int32_t *major, const int32_t *minor, int64_t n, Flags *flags);
void nonempty_flags(Env &env, const int32_t *ptr, int64_t n, int32_t *flag);
void max_group_len(Env &env, const int32_t *ptr, int64_t n, int32_t *out_max);
void sorted_ptr(Env &env, const int32_t *major, const int32_t *minor, int64_t n, int64_t ngroups, int32_t *ptr,
                bool check_dups, Flags *flags);
us_formatted *new_ell_of_rows(Env &env, const us_format_desc &desc, int64_t nrows, int64_t ncols, int64_t nnz, int64_t K,
                              int64_t clip, const int32_t *minor, const float *val, const int32_t *ptr, Flags *flags);
us_status build_from_sorted(Env &env, const Plan &plan, const us_format_desc &desc, int64_t nrows, int64_t ncols,
                            int64_t nnz, int32_t *major, int32_t *minor, float *val, Flags *flags, bool check_dups,
                            us_formatted **out, bool validated = false, bool major_is_temp = false);
us_status convert_with_plan(Env &env, const us_coo &coo, const Plan &plan, const us_format_desc &desc, us_formatted **out);

// sum_query.hip: the sum query over diagonals / rows / columns, DIA, and the decomposition it drives
enum { G_DIAG = 0, G_ROW = 1, G_COL = 2 };
struct CooLists { int32_t *r = nullptr, *c = nullptr; float *v = nullptr; };
CooLists alloc_lists(Env &env, int64_t n);
void free_lists(Env &env, CooLists &l);
us_status convert_dia(Env &env, const us_coo &coo, const Plan &plan, const us_format_desc &desc, Flags *flags,
                      us_formatted **out);
us_status decompose_sum(Env &env, const us_coo &coo, const Plan &pa, const us_format_desc &da, const Plan &pb,
                        const us_format_desc &db, const us_predicate &pred, int gkind, us_formatted **oa,
                        us_formatted **ob);

// blocked.hip: BCSR, BDIA, CSB
KeySpec blocked_keyspec(const Plan &plan, int64_t nrows, int64_t ncols);
// from entries sorted by the blocked tuple (keys built with ks)
us_status emit_blocked(Env &env, const Plan &plan, const us_format_desc &desc, int64_t nrows, int64_t ncols,
                       const KeySpec &ks, const uint64_t *skey, const float *sval, int64_t n, Flags *flags,
                       us_formatted **out, uint32_t *node_count = nullptr);   // node_count: SortOut::node_count when the sort filled it
us_status convert_blocked(Env &env, const us_coo &coo, const Plan &plan, const us_format_desc &desc, Flags *flags,
                          us_formatted **out);
us_status convert_csb(Env &env, const us_coo &coo, const Plan &plan, const us_format_desc &desc, Flags *flags,
                      us_formatted **out);

// cisr.hip
us_status convert_cisr(Env &env, const us_coo &coo, const Plan &plan, const us_format_desc &desc, Flags *flags,
                       us_formatted **out);

}  // namespace us
