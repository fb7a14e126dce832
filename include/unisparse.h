/*
 * unisparse.h -- C ABI of the MI355X (gfx950) sparse-format customization library.
 *
 * The calls follow the paper's own statement of the problem (Section 3, Figure 3c and
 * Section 6): a matrix arrives as COO; `decompose` splits it into two COO sub-tensors by a
 * `sum` query over groups of entries; `convert` turns a COO tensor into the storage that a
 * format encoding (index map + trim/merge mutation primitives, Section 4.1, Figure 7)
 * describes, i.e. the size/ptr/idx/val arrays inferred by the rules of Section 5.1; a
 * compute op (SpMV / SpMM, Figure 3c and Section 7.2) then runs over the formatted tensor.
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer (HBM of the current HIP device) unless its
 *     comment says "host".  Structs themselves (us_ctx, us_coo, descriptors) live on the host.
 *   - The library never takes ownership of caller memory.  Arrays of a us_formatted are
 *     obtained through us_ctx.alloc and released by us_free through us_ctx.free.
 *   - Work is enqueued on us_ctx.hip_stream.  us_convert / us_decompose synchronise that
 *     stream before returning (output sizes and the validation flags are data dependent:
 *     one read-back for most conversions, up to three for a decomposition); us_spmv /
 *     us_spmm only enqueue.
 *   - A us_formatted carries scratch memory that its products use (partial sums of rows cut by
 *     a tile boundary): every product over one us_formatted must be enqueued on ONE stream, one
 *     call at a time (two host threads, or two streams, multiplying the same tensor race on
 *     that scratch; make a second us_formatted for the second stream).  The `const` of the
 *     product calls covers the matrix arrays, not that scratch.
 *   - An array of a us_formatted may be allocated larger than the count us_formatted_array
 *     reports (the stored-row arrays of DCSR are sized before their count is known), and
 *     several arrays of one us_formatted may lie in one allocation (each 256-byte aligned):
 *     a pointer from us_formatted_array is for reading, never for us_ctx.free.
 *   - Every call returns a us_status; on error no output object is produced (*out = NULL)
 *     and nothing is leaked.  The library never aborts, throws or prints.
 *   - Indices are int32, values fp32 (fp32 accumulate), element counts must stay below 2^31.
 */
#ifndef UNISPARSE_H
#define UNISPARSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t us_status;
enum {
  US_OK = 0,
  US_ERR_NULL = -1,             /* a required pointer is NULL                                   */
  US_ERR_SHAPE = -2,            /* non-positive dims, bad N / leading dimension, entry beyond a fixed ELL width */
  US_ERR_INDEX_RANGE = -3,      /* a COO coordinate lies outside nrows x ncols                   */
  US_ERR_UNSUPPORTED_DESC = -4, /* descriptor matches none of the supported encodings           */
  US_ERR_DUPLICATE = -5,        /* two COO entries share one coordinate                          */
  US_ERR_ALLOC = -6,            /* allocator returned NULL                                       */
  US_ERR_OVERFLOW = -7,         /* an output array would need 2^31 or more elements             */
  US_ERR_HIP = -8,              /* a HIP runtime call or kernel launch failed                    */
  US_ERR_FORMAT_MISMATCH = -9,  /* compute op not available for this formatted tensor            */
  US_ERR_SCRATCH_LIMIT = -10    /* us_spmv_noalloc: the product needs more scratch than US_NOALLOC_SCRATCH_BYTES */
};

/* Execution context.  alloc/free may be NULL: the library then uses hipMalloc/hipFree.
 * alloc must return device memory aligned to at least 256 bytes, or NULL on failure. */
typedef struct us_ctx {
  void *(*alloc)(size_t bytes, void *user);
  void (*free)(void *ptr, void *user);
  void *user;
  void *hip_stream; /* hipStream_t, NULL = the null stream */
  void *profile;    /* us_profile* or NULL: per-kernel HIP-event timing (see us_profile_*) */
  /* How the Sort step (Figure 8) of the conversions made through this context finishes.
   *   US_SORT_FINISH_AUTO (0, what a zeroed us_ctx gives): by the target tuple -- in LDS for blocked tuples
   *     (BCSR, BDIA and the blocked #sum queries), whole-array digit passes for (row, col) tuples;
   *   US_SORT_FINISH_LDS: whole-array digit passes over the top key bits only, every bucket of equal top bits
   *     is then finished inside LDS;
   *   US_SORT_FINISH_PASSES: whole-array digit passes over all key bits.
   * The finish pays off when entries spread evenly over the buckets (block rows of a FEM-like matrix: COO->BCSR
   * of 50 M entries 27 % faster); heavy rows of a power-law matrix need extra splitting passes and gain nothing.
   * Results are identical in every mode; an input the finish cannot take (more than 262,144 entries sharing
   * their top key bits, or 2,048 sharing 8 more) is sorted again with whole-array passes by the same call. */
  int32_t sort_finish;
} us_ctx;
enum { US_SORT_FINISH_AUTO = 0, US_SORT_FINISH_LDS = 1, US_SORT_FINISH_PASSES = 2 };

/* Unsorted COO input (Figure 7, #COO): borrowed device arrays of length nnz; coordinates unique. */
typedef struct us_coo {
  int64_t nrows, ncols, nnz;
  const int32_t *row; /* d0 of every entry */
  const int32_t *col; /* d1 of every entry */
  const float *val;
} us_coo;

/* One destination expression of an index map (Figure 5a): e = c0*d0 + c1*d1 + c, optionally
 * followed by "/ factor" (floor) or "% factor", or the indirect function of ELL (Figure 7:
 * sum + enum grouped by the affine part / factor, traversed by the other dimension / factor2: factor = factor2 = 1
 * numbers the entries of a row, ELL; factor = bh, factor2 = bw numbers the blocks of a block row, blocked ELL), or
 * the indirect function of CISR-plus (Section 7.2.4: sum + reorder + schedule of the groups of the affine part into
 * `factor` partitions). */
enum { US_E_AFFINE = 0, US_E_DIV = 1, US_E_MOD = 2, US_E_INDIRECT_ENUM = 3, US_E_INDIRECT_SCHEDULE = 4 };
typedef struct us_expr {
  int32_t kind;
  int32_t c0, c1, c;
  int32_t factor;
  int32_t factor2; /* US_E_INDIRECT_ENUM only (0 is read as 1) */
} us_expr;

/* Format encoding: index map (major level first) + trim(S,E) + merge(L...), Section 4.1.
 * Supported encodings (anything else -> US_ERR_UNSUPPORTED_DESC):
 *   COO  (d0,d1) trim(0,1)              CSR  (d0,d1) merge(0) trim(1,1)
 *   DCSR (d0,d1) merge(0) trim(0,1)     CSC / DCSC: the same with map (d1,d0)
 *   DIA  (d1-d0,d0) merge(0) trim(0,0)  DIA variant (d1-d0,d1)
 *   BCSR (d0/bh,d1/bw,d0%bh,d1%bw) merge(0,1) trim(1,1), 1 <= bh,bw <= 16
 *   ELL  (indirect(d1),d0,d1) merge(0) trim(0,0)
 *   BELL (indirect(d1/bw),d0/bh,d1/bw,d0%bh,d1%bw) merge(0) trim(0,0), 1 <= bh,bw <= 16: blocked ELL, the BELL of
 *        Section 7.2.2 (its encoding is in a figure that is not available: this library's reading).  The indirect
 *        level numbers the blocks of a block row by ascending block column: a size K (the most blocks a block row
 *        holds, or ell_width if > 0), a size ceil(nrows/bh), one block column per (slot, block row) (slot-major,
 *        -1 = no block), then the dense bh x bw inner levels: val[((k*nbr + br)*bh + r)*bw + c]
 *   BDIA (d0/b,d1-d0,d0%b) merge(0) trim(1,1), 1 <= b <= 16 (the blocked DIA of Figure 3c)
 *   CSB  (d0/bh,d1/bw,d0%bh,d1%bw) merge(1) trim(2,3), 1 <= bh,bw <= 65536 and fewer than 2^31 blocks:
 *        a dense grid of blocks (two sizes), one ptr over the blocks, (d0%bh, d1%bw) per entry
 *   CISR-plus (schedule(d0),d0,d1) merge(0,1) trim(1,2), 1 <= partitions <= 65536 (Section 7.2.4): rows that
 *        hold entries are ordered by their number of entries, most first (equal ones by ascending row), and
 *        dealt to the partitions in turn (the k-th goes to partition k mod P: this library's reading of
 *        the schedule query, of which the paper only requires balance); stored as a size P, a row level (ptr over the partitions, row
 *        indices ascending inside a partition) and a column level (ptr over the stored rows, column indices) */
typedef struct us_format_desc {
  int32_t nlevels;
  us_expr level[5];
  int32_t trim_s, trim_e; /* -1,-1 = no trim */
  uint32_t merge_mask;    /* bit L set = merge(L) */
  int64_t ell_width;      /* ELL, BELL: 0 = longest (block) row, >0 = fixed number of slots */
} us_format_desc;

enum { US_F_COO = 0, US_F_CSR, US_F_DCSR, US_F_CSC, US_F_DCSC, US_F_DIA, US_F_DIA_VARIANT, US_F_BCSR, US_F_ELL, US_F_BDIA, US_F_CSB, US_F_CISR_PLUS, US_F_BELL };
/* Fill *out with the encoding of Figure 7 (Figure 3c for BDIA) for `format`; b0,b1 = block
 * height,width (BCSR, CSB, BELL), b0 = block height (BDIA), b0 = fixed width (ELL, 0 = longest row) or b0 = number of
 * partitions (CISR-plus).  host pointers. */
us_status us_desc_preset(int32_t format, int64_t b0, int64_t b1, us_format_desc *out);

/* Decomposition predicate: the `sum` query of Section 4.1.2 (groupBy map, stored entry -> 1)
 * compared with a threshold, as in unisparse.decompose(%A, %thld){query=#sum}; entries for
 * which it holds go to part A.
 *   US_P_SUM_GE_ABS              count(group) >= abs                     (the paper's %thld)
 *   US_P_SUM_GE_FRAC_OF_CAPACITY den*count(group) >= num*capacity(group), capacity = number of
 *                                in-bounds matrix positions of the group (diagonal length, ...)
 *   US_P_RANK_LT_ABS             rank of the entry in its row (ascending column) < abs
 *   US_P_RANK_LT_PERCENTILE      rank < K, K = nearest-rank num/den percentile of the row
 *                                lengths over all rows (empty rows included)
 * group maps supported: (d1-d0), (d0), (d1) for the sum predicates; (d0) for the rank ones;
 * (d0/b, d1-d0) with US_P_SUM_GE_ABS (the #sum query of Figure 3c) and (d0/bh, d1/bw) with US_P_SUM_GE_ABS
 * (entries per block, the threshold of the BELL/COO case study of Section 7.2.2), 1 <= b, bh, bw <= 16;
 * a part A stored as BDIA(b) / BCSR(bh,bw) / BELL(bh,bw) then needs no second sort. */
enum { US_P_SUM_GE_ABS = 0, US_P_SUM_GE_FRAC_OF_CAPACITY = 1, US_P_RANK_LT_ABS = 2, US_P_RANK_LT_PERCENTILE = 3 };
typedef struct us_predicate {
  us_expr group[2];
  int32_t ngroup;
  int32_t kind;
  int64_t num, den, abs;
} us_predicate;

typedef struct us_formatted us_formatted; /* opaque; owns arrays obtained through us_ctx.alloc */

/* COO -> target format (Figure 8: index-map alignment incl. Sort, then Trim/Fill/Merge).
 * The result is canonical: ordered by the full target tuple whatever the input order.
 * Errors: NULL, SHAPE, INDEX_RANGE, DUPLICATE, UNSUPPORTED_DESC, OVERFLOW, ALLOC, HIP. */
us_status us_convert(const us_ctx *ctx, const us_coo *coo, const us_format_desc *target, us_formatted **out);

/* Conversion between any two supported formats through the COO hub (Section 5.2: reversibility
 * and reachability; the cases of Table 5 such as CSR->CSC or DCSC->BCSR): the source is expanded
 * back to COO on the device (Split of ptr levels, inverse index map, bounds guard; slots of dense
 * levels holding +-0.0 and ELL pads are padding and are dropped), then converted as by us_convert.
 * The source is left untouched. */
us_status us_convert_formatted(const us_ctx *ctx, const us_formatted *src, const us_format_desc *target,
                               us_formatted **out);

/* decompose + convert of a hybrid (Figure 3c lines "decompose" and "convert"): entries that
 * satisfy `pred` form part A (stored as desc_a), the rest part B (desc_b).  Both parts keep
 * the shape of the whole matrix, so A*x = out_a*x + out_b*x. */
us_status us_decompose(const us_ctx *ctx, const us_coo *coo, const us_format_desc *desc_a,
                       const us_format_desc *desc_b, const us_predicate *pred,
                       us_formatted **out_a, us_formatted **out_b);

/* y = A x (accumulate = 0) or y += A x (accumulate != 0; the generic op of Figure 3c reads Y).
 * x: ncols floats, y: nrows floats, both device.  For a hybrid call it on part A, then on
 * part B with accumulate = 1.
 * Row-grouped layouts (COO, CSR, DCSR, CISR-plus, DIA and its variant, BCSR, BDIA, ELL, BELL) add in a fixed order: two
 * calls give the same bits.  Layouts whose leaves are not grouped by output row (CSC, DCSC, column-major
 * COO, CSB) scatter with fp32 atomics, so the last bits may differ from call to call; this holds for
 * us_spmm as well. */
us_status us_spmv(const us_ctx *ctx, const us_formatted *A, const float *x, float *y, int32_t accumulate);

/* us_spmv for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical results; the scratch of the
 * product (partial sums of rows cut by a tile boundary, which us_spmv keeps with the tensor and may have to
 * allocate or grow through us_ctx.alloc) is a fixed array of US_NOALLOC_SCRATCH_BYTES in the device memory of
 * every GPU the library runs on, held until the process ends.  The call makes no hipMalloc / hipFree, never
 * calls us_ctx.alloc / us_ctx.free and ignores us_ctx.profile (event creation allocates).
 * Limit: a product that needs more scratch returns US_ERR_SCRATCH_LIMIT and enqueues nothing.  Compressed rows
 * (CSR, DCSR, CISR-plus) take 8 bytes per 2048 stored rows + entries and row-major COO 8 bytes per 2048 entries,
 * each half rounded up to 256 bytes: tensors of up to 2^31 - 2048 rows + entries fit; the other layouts take none.
 * All calls on one GPU share the array: two calls that overlap in time on one GPU (two streams, two threads)
 * race on it, whatever tensors they multiply. */
#define US_NOALLOC_SCRATCH_BYTES (8u << 20)
us_status us_spmv_noalloc(const us_ctx *ctx, const us_formatted *A, const float *x, float *y, int32_t accumulate);

/* Y = A X or Y += A X with dense row-major X (ncols x N, leading dimension ldx >= N) and
 * Y (nrows x N, ldy >= N), device (Section 7.2.2). */
us_status us_spmm(const us_ctx *ctx, const us_formatted *A, const float *X, int64_t N, int64_t ldx,
                  float *Y, int64_t ldy, int32_t accumulate);

/* Level-wise view of the storage (Section 5.1).  level = tree level, which = one of:
 *   US_A_SIZE: *count = extent of a dense level (dev_ptr = NULL)
 *   US_A_PTR / US_A_IDX: int32 device array of *count entries
 *   US_A_VAL: fp32 value array (level ignored)
 * An array the format does not have yields *dev_ptr = NULL, *count = -1 and US_OK.
 * dtype (may be NULL) receives the element type of the array: US_T_INT32 for ptr / idx, US_T_FLOAT32 for val,
 * US_T_NONE for a size or an absent array. */
enum { US_A_SIZE = 0, US_A_PTR = 1, US_A_IDX = 2, US_A_VAL = 3 };
enum { US_T_NONE = 0, US_T_INT32 = 1, US_T_FLOAT32 = 2 };
us_status us_formatted_array(const us_formatted *f, int32_t level, int32_t which,
                             const void **dev_ptr, int64_t *count, int32_t *dtype);
us_status us_formatted_info(const us_formatted *f, int64_t *nrows, int64_t *ncols, int64_t *nnz,
                            us_format_desc *desc);
/* Releases a us_formatted (NULL is allowed).  us_free waits for ctx->hip_stream first, since products enqueued
 * earlier may still read the arrays: safe with any allocator.  us_free_async does not wait: for an allocator
 * whose free is ordered with that stream (memory freed while enqueued work still uses it is not handed to another
 * stream or to the host before that work is done -- PyTorch's caching allocator is such, for the stream the
 * memory was allocated on, and so is hipFreeAsync on the same stream); with hipFree itself the two are the same,
 * as it waits by itself. */
void us_free(const us_ctx *ctx, us_formatted *f);
void us_free_async(const us_ctx *ctx, us_formatted *f);
const char *us_status_str(us_status s); /* static storage */

/* Optional per-kernel timing: HIP events recorded on ctx->hip_stream around every kernel the
 * library launches while ctx->profile is set.  us_profile_collect synchronises the recorded
 * events and folds them into per-kernel totals; entry i (0 <= i < *n) is then read with
 * us_profile_entry: name (static storage), number of launches, summed milliseconds and the
 * summed algorithmic bytes (bytes each launch must read + write at least once). */
typedef struct us_profile us_profile;
us_status us_profile_create(us_profile **out);
void us_profile_destroy(us_profile *p);
us_status us_profile_reset(us_profile *p);
/* Only launches whose algorithmic bytes reach min_bytes are timed (0 = all): lets a timed region keep
 * the per-launch cost of event recording off the many tiny kernels.  With a threshold set the two
 * events of a launch travel in its dispatch (start and end of that kernel, nothing added to the
 * queue); with 0 they are recorded on the stream before and after the launch. */
us_status us_profile_set_min_bytes(us_profile *p, double min_bytes);
us_status us_profile_collect(us_profile *p, int32_t *n);
us_status us_profile_entry(const us_profile *p, int32_t i, const char **name, int64_t *launches,
                           double *total_ms, double *alg_bytes);

#ifdef __cplusplus
}
#endif
#endif /* UNISPARSE_H */
