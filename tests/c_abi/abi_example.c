/* The library used from plain C, without PyTorch: device memory from hipMalloc (the context's allocator
 * callbacks are NULL, so the library allocates with hipMalloc too), the null stream.
 *
 * Input: the 5x4 matrix A of the paper's figures (Section 4.2 prints its COO traversal), entries handed
 * over in scrambled order.  Prints the CSR arrays (Figure 7, #CSR), the DIA offsets of a COO -> CSR -> DIA
 * chain (Section 5.2, conversion through the COO hub) and y = A x; the test compares the text with what
 * the definition of the formats gives by hand. */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>

#include "unisparse.h"

#define HIP_OK(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { \
  fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_)); return 2; } } while (0)
#define US_OK_(call) do { us_status s_ = (call); if (s_ != US_OK) { \
  fprintf(stderr, "%s: %s\n", #call, us_status_str(s_)); return 3; } } while (0)

static int print_i32(const char *name, const void *dev, int64_t n) {
  int32_t *h = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
  HIP_OK(hipMemcpy(h, dev, sizeof(int32_t) * (size_t)n, hipMemcpyDeviceToHost));
  printf("%s", name);
  for (int64_t i = 0; i < n; ++i) printf(" %d", h[i]);
  printf("\n");
  free(h);
  return 0;
}
static int print_f32(const char *name, const void *dev, int64_t n) {
  float *h = (float *)malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));
  HIP_OK(hipMemcpy(h, dev, sizeof(float) * (size_t)n, hipMemcpyDeviceToHost));
  printf("%s", name);
  for (int64_t i = 0; i < n; ++i) printf(" %g", h[i]);
  printf("\n");
  free(h);
  return 0;
}

int main(void) {
  /* A: (0,0)=1 (1,1)=2 (2,1)=3 (2,2)=4 (2,3)=5 (4,3)=6, scrambled */
  const int32_t row[6] = {2, 4, 0, 2, 1, 2}, col[6] = {3, 3, 0, 1, 1, 2};
  const float val[6] = {5, 6, 1, 3, 2, 4}, x[4] = {1, 10, 100, 1000};
  int32_t *d_row, *d_col;
  float *d_val, *d_x, *d_y;
  HIP_OK(hipMalloc((void **)&d_row, sizeof row));
  HIP_OK(hipMalloc((void **)&d_col, sizeof col));
  HIP_OK(hipMalloc((void **)&d_val, sizeof val));
  HIP_OK(hipMalloc((void **)&d_x, sizeof x));
  HIP_OK(hipMalloc((void **)&d_y, 5 * sizeof(float)));
  HIP_OK(hipMemcpy(d_row, row, sizeof row, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(d_col, col, sizeof col, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(d_val, val, sizeof val, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(d_x, x, sizeof x, hipMemcpyHostToDevice));

  us_ctx ctx = {0};
  us_coo coo = {5, 4, 6, d_row, d_col, d_val};
  us_format_desc csr_desc, dia_desc;
  US_OK_(us_desc_preset(US_F_CSR, 0, 0, &csr_desc));
  US_OK_(us_desc_preset(US_F_DIA, 0, 0, &dia_desc));

  us_formatted *csr = NULL, *dia = NULL;
  US_OK_(us_convert(&ctx, &coo, &csr_desc, &csr));
  const void *p; int64_t n; int32_t t;
  US_OK_(us_formatted_array(csr, 1, US_A_PTR, &p, &n, &t));
  if (t != US_T_INT32) { printf("csr.ptr reported with element type %d\n", (int)t); return 2; }
  if (print_i32("csr.ptr", p, n)) return 2;
  US_OK_(us_formatted_array(csr, 1, US_A_IDX, &p, &n, NULL));
  if (print_i32("csr.idx", p, n)) return 2;
  US_OK_(us_formatted_array(csr, 0, US_A_VAL, &p, &n, &t));
  if (t != US_T_FLOAT32) { printf("csr.val reported with element type %d\n", (int)t); return 2; }
  if (print_f32("csr.val", p, n)) return 2;

  US_OK_(us_spmv(&ctx, csr, d_x, d_y, 0));
  HIP_OK(hipDeviceSynchronize());
  if (print_f32("y", d_y, 5)) return 2;

  US_OK_(us_convert_formatted(&ctx, csr, &dia_desc, &dia));
  US_OK_(us_formatted_array(dia, 0, US_A_IDX, &p, &n, NULL));
  if (print_i32("dia.offsets", p, n)) return 2;
  US_OK_(us_formatted_array(dia, 0, US_A_VAL, &p, &n, NULL));
  if (print_f32("dia.val", p, n)) return 2;
  US_OK_(us_spmv(&ctx, dia, d_x, d_y, 0));
  HIP_OK(hipDeviceSynchronize());
  if (print_f32("y_dia", d_y, 5)) return 2;

  /* a coordinate outside the matrix is reported, not executed */
  us_coo bad = {2, 4, 6, d_row, d_col, d_val};
  us_formatted *none = NULL;
  printf("bad %s\n", us_status_str(us_convert(&ctx, &bad, &csr_desc, &none)));

  us_free(&ctx, csr);
  us_free(&ctx, dia);
  HIP_OK(hipFree(d_row)); HIP_OK(hipFree(d_col)); HIP_OK(hipFree(d_val)); HIP_OK(hipFree(d_x)); HIP_OK(hipFree(d_y));
  return 0;
}
