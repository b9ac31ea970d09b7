/* libfusedmm.so used from plain C: no Python, no torch, nothing but the HIP runtime for device memory.
 * The GCN pattern with unit edge values is an SpMM (Table III row 3): on a ring-with-hubs graph whose
 * features are small integers every sum is exact in fp32, so the result must equal a closed form bit for bit:
 *     Z[u][k] = sum over stored (u, v) of Y[v][k],   Y[v][k] = (v + k) mod 7.
 * Prints "ok" and returns 0 on success.
 *
 *   python -m paper_2011_06391_amd.build example && ./paper_2011_06391_amd/example_c_abi
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>

#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "../../include/fusedmm.h"

#define HIP_OK(x)                                                               \
  do {                                                                          \
    hipError_t e_ = (x);                                                        \
    if (e_ != hipSuccess) {                                                     \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);     \
      return 1;                                                                 \
    }                                                                           \
  } while (0)
#define FMM_OK(x)                                                               \
  do {                                                                          \
    int s_ = (x);                                                               \
    if (s_ != FUSEDMM_OK) {                                                     \
      printf("fusedmm: %s at line %d\n", fusedmm_status_string(s_), __LINE__);  \
      return 1;                                                                 \
    }                                                                           \
  } while (0)

int main(void) {
  const int64_t m = 5000, n = 5000;
  const int32_t d = 96; /* between two instance sizes: runs masked on the 128 instance */
  /* row u: its two ring neighbours; every 50th row a hub of 1500 entries (split into chunks / tiles) */
  int64_t* rowptr = (int64_t*)malloc((size_t)(m + 1) * sizeof(int64_t));
  int64_t nnz = 0;
  int64_t u;
  if (!rowptr) return 1;
  for (u = 0; u < m; ++u) {
    rowptr[u] = nnz;
    nnz += (u % 50 == 0) ? 1500 : 2;
  }
  rowptr[m] = nnz;
  int32_t* colidx = (int32_t*)malloc((size_t)nnz * sizeof(int32_t));
  float* values = (float*)malloc((size_t)nnz * sizeof(float));
  float* Y = (float*)malloc((size_t)n * d * sizeof(float));
  float* Z = (float*)malloc((size_t)m * d * sizeof(float));
  if (!colidx || !values || !Y || !Z) return 1;
  for (u = 0; u < m; ++u) {
    int64_t e = rowptr[u];
    if (u % 50 == 0) {
      int64_t k;
      for (k = 0; k < 1500; ++k) colidx[e + k] = (int32_t)((3 * k + u % 3) % n); /* sorted: 3k + const < n */
    } else {
      int32_t a = (int32_t)((u + n - 1) % n), b = (int32_t)((u + 1) % n);
      colidx[e] = a < b ? a : b;
      colidx[e + 1] = a < b ? b : a;
    }
  }
  {
    int64_t i;
    for (i = 0; i < nnz; ++i) values[i] = 1.0f;
    for (i = 0; i < n * d; ++i) Y[i] = (float)(((i / d) + (i % d)) % 7);
  }

  int64_t* d_rowptr;
  int32_t* d_colidx;
  float *d_values, *d_Y, *d_Z;
  HIP_OK(hipMalloc((void**)&d_rowptr, (size_t)(m + 1) * sizeof(int64_t)));
  HIP_OK(hipMalloc((void**)&d_colidx, (size_t)nnz * sizeof(int32_t)));
  HIP_OK(hipMalloc((void**)&d_values, (size_t)nnz * sizeof(float)));
  HIP_OK(hipMalloc((void**)&d_Y, (size_t)n * d * sizeof(float)));
  HIP_OK(hipMalloc((void**)&d_Z, (size_t)m * d * sizeof(float)));
  HIP_OK(hipMemcpy(d_rowptr, rowptr, (size_t)(m + 1) * sizeof(int64_t), hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(d_colidx, colidx, (size_t)nnz * sizeof(int32_t), hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(d_values, values, (size_t)nnz * sizeof(float), hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(d_Y, Y, (size_t)n * d * sizeof(float), hipMemcpyHostToDevice));
  HIP_OK(hipMemset(d_Z, 0xff, (size_t)m * d * sizeof(float))); /* NaN everywhere: every entry must be written */

  fusedmm_plan_options_t options = {0};
  options.column_classes = 8; /* cut the hub rows by column class although Y is small */
  options.tile_row_min = 64;
  options.feature_dim_hint = d;
  fusedmm_plan_t* plan = NULL;
  FMM_OK(fusedmm_plan_create(&plan, m, n, nnz, d_rowptr, d_colidx, &options, NULL));
  int64_t tiled_rows = 0, partials = 0;
  FMM_OK(fusedmm_plan_stats(plan, NULL, NULL, NULL, NULL, &partials, &tiled_rows, NULL, NULL));
  fusedmm_ops_t ops;
  FMM_OK(fusedmm_ops_preset(FUSEDMM_PATTERN_GCN_SUM, &ops));
  FMM_OK(fusedmm_execute(plan, &ops, d, d_values, NULL, 0, d_Y, d, d_Z, d, NULL));
  HIP_OK(hipDeviceSynchronize());
  HIP_OK(hipMemcpy(Z, d_Z, (size_t)m * d * sizeof(float), hipMemcpyDeviceToHost));
  FMM_OK(fusedmm_plan_destroy(plan));

  int64_t wrong = 0;
  for (u = 0; u < m; ++u) {
    int32_t k;
    for (k = 0; k < d; ++k) {
      float want = 0.0f;
      int64_t e;
      for (e = rowptr[u]; e < rowptr[u + 1]; ++e) want += Y[(int64_t)colidx[e] * d + k];
      if (Z[u * d + k] != want) {
        if (wrong < 5) printf("Z[%lld][%d] = %g, expected %g\n", (long long)u, (int)k, (double)Z[u * d + k], (double)want);
        ++wrong;
      }
    }
  }
  printf("m = %lld, nnz = %lld, d = %d, tiled rows %lld, partial rows %lld: %s\n", (long long)m, (long long)nnz, (int)d,
         (long long)tiled_rows, (long long)partials, wrong ? "MISMATCH" : "ok");
  (void)hipFree(d_rowptr); (void)hipFree(d_colidx); (void)hipFree(d_values); (void)hipFree(d_Y); (void)hipFree(d_Z);
  free(rowptr); free(colidx); free(values); free(Y); free(Z);
  return wrong ? 1 : 0;
}
