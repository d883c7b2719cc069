/* A plain C99 caller of the library's C ABI: built and run by tests/test_c_caller.py (no GPU needed:
 * only host functions and argument checks that return before any launch are called). */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <stdint.h>
#include "mpq.h"

#define CHECK(cond) do { if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

int main(void) {
  CHECK(mpq_version() >= 100);
  CHECK(strcmp(mpq_strerror(MPQ_OK), "ok") == 0);
  CHECK(strlen(mpq_strerror(MPQ_ERR_TOO_LARGE)) > 0);

  /* Eq. 2 on the host: sqrt(sse / n) / max|x| */
  CHECK(mpq_eqe(4.0, 16, 0.5) == 1.0);

  /* latency of a configuration = sum of its layers' table entries; size = parameters * bits / 8 */
  const double table[3 * 2] = {10.0, 6.0, 20.0, 15.0, 5.0, 4.0}; /* [layer][width] */
  const int pick[3] = {0, 1, 1};
  double us = 0.0;
  CHECK(mpq_latency_estimate(table, 3, 2, pick, &us) == MPQ_OK);
  CHECK(us == 10.0 + 15.0 + 4.0);
  const int64_t params[2] = {1000, 3000};
  const int bits[2] = {8, 4};
  double bytes = 0.0;
  CHECK(mpq_model_size_bytes(params, bits, 2, &bytes) == MPQ_OK);
  CHECK(bytes == 1000.0 + 1500.0);

  /* a sweep plan is built in host memory from descriptors; the device pointers are never touched */
  mpq_sweep_tensor t;
  memset(&t, 0, sizeof t);
  t.x = (const float*)(uintptr_t)0x10000;
  t.rows = 100;
  t.cols = 4096;
  t.absmax_row = (float*)(uintptr_t)0x20000;
  t.absmax_tensor = (float*)(uintptr_t)0x30000;
  t.sse_tensor = (double*)(uintptr_t)0x40000;
  t.sse_row = (double*)(uintptr_t)0x50000;
  const size_t need = mpq_sweep_plan_bytes(&t, 1);
  CHECK(need > 0);
  void* plan = malloc(need);
  CHECK(plan != NULL);
  CHECK(mpq_sweep_plan_build(&t, 1, plan, need) == MPQ_OK);
  CHECK(mpq_sweep_plan_build(&t, 1, plan, need - 1) == MPQ_ERR_WORKSPACE);
  CHECK(mpq_quant_error_batch_workspace_bytes(plan, MPQ_PER_TENSOR, 2, 8) == (size_t)7 * 7 * 8); /* 7 chunks of 64 K */

  /* argument errors come back before anything is launched */
  CHECK(mpq_calibrate_absmax_batch(plan, NULL, NULL) == MPQ_ERR_NULL);
  CHECK(mpq_calibrate_quant_error_rows_batch(plan, (const void*)(uintptr_t)0x60000, 1, 8, NULL) == MPQ_ERR_BITS);
  CHECK(mpq_quant_error(NULL, 4, 4, MPQ_PER_TENSOR, NULL, 2, 8, NULL, NULL, 0, NULL) == MPQ_ERR_NULL);
  free(plan);
  printf("c caller ok, library version %d\n", mpq_version());
  return 0;
}
