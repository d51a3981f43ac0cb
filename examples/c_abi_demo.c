/*
 * Plain C program against the C ABI of libspt (include/spt.h): builds the 4 x 6 CSR matrix
 *     row 0: (0,0)=5 (0,1)=1      row 1: (1,0)=7 (1,1)=3
 *     row 2: (none)               row 3: (3,0)=8 (3,3)=4 (3,4)=9
 * on the device, multiplies it by x = (1,2,3,4,5,6), adds it to itself (sparse result) and
 * prints the results. No Python, no torch: hipMalloc / hipMemcpy and the library only.
 * Build: see paper_1804_10112_amd/build.py (build_example).
 */
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>

#include "../include/spt.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
  fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define CHECK_SPT(x) do { spt_status s_ = (x); if (s_ != SPT_OK) { \
  fprintf(stderr, "spt error %d: %s (line %d)\n", (int)s_, spt_last_error(), __LINE__); return 3; } } while (0)

static void* to_device(const void* host, size_t bytes) {
  void* d = NULL;
  if (hipMalloc(&d, bytes ? bytes : 4) != hipSuccess) return NULL;
  if (host && bytes && hipMemcpy(d, host, bytes, hipMemcpyHostToDevice) != hipSuccess) return NULL;
  return d;
}

int main(void) {
  const int32_t pos[5] = {0, 2, 4, 4, 7}, crd[7] = {0, 1, 0, 1, 0, 3, 4};
  const double vals[7] = {5, 1, 7, 3, 8, 4, 9}, x[6] = {1, 2, 3, 4, 5, 6};
  spt_tensor A = {0};
  A.order = 2;
  A.nlevels = 2;
  A.dtype = SPT_F64;
  A.level[0].kind = SPT_DENSE;
  A.level[0].mode = 0;
  A.level[0].N = 4;
  A.level[1].kind = SPT_COMPRESSED;
  A.level[1].mode = 1;
  A.level[1].flags = SPT_ORDERED | SPT_UNIQUE;
  A.level[1].N = 6;
  A.level[1].M = 4;
  A.level[1].pos = (const int32_t*)to_device(pos, sizeof pos);
  A.level[1].crd = (const int32_t*)to_device(crd, sizeof crd);
  A.vals = to_device(vals, sizeof vals);
  A.nvals = 7;
  double* dx = (double*)to_device(x, sizeof x);
  double* dy = (double*)to_device(NULL, 4 * sizeof(double));
  if (!A.level[1].pos || !A.level[1].crd || !A.vals || !dx || !dy) {
    fprintf(stderr, "device allocation failed\n");
    return 2;
  }

  size_t ws_bytes = spt_workspace_bytes(SPT_OP_SPMV, &A, 0);
  void* ws = to_device(NULL, ws_bytes);
  CHECK_SPT(spt_spmv(&A, dx, dy, ws, ws_bytes, NULL));
  double y[4];
  CHECK_HIP(hipMemcpy(y, dy, sizeof y, hipMemcpyDeviceToHost));
  printf("%s: y = %g %g %g %g\n", spt_version(), y[0], y[1], y[2], y[3]);
  const double want[4] = {7, 13, 0, 69};
  for (int i = 0; i < 4; ++i)
    if (y[i] != want[i]) { fprintf(stderr, "wrong y[%d]\n", i); return 1; }

  /* A + A with a CSR result: same structure, doubled values */
  size_t add_bytes = spt_add_workspace_bytes(&A, &A);
  void* add_ws = to_device(NULL, add_bytes);
  int32_t* opos = (int32_t*)to_device(NULL, 5 * 4);
  int32_t* ocrd = (int32_t*)to_device(NULL, 14 * 4);
  double* oval = (double*)to_device(NULL, 14 * 8);
  int64_t* onnz = (int64_t*)to_device(NULL, 8);
  CHECK_SPT(spt_add(&A, &A, opos, NULL, ocrd, NULL, oval, onnz, add_ws, add_bytes, NULL));
  int64_t n = 0;
  int32_t hp[5];
  double hv[14];
  CHECK_HIP(hipMemcpy(&n, onnz, 8, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(hp, opos, sizeof hp, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(hv, oval, 7 * 8, hipMemcpyDeviceToHost));
  printf("A + A: %lld entries, pos = %d %d %d %d %d, last value %g\n", (long long)n, hp[0], hp[1],
         hp[2], hp[3], hp[4], hv[6]);
  if (n != 7 || hp[4] != 7 || hp[2] != 4 || hv[6] != 18) { fprintf(stderr, "wrong sum\n"); return 1; }
  printf("ok\n");
  return 0;
}
