/* The C ABI used from plain C, with no Python and no torch: device buffers from the HIP runtime, one codec,
 * compress -> decompress -> norm, and a check of the round trip against the binning bound of Sec. IV-D
 * (every coefficient moves by at most N_k / (2 r), so a block's L2 error is at most sqrt(prod(i)) N_k / (2 r)).
 * Built by paper_2406_11209_amd/build.py next to libpbz.so; prints "ok" and returns 0 on success. */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include "pbz.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP: %s (line %d)\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define CHECK_PBZ(x) do { int s_ = (x); if (s_ != PBZ_OK) { fprintf(stderr, "pbz: %s (line %d)\n", pbz_status_string(s_), __LINE__); return 3; } } while (0)

int main(void) {
  const int64_t shape[3] = {20, 36, 40};          /* not multiples of the block in the first dimension */
  const int64_t block[3] = {4, 4, 4};
  const size_t n = (size_t)(shape[0] * shape[1] * shape[2]);
  double* host = (double*)malloc(n * sizeof(double));
  double* back = (double*)malloc(n * sizeof(double));
  if (!host || !back) return 1;
  for (size_t i = 0; i < n; ++i) {
    const double z = (double)(i / (size_t)(shape[1] * shape[2])), y = (double)((i / (size_t)shape[2]) % (size_t)shape[1]), x = (double)(i % (size_t)shape[2]);
    host[i] = sin(0.3 * z) * cos(0.2 * y) + 0.05 * x;
  }

  pbz_codec* codec = NULL;
  CHECK_PBZ(pbz_codec_create(&codec, 3, block, PBZ_F64, PBZ_I16, NULL));
  int64_t n_blocks = 0, kept = 0;
  size_t n_bytes = 0, f_bytes = 0, ws_bytes = 0;
  CHECK_PBZ(pbz_layout(codec, shape, &n_blocks, &kept, &n_bytes, &f_bytes, &ws_bytes));

  void *d_x = NULL, *d_y = NULL, *d_N = NULL, *d_F = NULL, *d_ws = NULL;
  double* d_out = NULL;
  CHECK_HIP(hipMalloc(&d_x, n * sizeof(double)));
  CHECK_HIP(hipMalloc(&d_y, n * sizeof(double)));
  CHECK_HIP(hipMalloc(&d_N, n_bytes));
  CHECK_HIP(hipMalloc(&d_F, f_bytes));
  CHECK_HIP(hipMalloc(&d_ws, ws_bytes));
  CHECK_HIP(hipMalloc((void**)&d_out, sizeof(double)));
  CHECK_HIP(hipMemcpy(d_x, host, n * sizeof(double), hipMemcpyHostToDevice));

  CHECK_PBZ(pbz_compress(codec, d_x, PBZ_F64, shape, d_N, d_F, NULL));
  CHECK_PBZ(pbz_decompress(codec, d_N, d_F, shape, d_y, PBZ_F64, NULL));
  CHECK_PBZ(pbz_norm2(codec, n_blocks, d_N, d_F, d_out, d_ws, ws_bytes, NULL));
  CHECK_HIP(hipDeviceSynchronize());

  double norm = 0.0;
  double* N_host = (double*)malloc(n_bytes);
  if (!N_host) return 1;
  CHECK_HIP(hipMemcpy(back, d_y, n * sizeof(double), hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(N_host, d_N, n_bytes, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(&norm, d_out, sizeof(double), hipMemcpyDeviceToHost));

  double err2 = 0.0, bound2 = 0.0, ref2 = 0.0;
  for (size_t i = 0; i < n; ++i) {
    err2 += (back[i] - host[i]) * (back[i] - host[i]);
    ref2 += host[i] * host[i];
  }
  for (int64_t k = 0; k < n_blocks; ++k) bound2 += 64.0 * (N_host[k] / (2.0 * 32767.0)) * (N_host[k] / (2.0 * 32767.0));
  printf("blocks %lld  kept %lld  kernel %s\n", (long long)n_blocks, (long long)kept, pbz_kernel_name(codec, "compress", shape, PBZ_F64));
  printf("round-trip L2 error %.3e (bound %.3e)  ||x|| %.6f  compressed-space norm %.6f\n", sqrt(err2), sqrt(bound2), sqrt(ref2), norm);
  int ok = sqrt(err2) <= sqrt(bound2) * (1.0 + 1e-9) && fabs(norm - sqrt(ref2)) <= sqrt(bound2) + 1e-9;
  /* the padded part of the last block row along z carries coefficients too, but its samples are zero: the norm of
   * the uncropped decompressed array differs from ||x|| by at most the same bound */

  pbz_codec_destroy(codec);
  hipFree(d_x); hipFree(d_y); hipFree(d_N); hipFree(d_F); hipFree(d_ws); hipFree(d_out);
  free(host); free(back); free(N_host);
  printf(ok ? "ok\n" : "FAILED\n");
  return ok ? 0 : 4;
}
