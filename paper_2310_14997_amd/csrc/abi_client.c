/*
 * Plain C client of libspcfg: no Python, no PyTorch.  Reads one batch from a binary file, runs
 * spcfg_inside_forward_backward through the C ABI and writes the results to another file.  Used by the tests to
 * show that the boundary stands on its own; it is also the shortest complete usage example of the library.
 *
 * Input file (little endian): int32 N, P, B, n_max; int32 lengths[B]; float log_root[N], L[N*M], R[N*M],
 * log_emit[B*n_max*P]  (M = N + P).  Output file: float logZ[B], grad_L[N*M], grad_R[N*M], grad_log_root[N],
 * grad_log_emit[B*n_max*P].
 */
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/spcfg.h"

#define CHECK_HIP(x)                                                              \
  do {                                                                            \
    hipError_t e_ = (x);                                                          \
    if (e_ != hipSuccess) {                                                       \
      fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
      return 2;                                                                   \
    }                                                                             \
  } while (0)

static float* upload(const float* h, size_t n) {
  float* d = NULL;
  if (hipMalloc((void**)&d, n * sizeof(float)) != hipSuccess) return NULL;
  if (hipMemcpy(d, h, n * sizeof(float), hipMemcpyHostToDevice) != hipSuccess) return NULL;
  return d;
}

int main(int argc, char** argv) {
  if (argc != 3) {
    fprintf(stderr, "usage: %s <input file> <output file>\n", argv[0]);
    return 1;
  }
  FILE* f = fopen(argv[1], "rb");
  if (!f) { perror("input"); return 1; }
  int32_t hdr[4];
  if (fread(hdr, sizeof(int32_t), 4, f) != 4) return 1;
  const int32_t N = hdr[0], P = hdr[1], B = hdr[2], n_max = hdr[3];
  const size_t M = (size_t)N + P, nW = (size_t)N * M, nE = (size_t)B * n_max * P;
  int32_t* lengths = (int32_t*)malloc(sizeof(int32_t) * B);
  float* host = (float*)malloc(sizeof(float) * (N + 2 * nW + nE));
  if (!lengths || !host) return 1;
  if (fread(lengths, sizeof(int32_t), B, f) != (size_t)B) return 1;
  if (fread(host, sizeof(float), N + 2 * nW + nE, f) != N + 2 * nW + nE) return 1;
  fclose(f);

  spcfg_config cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.struct_size = sizeof cfg;
  cfg.N = N; cfg.P = P; cfg.max_B = B; cfg.max_n = n_max; cfg.precision = SPCFG_PRECISION_FP32;
  size_t ws_bytes = 0;
  int rc = spcfg_workspace_bytes_for(&cfg, lengths, B, n_max, &ws_bytes);
  if (rc != SPCFG_OK) { fprintf(stderr, "workspace query: %s\n", spcfg_strerror(rc)); return 3; }

  float* d_root = upload(host, N);
  float* d_L = upload(host + N, nW);
  float* d_R = upload(host + N + nW, nW);
  float* d_emit = upload(host + N + 2 * nW, nE);
  if (!d_root || !d_L || !d_R || !d_emit) { fprintf(stderr, "upload failed\n"); return 2; }
  void* ws = NULL;
  float *d_logZ, *d_gL, *d_gR, *d_groot, *d_gemit;
  CHECK_HIP(hipMalloc(&ws, ws_bytes));
  CHECK_HIP(hipMalloc((void**)&d_logZ, sizeof(float) * B));
  CHECK_HIP(hipMalloc((void**)&d_gL, sizeof(float) * nW));
  CHECK_HIP(hipMalloc((void**)&d_gR, sizeof(float) * nW));
  CHECK_HIP(hipMalloc((void**)&d_groot, sizeof(float) * N));
  CHECK_HIP(hipMalloc((void**)&d_gemit, sizeof(float) * nE));

  rc = spcfg_inside_forward_backward(&cfg, d_root, d_L, d_R, d_emit, lengths, B, n_max, NULL, d_logZ, d_gL, d_gR,
                                     d_groot, d_gemit, ws, ws_bytes, NULL);
  if (rc != SPCFG_OK) {
    fprintf(stderr, "spcfg_inside_forward_backward: %s %s\n", spcfg_strerror(rc), spcfg_last_hip_error());
    return 3;
  }
  CHECK_HIP(hipDeviceSynchronize());

  float* out = (float*)malloc(sizeof(float) * (B + 2 * nW + N + nE));
  if (!out) return 1;
  CHECK_HIP(hipMemcpy(out, d_logZ, sizeof(float) * B, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(out + B, d_gL, sizeof(float) * nW, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(out + B + nW, d_gR, sizeof(float) * nW, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(out + B + 2 * nW, d_groot, sizeof(float) * N, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(out + B + 2 * nW + N, d_gemit, sizeof(float) * nE, hipMemcpyDeviceToHost));
  f = fopen(argv[2], "wb");
  if (!f) { perror("output"); return 1; }
  fwrite(out, sizeof(float), B + 2 * nW + N + nE, f);
  fclose(f);
  printf("ok: %d sentences, log Z[0] = %f\n", (int)B, out[0]);
  return 0;
}
