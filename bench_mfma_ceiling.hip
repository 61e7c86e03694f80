// What the matrix pipes of this chip sustain, for bench.py's roofline figures: a register-only loop of
// v_mfma_f32_32x32x16_bf16 (the instruction of the projection and rule-gradient products) on every SIMD, timed with HIP
// events, with the shader clock read from inside the kernel (shader-cycle counter against the fixed 100 MHz counter).
// Three operand patterns: constant values; random values that stay the same from instruction to instruction; random
// values that change with every instruction (four operand pairs in rotation), which is what a product sees.
// Prints one JSON object.  Measurement aid only: nothing in the library depends on it.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)

// PATTERN 0: all operands 1.0; 1: one random operand pair per lane; 2: four random pairs per lane, one per instruction
template <int PATTERN>
__global__ void __launch_bounds__(256) k_mfma_loop(long long* clocks, float* sink, int iters) {
  floatx16 acc[4];
  for (int i = 0; i < 4; ++i)
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  bf16x8 a[4], b[4];
  unsigned seed = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
  for (int q = 0; q < 4; ++q)
    for (int i = 0; i < 8; ++i) {
      seed = seed * 1664525u + 1013904223u;
      const float x = ((int)(seed >> 8) % 2001 - 1000) * 0.001f;
      seed = seed * 1664525u + 1013904223u;
      const float y = ((int)(seed >> 8) % 2001 - 1000) * 0.001f;
      a[q][i] = (__bf16)(PATTERN == 0 ? 1.0f : x);
      b[q][i] = (__bf16)(PATTERN == 0 ? 1.0f : y);
    }
  const long long c0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int p = PATTERN == 2 ? q : 0;
        acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[p], b[p], acc[q], 0, 0, 0);
      }
    }
  }
  const long long c1 = clock64(), w1 = wall_clock64();
  float s = 0;
  for (int i = 0; i < 4; ++i)
    for (int v = 0; v < 16; ++v) s += acc[i][v];
  sink[blockIdx.x * 256 + threadIdx.x] = s;
  if (threadIdx.x == 0) { clocks[blockIdx.x * 2] = c1 - c0; clocks[blockIdx.x * 2 + 1] = w1 - w0; }
}

int main() {
  const int wgs = 256, iters = 20000;  // one workgroup of four wavefronts per CU, 640 000 instructions per wavefront
  long long* clocks; float* sink;
  CK(hipMalloc(&clocks, wgs * 16)); CK(hipMalloc(&sink, (size_t)wgs * 256 * 4));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  const char* names[3] = {"constant_operands", "random_operands_fixed", "random_operands_changing"};
  printf("{\"instruction\": \"v_mfma_f32_32x32x16_bf16\", \"published_peak_tflops\": 2500.0");
  for (int pattern = 0; pattern < 3; ++pattern) {
    float best = 1e30f; long long h[2] = {0, 1};
    for (int rep = 0; rep < 3; ++rep) {
      CK(hipEventRecord(e0, 0));
      if (pattern == 0) hipLaunchKernelGGL((k_mfma_loop<0>), dim3(wgs), dim3(256), 0, 0, clocks, sink, iters);
      else if (pattern == 1) hipLaunchKernelGGL((k_mfma_loop<1>), dim3(wgs), dim3(256), 0, 0, clocks, sink, iters);
      else hipLaunchKernelGGL((k_mfma_loop<2>), dim3(wgs), dim3(256), 0, 0, clocks, sink, iters);
      CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1)); CK(hipGetLastError());
      float ms; CK(hipEventElapsedTime(&ms, e0, e1));
      if (ms < best) { best = ms; CK(hipMemcpy(h, clocks, 16, hipMemcpyDeviceToHost)); }
    }
    const double n_mfma = (double)iters * 32;  // per wavefront
    const double tflops = (double)wgs * 4 * n_mfma * 32768.0 / (best * 1e-3) / 1e12;
    printf(", \"%s\": {\"ms\": %.3f, \"shader_MHz\": %.0f, \"cycles_per_instruction\": %.2f, \"tflops\": %.0f, \"frac_of_published\": %.3f}",
           names[pattern], best, 100.0 * h[0] / h[1], (double)h[0] / n_mfma, tflops, tflops / 2500.0);
  }
  printf("}\n");
  return 0;
}
