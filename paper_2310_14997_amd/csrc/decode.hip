// Minimum-Bayes-risk tree decoding from span posteriors: the binary bracketing that maximises the sum of
// mu(i,j) over its spans of width >= 2, by CKY over split points,
//   best(i,j) = mu(i,j) + max_{i<k<j} best(i,k) + best(k,j),   best(i,i+1) = 0,
// smallest k on ties.  This is the tree used to score a grammar as a parser (Sec. 4, "Evaluation").
// One workgroup per sentence; widths are taken in order with a barrier between them, one wavefront per
// span with its lanes over the split points.  The chart is kept twice, by start and by end position, so
// that both children are read along contiguous runs; it lives in LDS when it fits and in caller-provided
// scratch otherwise.  Integer split table and the read-out stack live in the scratch.
#include "spcfg_internal.h"

namespace spcfg {
namespace {

constexpr int kDecodeThreads = 1024;
constexpr size_t kDecodeLdsMax = 64 * 1024;

__global__ void __launch_bounds__(kDecodeThreads)
k_mbr_decode(LenArg la, int n_max, int use_lds, const float* __restrict__ mu, float* __restrict__ gchart,
             int32_t* __restrict__ gsplit, int32_t* __restrict__ tree_spans, float* __restrict__ tree_score) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int b = blockIdx.x;
  const int n = la.v[b];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
  const int64_t nn = (int64_t)n_max * n_max;
  // byS[i * n_max + (k-1)] = best(i,k); byE[(j-1) * n_max + k] = best(k,j)
  float* byS = use_lds ? reinterpret_cast<float*>(smem) : gchart + (int64_t)b * 2 * nn;
  float* byE = byS + nn;
  int32_t* split = gsplit + (int64_t)b * nn;
  const float* m = mu + (int64_t)b * nn;

  for (int i = tid; i < n; i += blockDim.x) {  // width 1
    byS[i * n_max + i] = 0.0f;
    byE[i * n_max + i] = 0.0f;
  }
  __syncthreads();
  for (int w = 2; w <= n; ++w) {
    for (int i = wave; i + w <= n; i += nwaves) {
      const int j = i + w;
      const float* left = byS + (int64_t)i * n_max;         // left[k-1]  = best(i,k)
      const float* right = byE + (int64_t)(j - 1) * n_max;  // right[k]   = best(k,j)
      float bv = -INFINITY;
      int bk = 0x7fffffff;
      for (int k = i + 1 + lane; k < j; k += 64) {
        const float v = left[k - 1] + right[k];
        if (v > bv) { bv = v; bk = k; }  // k increases within a lane: the first maximum is kept
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int ok = __shfl_xor(bk, o, 64);
        if (ov > bv || (ov == bv && ok < bk)) { bv = ov; bk = ok; }
      }
      // No candidate compares greater than -inf when every sum is -inf or NaN (scores are the caller's data): the
      // split then defaults to the smallest one, so the table only ever holds split points inside the span.
      if (bk <= i || bk >= j) bk = i + 1;
      if (lane == 0) {
        const float v = m[(int64_t)i * n_max + (j - 1)] + bv;
        byS[(int64_t)i * n_max + (j - 1)] = v;
        byE[(int64_t)(j - 1) * n_max + i] = v;
        split[(int64_t)i * n_max + (j - 1)] = bk;
      }
    }
    __syncthreads();
  }
  // read-out in pre-order with an explicit stack (at most n-1 pending spans of width >= 2)
  if (tid == 0) {
    int32_t* out = tree_spans + (int64_t)b * (n_max - 1) * 2;
    // the by-end chart in the scratch is unused (LDS chart) or dead (best(0,n) is known): reuse it as the stack
    int32_t* stack = reinterpret_cast<int32_t*>(gchart + (int64_t)b * 2 * nn + nn);
    tree_score[b] = byS[n - 1];
    int sp = 0, cnt = 0;
    stack[0] = 0; stack[1] = n; sp = 1;
    while (sp > 0 && cnt < n - 1) {  // a binary tree over n words has n - 1 spans of width >= 2
      --sp;
      const int i = stack[2 * sp], j = stack[2 * sp + 1];
      out[2 * cnt] = i; out[2 * cnt + 1] = j; ++cnt;
      const int k = split[(int64_t)i * n_max + (j - 1)];
      if (j - k >= 2) { stack[2 * sp] = k; stack[2 * sp + 1] = j; ++sp; }
      if (k - i >= 2) { stack[2 * sp] = i; stack[2 * sp + 1] = k; ++sp; }
    }
    for (; cnt < n_max - 1; ++cnt) { out[2 * cnt] = -1; out[2 * cnt + 1] = -1; }
  }
}

}  // namespace
}  // namespace spcfg

using namespace spcfg;

extern "C" {

int spcfg_mbr_decode_scratch_bytes(int32_t B, int32_t n_max, size_t* out_bytes) {
  if (!out_bytes) return SPCFG_ERR_ARG;
  if (B < 1 || B > kMaxB || n_max < 2 || n_max > kMaxLen) return SPCFG_ERR_SHAPE;
  *out_bytes = (size_t)B * n_max * n_max * 12;  // chart by start, chart by end, split points
  return SPCFG_OK;
}

int spcfg_mbr_decode(const float* span_post, const int32_t* lengths, int32_t B, int32_t n_max, int32_t* tree_spans,
                     float* tree_score, void* scratch, size_t scratch_bytes, void* hip_stream) {
  if (!span_post || !lengths || !tree_spans || !tree_score || !scratch) return SPCFG_ERR_ARG;
  size_t need = 0;
  int rc = spcfg_mbr_decode_scratch_bytes(B, n_max, &need);
  if (rc) return rc;
  if (((uintptr_t)scratch & 15) != 0 || scratch_bytes < need) return SPCFG_ERR_WORKSPACE;
  LenArg la;
  for (int b = 0; b < B; ++b) {
    if (lengths[b] < 2 || lengths[b] > n_max) return SPCFG_ERR_LENGTH;
    la.v[b] = lengths[b];
  }
  const size_t nn = (size_t)n_max * n_max;
  const size_t lds = 2 * nn * sizeof(float);
  const int use_lds = lds <= kDecodeLdsMax;
  float* gchart = static_cast<float*>(scratch);
  int32_t* gsplit = reinterpret_cast<int32_t*>(gchart + 2 * nn * B);
  hipLaunchKernelGGL(k_mbr_decode, dim3(B), dim3(kDecodeThreads), use_lds ? lds : 0, (hipStream_t)hip_stream, la, n_max,
                     use_lds, span_post, gchart, gsplit, tree_spans, tree_score);
  return hipGetLastError() == hipSuccess ? SPCFG_OK : SPCFG_ERR_HIP;
}

}  // extern "C"
