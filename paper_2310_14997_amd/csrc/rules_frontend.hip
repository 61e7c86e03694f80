// Rule-probability front-end and its backward: the four softmaxes that end the neural parameterisation
// (App. A) - root over the nonterminals, left and right productions over N u P children per parent,
// emissions over the vocabulary per preterminal - and the per-token gather of the emission table that the
// inside pass consumes.  All kernels are memory-bound row reductions or elementwise passes; results are
// deterministic (the token scatter of the emission gradient walks the tokens in a fixed order inside the
// one wavefront that owns a block of the table).
#include <cmath>

#include "spcfg_internal.h"

namespace spcfg {

namespace {

__device__ __forceinline__ float wmax(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wsum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float bmax(float v, float* red) {
  v = wmax(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = red[0];
  for (int i = 1; i < (int)(blockDim.x >> 6); ++i) r = fmaxf(r, red[i]);
  return r;
}
__device__ __forceinline__ float bsum(float v, float* red) {
  v = wsum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = 0.0f;
  for (int i = 0; i < (int)(blockDim.x >> 6); ++i) r += red[i];  // fixed order
  return r;
}

// mode 0: out = softmax(row); mode 1: out = log_softmax(row); mode 2: out[row] = logsumexp(row) only
__global__ void __launch_bounds__(256) k_row_softmax(const float* __restrict__ z, int64_t cols, float* __restrict__ out,
                                                     int mode) {
  __shared__ float red[4];
  const float* row = z + (int64_t)blockIdx.x * cols;
  float m = -INFINITY;
  for (int64_t c = threadIdx.x; c < cols; c += 256) m = fmaxf(m, row[c]);
  m = bmax(m, red);
  float s = 0.0f;
  for (int64_t c = threadIdx.x; c < cols; c += 256) s += expf(row[c] - m);
  s = bsum(s, red);
  if (mode == 2) {
    if (threadIdx.x == 0) out[blockIdx.x] = m + logf(s);
    return;
  }
  float* o = out + (int64_t)blockIdx.x * cols;
  const float inv = 1.0f / s, ls = logf(s);
  for (int64_t c = threadIdx.x; c < cols; c += 256) o[c] = mode == 0 ? expf(row[c] - m) * inv : (row[c] - m) - ls;
}

// log_emit[b, i, T] = emis_logits[T, tok] - lse[T] for i < n_b, 0 on padding; an out-of-range token id gives NaN.
__global__ void __launch_bounds__(256) k_gather_emit(LenArg la, int n_max, int P, int V,
                                                     const float* __restrict__ emis, const float* __restrict__ lse,
                                                     const int32_t* __restrict__ tokens, float* __restrict__ out) {
  const int b = blockIdx.x / n_max, i = blockIdx.x % n_max;
  float* o = out + (int64_t)blockIdx.x * P;
  if (i >= la.v[b]) {
    for (int t = threadIdx.x; t < P; t += 256) o[t] = 0.0f;
    return;
  }
  const int tok = tokens[blockIdx.x];
  const bool ok = (unsigned)tok < (unsigned)V;
  for (int t = threadIdx.x; t < P; t += 256) o[t] = ok ? emis[(int64_t)t * V + tok] - lse[t] : NAN;
}

// softmax backward per row: dz = p * (g - sum_j p_j g_j)
__global__ void __launch_bounds__(256) k_softmax_bwd(const float* __restrict__ p, const float* __restrict__ g,
                                                     int64_t cols, float* __restrict__ dz) {
  __shared__ float red[4];
  const int64_t base = (int64_t)blockIdx.x * cols;
  float d = 0.0f;
  for (int64_t c = threadIdx.x; c < cols; c += 256) d = fmaf(p[base + c], g[base + c], d);
  d = bsum(d, red);
  for (int64_t c = threadIdx.x; c < cols; c += 256) dz[base + c] = p[base + c] * (g[base + c] - d);
}

// log-softmax backward for the root: dz = g - exp(log_root) * sum_j g_j
__global__ void __launch_bounds__(256) k_logsoftmax_bwd(const float* __restrict__ logp, const float* __restrict__ g, int n,
                                                        float* __restrict__ dz) {
  __shared__ float red[4];
  float s = 0.0f;
  for (int c = threadIdx.x; c < n; c += 256) s += g[c];
  s = bsum(s, red);
  for (int c = threadIdx.x; c < n; c += 256) dz[c] = g[c] - expf(logp[c]) * s;
}

// part[c][T] = sum of grad_log_emit[b, i, T] over the real token positions p = b * n_max + i with p % kColChunks == c
// (position order inside a chunk); tot[T] = sum_c part[c][T] in chunk order.  Deterministic two-level sum.
constexpr int kColChunks = 32;
__global__ void __launch_bounds__(64) k_emit_colsum_part(LenArg la, int B, int n_max, int P, const float* __restrict__ ge,
                                                         float* __restrict__ part) {
  const int t = blockIdx.x * 64 + threadIdx.x;
  const int c = blockIdx.y;
  if (t >= P) return;
  float s = 0.0f;
  for (int p = c; p < B * n_max; p += kColChunks) {
    const int b = p / n_max, i = p - b * n_max;
    if (i < la.v[b]) s += ge[(int64_t)p * P + t];
  }
  part[(int64_t)c * P + t] = s;
}
__global__ void __launch_bounds__(256) k_emit_colsum_final(int P, float* __restrict__ part) {  // tot -> part[0]
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= P) return;
  float s = 0.0f;
  for (int c = 0; c < kColChunks; ++c) s += part[(int64_t)c * P + t];
  part[t] = s;
}

// d emis[T, v] = sum_{(b,i): tok = v} grad_log_emit[b, i, T]  -  softmax(emis[T, :])[v] * tot[T].
// One wavefront owns a block of 64 preterminals x kVChunk vocabulary entries: it accumulates the token
// contributions of its block in LDS (lane = preterminal, so every LDS word has one owner; tokens are walked in
// order, which fixes the summation order of repeated tokens), then writes the block once, coalesced along v.
constexpr int kVChunk = 128;
__global__ void __launch_bounds__(64) k_emis_grad(LenArg la, int B, int n_max, int P, int V,
                                                  const int32_t* __restrict__ tokens, const float* __restrict__ ge,
                                                  const float* __restrict__ emis, const float* __restrict__ lse,
                                                  const float* __restrict__ tot, float* __restrict__ d) {
  __shared__ float tile[kVChunk][65];
  const int lane = threadIdx.x;
  const int t0 = blockIdx.x * 64, v0 = blockIdx.y * kVChunk;
  const int v1 = min(v0 + kVChunk, V);
  for (int v = 0; v < kVChunk; ++v) tile[v][lane] = 0.0f;
  const int t = t0 + lane;
  for (int b = 0; b < B; ++b) {
    const int n = la.v[b];
    for (int i0 = 0; i0 < n; i0 += 64) {
      // one coalesced load of up to 64 token ids, then a ballot of those that fall into this block
      const int i = i0 + lane;
      const int mytok = i < n ? tokens[b * n_max + i] : -1;
      unsigned long long hit = __ballot(mytok >= v0 && mytok < v1);
      while (hit) {  // ascending position order
        const int j = __ffsll((long long)hit) - 1;
        hit &= hit - 1;
        const int tok = __shfl(mytok, j, 64);
        if (t < P) tile[tok - v0][lane] += ge[((int64_t)b * n_max + i0 + j) * P + t];
      }
    }
  }
  __syncthreads();
  // write-out: lanes along v (two columns per lane), eight preterminal rows in flight
  const int va = v0 + lane, vb = v0 + 64 + lane;
  const bool oka = va < v1, okb = vb < v1;
  const int rows = min(64, P - t0);
  for (int r0 = 0; r0 < rows; r0 += 8) {
    float ea[8], eb[8], ls[8], ts[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int tr = t0 + min(r0 + u, rows - 1);
      const int64_t base = (int64_t)tr * V;
      ea[u] = oka ? emis[base + va] : 0.0f;
      eb[u] = okb ? emis[base + vb] : 0.0f;
      ls[u] = lse[tr];
      ts[u] = tot[tr];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (r0 + u >= rows) break;
      const int64_t base = (int64_t)(t0 + r0 + u) * V;
      if (oka) d[base + va] = tile[va - v0][r0 + u] - expf(ea[u] - ls[u]) * ts[u];
      if (okb) d[base + vb] = tile[vb - v0][r0 + u] - expf(eb[u] - ls[u]) * ts[u];
    }
  }
}

int check(int N, int P, int V, int B, int n_max, const int32_t* lengths, LenArg* la) {
  if (N < 1 || P < 1 || V < 1 || N > (1 << 16) || P > (1 << 16) || V > (1 << 24)) return SPCFG_ERR_SHAPE;
  if (B < 1 || B > kMaxB || n_max < 1 || n_max > kMaxLen) return SPCFG_ERR_SHAPE;
  if (!lengths) return SPCFG_ERR_ARG;
  for (int b = 0; b < B; ++b) {
    if (lengths[b] < 0 || lengths[b] > n_max) return SPCFG_ERR_LENGTH;
    la->v[b] = lengths[b];
  }
  return SPCFG_OK;
}

int status() { return hipGetLastError() == hipSuccess ? SPCFG_OK : SPCFG_ERR_HIP; }

}  // namespace
}  // namespace spcfg

using namespace spcfg;

extern "C" {

int spcfg_rules_forward(int32_t N, int32_t P, int32_t V, const float* root_logits, const float* L_logits,
                        const float* R_logits, const float* emis_logits, const int32_t* tokens, const int32_t* lengths,
                        int32_t B, int32_t n_max, float* log_root, float* L, float* R, float* log_emit, float* emis_lse,
                        void* hip_stream) {
  LenArg la;
  int rc = check(N, P, V, B, n_max, lengths, &la);
  if (rc) return rc;
  if (!root_logits || !L_logits || !R_logits || !emis_logits || !tokens || !log_root || !L || !R || !log_emit ||
      !emis_lse)
    return SPCFG_ERR_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  const int64_t M = (int64_t)N + P;
  hipLaunchKernelGGL(k_row_softmax, dim3(1), dim3(256), 0, st, root_logits, (int64_t)N, log_root, 1);
  hipLaunchKernelGGL(k_row_softmax, dim3(N), dim3(256), 0, st, L_logits, M, L, 0);
  hipLaunchKernelGGL(k_row_softmax, dim3(N), dim3(256), 0, st, R_logits, M, R, 0);
  hipLaunchKernelGGL(k_row_softmax, dim3(P), dim3(256), 0, st, emis_logits, (int64_t)V, emis_lse, 2);
  hipLaunchKernelGGL(k_gather_emit, dim3(B * n_max), dim3(256), 0, st, la, n_max, P, V, emis_logits, emis_lse, tokens,
                     log_emit);
  return status();
}

int spcfg_rules_backward(int32_t N, int32_t P, int32_t V, const float* log_root, const float* L, const float* R,
                         const float* emis_logits, const float* emis_lse, const int32_t* tokens,
                         const int32_t* lengths, int32_t B, int32_t n_max, const float* grad_log_root,
                         const float* grad_L, const float* grad_R, const float* grad_log_emit, float* grad_root_logits,
                         float* grad_L_logits, float* grad_R_logits, float* grad_emis_logits, float* scratch,
                         void* hip_stream) {
  LenArg la;
  int rc = check(N, P, V, B, n_max, lengths, &la);
  if (rc) return rc;
  if (!log_root || !L || !R || !emis_logits || !emis_lse || !tokens || !grad_log_root || !grad_L || !grad_R ||
      !grad_log_emit || !grad_root_logits || !grad_L_logits || !grad_R_logits || !grad_emis_logits || !scratch)
    return SPCFG_ERR_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  const int64_t M = (int64_t)N + P;
  hipLaunchKernelGGL(k_logsoftmax_bwd, dim3(1), dim3(256), 0, st, log_root, grad_log_root, N, grad_root_logits);
  hipLaunchKernelGGL(k_softmax_bwd, dim3(N), dim3(256), 0, st, L, grad_L, M, grad_L_logits);
  hipLaunchKernelGGL(k_softmax_bwd, dim3(N), dim3(256), 0, st, R, grad_R, M, grad_R_logits);
  hipLaunchKernelGGL(k_emit_colsum_part, dim3((P + 63) / 64, kColChunks), dim3(64), 0, st, la, B, n_max, P,
                     grad_log_emit, scratch);
  hipLaunchKernelGGL(k_emit_colsum_final, dim3((P + 255) / 256), dim3(256), 0, st, P, scratch);
  hipLaunchKernelGGL(k_emis_grad, dim3((P + 63) / 64, (V + kVChunk - 1) / kVChunk), dim3(64), 0, st, la, B, n_max, P, V,
                     tokens, grad_log_emit, emis_logits, emis_lse, scratch, grad_emis_logits);
  return status();
}

}  // extern "C"
