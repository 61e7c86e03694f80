// Span plan, weight packing, leaf preparation, split-point reductions (forward and reverse) and root
// reductions for the simple-PCFG inside pass on gfx950.  All kernels are deterministic (no atomics).
#include <type_traits>

#include "gemm_nt_common.h"

namespace spcfg {

namespace {


__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ int wave_max_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Block-wide reductions through LDS; `red` needs one slot per wave (<= 16). All threads get the result.
__device__ __forceinline__ float block_max(float v, float* red) {
  v = wave_max(v);
  const int wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  float r = red[0];
  for (int i = 1; i < nw; ++i) r = fmaxf(r, red[i]);
  return r;
}
__device__ __forceinline__ int block_max_i(int v, int* red) {
  v = wave_max_i(v);
  const int wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  int r = red[0];
  for (int i = 1; i < nw; ++i) r = max(r, red[i]);
  return r;
}
__device__ __forceinline__ double block_sum_d(double v, double* red) {
  v = wave_sum_d(v);
  const int wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  double r = 0.0;
  for (int i = 0; i < nw; ++i) r += red[i];
  return r;
}

typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
// bf16 copy of four consecutive values (round to nearest even): the operand the bf16 projection products read
__device__ __forceinline__ void store_bf16x4(void* base, int64_t idx, float4 v) {
  bf16x4_t r;
  r[0] = (__bf16)v.x; r[1] = (__bf16)v.y; r[2] = (__bf16)v.z; r[3] = (__bf16)v.w;
  *reinterpret_cast<bf16x4_t*>(static_cast<__bf16*>(base) + idx) = r;
}

// Operand planes of four consecutive values for the projection products: with three planes the exact cut
// x = hi + mid + lo into bf16 pieces (nt::Split3), with two planes hi = bf16(x) and lo = bf16(x - hi) (the first two
// pieces of the same cut), with one plane the bf16 rounding.  Plane p starts at base + p * plane_stride elements.
__device__ __forceinline__ void store_planes4(void* base, int planes, int64_t plane_stride, int64_t idx, float4 v) {
  if (planes >= 2) {
    unsigned h0, m0, l0, h1, m1, l1;
    nt::Split3::cut2(v.x, v.y, h0, m0, l0);
    nt::Split3::cut2(v.z, v.w, h1, m1, l1);
    uint16_t* b = static_cast<uint16_t*>(base) + idx;
    *reinterpret_cast<uint2*>(b) = uint2{h0, h1};
    *reinterpret_cast<uint2*>(b + plane_stride) = uint2{m0, m1};
    if (planes == 3) *reinterpret_cast<uint2*>(b + 2 * plane_stride) = uint2{l0, l1};
  } else {
    store_bf16x4(base, idx, v);
  }
}

// 2^d as a float for an integer d (0 below the fp32 range); exact.
__device__ __forceinline__ float pow2i(int d) { return d < -160 ? 0.0f : ldexpf(1.0f, min(d, 127)); }

__device__ __forceinline__ int add_exp(int a, int b) { return (a == kExpZero || b == kExpZero) ? kExpZero : a + b; }

// A stored vector has a raw exponent m and the bit pattern of its largest magnitude (kept by integer
// atomicMax, which is exact and order-independent).  Its normalising shift f puts that maximum into
// [0.5, 1): the vector's consumers use the exponent m + f and the scale 2^-f.
__device__ __forceinline__ int norm_shift(uint32_t maxbits) { return max((int)((maxbits >> 23) & 0xffu) - 126, -126); }
__device__ __forceinline__ int norm_exp(int m, uint32_t maxbits) {
  return (maxbits == 0u || m == kExpZero) ? kExpZero : m + norm_shift(maxbits);
}
__device__ __forceinline__ float norm_scale(uint32_t maxbits) {
  return maxbits == 0u ? 0.0f : ldexpf(1.0f, -norm_shift(maxbits));
}

// A projected half row (eta or zeta of a span) is stored as 2^-f * [L or R] * (stored inside vector), with the
// exponent m + f of its inside vector (f = norm_shift(tmaxb)).  Its producer also records
//   psum = max_B (biased exponent of max_A W[A,B]) + (biased exponent of the stored inside entry B)      (0: all zero)
// so that the largest entry of W * (stored inside vector) lies in [2^(psum - 254), 4 N 2^(psum - 254)).  The
// consumers read the half row as 2^-g * stored with g = (psum - 253) - f (clamped to the fp32 exponent range): its
// largest entry is then in [0.5, 2 N), and products of two such values cannot leave the fp32 range however small
// (or large) the grammar's weights are.
__device__ __forceinline__ int bexp(float x) { return (int)((__float_as_uint(x) >> 23) & 0xffu); }
__device__ __forceinline__ int bexp_sum(float w, float x) {
  const int a = bexp(w), b = bexp(x);
  return (a == 0 || b == 0) ? 0 : a + b;
}
__device__ __forceinline__ int proj_shift(uint32_t tmaxbits, int psum) {
  return min(max((psum - 253) - norm_shift(tmaxbits), -126), 126);
}
__device__ __forceinline__ int proj_exp(int m, uint32_t tmaxbits, int psum) {
  const int e = norm_exp(m, tmaxbits);
  return (e == kExpZero || psum == 0) ? kExpZero : e + proj_shift(tmaxbits, psum);
}

// ------------------------------------------------------------------------------------------ span plan
// Width-synchronous schedule (Sec. 3.2, span-level parallelism): rows are ordered by width.  Within a width the
// order is: the prefix spans (i = 0) of all sentences, then the other spans that do not end the sentence
// (sentence by sentence, by start), then the suffix spans (j = n, i > 0).  A prefix span is never a right
// child and a suffix span never a left child, so the first two blocks are exactly the rows whose left projection
// (eta) is used and the last two blocks those whose right projection (zeta) is used: each is one contiguous row
// range for the projection products.  Width 1, and every width when each sentence has its own grammar, keep the
// plain (sentence, start) order; the three tables then describe that order.
//   rowtab[0 * stride + w * B + b]  row of span (0, w) of sentence b (-1 if the sentence is shorter)
//   rowtab[1 * stride + w * B + b]  row of span (1, 1 + w) (the spans 1 .. n-w-1 follow each other)
//   rowtab[2 * stride + w * B + b]  row of span (n - w, n)
__device__ __forceinline__ int row_of(const int32_t* __restrict__ rowtab, int stride, int B, int w, int b, int i,
                                      int n) {
  const int which = i == 0 ? 0 : (i == n - w ? 2 : 1);
  return rowtab[which * stride + w * B + b] + (which == 1 ? i - 1 : 0);
}

__global__ void k_plan_rowbase(LenArg la, int B, int n_max, int by_sentence, int32_t* __restrict__ lens,
                               int32_t* __restrict__ rowtab, int32_t* __restrict__ rootrow,
                               int32_t* __restrict__ counters, int n_counters) {
  __shared__ int s_w[kMaxLen + 2];
  const int stride = (n_max + 1) * B;
  for (int t = threadIdx.x; t < n_counters; t += blockDim.x) counters[t] = 0;  // GEMM arrival counters
  for (int b = threadIdx.x; b < B; b += blockDim.x) lens[b] = la.v[b];
  for (int w = 1 + threadIdx.x; w <= n_max; w += blockDim.x) {
    int s = 0;
    for (int b = 0; b < B; ++b) s += max(0, la.v[b] - w + 1);
    s_w[w] = s;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int w = 1; w <= n_max; ++w) {
      int s = s_w[w];
      s_w[w] = run;
      run += s;
    }
  }
  __syncthreads();
  for (int w = 1 + threadIdx.x; w <= n_max; w += blockDim.x) {
    const int base = s_w[w];
    int* tp = rowtab + w * B;
    int* tm = rowtab + stride + w * B;
    int* ts = rowtab + 2 * stride + w * B;
    if (by_sentence || w == 1) {
      int run = base;
      for (int b = 0; b < B; ++b) {
        const int cnt = la.v[b] - w + 1;
        tp[b] = cnt > 0 ? run : -1;
        tm[b] = cnt > 0 ? run + 1 : -1;
        ts[b] = cnt > 0 ? run + cnt - 1 : -1;
        if (cnt == 1) rootrow[b] = run;
        run += max(0, cnt);
      }
    } else {
      int n_pre = 0, n_mid = 0;
      for (int b = 0; b < B; ++b) {
        const int cnt = la.v[b] - w + 1;
        n_pre += cnt > 0 ? 1 : 0;
        n_mid += max(0, cnt - 2);
      }
      int rp = base, rm = base + n_pre, rs = base + n_pre + n_mid;
      for (int b = 0; b < B; ++b) {
        const int cnt = la.v[b] - w + 1;
        if (cnt <= 0) { tp[b] = tm[b] = ts[b] = -1; continue; }
        tp[b] = rp;
        tm[b] = rm;
        ts[b] = cnt >= 2 ? rs : rp;  // a span that is the whole sentence is both: it sits in the prefix block
        if (cnt == 1) rootrow[b] = rp;
        rp += 1;
        rm += max(0, cnt - 2);
        rs += cnt >= 2 ? 1 : 0;
      }
    }
  }
}

__global__ void k_plan_rows(int B, int stride, const int32_t* __restrict__ lens, const int32_t* __restrict__ rowtab,
                            int32_t* __restrict__ row_b, int32_t* __restrict__ row_i,
                            int32_t* __restrict__ rootmask, uint32_t* __restrict__ tmaxb,
                            uint32_t* __restrict__ umaxb, int32_t* __restrict__ hmaxb,
                            int32_t* __restrict__ zmaxb) {
  const int w = blockIdx.x + 1, b = blockIdx.y;
  const int n = lens[b];
  if (w > n) return;
  for (int i = threadIdx.x; i <= n - w; i += blockDim.x) {
    const int r = row_of(rowtab, stride, B, w, b, i, n);
    row_b[r] = b;
    row_i[r] = i;
    rootmask[r] = (w == n) ? 1 : 0;
    tmaxb[r] = 0u;
    umaxb[r] = 0u;
    hmaxb[r] = 0;
    zmaxb[r] = 0;
  }
}

// Rows of width >= 2 listed sentence by sentence (width, then start): the reduction order of the per-sentence
// rule gradients.  Sentence b owns entries [sum_{b'<b} n_b'(n_b'-1)/2, + n_b(n_b-1)/2).
__global__ void k_plan_sentrows(int B, int stride, const int32_t* __restrict__ lens,
                                const int32_t* __restrict__ rowtab, int32_t* __restrict__ sentrows,
                                int32_t* __restrict__ sentoff) {
  const int w = blockIdx.x + 2, b = blockIdx.y;
  const int n = lens[b];
  if (w > n) return;
  int64_t off = 0;
  for (int bb = 0; bb < b; ++bb) off += (int64_t)lens[bb] * (lens[bb] - 1) / 2;
  if (w == 2 && threadIdx.x == 0) sentoff[b] = (int32_t)off;
  // spans of widths 2..w-1 of this sentence: sum_{v=2}^{w-1} (n - v + 1)
  off += (int64_t)(w - 2) * (n + 1) - ((int64_t)w * (w - 1) / 2 - 1);
  for (int i = threadIdx.x; i <= n - w; i += blockDim.x) sentrows[off + i] = row_of(rowtab, stride, B, w, b, i, n);
}

// ------------------------------------------------------------------------------------------ weights
// Stacks [L;R] (Sec. 3.2, kernel fusion: one matrix product for both projections) into zero-padded,
// K-contiguous operands: Wn [2Np x Np] / Wp [2Np x Pp] for the forward products and their transposes
// Wtn [Np x 2Np] / Wtp [Pp x 2Np] for the reverse products.
// Element store of a packed panel: OutT float or __bf16 writes the value; uint16_t writes the first NPL bf16 pieces
// of the cut (nt::Split3) into planes `stride` elements apart.  A null panel is skipped.
template <int NPL, typename OutT> __device__ __forceinline__ void put_w(OutT* w, int64_t, int64_t at, float v) {
  if (w != nullptr) w[at] = (OutT)v;
}
template <int NPL> __device__ __forceinline__ void put_w(uint16_t* w, int64_t stride, int64_t at, float v) {
  if (w == nullptr) return;
  unsigned h, m, l;
  nt::Split3::cut2(v, 0.0f, h, m, l);
  w[at] = (uint16_t)h; w[stride + at] = (uint16_t)m;
  if (NPL == 3) w[2 * stride + at] = (uint16_t)l;
}
// OutT = uint16_t: NPL (2 or 3) bf16 planes per panel (plane strides 2Np*Np resp. 2Np*Pp elements; a grammar's
// panel set is then NPL times as long)
template <typename OutT, int NPL>
__global__ void k_pack_weights(const float* __restrict__ L, const float* __restrict__ R, int N, int P, int Np,
                               int Pp, OutT* __restrict__ Wn, OutT* __restrict__ Wp, OutT* __restrict__ Wtn,
                               OutT* __restrict__ Wtp, uint32_t* __restrict__ colmax) {
  const int64_t sn = 2 * (int64_t)Np * Np, sp = 2 * (int64_t)Np * Pp;
  __shared__ float tile[32][33];
  const int M = N + P;
  const int gi = blockIdx.z >> 1, lr = blockIdx.z & 1;  // grammar, left / right factor
  const float* src = (lr ? R : L) + (int64_t)gi * N * M;
  if (Wn) Wn += (int64_t)gi * NPL * sn;
  if (Wtn) Wtn += (int64_t)gi * NPL * sn;
  if (Wp) Wp += (int64_t)gi * NPL * sp;
  if (Wtp) Wtp += (int64_t)gi * NPL * sp;
  const int half = lr * Np;
  const int c0 = blockIdx.x * 32;  // padded column: [0,Np) nonterminal part, [Np, Np+Pp) preterminal part
  const int a0 = blockIdx.y * 32;
  const bool ppart = c0 >= Np;
  const int cc0 = ppart ? c0 - Np : c0;
  const int tx = threadIdx.x, ty = threadIdx.y;  // 32 x 8
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int a = a0 + ty + 8 * q, c = cc0 + tx;
    float v = 0.0f;
    if (a < N && c < (ppart ? P : N)) v = src[(int64_t)a * M + (ppart ? N + c : c)];
    tile[ty + 8 * q][tx] = v;
    if (ppart) put_w<NPL>(Wp, sp, (int64_t)(half + a) * Pp + c, v); else put_w<NPL>(Wn, sn, (int64_t)(half + a) * Np + c, v);
  }
  __syncthreads();
  if (colmax != nullptr && ty == 0) {
    // colmax[(g * 2 + lr) * (Np + Pp) + c] = max_A W[A, c] over the padded columns c (nonterminals [0, Np), then
    // preterminals): feeds the exponent bounds of the projections (see proj_shift).  Weights are non-negative, so the
    // maximum of the bit patterns is the maximum of the values; the array is zeroed before this kernel.
    float m = 0.0f;
#pragma unroll
    for (int q = 0; q < 32; ++q) m = fmaxf(m, tile[q][tx]);
    if (m > 0.0f) atomicMax(colmax + (int64_t)blockIdx.z * (Np + Pp) + c0 + tx, __float_as_uint(m));
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int c = cc0 + ty + 8 * q, a = a0 + tx;
    const float v = tile[tx][ty + 8 * q];
    if (ppart) put_w<NPL>(Wtp, sp, (int64_t)c * (2 * Np) + half + a, v); else put_w<NPL>(Wtn, sn, (int64_t)c * (2 * Np) + half + a, v);
  }
}

// Operand planes of the rule-gradient product on planes: the three bf16 pieces of sc[s] * X[s][.] for s < S, zero for
// the rows up to the end of the last 32-row step (the product reads whole steps).  One thread per four columns.
__global__ void k_scaled_planes(const float* __restrict__ X, int64_t ld, const float* __restrict__ sc, int64_t S,
                                uint16_t* __restrict__ planes, int64_t plane_stride) {
  const int64_t s = blockIdx.x;
  const int c = (blockIdx.y * blockDim.x + threadIdx.x) * 4;
  if (c >= ld) return;
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (s < S) {
    const float f = sc[s];
    const float4 x = *reinterpret_cast<const float4*>(X + s * ld + c);
    v = make_float4(f * x.x, f * x.y, f * x.z, f * x.w);
  }
  store_planes4(planes, 3, plane_stride, s * ld + c, v);
}

__global__ void k_zero_plane_rows(uint16_t* __restrict__ planes, int64_t plane_stride, int64_t first, int64_t count) {
  uint16_t* p = planes + (int64_t)blockIdx.y * plane_stride + first;
  for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 8; i < count; i += (int64_t)gridDim.x * blockDim.x * 8)
    *reinterpret_cast<uint4*>(p + i) = uint4{0u, 0u, 0u, 0u};  // count and first are multiples of 8 elements
}

__global__ void k_zero_u32(uint32_t* __restrict__ p, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0u;
}

// Xt[c][s] = bf16(sc[s] * X[s][c]) for s < S, 0 for S <= s < Spad: the reduction-major operands of the
// rule-gradient product, transposed so that the bf16 GEMM reads both K-contiguously.
__global__ void k_transpose_bf16(const float* __restrict__ X, int64_t ldx, const float* __restrict__ sc, int64_t S,
                                 int64_t Spad, __bf16* __restrict__ Xt) {
  __shared__ float tile[64][65];
  const int64_t s0 = (int64_t)blockIdx.x * 64;
  const int c0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;  // 64 x 4
#pragma unroll 4
  for (int q = 0; q < 16; ++q) {
    const int64_t s = s0 + ty + 4 * q;
    float v = 0.0f;
    if (s < S) v = X[s * ldx + c0 + tx] * (sc ? sc[s] : 1.0f);
    tile[ty + 4 * q][tx] = v;
  }
  __syncthreads();
  const int c = threadIdx.x >> 2, sq = (threadIdx.x & 3) * 16;
  __bf16* out = Xt + (int64_t)(c0 + c) * Spad + s0 + sq;
#pragma unroll
  for (int j = 0; j < 16; ++j) out[j] = (__bf16)tile[sq + j][c];
}

// ------------------------------------------------------------------------------------------ leaves
// Base case (Sec. 3.1): the inside vector of token i is its emission vector; it is stored as
// exp(e - max e) with the maximum kept aside (it re-enters only in log Z).
__global__ void k_leaf_prep(const float* __restrict__ log_emit, int P, int Pp, int n_max,
                            const int32_t* __restrict__ row_b, const int32_t* __restrict__ row_i,
                            float* __restrict__ leafE, float* __restrict__ xs, int32_t* __restrict__ mexp,
                            uint32_t* __restrict__ tmaxb, uint16_t* __restrict__ leafEb, int planes,
                            int64_t plane_stride, const float* __restrict__ colmax, int Np, int per_sentence,
                            int32_t* __restrict__ hmaxb, int32_t* __restrict__ zmaxb) {
  __shared__ float red[16];
  __shared__ int redi[16];
  const int r = blockIdx.x;
  const float* e = log_emit + ((int64_t)row_b[r] * n_max + row_i[r]) * P;
  float mx = -INFINITY;
  for (int t = threadIdx.x; t < P; t += blockDim.x) mx = fmaxf(mx, e[t]);
  mx = block_max(mx, red);
  const bool dead = !(mx > -INFINITY);
  const float x = dead ? 0.0f : mx;
  float* out = leafE + (int64_t)r * Pp;
  const float* cmL = colmax + (int64_t)(per_sentence ? row_b[r] : 0) * 2 * (Np + Pp) + Np;  // preterminal columns of L
  const float* cmR = cmL + (Np + Pp);
  int hs = 0, zs = 0;
  for (int t = threadIdx.x; t < Pp; t += blockDim.x) {
    const float v = (t < P && !dead) ? expf(e[t] - x) : 0.0f;
    out[t] = v;
    hs = max(hs, bexp_sum(cmL[t], v));
    zs = max(zs, bexp_sum(cmR[t], v));
    if (leafEb) {
      if (planes == 3) put_w<3>(leafEb, plane_stride, (int64_t)r * Pp + t, v);
      else if (planes == 2) put_w<2>(leafEb, plane_stride, (int64_t)r * Pp + t, v);
      else reinterpret_cast<__bf16*>(leafEb)[(int64_t)r * Pp + t] = (__bf16)v;
    }
  }
  hs = block_max_i(hs, redi);
  zs = block_max_i(zs, redi);
  if (threadIdx.x == 0) {
    xs[r] = x;
    mexp[r] = dead ? kExpZero : 0;
    tmaxb[r] = dead ? 0u : __float_as_uint(1.0f);  // the largest entry is exactly 1
    hmaxb[r] = hs;
    zmaxb[r] = zs;
  }
}

// ------------------------------------------------------------------------------------------ forward split
// beta_ij = sum_k eta_ik * zeta_kj (Sec. 3.1 vector form) for every span of one width, in the scaled
// representation: T = sum_k 2^(d_k - m) etat_ik * zetat_kj with d_k = e_ik + e_kj, m = max_k d_k.
// One wavefront per (span, block of 256 nonterminals): split-point rows and coefficients are staged in
// LDS, eight split points (16 row loads) are in flight per lane, the per-span maximum that drives the
// rescaling of Sec. 3.2 is a wavefront reduction followed by one integer atomicMax, and nothing per split
// point goes to HBM.  The normalisation itself is applied by the projection GEMM's epilogue.
// KG = 4 is the shape for launches with few spans and many split points (the late widths), which would leave
// most of the chip idle: the wavefront covers 64 nonterminals and its four groups of 16 lanes take every fourth
// split point, so four times as many wavefronts run and each walks a quarter of the split points.
constexpr int kChunk = 256;  // nonterminals per wavefront (4 per lane) when KG = 1

template <int KG>
__global__ void __launch_bounds__(64)
k_split_fwd(int w, int64_t row0, int B, int Np, int64_t S1, int stride, const int32_t* __restrict__ lens,
            const int32_t* __restrict__ rowtab, const int32_t* __restrict__ row_b,
            const int32_t* __restrict__ row_i, const float* __restrict__ HZ,
            float* __restrict__ T, int32_t* __restrict__ mexp, uint32_t* __restrict__ tmaxb, void* __restrict__ Tb,
            int planes, int64_t plane_stride, int32_t* __restrict__ hmaxb, int32_t* __restrict__ zmaxb,
            const float* __restrict__ colmax, int Pp, int per_sentence) {
  extern __shared__ __align__(16) unsigned char smem[];
  float* s_c = reinterpret_cast<float*>(smem);                 // [w-1] coefficient of the left child's eta
  float* s_cz = s_c + (w - 1);                                 // [w-1] coefficient of the right child's zeta
  int32_t* s_l = reinterpret_cast<int32_t*>(s_cz + (w - 1));   // [w-1] row of the left child
  int32_t* s_r = s_l + (w - 1);                                // [w-1] row of the right child
  const int lane = threadIdx.x;
  const int64_t r = row0 + blockIdx.x;
  const int b = row_b[r], i = row_i[r];
  const int n = lens[b];
  int dmax = kExpZero;
  for (int k = 1 + lane; k < w; k += 64) {
    const int lr = row_of(rowtab, stride, B, k, b, i, n);          // span (i, i+k)
    const int rr = row_of(rowtab, stride, B, w - k, b, i + k, n);  // span (i+k, i+w)
    s_l[k - 1] = lr;
    s_r[k - 1] = rr;
    const int d = add_exp(proj_exp(mexp[lr], tmaxb[lr], hmaxb[lr]), proj_exp(mexp[rr], tmaxb[rr], zmaxb[rr]));
    s_c[k - 1] = __int_as_float(d);
    s_cz[k - 1] = __int_as_float(proj_shift(tmaxb[lr], hmaxb[lr]));  // eta's shift, used once m is known
    dmax = max(dmax, d);
  }
  const int m = wave_max_i(dmax);
  __syncthreads();
  // the term of split point k is 2^(d_k - m) * (2^-gh eta) * (2^-gz zeta): the first two factors go with eta
  // (coefficient 2^(d_k - m - gh)), the last with zeta (coefficient 2^-gz); both products stay at or below 1
  for (int k = lane; k < w - 1; k += 64) {
    const int d = __float_as_int(s_c[k]);
    const int gh = __float_as_int(s_cz[k]);
    s_c[k] = (d == kExpZero) ? 0.0f : pow2i(d - m - gh);
    s_cz[k] = (d == kExpZero) ? 0.0f : pow2i(-proj_shift(tmaxb[s_r[k]], zmaxb[s_r[k]]));
  }
  __syncthreads();

  const int64_t ld = 2 * (int64_t)Np;
  constexpr int LG = 64 / KG;          // lanes per split-point group
  const int kg = lane / LG;            // this lane's group: it takes the split points kg, kg + KG, ...
  const int a = blockIdx.y * (LG * 4) + (lane % LG) * 4;
  float tmax = 0.0f;
  int hsum = 0, zsum = 0;
  if (a < Np) {  // always true for KG > 1 (the padded width is a multiple of 64): the shuffles below see every lane
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    const float* hz_l = HZ + a;
    const float* hz_r = HZ + Np + a;
    int k = 0;
    for (; k + 8 * KG <= w - 1; k += 8 * KG) {
      float4 h[8], z[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        h[u] = *reinterpret_cast<const float4*>(hz_l + s_l[k + u * KG + kg] * ld);
        z[u] = *reinterpret_cast<const float4*>(hz_r + s_r[k + u * KG + kg] * ld);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const float c = s_c[k + u * KG + kg], cz = s_cz[k + u * KG + kg];
        acc.x = fmaf(c * h[u].x, cz * z[u].x, acc.x);
        acc.y = fmaf(c * h[u].y, cz * z[u].y, acc.y);
        acc.z = fmaf(c * h[u].z, cz * z[u].z, acc.z);
        acc.w = fmaf(c * h[u].w, cz * z[u].w, acc.w);
      }
    }
    for (; k < w - 1; k += 4 * KG) {  // remainder in masked groups of four: no serial chain of dependent loads
      float4 h[4], z[4];
      float c[4], cz[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int idx = k + u * KG + kg;
        const int kk = min(idx, w - 2);
        c[u] = (idx < w - 1) ? s_c[kk] : 0.0f;
        cz[u] = s_cz[kk];
        h[u] = *reinterpret_cast<const float4*>(hz_l + s_l[kk] * ld);
        z[u] = *reinterpret_cast<const float4*>(hz_r + s_r[kk] * ld);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        acc.x = fmaf(c[u] * h[u].x, cz[u] * z[u].x, acc.x);
        acc.y = fmaf(c[u] * h[u].y, cz[u] * z[u].y, acc.y);
        acc.z = fmaf(c[u] * h[u].z, cz[u] * z[u].z, acc.z);
        acc.w = fmaf(c[u] * h[u].w, cz[u] * z[u].w, acc.w);
      }
    }
    if (KG > 1) {  // sum of the groups' partial sums, in a fixed order
#pragma unroll
      for (int o = LG; o < 64; o <<= 1) {
        acc.x += __shfl_xor(acc.x, o, 64);
        acc.y += __shfl_xor(acc.y, o, 64);
        acc.z += __shfl_xor(acc.z, o, 64);
        acc.w += __shfl_xor(acc.w, o, 64);
      }
    }
    if (kg == 0) {
      *reinterpret_cast<float4*>(T + (r - S1) * Np + a) = acc;
      if (Tb) store_planes4(Tb, planes, plane_stride, (r - S1) * Np + a, acc);
    }
    tmax = fmaxf(fmaxf(acc.x, acc.y), fmaxf(acc.z, acc.w));
    // exponent bounds of this vector's two projections (see proj_shift)
    const float* cmL = colmax + (int64_t)(per_sentence ? b : 0) * 2 * (Np + Pp) + a;
    const float4 wl = *reinterpret_cast<const float4*>(cmL), wr = *reinterpret_cast<const float4*>(cmL + Np + Pp);
    hsum = max(max(bexp_sum(wl.x, acc.x), bexp_sum(wl.y, acc.y)), max(bexp_sum(wl.z, acc.z), bexp_sum(wl.w, acc.w)));
    zsum = max(max(bexp_sum(wr.x, acc.x), bexp_sum(wr.y, acc.y)), max(bexp_sum(wr.z, acc.z), bexp_sum(wr.w, acc.w)));
  }
  tmax = wave_max(tmax);
  hsum = wave_max_i(hsum);
  zsum = wave_max_i(zsum);
  if (lane == 0) {
    if (tmax > 0.0f && m != kExpZero) atomicMax(&tmaxb[r], __float_as_uint(tmax));
    if (hsum > 0 && m != kExpZero) atomicMax(&hmaxb[r], hsum);
    if (zsum > 0 && m != kExpZero) atomicMax(&zmaxb[r], zsum);
    if (blockIdx.y == 0) mexp[r] = m;
  }
}

// ------------------------------------------------------------------------------------------ root
// Z = sum_A pi(S->A) beta_0n[A] (rule S -> A, Sec. 2).
__global__ void k_root_fwd(int B, int N, int Np, int64_t S1, const int32_t* __restrict__ lens,
                           const int32_t* __restrict__ rowbase, const int32_t* __restrict__ rootrow,
                           const float* __restrict__ log_root, const float* __restrict__ T,
                           const int32_t* __restrict__ mexp, const uint32_t* __restrict__ tmaxb,
                           const float* __restrict__ xs, float* __restrict__ logZ, float* __restrict__ ztil,
                           float* __restrict__ rmaxs, int64_t root_stride) {
  __shared__ float redf[16];
  __shared__ double redd[16];
  const int b = blockIdx.x;
  log_root += b * root_stride;
  const int64_t r = rootrow[b];
  float rm = -INFINITY;
  for (int a = threadIdx.x; a < N; a += blockDim.x) rm = fmaxf(rm, log_root[a]);
  rm = block_max(rm, redf);
  const bool deadroot = !(rm > -INFINITY);
  const float rmx = deadroot ? 0.0f : rm;
  const float* t = T + (r - S1) * Np;
  const float fs = norm_scale(tmaxb[r]);
  double z = 0.0;
  for (int a = threadIdx.x; a < N; a += blockDim.x) z += (double)expf(log_root[a] - rmx) * (double)(t[a] * fs);
  z = block_sum_d(z, redd);
  double sx = 0.0;
  const int n = lens[b];
  const int leaf0 = rowbase[1 * B + b];  // width 1 keeps the (sentence, start) order
  for (int i = threadIdx.x; i < n; i += blockDim.x) sx += (double)xs[leaf0 + i];
  sx = block_sum_d(sx, redd);
  if (threadIdx.x == 0) {
    const int e = norm_exp(mexp[r], tmaxb[r]);
    const bool dead = deadroot || e == kExpZero || !(z > 0.0);
    logZ[b] = dead ? -INFINITY : (float)((double)rmx + log(z) + (double)e * 0.6931471805599453094 + sx);
    ztil[b] = dead ? 0.0f : (float)z;
    rmaxs[b] = rmx;
  }
}

// d logZ / d beta_0n[A] = pi(S->A) / Z.  Scaled adjoint of the root span: BH = g * r[A] / Zt, exponent -e_0n.
__global__ void k_root_bwd(int N, int Np, int64_t S1, const int32_t* __restrict__ rootrow,
                           const float* __restrict__ log_root, const float* __restrict__ grad_logZ,
                           const float* __restrict__ ztil, const float* __restrict__ rmaxs,
                           const int32_t* __restrict__ mexp, const uint32_t* __restrict__ tmaxb,
                           float* __restrict__ BH, float* __restrict__ UV, int32_t* __restrict__ uexp,
                           uint32_t* __restrict__ umaxb, float* __restrict__ gsc, int64_t root_stride,
                           uint16_t* __restrict__ UVb, int planes, int64_t plane_stride) {
  const int b = blockIdx.x;
  log_root += b * root_stride;
  const int64_t r = rootrow[b];
  const float g = grad_logZ ? grad_logZ[b] : 1.0f;
  const float zt = ztil[b];
  const bool dead = !(zt > 0.0f) || g == 0.0f;
  const float s = dead ? 0.0f : g / zt;
  const float rmx = rmaxs[b];
  float* bh = BH + (r - S1) * Np;
  float* uv = UV + r * 2 * (int64_t)Np;
  for (int a = threadIdx.x; a < Np; a += blockDim.x) {
    bh[a] = (a < N && !dead) ? s * expf(log_root[a] - rmx) : 0.0f;
    uv[a] = 0.0f;
    uv[Np + a] = 0.0f;
    if (UVb) {
      for (int pl = 0; pl < planes; ++pl) {  // bf16 zero is the all-zero bit pattern
        UVb[pl * plane_stride + r * 2 * (int64_t)Np + a] = 0;
        UVb[pl * plane_stride + r * 2 * (int64_t)Np + Np + a] = 0;
      }
    }
  }
  if (threadIdx.x == 0) {
    // consumers read the exponent of BH as uexp + norm_shift(umaxb); 0.5 has shift 0
    uexp[r] = dead ? kExpZero : -norm_exp(mexp[r], tmaxb[r]);
    umaxb[r] = dead ? 0u : __float_as_uint(0.5f);
    gsc[r] = 0.0f;
  }
}

// grad_log_root[A] = sum_b g_b * pi(S->A) beta_0n[A] / Z_b  (root posteriors); fixed summation order.
__global__ void k_grad_log_root(int B, int N, int Np, int64_t S1, const int32_t* __restrict__ rootrow,
                                const float* __restrict__ log_root, const float* __restrict__ grad_logZ,
                                const float* __restrict__ ztil, const float* __restrict__ rmaxs,
                                const float* __restrict__ T, const uint32_t* __restrict__ tmaxb,
                                float* __restrict__ grad_log_root, int accumulate, int per_sentence) {
  const int a = blockIdx.x * blockDim.x + threadIdx.x;
  if (a >= N) return;
  int b_lo = 0, b_hi = B;
  if (per_sentence) {  // one root vector and one gradient per sentence: no sum over the batch
    b_lo = blockIdx.y; b_hi = b_lo + 1;
    log_root += (int64_t)b_lo * N;
    grad_log_root += (int64_t)b_lo * N;
  }
  const float lr = log_root[a];
  float acc = 0.0f;
  for (int b0 = b_lo; b0 < b_hi; b0 += 8) {  // eight sentences' loads in flight; summed in sentence order
    float t[8], coef[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int b = min(b0 + u, b_hi - 1);
      const float zt = ztil[b];
      const int64_t r = rootrow[b];
      const float g = grad_logZ ? grad_logZ[b] : 1.0f;
      const bool on = b0 + u < b_hi && zt > 0.0f;
      t[u] = T[(r - S1) * Np + a] * norm_scale(tmaxb[r]);  // the root span's inside vector: always written, finite
      coef[u] = on ? g * expf(lr - rmaxs[b]) / zt : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += coef[u] * t[u];
  }
  grad_log_root[a] = accumulate ? grad_log_root[a] + acc : acc;
}

// ------------------------------------------------------------------------------------------ reverse split
// Reverse of the split-point sum in gather form (Sec. 3.2 "Recomputation": the per-split products are
// recomputed from the stored projections, never saved).  For the span (i,j):
//   adjoint of eta_ij  = sum_{j'>j} adj(beta_ij') * zeta_jj'     (as the left child of (i,j'))
//   adjoint of zeta_ij = sum_{i'<i} adj(beta_i'j) * eta_i'i      (as the right child of (i',j))
// Both are written with one common exponent so that they can be projected back through [L;R] together;
// as in the forward pass one wavefront handles (span, 256 nonterminals) and the normalisation by the
// largest magnitude is left to the GEMM epilogue.
__global__ void __launch_bounds__(64)
k_split_bwd(int w, int64_t row0, int B, int Np, int64_t S1, int stride, const int32_t* __restrict__ lens,
            const int32_t* __restrict__ rowtab, const int32_t* __restrict__ row_b,
            const int32_t* __restrict__ row_i, const int32_t* __restrict__ rootmask,
            const float* __restrict__ HZ, const float* __restrict__ BH, const int32_t* __restrict__ mexp,
            const uint32_t* __restrict__ tmaxb, float* __restrict__ UV, int32_t* __restrict__ uexp,
            uint32_t* __restrict__ umaxb, float* __restrict__ gsc, void* __restrict__ UVb, int planes,
            int64_t plane_stride, const int32_t* __restrict__ hmaxb, const int32_t* __restrict__ zmaxb) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x;
  const int64_t r = row0 + blockIdx.x;
  if (rootmask[r]) return;  // the root span has no parent; its adjoint comes from k_root_bwd
  const int b = row_b[r], i = row_i[r];
  const int n = lens[b];
  const int j = i + w;
  const int nl = n - j;  // parents (i, j'), j' = j+1..n   (this span is their left child)
  const int nr = i;      // parents (i', j), i' = 0..i-1   (this span is their right child)
  const int nt = nl + nr;
  float* s_c = reinterpret_cast<float*>(smem);             // [nt] coefficient of the parent's adjoint
  float* s_cs = s_c + nt;                                  // [nt] coefficient of the sibling's projection
  int32_t* s_p = reinterpret_cast<int32_t*>(s_cs + nt);    // [nt] parent row (index into BH: row - S1)
  int32_t* s_s = s_p + nt;                                 // [nt] sibling row

  int dmax = kExpZero;
  for (int t = lane; t < nt; t += 64) {
    int pr, sr;
    if (t < nl) {
      const int jp = j + 1 + t;
      pr = row_of(rowtab, stride, B, jp - i, b, i, n);   // parent (i, j')
      sr = row_of(rowtab, stride, B, jp - j, b, j, n);   // sibling (j, j'), used through its zeta
    } else {
      const int ip = t - nl;
      pr = row_of(rowtab, stride, B, j - ip, b, ip, n);  // parent (i', j)
      sr = row_of(rowtab, stride, B, i - ip, b, ip, n);  // sibling (i', i), used through its eta
    }
    s_p[t] = pr - (int)S1;
    s_s[t] = sr;
    const int sb = t < nl ? zmaxb[sr] : hmaxb[sr];  // the sibling's zeta (this span is the left child) or eta
    const int d = add_exp(norm_exp(uexp[pr], umaxb[pr]), proj_exp(mexp[sr], tmaxb[sr], sb));
    s_c[t] = __int_as_float(d);
    s_cs[t] = pow2i(-proj_shift(tmaxb[sr], sb));
    dmax = max(dmax, d);
  }
  const int m = wave_max_i(dmax);
  __syncthreads();
  for (int t = lane; t < nt; t += 64) {
    const int d = __float_as_int(s_c[t]);
    s_c[t] = (d == kExpZero) ? 0.0f : pow2i(d - m);
    if (d == kExpZero) s_cs[t] = 0.0f;
  }
  __syncthreads();

  const int64_t ld = 2 * (int64_t)Np;
  const int a = blockIdx.y * kChunk + lane * 4;
  float amax = 0.0f;
  if (a < Np) {
    float4 u = make_float4(0.f, 0.f, 0.f, 0.f), v = make_float4(0.f, 0.f, 0.f, 0.f);
    const float* bh = BH + a;
    // left-child role: sibling zeta (second half of HZ); right-child role: sibling eta (first half)
#define SPCFG_GATHER(ACC, T0, T1, HZOFF)                                                        \
  {                                                                                             \
    int t = (T0);                                                                               \
    for (; t + 8 <= (T1); t += 8) {                                                             \
      float4 gq[8], sq[8];                                                                      \
      _Pragma("unroll") for (int q = 0; q < 8; ++q) {                                           \
        gq[q] = *reinterpret_cast<const float4*>(bh + (int64_t)s_p[t + q] * Np);                \
        sq[q] = *reinterpret_cast<const float4*>(HZ + s_s[t + q] * ld + (HZOFF) + a);           \
      }                                                                                         \
      _Pragma("unroll") for (int q = 0; q < 8; ++q) {                                           \
        const float c = s_c[t + q], cs = s_cs[t + q];                                           \
        ACC.x = fmaf(c * gq[q].x, cs * sq[q].x, ACC.x);                                         \
        ACC.y = fmaf(c * gq[q].y, cs * sq[q].y, ACC.y);                                         \
        ACC.z = fmaf(c * gq[q].z, cs * sq[q].z, ACC.z);                                         \
        ACC.w = fmaf(c * gq[q].w, cs * sq[q].w, ACC.w);                                         \
      }                                                                                         \
    }                                                                                           \
    for (; t < (T1); t += 4) {                                                                  \
      float4 gq[4], sq[4];                                                                      \
      float cq[4], cs[4];                                                                       \
      _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                           \
        const int tt = min(t + q, (T1)-1);                                                      \
        cq[q] = (t + q < (T1)) ? s_c[tt] : 0.0f;                                                \
        cs[q] = s_cs[tt];                                                                       \
        gq[q] = *reinterpret_cast<const float4*>(bh + (int64_t)s_p[tt] * Np);                   \
        sq[q] = *reinterpret_cast<const float4*>(HZ + s_s[tt] * ld + (HZOFF) + a);              \
      }                                                                                         \
      _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                           \
        ACC.x = fmaf(cq[q] * gq[q].x, cs[q] * sq[q].x, ACC.x);                                  \
        ACC.y = fmaf(cq[q] * gq[q].y, cs[q] * sq[q].y, ACC.y);                                  \
        ACC.z = fmaf(cq[q] * gq[q].z, cs[q] * sq[q].z, ACC.z);                                  \
        ACC.w = fmaf(cq[q] * gq[q].w, cs[q] * sq[q].w, ACC.w);                                  \
      }                                                                                         \
    }                                                                                           \
  }
    SPCFG_GATHER(u, 0, nl, Np)
    SPCFG_GATHER(v, nl, nt, 0)
#undef SPCFG_GATHER
    float* out = UV + r * ld;
    *reinterpret_cast<float4*>(out + a) = u;
    *reinterpret_cast<float4*>(out + Np + a) = v;
    if (UVb) {
      store_planes4(UVb, planes, plane_stride, r * ld + a, u);
      store_planes4(UVb, planes, plane_stride, r * ld + Np + a, v);
    }
    amax = fmaxf(fmaxf(fmaxf(fabsf(u.x), fabsf(u.y)), fmaxf(fabsf(u.z), fabsf(u.w))),
                 fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
  }
  amax = wave_max(amax);
  if (lane == 0) {
    if (amax > 0.0f && m != kExpZero) atomicMax(&umaxb[r], __float_as_uint(amax));
    if (blockIdx.y == 0) {
      uexp[r] = m;
      // scale that turns UV[r] (x) (stored inside vector of the row) into its contribution to dZ/d[L;R]
      const int me = mexp[r];
      gsc[r] = (m == kExpZero || me == kExpZero) ? 0.0f : pow2i(max(m + me, -160));
    }
  }
}

// grad_log_emit is zero at padded token positions.
__global__ void k_zero_pad_emit(int P, int n_max, const int32_t* __restrict__ lens, float* __restrict__ g) {
  const int b = blockIdx.x;
  const int n = lens[b];
  float* base = g + ((int64_t)b * n_max + n) * P;
  const int64_t cnt = (int64_t)(n_max - n) * P;
  for (int64_t t = threadIdx.x; t < cnt; t += blockDim.x) base[t] = 0.0f;
}

// ------------------------------------------------------------------------------------------ span posteriors
// mu(i,j) = sum_A beta_ij[A] * d logZ / d beta_ij[A]: the posterior probability that some nonterminal spans
// (i,j) (inside-outside by back-propagation, Sec. 3.2).  Both factors are still in the workspace after the
// reverse pass: beta = 2^mexp * T and its adjoint = 2^(uexp + f') * BH.  One wavefront per (sentence, i, j-1)
// entry of the dense output; entries that are no span get 0 / -1.  Width-1 spans carry the same mass as the
// root span (both are in every tree), so they read the root row.  label = first arg-max nonterminal.
__global__ void __launch_bounds__(64)
k_span_marginals(int B, int N, int Np, int n_max, int64_t S1, const int32_t* __restrict__ lens,
                 const int32_t* __restrict__ rowtab, const float* __restrict__ T, const float* __restrict__ BH,
                 const int32_t* __restrict__ mexp, const int32_t* __restrict__ uexp,
                 const uint32_t* __restrict__ umaxb, float* __restrict__ mu, int32_t* __restrict__ label) {
  const int lane = threadIdx.x;
  const int b = blockIdx.y;
  const int i = blockIdx.x / n_max, j = blockIdx.x % n_max + 1;
  const int n = lens[b];
  const int64_t out = ((int64_t)b * n_max + i) * n_max + (j - 1);
  if (j <= i || j > n) {
    if (lane == 0) {
      mu[out] = 0.0f;
      if (label) label[out] = -1;
    }
    return;
  }
  const int w = j - i;
  const int stride = (n_max + 1) * B;
  const int64_t r = (w == 1) ? rowtab[n * B + b] : row_of(rowtab, stride, B, w, b, i, n);
  const float* t = T + (r - S1) * Np;
  const float* h = BH + (r - S1) * Np;
  float sum = 0.0f, best = 0.0f;
  int arg = -1;
  for (int a = lane * 4; a < Np; a += 256) {
    const float4 x = *reinterpret_cast<const float4*>(t + a);
    const float4 y = *reinterpret_cast<const float4*>(h + a);
    const float p0 = x.x * y.x, p1 = x.y * y.y, p2 = x.z * y.z, p3 = x.w * y.w;
    sum += (p0 + p1) + (p2 + p3);
    if (p0 > best) { best = p0; arg = a; }
    if (p1 > best) { best = p1; arg = a + 1; }
    if (p2 > best) { best = p2; arg = a + 2; }
    if (p3 > best) { best = p3; arg = a + 3; }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    sum += __shfl_xor(sum, o, 64);
    const float ob = __shfl_xor(best, o, 64);
    const int oa = __shfl_xor(arg, o, 64);
    if (ob > best || (ob == best && oa >= 0 && (arg < 0 || oa < arg))) { best = ob; arg = oa; }
  }
  if (lane == 0) {
    const int d = add_exp(mexp[r], norm_exp(uexp[r], umaxb[r]));
    const float m = (d == kExpZero) ? 0.0f : pow2i(d) * sum;
    mu[out] = m;
    if (label) label[out] = (w >= 2 && m > 0.0f && arg < N) ? arg : -1;
  }
}

}  // namespace

void launch_plan(const Layout& ly, const Ptrs& p, const LenArg& lens, hipStream_t st) {
  launch_k(k_plan_rowbase, dim3(1), dim3(256), 0, st, lens, ly.B, ly.n_max, ly.G > 1 ? 1 : 0, p.lens, p.rowbase,
           p.rootrow,
                     p.counters, ly.n_counters);
  launch_k(k_plan_rows, dim3(ly.n_max, ly.B), dim3(64), 0, st, ly.B, (ly.n_max + 1) * ly.B, p.lens, p.rowbase, p.row_b, p.row_i,
                     p.rootmask, p.tmaxb, p.umaxb, p.hmaxb, p.zmaxb);
}

void launch_plan_sentrows(const Layout& ly, const Ptrs& p, hipStream_t st) {
  if (ly.n_max < 2) return;
  launch_k(k_plan_sentrows, dim3(ly.n_max - 1, ly.B), dim3(64), 0, st, ly.B, (ly.n_max + 1) * ly.B, p.lens, p.rowbase, p.sentrows,
                     p.sentoff);
}

void launch_pack_weights(const Layout& ly, const Ptrs& p, const float* L, const float* R, hipStream_t st) {
  dim3 grid((ly.Np + ly.Pp) / 32, ly.Np / 32, 2 * ly.G);
  uint32_t* cm = reinterpret_cast<uint32_t*>(p.colmax);
  const int64_t ncm = 2 * (int64_t)(ly.Np + ly.Pp) * ly.G;
  launch_k(k_zero_u32, dim3((unsigned)((ncm + 255) / 256 < 1024 ? (ncm + 255) / 256 : 1024)), dim3(256), 0, st, cm, ncm);
  if (ly.planes == 3)  // the panels once more as three bf16 planes
    launch_k(k_pack_weights<uint16_t, 3>, grid, dim3(32, 8), 0, st, L, R, ly.N, ly.P, ly.Np, ly.Pp,
                       (uint16_t*)p.Wn3, (uint16_t*)p.Wp3, (uint16_t*)p.Wtn3, (uint16_t*)p.Wtp3, (uint32_t*)nullptr);
  if (ly.planes == 2)  // the panels of the forward products as two bf16 planes
    launch_k(k_pack_weights<uint16_t, 2>, grid, dim3(32, 8), 0, st, L, R, ly.N, ly.P, ly.Np, ly.Pp,
                       (uint16_t*)p.Wn3, (uint16_t*)p.Wp3, (uint16_t*)nullptr, (uint16_t*)nullptr, (uint32_t*)nullptr);
  if (ly.fwd_fp32) {  // fp32 panels for the forward products, bf16 panels for the reverse ones
    launch_k(k_pack_weights<float, 1>, grid, dim3(32, 8), 0, st, L, R, ly.N, ly.P, ly.Np, ly.Pp, p.Wn, p.Wp,
                       (float*)nullptr, (float*)nullptr, cm);
    launch_k(k_pack_weights<__bf16, 1>, grid, dim3(32, 8), 0, st, L, R, ly.N, ly.P, ly.Np, ly.Pp,
                       (__bf16*)nullptr, (__bf16*)nullptr, (__bf16*)p.Wtn, (__bf16*)p.Wtp, (uint32_t*)nullptr);
    return;
  }
  if (ly.planes == 2)  // single bf16 panels of the reverse products only
    launch_k(k_pack_weights<__bf16, 1>, grid, dim3(32, 8), 0, st, L, R, ly.N, ly.P, ly.Np, ly.Pp,
                       (__bf16*)nullptr, (__bf16*)nullptr, (__bf16*)p.Wtn, (__bf16*)p.Wtp, cm);
  else if (ly.bf16)
    launch_k(k_pack_weights<__bf16, 1>, grid, dim3(32, 8), 0, st, L, R, ly.N, ly.P, ly.Np, ly.Pp,
                       (__bf16*)p.Wn, (__bf16*)p.Wp, (__bf16*)p.Wtn, (__bf16*)p.Wtp, cm);
  else
    launch_k(k_pack_weights<float, 1>, grid, dim3(32, 8), 0, st, L, R, ly.N, ly.P, ly.Np, ly.Pp, p.Wn, p.Wp,
                       p.Wtn, p.Wtp, cm);
}

void launch_scaled_planes(const float* X, int64_t ld, const float* sc, int64_t S, int64_t Srows, void* planes,
                          int64_t plane_stride, hipStream_t st) {
  if (Srows <= 0) return;
  const dim3 grid((unsigned)Srows, (unsigned)((ld / 4 + 255) / 256));
  launch_k(k_scaled_planes, grid, dim3(256), 0, st, X, ld, sc, S, static_cast<uint16_t*>(planes), plane_stride);
}

void launch_zero_plane_rows(void* planes, int64_t plane_stride, int64_t ld, int64_t row0, int64_t rows, hipStream_t st) {
  const int64_t count = rows * ld;  // ld is a multiple of 64
  launch_k(k_zero_plane_rows, dim3((unsigned)((count / 8 + 255) / 256 < 256 ? (count / 8 + 255) / 256 : 256), 3), dim3(256), 0, st,
           static_cast<uint16_t*>(planes), plane_stride, row0 * ld, count);
}

void launch_transpose_bf16(const float* X, int64_t ldx, int cols, const float* sc, int64_t S, int64_t Spad, void* Xt,
                           hipStream_t st) {
  dim3 grid((unsigned)(Spad / 64), (unsigned)(cols / 64));
  launch_k(k_transpose_bf16, grid, dim3(256), 0, st, X, ldx, sc, S, Spad, (__bf16*)Xt);
}

void launch_leaf_prep(const Layout& ly, const Ptrs& p, const float* log_emit, bool write_planes, hipStream_t st) {
  launch_k(k_leaf_prep, dim3((unsigned)ly.S1), dim3(256), 0, st, log_emit, ly.P, ly.Pp, ly.n_max, p.row_b,
                     p.row_i, p.leafE, p.xs, p.mexp, p.tmaxb, static_cast<uint16_t*>(write_planes ? p.leafEb : nullptr), ly.planes,
                     (int64_t)ly.S1 * ly.Pp, p.colmax, ly.Np, ly.G > 1 ? 1 : 0, p.hmaxb, p.zmaxb);
}

void launch_split_fwd(const Layout& ly, const Ptrs& p, int w, int64_t row0, int64_t rows, bool write_planes,
                      hipStream_t st) {
  void* Tb = write_planes ? p.Tb : nullptr;
  const size_t sh = (size_t)(w - 1) * 16;
  const int chunks = (ly.Np + kChunk - 1) / kChunk;
  if (rows * chunks < 1024 && w - 1 >= 64) {  // fewer than one wavefront per SIMD, long chains of split points
    const dim3 grid((unsigned)rows, (unsigned)(ly.Np / 64));
    launch_k(k_split_fwd<4>, grid, dim3(64), sh, st, w, row0, ly.B, ly.Np, ly.S1, (ly.n_max + 1) * ly.B, p.lens, p.rowbase, p.row_b, p.row_i, p.HZ,
             p.T, p.mexp, p.tmaxb, Tb, ly.planes, (int64_t)ly.S2 * ly.Np, p.hmaxb, p.zmaxb, p.colmax, ly.Pp,
             ly.G > 1 ? 1 : 0);
    return;
  }
  const dim3 grid((unsigned)rows, (unsigned)chunks);
  launch_k(k_split_fwd<1>, grid, dim3(64), sh, st, w, row0, ly.B, ly.Np, ly.S1, (ly.n_max + 1) * ly.B, p.lens, p.rowbase, p.row_b, p.row_i, p.HZ,
           p.T, p.mexp, p.tmaxb, Tb, ly.planes, (int64_t)ly.S2 * ly.Np, p.hmaxb, p.zmaxb, p.colmax, ly.Pp,
           ly.G > 1 ? 1 : 0);
}

void launch_root_fwd(const Layout& ly, const Ptrs& p, const float* log_root, float* logZ, hipStream_t st) {
  launch_k(k_root_fwd, dim3(ly.B), dim3(256), 0, st, ly.B, ly.N, ly.Np, ly.S1, p.lens, p.rowbase,
                     p.rootrow, log_root, p.T, p.mexp, p.tmaxb, p.xs, logZ, p.ztil, p.rmax,
                     (int64_t)(ly.G > 1 ? ly.N : 0));
}

void launch_root_bwd(const Layout& ly, const Ptrs& p, const float* log_root, const float* grad_logZ,
                     float* grad_log_root, int accumulate, hipStream_t st) {
  launch_k(k_root_bwd, dim3(ly.B), dim3(256), 0, st, ly.N, ly.Np, ly.S1, p.rootrow, log_root, grad_logZ,
                     p.ztil, p.rmax, p.mexp, p.tmaxb, p.BH, p.UV, p.uexp, p.umaxb, p.gsc,
                     (int64_t)(ly.G > 1 ? ly.N : 0), static_cast<uint16_t*>(p.UVb), ly.planes_bwd,
                     ly.uvb_plane);
  launch_k(k_grad_log_root, dim3((ly.N + 255) / 256, ly.G > 1 ? ly.B : 1), dim3(256), 0, st, ly.B, ly.N,
                     ly.Np, ly.S1, p.rootrow, log_root, grad_logZ, p.ztil, p.rmax, p.T, p.tmaxb, grad_log_root,
                     accumulate, ly.G > 1 ? 1 : 0);
}

void launch_split_bwd(const Layout& ly, const Ptrs& p, int w, int64_t row0, int64_t rows, bool write_planes,
                      hipStream_t st) {
  const size_t sh = (size_t)ly.n_max * 16;
  const dim3 grid((unsigned)rows, (unsigned)((ly.Np + kChunk - 1) / kChunk));
  launch_k(k_split_bwd, grid, dim3(64), sh, st, w, row0, ly.B, ly.Np, ly.S1, (ly.n_max + 1) * ly.B, p.lens, p.rowbase, p.row_b,
                     p.row_i, p.rootmask, p.HZ, p.BH, p.mexp, p.tmaxb, p.UV, p.uexp, p.umaxb, p.gsc, write_planes ? p.UVb : nullptr, ly.planes_bwd,
                     ly.uvb_plane, p.hmaxb, p.zmaxb);
}

void launch_zero_pad_emit(const Layout& ly, const Ptrs& p, float* grad_log_emit, hipStream_t st) {
  launch_k(k_zero_pad_emit, dim3(ly.B), dim3(256), 0, st, ly.P, ly.n_max, p.lens, grad_log_emit);
}

void launch_span_marginals(const Layout& ly, const Ptrs& p, float* mu, int32_t* label, hipStream_t st) {
  const dim3 grid((unsigned)(ly.n_max * ly.n_max), (unsigned)ly.B);
  launch_k(k_span_marginals, grid, dim3(64), 0, st, ly.B, ly.N, ly.Np, ly.n_max, ly.S1, p.lens, p.rowbase,
                     p.T, p.BH, p.mexp, p.uexp, p.umaxb, mu, label);
}

}  // namespace spcfg
