// bf16-operand MFMA GEMM (fp32 accumulate) for the projections in SPCFG_PRECISION_BF16:
//   C[r][c] = sum_k A[r][k] * Bm[c][k],  Bm = packed bf16 [L;R] panel, A = fp32 chart rows rounded to bf16
// while they are staged into LDS (or rows that are bf16 already: the transposed operands of the rule-gradient
// product).  Same tiling, work sharing and epilogues as the fp32 kernel; one K-step is 64 values, and every
// MFMA operand is one 16-byte LDS read of 8 consecutive bf16 (v_mfma_f32_32x32x16_bf16: lane l holds row
// l % 32, k = 8 * (l / 32) .. + 7).
#include "gemm_nt_common.h"

namespace spcfg {

namespace {

using namespace nt;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
constexpr int BK = 64;  // bf16 values per K-step

__device__ __forceinline__ bf16x4 to_bf16(floatx4 x) {
  bf16x4 r;
  r[0] = (__bf16)x[0]; r[1] = (__bf16)x[1]; r[2] = (__bf16)x[2]; r[3] = (__bf16)x[3];
  return r;
}

// A_BF16 = false: A rows are fp32 (16 chunks of 16 bytes per K-step row, 16 rows per staging pass);
// A_BF16 = true : A rows are bf16 (8 chunks per row, 32 rows per pass).
template <int EPI, int BM, bool A_BF16>
__global__ void __launch_bounds__(256, 2) k_gemm_nt16(NtArgs g, int ipw, int total_iters) {
  using G = Geo<BM>;
  extern __shared__ __align__(16) float lds[];
  __shared__ int s_last;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave % G::WM, wn = wave / G::WM;
  const int tiles_m = (g.rows + BM - 1) / BM;
  const int KT = g.K / BK;
  // staging of Bm (and of a bf16 A): 8 chunks of 16 bytes per row, 32 rows per pass
  const int lc8 = tid & 7, lr8 = tid >> 3;
  // staging of an fp32 A: 16 chunks of 16 bytes (4 floats) per row, 16 rows per pass; 8 bytes of bf16 out
  const int lc16 = tid & 15, lr16 = tid >> 4;
  constexpr int QA = A_BF16 ? BM / 32 : BM / 16;  // chunks of A per thread and K-step
  const int frag_row = lane & 31, frag_h = lane >> 5;
  const int a_off = (wm * G::MI * 32 + frag_row) * LDT + frag_h * 4;  // in words; chunk c adds 8 words
  const int b_off = BM * LDT + (wn * G::NI * 32 + frag_row) * LDT + frag_h * 4;

  const int wg = renumbered_wg();
  const int wg_begin = wg * ipw;
  const int wg_end = min(wg_begin + ipw, total_iters);
  int it = wg_begin;
  while (it < wg_end) {
    const int tile = it / KT;
    const int k0 = it - tile * KT;
    const int k1 = min(KT, k0 + (wg_end - it));
    const int tile_m = tile % tiles_m, tile_n = tile / tiles_m;
    const int row0 = tile_m * BM, col0 = tile_n * BN;

    // element offsets of this thread's chunks (row clamped into range: out-of-range rows are never stored)
    int64_t oa[QA], ob[4];
#pragma unroll
    for (int q = 0; q < QA; ++q)
      oa[q] = A_BF16 ? (int64_t)min(row0 + lr8 + 32 * q, g.rows - 1) * g.lda + lc8 * 8
                     : (int64_t)min(row0 + lr16 + 16 * q, g.rows - 1) * g.lda + lc16 * 4;
#pragma unroll
    for (int q = 0; q < 4; ++q) ob[q] = (int64_t)min(col0 + lr8 + 32 * q, g.cols - 1) * g.ldb + lc8 * 8;
    const float* Af = static_cast<const float*>(g.A);
    const __bf16* Ah = static_cast<const __bf16*>(g.A);
    const __bf16* Bh = static_cast<const __bf16*>(g.Bm);

    floatx4 ra0, ra1, ra2, ra3, ra4, ra5, ra6, ra7, rb0, rb1, rb2, rb3;  // named: arrays would go to scratch
#define SPCFG_LDA(R, Q, KOFF)                                                                     \
  if (QA > (Q))                                                                                   \
    R = A_BF16 ? *reinterpret_cast<const floatx4*>(Ah + oa[(Q) < QA ? (Q) : 0] + (KOFF))          \
               : *reinterpret_cast<const floatx4*>(Af + oa[(Q) < QA ? (Q) : 0] + (KOFF));
#define SPCFG_LOAD_TILE(KOFF)                                                                     \
  SPCFG_LDA(ra0, 0, KOFF) SPCFG_LDA(ra1, 1, KOFF) SPCFG_LDA(ra2, 2, KOFF) SPCFG_LDA(ra3, 3, KOFF) \
  SPCFG_LDA(ra4, 4, KOFF) SPCFG_LDA(ra5, 5, KOFF) SPCFG_LDA(ra6, 6, KOFF) SPCFG_LDA(ra7, 7, KOFF) \
  rb0 = *reinterpret_cast<const floatx4*>(Bh + ob[0] + (KOFF));                                   \
  rb1 = *reinterpret_cast<const floatx4*>(Bh + ob[1] + (KOFF));                                   \
  rb2 = *reinterpret_cast<const floatx4*>(Bh + ob[2] + (KOFF));                                   \
  rb3 = *reinterpret_cast<const floatx4*>(Bh + ob[3] + (KOFF));
#define SPCFG_STA(R, Q, DST)                                                                      \
  if (QA > (Q)) {                                                                                 \
    if (A_BF16) *reinterpret_cast<floatx4*>((DST) + (lr8 + 32 * (Q)) * LDT + lc8 * 4) = R;        \
    else *reinterpret_cast<bf16x4*>((DST) + (lr16 + 16 * (Q)) * LDT + lc16 * 2) = to_bf16(R);     \
  }
#define SPCFG_STORE_TILE(DST)                                                                     \
  SPCFG_STA(ra0, 0, DST) SPCFG_STA(ra1, 1, DST) SPCFG_STA(ra2, 2, DST) SPCFG_STA(ra3, 3, DST)     \
  SPCFG_STA(ra4, 4, DST) SPCFG_STA(ra5, 5, DST) SPCFG_STA(ra6, 6, DST) SPCFG_STA(ra7, 7, DST)     \
  *reinterpret_cast<floatx4*>((DST) + BM * LDT + (lr8) * LDT + lc8 * 4) = rb0;                    \
  *reinterpret_cast<floatx4*>((DST) + BM * LDT + (lr8 + 32) * LDT + lc8 * 4) = rb1;               \
  *reinterpret_cast<floatx4*>((DST) + BM * LDT + (lr8 + 64) * LDT + lc8 * 4) = rb2;               \
  *reinterpret_cast<floatx4*>((DST) + BM * LDT + (lr8 + 96) * LDT + lc8 * 4) = rb3;

    floatx16 acc[G::MI][G::NI];
#pragma unroll
    for (int mi = 0; mi < G::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < G::NI; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

    SPCFG_LOAD_TILE(k0 * BK)
    SPCFG_STORE_TILE(lds)
    __syncthreads();

    for (int kt = k0; kt < k1; ++kt) {
      const int buf = (kt - k0) & 1;
      const int kn = min(kt + 1, k1 - 1) * BK;  // the last step re-reads itself (stored, never used)
      SPCFG_LOAD_TILE(kn)
      __builtin_amdgcn_sched_barrier(0);  // keep the prefetch loads at the top of the step
      const float* as = lds + buf * G::kStage + a_off;
      const float* bs = lds + buf * G::kStage + b_off;
#define SPCFG_FRAGS(C)                                                                                      \
  _Pragma("unroll") for (int mi = 0; mi < G::MI; ++mi) a[mi] =                                              \
      *reinterpret_cast<const bf16x8*>(as + mi * 32 * LDT + (C)*8);                                         \
  _Pragma("unroll") for (int ni = 0; ni < G::NI; ++ni) b[ni] =                                              \
      *reinterpret_cast<const bf16x8*>(bs + ni * 32 * LDT + (C)*8);
#define SPCFG_MFMAS                                                                                         \
  _Pragma("unroll") for (int mi = 0; mi < G::MI; ++mi) _Pragma("unroll") for (int ni = 0; ni < G::NI; ++ni) \
      acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
#define SPCFG_CHUNK(C)      \
  {                         \
    bf16x8 a[G::MI], b[G::NI]; \
    SPCFG_FRAGS(C)          \
    SPCFG_MFMAS             \
  }
      SPCFG_CHUNK(0)
      SPCFG_CHUNK(1)
      SPCFG_CHUNK(2)
      {
        bf16x8 a[G::MI], b[G::NI];
        SPCFG_FRAGS(3)  // fetched before the LDS stores below so that their latency hides behind chunk 2
        __builtin_amdgcn_sched_barrier(0);
        SPCFG_STORE_TILE(lds + (buf ^ 1) * G::kStage)
        __builtin_amdgcn_sched_barrier(0);
        SPCFG_MFMAS
      }
#undef SPCFG_CHUNK
#undef SPCFG_MFMAS
#undef SPCFG_FRAGS
      __builtin_amdgcn_sched_barrier(0);
      __syncthreads();
    }
#undef SPCFG_LDA
#undef SPCFG_LOAD_TILE
#undef SPCFG_STA
#undef SPCFG_STORE_TILE

    finish_tile<BM>(g.partial, g.counters, acc, tile, k0, k1, KT, ipw, wg, it, wg_begin, tid, &s_last,
                    [&](floatx16(&t)[G::MI][G::NI]) { epilogue<EPI, BM>(g, t, row0, col0, wm, wn, lane, g.rows); });
    it += k1 - k0;
  }
}

template <int EPI, int BM, bool A_BF16>
void launch(const NtArgs& a, hipStream_t st) {
  using G = Geo<BM>;
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_nt16<EPI, BM, A_BF16>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)G::kLdsBytes);
    attr_set = true;
  }
  launch_shared(k_gemm_nt16<EPI, BM, A_BF16>, a, BM, BK, G::kLdsBytes, st);
}

template <int EPI, bool A_BF16>
void launch_bm(const NtArgs& a, hipStream_t st) {
  switch (chosen_bm(a)) {
    case 32: launch<EPI, 32, A_BF16>(a, st); break;
    case 64: launch<EPI, 64, A_BF16>(a, st); break;
    default: launch<EPI, 128, A_BF16>(a, st); break;
  }
}

}  // namespace

void launch_gemm_nt16(const NtArgs& a, hipStream_t st) {
  if (a.rows <= 0 || a.cols <= 0) return;
  if (a.a_bf16) {  // only the rule-gradient product has both operands in bf16
    launch<NT_EPI_GRAD, 128, true>(a, st);
    return;
  }
  switch (a.epilogue) {
    case NT_EPI_ROWSCALE: launch_bm<NT_EPI_ROWSCALE, false>(a, st); break;
    case NT_EPI_MASKROWS: launch_bm<NT_EPI_MASKROWS, false>(a, st); break;
    default: launch_bm<NT_EPI_LEAF_EMIT, false>(a, st); break;
  }
}

}  // namespace spcfg
