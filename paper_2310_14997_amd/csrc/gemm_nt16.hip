// bf16-operand MFMA GEMM (fp32 accumulate) for the projections in SPCFG_PRECISION_BF16:
//   C[r][c] = sum_k A[r][k] * Bm[c][k],  Bm = packed bf16 [L;R] panel, A = the bf16 copy of the chart rows that
// their producers write next to the fp32 ones (or the transposed operands of the rule-gradient product).
// Same tiling, work sharing and epilogues as the fp32 kernel; one K-step is 64 values, and every
// MFMA operand is one 16-byte LDS read of 8 consecutive bf16 (v_mfma_f32_32x32x16_bf16: lane l holds row
// l % 32, k = 8 * (l / 32) .. + 7).
#include "gemm_nt_common.h"

namespace spcfg {

namespace {

using namespace nt;
constexpr int BK = 64;  // bf16 values per K-step

template <int EPI, int BM, bool GROUPED>
__global__ void __launch_bounds__(256, 2) k_gemm_nt16(NtArgs g, int ipw, int total_iters) {
  using G = Geo<BM>;
  extern __shared__ __align__(16) float lds[];
  __shared__ int s_last;
  // grouped mode (one grammar per sentence): first row tile, first row and row count of every sentence
  __shared__ int s_tile0[GROUPED ? kMaxB + 1 : 1], s_row0[GROUPED ? kMaxB : 1], s_cnt[GROUPED ? kMaxB : 1];
  __shared__ int s_wsum[4];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave % G::WM, wn = wave / G::WM;
  int tiles_m = (g.rows + BM - 1) / BM;
  if (GROUPED) tiles_m = build_group_table<BM>(g, s_tile0, s_row0, s_cnt, s_wsum, tid);
  const int KT = g.K / BK;
  // staging of both operands: 8 chunks of 16 bytes (8 bf16) per row and K-step, 32 rows per pass
  const int lc8 = tid & 7, lr8 = tid >> 3;
  constexpr int QA = BM / 32;  // chunks of A per thread and K-step
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
    int row0 = tile_m * BM, row_end = g.rows;
    const int col0 = tile_n * BN;
    const __bf16* Bh = static_cast<const __bf16*>(g.Bm);
    if (GROUPED) Bh += (int64_t)find_group<BM>(g, s_tile0, s_row0, s_cnt, tile_m, &row0, &row_end) * g.grp_b_stride;

    // element offsets of this thread's chunks (row clamped into range: out-of-range rows are never stored)
    int64_t oa[QA], ob[4];
#pragma unroll
    for (int q = 0; q < QA; ++q)
      oa[q] = (int64_t)min(row0 + lr8 + 32 * q, row_end - 1) * g.lda + lc8 * 8;
#pragma unroll
    for (int q = 0; q < 4; ++q) ob[q] = (int64_t)min(col0 + lr8 + 32 * q, g.cols - 1) * g.ldb + lc8 * 8;
    const __bf16* Ah = static_cast<const __bf16*>(g.A);

    floatx4 ra0, ra1, ra2, ra3, rb0, rb1, rb2, rb3;  // 8 bf16 each; named: arrays would go to scratch
#define SPCFG_LDA(R, Q, KOFF) \
  if (QA > (Q)) R = *reinterpret_cast<const floatx4*>(Ah + oa[(Q) < QA ? (Q) : 0] + (KOFF));
#define SPCFG_LOAD_TILE(KOFF)                                                                     \
  SPCFG_LDA(ra0, 0, KOFF) SPCFG_LDA(ra1, 1, KOFF) SPCFG_LDA(ra2, 2, KOFF) SPCFG_LDA(ra3, 3, KOFF) \
  rb0 = *reinterpret_cast<const floatx4*>(Bh + ob[0] + (KOFF));                                   \
  rb1 = *reinterpret_cast<const floatx4*>(Bh + ob[1] + (KOFF));                                   \
  rb2 = *reinterpret_cast<const floatx4*>(Bh + ob[2] + (KOFF));                                   \
  rb3 = *reinterpret_cast<const floatx4*>(Bh + ob[3] + (KOFF));
#define SPCFG_STA(R, Q, DST) \
  if (QA > (Q)) *reinterpret_cast<floatx4*>((DST) + (lr8 + 32 * (Q)) * LDT + lc8 * 4) = R;
#define SPCFG_STORE_TILE(DST)                                                                     \
  SPCFG_STA(ra0, 0, DST) SPCFG_STA(ra1, 1, DST) SPCFG_STA(ra2, 2, DST) SPCFG_STA(ra3, 3, DST)     \
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

    finish_tile<BM>(g.partial, g.counters, acc, tile, tile * KT, k0, k1, KT, ipw, wg, it, wg_begin, tid, &s_last,
                    [&](floatx16(&t)[G::MI][G::NI]) { epilogue<EPI, BM>(g, t, row0, col0, wm, wn, lane, row_end); });
    it += k1 - k0;
  }
}

template <int EPI, int BM, bool GROUPED>
void launch(const NtArgs& a, hipStream_t st) {
  using G = Geo<BM>;
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_nt16<EPI, BM, GROUPED>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)G::kLdsBytes);
    attr_set = true;
  }
  launch_shared(k_gemm_nt16<EPI, BM, GROUPED>, a, BM, BK, G::kLdsBytes, st);
}

template <int EPI>
void launch_bm(const NtArgs& a, hipStream_t st) {
  if (a.grouped) {
    switch (chosen_bm(a)) {
      case 32: launch<EPI, 32, true>(a, st); break;
      case 64: launch<EPI, 64, true>(a, st); break;
      default: launch<EPI, 128, true>(a, st); break;
    }
    return;
  }
  switch (chosen_bm(a)) {
    case 32: launch<EPI, 32, false>(a, st); break;
    case 64: launch<EPI, 64, false>(a, st); break;
    default: launch<EPI, 128, false>(a, st); break;
  }
}

}  // namespace

void launch_gemm_nt16(const NtArgs& a, hipStream_t st) {
  if (a.rows <= 0 || a.cols <= 0 || !a.a_bf16 || !a.b_bf16) return;  // both operands are bf16 here
  switch (a.epilogue) {
    case NT_EPI_GRAD: launch<NT_EPI_GRAD, 128, false>(a, st); break;
    case NT_EPI_ROWSCALE: launch_bm<NT_EPI_ROWSCALE>(a, st); break;
    case NT_EPI_MASKROWS: launch_bm<NT_EPI_MASKROWS>(a, st); break;
    default: launch_bm<NT_EPI_LEAF_EMIT>(a, st); break;
  }
}

}  // namespace spcfg
