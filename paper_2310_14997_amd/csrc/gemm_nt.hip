// fp32-operand MFMA GEMM for the stacked projections (Sec. 3.2: [eta | zeta] = [L;R] * beta for all spans of one
// width at once) and for their reverse:  C[r][c] = sum_k A[r][k] * Bm[c][k], both operands K-contiguous.
//
// gfx950 mapping: 128x128x32 tile per 256-thread workgroup (4 wavefronts, 2x2, 64x64 each = 2x2 tiles of 32x32;
// shorter tiles for widths with few spans), global -> registers -> LDS, one K-step of loads in flight.
// Two inner loops:
//  * default: fp32 products from bf16 matrix instructions (nt::Split3): the staged registers are cut into three
//    bf16 planes on their way into a single LDS stage; per K-step a matrix phase (16-byte operand reads,
//    v_mfma_f32_32x32x16_bf16), a barrier, the cut of the next step, a barrier;
//  * SPCFG_FLAG_FP32_MFMA: v_mfma_f32_32x32x2_f32 on fp32 tiles in two LDS stages, one barrier per K-step; each
//    lane fetches its operands as one 16-byte LDS read covering four K values (the K order inside an 8-wide chunk
//    is permuted identically for both operands, which leaves the sum over K unchanged).
// Work sharing across workgroups and the epilogues are in gemm_nt_common.h.
#include "gemm_nt_common.h"

namespace spcfg {

namespace {

using namespace nt;
constexpr int BK = 32;
// Split-product path: the tile lies in LDS already cut into its three bf16 planes (each thread cuts the 32
// values it stages, so every value is cut once per workgroup and not once per wavefront that multiplies it).
// One K-step of a row is 32 bf16 = 64 bytes per plane, rows lie back to back, and the 16-byte chunk index of a row
// is XORed with bits 2..3 of the row number: the 16-byte operand reads of 16 consecutive rows and the 8-byte stores of
// a wavefront (8 rows of 64 bytes) then touch every bank equally.  One stage: three planes of BM + 128 rows.
constexpr int PRS = 16;  // plane row stride in 4-byte words
__device__ __forceinline__ int plane_swz(int row) { return (row >> 2) & 3; }
template <int BM> constexpr int kPlaneWords = (BM + BN) * PRS;
template <int BM, bool X3> constexpr size_t kLdsBytesNT = X3 ? (size_t)3 * kPlaneWords<BM> * 4 : Geo<BM>::kLdsBytes;

// MODE 0: one product; 1: grouped (one grammar per sentence); 2: parts (several row ranges with their own
// column block and K range in one launch, see NtArgs).
// X3: fp32 products from bf16 matrix instructions (Split3) instead of fp32 ones.
template <int EPI, int BM, int MODE, bool X3>
__global__ void __launch_bounds__(256, 2) k_gemm_nt(NtArgs g, int ipw, int total_iters) {
  constexpr bool GROUPED = MODE == 1, PARTS = MODE == 2;
  using G = Geo<BM>;
  extern __shared__ __align__(16) float lds[];
  __shared__ int s_last;
  // grouped mode: first row tile, first row and row count of every sentence
  __shared__ int s_tile0[GROUPED ? kMaxB + 1 : 1], s_row0[GROUPED ? kMaxB : 1], s_cnt[GROUPED ? kMaxB : 1];
  __shared__ int s_wsum[4];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave % G::WM, wn = wave / G::WM;
  int tiles_m = (g.rows + BM - 1) / BM;
  if (GROUPED) tiles_m = build_group_table<BM>(g, s_tile0, s_row0, s_cnt, s_wsum, tid);
  const int KT = g.K / BK;
  const int lc4 = tid & 7, lr = tid >> 3;  // staging: 8 float4 per tile row, 32 rows per pass
  const int lds_st = lr * LDT + lc4 * 4;
  const int frag_row = lane & 31, frag_k = (lane >> 5) * 4;
  const int a_off = (wm * G::MI * 32 + frag_row) * LDT + frag_k;
  const int b_off = BM * LDT + (wn * G::NI * 32 + frag_row) * LDT + frag_k;

  const int wg = renumbered_wg();
  const int wg_begin = wg * ipw;
  const int wg_end = min(wg_begin + ipw, total_iters);
  int it = wg_begin;
  while (it < wg_end) {
    int tile, ustart, KTt = KT, k0, tile_m, tile_n, row0, row_end = g.rows, c_shift = 0, kbeg = 0;
    if (PARTS) {
      // which part does unit `it` belong to?  (at most three parts; each is tiles * K-steps units long)
      const int tiles_n = (g.cols + BN - 1) / BN;
      int p = 0, ubase = 0, tbase = 0;
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        if (p == q && q + 1 < g.parts) {
          const int tq = ((g.prt_rows[q] + BM - 1) / BM) * tiles_n;
          if (it >= ubase + tq * g.prt_kt[q]) { ubase += tq * g.prt_kt[q]; tbase += tq; p = q + 1; }
        }
      }
      const int tm = (g.prt_rows[p] + BM - 1) / BM;
      KTt = g.prt_kt[p];
      const int u = it - ubase;
      const int tl = u / KTt;
      k0 = u - tl * KTt;
      tile = tbase + tl;
      ustart = ubase + tl * KTt;
      tile_m = tl % tm; tile_n = tl / tm;
      row0 = g.prt_row0[p] + tile_m * BM;
      row_end = g.prt_row0[p] + g.prt_rows[p];
      c_shift = g.prt_c0[p];
      kbeg = g.prt_kbeg[p];
    } else {
      tile = it / KT;
      k0 = it - tile * KT;
      ustart = tile * KT;
      tile_m = tile % tiles_m; tile_n = tile / tiles_m;
      row0 = tile_m * BM;
    }
    const int k1 = min(KTt, k0 + (wg_end - it));
    const int col0 = tile_n * BN;
    // Position p of the tile's K loop is K-step (p + krot) mod KTt: the workgroup that owns the tile's first position is
    // then at K-step (its own step count) mod KTt, so workgroups running side by side on an XCD read the same K range
    // of the operand rows they share at the same time and that XCD's L2 fetches them once.  Shares and partial tiles are
    // made of positions; the order of the sum stays fixed by the launch geometry.
    const int krot = (ustart % ipw) % KTt;
    auto kstep_of = [&](int p) { const int q = p + krot; return q >= KTt ? q - KTt : q; };
    // parts: the part's column block of Bm (rows of the K-contiguous panel) and its K range
    const float* bmat = static_cast<const float*>(g.Bm) + (int64_t)c_shift * g.ldb + (int64_t)kbeg * BK;
    const float* amat = static_cast<const float*>(g.A) + (int64_t)kbeg * BK;
    if (GROUPED) bmat += (int64_t)find_group<BM>(g, s_tile0, s_row0, s_cnt, tile_m, &row0, &row_end) * g.grp_b_stride;

    const float* ga[G::QA];
    const float* gb[4];
#pragma unroll
    for (int q = 0; q < G::QA; ++q)
      ga[q] = amat + (int64_t)min(row0 + lr + 32 * q, row_end - 1) * g.lda + lc4 * 4;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      gb[q] = bmat + (int64_t)min(col0 + lr + 32 * q, g.cols - 1) * g.ldb + lc4 * 4;
    float4 ra0, ra1, ra2, ra3, rb0, rb1, rb2, rb3;  // named scalars: arrays here end up in scratch memory
    floatx16 acc[G::MI][G::NI];
#pragma unroll
    for (int mi = 0; mi < G::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < G::NI; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

#define SPCFG_LOAD_TILE(KOFF)                                                    \
  ra0 = *reinterpret_cast<const float4*>(ga[0] + (KOFF));                         \
  if (G::QA > 1) ra1 = *reinterpret_cast<const float4*>(ga[G::QA > 1 ? 1 : 0] + (KOFF)); \
  if (G::QA > 2) ra2 = *reinterpret_cast<const float4*>(ga[G::QA > 2 ? 2 : 0] + (KOFF)); \
  if (G::QA > 2) ra3 = *reinterpret_cast<const float4*>(ga[G::QA > 2 ? 3 : 0] + (KOFF)); \
  rb0 = *reinterpret_cast<const float4*>(gb[0] + (KOFF));                         \
  rb1 = *reinterpret_cast<const float4*>(gb[1] + (KOFF));                         \
  rb2 = *reinterpret_cast<const float4*>(gb[2] + (KOFF));                         \
  rb3 = *reinterpret_cast<const float4*>(gb[3] + (KOFF));
#define SPCFG_STORE_TILE(DST)                                                    \
  *reinterpret_cast<float4*>((DST)) = ra0;                                        \
  if (G::QA > 1) *reinterpret_cast<float4*>((DST) + 32 * LDT) = ra1;              \
  if (G::QA > 2) *reinterpret_cast<float4*>((DST) + 64 * LDT) = ra2;              \
  if (G::QA > 2) *reinterpret_cast<float4*>((DST) + 96 * LDT) = ra3;              \
  *reinterpret_cast<float4*>((DST) + BM * LDT) = rb0;                             \
  *reinterpret_cast<float4*>((DST) + BM * LDT + 32 * LDT) = rb1;                  \
  *reinterpret_cast<float4*>((DST) + BM * LDT + 64 * LDT) = rb2;                  \
  *reinterpret_cast<float4*>((DST) + BM * LDT + 96 * LDT) = rb3;
    SPCFG_LOAD_TILE(kstep_of(k0) * BK)
    if constexpr (!X3) {
      SPCFG_STORE_TILE(lds + lds_st)
      __syncthreads();
    }

    // MFMA operands of one 8-wide K chunk: named scalars (arrays next to scheduling barriers go to scratch)
#define SPCFG_FRAGS(A0, A1, B0, B1, AS, BS, KC)                                         \
  A0 = *reinterpret_cast<const float4*>((AS) + (KC)*8);                                  \
  if (G::MI > 1) A1 = *reinterpret_cast<const float4*>((AS) + 32 * LDT + (KC)*8);        \
  B0 = *reinterpret_cast<const float4*>((BS) + (KC)*8);                                  \
  if (G::NI > 1) B1 = *reinterpret_cast<const float4*>((BS) + 32 * LDT + (KC)*8);
#define SPCFG_MFMA1(A0, A1, B0, B1, C)                                                                      \
  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(A0.C, B0.C, acc[0][0], 0, 0, 0);                          \
  if (G::NI > 1) acc[0][G::NI - 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(A0.C, B1.C, acc[0][G::NI - 1], 0, 0, 0); \
  if (G::MI > 1) acc[G::MI - 1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(A1.C, B0.C, acc[G::MI - 1][0], 0, 0, 0); \
  if (G::MI > 1 && G::NI > 1)                                                                                \
    acc[G::MI - 1][G::NI - 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(A1.C, B1.C, acc[G::MI - 1][G::NI - 1], 0, 0, 0);
#define SPCFG_MFMA4(A0, A1, B0, B1) \
  SPCFG_MFMA1(A0, A1, B0, B1, x) SPCFG_MFMA1(A0, A1, B0, B1, y) SPCFG_MFMA1(A0, A1, B0, B1, z) SPCFG_MFMA1(A0, A1, B0, B1, w)

    if constexpr (X3) {
    // fp32 products from bf16 matrix instructions (nt::Split3 describes the cut).  Single LDS stage: matrix phase
    // on the stage (24 16-byte operand reads and 48 matrix instructions per wavefront, no vector work), barrier,
    // cut the staged registers of the next step into the stage, barrier.  The two phases of the two workgroups
    // of a CU interleave.
    uint32_t* ldsu = reinterpret_cast<uint32_t*>(lds);
    constexpr int PL = kPlaneWords<BM>;
    // this thread's 4 values (half a 16-byte chunk) of row lr (+ 32 q: the same swizzle)
    const int st_off = lr * PRS + (((lc4 >> 1) ^ plane_swz(lr)) * 4) + (lc4 & 1) * 2;
    // 8 values of chunk 0; chunk 1 is the offset with bit 3 flipped (the next two 16-byte pieces of the row)
    const int fsw = (((lane >> 5) ^ plane_swz(frag_row)) * 4);
    const int fa_off = (wm * G::MI * 32 + frag_row) * PRS + fsw;
    const int fb_off = (BM + wn * G::NI * 32 + frag_row) * PRS + fsw;
#define SPCFG_CUT_STORE1(V, ROWOFF)                                                            \
  {                                                                                            \
    unsigned h0_, m0_, l0_, h1_, m1_, l1_;                                                     \
    Split3::cut2(V.x, V.y, h0_, m0_, l0_);                                                     \
    Split3::cut2(V.z, V.w, h1_, m1_, l1_);                                                     \
    *reinterpret_cast<uint2*>(ldsu + st_off + (ROWOFF)*PRS) = uint2{h0_, h1_};                 \
    *reinterpret_cast<uint2*>(ldsu + PL + st_off + (ROWOFF)*PRS) = uint2{m0_, m1_};            \
    *reinterpret_cast<uint2*>(ldsu + 2 * PL + st_off + (ROWOFF)*PRS) = uint2{l0_, l1_};        \
  }
#define SPCFG_CUT_STORE                                             \
  SPCFG_CUT_STORE1(ra0, 0)                                          \
  if (G::QA > 1) SPCFG_CUT_STORE1(ra1, 32)                          \
  if (G::QA > 2) SPCFG_CUT_STORE1(ra2, 64)                          \
  if (G::QA > 2) SPCFG_CUT_STORE1(ra3, 96)                          \
  SPCFG_CUT_STORE1(rb0, BM) SPCFG_CUT_STORE1(rb1, BM + 32) SPCFG_CUT_STORE1(rb2, BM + 64) SPCFG_CUT_STORE1(rb3, BM + 96)
#define SPCFG_OPER(PLANE, OFF, C) \
  __builtin_bit_cast(bf16x8, *reinterpret_cast<const uintx4*>(ldsu + (PLANE)*PL + ((OFF) ^ (8 * (C)))))
#define SPCFG_MFMA_T(X, Y)                                                                                    \
  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0##X, b0##Y, acc[0][0], 0, 0, 0);                        \
  if (G::NI > 1) acc[0][G::NI - 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0##X, b1##Y, acc[0][G::NI - 1], 0, 0, 0); \
  if (G::MI > 1) acc[G::MI - 1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1##X, b0##Y, acc[G::MI - 1][0], 0, 0, 0); \
  if (G::MI > 1 && G::NI > 1)                                                                                  \
    acc[G::MI - 1][G::NI - 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1##X, b1##Y, acc[G::MI - 1][G::NI - 1], 0, 0, 0);
#define SPCFG_CHUNK(C)                                                                             \
  {                                                                                                \
    const bf16x8 a0h = SPCFG_OPER(0, fa_off, C), a0m = SPCFG_OPER(1, fa_off, C), a0l = SPCFG_OPER(2, fa_off, C); \
    const bf16x8 b0h = SPCFG_OPER(0, fb_off, C), b0m = SPCFG_OPER(1, fb_off, C), b0l = SPCFG_OPER(2, fb_off, C); \
    bf16x8 a1h = a0h, a1m = a0m, a1l = a0l, b1h = b0h, b1m = b0m, b1l = b0l;                       \
    if (G::MI > 1) {                                                                               \
      a1h = SPCFG_OPER(0, fa_off + 32 * PRS, C); a1m = SPCFG_OPER(1, fa_off + 32 * PRS, C);        \
      a1l = SPCFG_OPER(2, fa_off + 32 * PRS, C);                                                   \
    }                                                                                              \
    if (G::NI > 1) {                                                                               \
      b1h = SPCFG_OPER(0, fb_off + 32 * PRS, C); b1m = SPCFG_OPER(1, fb_off + 32 * PRS, C);        \
      b1l = SPCFG_OPER(2, fb_off + 32 * PRS, C);                                                   \
    }                                                                                              \
    SPCFG_MFMA_T(l, h) SPCFG_MFMA_T(h, l) SPCFG_MFMA_T(m, m) SPCFG_MFMA_T(m, h) SPCFG_MFMA_T(h, m) SPCFG_MFMA_T(h, h) \
  }
    SPCFG_CUT_STORE  // the first step (the stage is free: the previous tile segment ended with a barrier)
    __syncthreads();
    for (int kt = k0; kt < k1; ++kt) {
      const bool more = kt + 1 < k1;  // uniform over the workgroup
      if (more) { SPCFG_LOAD_TILE(kstep_of(kt + 1) * BK) }
      __builtin_amdgcn_sched_barrier(0);  // keep the prefetch loads at the top of the step
      SPCFG_CHUNK(0)
      SPCFG_CHUNK(1)
      __builtin_amdgcn_sched_barrier(0);
      if (more) {
        __syncthreads();  // every wavefront has read its operands of this step
        SPCFG_CUT_STORE
        __syncthreads();
      }
    }
#undef SPCFG_CUT_STORE1
#undef SPCFG_CUT_STORE
#undef SPCFG_OPER
#undef SPCFG_MFMA_T
#undef SPCFG_CHUNK
    } else {
    float4 pa0, pa1, pb0, pb1;  // chunk 0 of the current K-step, fetched one step ahead (behind the barrier)
    float4 qa0, qa1, qb0, qb1;  // chunks 1..3
    SPCFG_FRAGS(pa0, pa1, pb0, pb1, lds + a_off, lds + b_off, 0)

    for (int kt = k0; kt < k1; ++kt) {
      const int buf = (kt - k0) & 1;
      // prefetch the next K-step into registers (the last iteration re-reads its own step)
      const int kn = kstep_of(min(kt + 1, k1 - 1)) * BK;
      SPCFG_LOAD_TILE(kn)
      // Pinned schedule (left alone, the compiler sinks the prefetch loads down to their LDS stores and exposes
      // the memory latency in every K-step): loads, chunks 0-2, LDS stores of the prefetched tile (the loads
      // have landed by then), barrier, operands of the NEXT step's chunk 0, and only then the MFMAs of chunk 3,
      // so that the LDS latency right after the barrier hides behind a quarter step of matrix work.
      __builtin_amdgcn_sched_barrier(0);
      const float* as = lds + buf * G::kStage + a_off;
      const float* bs = lds + buf * G::kStage + b_off;
      SPCFG_MFMA4(pa0, pa1, pb0, pb1)
      SPCFG_FRAGS(qa0, qa1, qb0, qb1, as, bs, 1)
      SPCFG_MFMA4(qa0, qa1, qb0, qb1)
      SPCFG_FRAGS(qa0, qa1, qb0, qb1, as, bs, 2)
      SPCFG_MFMA4(qa0, qa1, qb0, qb1)
      SPCFG_FRAGS(qa0, qa1, qb0, qb1, as, bs, 3)
      __builtin_amdgcn_sched_barrier(0);
      SPCFG_STORE_TILE(lds + (buf ^ 1) * G::kStage + lds_st)
      __builtin_amdgcn_sched_barrier(0);
      __syncthreads();
      __builtin_amdgcn_sched_barrier(0);
      SPCFG_FRAGS(pa0, pa1, pb0, pb1, lds + (buf ^ 1) * G::kStage + a_off, lds + (buf ^ 1) * G::kStage + b_off, 0)
      __builtin_amdgcn_sched_barrier(0);
      SPCFG_MFMA4(qa0, qa1, qb0, qb1)
    }
    }
    __syncthreads();  // every wavefront has fetched its last operands before the LDS tiles are reused
#undef SPCFG_FRAGS
#undef SPCFG_MFMA1
#undef SPCFG_MFMA4

    finish_tile<BM>(g.partial, g.counters, acc, tile, ustart, k0, k1, KTt, ipw, wg, it, wg_begin, tid, &s_last,
                    [&](floatx16(&t)[G::MI][G::NI]) {
                      epilogue<EPI, BM>(g, t, row0, col0, wm, wn, lane, row_end, c_shift);
                    });
    it += k1 - k0;
  }
}

template <int EPI, int BM, int MODE, bool X3>
void launch_x(const NtArgs& a, hipStream_t st) {
  using G = Geo<BM>;
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_nt<EPI, BM, MODE, X3>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytesNT<BM, X3>);
    attr_set = true;
  }
  launch_shared(k_gemm_nt<EPI, BM, MODE, X3>, a, BM, BK, kLdsBytesNT<BM, X3>, st);
}

template <int EPI, int BM, int MODE>
void launch(const NtArgs& a, hipStream_t st) {
  if (a.fp32_mfma) launch_x<EPI, BM, MODE, false>(a, st); else launch_x<EPI, BM, MODE, true>(a, st);
}

template <int EPI>
void launch_bm(const NtArgs& a, hipStream_t st) {
  if (a.grouped) {
    switch (chosen_bm(a)) {
      case 32: launch<EPI, 32, 1>(a, st); break;
      case 64: launch<EPI, 64, 1>(a, st); break;
      default: launch<EPI, 128, 1>(a, st); break;
    }
    return;
  }
  if (a.parts > 0) {
    switch (chosen_bm(a)) {
      case 32: launch<EPI, 32, 2>(a, st); break;
      case 64: launch<EPI, 64, 2>(a, st); break;
      default: launch<EPI, 128, 2>(a, st); break;
    }
    return;
  }
  switch (chosen_bm(a)) {
    case 32: launch<EPI, 32, 0>(a, st); break;
    case 64: launch<EPI, 64, 0>(a, st); break;
    default: launch<EPI, 128, 0>(a, st); break;
  }
}

}  // namespace

// number of arrival counters a launch can need (upper bound over the tile heights used)
int gemm_nt_tiles(int rows, int cols) { return ((rows + 31) / 32) * ((cols + nt::BN - 1) / nt::BN); }
size_t gemm_nt_partial_bytes(int max_wgs) { return (size_t)2 * max_wgs * nt::Geo<128>::kSlotFloats * sizeof(float); }

// Parts that cover all columns over different K ranges of the same rows (the reverse product: the adjoint half
// they leave out is zero) can also run as one plain product.  Each part rounds its rows up to whole tiles, so with
// few prefix / suffix rows per width and tall tiles the plain product has fewer (tile, K-step) units: then the parts
// are dropped.  Returns whether the launch keeps its parts.
bool gemm_nt_keep_parts(NtArgs& a) {
  if (a.parts == 0) return false;
  const int bm = nt::chosen_bm(a);
  int units_parts = 0;
  for (int p = 0; p < a.parts; ++p) {
    if (a.prt_c0[p] != 0) return true;  // parts with their own column blocks (the forward product) stay
    units_parts += ((a.prt_rows[p] + bm - 1) / bm) * a.prt_kt[p];
  }
  if (((a.rows + bm - 1) / bm) * (a.K / BK) > units_parts) return true;
  a.parts = 0;
  return false;
}

bool gemm_nt_reads_planes(const NtArgs& a) {
  if (!a.planes3 || a.b_bf16 || a.rows <= 0 || a.cols <= 0 || a.grouped) return false;
  return a.planes3 == 2 || nt::chosen_bm(a) == 128;
}

void launch_gemm_nt(const NtArgs& a, hipStream_t st) {
  if (a.rows <= 0 || a.cols <= 0) return;
  if (a.b_bf16) { launch_gemm_nt16(a, st); return; }
  if (a.planes3) {
    // tall row tiles: the kernel on pre-cut operands; short ones keep the fp32 operands (fewer panel bytes)
    if (gemm_nt_reads_planes(a)) { launch_gemm_nt3(a, st); return; }
    NtArgs b = a;
    b.planes3 = 0;
    launch_gemm_nt(b, st);
    return;
  }
  switch (a.epilogue) {
    case NT_EPI_ROWSCALE: launch_bm<NT_EPI_ROWSCALE>(a, st); break;
    case NT_EPI_MASKROWS: launch_bm<NT_EPI_MASKROWS>(a, st); break;
    default: launch_bm<NT_EPI_LEAF_EMIT>(a, st); break;
  }
}

}  // namespace spcfg
