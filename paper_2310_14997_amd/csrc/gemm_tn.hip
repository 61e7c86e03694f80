// fp32-operand MFMA GEMM for the rule gradients:  d/d[L;R][a][b] = sum_s sc[s] * UV[s][a] * X[s][b], where s runs over
// every span row, UV holds the scaled adjoints of [eta | zeta] and X the stored inside vectors (chain rule
// through the stacked projection of Sec. 3.2).  Both operands are reduction-major, so tiles go to LDS as
// they lie in memory ([s][a], [s][b]) and every MFMA operand is a conflict-free 4-byte LDS read.
// 128x128 output tile, 32 span rows per step, 4 wavefronts (2x2) of 2x2 tiles of 32x32: by default fp32 products
// from bf16 matrix instructions (nt::Split3, fragments cut in registers), with SPCFG_FLAG_FP32_MFMA
// v_mfma_f32_32x32x2_f32.  The per-row power-of-two scale is applied to the A fragments in registers.  The (tile, K-step) space is
// shared among workgroups as in the projection GEMMs, so grammars with few output tiles still fill the chip.
#include "gemm_nt_common.h"

namespace spcfg {

namespace {

using nt::floatx16;
using nt::floatx4;
typedef float floatx8 __attribute__((ext_vector_type(8)));

constexpr int TM = 128, TN = 128, TK = 32;
constexpr int kStageT = (TM + TN) * TK + TK;  // A tile, B tile, scales
constexpr size_t kLdsBytesT = 2 * kStageT * sizeof(float);

// 16 bytes per lane straight from global memory into LDS (lane l lands at lds_base + 16 l; the LDS base is
// uniform over the wavefront).  The builtin exists in the device pass only.
__device__ __forceinline__ void dma16(const float* gptr, float* lds_base) {
#if defined(__HIP_DEVICE_COMPILE__)
  typedef __attribute__((address_space(3))) float lds_float;
  __builtin_amdgcn_global_load_lds(gptr, (lds_float*)lds_base, 16, 0, 0);
#else
  (void)gptr; (void)lds_base;
#endif
}

// MODE 0: one reduction over the contiguous rows [0, S).  MODE 1, 2: one reduction per sentence (grouped mode of
// TnArgs); every workgroup share is a whole number of output tiles, so no partial tiles are exchanged.
// X3: fp32 products from bf16 matrix instructions (nt::Split3) instead of fp32 ones.
template <int MODE, bool X3>
__global__ void __launch_bounds__(256, 2) k_gemm_tn(TnArgs g, int ipw, int total_iters) {
  extern __shared__ __align__(16) float lds[];
  __shared__ int s_last;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1;
  const int tiles_a = (2 * g.Np) / TM;
  const int KT = MODE ? g.grp_kt_max : (int)((g.S + TK - 1) / TK);
  const int wg = nt::renumbered_wg();
  const int wg_begin = wg * ipw;
  const int wg_end = min(wg_begin + ipw, total_iters);
  int it = wg_begin;
  while (it < wg_end) {
  const int tile = it / KT;
  const int k0 = it - tile * KT;
  int k1 = min(KT, k0 + (wg_end - it));
  const int advance = k1 - k0;
  int tile_l = tile, KTg = KT;
  int64_t S = g.S, rbase = 0;
  const int32_t* rl = nullptr;
  float* gL = g.gL;
  float* gR = g.gR;
  if (MODE) {
    const int tiles_pg = tiles_a * ((g.cols + TN - 1) / TN);
    const int grp = tile / tiles_pg;
    tile_l = tile - grp * tiles_pg;
    const int n = g.grp_lens[grp];
    S = MODE == 1 ? (int64_t)n * (n - 1) / 2 : n;
    if (MODE == 1) rl = g.rowlist + g.grp_off[grp]; else rbase = g.grp_base[grp];
    KTg = (int)((S + TK - 1) / TK);
    k1 = min(k1, KTg);
    gL += grp * g.grp_gstride;
    gR += grp * g.grp_gstride;
  }
  int tile_a = tile_l % tiles_a, tile_b = tile_l / tiles_a;
  if (MODE == 0) {
    // 64 consecutive tiles (the tiles one XCD works on at a time: workgroups are renumbered into contiguous runs
    // per XCD) form an 8 x 8 block of the output, so that XCD's L2 fetches 16 operand panels for them and not 34
    const int tiles_bb = (g.cols + TN - 1) / TN;
    if ((tiles_a & 7) == 0 && (tiles_bb & 7) == 0) {
      const int blk = tile_l >> 6, l = tile_l & 63, blocks_a = tiles_a >> 3;
      tile_a = (blk % blocks_a) * 8 + (l & 7);
      tile_b = (blk / blocks_a) * 8 + (l >> 3);
    }
  }
  const int a0 = tile_a * TM, b0 = tile_b * TN;

  const int lc4 = tid & 31, lr = tid >> 5;  // 32 float4 per tile row, 8 rows per pass
  const bool bcol_ok = (b0 + lc4 * 4) < (int)g.ldb;  // ldb is the padded column count of X
  const float* gA = g.A + a0 + lc4 * 4;
  const float* gB = g.Bm + (bcol_ok ? b0 + lc4 * 4 : 0);
  // Tiles go straight from global memory into LDS (16 bytes per lane, lane l of a wavefront lands at base +
  // 16 l): thread (lr, lc4) moves columns 4 lc4 .. +3 of tile row lr + 8 q, and a wavefront's two rows are
  // contiguous in the [row][128] LDS tile.  Rows past the end are read from the last valid row (always in
  // bounds, finite) and contribute nothing because their scale is staged as 0; columns past the padded width
  // of X are read from column 0 and only feed output columns that the epilogue drops.
  float rsc = 0.0f;
  const int uw = __builtin_amdgcn_readfirstlane(wave);
#define SPCFG_TN_DMA1(Q, BUF, S0)                                                                        \
  {                                                                                                      \
    const int64_t s = (S0) + lr + 8 * (Q);                                                               \
    const int64_t sc = s < S ? s : S - 1;                                                                \
    const int64_t sr = MODE == 1 ? (int64_t)rl[sc] : rbase + sc;                                         \
    dma16(gA + sr * g.lda, lds + (BUF)*kStageT + (8 * (Q) + 2 * uw) * TM);                               \
    dma16(gB + (MODE == 1 ? sr - g.brow0 : sr) * g.ldb, lds + (BUF)*kStageT + TM * TK + (8 * (Q) + 2 * uw) * TN); \
  }
#define SPCFG_TN_DMA(BUF, S0)                                                                            \
  SPCFG_TN_DMA1(0, BUF, S0) SPCFG_TN_DMA1(1, BUF, S0) SPCFG_TN_DMA1(2, BUF, S0) SPCFG_TN_DMA1(3, BUF, S0) \
  if (tid < TK) rsc = ((S0) + tid < S) ? g.sc[MODE == 1 ? (int64_t)rl[(S0) + tid] : rbase + (S0) + tid] : 0.0f;
#define SPCFG_TN_STORE_SC(BUF) \
  if (tid < TK) lds[(BUF)*kStageT + (TM + TN) * TK + tid] = rsc;

  floatx16 acc[2][2];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

  SPCFG_TN_DMA(0, (int64_t)k0 * TK)
  SPCFG_TN_STORE_SC(0)
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  const int fcol = lane & 31, fk = lane >> 5;
  if constexpr (X3) {
  // One 32x32x16 instruction takes 8 reduction rows per lane: rows 16 c + 8 (lane / 32) .. + 7 of chunk c of
  // the step, read as 4-byte LDS words (the tile lies [row][column]).  The span scale (a power of two) goes
  // into the A values before they are cut into bf16 pieces.
#define SPCFG_TN_RAW(P, AS, BS, SS, C)                                          \
  {                                                                             \
    const int kb_ = 16 * (C) + 8 * fk;                                          \
    P##s0 = *reinterpret_cast<const float4*>((SS) + kb_);                       \
    P##s1 = *reinterpret_cast<const float4*>((SS) + kb_ + 4);                   \
    _Pragma("unroll") for (int j = 0; j < 8; ++j) {                             \
      P##a0[j] = (AS)[(kb_ + j) * TM];                                          \
      P##a1[j] = (AS)[(kb_ + j) * TM + 32];                                     \
      P##b0[j] = (BS)[(kb_ + j) * TN];                                          \
      P##b1[j] = (BS)[(kb_ + j) * TN + 32];                                     \
    }                                                                           \
  }
#define SPCFG_TN_T(X, Y)                                                                             \
    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A0.X(), B0.Y(), acc[0][0], 0, 0, 0);           \
    acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A0.X(), B1.Y(), acc[0][1], 0, 0, 0);           \
    acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A1.X(), B0.Y(), acc[1][0], 0, 0, 0);           \
    acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A1.X(), B1.Y(), acc[1][1], 0, 0, 0);
#define SPCFG_TN_GROUP(P)                                                                            \
  {                                                                                                  \
    nt::Split3 A0, A1, B0, B1;                                                                       \
    A0.cut(float4{P##a0[0] * P##s0.x, P##a0[1] * P##s0.y, P##a0[2] * P##s0.z, P##a0[3] * P##s0.w},   \
           float4{P##a0[4] * P##s1.x, P##a0[5] * P##s1.y, P##a0[6] * P##s1.z, P##a0[7] * P##s1.w});  \
    A1.cut(float4{P##a1[0] * P##s0.x, P##a1[1] * P##s0.y, P##a1[2] * P##s0.z, P##a1[3] * P##s0.w},   \
           float4{P##a1[4] * P##s1.x, P##a1[5] * P##s1.y, P##a1[6] * P##s1.z, P##a1[7] * P##s1.w});  \
    B0.cut(float4{P##b0[0], P##b0[1], P##b0[2], P##b0[3]}, float4{P##b0[4], P##b0[5], P##b0[6], P##b0[7]}); \
    B1.cut(float4{P##b1[0], P##b1[1], P##b1[2], P##b1[3]}, float4{P##b1[4], P##b1[5], P##b1[6], P##b1[7]}); \
    SPCFG_TN_T(l, h) SPCFG_TN_T(h, l) SPCFG_TN_T(m, m) SPCFG_TN_T(m, h) SPCFG_TN_T(h, m) SPCFG_TN_T(h, h) \
  }
  floatx8 xa0, xa1, xb0, xb1, ya0, ya1, yb0, yb1;
  float4 xs0, xs1, ys0, ys1;
  {
    const float* as = lds + wm * 64 + fcol;
    const float* bs = lds + TM * TK + wn * 64 + fcol;
    const float* ss = lds + (TM + TN) * TK;
    SPCFG_TN_RAW(x, as, bs, ss, 0)
  }
  for (int kt = k0; kt < k1; ++kt) {
    const int buf = (kt - k0) & 1;
    const int64_t sn = (int64_t)(kt + 1 < k1 ? kt + 1 : kt) * TK;  // the last step re-reads itself (never used)
    SPCFG_TN_DMA(buf ^ 1, sn)  // the other stage: everybody left it at the last barrier
    __builtin_amdgcn_sched_barrier(0);  // keep the loads at the top of the step
    const float* as = lds + buf * kStageT + wm * 64 + fcol;
    const float* bs = lds + buf * kStageT + TM * TK + wn * 64 + fcol;
    const float* ss = lds + buf * kStageT + (TM + TN) * TK;
    SPCFG_TN_RAW(y, as, bs, ss, 1)
    SPCFG_TN_GROUP(x)
    __builtin_amdgcn_sched_barrier(0);
    SPCFG_TN_STORE_SC(buf ^ 1)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // my part of the next tile has landed in LDS
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    {
      const float* as2 = lds + (buf ^ 1) * kStageT + wm * 64 + fcol;
      const float* bs2 = lds + (buf ^ 1) * kStageT + TM * TK + wn * 64 + fcol;
      const float* ss2 = lds + (buf ^ 1) * kStageT + (TM + TN) * TK;
      SPCFG_TN_RAW(x, as2, bs2, ss2, 0)
    }
    __builtin_amdgcn_sched_barrier(0);
    SPCFG_TN_GROUP(y)
  }
#undef SPCFG_TN_RAW
#undef SPCFG_TN_T
#undef SPCFG_TN_GROUP
  } else {
  // operands of one K pair: named scalars, double-buffered by hand so that the LDS reads of pair kk+2 are in
  // flight while the MFMAs of pair kk execute
  // (the span scale is multiplied in when the pair is used, not when it is fetched: a use right behind
  // the LDS read would wait for it)
#define SPCFG_TN_FRAGS(P, AS, BS, SS, KK)                                  \
  {                                                                        \
    const int k_ = (KK) + fk;                                              \
    P##s = (SS)[k_];                                                       \
    P##a0 = (AS)[k_ * TM];                                                 \
    P##a1 = (AS)[k_ * TM + 32];                                            \
    P##b0 = (BS)[k_ * TN];                                                 \
    P##b1 = (BS)[k_ * TN + 32];                                            \
  }
#define SPCFG_TN_MFMA(P)                                                                          \
  {                                                                                               \
    const float a0_ = P##a0 * P##s, a1_ = P##a1 * P##s;                                           \
    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0_, P##b0, acc[0][0], 0, 0, 0);             \
    acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0_, P##b1, acc[0][1], 0, 0, 0);             \
    acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1_, P##b0, acc[1][0], 0, 0, 0);             \
    acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1_, P##b1, acc[1][1], 0, 0, 0);             \
  }
  float xa0, xa1, xb0, xb1, xs, ya0, ya1, yb0, yb1, ys;
  {
    const float* as = lds + wm * 64 + fcol;
    const float* bs = lds + TM * TK + wn * 64 + fcol;
    const float* ss = lds + (TM + TN) * TK;
    SPCFG_TN_FRAGS(x, as, bs, ss, 0)
  }
  for (int kt = k0; kt < k1; ++kt) {
    const int buf = (kt - k0) & 1;
    const int64_t sn = (int64_t)(kt + 1 < k1 ? kt + 1 : kt) * TK;  // the last step re-reads itself (never used)
    SPCFG_TN_DMA(buf ^ 1, sn)  // the other stage: everybody left it at the last barrier
    __builtin_amdgcn_sched_barrier(0);  // keep the loads at the top of the step
    const float* as = lds + buf * kStageT + wm * 64 + fcol;
    const float* bs = lds + buf * kStageT + TM * TK + wn * 64 + fcol;
    const float* ss = lds + buf * kStageT + (TM + TN) * TK;
    // pairs 0..29 in two-pair stages: x holds pair kk, y pair kk+2
#pragma unroll
    for (int kk = 0; kk < TK - 4; kk += 4) {
      SPCFG_TN_FRAGS(y, as, bs, ss, kk + 2)
      SPCFG_TN_MFMA(x)
      __builtin_amdgcn_sched_barrier(0);
      SPCFG_TN_FRAGS(x, as, bs, ss, kk + 4)
      SPCFG_TN_MFMA(y)
      __builtin_amdgcn_sched_barrier(0);
      if (kk == 20) {  // the next step's scales, behind three quarters of the MFMA work
        SPCFG_TN_STORE_SC(buf ^ 1)
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // here x holds pair TK-4; fetch the last pair, then the barrier, then the next step's first pair, and only
    // then the last MFMAs: the LDS latency behind the barrier hides under them
    SPCFG_TN_FRAGS(y, as, bs, ss, TK - 2)
    SPCFG_TN_MFMA(x)
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // my part of the next tile has landed in LDS
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    {
      const float* as2 = lds + (buf ^ 1) * kStageT + wm * 64 + fcol;
      const float* bs2 = lds + (buf ^ 1) * kStageT + TM * TK + wn * 64 + fcol;
      const float* ss2 = lds + (buf ^ 1) * kStageT + (TM + TN) * TK;
      SPCFG_TN_FRAGS(x, as2, bs2, ss2, 0)
    }
    __builtin_amdgcn_sched_barrier(0);
    SPCFG_TN_MFMA(y)
  }
  }
  __syncthreads();  // all operands fetched before the LDS tiles are reused by the next tile segment
#undef SPCFG_TN_FRAGS
#undef SPCFG_TN_MFMA
#undef SPCFG_TN_DMA
#undef SPCFG_TN_DMA1
#undef SPCFG_TN_STORE_SC

  nt::finish_tile<128>(g.partial, g.counters, acc, tile, tile * KT, k0, k1, KTg, ipw, wg, it, wg_begin, tid, &s_last,
                       [&](floatx16(&t)[2][2]) {
    // accumulator layout of a 32x32 tile: column = lane % 32, row = 8*(v/4) + 4*(lane/32) + v%4
#pragma unroll
    for (int mi = 0; mi < 2; ++mi) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int ar = a0 + wm * 64 + mi * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        const int half = ar >= g.Np;
        const int arow = ar - half * g.Np;
        if (arow >= g.N) continue;
        float* dst = (half ? gR : gL) + (int64_t)arow * g.ldg + g.col0;
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
          const int c = b0 + wn * 64 + ni * 32 + (lane & 31);
          if (c >= g.cols) continue;
          const float val = t[mi][ni][v];
          dst[c] = g.accumulate ? dst[c] + val : val;
        }
      }
    }
  });
  it += advance;
  }  // share loop
}

}  // namespace

void launch_gemm_tn(const TnArgs& a, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    const void* kernels[6] = {
        reinterpret_cast<const void*>(&k_gemm_tn<0, false>), reinterpret_cast<const void*>(&k_gemm_tn<1, false>),
        reinterpret_cast<const void*>(&k_gemm_tn<2, false>), reinterpret_cast<const void*>(&k_gemm_tn<0, true>),
        reinterpret_cast<const void*>(&k_gemm_tn<1, true>),  reinterpret_cast<const void*>(&k_gemm_tn<2, true>)};
    for (const void* k : kernels)
      (void)hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytesT);
    attr_set = true;
  }
  const int tiles = ((2 * a.Np) / TM) * ((a.cols + TN - 1) / TN);
  if (a.grp_mode) {
    // one workgroup per (sentence, output tile); the hardware scheduler balances sentences of different length
    if (a.ngroups <= 0 || a.grp_kt_max <= 0) return;
    const int64_t tiles_total = (int64_t)a.ngroups * tiles;
    const int64_t total64 = tiles_total * a.grp_kt_max;
    if (total64 >= ((int64_t)1 << 31)) return;  // guarded by the row-count limit of the layout
    auto kernel = a.grp_mode == 1 ? (a.fp32_mfma ? k_gemm_tn<1, false> : k_gemm_tn<1, true>)
                                  : (a.fp32_mfma ? k_gemm_tn<2, false> : k_gemm_tn<2, true>);
    launch_k(kernel, dim3((unsigned)tiles_total), dim3(256), kLdsBytesT, st, a, a.grp_kt_max, (int)total64);
    return;
  }
  if (a.S <= 0) return;
  if (tiles > a.n_counters) { launch_refused("rule-gradient product: more output tiles than arrival counters"); return; }
  const int KT = (int)((a.S + TK - 1) / TK);
  const int64_t total64 = (int64_t)tiles * KT;
  if (total64 >= ((int64_t)1 << 31)) return;  // guarded by the row-count limit of the layout
  const int total = (int)total64;
  int Gn = a.max_wgs < 512 ? a.max_wgs : 512;
  if (Gn > total / 2) Gn = total / 2 > 0 ? total / 2 : 1;
  int ipw = (total + Gn - 1) / Gn;
  Gn = (total + ipw - 1) / ipw;
  launch_k(a.fp32_mfma ? k_gemm_tn<0, false> : k_gemm_tn<0, true>, dim3(Gn), dim3(256), kLdsBytesT, st, a, ipw, total);
}

}  // namespace spcfg
