// fp32 MFMA GEMM for the stacked projections (Sec. 3.2: [eta | zeta] = [L;R] * beta for all spans of one
// width at once) and for their reverse:  C[r][c] = sum_k A[r][k] * Bm[c][k], both operands K-contiguous.
//
// gfx950 mapping: 128x128x32 tile per 256-thread workgroup (4 wavefronts, 2x2, 64x64 each = 2x2 tiles of
// v_mfma_f32_32x32x2_f32).  Global -> registers -> LDS with two LDS stages and one barrier per K-step.
// Each lane fetches its MFMA operands as one 16-byte LDS read covering four K values; the K order inside
// an 8-wide chunk is permuted identically for both operands (lanes 0-31 take k0..k0+3, lanes 32-63
// k0+4..k0+7), which leaves the sum over K unchanged.
//
// The number of span rows shrinks with the width (from thousands to a handful), so a tile-per-workgroup
// launch would leave most of the 256 CUs idle for most widths.  Instead the (tile, K-step) iteration space is
// cut into equal contiguous shares, one per workgroup.  A workgroup whose share covers only part of a
// tile's K range writes its partial accumulators to a scratch slot and bumps the tile's arrival counter;
// whichever workgroup arrives last sums the slots in fixed order (so the result does not depend on the
// arrival order) and runs the epilogue.  Nobody waits on anybody: there is no spinning.
#include "spcfg_internal.h"
#ifdef SPCFG_TUNING
#include <cstdlib>
#endif

namespace spcfg {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Partial tiles travel between workgroups (possibly on different XCDs, whose L2 caches are not coherent
// with each other) as relaxed agent-scope atomic 8-byte accesses: stores write through, loads read the
// coherent copy, and neither needs a cache write-back or invalidate.
struct F2 { float a, b; };
__device__ __forceinline__ void st_agent(float* p, float a, float b) {
  const F2 v{a, b};
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), __builtin_bit_cast(unsigned long long, v),
                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ F2 ld_agent(const float* p) {
  return __builtin_bit_cast(F2, __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED,
                                                  __HIP_MEMORY_SCOPE_AGENT));
}

constexpr int BN = 128, BK = 32;
constexpr int LDT = BK + 4;  // LDS row stride in floats: 16-byte aligned rows, conflict-free 16-byte reads

// Tile geometry for a row-tile height BM (spans per tile).  Widths with few spans use shorter tiles so that
// the matrix cores do not multiply padding rows.
template <int BM> struct Geo {
  static constexpr int WM = BM == 32 ? 1 : 2;            // wavefronts along rows
  static constexpr int WN = 4 / WM;                      // wavefronts along columns
  static constexpr int MI = BM / (32 * WM);              // 32x32 MFMA tiles per wavefront along rows
  static constexpr int NI = BN / (32 * WN);              // ... along columns
  static constexpr int QA = BM / 32;                     // float4 of A staged per thread and K-step
  static constexpr int kStage = (BM + BN) * LDT;
  static constexpr size_t kLdsBytes = 2 * kStage * sizeof(float);
  static constexpr int kSlotFloats = BM * BN;
};

template <int EPI, int BM>
__device__ __forceinline__ void epilogue(const NtArgs& g, floatx16 (&acc)[Geo<BM>::MI][Geo<BM>::NI], int row0, int col0,
                                         int wm, int wn, int lane) {
  using G = Geo<BM>;
  // accumulator layout of a 32x32 tile: column = lane % 32, row = 8*(v/4) + 4*(lane/32) + v%4
#pragma unroll
  for (int mi = 0; mi < G::MI; ++mi) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int r = row0 + (wm * G::MI + mi) * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      if (r >= g.rows) continue;
      float scale = 1.0f;
      int64_t drow = r;
      if (EPI == NT_EPI_MASKROWS) {
        if (g.rowmask[r]) continue;
      }
      if (EPI == NT_EPI_ROWSCALE || EPI == NT_EPI_MASKROWS) {
        // normalising shift of the input row: brings its largest magnitude into [0.5, 1)
        const uint32_t mb = g.rowmaxb[r];
        const int f = max((int)((mb >> 23) & 0xffu) - 126, -126);
        scale = mb == 0u ? 0.0f : ldexpf(1.0f, -f);
      }
      if (EPI == NT_EPI_LEAF_EMIT) {
        const int q = g.rowexp[r];
        scale = (q == kExpZero || q < -160) ? 0.0f : ldexpf(1.0f, min(q, 127));
        drow = (int64_t)g.row_b[r] * g.n_max + g.row_i[r];
      }
#pragma unroll
      for (int ni = 0; ni < G::NI; ++ni) {
        const int c = col0 + (wn * G::NI + ni) * 32 + (lane & 31);
        if (c >= g.cols) continue;
        float val = acc[mi][ni][v] * scale;
        if (EPI == NT_EPI_LEAF_EMIT) val *= g.E[(int64_t)r * g.lde + c];
        g.C[drow * g.ldc + c] = val;
      }
    }
  }
}

template <int EPI, int BM>
__global__ void __launch_bounds__(256, 2) k_gemm_nt(NtArgs g, int ipw, int total_iters) {
  using G = Geo<BM>;
  extern __shared__ __align__(16) float lds[];
  __shared__ int s_last;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave % G::WM, wn = wave / G::WM;
  const int tiles_m = (g.rows + BM - 1) / BM;
  const int KT = g.K / BK;
  const int lc4 = tid & 7, lr = tid >> 3;  // staging: 8 float4 per tile row, 32 rows per pass
  const int lds_st = lr * LDT + lc4 * 4;
  const int frag_row = lane & 31, frag_k = (lane >> 5) * 4;
  const int a_off = (wm * G::MI * 32 + frag_row) * LDT + frag_k;
  const int b_off = BM * LDT + (wn * G::NI * 32 + frag_row) * LDT + frag_k;

  // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Renumber them so that every XCD
  // owns one contiguous run of shares, i.e. a contiguous run of tiles: the [L;R] panels it streams are then
  // (nearly) disjoint from those of the other XCDs instead of every L2 fetching all of them.
  const int nwg = gridDim.x, xcd = blockIdx.x & 7, qx = nwg >> 3, rx = nwg & 7;
  const int wg = xcd * qx + min(xcd, rx) + (blockIdx.x >> 3);
  const int wg_begin = wg * ipw;
  const int wg_end = min(wg_begin + ipw, total_iters);
  int it = wg_begin;
  while (it < wg_end) {
    const int tile = it / KT;
    const int k0 = it - tile * KT;
    const int k1 = min(KT, k0 + (wg_end - it));
    const int tile_m = tile % tiles_m, tile_n = tile / tiles_m;
    const int row0 = tile_m * BM, col0 = tile_n * BN;

    const float* ga[G::QA];
    const float* gb[4];
#pragma unroll
    for (int q = 0; q < G::QA; ++q)
      ga[q] = g.A + (int64_t)min(row0 + lr + 32 * q, g.rows - 1) * g.lda + lc4 * 4;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      gb[q] = g.Bm + (int64_t)min(col0 + lr + 32 * q, g.cols - 1) * g.ldb + lc4 * 4;
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
    SPCFG_LOAD_TILE(k0 * BK)
    SPCFG_STORE_TILE(lds + lds_st)
    __syncthreads();

    for (int kt = k0; kt < k1; ++kt) {
      const int buf = (kt - k0) & 1;
      // prefetch the next K-step into registers (the last iteration re-reads its own step)
      const int kn = min(kt + 1, k1 - 1) * BK;
      SPCFG_LOAD_TILE(kn)
      // Pin the schedule: the compiler otherwise sinks the prefetch loads down to their LDS stores and exposes
      // the full memory latency in every K-step.  Order: loads first, three quarters of the MFMA work, then the
      // LDS stores of the prefetched tile (by then the loads have landed), then the last quarter, then the barrier.
      __builtin_amdgcn_sched_barrier(0);
      const float* as = lds + buf * G::kStage + a_off;
      const float* bs = lds + buf * G::kStage + b_off;
#define SPCFG_MFMA_STEP(C)                                                                             \
  _Pragma("unroll") for (int mi = 0; mi < G::MI; ++mi) _Pragma("unroll") for (int ni = 0; ni < G::NI; ++ni) \
      acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mi].C, b[ni].C, acc[mi][ni], 0, 0, 0);
#define SPCFG_FRAGS(KC)                                                                                     \
  _Pragma("unroll") for (int mi = 0; mi < G::MI; ++mi) a[mi] =                                              \
      *reinterpret_cast<const float4*>(as + mi * 32 * LDT + (KC)*8);                                        \
  _Pragma("unroll") for (int ni = 0; ni < G::NI; ++ni) b[ni] =                                              \
      *reinterpret_cast<const float4*>(bs + ni * 32 * LDT + (KC)*8);
#define SPCFG_KCHUNK(KC)                                                                                    \
  {                                                                                                         \
    float4 a[G::MI], b[G::NI];                                                                              \
    SPCFG_FRAGS(KC)                                                                                         \
    SPCFG_MFMA_STEP(x) SPCFG_MFMA_STEP(y) SPCFG_MFMA_STEP(z) SPCFG_MFMA_STEP(w)                             \
  }
      SPCFG_KCHUNK(0)
      SPCFG_KCHUNK(1)
      SPCFG_KCHUNK(2)
      {
        float4 a[G::MI], b[G::NI];
        SPCFG_FRAGS(3)  // fetched before the LDS stores below so that their latency hides behind chunk 2
        __builtin_amdgcn_sched_barrier(0);
        SPCFG_STORE_TILE(lds + (buf ^ 1) * G::kStage + lds_st)
        __builtin_amdgcn_sched_barrier(0);
        SPCFG_MFMA_STEP(x) SPCFG_MFMA_STEP(y) SPCFG_MFMA_STEP(z) SPCFG_MFMA_STEP(w)
      }
#undef SPCFG_FRAGS
#undef SPCFG_KCHUNK
#undef SPCFG_MFMA_STEP
      __builtin_amdgcn_sched_barrier(0);
      __syncthreads();
    }

    if (k0 == 0 && k1 == KT) {
      epilogue<EPI, BM>(g, acc, row0, col0, wm, wn, lane);
    } else {
      // partial tile: publish, count arrivals, last arriver reduces in fixed order
      const int first_g = (tile * KT) / ipw;
      const int last_g = (tile * KT + KT - 1) / ipw;
      const int parts = last_g - first_g + 1;
      float* slot = g.partial + (size_t)(2 * wg + (it != wg_begin ? 1 : 0)) * G::kSlotFloats;
#pragma unroll
      for (int mi = 0; mi < G::MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < G::NI; ++ni)
#pragma unroll
          for (int j = 0; j < 8; ++j)
            st_agent(slot + (((mi * G::NI + ni) * 8 + j) * 256 + tid) * 2, acc[mi][ni][2 * j], acc[mi][ni][2 * j + 1]);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // my stores have landed before the arrival is counted
      __syncthreads();
      if (tid == 0)
        s_last = (__hip_atomic_fetch_add(&g.counters[tile], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                  parts - 1) ? 1 : 0;
      __syncthreads();
      if (s_last) {
        // one 32x32 accumulator tile at a time (8 loads in flight per lane), parts in ascending order
        const int odd0 = (tile * KT != first_g * ipw) ? 1 : 0;
#pragma unroll
        for (int mi = 0; mi < G::MI; ++mi)
#pragma unroll
          for (int ni = 0; ni < G::NI; ++ni) {
            floatx16 sum;
#pragma unroll
            for (int v = 0; v < 16; ++v) sum[v] = 0.0f;
            const size_t off = (size_t)((mi * G::NI + ni) * 8 * 256 + tid) * 2;
            for (int p0 = 0; p0 < parts; p0 += 4) {  // four parts (32 loads per lane) in flight
              F2 x[4][8];
#pragma unroll
              for (int u = 0; u < 4; ++u) {
                const int p = min(p0 + u, parts - 1);
                const float* src = g.partial + (size_t)(2 * (first_g + p) + (p == 0 ? odd0 : 0)) * G::kSlotFloats + off;
#pragma unroll
                for (int j = 0; j < 8; ++j) x[u][j] = ld_agent(src + j * 512);
              }
#pragma unroll
              for (int u = 0; u < 4; ++u) {
                const float keep = (p0 + u < parts) ? 1.0f : 0.0f;  // the clamped duplicate of the last part adds nothing
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                  sum[2 * j] += keep * x[u][j].a;
                  sum[2 * j + 1] += keep * x[u][j].b;
                }
              }
            }
            acc[mi][ni] = sum;
          }
        epilogue<EPI, BM>(g, acc, row0, col0, wm, wn, lane);
        if (tid == 0)  // ready for the next launch on this stream
          __hip_atomic_store(&g.counters[tile], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    it += k1 - k0;
  }
}

// Tile height and workgroup count per launch, from a sweep on MI355X (256 CUs): what matters is the amount
// of work relative to the machine, so the thresholds are in multiply-accumulates (rows * cols * K).  Small
// launches want short tiles (finer shares, less padding) and one workgroup per CU; large ones tall tiles
// (less LDS and L2 traffic per flop) and two workgroups per CU.
int pick_bm(int rows, int cols, int K) {
  const double work = (double)rows * cols * K;
  if (rows <= 32 || work <= 2.7e9) return 32;
  if (rows <= 64 || work <= 7.6e9) return 64;
  return 128;
}
int pick_wgs(int rows, int cols, int K) { return (double)rows * cols * K <= 1.25e9 ? 256 : 512; }

template <int EPI, int BM>
void launch(const NtArgs& a, hipStream_t st) {
  using G = Geo<BM>;
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_nt<EPI, BM>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)G::kLdsBytes);
    attr_set = true;
  }
  const int tiles = ((a.rows + BM - 1) / BM) * ((a.cols + BN - 1) / BN);
  const int KT = a.K / BK;
  const int total = tiles * KT;
  int Gn = pick_wgs(a.rows, a.cols, a.K);
  if (Gn > a.max_wgs) Gn = a.max_wgs;
  if (Gn > total / 2) Gn = total / 2 > 0 ? total / 2 : 1;  // at least two K-steps per share
#ifdef SPCFG_TUNING
  if (getenv("SPCFG_NT_G")) Gn = atoi(getenv("SPCFG_NT_G"));
  if (Gn > total) Gn = total;
#endif
  int ipw = (total + Gn - 1) / Gn;
  Gn = (total + ipw - 1) / ipw;
  hipLaunchKernelGGL((k_gemm_nt<EPI, BM>), dim3(Gn), dim3(256), G::kLdsBytes, st, a, ipw, total);
}

template <int EPI>
void launch_bm(const NtArgs& a, hipStream_t st) {
  int bm = pick_bm(a.rows, a.cols, a.K);
#ifdef SPCFG_TUNING
  if (getenv("SPCFG_NT_BM")) bm = atoi(getenv("SPCFG_NT_BM"));
#endif
  switch (bm) {
    case 32: launch<EPI, 32>(a, st); break;
    case 64: launch<EPI, 64>(a, st); break;
    default: launch<EPI, 128>(a, st); break;
  }
}

}  // namespace

// number of arrival counters a launch can need (upper bound over the tile heights used)
int gemm_nt_tiles(int rows, int cols) { return ((rows + 31) / 32) * ((cols + BN - 1) / BN); }
size_t gemm_nt_partial_bytes(int max_wgs) { return (size_t)2 * max_wgs * Geo<128>::kSlotFloats * sizeof(float); }

void launch_gemm_nt(const NtArgs& a, hipStream_t st) {
  if (a.rows <= 0 || a.cols <= 0) return;
  switch (a.epilogue) {
    case NT_EPI_ROWSCALE: launch_bm<NT_EPI_ROWSCALE>(a, st); break;
    case NT_EPI_MASKROWS: launch_bm<NT_EPI_MASKROWS>(a, st); break;
    default: launch_bm<NT_EPI_LEAF_EMIT>(a, st); break;
  }
}

}  // namespace spcfg
