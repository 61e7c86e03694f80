// Shared pieces of the NT projection GEMMs (fp32 and bf16 operand variants): tile geometry, epilogues,
// and the work sharing across workgroups.
//
// The number of span rows shrinks with the width (from thousands to a handful), so a tile-per-workgroup
// launch would leave most of the 256 CUs idle for most widths.  Instead the (tile, K-step) iteration space is
// cut into equal contiguous shares, one per workgroup.  A workgroup whose share covers only part of a
// tile's K range writes its partial accumulators to a scratch slot and bumps the tile's arrival counter;
// whichever workgroup arrives last sums the slots in fixed order (so the result does not depend on the
// arrival order) and runs the epilogue.  Nobody waits on anybody: there is no spinning.
#pragma once
#include "spcfg_internal.h"

namespace spcfg {
namespace nt {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

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

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
// fp32 products from bf16 matrix instructions (the bf16 rate of the matrix cores is 16 times the fp32 rate):
// every operand x is cut into three bf16 pieces, hi = bf16(x), mid = bf16(x - hi), lo = x - hi - mid (both
// conversions round to nearest; the differences are exact and lo has at most 8 significant bits left), so
// hi + mid + lo is x exactly, and the six largest of the nine piece products are accumulated in fp32
// (hi*hi, hi*mid, mid*hi, mid*mid, hi*lo, lo*hi).  With |mid| <= 2^-8 |x| and |lo| <= 2^-16 |x| the three dropped
// products are below 2^-23 |x y|, the size of an fp32 rounding error, and have either sign.  Measured against the
// fp64 result of a whole forward-backward pass this is as accurate as the fp32 matrix instructions; cutting
// by truncation instead (two cheaper operations per value) biases every product downwards and was 13 times less
// accurate on the gradients.  Pieces of 8 values are packed as one MFMA operand.
struct Split3 {
  uintx4 hi, mid, lo;
  __device__ __forceinline__ static unsigned pack_rne(float x0, float x1) {
    typedef float floatx2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(unsigned, __builtin_convertvector(floatx2{x0, x1}, bf16x2));  // v_cvt_pk_bf16_f32
  }
  __device__ __forceinline__ static void cut2(float x0, float x1, unsigned& h, unsigned& m, unsigned& l) {
    h = pack_rne(x0, x1);
    const float r0 = x0 - __uint_as_float(h << 16), r1 = x1 - __uint_as_float(h & 0xffff0000u);
    m = pack_rne(r0, r1);
    const float s0 = r0 - __uint_as_float(m << 16), s1 = r1 - __uint_as_float(m & 0xffff0000u);
    l = __builtin_amdgcn_perm(__float_as_uint(s1), __float_as_uint(s0), 0x07060302u);  // upper halves; exact
  }
  __device__ __forceinline__ void cut(const float4& u, const float4& v) {
    unsigned h0, h1, h2, h3, m0, m1, m2, m3, l0, l1, l2, l3;
    cut2(u.x, u.y, h0, m0, l0);
    cut2(u.z, u.w, h1, m1, l1);
    cut2(v.x, v.y, h2, m2, l2);
    cut2(v.z, v.w, h3, m3, l3);
    hi = uintx4{h0, h1, h2, h3};
    mid = uintx4{m0, m1, m2, m3};
    lo = uintx4{l0, l1, l2, l3};
  }
  __device__ __forceinline__ bf16x8 h() const { return __builtin_bit_cast(bf16x8, hi); }
  __device__ __forceinline__ bf16x8 m() const { return __builtin_bit_cast(bf16x8, mid); }
  __device__ __forceinline__ bf16x8 l() const { return __builtin_bit_cast(bf16x8, lo); }
};


constexpr int BN = 128;
// One K-step is 128 bytes of every tile row (32 fp32 or 64 bf16 values); LDS rows are 144 bytes apart
// (16-byte aligned, and 16-byte reads of 8 consecutive rows touch all banks once).
constexpr int LDT = 36;  // LDS row stride in 4-byte words

// Tile geometry for a row-tile height BM (spans per tile).  Widths with few spans use shorter tiles so that
// the matrix cores do not multiply padding rows.
template <int BM> struct Geo {
  static constexpr int WM = BM == 32 ? 1 : 2;            // wavefronts along rows
  static constexpr int WN = 4 / WM;                      // wavefronts along columns
  static constexpr int MI = BM / (32 * WM);              // 32x32 MFMA tiles per wavefront along rows
  static constexpr int NI = BN / (32 * WN);              // ... along columns
  static constexpr int QA = BM / 32;                     // 16-byte chunks of A staged per thread and K-step
  static constexpr int kStage = (BM + BN) * LDT;         // words per LDS stage
  static constexpr size_t kLdsBytes = 2 * kStage * sizeof(float);
  static constexpr int kSlotFloats = BM * BN;
};

template <int EPI, int BM>
__device__ __forceinline__ void epilogue(const NtArgs& g, floatx16 (&acc)[Geo<BM>::MI][Geo<BM>::NI], int row0, int col0,
                                         int wm, int wn, int lane, int row_end, int c_shift = 0) {
  using G = Geo<BM>;
  // accumulator layout of a 32x32 tile: column = lane % 32, row = 8*(v/4) + 4*(lane/32) + v%4
#pragma unroll
  for (int mi = 0; mi < G::MI; ++mi) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int r = row0 + (wm * G::MI + mi) * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      if (r >= row_end) continue;
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
      if (EPI == NT_EPI_GRAD) {  // rows are the stacked parents [L;R]: scatter into grad_L / grad_R
        const int half = r >= g.Np ? 1 : 0;
        const int arow = r - half * g.Np;
        if (arow >= g.Nvalid) continue;
        float* dst = (half ? g.gR : g.gL) + (int64_t)arow * g.ldg + g.col0;
#pragma unroll
        for (int ni = 0; ni < G::NI; ++ni) {
          const int c = col0 + (wn * G::NI + ni) * 32 + (lane & 31);
          if (c >= g.cols) continue;
          dst[c] = g.accumulate ? dst[c] + acc[mi][ni][v] : acc[mi][ni][v];
        }
        continue;
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
        g.C[drow * g.ldc + c + c_shift] = val;  // c_shift: column block of this part of the launch
      }
    }
  }
}

// Share of the (tile, K-step) space of this workgroup.  Workgroups are dealt round-robin to the 8 XCDs (each
// with its own L2); they are renumbered so that every XCD owns one contiguous run of shares, i.e. a
// contiguous run of tiles: the [L;R] panels it streams are then (nearly) disjoint from those of the other
// XCDs instead of every L2 fetching all of them.
__device__ __forceinline__ int renumbered_wg() {
  const int nwg = gridDim.x, xcd = blockIdx.x & 7, qx = nwg >> 3, rx = nwg & 7;
  return xcd * qx + min(xcd, rx) + (blockIdx.x >> 3);
}

// Grouped mode (one grammar per sentence): table of the sentences' first row tile, first row and row count in
// LDS, built by every workgroup with one block scan over the lengths (four sentences per thread); returns
// the number of row tiles of the launch.  s_tile0 has ngroups + 1 entries.
template <int BM>
__device__ __forceinline__ int build_group_table(const NtArgs& g, int* s_tile0, int* s_row0, int* s_cnt, int* s_wsum,
                                                 int tid) {
  const int lane = tid & 63, wave = tid >> 6;
  int c[4], local = 0;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int b = 4 * tid + q;
    int cnt = 0;
    if (b < g.ngroups) {
      cnt = max(0, g.grp_lens[b] - g.grp_w + 1);
      s_cnt[b] = cnt;
      s_row0[b] = cnt > 0 ? (int)(g.grp_rowbase[b] - g.grp_row_first) : 0;
    }
    c[q] = (cnt + BM - 1) / BM;
    local += c[q];
  }
  int x = local;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int y = __shfl_up(x, o, 64);
    if (lane >= o) x += y;
  }
  if (lane == 63) s_wsum[wave] = x;
  __syncthreads();
  int base = 0;
  for (int i = 0; i < wave; ++i) base += s_wsum[i];
  int excl = base + x - local;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int b = 4 * tid + q;
    if (b < g.ngroups) s_tile0[b] = excl;
    excl += c[q];
  }
  const int tiles_m = s_wsum[0] + s_wsum[1] + s_wsum[2] + s_wsum[3];
  if (tid == 0) s_tile0[g.ngroups] = tiles_m;
  __syncthreads();
  return tiles_m;
}
// The sentence whose row tiles contain tile_m (s_tile0[b] <= tile_m < s_tile0[b + 1]); sets the tile's first row
// and the end of the sentence's rows.
template <int BM>
__device__ __forceinline__ int find_group(const NtArgs& g, const int* s_tile0, const int* s_row0, const int* s_cnt,
                                          int tile_m, int* row0, int* row_end) {
  int lo = 0, hi = g.ngroups;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (s_tile0[mid] <= tile_m) lo = mid; else hi = mid;
  }
  *row0 = s_row0[lo] + (tile_m - s_tile0[lo]) * BM;
  *row_end = s_row0[lo] + s_cnt[lo];
  return lo;
}

// After the K loop of one tile segment [k0, k1): run the epilogue if the segment is the whole tile, else
// publish the partial tile, count the arrival, and let the last arriver reduce in fixed order.
template <int BM, typename Epi>
__device__ __forceinline__ void finish_tile(float* partial, int32_t* counters, floatx16 (&acc)[Geo<BM>::MI][Geo<BM>::NI],
                                            int tile, int ustart, int k0, int k1, int KT, int ipw, int wg, int it,
                                            int wg_begin, int tid, int* s_last_ptr, Epi&& run_epilogue) {
  using G = Geo<BM>;
  int& s_last = *s_last_ptr;
  if (k0 == 0 && k1 == KT) {
    run_epilogue(acc);
  } else {
    // partial tile: publish, count arrivals, last arriver reduces in fixed order
    // ustart = index of the tile's first K-step in the launch's unit space; shares are ipw units long
    const int first_g = ustart / ipw;
    const int last_g = (ustart + KT - 1) / ipw;
    const int parts = last_g - first_g + 1;
    float* slot = partial + (size_t)(2 * wg + (it != wg_begin ? 1 : 0)) * G::kSlotFloats;
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
      s_last = (__hip_atomic_fetch_add(&counters[tile], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                parts - 1) ? 1 : 0;
    __syncthreads();
    if (s_last) {
      // one 32x32 accumulator tile at a time (8 loads in flight per lane), parts in ascending order
      const int odd0 = (ustart != first_g * ipw) ? 1 : 0;
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
              const float* src = partial + (size_t)(2 * (first_g + p) + (p == 0 ? odd0 : 0)) * G::kSlotFloats + off;
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
      run_epilogue(acc);
      if (tid == 0)  // ready for the next launch on this stream
        __hip_atomic_store(&counters[tile], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

// Tile height per launch, from a sweep on MI355X (256 CUs): what matters is the amount of work relative to the
// machine, so the thresholds are in multiply-accumulates (rows * cols * K).  Small launches want short tiles
// (finer shares, less padding), large ones tall tiles (less LDS and L2 traffic per flop).
inline double work_of(const NtArgs& a) {
  if (a.parts == 0) return (double)(a.grouped ? a.grp_max_rows : a.rows) * a.cols * a.K;
  double w = 0;
  for (int p = 0; p < a.parts; ++p) w += (double)a.prt_rows[p] * a.cols * a.prt_kt[p] * 32;
  return w;
}
// fp32 operands (split products): repeated sweeps at N = 2048 put the changes at 190 rows (32 -> 64 for both
// shapes) and at 380 rows (64 -> 128) for the forward shape (2N columns, K = N; 128 is 20 % faster at 500-900
// rows) resp. 520 rows for the reverse shape (N columns, K = 2N; equal from there on); at N = 1024 the short tile
// wins at every row count that occurs, which the same amounts of work reproduce.  bf16 operands keep the
// thresholds of their own sweep.
inline int pick_bm(int rows, double work, bool bf16, bool wide) {
  const double t64 = bf16 ? 2.7e9 : 1.6e9, t128 = bf16 ? 7.6e9 : (wide ? 3.2e9 : 4.3e9);
  if (rows <= 32 || work <= t64) return 32;
  if (rows <= 64 || work <= t128) return 64;
  return 128;
}
// Workgroups of a launch from its (tile, K-step) units (counted in steps of 32 K values): few units want few
// workgroups (every further share of a tile is one more partial tile for the reducing workgroup to read), many want
// two workgroups per CU.  Sweeps at N = 1024 and 2048, 4 to 150 rows, forward and reverse shapes: 128 workgroups are
// best below 1024 units, 256 below 4096, 512 above (each within 3 % of the best of the three everywhere).
inline int pick_wgs(int total_units, int bk_elems) {
  const int64_t u = (int64_t)total_units * bk_elems / 32;
  return u < 1024 ? 128 : (u < 4096 ? 256 : 512);
}


// Launch helper: splits total = tiles * KT K-steps into equal shares.
template <typename Kernel>
void launch_shared(Kernel kernel, const NtArgs& a, int BM, int BKelems, size_t lds_bytes, hipStream_t st) {
  const int tiles_m = a.grouped ? a.grp_tiles_m[BM == 32 ? 0 : (BM == 64 ? 1 : 2)] : (a.rows + BM - 1) / BM;
  int tiles = tiles_m * ((a.cols + BN - 1) / BN);
  const int KT = a.K / BKelems;
  int total = tiles * KT;
  if (a.parts > 0) {  // several products in one launch: each part has its own rows and K range
    tiles = 0; total = 0;
    for (int p = 0; p < a.parts; ++p) {
      const int tp = ((a.prt_rows[p] + BM - 1) / BM) * ((a.cols + BN - 1) / BN);
      tiles += tp;
      total += tp * a.prt_kt[p];
    }
    if (total == 0) return;
  }
  if (tiles > a.n_counters) { launch_refused("projection product: more output tiles than arrival counters"); return; }
  int Gn = pick_wgs(total, BKelems);
  const int cap = a.max_wgs * (128 / BM);  // the partial-tile scratch holds 2 * max_wgs slots of 128 x 128
  if (Gn > cap) Gn = cap;
  if (Gn > total / 2) Gn = total / 2 > 0 ? total / 2 : 1;  // at least two K-steps per share
  int ipw = (total + Gn - 1) / Gn;
  Gn = (total + ipw - 1) / ipw;
  launch_k(kernel, dim3(Gn), dim3(256), lds_bytes, st, a, ipw, total);
}

inline int chosen_bm(const NtArgs& a) {
  // wide = more columns than K (the forward projection; a two-part launch is one)
  int bm = pick_bm(a.grouped ? a.grp_max_rows : a.rows, work_of(a), a.a_bf16 != 0, a.parts == 2 || a.cols > a.K);
  return bm;
}

}  // namespace nt
}  // namespace spcfg
