// Projection GEMM on operands that arrive already cut into bf16 planes (Sec. 3.2: [eta | zeta] = [L;R] * beta
// for all spans of one width at once, and the reverse product):  C[r][c] = sum_k A[r][k] * Bm[c][k].
// Three planes (fp32 mode): A = Ah + Am + Al, Bm = Bh + Bm + Bl exactly (nt::Split3) and the six significant piece
// products accumulated in fp32.  Two planes (forward products of the bf16 mode): hi = bf16(x), lo = bf16(x - hi), products
// lo*hi, hi*lo, hi*hi: operands good to 2^-17 instead of 2^-9, which keeps log Z inside its bound on peaked grammars
// and long sentences, where single bf16 roundings add up over the hundreds of projections of a tree.
// The producers of the chart rows and the weight packing write the planes, so this kernel does no conversion work:
//
//  * tiles go straight from global memory into LDS (global_load_lds_dwordx4, 1 KB per wavefront instruction = 16 rows of
//    one plane and K-step), into a ring of NS stages; the loads of step t + NS - 1 are issued while step t is multiplied;
//  * LDS rows are 64 bytes (32 bf16) without padding; the 16-byte chunk index is XORed with bits 2..3 of the row, which
//    makes the 16-byte operand reads of 16 consecutive rows conflict-free (the loads apply the same permutation on the
//    global side, four lanes per row);
//  * one 256-thread workgroup per CU (the ring takes 120-150 KB of LDS), 4 wavefronts as in the other projection kernels;
//  * the instruction order of a K-step is written out: operand reads are inline assembly (so every wait is placed by
//    hand), matrix instructions, reads and loads alternate, and the one barrier per step sits behind the first matrix
//    instructions of the step's second half, so the matrix pipe has work while the wavefronts meet.
// Work sharing across workgroups, parts and epilogues are those of gemm_nt_common.h.
#include <type_traits>
#include <utility>

#include "gemm_nt_common.h"

namespace spcfg {

namespace {

using namespace nt;

constexpr int BK3 = 32;  // K values per step: one 64-byte row per plane

template <int BM, int NPL> struct Geo3 {
  using G = Geo<BM>;
  static constexpr int PTA = BM * 64, PTB = BN * 64;        // bytes of one plane tile of A / of Bm
  static constexpr int STAGE = NPL * (PTA + PTB);            // [A hi | A mid | A lo | B hi | B mid | B lo]
  static constexpr int NS = (BM == 128 ? 3 : (BM == 64 ? 4 : 5)) + (NPL == 2 ? 1 : 0);
  static constexpr int NDT = NPL * (BM / 16) + NPL * (BN / 16);  // 1 KB load instructions per stage
  static constexpr int ND = (NDT + 3) / 4;                   // per wavefront (the last ones repeat when uneven)
  static constexpr int NF = G::MI + G::NI;                   // operand fragments per plane and 16-wide chunk
  static constexpr int NR = NPL * NF;                        // operand reads per chunk
  static constexpr int NM = (NPL == 3 ? 6 : 3) * G::MI * G::NI;  // matrix instructions per chunk
  static constexpr int RPF = (NR + NM - 1) / NM;             // operand reads behind each of them in the first half
  static constexpr int NB = NM >= 12 ? 2 : 1;                // matrix instructions ahead of the barrier
  static constexpr size_t kLds = (size_t)NS * STAGE;
};

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

__device__ __forceinline__ void dma16(const void* gptr, unsigned lds_addr) {
#if defined(__HIP_DEVICE_COMPILE__)
  typedef __attribute__((address_space(3))) unsigned char lds_u8;
  __builtin_amdgcn_global_load_lds(gptr, (lds_u8*)(uintptr_t)lds_addr, 16, 0, 0);
#else
  (void)gptr; (void)lds_addr;
#endif
}
__device__ __forceinline__ unsigned lds_address(const void* p) {
#if defined(__HIP_DEVICE_COMPILE__)
  typedef __attribute__((address_space(3))) unsigned char lds_u8;
  return (unsigned)(uintptr_t)(lds_u8*)p;
#else
  (void)p; return 0;
#endif
}
__device__ __forceinline__ int swz(int row) { return (row >> 2) & 3; }

// Makes every register of F[NPL][NF] an in/out operand of an empty statement: instructions that use them stay behind it.
template <int NPL, int NF, int R = 0>
__device__ __forceinline__ void tie_registers(uintx4 (&F)[NPL][NF]) {
  if constexpr (R < NPL * NF) {
    asm volatile("" : "+v"(F[R / NF][R % NF]));
    tie_registers<NPL, NF, R + 1>(F);
  }
}

#define SPCFG_SB __builtin_amdgcn_sched_barrier(0);

// MODE 0: one product; 2: parts (see NtArgs).
template <int EPI, int BM, int MODE, int NPL>
__global__ void __launch_bounds__(256, 1) k_gemm_nt3(NtArgs g, int ipw, int total_iters, int mgroups) {
  constexpr bool PARTS = MODE == 2;
  using G = Geo<BM>;
  using Q = Geo3<BM, NPL>;
  constexpr int MI = G::MI, NI = G::NI, NS = Q::NS, ND = Q::ND, NF = Q::NF, NR = Q::NR, NM = Q::NM, NB = Q::NB;
  extern __shared__ __align__(16) unsigned char lds3[];
  __shared__ int s_last;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int uw = __builtin_amdgcn_readfirstlane(wave);
  const int wm = wave % G::WM, wn = wave / G::WM;
  const int tiles_m = (g.rows + BM - 1) / BM;
  const int KT = g.K / BK3;
  const unsigned lds0 = lds_address(lds3);
  // operand fragments: lane l holds row l % 32 and the 16-byte chunk l / 32 of the 32-byte K range of a chunk
  const int fr = lane & 31, fh = lane >> 5;
  const unsigned frag_sw = (unsigned)((fh ^ swz(fr)) * 16);
  // byte offsets inside a stage of chunk 0; chunk 1 flips bit 5 of the offset (the next two 16-byte pieces of the row)
  const unsigned a_rel = (wm * MI * 32 + fr) * 64 + frag_sw;
  const unsigned b_rel = NPL * Q::PTA + (wn * NI * 32 + fr) * 64 + frag_sw;
  const unsigned a_frag = lds0 + a_rel, b_frag = lds0 + b_rel;
  const unsigned a_frag1 = lds0 + (a_rel ^ 32u), b_frag1 = lds0 + (b_rel ^ 32u);
  // this wavefront's load instructions: entry e = uw + 4 j of the stage's list (A planes first, then Bm planes)
  int e_isA[ND], e_plane[ND], e_rg[ND];
  unsigned e_lds[ND];
#pragma unroll
  for (int j = 0; j < ND; ++j) {
    const int e = min(uw + 4 * j, Q::NDT - 1);
    const bool isA = e < NPL * (BM / 16);
    const int ee = isA ? e : e - NPL * (BM / 16);
    const int per = isA ? BM / 16 : BN / 16;
    e_isA[j] = isA; e_plane[j] = ee / per; e_rg[j] = ee % per;
    e_lds[j] = (isA ? e_plane[j] * Q::PTA : NPL * Q::PTA + e_plane[j] * Q::PTB) + e_rg[j] * 1024;
  }

  const int wg = renumbered_wg();
  const int wg_begin = wg * ipw;
  const int wg_end = min(wg_begin + ipw, total_iters);
  int it = wg_begin;
  while (it < wg_end) {
    int tile, ustart, KTt = KT, k0, tile_m, tile_n, row0, row_end = g.rows, c_shift = 0, kbeg = 0;
    if (PARTS) {
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
      // tile order: the row tiles in mgroups groups, one group after the other, inside a group row tile fastest: with
      // consecutive shares on one XCD, that XCD's concurrently running tiles form a block of (row tiles of a group) x
      // (a slice of the column tiles), whose operand rows its L2 fetches once
      const int rpg = (tiles_m + mgroups - 1) / mgroups, per = rpg * ((g.cols + BN - 1) / BN);
      const int gi = tile / per, rem = tile - gi * per, gm = min(rpg, tiles_m - gi * rpg);
      tile_m = gi * rpg + rem % gm; tile_n = rem / gm;
      row0 = tile_m * BM;
    }
    const int k1 = min(KTt, k0 + (wg_end - it));
    const int col0 = tile_n * BN;
    // The tile's K-steps are taken in rotated order: position p of the tile's K loop is K-step (p + krot) mod KTt, with
    // krot chosen so that the workgroup that owns the tile's first position is at K-step (its own step count) mod KTt.
    // Workgroups that run side by side on an XCD then read the same K range of the operand rows they share at the same
    // time, whatever the share size is, and that XCD's L2 fetches those rows once.  (Positions, not K-steps, are what
    // the shares and the partial tiles are made of; the order of the sum is still fixed by the launch geometry.)
    const int krot = (ustart % ipw) % KTt;
    const uint16_t* amat = static_cast<const uint16_t*>(g.A3) + (int64_t)kbeg * BK3;
    const uint16_t* bmat = static_cast<const uint16_t*>(g.Bm3) + (int64_t)c_shift * g.ldb + (int64_t)kbeg * BK3;
    // global address of this lane's 16 bytes of every load instruction at K-step 0: row rg * 16 + lane / 4 of the
    // plane tile (clamped into the operand: rows past the end are never stored), chunk (lane % 4) ^ swz(row)
    const unsigned char* gp[ND];
#pragma unroll
    for (int j = 0; j < ND; ++j) {
      const int r = e_rg[j] * 16 + (lane >> 2);
      const int c = (lane & 3) ^ swz(r);
      const uint16_t* base = e_isA[j]
          ? amat + (int64_t)e_plane[j] * g.a_plane + (int64_t)min(row0 + r, row_end - 1) * g.lda
          : bmat + (int64_t)e_plane[j] * g.b_plane + (int64_t)min(col0 + r, g.cols - 1) * g.ldb;
      gp[j] = reinterpret_cast<const unsigned char*>(base + c * 8);
    }

    floatx16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

    // operand registers of two chunks: [plane][fragment], fragments 0..MI-1 of A, MI..MI+NI-1 of Bm
    uintx4 X[NPL][NF], Y[NPL][NF];
    auto load_stage = [&](int stage, int kpos) {  // all of this wavefront's loads of one K-step
      const int kr = kpos + krot;
      const int64_t koff = (int64_t)(kr >= KTt ? kr - KTt : kr) * 64;
      static_for<0, ND>([&](auto j) { dma16(gp[j] + koff, lds0 + stage * Q::STAGE + e_lds[j]); });
    };
    auto read_one = [&](uintx4(&F)[NPL][NF], auto r, unsigned aa, unsigned ba) {
      constexpr int pl = decltype(r)::value / NF, f = decltype(r)::value % NF;
      if constexpr (f < MI) {
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(F[pl][f]) : "v"(aa), "n"(pl * Q::PTA + f * 2048));
      } else {
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(F[pl][f]) : "v"(ba), "n"(pl * Q::PTB + (f - MI) * 2048));
      }
    };
    auto mfma_one = [&](uintx4(&F)[NPL][NF], auto i) {
      // piece products, small terms first.  Three planes (0 hi, 1 mid, 2 lo): lo*hi, hi*lo, mid*mid, mid*hi, hi*mid,
      // hi*hi; two planes (0 hi, 1 lo): lo*hi, hi*lo, hi*hi
      constexpr int pp = decltype(i)::value / (MI * NI), rem = decltype(i)::value % (MI * NI);
      constexpr int mi = rem / NI, ni = rem % NI;
      constexpr int pa = NPL == 3 ? (pp == 0 ? 2 : (pp == 2 || pp == 3 ? 1 : 0)) : (pp == 0 ? 1 : 0);
      constexpr int pb = NPL == 3 ? (pp == 1 ? 2 : (pp == 2 || pp == 4 ? 1 : 0)) : (pp == 1 ? 1 : 0);
      acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, F[pa][mi]),
                                                           __builtin_bit_cast(bf16x8, F[pb][MI + ni]), acc[mi][ni], 0, 0, 0);
    };
    auto wait_reads = [&](uintx4(&F)[NPL][NF]) {  // every operand read has landed; ties the registers to the wait
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      tie_registers<NPL, NF>(F);
    };

    // prologue: the first NS - 1 steps in flight (steps past the end repeat the last one: the count of loads in flight
    // stays the same in every step, and the repeated data lands in a stage that is never read)
    static_for<0, NS - 1>([&](auto s) { load_stage(decltype(s)::value, min(k0 + decltype(s)::value, k1 - 1)); });
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(ND * (NS - 2)) : "memory");
    __builtin_amdgcn_s_barrier();
    SPCFG_SB
    static_for<0, NR>([&](auto r) { read_one(X, r, a_frag, b_frag); });
    int cur = 0;
    for (int kt = k0; kt < k1; ++kt) {
      const int nxt = cur + 1 == NS ? 0 : cur + 1;
      const int fill = cur == 0 ? NS - 1 : cur - 1;   // the stage of step kt - 1: free since that step's barrier
      const int kfill = min(kt + NS - 1, k1 - 1) + krot;
      const int64_t koff = (int64_t)(kfill >= KTt ? kfill - KTt : kfill) * 64;
      const unsigned fill_lds = lds0 + fill * Q::STAGE;
      const unsigned aa1 = a_frag1 + cur * Q::STAGE, ba1 = b_frag1 + cur * Q::STAGE;
      const unsigned aa0 = a_frag + nxt * Q::STAGE, ba0 = b_frag + nxt * Q::STAGE;
      SPCFG_SB
      wait_reads(X);
      SPCFG_SB
      // first half: products of chunk 0, reads of chunk 1, loads of step kt + NS - 1
      static_for<0, NM>([&](auto i) {
        constexpr int iv = decltype(i)::value;
        mfma_one(X, i);
        SPCFG_SB
        static_for<0, Q::RPF>([&](auto q) {
          constexpr int r = iv * Q::RPF + decltype(q)::value;
          if constexpr (r < NR) read_one(Y, std::integral_constant<int, r>{}, aa1, ba1);
        });
        static_for<0, ND>([&](auto j) {
          if constexpr ((decltype(j)::value * NM) / ND == iv) dma16(gp[decltype(j)::value] + koff, fill_lds + e_lds[decltype(j)::value]);
        });
        SPCFG_SB
      });
      wait_reads(Y);
      SPCFG_SB
      // second half: products of chunk 1; behind the first of them the barrier (every wavefront's loads of step kt + 1
      // have landed, every wavefront has its operands of step kt), then the reads of the next step's chunk 0
      static_for<0, NB>([&](auto i) { mfma_one(Y, i); });
      SPCFG_SB
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(ND * (NS - 2)) : "memory");
      __builtin_amdgcn_s_barrier();
      SPCFG_SB
      constexpr int RS = NM - NB;                              // matrix instructions left
      constexpr int RPS = (NR + (RS > 1 ? RS - 2 : 0)) / (RS > 1 ? RS - 1 : 1);  // reads per slot, tail slots free
      static_for<NB, NM>([&](auto i) {
        constexpr int s = decltype(i)::value - NB;
        mfma_one(Y, i);
        SPCFG_SB
        static_for<0, RPS>([&](auto q) {
          constexpr int r = s * RPS + decltype(q)::value;
          if constexpr (r < NR) read_one(X, std::integral_constant<int, r>{}, aa0, ba0);
        });
        SPCFG_SB
      });
      cur = nxt;
    }
    wait_reads(X);  // the last step read ahead into a stage without data: nothing of it is used
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();  // every load has landed and every operand is in registers before the ring is reused

    finish_tile<BM>(g.partial, g.counters, acc, tile, ustart, k0, k1, KTt, ipw, wg, it, wg_begin, tid, &s_last,
                    [&](floatx16(&t)[MI][NI]) { epilogue<EPI, BM>(g, t, row0, col0, wm, wn, lane, row_end, c_shift); });
    it += k1 - k0;
  }
}

template <int EPI, int BM, int MODE, int NPL>
void launch3(const NtArgs& a, hipStream_t st) {
  using Q = Geo3<BM, NPL>;
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_nt3<EPI, BM, MODE, NPL>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)Q::kLds);
    attr_set = true;
  }
  // shares of the (tile, K-step) space: at most one workgroup per CU
  const int tiles_n = (a.cols + BN - 1) / BN;
  int tiles = ((a.rows + BM - 1) / BM) * tiles_n;
  const int KT = a.K / BK3;
  int total = tiles * KT;
  if (a.parts > 0) {
    tiles = 0; total = 0;
    for (int p = 0; p < a.parts; ++p) {
      const int tp = ((a.prt_rows[p] + BM - 1) / BM) * tiles_n;
      tiles += tp;
      total += tp * a.prt_kt[p];
    }
    if (total == 0) return;
  }
  if (tiles > a.n_counters) { launch_refused("projection product: more output tiles than arrival counters"); return; }
  int Gn = 256;
  const int cap = a.max_wgs * (128 / BM);  // the partial-tile scratch holds 2 * max_wgs slots of 128 x 128
  if (Gn > cap) Gn = cap;
  if (Gn > total / 2) Gn = total / 2 > 0 ? total / 2 : 1;  // at least two K-steps per share
  int ipw = (total + Gn - 1) / Gn;
  Gn = (total + ipw - 1) / ipw;
  // Every XCD has an L2 of its own and runs consecutive shares, so what the launch fetches past L2 is, per XCD, the
  // operand rows of the block of tiles it runs at a time: (a + b) row panels for a block of a row tiles x b column tiles.
  // Row-tile groups (1, 2 or 4) make that block as square as the tile counts allow.
  int mgroups = 1;
  if (a.parts == 0) {
    const int tiles_m = (a.rows + BM - 1) / BM, passes = tiles / 256 > 0 ? tiles / 256 : 1;
    int best = 1 << 30;
    for (int mg = 1; mg <= 4; mg *= 2) {
      if (mg > 1 && tiles_m < 2 * mg) break;
      const int am = tiles_m / (mg * passes) > 0 ? tiles_m / (mg * passes) : 1, bn = tiles_n * mg / 8 > 0 ? tiles_n * mg / 8 : 1;
      if (am + bn < best) { best = am + bn; mgroups = mg; }
    }
  }
  launch_k(k_gemm_nt3<EPI, BM, MODE, NPL>, dim3(Gn), dim3(256), Q::kLds, st, a, ipw, total, mgroups);
}

template <int EPI, int NPL>
void launch_bm3(const NtArgs& a, hipStream_t st) {
  const int bm = chosen_bm(a);
  if (a.parts > 0) {
    switch (bm) {
      case 32: launch3<EPI, 32, 2, NPL>(a, st); break;
      case 64: launch3<EPI, 64, 2, NPL>(a, st); break;
      default: launch3<EPI, 128, 2, NPL>(a, st); break;
    }
    return;
  }
  switch (bm) {
    case 32: launch3<EPI, 32, 0, NPL>(a, st); break;
    case 64: launch3<EPI, 64, 0, NPL>(a, st); break;
    default: launch3<EPI, 128, 0, NPL>(a, st); break;
  }
}

template <int EPI>
void launch_tall3(const NtArgs& a, hipStream_t st) {
  if (a.parts > 0) launch3<EPI, 128, 2, 3>(a, st); else launch3<EPI, 128, 0, 3>(a, st);
}

}  // namespace

// planes3 == 3: the launches with 128-row tiles of the fp32 mode (gemm_nt_reads_planes); planes3 == 2: every forward
// product of the bf16 mode.
void launch_gemm_nt3(const NtArgs& a, hipStream_t st) {
  if (a.rows <= 0 || a.cols <= 0 || !a.planes3 || a.grouped) return;
  if (a.planes3 == 2) {
    if (a.epilogue != NT_EPI_ROWSCALE) { launch_refused("two-plane projection product: forward epilogue only"); return; }
    launch_bm3<NT_EPI_ROWSCALE, 2>(a, st);
    return;
  }
  switch (a.epilogue) {
    case NT_EPI_ROWSCALE: launch_tall3<NT_EPI_ROWSCALE>(a, st); break;
    case NT_EPI_MASKROWS: launch_tall3<NT_EPI_MASKROWS>(a, st); break;
    default: launch_tall3<NT_EPI_LEAF_EMIT>(a, st); break;
  }
}

}  // namespace spcfg
