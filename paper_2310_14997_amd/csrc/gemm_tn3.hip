// Rule-gradient GEMM on operands that arrive already cut into three bf16 planes:
//   d/d[L;R][a][b] = sum_s A[s][a] * B[s][b],  A = adjoint rows of [eta | zeta], B = scale[s] * inside vector of row s
// (chain rule through the stacked projection of Sec. 3.2; the per-span power-of-two scale is folded into B's planes
// by their producer, so this kernel does no vector work).  Both operands are reduction-major ([s][column]): tiles of
// 32 span rows x 128 columns go straight from global memory into LDS as they lie (global_load_lds_dwordx4, 1 KB per
// wavefront instruction = 4 rows of 256 bytes), into a ring of three stages, and the matrix operands - eight
// consecutive reduction rows of one column per lane - come out of LDS through the transposing read
// ds_read_b64_tr_b16: within 16 lanes, lane i passes the address of row k0 + i/4, columns 4 (i mod 4) .. + 3, and lane
// j receives column j of rows k0 .. k0 + 3.  The 64-byte blocks of an LDS row are XORed with (row mod 4) on the way in
// (the loads pick their global columns accordingly), which makes those reads conflict-free.
// Exact three-piece cut and six piece products as in the projection kernels (nt::Split3); 128 x 128 output tile,
// 4 wavefronts (2 x 2) of 2 x 2 tiles of 32 x 32, one workgroup per CU, the instruction order of a step written out
// as in gemm_nt3.hip.  Rows past the end of the reduction contribute nothing: B's planes are zero there (its producer
// pads them to whole steps) and A's are finite (zeroed padding rows, or rows of the next block).
#include <type_traits>
#include <utility>

#include "gemm_nt_common.h"

namespace spcfg {

namespace {

using namespace nt;

typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));

constexpr int T3M = 128, T3N = 128, T3K = 32;
constexpr int kOpnd = T3K * 256;            // bytes of one operand tile of one plane: 32 rows of 128 bf16
constexpr int kPlane = 2 * kOpnd;           // [A tile | B tile]
constexpr int kStage3 = 3 * kPlane;         // three planes
constexpr int kNS = 3;
constexpr size_t kLdsTn3 = (size_t)kNS * kStage3;
constexpr int kND = 12;                     // 1 KB load instructions per wavefront and stage (48 per workgroup)
constexpr int kNF = 4;                      // operand fragments per plane and 16-row chunk (2 of A, 2 of B)
constexpr int kNR = 3 * kNF * 2;            // transposing reads per chunk (two per fragment: rows 0..3 and 4..7 of its 8)
constexpr int kNM = 6 * 2 * 2;              // matrix instructions per chunk
constexpr int kNB = 2;                      // matrix instructions ahead of the barrier

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

// One operand fragment of one plane: eight reduction rows of a column per lane, as two 64-bit halves.
struct Frag { uintx2 lo, hi; };
__device__ __forceinline__ bf16x8 operand(const Frag& f) {
  return __builtin_bit_cast(bf16x8, uintx4{f.lo[0], f.lo[1], f.hi[0], f.hi[1]});
}
template <int R = 0>
__device__ __forceinline__ void tie_frags(Frag (&F)[3][kNF]) {
  if constexpr (R < 3 * kNF) {
    asm volatile("" : "+v"(F[R / kNF][R % kNF].lo), "+v"(F[R / kNF][R % kNF].hi));
    tie_frags<R + 1>(F);
  }
}

#define SPCFG_SB __builtin_amdgcn_sched_barrier(0);

__global__ void __launch_bounds__(256, 1) k_gemm_tn3(Tn3Args g, int ipw, int total_iters) {
  extern __shared__ __align__(16) unsigned char lds3[];
  __shared__ int s_last;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int uw = __builtin_amdgcn_readfirstlane(wave);
  const int wm = wave & 1, wn = wave >> 1;
  const int tiles_a = (2 * g.Np) / T3M;
  const int tiles_b = (g.cols + T3N - 1) / T3N;
  const int KT = g.KT;
  const unsigned lds0 = lds_address(lds3);
  // transposing reads: lane = 16 q + i reads row 8 (q / 2) + i / 4 of the chunk, columns 32 f + 16 (q % 2) + 4 (i % 4) .. + 3
  // of fragment f's 32 columns, whose 64-byte block is f XOR (row mod 4)
  const int li = lane & 15, lq = lane >> 4;
  const unsigned row_in = (unsigned)(8 * (lq >> 1) + (li >> 2));
  const unsigned in_blk = (unsigned)(32 * (lq & 1) + 8 * (li & 3));
  unsigned fbase[kNF];  // byte offset inside a stage of fragment f, plane 0, chunk 0, first half
#pragma unroll
  for (int f = 0; f < kNF; ++f) {
    const unsigned blk = (unsigned)((f < 2 ? wm : wn) * 2 + (f & 1));
    fbase[f] = (f < 2 ? 0u : (unsigned)kOpnd) + row_in * 256u + ((blk ^ (unsigned)(li >> 2)) * 64u) + in_blk;
  }
  // this wavefront's load instructions: entry e = uw + 4 t of the stage's 48: plane e / 16 = t / 4, operand A for
  // (e % 16) < 8, i.e. t % 4 < 2, rows 4 ((e % 16) % 8) .. + 3; lane l lands at + 16 l: row l / 16 of the four, 16-byte
  // chunk l % 16
  int e_row[kND];
  unsigned e_lds[kND];
#pragma unroll
  for (int t = 0; t < kND; ++t) {
    const int j = (uw + 4 * t) & 15;
    e_row[t] = 4 * (j & 7) + (lane >> 4);
    e_lds[t] = (unsigned)((t / 4) * kPlane + ((t % 4) < 2 ? 0 : kOpnd) + (j & 7) * 1024);
  }
  const int c16 = lane & 15;
  // global column (elements) of this lane's 16 bytes: 64-byte block (c16 / 4) XOR (row mod 4), 16-byte piece c16 % 4
  const int gcol = (((c16 >> 2) ^ (lane >> 4)) * 32) + (c16 & 3) * 8;

  const int wg = renumbered_wg();
  const int wg_begin = wg * ipw;
  const int wg_end = min(wg_begin + ipw, total_iters);
  int it = wg_begin;
  while (it < wg_end) {
    const int tile = it / KT;
    const int k0 = it - tile * KT;
    const int k1 = min(KT, k0 + (wg_end - it));
    int tile_a = tile % tiles_a, tile_b = tile / tiles_a;
    // 64 consecutive tiles (what one XCD works on at a time) form an 8 x 8 block of the output: its L2 fetches 16 operand
    // panels for them and not 34
    if ((tiles_a & 7) == 0 && (tiles_b & 7) == 0) {
      const int blk = tile >> 6, l = tile & 63, blocks_a = tiles_a >> 3;
      tile_a = (blk % blocks_a) * 8 + (l & 7);
      tile_b = (blk / blocks_a) * 8 + (l >> 3);
    }
    const int a0 = tile_a * T3M, b0 = tile_b * T3N;
    // position p of the tile's K loop is step (p + krot) mod KT (see gemm_nt3.hip: shares of any size stay in phase)
    const int krot = ((tile * KT) % ipw) % KT;

    const unsigned char* gp[kND];
#pragma unroll
    for (int t = 0; t < kND; ++t) {
      if ((t % 4) < 2) {
        gp[t] = reinterpret_cast<const unsigned char*>(g.A3 + (int64_t)(t / 4) * g.a_plane + (int64_t)e_row[t] * g.lda +
                                                       a0 + gcol);
      } else {
        const int c = b0 + gcol;  // columns past the padded width are read from column 0 and feed dropped outputs only
        gp[t] = reinterpret_cast<const unsigned char*>(g.B3 + (int64_t)(t / 4) * g.b_plane + (int64_t)e_row[t] * g.ldb +
                                                       (c < (int)g.ldb ? c : 0));
      }
    }
    const int64_t step_a = 2 * (int64_t)T3K * g.lda, step_b = 2 * (int64_t)T3K * g.ldb;  // bytes per K-step

    floatx16 acc[2][2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

    Frag X[3][kNF], Y[3][kNF];
    auto load_stage = [&](int stage, int kpos) {
      const int kr = kpos + krot;
      const int64_t ks = kr >= KT ? kr - KT : kr;
      static_for<0, kND>([&](auto t) {
        constexpr int tv = decltype(t)::value;
        dma16(gp[tv] + ks * ((tv % 4) < 2 ? step_a : step_b), lds0 + stage * kStage3 + e_lds[tv]);
      });
    };
    // read r of a chunk: plane r / 8, fragment (r % 8) / 2, half r % 2
    auto read_one = [&](Frag(&F)[3][kNF], auto r, unsigned stage_chunk) {
      constexpr int pl = decltype(r)::value / 8, f = (decltype(r)::value % 8) / 2, h = decltype(r)::value % 2;
      const unsigned addr = stage_chunk + fbase[f];
      if constexpr (h == 0) {
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(F[pl][f].lo) : "v"(addr), "n"(pl * kPlane));
      } else {
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(F[pl][f].hi) : "v"(addr), "n"(pl * kPlane + 1024));
      }
    };
    auto mfma_one = [&](Frag(&F)[3][kNF], auto i) {
      // piece products, small terms first: lo*hi, hi*lo, mid*mid, mid*hi, hi*mid, hi*hi (planes: 0 hi, 1 mid, 2 lo)
      constexpr int pp = decltype(i)::value / 4, rem = decltype(i)::value % 4;
      constexpr int mi = rem / 2, ni = rem % 2;
      constexpr int pa = pp == 0 ? 2 : (pp == 2 || pp == 3 ? 1 : 0);
      constexpr int pb = pp == 1 ? 2 : (pp == 2 || pp == 4 ? 1 : 0);
      acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(operand(F[pa][mi]), operand(F[pb][2 + ni]), acc[mi][ni], 0, 0, 0);
    };
    auto wait_reads = [&](Frag(&F)[3][kNF]) {
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      tie_frags(F);
    };

    // prologue: the first two steps in flight (steps past the end repeat the last one into a stage that is never read)
    static_for<0, kNS - 1>([&](auto s) { load_stage(decltype(s)::value, min(k0 + decltype(s)::value, k1 - 1)); });
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kND * (kNS - 2)) : "memory");
    __builtin_amdgcn_s_barrier();
    SPCFG_SB
    static_for<0, kNR>([&](auto r) { read_one(X, r, lds0); });
    int cur = 0;
    for (int kt = k0; kt < k1; ++kt) {
      const int nxt = cur + 1 == kNS ? 0 : cur + 1;
      const int fill = cur == 0 ? kNS - 1 : cur - 1;  // the stage of step kt - 1: free since that step's barrier
      const int kfill = min(kt + kNS - 1, k1 - 1) + krot;
      const int64_t ks = kfill >= KT ? kfill - KT : kfill;
      const int64_t off_a = ks * step_a, off_b = ks * step_b;
      const unsigned fill_lds = lds0 + fill * kStage3;
      const unsigned chunk1 = lds0 + cur * kStage3 + 16 * 256;  // rows 16..31 of this step
      const unsigned chunk0n = lds0 + nxt * kStage3;            // rows 0..15 of the next step
      SPCFG_SB
      wait_reads(X);
      SPCFG_SB
      // first half: products of rows 0..15, reads of rows 16..31, loads of step kt + 2
      static_for<0, kNM>([&](auto i) {
        constexpr int iv = decltype(i)::value;
        mfma_one(X, i);
        SPCFG_SB
        static_for<0, 2>([&](auto q) {  // two reads behind each of the first twelve: all have landed by the end of the half
          constexpr int r = iv * 2 + decltype(q)::value;
          if constexpr (r < kNR) read_one(Y, std::integral_constant<int, r>{}, chunk1);
        });
        static_for<0, kND>([&](auto t) {
          constexpr int tv = decltype(t)::value;
          if constexpr ((tv * kNM) / kND == iv) dma16(gp[tv] + ((tv % 4) < 2 ? off_a : off_b), fill_lds + e_lds[tv]);
        });
        SPCFG_SB
      });
      wait_reads(Y);
      SPCFG_SB
      // second half: products of rows 16..31; behind the first two the barrier (every wavefront's loads of step kt + 1
      // have landed, every wavefront has its operands of step kt), then the reads of the next step's rows 0..15
      static_for<0, kNB>([&](auto i) { mfma_one(Y, i); });
      SPCFG_SB
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kND * (kNS - 2)) : "memory");
      __builtin_amdgcn_s_barrier();
      SPCFG_SB
      static_for<kNB, kNM>([&](auto i) {
        constexpr int s = decltype(i)::value - kNB;
        mfma_one(Y, i);
        SPCFG_SB
        static_for<0, 2>([&](auto q) {
          constexpr int r = s * 2 + decltype(q)::value;
          if constexpr (r < kNR) read_one(X, std::integral_constant<int, r>{}, chunk0n);
        });
        SPCFG_SB
      });
      cur = nxt;
    }
    wait_reads(X);  // the last step read ahead into a stage without new data: nothing of it is used
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();  // every load has landed and every operand is in registers before the ring is reused

    finish_tile<128>(g.partial, g.counters, acc, tile, tile * KT, k0, k1, KT, ipw, wg, it, wg_begin, tid, &s_last,
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
          float* dst = (half ? g.gR : g.gL) + (int64_t)arow * g.ldg + g.col0;
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
    it += k1 - k0;
  }
}

}  // namespace

void launch_gemm_tn3(const Tn3Args& a, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_tn3), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)kLdsTn3);
    attr_set = true;
  }
  if (a.KT <= 0 || a.cols <= 0) return;
  const int tiles = ((2 * a.Np) / T3M) * ((a.cols + T3N - 1) / T3N);
  if (tiles > a.n_counters) { launch_refused("rule-gradient product: more output tiles than arrival counters"); return; }
  const int64_t total64 = (int64_t)tiles * a.KT;
  if (total64 >= ((int64_t)1 << 31)) { launch_refused("rule-gradient product: too many (tile, step) units"); return; }
  const int total = (int)total64;
  int Gn = 256;  // one workgroup per CU
  if (Gn > a.max_wgs) Gn = a.max_wgs;  // the partial-tile scratch holds 2 * max_wgs slots
  if (Gn > total / 2) Gn = total / 2 > 0 ? total / 2 : 1;
  int ipw = (total + Gn - 1) / Gn;
  Gn = (total + ipw - 1) / ipw;
  launch_k(k_gemm_tn3, dim3(Gn), dim3(256), kLdsTn3, st, a, ipw, total);
}

}  // namespace spcfg
