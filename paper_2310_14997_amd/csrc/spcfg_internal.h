// Internal declarations shared by the host scheduler and the kernel launchers of libspcfg.
//
// Representation (paper Sec. 3.2 rescales by the per-span maximum in log space; here the same
// rescaling is done with exact powers of two):  every chart vector v of a span is stored as an fp32
// vector vt plus one integer exponent e per span, v = 2^e * vt.  Scaling by a power of two is exact in
// fp32, so the only rounding is that of the probability-space products and sums themselves.
//   leaf row r:        leafE[r] = exp(e_i - max e_i)          (exponent 0; the max is added back into logZ)
//   span row r (w>=2): T[r]     = sum_k 2^(d_k - m) * eta_ik * zeta_kj,  m = max_k d_k   (exponent mexp[r] = m)
//   every non-root row: HZ[r]   = [eta | zeta] = 2^-f * [L;R] * (leafE[r] or T[r])        (exponent mexp[r] + f)
//                      eta and zeta each have a normalising shift of their own on top: the producer of the inside
//                      vector records hmaxb[r] = max_B (exponent of max_A L[A,B]) + (exponent of its entry B), zmaxb
//                      likewise with R, which bounds the largest entry of eta (zeta) from below to within a factor 4N.
//                      A grammar whose weights are tiny everywhere gives tiny projections, and with these shifts the
//                      split products eta * zeta stay inside the fp32 range
//                      Halves that no span ever reads are left unwritten when the launch is cut into parts (shared
//                      grammar, width >= 2, Np a multiple of 128): zeta of the prefix rows (i = 0) and eta of the
//                      suffix rows (j = n) of HZ hold whatever the workspace held before the call.  No kernel reads them (the split kernels pick a child's half by
//                      its position); anything added later that walks HZ must do the same.  A test runs with a
//                      workspace pre-filled with 0xFF bytes to catch a read of such a half.
//   reverse pass:      UV[r]    = unnormalised adjoints of [eta | zeta]                   (exponent uexp[r])
//                      BH[r]    = 2^-f' * UV[r] * [L;R]  = scaled adjoint of beta         (exponent uexp[r] + f')
// f (f') is the shift that brings the largest magnitude of T[r] (UV[r]) into [0.5, 1).  The split kernels
// record that magnitude's bit pattern in tmaxb[r] (umaxb[r]) with an integer atomicMax; the GEMM epilogue
// applies 2^-f, and every consumer derives the exponent from (mexp, tmaxb) or (uexp, umaxb).
// Rows are ordered by width, then sentence, then start position, so each width is one contiguous block.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

#include <tuple>
#include <utility>

#include "../../include/spcfg.h"

namespace spcfg {

constexpr int kPad = 64;                 // N and P are padded to multiples of this (zero filled)
constexpr int kExpZero = -(1 << 24);     // exponent marking an all-zero vector
constexpr int kMaxB = 960;               // lengths travel as one kernel argument
constexpr int kMaxLen = 1024;

inline int round_up(int x, int m) { return (x + m - 1) / m * m; }

struct Layout {
  int N, P, Np, Pp, B, n_max;
  int G;                 // number of grammars: 1 (shared by the batch) or B (one per sentence)
  int bf16;              // projections with bf16 operands: packed weights are bf16, transposed bf16 copies for the rule gradients
  int planes;            // bf16 planes that producers write beside every fp32 chart row for the forward projection products:
                         // 0 none (fp32 operands are staged and cut in the kernel), 1 the bf16 rounding (bf16 mode, one
                         // grammar per sentence), 2 hi + lo (bf16 mode, shared grammar), 3 the exact cut hi + mid + lo
                         // of every fp32 value (fp32 mode, shared grammar)
  int planes_bwd;        // the same for the adjoint rows of the reverse products: 0, 1 (bf16 mode) or 3
  int tn3;               // rule gradients on operand planes (fp32 mode, shared grammar): Tg3 / Eg3 below, padded UVb
  int64_t S1p32, S2p32;  // row counts rounded up to whole 32-row steps of that product
  int64_t uvb_plane;     // elements between the planes of UVb: (Sall [+ 32 zeroed rows]) * 2Np
  int fwd_fp32;          // bf16 mode with one grammar per sentence: the forward products read fp32 operands (Wn / Wp are
                         // fp32 then, Wtn / Wtp bf16)
  int64_t S1pad, S2pad;  // row counts rounded up to 64 (K of the bf16 rule-gradient product)
  int64_t S1, S2, Sall;  // leaf rows, rows of width >= 2, all rows
  // byte offsets into the workspace
  size_t lens, rowbase, row_b, row_i, rootmask, rootrow, mexp, uexp, tmaxb, umaxb, hmaxb, zmaxb, gsc, xs, ztil, rmax;
  size_t leafE, T, HZ, UV, BH, Wn, Wp, Wtn, Wtp, partial, counters;
  size_t colmax;  // [G][2][Np + Pp]: largest entry of every column of L (then of R), nonterminal columns first
  size_t Wn3, Wp3, Wtn3, Wtp3;  // the packed panels once more, cut into bf16 planes: Wn3 / Wp3 `planes` of them (if >= 2), Wtn3 / Wtp3 three (planes_bwd == 3)
  size_t UVt_n, Tt, UVt_p, Et;  // bf16 mode only
  size_t Tg3, Eg3;              // tn3: three bf16 planes of gsc[s] * T[s] ([3][S2p32][Np]) and of gsc[s] * leafE[s] ([3][S1p32][Pp])
  size_t Tb, UVb, leafEb;       // planes > 0: bf16 planes of T, UV, leafE ([planes][rows][cols]), written by their producers
  size_t sentrows, sentoff;     // per-sentence grammars only: rows of width >= 2 listed sentence by sentence, first entry of each
  int n_counters;
  int gemm_wgs;          // workgroups the partial-tile scratch is sized for (kGemmWgs, fewer for the static scratch)
  size_t total;
};

struct Ptrs {  // device pointers resolved from a Layout
  int32_t *lens, *rowbase, *row_b, *row_i, *rootmask, *rootrow, *mexp, *uexp;
  uint32_t *tmaxb, *umaxb;
  int32_t *hmaxb, *zmaxb;  // biased-exponent sums (see above); 0 = the projection is all zero
  float* colmax;
  float *gsc, *xs, *ztil, *rmax;
  float *leafE, *T, *HZ, *UV, *BH, *Wn, *Wp, *Wtn, *Wtp, *partial;  // W* hold bf16 data in bf16 mode
  void *UVt_n, *Tt, *UVt_p, *Et;
  void *Tg3, *Eg3;
  void *Tb, *UVb, *leafEb;  // null when the layout has no planes
  void *Wn3, *Wp3, *Wtn3, *Wtp3;
  int32_t* counters;
  int32_t* sentrows; int32_t* sentoff;
};

struct LenArg {  // lengths passed by value: no host buffer has to outlive the call
  int32_t v[kMaxB];
};

// ---- kernel launch ------------------------------------------------------------------------------------
// While per-kernel-class timing is enabled every launch carries a start and a stop event that are bound to the
// kernel's own dispatch (hipExtLaunchKernel), so the measured time is the kernel's and nothing is inserted
// between two kernels; otherwise the events are null and the launch is an ordinary one.
struct LaunchEvents { hipEvent_t start = nullptr, stop = nullptr; };
LaunchEvents prof_launch_events();  // a fresh pair charged to the current kernel class, or nulls

template <typename... P, typename... A, size_t... I>
inline void launch_k_impl(void (*kernel)(P...), dim3 grid, dim3 block, size_t shmem, hipStream_t st,
                          std::index_sequence<I...>, A&&... args) {
  std::tuple<P...> vals{static_cast<P>(std::forward<A>(args))...};  // copies with the kernel's parameter types
  void* ptrs[sizeof...(P) > 0 ? sizeof...(P) : 1] = {static_cast<void*>(&std::get<I>(vals))...};
  const LaunchEvents ev = prof_launch_events();
  if (ev.start && ev.stop)
    (void)hipExtLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, shmem, st, ev.start, ev.stop, 0);
  else
    (void)hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, shmem, st);
}
template <typename... P, typename... A>
inline void launch_k(void (*kernel)(P...), dim3 grid, dim3 block, size_t shmem, hipStream_t st, A&&... args) {
  static_assert(sizeof...(P) == sizeof...(A), "argument count does not match the kernel");
  launch_k_impl(kernel, grid, block, shmem, st, std::index_sequence_for<P...>{}, std::forward<A>(args)...);
}

// A launcher that finds its launch outside what the workspace was sized for does not launch and reports it here;
// the API call then returns SPCFG_ERR_WORKSPACE.
void launch_refused(const char* what);

// ---- launchers (each only enqueues on `st`) -------------------------------------------------------
void launch_plan(const Layout& ly, const Ptrs& p, const LenArg& lens, hipStream_t st);
void launch_plan_sentrows(const Layout& ly, const Ptrs& p, hipStream_t st);
void launch_pack_weights(const Layout& ly, const Ptrs& p, const float* L, const float* R, hipStream_t st);
void launch_transpose_bf16(const float* X, int64_t ldx, int cols, const float* sc, int64_t S, int64_t Spad, void* Xt,
                           hipStream_t st);
void launch_leaf_prep(const Layout& ly, const Ptrs& p, const float* log_emit, bool write_planes, hipStream_t st);
// write_planes: also write the operand planes of the rows (the projection launch of this width reads them)
void launch_split_fwd(const Layout& ly, const Ptrs& p, int w, int64_t row0, int64_t rows, bool write_planes,
                      hipStream_t st);
// log_root (and grad_log_root) hold one vector per grammar: [G x N]
void launch_root_fwd(const Layout& ly, const Ptrs& p, const float* log_root, float* logZ, hipStream_t st);
void launch_root_bwd(const Layout& ly, const Ptrs& p, const float* log_root, const float* grad_logZ,
                     float* grad_log_root, int accumulate, hipStream_t st);
void launch_split_bwd(const Layout& ly, const Ptrs& p, int w, int64_t row0, int64_t rows, bool write_planes,
                      hipStream_t st);
void launch_zero_pad_emit(const Layout& ly, const Ptrs& p, float* grad_log_emit, hipStream_t st);
void launch_span_marginals(const Layout& ly, const Ptrs& p, float* mu, int32_t* label, hipStream_t st);

// C[r][c] = sum_k A[r][k] * Bm[c][k]   (both operands K-contiguous), r < rows, c < cols, K % 32 == 0.
enum NtEpilogue { NT_EPI_ROWSCALE = 0, NT_EPI_MASKROWS = 1, NT_EPI_LEAF_EMIT = 2, NT_EPI_GRAD = 3 };
struct NtArgs {
  // fp32 mode: A, Bm are float.  bf16 mode (a_bf16 = b_bf16 = 1): both point to bf16 data.  lda/ldb count
  // elements; K % 64 == 0 in bf16 mode.
  const void* A; int64_t lda;
  const void* Bm; int64_t ldb;
  int a_bf16, b_bf16;
  float* C; int64_t ldc;
  int rows, cols, K;
  int epilogue;
  const uint32_t* rowmaxb;  // ROWSCALE, MASKROWS: C = 2^-f(rowmaxb[r]) * acc (normalising shift of the A row)
  const int32_t* rowmask;   // MASKROWS: rows with rowmask[r] != 0 are left untouched
  // LEAF_EMIT: C[dst[r] * ldc + c] = acc * E[r][c] * 2^rowexp[r], c < cols
  const float* E; int64_t lde;
  const int32_t* rowexp;
  const int32_t* row_b; const int32_t* row_i; int n_max;
  // GRAD: rows are stacked parents; row r -> (r < Np ? gL : gR)[(r mod Np) * ldg + col0 + c], rows >= Nvalid per half dropped
  float* gL; float* gR; int64_t ldg; int col0, Np, Nvalid, accumulate;
  // work sharing across workgroups: scratch for partial tiles and per-tile arrival counters (zero between launches)
  float* partial; int32_t* counters; int max_wgs;
  int n_counters;  // capacity of `counters`: a launch with more output tiles is refused (see launch_refused)
  // Grouped mode (one grammar per sentence): the rows of the launch are the spans of one width, sentence
  // after sentence; sentence b owns rows [grp_rowbase[b] - grp_row_first, + max(0, grp_lens[b] - grp_w + 1)) and
  // multiplies them with its own operand Bm + b * grp_b_stride.  Row tiles never straddle two sentences.
  int grouped, ngroups, grp_w;
  const int32_t* grp_lens; const int32_t* grp_rowbase; int64_t grp_row_first; int64_t grp_b_stride;
  int grp_tiles_m[3];  // host: number of row tiles for tile heights 32, 64, 128
  int grp_max_rows;    // host: largest row count of one sentence
  // Parts mode (fp32, shared grammar, width >= 2): `parts` products in one launch.  Part p multiplies the rows
  // [prt_row0[p], + prt_rows[p]) with the columns [prt_c0[p], + cols) of Bm / C over the K-steps
  // [prt_kbeg[p], + prt_kt[p]) (steps of 32 values).  The span plan puts the prefix spans first and the suffix
  // spans last within a width, so "rows whose eta is used", "rows whose zeta is used" (forward: two parts, one
  // column block each) and "prefix / middle / suffix rows" (reverse: the adjoint of zeta resp. eta is zero, half
  // of K is skipped) are contiguous ranges.
  int fp32_mfma;  // 1: fp32 matrix instructions instead of the split-bf16 scheme (fp32 operands only)
  // planes3 = 3: both operands are also given as three bf16 planes (the exact cut hi + mid + lo of every fp32 value,
  // nt::Split3), written by their producers: A3 = [3][..][lda] with planes a_plane elements apart, Bm3 likewise with
  // b_plane; the launches with tall row tiles run on them in gemm_nt3.hip.  A / Bm stay the fp32 operands, which the
  // launches with short row tiles use (their time goes into reading the panel once, and the fp32 panel is a third
  // shorter than its three planes).  planes3 = 2: two planes (hi, lo) and every launch runs on them (forward products
  // of the bf16 mode).
  int planes3; int64_t a_plane, b_plane;
  const void* A3; const void* Bm3;
  int parts;
  int prt_row0[3], prt_rows[3], prt_c0[3], prt_kbeg[3], prt_kt[3];
};
void launch_gemm_nt(const NtArgs& a, hipStream_t st);
void launch_gemm_nt16(const NtArgs& a, hipStream_t st);  // bf16-operand variant (called through launch_gemm_nt)
void launch_gemm_nt3(const NtArgs& a, hipStream_t st);   // pre-cut three-plane operands (called through launch_gemm_nt)
bool gemm_nt_keep_parts(NtArgs& a);             // drops the parts of a launch that would not save work
bool gemm_nt_reads_planes(const NtArgs& a);     // whether launch_gemm_nt will read the plane operands (A3 / Bm3)
int gemm_nt_tiles(int rows, int cols);           // number of output tiles (= arrival counters needed)
size_t gemm_nt_partial_bytes(int max_wgs);       // scratch needed for partial tiles
constexpr int kGemmWgs = 512;                    // workgroups per projection launch: 2 per CU on 256 CUs

// C[a][b] (+)= sum_s sc[s] * A[s][a] * Bm[s][b]   (both operands reduction-major), written into grad_L / grad_R.
struct TnArgs {
  int fp32_mfma;                    // 1: fp32 matrix instructions instead of the split-bf16 scheme
  const float* A; int64_t lda;     // UV rows [S x 2Np]
  const float* Bm; int64_t ldb;    // T rows [S x Np] or leafE rows [S x Pp]
  const float* sc;                 // [S]
  int64_t S;
  int Np;                          // rows a in [0,Np) -> grad_L, [Np, 2Np) -> grad_R
  int N;                           // valid rows per half
  int cols;                        // valid output columns
  float* gL; float* gR; int64_t ldg; int col0;  // destination column offset (0 or N)
  int accumulate;
  float* partial; int32_t* counters; int max_wgs;  // work sharing scratch, as in NtArgs
  int n_counters;
  // Grouped mode (one grammar per sentence): sentence b reduces over its own rows only and writes gL / gR + b * grp_gstride;
  // A, Bm, sc are then the whole arrays, indexed by span row.
  //   grp_mode 1: rows rowlist[grp_off[b] + s], s < n_b (n_b - 1) / 2  (spans of width >= 2; the Bm row is row - brow0)
  //   grp_mode 2: rows grp_base[b] + s, s < n_b                        (leaves)
  int grp_mode, ngroups;
  const int32_t* grp_lens; const int32_t* grp_off; const int32_t* grp_base; const int32_t* rowlist;
  int64_t brow0, grp_gstride;
  int grp_kt_max;  // number of 32-row steps of the longest per-sentence reduction
};
void launch_gemm_tn(const TnArgs& a, hipStream_t st);

// The same product on operands that their producers have cut into three bf16 planes (gemm_tn3.hip): A3 = planes of the
// adjoint rows UV ([3][..][lda], planes a_plane elements apart, pointing at the first row of the block), B3 = planes of
// scale[s] * (inside vector of row s), zero from row S to the end of the last 32-row step.  A3 must be readable (and
// finite) for 31 rows past the end of the reduction.
struct Tn3Args {
  const uint16_t* A3; int64_t a_plane, lda;
  const uint16_t* B3; int64_t b_plane, ldb;
  int KT;                           // 32-row steps of the reduction: ceil(S / 32)
  int Np, N, cols;                  // as in TnArgs
  float* gL; float* gR; int64_t ldg; int col0;
  int accumulate;
  float* partial; int32_t* counters; int max_wgs, n_counters;
};
void launch_gemm_tn3(const Tn3Args& a, hipStream_t st);
// planes of sc[s] * X[s][.] for s < S and of zero for S <= s < Srows (X is [S x ld], ld a multiple of 4)
void launch_scaled_planes(const float* X, int64_t ld, const float* sc, int64_t S, int64_t Srows, void* planes,
                          int64_t plane_stride, hipStream_t st);
// zeroes rows [row0, row0 + rows) of every plane of a [3][..][ld] array of bf16
void launch_zero_plane_rows(void* planes, int64_t plane_stride, int64_t ld, int64_t row0, int64_t rows, hipStream_t st);

}  // namespace spcfg
