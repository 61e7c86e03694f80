// C ABI of libspcfg: argument checks, workspace layout, the width-synchronous schedule (Sec. 3.2,
// span-level parallelism: one launch handles every span of one width across the batch) and optional
// per-kernel-class timing with HIP events.
#include <cstdio>
#include <atomic>
#include <cstring>
#include <mutex>
#include <vector>

#include "spcfg_internal.h"

namespace spcfg {

namespace {

thread_local char g_hip_err[256] = "";
thread_local const char* g_refused = nullptr;  // set by a launcher that refused to launch

struct Plan {            // host-side copy of the span schedule
  std::vector<int64_t> off;   // off[w] = first row of width w (1-based), off[n_max+1] = Sall
  std::vector<int64_t> cnt;   // cnt[w] = number of spans of width w
  LenArg lens;
};

size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

int check_cfg(const spcfg_config* c) {
  if (!c || c->struct_size != sizeof(spcfg_config)) return SPCFG_ERR_ARG;
  if (c->N < 1 || c->P < 1 || c->N > (1 << 16) || c->P > (1 << 16)) return SPCFG_ERR_SHAPE;
  if (c->max_B < 1 || c->max_B > kMaxB || c->max_n < 2 || c->max_n > kMaxLen) return SPCFG_ERR_SHAPE;
  if (c->precision != SPCFG_PRECISION_FP32 && c->precision != SPCFG_PRECISION_BF16) return SPCFG_ERR_UNSUPPORTED;
  if (c->flags & ~(uint32_t)(SPCFG_FLAG_ACCUMULATE_GRADS | SPCFG_FLAG_PER_SENTENCE_GRAMMAR | SPCFG_FLAG_FP32_MFMA |
                              SPCFG_FLAG_BF16_SINGLE_FORWARD)) return SPCFG_ERR_UNSUPPORTED;
  return SPCFG_OK;
}

// Byte layout of the workspace for a batch with S1 leaf rows and S2 rows of width >= 2.
Layout make_layout(int N, int P, int B, int n_max, int64_t S1, int64_t S2, int bf16, int per_sentence, int fp32_mfma,
                   int bf16_single, int gemm_wgs = kGemmWgs) {
  Layout ly{};
  ly.gemm_wgs = gemm_wgs;
  // Operand planes for the projection products.  fp32 mode with a shared grammar: the exact three-piece cut, forward
  // and reverse (the products then never cut operands themselves).  bf16 mode with a shared grammar: two pieces
  // (hi + lo) for the forward products, which decide log Z, the plain bf16 rounding for the reverse ones; with one
  // grammar per sentence the forward products run on fp32 operands instead (the grouped kernel cuts them itself; there
  // is no grouped kernel on planes), the reverse ones on one plane; one plane both ways when the caller asks for single
  // bf16 operands.
  const bool shared = !(per_sentence && B > 1);
  ly.fwd_fp32 = bf16 && !shared && !bf16_single;
  ly.planes = bf16 ? (bf16_single ? 1 : (shared ? 2 : 0)) : (!shared || fp32_mfma ? 0 : 3);
  ly.planes_bwd = bf16 ? 1 : ly.planes;
  ly.N = N; ly.P = P; ly.B = B; ly.n_max = n_max; ly.bf16 = bf16;
  ly.G = per_sentence ? B : 1;
  ly.S1pad = (S1 + 63) / 64 * 64; ly.S2pad = (S2 + 63) / 64 * 64;
  ly.Np = round_up(N, kPad);
  ly.Pp = round_up(P, kPad);
  ly.S1 = S1; ly.S2 = S2; ly.Sall = S1 + S2;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
  const size_t i4 = sizeof(int32_t), f4 = sizeof(float);
  ly.lens = take(i4 * B);
  ly.rowbase = take(i4 * 3 * (size_t)(n_max + 1) * B);  // three tables, see the span plan kernel
  ly.rootrow = take(i4 * B);
  ly.ztil = take(f4 * B);
  ly.rmax = take(f4 * B);
  ly.row_b = take(i4 * ly.Sall);
  ly.row_i = take(i4 * ly.Sall);
  ly.rootmask = take(i4 * ly.Sall);
  ly.mexp = take(i4 * ly.Sall);
  ly.uexp = take(i4 * ly.Sall);
  ly.tmaxb = take(i4 * ly.Sall);
  ly.umaxb = take(i4 * ly.Sall);
  ly.hmaxb = take(i4 * ly.Sall);
  ly.zmaxb = take(i4 * ly.Sall);
  ly.colmax = take(f4 * 2 * (size_t)(ly.Np + ly.Pp) * ly.G);
  ly.gsc = take(f4 * ly.Sall);
  ly.xs = take(f4 * S1);
  // One arrival counter per output tile of the largest launch: at most max(S1, S2) rows (one width; grouped
  // launches round every sentence's rows up to whole row tiles, at most one extra tile per sentence) and
  // max(2Np, Pp) columns (the projections write 2Np columns, the leaf reverse product P of them).  A launch cut
  // into up to three row ranges rounds each of them up to whole row tiles: two extra tiles of 32 rows (also with
  // the per-sentence flag when the batch is a single sentence: that runs as a shared grammar).
  ly.n_counters = gemm_nt_tiles((int)(S1 > S2 ? S1 : S2) + 64 + (per_sentence ? 32 * B : 0),
                                2 * ly.Np > ly.Pp ? 2 * ly.Np : ly.Pp);
  {  // the bf16 rule-gradient product has 2Np rows and up to max(Np, Pp) columns
    const int g = (2 * ly.Np / 128 + 1) * ((ly.Np > ly.Pp ? ly.Np : ly.Pp) / 128 + 1);
    if (g > ly.n_counters) ly.n_counters = g;
  }
  ly.counters = take(i4 * (size_t)ly.n_counters);
  ly.partial = take(gemm_nt_partial_bytes(gemm_wgs));
  const size_t w4 = bf16 ? 2 : 4;  // bytes per packed weight
  const size_t w4f = (bf16 && !ly.fwd_fp32) ? 2 : 4;  // ... of the forward panels
  ly.Wn = take(w4f * 2 * (size_t)ly.Np * ly.Np * ly.G);
  ly.Wp = take(w4f * 2 * (size_t)ly.Np * ly.Pp * ly.G);
  ly.Wtn = take(w4 * 2 * (size_t)ly.Np * ly.Np * ly.G);
  ly.Wtp = take(w4 * 2 * (size_t)ly.Np * ly.Pp * ly.G);
  if (ly.planes >= 2) {
    ly.Wn3 = take(2 * (size_t)ly.planes * 2 * ly.Np * ly.Np); ly.Wp3 = take(2 * (size_t)ly.planes * 2 * ly.Np * ly.Pp);
  }
  if (ly.planes_bwd == 3) {
    ly.Wtn3 = take(6 * 2 * (size_t)ly.Np * ly.Np); ly.Wtp3 = take(6 * 2 * (size_t)ly.Np * ly.Pp);
  }
  if (per_sentence) { ly.sentrows = take(i4 * (size_t)S2); ly.sentoff = take(i4 * (size_t)B); }
  if (bf16) {
    ly.UVt_n = take(2 * 2 * (size_t)ly.Np * ly.S2pad);
    ly.Tt = take(2 * (size_t)ly.Np * ly.S2pad);
    ly.UVt_p = take(2 * 2 * (size_t)ly.Np * ly.S1pad);
    ly.Et = take(2 * (size_t)ly.Pp * ly.S1pad);
  }
  if (ly.planes > 0) {
    ly.Tb = take(2 * (size_t)ly.planes * S2 * ly.Np);
    ly.leafEb = take(2 * (size_t)ly.planes * S1 * ly.Pp);
  }
  // rule gradients on planes (fp32 mode, shared grammar): the adjoint planes get 32 zeroed rows behind the last row (the
  // product reads whole 32-row steps), and the scaled inside vectors get planes of their own, padded to whole steps
  ly.tn3 = ly.planes_bwd == 3;
  ly.S1p32 = (S1 + 31) / 32 * 32; ly.S2p32 = (S2 + 31) / 32 * 32;
  ly.uvb_plane = (ly.Sall + (ly.tn3 ? 32 : 0)) * 2 * ly.Np;
  if (ly.planes_bwd > 0) ly.UVb = take(2 * (size_t)ly.planes_bwd * ly.uvb_plane);
  if (ly.tn3) {
    ly.Tg3 = take(6 * (size_t)ly.S2p32 * ly.Np);
    ly.Eg3 = take(6 * (size_t)ly.S1p32 * ly.Pp);
  }
  ly.leafE = take(f4 * (size_t)S1 * ly.Pp);
  ly.T = take(f4 * (size_t)S2 * ly.Np);
  ly.BH = take(f4 * (size_t)S2 * ly.Np);
  ly.HZ = take(f4 * (size_t)ly.Sall * 2 * ly.Np);
  ly.UV = take(f4 * (size_t)ly.Sall * 2 * ly.Np);
  ly.total = o;
  return ly;
}

Ptrs resolve(const Layout& ly, void* ws) {
  unsigned char* b = static_cast<unsigned char*>(ws);
  Ptrs p;
  p.lens = (int32_t*)(b + ly.lens); p.rowbase = (int32_t*)(b + ly.rowbase); p.rootrow = (int32_t*)(b + ly.rootrow);
  p.row_b = (int32_t*)(b + ly.row_b); p.row_i = (int32_t*)(b + ly.row_i); p.rootmask = (int32_t*)(b + ly.rootmask);
  p.mexp = (int32_t*)(b + ly.mexp); p.uexp = (int32_t*)(b + ly.uexp);
  p.tmaxb = (uint32_t*)(b + ly.tmaxb); p.umaxb = (uint32_t*)(b + ly.umaxb);
  p.hmaxb = (int32_t*)(b + ly.hmaxb); p.zmaxb = (int32_t*)(b + ly.zmaxb); p.colmax = (float*)(b + ly.colmax);
  p.gsc = (float*)(b + ly.gsc); p.xs = (float*)(b + ly.xs);
  p.ztil = (float*)(b + ly.ztil); p.rmax = (float*)(b + ly.rmax);
  p.leafE = (float*)(b + ly.leafE); p.T = (float*)(b + ly.T); p.HZ = (float*)(b + ly.HZ);
  p.UV = (float*)(b + ly.UV); p.BH = (float*)(b + ly.BH);
  p.partial = (float*)(b + ly.partial); p.counters = (int32_t*)(b + ly.counters);
  p.sentrows = (int32_t*)(b + ly.sentrows); p.sentoff = (int32_t*)(b + ly.sentoff);
  p.Tb = ly.planes ? b + ly.Tb : nullptr; p.UVb = ly.planes_bwd ? b + ly.UVb : nullptr; p.leafEb = ly.planes ? b + ly.leafEb : nullptr;
  p.UVt_n = b + ly.UVt_n; p.Tt = b + ly.Tt; p.UVt_p = b + ly.UVt_p; p.Et = b + ly.Et;
  p.Tg3 = b + ly.Tg3; p.Eg3 = b + ly.Eg3;
  p.Wn3 = b + ly.Wn3; p.Wp3 = b + ly.Wp3; p.Wtn3 = b + ly.Wtn3; p.Wtp3 = b + ly.Wtp3;
  p.Wn = (float*)(b + ly.Wn); p.Wp = (float*)(b + ly.Wp); p.Wtn = (float*)(b + ly.Wtn); p.Wtp = (float*)(b + ly.Wtp);
  return p;
}

int make_plan(const spcfg_config* cfg, const int32_t* lengths, int B, int n_max, Plan* plan, Layout* ly,
              int gemm_wgs = kGemmWgs) {
  if (!lengths) return SPCFG_ERR_ARG;
  if (B < 1 || B > cfg->max_B || n_max < 2 || n_max > cfg->max_n) return SPCFG_ERR_SHAPE;
  for (int b = 0; b < B; ++b)
    if (lengths[b] < 2 || lengths[b] > n_max) return SPCFG_ERR_LENGTH;
  plan->off.assign(n_max + 2, 0);
  plan->cnt.assign(n_max + 2, 0);
  for (int b = 0; b < B; ++b) {
    plan->lens.v[b] = lengths[b];
    for (int w = 1; w <= lengths[b]; ++w) plan->cnt[w] += lengths[b] - w + 1;
  }
  int64_t run = 0;
  for (int w = 1; w <= n_max + 1; ++w) {
    plan->off[w] = run;
    if (w <= n_max) run += plan->cnt[w];
  }
  const int64_t S1 = plan->cnt[1], Sall = run;
  if (Sall >= (int64_t)1 << 30) return SPCFG_ERR_SHAPE;
  *ly = make_layout(cfg->N, cfg->P, B, n_max, S1, Sall - S1, cfg->precision == SPCFG_PRECISION_BF16,
                    (cfg->flags & SPCFG_FLAG_PER_SENTENCE_GRAMMAR) != 0, (cfg->flags & SPCFG_FLAG_FP32_MFMA) != 0,
                    (cfg->flags & SPCFG_FLAG_BF16_SINGLE_FORWARD) != 0, gemm_wgs);
  return SPCFG_OK;
}

// ---- profiling -------------------------------------------------------------------------------------
// A Scope names the kernel class of the launches made during its lifetime; every such launch gets its own
// start/stop event pair (see launch_k), so a class's time is the sum of its kernels' own durations.
// The counters are process-wide; a mutex guards them, and the class that a thread's launches are charged to is that
// thread's own, so concurrent callers do not corrupt the records (their launches simply add up).
thread_local int t_cur_cls = -1;
struct Prof {
  std::atomic<bool> on{false};
  std::mutex mu;
  struct Rec { hipEvent_t a, b; int cls; };
  std::vector<Rec> recs;
  std::vector<hipEvent_t> pool;
  double work[SPCFG_PROF_CLASSES] = {0};
  int64_t launches[SPCFG_PROF_CLASSES] = {0};
  hipEvent_t get() {
    if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
  void recycle() {
    for (auto& r : recs) { pool.push_back(r.a); pool.push_back(r.b); }
    recs.clear();
  }
} g_prof;

struct Scope {
  int prev;
  Scope(hipStream_t, int c, double work, int nlaunch = 1) : prev(t_cur_cls) {
    if (!g_prof.on) return;
    t_cur_cls = c;
    std::lock_guard<std::mutex> lock(g_prof.mu);
    g_prof.work[c] += work;
    g_prof.launches[c] += nlaunch;
  }
  ~Scope() { t_cur_cls = prev; }
};

}  // namespace

void launch_refused(const char* what) { g_refused = what; }

LaunchEvents prof_launch_events() {
  LaunchEvents ev;
  if (!g_prof.on || t_cur_cls < 0) return ev;
  std::lock_guard<std::mutex> lock(g_prof.mu);
  ev.start = g_prof.get();
  ev.stop = g_prof.get();
  if (!ev.start || !ev.stop) {
    if (ev.start) g_prof.pool.push_back(ev.start);
    if (ev.stop) g_prof.pool.push_back(ev.stop);
    return LaunchEvents{};
  }
  g_prof.recs.push_back({ev.start, ev.stop, t_cur_cls});
  return ev;
}

namespace {

int hip_status() {
  if (g_refused) {
    snprintf(g_hip_err, sizeof(g_hip_err), "%s", g_refused);
    g_refused = nullptr;
    (void)hipGetLastError();
    return SPCFG_ERR_WORKSPACE;
  }
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) return SPCFG_OK;
  snprintf(g_hip_err, sizeof(g_hip_err), "%s", hipGetErrorString(e));
  return SPCFG_ERR_HIP;
}

int check_ws(const Layout& ly, void* ws, size_t bytes) {
  if (!ws) return SPCFG_ERR_ARG;
  if (((uintptr_t)ws & 255) != 0 || bytes < ly.total) return SPCFG_ERR_WORKSPACE;
  return SPCFG_OK;
}

// Shared grammar, fp32, width >= 2: the rows of a width are ordered [prefix spans | middle spans | suffix spans]
// (a span that is both, i.e. a root, counts as prefix).  A prefix span is never a right child and a suffix span
// never a left child, so one of their two projections (forward) resp. one half of their adjoint (reverse, it
// is zero) takes no part: the launch is cut into parts that leave those products out.
struct WidthBlocks { int nP, nM, nS; };
WidthBlocks width_blocks(const Plan& plan, const Layout& ly, int w) {
  WidthBlocks k{0, 0, 0};
  for (int b = 0; b < ly.B; ++b) {
    const int cnt = plan.lens.v[b] - w + 1;
    if (cnt >= 1) ++k.nP;
    if (cnt >= 2) ++k.nS;
    if (cnt >= 3) k.nM += cnt - 2;
  }
  return k;
}
// (the bf16 mode has a kernel with parts for its forward products only)
bool use_parts(const Layout& ly, int w, bool forward_product) {
  return ly.G == 1 && (!ly.bf16 || (forward_product && ly.planes == 2)) && w >= 2;
}
void set_part(NtArgs& a, int i, int row0, int rows, int c0, int kbeg, int kt) {
  a.prt_row0[i] = row0; a.prt_rows[i] = rows; a.prt_c0[i] = c0; a.prt_kbeg[i] = kbeg; a.prt_kt[i] = kt;
}

// One grammar per sentence: the launch for width w multiplies each sentence's rows with that sentence's panel.
void set_groups(NtArgs& a, const Plan& plan, const Layout& ly, const Ptrs& p, int w, int64_t row0, int64_t b_stride) {
  if (ly.G == 1) return;
  a.grouped = 1; a.ngroups = ly.B; a.grp_w = w;
  a.grp_lens = p.lens; a.grp_rowbase = p.rowbase + (size_t)w * ly.B; a.grp_row_first = row0; a.grp_b_stride = b_stride;
  a.grp_tiles_m[0] = a.grp_tiles_m[1] = a.grp_tiles_m[2] = 0;
  a.grp_max_rows = 0;
  for (int b = 0; b < ly.B; ++b) {
    const int cnt = plan.lens.v[b] - w + 1;
    if (cnt <= 0) continue;
    a.grp_tiles_m[0] += (cnt + 31) / 32; a.grp_tiles_m[1] += (cnt + 63) / 64; a.grp_tiles_m[2] += (cnt + 127) / 128;
    if (cnt > a.grp_max_rows) a.grp_max_rows = cnt;
  }
}

int forward(const spcfg_config* cfg, const Plan& plan, const Layout& ly, const Ptrs& p, const float* log_root,
            const float* L, const float* R, const float* log_emit, float* logZ, hipStream_t st) {
  const int n_max = ly.n_max;
  const int64_t Np = ly.Np, Pp = ly.Pp;
  const int fp32_mfma = (cfg->flags & SPCFG_FLAG_FP32_MFMA) ? 1 : 0;
  // width 1: [eta | zeta] = [L_P ; R_P] * emission vector
  NtArgs leaf{};
  leaf.partial = p.partial; leaf.counters = p.counters; leaf.max_wgs = ly.gemm_wgs; leaf.n_counters = ly.n_counters; leaf.b_bf16 = ly.bf16 && !ly.fwd_fp32; leaf.fp32_mfma = fp32_mfma;
  leaf.A = p.leafE; leaf.lda = Pp; leaf.Bm = p.Wp; leaf.ldb = Pp; leaf.C = p.HZ; leaf.ldc = 2 * Np;
  if (ly.bf16 && !ly.fwd_fp32) { leaf.A = p.leafEb; leaf.a_bf16 = 1; }
  if (ly.planes >= 2) {
    leaf.A3 = p.leafEb; leaf.Bm3 = p.Wp3; leaf.planes3 = ly.planes; leaf.a_plane = ly.S1 * Pp; leaf.b_plane = 2 * Np * Pp;
    leaf.a_bf16 = 0; leaf.b_bf16 = 0;
  }
  leaf.rows = (int)ly.S1; leaf.cols = (int)(2 * Np); leaf.K = (int)Pp;
  leaf.epilogue = NT_EPI_ROWSCALE; leaf.rowmaxb = p.tmaxb;
  set_groups(leaf, plan, ly, p, 1, 0, 2 * Np * Pp);
  {
    Scope s(st, SPCFG_PROF_SETUP, 4.0 * 2 * (double)ly.N * (ly.N + ly.P) * 3 + 8.0 * ly.S1 * ly.P, 4);
    launch_plan(ly, p, plan.lens, st);
    if (ly.G > 1) launch_plan_sentrows(ly, p, st);
    launch_pack_weights(ly, p, L, R, st);
    // operand planes are written only for the launches that read them (bf16 mode: all of them)
    launch_leaf_prep(ly, p, log_emit, (ly.bf16 && !ly.fwd_fp32) || gemm_nt_reads_planes(leaf), st);
  }
  {
    Scope s(st, SPCFG_PROF_GEMM_FWD, 4.0 * ly.N * (double)ly.P * ly.S1);
    launch_gemm_nt(leaf, st);
  }
  for (int w = 2; w <= n_max; ++w) {
    const int64_t row0 = plan.off[w], rows = plan.cnt[w];
    if (rows == 0) continue;
    const double split_bytes = 4.0 * ly.N * (double)rows * (2.0 * (w - 1) + 1.0);
    if (w == n_max) {  // every span of the largest width is a root span: never a child, not projected
      Scope s(st, SPCFG_PROF_SPLIT_FWD, split_bytes);
      launch_split_fwd(ly, p, w, row0, rows, false, st);
      break;
    }
    NtArgs a{};
    double skipped = 0.0;
    a.partial = p.partial; a.counters = p.counters; a.max_wgs = ly.gemm_wgs; a.n_counters = ly.n_counters; a.b_bf16 = ly.bf16 && !ly.fwd_fp32; a.fp32_mfma = fp32_mfma;
    a.A = p.T + (row0 - ly.S1) * Np; a.lda = Np; a.Bm = p.Wn; a.ldb = Np;
    if (ly.bf16 && !ly.fwd_fp32) { a.A = static_cast<const uint16_t*>(p.Tb) + (row0 - ly.S1) * Np; a.a_bf16 = 1; }
    if (ly.planes >= 2) {
      a.A3 = static_cast<const uint16_t*>(p.Tb) + (row0 - ly.S1) * Np; a.Bm3 = p.Wn3;
      a.planes3 = ly.planes; a.a_plane = ly.S2 * Np; a.b_plane = 2 * Np * Np;
      a.a_bf16 = 0; a.b_bf16 = 0;
    }
    a.C = p.HZ + row0 * 2 * Np; a.ldc = 2 * Np;
    a.rows = (int)rows; a.cols = (int)(2 * Np); a.K = (int)Np;
    a.epilogue = NT_EPI_ROWSCALE; a.rowmaxb = p.tmaxb + row0;
    // eta for the prefix and middle rows, zeta for the middle and suffix rows (when Np is not a whole number of
    // 128-column tiles the two column blocks would each pad their last tile: one product of 2Np columns then)
    if (use_parts(ly, w, true) && Np % 128 == 0) {
      const WidthBlocks k = width_blocks(plan, ly, w);
      const int kt = (int)(Np / 32);
      // the profile counts the executed flop: one of the two projections is left out for k.nP + k.nS rows
      skipped = 2.0 * ly.N * (double)ly.N * (k.nP + k.nS);
      a.parts = 2; a.cols = (int)Np;
      set_part(a, 0, 0, k.nP + k.nM, 0, 0, kt);
      set_part(a, 1, k.nP, k.nM + k.nS, (int)Np, 0, kt);
    }
    set_groups(a, plan, ly, p, w, row0, 2 * Np * Np);
    {
      Scope s(st, SPCFG_PROF_SPLIT_FWD, split_bytes);
      launch_split_fwd(ly, p, w, row0, rows, (ly.bf16 && !ly.fwd_fp32) || gemm_nt_reads_planes(a), st);
    }
    Scope s(st, SPCFG_PROF_GEMM_FWD, 4.0 * ly.N * (double)ly.N * rows - skipped);
    launch_gemm_nt(a, st);
  }
  {
    Scope s(st, SPCFG_PROF_ROOT, 8.0 * ly.N * ly.B);
    launch_root_fwd(ly, p, log_root, logZ, st);
  }
  (void)cfg;
  return hip_status();
}

int backward(const spcfg_config* cfg, const Plan& plan, const Layout& ly, const Ptrs& p, const float* log_root,
             const float* grad_logZ, float* grad_L, float* grad_R, float* grad_log_root, float* grad_log_emit,
             hipStream_t st) {
  const int n_max = ly.n_max;
  const int64_t Np = ly.Np, Pp = ly.Pp;
  const int fp32_mfma = (cfg->flags & SPCFG_FLAG_FP32_MFMA) ? 1 : 0;
  const int acc = (cfg->flags & SPCFG_FLAG_ACCUMULATE_GRADS) ? 1 : 0;
  {
    Scope s(st, SPCFG_PROF_ROOT, 16.0 * ly.N * ly.B, 3);
    launch_root_bwd(ly, p, log_root, grad_logZ, grad_log_root, acc, st);
    launch_zero_pad_emit(ly, p, grad_log_emit, st);
  }
  for (int w = n_max - 1; w >= 1; --w) {  // spans of width n_max are all roots
    const int64_t row0 = plan.off[w], rows = plan.cnt[w];
    if (rows == 0) continue;
    // per span: (n - w) terms, two vector reads each, plus the two output vectors
    double terms = 0;
    for (int b = 0; b < ly.B; ++b) {
      const int n = plan.lens.v[b];
      if (n > w) terms += (double)(n - w + 1) * (n - w);
    }
    const double split_bytes = 4.0 * ly.N * (2.0 * terms + 2.0 * rows);  // reads + the two output vectors
    NtArgs a{};
    double gemm_flop;
    a.partial = p.partial; a.counters = p.counters; a.max_wgs = ly.gemm_wgs; a.n_counters = ly.n_counters; a.b_bf16 = ly.bf16; a.fp32_mfma = fp32_mfma;
    a.A = p.UV + row0 * 2 * Np; a.lda = 2 * Np; a.K = (int)(2 * Np); a.rows = (int)rows;
    if (ly.bf16) { a.A = static_cast<const uint16_t*>(p.UVb) + row0 * 2 * Np; a.a_bf16 = 1; }
    if (ly.planes_bwd == 3) {
      a.A3 = static_cast<const uint16_t*>(p.UVb) + row0 * 2 * Np; a.Bm3 = w >= 2 ? p.Wtn3 : p.Wtp3;
      a.planes3 = 3; a.a_plane = ly.uvb_plane; a.b_plane = 2 * Np * (w >= 2 ? Np : Pp);
    }
    if (w >= 2) {
      gemm_flop = 4.0 * ly.N * (double)ly.N * rows;
      a.Bm = p.Wtn; a.ldb = 2 * Np; a.C = p.BH + (row0 - ly.S1) * Np; a.ldc = Np; a.cols = (int)Np;
      a.epilogue = NT_EPI_MASKROWS; a.rowmask = p.rootmask + row0; a.rowmaxb = p.umaxb + row0;
      if (use_parts(ly, w, false)) {  // prefix rows: only the eta adjoint (first half of K); suffix rows: only zeta's
        const WidthBlocks k = width_blocks(plan, ly, w);
        const int kt = (int)(Np / 32);
        a.parts = 3;
        set_part(a, 0, 0, k.nP, 0, 0, kt);
        set_part(a, 1, k.nP, k.nM, 0, 0, 2 * kt);
        set_part(a, 2, k.nP + k.nM, k.nS, 0, kt, kt);
        // (the profile counts the executed flop)
        if (gemm_nt_keep_parts(a)) gemm_flop -= 2.0 * ly.N * (double)ly.N * (k.nP + k.nS);
      }
      set_groups(a, plan, ly, p, w, row0, 2 * Np * Np);
    } else {
      gemm_flop = 4.0 * ly.N * (double)ly.P * rows;
      a.Bm = p.Wtp; a.ldb = 2 * Np; a.C = grad_log_emit; a.ldc = ly.P; a.cols = ly.P;
      a.epilogue = NT_EPI_LEAF_EMIT; a.E = p.leafE; a.lde = Pp; a.rowexp = p.uexp;
      a.row_b = p.row_b; a.row_i = p.row_i; a.n_max = n_max;
      set_groups(a, plan, ly, p, 1, 0, 2 * Np * Pp);
    }
    {
      Scope s(st, SPCFG_PROF_SPLIT_BWD, split_bytes);
      // (the rule-gradient product on planes reads the adjoint planes of every row)
      launch_split_bwd(ly, p, w, row0, rows, ly.bf16 || (ly.tn3 && !fp32_mfma) || gemm_nt_reads_planes(a), st);
    }
    {
      Scope s(st, SPCFG_PROF_GEMM_BWD, gemm_flop);
      launch_gemm_nt(a, st);
    }
  }
  {
    // (launches of the class: the two products, plus what prepares their operands: planes or transposes)
    Scope s(st, SPCFG_PROF_GEMM_GRAD, 4.0 * ly.N * ((double)ly.N * ly.S2 + (double)ly.P * ly.S1),
            (ly.tn3 && !fp32_mfma && ly.G == 1) ? 5 : ((ly.bf16 && ly.G == 1) ? 6 : 2));
    if (ly.G > 1) {
      // one reduction per sentence over its own spans of width >= 2 (listed in sentrows), one over its leaves
      int n_longest = 2;
      for (int b = 0; b < ly.B; ++b) n_longest = plan.lens.v[b] > n_longest ? plan.lens.v[b] : n_longest;
      TnArgs t{};
      t.fp32_mfma = fp32_mfma;
      t.Np = (int)Np; t.N = ly.N; t.gL = grad_L; t.gR = grad_R; t.ldg = ly.N + ly.P; t.accumulate = acc;
      t.ngroups = ly.B; t.grp_lens = p.lens; t.grp_gstride = (int64_t)ly.N * (ly.N + ly.P);
      t.A = p.UV; t.lda = 2 * Np; t.sc = p.gsc;
      t.grp_mode = 1; t.rowlist = p.sentrows; t.grp_off = p.sentoff; t.brow0 = ly.S1;
      t.Bm = p.T; t.ldb = Np; t.cols = ly.N; t.col0 = 0;
      t.grp_kt_max = (int)(((int64_t)n_longest * (n_longest - 1) / 2 + 31) / 32);
      launch_gemm_tn(t, st);
      t.grp_mode = 2; t.grp_base = p.rowbase + ly.B;  // first leaf row of every sentence
      t.Bm = p.leafE; t.ldb = Pp; t.cols = ly.P; t.col0 = ly.N;
      t.grp_kt_max = (n_longest + 31) / 32;
      launch_gemm_tn(t, st);
    } else if (ly.tn3 && !fp32_mfma) {
      // on planes: the adjoint rows as their producers cut them, the inside vectors times the span scale cut here
      launch_scaled_planes(p.T, Np, p.gsc + ly.S1, ly.S2, ly.S2p32, p.Tg3, ly.S2p32 * Np, st);
      launch_scaled_planes(p.leafE, Pp, p.gsc, ly.S1, ly.S1p32, p.Eg3, ly.S1p32 * Pp, st);
      launch_zero_plane_rows(p.UVb, ly.uvb_plane, 2 * Np, ly.Sall, 32, st);
      Tn3Args t{};
      t.partial = p.partial; t.counters = p.counters; t.max_wgs = ly.gemm_wgs; t.n_counters = ly.n_counters;
      t.Np = (int)Np; t.N = ly.N; t.gL = grad_L; t.gR = grad_R; t.ldg = ly.N + ly.P; t.accumulate = acc;
      t.a_plane = ly.uvb_plane; t.lda = 2 * Np;
      t.A3 = static_cast<const uint16_t*>(p.UVb) + ly.S1 * 2 * Np; t.B3 = static_cast<const uint16_t*>(p.Tg3);
      t.b_plane = ly.S2p32 * Np; t.ldb = Np; t.KT = (int)(ly.S2p32 / 32); t.cols = ly.N; t.col0 = 0;
      launch_gemm_tn3(t, st);
      t.A3 = static_cast<const uint16_t*>(p.UVb); t.B3 = static_cast<const uint16_t*>(p.Eg3);
      t.b_plane = ly.S1p32 * Pp; t.ldb = Pp; t.KT = (int)(ly.S1p32 / 32); t.cols = ly.P; t.col0 = ly.N;
      launch_gemm_tn3(t, st);
    } else if (!ly.bf16) {
      TnArgs t{};
      t.fp32_mfma = fp32_mfma;
      t.partial = p.partial; t.counters = p.counters; t.max_wgs = ly.gemm_wgs; t.n_counters = ly.n_counters;
      t.Np = (int)Np; t.N = ly.N; t.gL = grad_L; t.gR = grad_R; t.ldg = ly.N + ly.P; t.accumulate = acc;
      t.A = p.UV + ly.S1 * 2 * Np; t.lda = 2 * Np; t.Bm = p.T; t.ldb = Np; t.sc = p.gsc + ly.S1; t.S = ly.S2;
      t.cols = ly.N; t.col0 = 0;
      launch_gemm_tn(t, st);
      t.A = p.UV; t.Bm = p.leafE; t.ldb = Pp; t.sc = p.gsc; t.S = ly.S1; t.cols = ly.P; t.col0 = ly.N;
      launch_gemm_tn(t, st);
    } else {
      // both operands transposed to bf16 (span scale folded into the adjoint rows), then the NT kernel
      launch_transpose_bf16(p.UV + ly.S1 * 2 * Np, 2 * Np, (int)(2 * Np), p.gsc + ly.S1, ly.S2, ly.S2pad, p.UVt_n, st);
      launch_transpose_bf16(p.T, Np, (int)Np, nullptr, ly.S2, ly.S2pad, p.Tt, st);
      launch_transpose_bf16(p.UV, 2 * Np, (int)(2 * Np), p.gsc, ly.S1, ly.S1pad, p.UVt_p, st);
      launch_transpose_bf16(p.leafE, Pp, (int)Pp, nullptr, ly.S1, ly.S1pad, p.Et, st);
      NtArgs a{};
      a.partial = p.partial; a.counters = p.counters; a.max_wgs = ly.gemm_wgs; a.n_counters = ly.n_counters; a.a_bf16 = 1; a.b_bf16 = 1;
      a.epilogue = NT_EPI_GRAD; a.gL = grad_L; a.gR = grad_R; a.ldg = ly.N + ly.P; a.Np = (int)Np; a.Nvalid = ly.N;
      a.accumulate = acc; a.rows = (int)(2 * Np);
      a.A = p.UVt_n; a.lda = ly.S2pad; a.Bm = p.Tt; a.ldb = ly.S2pad; a.K = (int)ly.S2pad; a.cols = ly.N; a.col0 = 0;
      launch_gemm_nt(a, st);
      a.A = p.UVt_p; a.lda = ly.S1pad; a.Bm = p.Et; a.ldb = ly.S1pad; a.K = (int)ly.S1pad; a.cols = ly.P; a.col0 = ly.N;
      launch_gemm_nt(a, st);
    }
  }
  return hip_status();
}

}  // namespace
}  // namespace spcfg

using namespace spcfg;

// ---- static device scratch for the entry point that allocates nothing ---------------------------------------
// One array per GPU (every device that loads the library's code object holds its own copy at its own address).
// In host code the array's name only stands for the symbol: the device address comes from hipGetSymbolAddress,
// once per device, and that pointer is what the kernels get.
#ifndef SPCFG_HOST_CHECKS_BUILD  // (the host-only build of tests/sanitize has no device code object to hold it)
static __device__ __align__(256) unsigned char scratch[SPCFG_STATIC_SCRATCH_BYTES];
#endif

namespace {
constexpr int kStaticGemmWgs = 64;   // partial-tile scratch of the static buffer: 2 * 64 slots of 64 KiB = 8 MiB
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {nullptr};
std::mutex g_scratch_mutex;

// Device address of this device's copy of `scratch` (looked up on the first call on a device, with that device
// current), or nullptr with the HIP error text recorded.
void* static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    snprintf(g_hip_err, sizeof(g_hip_err), "no current HIP device below %d", kMaxDevices);
    (void)hipGetLastError();
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
#ifndef SPCFG_HOST_CHECKS_BUILD
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
#else
    const hipError_t e = hipErrorNotSupported;
#endif
    if (e != hipSuccess || !ptr) {
      snprintf(g_hip_err, sizeof(g_hip_err), "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
      (void)hipGetLastError();
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

extern "C" {

int spcfg_inside_static(const spcfg_config* cfg, const float* log_root, const float* L, const float* R,
                        const float* log_emit, const int32_t* lengths, int32_t B, int32_t n_max, float* logZ,
                        void* hip_stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if (!log_root || !L || !R || !log_emit || !logZ) return SPCFG_ERR_ARG;
  Plan plan; Layout ly;
  rc = make_plan(cfg, lengths, B, n_max, &plan, &ly, kStaticGemmWgs);
  if (rc) return rc;
  if (ly.total > (size_t)SPCFG_STATIC_SCRATCH_BYTES) return SPCFG_ERR_STATIC_CAPACITY;
  void* ws = static_scratch();
  if (!ws) return SPCFG_ERR_HIP;
  return forward(cfg, plan, ly, resolve(ly, ws), log_root, L, R, log_emit, logZ, (hipStream_t)hip_stream);
}

int spcfg_workspace_bytes(const spcfg_config* cfg, size_t* out_bytes) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if (!out_bytes) return SPCFG_ERR_ARG;
  const int64_t S1 = (int64_t)cfg->max_B * cfg->max_n;
  const int64_t Sall = (int64_t)cfg->max_B * cfg->max_n * (cfg->max_n + 1) / 2;
  if (Sall >= (int64_t)1 << 30) return SPCFG_ERR_SHAPE;
  *out_bytes = make_layout(cfg->N, cfg->P, cfg->max_B, cfg->max_n, S1, Sall - S1,
                           cfg->precision == SPCFG_PRECISION_BF16,
                           (cfg->flags & SPCFG_FLAG_PER_SENTENCE_GRAMMAR) != 0,
                           (cfg->flags & SPCFG_FLAG_FP32_MFMA) != 0,
                           (cfg->flags & SPCFG_FLAG_BF16_SINGLE_FORWARD) != 0).total;
  return SPCFG_OK;
}

int spcfg_workspace_bytes_for(const spcfg_config* cfg, const int32_t* lengths, int32_t B, int32_t n_max,
                              size_t* out_bytes) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if (!out_bytes) return SPCFG_ERR_ARG;
  Plan plan; Layout ly;
  rc = make_plan(cfg, lengths, B, n_max, &plan, &ly);
  if (rc) return rc;
  *out_bytes = ly.total;
  return SPCFG_OK;
}

int spcfg_inside(const spcfg_config* cfg, const float* log_root, const float* L, const float* R,
                 const float* log_emit, const int32_t* lengths, int32_t B, int32_t n_max, float* logZ,
                 void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if (!log_root || !L || !R || !log_emit || !logZ) return SPCFG_ERR_ARG;
  Plan plan; Layout ly;
  rc = make_plan(cfg, lengths, B, n_max, &plan, &ly);
  if (rc) return rc;
  rc = check_ws(ly, workspace, workspace_bytes);
  if (rc) return rc;
  return forward(cfg, plan, ly, resolve(ly, workspace), log_root, L, R, log_emit, logZ, (hipStream_t)hip_stream);
}

int spcfg_inside_backward(const spcfg_config* cfg, const float* log_root, const float* L, const float* R,
                          const float* log_emit, const int32_t* lengths, int32_t B, int32_t n_max,
                          const float* grad_logZ, float* grad_L, float* grad_R, float* grad_log_root,
                          float* grad_log_emit, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if (!log_root || !L || !R || !log_emit || !grad_L || !grad_R || !grad_log_root || !grad_log_emit)
    return SPCFG_ERR_ARG;
  Plan plan; Layout ly;
  rc = make_plan(cfg, lengths, B, n_max, &plan, &ly);
  if (rc) return rc;
  rc = check_ws(ly, workspace, workspace_bytes);
  if (rc) return rc;
  return backward(cfg, plan, ly, resolve(ly, workspace), log_root, grad_logZ, grad_L, grad_R, grad_log_root,
                  grad_log_emit, (hipStream_t)hip_stream);
}

int spcfg_inside_forward_backward(const spcfg_config* cfg, const float* log_root, const float* L,
                                  const float* R, const float* log_emit, const int32_t* lengths, int32_t B,
                                  int32_t n_max, const float* grad_logZ, float* logZ, float* grad_L,
                                  float* grad_R, float* grad_log_root, float* grad_log_emit, void* workspace,
                                  size_t workspace_bytes, void* hip_stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if (!log_root || !L || !R || !log_emit || !logZ || !grad_L || !grad_R || !grad_log_root || !grad_log_emit)
    return SPCFG_ERR_ARG;
  Plan plan; Layout ly;
  rc = make_plan(cfg, lengths, B, n_max, &plan, &ly);
  if (rc) return rc;
  rc = check_ws(ly, workspace, workspace_bytes);
  if (rc) return rc;
  const Ptrs p = resolve(ly, workspace);
  rc = forward(cfg, plan, ly, p, log_root, L, R, log_emit, logZ, (hipStream_t)hip_stream);
  if (rc) return rc;
  return backward(cfg, plan, ly, p, log_root, grad_logZ, grad_L, grad_R, grad_log_root, grad_log_emit,
                  (hipStream_t)hip_stream);
}

int spcfg_span_marginals(const spcfg_config* cfg, const int32_t* lengths, int32_t B, int32_t n_max,
                         const void* workspace, size_t workspace_bytes, float* span_post, int32_t* span_label,
                         void* hip_stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if (!span_post) return SPCFG_ERR_ARG;
  Plan plan; Layout ly;
  rc = make_plan(cfg, lengths, B, n_max, &plan, &ly);
  if (rc) return rc;
  rc = check_ws(ly, const_cast<void*>(workspace), workspace_bytes);
  if (rc) return rc;
  launch_span_marginals(ly, resolve(ly, const_cast<void*>(workspace)), span_post, span_label, (hipStream_t)hip_stream);
  return hip_status();
}

const char* spcfg_strerror(int code) {
  switch (code) {
    case SPCFG_OK: return "ok";
    case SPCFG_ERR_ARG: return "invalid argument (null pointer or bad struct_size)";
    case SPCFG_ERR_SHAPE: return "shape out of range or above the configured capacity";
    case SPCFG_ERR_LENGTH: return "sentence length below 2 or above n_max";
    case SPCFG_ERR_WORKSPACE: return "workspace misaligned or too small";
    case SPCFG_ERR_UNSUPPORTED: return "precision or flag not supported";
    case SPCFG_ERR_HIP: return "HIP runtime error";
    case SPCFG_ERR_STATIC_CAPACITY: return "batch needs more scratch than the static device buffer of spcfg_inside_static holds";
    default: return "unknown error code";
  }
}

const char* spcfg_last_hip_error(void) { return g_hip_err; }

int spcfg_profile_enable(int on) {
  std::lock_guard<std::mutex> lock(g_prof.mu);
  g_prof.on = on != 0;
  if (g_prof.on) {
    g_prof.recycle();
    for (int c = 0; c < SPCFG_PROF_CLASSES; ++c) { g_prof.work[c] = 0; g_prof.launches[c] = 0; }
  }
  return SPCFG_OK;
}

int spcfg_profile_read(double* ms, int64_t* launches, double* work) {
  if (!ms || !launches || !work) return SPCFG_ERR_ARG;
  std::lock_guard<std::mutex> lock(g_prof.mu);
  for (int c = 0; c < SPCFG_PROF_CLASSES; ++c) ms[c] = 0.0;
  int rc = SPCFG_OK;
  for (auto& r : g_prof.recs) {
    float t = 0.0f;
    if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&t, r.a, r.b) != hipSuccess) rc = SPCFG_ERR_HIP;
    ms[r.cls] += t;
  }
  g_prof.recycle();
  for (int c = 0; c < SPCFG_PROF_CLASSES; ++c) {
    launches[c] = g_prof.launches[c];
    work[c] = g_prof.work[c];
    g_prof.launches[c] = 0;
    g_prof.work[c] = 0;
  }
  return rc;
}

const char* spcfg_profile_class_name(int cls) {
  static const char* names[SPCFG_PROF_CLASSES] = {"setup", "gemm_fwd", "split_fwd", "root", "split_bwd", "gemm_bwd",
                                                  "gemm_grad"};
  return (cls >= 0 && cls < SPCFG_PROF_CLASSES) ? names[cls] : "?";
}

}  // extern "C"
