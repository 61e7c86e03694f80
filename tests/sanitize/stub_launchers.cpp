// Kernel launchers replaced by no-ops: lets the host side of the library (argument checks, workspace layout, span
// plan, the width-synchronous schedule of both passes) run under AddressSanitizer / UBSan without a GPU.
#include "spcfg_internal.h"
namespace spcfg {
static long g_launches = 0;
long stub_launch_count() { return g_launches; }
void launch_plan(const Layout&, const Ptrs&, const LenArg&, hipStream_t) { ++g_launches; }
void launch_plan_sentrows(const Layout&, const Ptrs&, hipStream_t) { ++g_launches; }
void launch_pack_weights(const Layout&, const Ptrs&, const float*, const float*, hipStream_t) { ++g_launches; }
void launch_transpose_bf16(const float*, int64_t, int, const float*, int64_t, int64_t, void*, hipStream_t) { ++g_launches; }
void launch_leaf_prep(const Layout&, const Ptrs&, const float*, bool, hipStream_t) { ++g_launches; }
void launch_split_fwd(const Layout&, const Ptrs&, int, int64_t, int64_t, bool, hipStream_t) { ++g_launches; }
void launch_root_fwd(const Layout&, const Ptrs&, const float*, float*, hipStream_t) { ++g_launches; }
void launch_root_bwd(const Layout&, const Ptrs&, const float*, const float*, float*, int, hipStream_t) { ++g_launches; }
void launch_split_bwd(const Layout&, const Ptrs&, int, int64_t, int64_t, bool, hipStream_t) { ++g_launches; }
void launch_zero_pad_emit(const Layout&, const Ptrs&, float*, hipStream_t) { ++g_launches; }
void launch_span_marginals(const Layout&, const Ptrs&, float*, int32_t*, hipStream_t) { ++g_launches; }
void launch_gemm_nt(const NtArgs& a, hipStream_t) {
  // what the real launcher relies on: parts lie inside the launch's rows
  for (int p = 0; p < a.parts; ++p)
    if (a.prt_row0[p] < 0 || a.prt_rows[p] < 0 || a.prt_row0[p] + a.prt_rows[p] > a.rows) __builtin_trap();
  ++g_launches;
}
void launch_gemm_tn(const TnArgs&, hipStream_t) { ++g_launches; }
void launch_gemm_tn3(const Tn3Args& a, hipStream_t) { if (a.KT < 0) __builtin_trap(); ++g_launches; }
void launch_scaled_planes(const float*, int64_t, const float*, int64_t S, int64_t Srows, void*, int64_t, hipStream_t) {
  if (Srows < S || Srows % 32 != 0) __builtin_trap();  // the product reads whole 32-row steps
  ++g_launches;
}
void launch_zero_plane_rows(void*, int64_t, int64_t, int64_t, int64_t, hipStream_t) { ++g_launches; }
bool gemm_nt_keep_parts(NtArgs& a) { return a.parts != 0; }
bool gemm_nt_reads_planes(const NtArgs& a) { return a.planes3 != 0 && a.rows >= 380; }
int gemm_nt_tiles(int rows, int cols) { return ((rows + 31) / 32) * ((cols + 127) / 128); }
size_t gemm_nt_partial_bytes(int max_wgs) { return (size_t)2 * max_wgs * 128 * 128 * 4; }
}  // namespace spcfg
