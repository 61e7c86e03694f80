// Host-side checks of the C ABI under AddressSanitizer / UBSan (no GPU, kernel launchers stubbed): every argument
// check of tests/test_abi.py, workspace queries over a range of shapes, and dry runs of the whole schedule.
#include <cstdio>
#include <cstdlib>
#include <vector>
#include "../../include/spcfg.h"
namespace spcfg { long stub_launch_count(); }
#define EXPECT(cond) do { if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); return 1; } } while (0)
int main() {
  void* fake = (void*)4096;
  const float* ff = (const float*)fake; float* fm = (float*)fake;
  spcfg_config cfg{sizeof(spcfg_config), 8, 8, 4, 6, SPCFG_PRECISION_FP32, 0};
  size_t bytes = 0;
  EXPECT(spcfg_workspace_bytes(&cfg, &bytes) == 0 && bytes > 0);
  EXPECT(spcfg_workspace_bytes(nullptr, &bytes) == SPCFG_ERR_ARG);
  EXPECT(spcfg_workspace_bytes(&cfg, nullptr) == SPCFG_ERR_ARG);
  { spcfg_config c = cfg; c.N = 0; EXPECT(spcfg_workspace_bytes(&c, &bytes) == SPCFG_ERR_SHAPE); }
  { spcfg_config c = cfg; c.max_B = 5000; EXPECT(spcfg_workspace_bytes(&c, &bytes) == SPCFG_ERR_SHAPE); }
  { spcfg_config c = cfg; c.precision = 7; EXPECT(spcfg_workspace_bytes(&c, &bytes) == SPCFG_ERR_UNSUPPORTED); }
  { spcfg_config c = cfg; c.flags = 64; EXPECT(spcfg_workspace_bytes(&c, &bytes) == SPCFG_ERR_UNSUPPORTED); }
  { spcfg_config c = cfg; c.struct_size = 4; EXPECT(spcfg_workspace_bytes(&c, &bytes) == SPCFG_ERR_ARG); }
  int32_t lens2[2] = {3, 4};
  EXPECT(spcfg_workspace_bytes_for(&cfg, lens2, 2, 6, &bytes) == 0);
  { int32_t bad[2] = {1, 3}; EXPECT(spcfg_workspace_bytes_for(&cfg, bad, 2, 6, &bytes) == SPCFG_ERR_LENGTH); }
  { int32_t bad[2] = {7, 3}; EXPECT(spcfg_workspace_bytes_for(&cfg, bad, 2, 6, &bytes) == SPCFG_ERR_LENGTH); }
  EXPECT(spcfg_workspace_bytes_for(&cfg, lens2, 2, 9, &bytes) == SPCFG_ERR_SHAPE);
  EXPECT(spcfg_inside(&cfg, nullptr, nullptr, nullptr, nullptr, lens2, 2, 6, nullptr, nullptr, 0, nullptr) == SPCFG_ERR_ARG);
  EXPECT(spcfg_inside(&cfg, ff, ff, ff, ff, lens2, 2, 6, fm, nullptr, 0, nullptr) == SPCFG_ERR_ARG);
  EXPECT(spcfg_inside(&cfg, ff, ff, ff, ff, lens2, 2, 6, fm, (void*)256, 16, nullptr) == SPCFG_ERR_WORKSPACE);
  EXPECT(spcfg_inside(&cfg, ff, ff, ff, ff, lens2, 2, 6, fm, (void*)100, (size_t)1 << 40, nullptr) == SPCFG_ERR_WORKSPACE);
  EXPECT(spcfg_inside_static(&cfg, nullptr, ff, ff, ff, lens2, 2, 6, fm, nullptr) == SPCFG_ERR_ARG);
  { spcfg_config big{sizeof(spcfg_config), 2048, 2048, 64, 40, 0, 0}; std::vector<int32_t> full(64, 40);
    EXPECT(spcfg_inside_static(&big, ff, ff, ff, ff, full.data(), 64, 40, fm, nullptr) == SPCFG_ERR_STATIC_CAPACITY); }
  for (int c = -9; c < 2; ++c) EXPECT(spcfg_strerror(c) != nullptr && spcfg_strerror(c)[0] != 0);
  // dry runs of the whole schedule (the launchers are no-ops; the "device" pointers are never dereferenced)
  const long before = spcfg::stub_launch_count();
  int runs = 0;
  for (int precision = 0; precision < 2; ++precision)
    for (unsigned flags : {0u, 2u, 4u, 1u | 2u | 4u})
      for (int shape = 0; shape < 5; ++shape) {
        std::vector<int32_t> lens;
        int N = 30, P = 60;
        if (shape == 0) lens = {2};
        if (shape == 1) lens = {10, 3, 7, 2, 9, 5};
        if (shape == 2) { lens.assign(960, 3); lens[7] = 5; N = 5; P = 6; }
        if (shape == 3) { lens = {1024}; N = 4; P = 7; }
        if (shape == 4) { lens.assign(64, 40); lens[3] = 2; N = 2048; P = 2048; }
        int n_max = 0; for (int x : lens) n_max = x > n_max ? x : n_max;
        spcfg_config c{sizeof(spcfg_config), N, P, (int32_t)lens.size(), n_max, precision, flags};
        size_t need = 0, cap = 0;
        EXPECT(spcfg_workspace_bytes_for(&c, lens.data(), (int32_t)lens.size(), n_max, &need) == 0);
        EXPECT(spcfg_workspace_bytes(&c, &cap) == 0 && need <= cap);
        const int rc = spcfg_inside_forward_backward(&c, ff, ff, ff, ff, lens.data(), (int32_t)lens.size(), n_max, nullptr, fm, fm, fm, fm,
                                                     fm, (void*)(size_t)(1 << 20), need, nullptr);
        EXPECT(rc == SPCFG_OK || rc == SPCFG_ERR_HIP);  // without a GPU the runtime's last-error query may report one
        EXPECT(spcfg_span_marginals(&c, lens.data(), (int32_t)lens.size(), n_max, (void*)(size_t)(1 << 20), need, fm, nullptr, nullptr) != SPCFG_ERR_ARG);
        ++runs;
      }
  EXPECT(spcfg::stub_launch_count() - before > 100);
  printf("host checks passed: %d dry runs, %ld stubbed launches\n", runs, spcfg::stub_launch_count() - before);
  return 0;
}
