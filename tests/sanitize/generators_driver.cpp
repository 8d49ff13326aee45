// Walks every entry point of the workload generators on small sizes; built with
// -fsanitize=address,undefined by tests/test_sanitizers.py, which fails on any report.
#include "../../workloads/gen.cpp"

#include <cstdio>
#include <vector>

static int export_and_check(wl_pattern* p, const char* what) {
  if (!p) { std::printf("%s: no pattern\n", what); return 1; }
  const int64_t nr = wl_pattern_rows(p), nc = wl_pattern_cols(p), nnz = wl_pattern_nnz(p);
  std::vector<int32_t> rp((size_t)nr + 1), ci((size_t)nnz + 1);
  if (wl_pattern_export(p, rp.data(), ci.data()) != 0) { std::printf("%s: export failed\n", what); return 1; }
  wl_pattern_free(p);
  if (rp[0] != 0 || rp[(size_t)nr] != nnz) { std::printf("%s: bad offsets\n", what); return 1; }
  for (int64_t i = 0; i < nr; ++i)
    for (int32_t k = rp[(size_t)i]; k < rp[(size_t)i + 1]; ++k) {
      if (ci[(size_t)k] < 0 || ci[(size_t)k] >= nc) { std::printf("%s: column out of range\n", what); return 1; }
      if (k > rp[(size_t)i] && ci[(size_t)k] <= ci[(size_t)k - 1]) { std::printf("%s: row not ascending\n", what); return 1; }
    }
  return 0;
}

int main() {
  int bad = 0;
  bad += export_and_check(wl_erdos_renyi(500, 16.0 / 499.0, 0x6D670001ull), "erdos_renyi");
  bad += export_and_check(wl_chung_lu(3000, 60e3, 2.1, 700.0, 1, 3), "chung_lu relabelled");
  bad += export_and_check(wl_chung_lu(1000, 9e3, 2.3, 300.0, 0, 4), "chung_lu degree order");
  bad += export_and_check(wl_rmat(10, 8000, 0.57, 0.19, 0.19, 5), "rmat");
  bad += export_and_check(wl_row_block(700, 5000, 9000.0, 2.5, 300.0, 1.6, 6), "row_block");
  std::vector<float> f(1001);
  wl_normal_f32(7, 1, 12345, (int64_t)f.size(), f.data());
  wl_uniform_f32(7, 2, 0, (int64_t)f.size(), -0.25, 0.25, f.data());
  std::vector<int32_t> l(777);
  wl_labels_i32(7, 3, (int64_t)l.size(), 41, l.data());
  for (int32_t x : l) bad += (x < 0 || x >= 41);
  if (bad) { std::printf("generator walk failed\n"); return 1; }
  std::printf("generator walk ok\n");
  return 0;
}
