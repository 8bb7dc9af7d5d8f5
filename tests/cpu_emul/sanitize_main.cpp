// Test infrastructure: the library's kernels in the host-thread build, run under AddressSanitizer and
// UndefinedBehaviorSanitizer on two small cases (fixed thresholds, then a budget). No oracle here: the run must be
// clean and the member counts must add up; tests/test_cpu_emulation.py compares the same build with the oracle.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/sttm.h"

static uint32_t g_state = 12345u;
static float rnd() {  // small deterministic generator of values in [-1, 1)
  g_state = g_state * 1664525u + 1013904223u;
  return (float)((g_state >> 8) & 0xffff) / 32768.f - 1.f;
}

static int run_case(int B, int T, int H, int W, int D, int dtype, bool budget, int cell_dots, int order) {
  const int N = B * T * H * W;
  sttm_ctx* c = nullptr;
  if (sttm_create(&c, 0, nullptr) != STTM_OK) return 10;
  sttm_set_cell_dots(c, cell_dots);
  sttm_set_output_order(c, order);
  const size_t need = sttm_workspace_bytes(B, T, H, W, D, dtype, 1);
  // exact-size heap blocks: a store one byte past any of them is an error the sanitizer reports
  void* ws = nullptr;
  if (posix_memalign(&ws, 256, need)) return 11;
  memset(ws, 0xA5, need);
  if (sttm_set_workspace(c, ws, need) != STTM_OK) return 12;
  const size_t esz = dtype == STTM_F32 ? 4 : 2;
  void* x = nullptr;
  if (posix_memalign(&x, 16, (size_t)N * D * esz)) return 13;
  // blocks of 2x2 cells share a base vector, so that something merges
  std::vector<float> base((size_t)B * T * ((H + 1) / 2) * ((W + 1) / 2) * D);
  for (auto& v : base) v = rnd();
  for (int i = 0; i < N; ++i) {
    const int f = i / (H * W), cell = i % (H * W), y = cell / W, xx = cell % W;
    const size_t bi = ((size_t)(f / 2) * ((H + 1) / 2) + y / 2) * ((W + 1) / 2) + xx / 2;  // frames pair up too
    for (int d = 0; d < D; ++d) {
      const float v = base[(bi % (base.size() / D)) * D + d] + 0.05f * rnd();
      if (dtype == STTM_F32) {
        ((float*)x)[(size_t)i * D + d] = v;
      } else {
        uint32_t u;
        memcpy(&u, &v, 4);
        ((uint16_t*)x)[(size_t)i * D + d] = (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
      }
    }
  }
  std::vector<int32_t> node_map(N), cluster(N), counts(N), out_ids(N), survived(N), reassigned(N), tyxl(4 * (size_t)N);
  std::vector<uint8_t> level(N);
  std::vector<float> mpos(N);
  std::vector<int64_t> offsets(B + 1);
  void* merged = nullptr;
  if (posix_memalign(&merged, 16, (size_t)N * D * esz)) return 14;
  std::vector<float> tau(B, 0.8f);
  std::vector<double> keep(B, 0.5);
  int rc;
  if (budget) {
    rc = sttm_spatial_stats(c, x, dtype, B, T, H, W, D, 1);
    if (!rc) rc = sttm_budget_threshold(c, STTM_STAGE_SPATIAL, keep.data(), nullptr);
    if (!rc) rc = sttm_spatial_quadtree(c, x, dtype, B, T, H, W, D, 1, nullptr, node_map.data(), level.data());
    if (!rc) rc = sttm_temporal_stats(c, x, node_map.data(), level.data());
    if (!rc) rc = sttm_budget_threshold(c, STTM_STAGE_TEMPORAL, keep.data(), tau.data());
    if (!rc) rc = sttm_temporal_merge(c, x, node_map.data(), level.data(), nullptr, cluster.data());
  } else {
    rc = sttm_spatial_quadtree(c, x, dtype, B, T, H, W, D, 1, tau.data(), node_map.data(), level.data());
    if (!rc) rc = sttm_temporal_merge(c, x, node_map.data(), level.data(), tau.data(), cluster.data());
  }
  int64_t K = -1;
  if (!rc)
    rc = sttm_reduce(c, x, cluster.data(), node_map.data(), level.data(), dtype, N, merged, counts.data(), out_ids.data(),
                     offsets.data(), &K);
  if (!rc)
    rc = sttm_positions(c, cluster.data(), node_map.data(), level.data(), offsets.data(), N, survived.data(),
                        reassigned.data(), mpos.data(), tyxl.data());
  if (rc) {
    fprintf(stderr, "status %d: %s\n", rc, sttm_last_error(c));
    return 20 + rc;
  }
  if (!rc) {  // the reduce stage for callers that cannot allocate: same rows, bit for bit
    std::vector<int32_t> counts2(N), ids2(N);
    std::vector<int64_t> off2(B + 1);
    void* merged2 = nullptr;
    if (posix_memalign(&merged2, 16, (size_t)N * D * esz)) return 15;
    rc = sttm_reduce_noalloc(c, x, dtype, B, T, H, W, D, cluster.data(), dtype, N, merged2, counts2.data(), ids2.data(),
                             off2.data());
    if (!rc && (off2[B] != K || memcmp(merged, merged2, (size_t)K * D * esz) ||
                memcmp(counts.data(), counts2.data(), (size_t)K * 4) || memcmp(out_ids.data(), ids2.data(), (size_t)K * 4))) {
      fprintf(stderr, "sttm_reduce_noalloc differs from sttm_reduce\n");
      return 41;
    }
    free(merged2);
  }
  if (rc) {
    fprintf(stderr, "status %d: %s\n", rc, sttm_last_error(c));
    return 20 + rc;
  }
  long long total = 0;
  for (int64_t k = 0; k < K; ++k) total += counts[k];
  if (total != N || offsets[B] != K || K < 1) {
    fprintf(stderr, "counts add up to %lld of %d tokens, K = %lld\n", total, N, (long long)K);
    return 40;
  }
  sttm_destroy(c);
  free(ws);
  free(x);
  free(merged);
  printf("case B=%d T=%d %dx%d D=%d dtype=%d budget=%d: K=%lld of %d\n", B, T, H, W, D, dtype, (int)budget, (long long)K, N);
  return 0;
}

int main() {
  int rc = run_case(1, 3, 5, 6, 16, STTM_F32, false, 1, 0);
  if (!rc) rc = run_case(2, 3, 9, 7, 24, STTM_BF16, true, 2, 1);
  return rc;
}
