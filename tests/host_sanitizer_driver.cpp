// Walks the host-only entry points of libvorta (plan construction, index tables, route
// bookkeeping, router) under AddressSanitizer / UBSan.  Built and run by
// tests/test_host_tables.py; links vorta_host.cpp alone (it has no reference into the device side).
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "vorta_internal.h"

static int failures = 0;
#define EXPECT(cond)                                                   \
  do {                                                                 \
    if (!(cond)) {                                                     \
      std::printf("line %d: %s failed (%s)\n", __LINE__, #cond, vorta_last_error()); \
      ++failures;                                                      \
    }                                                                  \
  } while (0)

static vorta_layer_desc desc(int F, int H, int W, int n_text, int heads, const int tile[3], const int window[3],
                             const int bucket[3], int mode, int num, int den) {
  vorta_layer_desc d;
  std::memset(&d, 0, sizeof(d));
  d.F = F; d.H = H; d.W = W; d.n_text = n_text; d.heads = heads; d.head_dim = 128;
  d.dtype = VORTA_BF16; d.layout = VORTA_LAYOUT_HND;
  for (int a = 0; a < 3; ++a) { d.tile[a] = tile[a]; d.window[a] = window[a]; d.bucket[a] = bucket[a]; }
  d.center_mode = mode; d.keep_num = num; d.keep_den = den;
  return d;
}

static void walk(const vorta_layer_desc& d) {
  vorta_plan* p = nullptr;
  EXPECT(vorta_plan_create(&d, &p) == VORTA_OK);
  if (!p) return;
  vorta_plan_info info;
  EXPECT(vorta_plan_info_get(p, &info) == VORTA_OK);
  std::vector<int32_t> perm((size_t)info.n_video), row0((size_t)info.n_tiles + 1), boxes((size_t)info.n_tiles * 6),
      runs((size_t)info.n_tiles * info.max_runs * 2), n_runs((size_t)info.n_tiles), sb((size_t)info.n_buckets + 1);
  EXPECT(vorta_tile_permutation(p, perm.data()) == VORTA_OK);
  EXPECT(vorta_tile_row0(p, row0.data()) == VORTA_OK);
  EXPECT(vorta_window_boxes(p, boxes.data()) == VORTA_OK);
  EXPECT(vorta_window_runs(p, runs.data(), n_runs.data()) == VORTA_OK);
  EXPECT(vorta_bcs_slot_bases(p, sb.data()) == VORTA_OK);
  EXPECT(row0.back() == info.n_video && sb.back() == info.n_core);
  for (int t = 0; t < info.n_tiles; ++t)
    for (int r = 0; r < n_runs[t]; ++r) {
      const int32_t* run = &runs[((size_t)t * info.max_runs + r) * 2];
      EXPECT(run[0] >= 0 && run[1] > 0 && (int64_t)run[0] + run[1] <= info.n_tokens);
    }
  std::vector<uint8_t> routes((size_t)d.heads);
  for (int h = 0; h < d.heads; ++h) routes[h] = (uint8_t)(h % 3);
  std::vector<int32_t> by_route((size_t)d.heads);
  int32_t counts[3];
  EXPECT(vorta_route_partition(p, routes.data(), by_route.data(), counts) == VORTA_OK);
  EXPECT(counts[0] + counts[1] + counts[2] == d.heads);
  size_t bytes = 0, off[12];
  EXPECT(vorta_workspace_bytes(p, routes.data(), &bytes) == VORTA_OK && bytes >= 256);
  EXPECT(vorta_workspace_layout(p, routes.data(), off) == VORTA_OK);
  EXPECT(vorta_soft_mixture_workspace_bytes(p, &bytes) == VORTA_OK);
  routes[0] = 9;
  EXPECT(vorta_route_partition(p, routes.data(), by_route.data(), counts) == VORTA_EROUTE);
  EXPECT(vorta_plan_destroy(p) == VORTA_OK);
}

int main() {
  const int t1[3] = {2, 4, 4}, w3[3] = {3, 3, 3}, b[3] = {2, 3, 2};
  walk(desc(4, 8, 8, 0, 2, t1, w3, b, VORTA_CENTER_CLAMP, 1, 2));
  const int t2[3] = {2, 3, 4}, w2[3] = {1, 2, 5};
  for (int mode = 0; mode < 3; ++mode) walk(desc(5, 7, 6, 9, 5, t2, w2, b, mode, 2, 3));
  const int huge[3] = {2147483647, 70000, 3}, wide[3] = {2147483647, 1, 2147483646}, bb[3] = {2147483647, 2, 1};
  for (int mode = 0; mode < 3; ++mode) walk(desc(3, 5, 7, 1, 128, huge, wide, bb, mode, 1, 4));
  const int one[3] = {1, 1, 1};
  walk(desc(1, 1, 1, 0, 1, one, one, one, VORTA_CENTER_BLOCK, 1, 1));
  walk(desc(21, 45, 80, 0, 40, (const int[3]){3, 5, 8}, w3, b, VORTA_CENTER_CLAMP, 1, 2));
  vorta_layer_desc roped = desc(5, 7, 6, 9, 5, t2, w2, b, 0, 1, 2);
  roped.rope_dims[0] = 44; roped.rope_dims[1] = 42; roped.rope_dims[2] = 42; roped.rope_theta = 0.f;
  walk(roped);

  // rejected descriptions leave no plan behind
  vorta_plan* p = nullptr;
  vorta_layer_desc bad = desc(4, 8, 8, 0, 2, t1, w3, b, 0, 1, 2);
  bad.tile[1] = 0;
  EXPECT(vorta_plan_create(&bad, &p) == VORTA_ESHAPE && p == nullptr);
  bad = desc(4, 8, 8, 0, 2, t1, w3, b, 7, 1, 2);
  EXPECT(vorta_plan_create(&bad, &p) == VORTA_EINVAL && p == nullptr);
  bad = desc(2147483647, 2147483647, 2147483647, 2147483647, 2, t1, w3, b, 0, 1, 2);
  EXPECT(vorta_plan_create(&bad, &p) == VORTA_ESHAPE && p == nullptr);
  EXPECT(vorta_plan_create(nullptr, &p) == VORTA_EINVAL);
  EXPECT(vorta_plan_destroy(nullptr) == VORTA_OK);

  // router (Eq. 3, Eq. 4)
  const int heads = 7, d_t = 33;
  std::vector<float> t(d_t), w((size_t)heads * d_t * 3), alpha((size_t)heads * 3);
  for (int i = 0; i < d_t; ++i) t[i] = 0.01f * (float)(i - 16);
  for (size_t i = 0; i < w.size(); ++i) w[i] = 0.001f * (float)((int)(i * 37 % 101) - 50);
  EXPECT(vorta_router_gates(t.data(), w.data(), d_t, heads, alpha.data()) == VORTA_OK);
  std::vector<uint8_t> routes((size_t)heads);
  EXPECT(vorta_route_select(alpha.data(), heads, routes.data()) == VORTA_OK);
  for (int h = 0; h < heads; ++h) EXPECT(routes[h] <= 2);
  EXPECT(vorta_router_gates(t.data(), w.data(), 0, heads, alpha.data()) == VORTA_EINVAL);

  if (failures) {
    std::printf("%d check(s) failed\n", failures);
    return 1;
  }
  std::printf("host entry points clean\n");
  return 0;
}
