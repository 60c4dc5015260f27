// Host-only exercise of the library's pure host code and of the oracle under AddressSanitizer and
// UBSan (built and run by tests/test_host_sanitized.py; no GPU, no HIP runtime).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "noloco.h"

extern "C" {
int oracle_plan_groups(uint64_t, uint64_t, int32_t, int32_t, int32_t*, int32_t*);
int oracle_plan_routes(uint64_t, uint64_t, uint64_t, int32_t, int32_t, int32_t*, int32_t*);
int oracle_outer_step_f32(float*, float*, void*, int32_t, int64_t, int32_t, const int64_t*, const int64_t*,
                          int32_t, float, float, float, const int32_t*, const int32_t*, int32_t);
int oracle_replica_spread(const void*, int32_t, int64_t, int32_t, const int64_t*, const int64_t*, int32_t,
                          int32_t, double*);
}

#define CHECK(cond) do { if (!(cond)) { std::printf("CHECK failed at line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

int main() {
  // planners, product against oracle, exact-size buffers so that any overrun is caught
  for (int32_t W : {1, 2, 3, 8, 64, 96, 1000}) {
    for (int32_t n = 1; n <= W; ++n) {
      if (W % n != 0 || (W > 100 && n > 8 && n != W)) continue;
      std::vector<int32_t> m1(W), o1(W / n + 1), m2(W), o2(W / n + 1);
      CHECK(noloco_plan_groups(5, 77, W, n, m1.data(), o1.data()) == NOLOCO_OK);
      CHECK(oracle_plan_groups(5, 77, W, n, m2.data(), o2.data()) == 0);
      CHECK(m1 == m2 && o1 == o2);
    }
  }
  CHECK(noloco_plan_groups(0, 0, 8, 3, nullptr, nullptr) == NOLOCO_ERR_NULL);
  {
    std::vector<int32_t> m(8), o(9);
    CHECK(noloco_plan_groups(0, 0, 8, 3, m.data(), o.data()) == NOLOCO_ERR_BAD_GROUPING);
    CHECK(noloco_plan_groups(~0ull, ~0ull, 8, 8, m.data(), o.data()) == NOLOCO_OK);
  }
  for (int32_t stages : {1, 2, 5}) {
    for (int32_t W : {1, 7, 64}) {
      std::vector<int32_t> s1((stages - 1) * W), r1((stages - 1) * W), s2(s1.size()), r2(r1.size());
      CHECK(noloco_plan_routes(9, 3, 4, stages, W, s1.data(), r1.data()) == NOLOCO_OK);
      CHECK(oracle_plan_routes(9, 3, 4, stages, W, s2.data(), r2.data()) == 0);
      CHECK(s1 == s2 && r1 == r2);
    }
  }
  // segment merging
  {
    std::vector<noloco_segment> segs = {{10, 5}, {0, 10}, {20, 3}, {15, 0}, {23, 1}};
    std::vector<noloco_segment> runs(segs.size());
    int32_t count = -1;
    CHECK(noloco_merge_segments(segs.data(), 5, 64, runs.data(), &count) == NOLOCO_OK && count == 2);
    CHECK(runs[0].offset == 0 && runs[0].numel == 15 && runs[1].offset == 20 && runs[1].numel == 4);
    CHECK(noloco_merge_segments(segs.data(), 5, 23, runs.data(), &count) == NOLOCO_ERR_SEGMENT_OVERLAP);
    CHECK(noloco_merge_segments(nullptr, 0, 64, nullptr, &count) == NOLOCO_OK && count == 0);
    noloco_segment huge = {INT64_MAX - 2, 5};
    CHECK(noloco_merge_segments(&huge, 1, INT64_MAX, nullptr, &count) == NOLOCO_ERR_SEGMENT_OVERLAP);
  }
  // latency model
  {
    double out[4];
    CHECK(noloco_sim_tree_vs_pair(1, 64, 0.0, 0.5, 200, out) == NOLOCO_OK && out[0] > out[2]);
    CHECK(noloco_sim_tree_vs_pair(1, 48, 0.0, 0.5, 200, out) == NOLOCO_ERR_INVALID_ARG);
    CHECK(noloco_sim_barrier_penalty(1, 64, 2, 10, 20, 1.0, 0.7, out) == NOLOCO_OK && out[0] >= out[1]);
  }
  // oracle step and spread on exact-size buffers with ragged segments
  {
    const int32_t W = 6;
    const int64_t S = 64;
    std::vector<float> phi(W * S, 0.5f), delta(W * S, 0.25f), theta(W * S, 0.75f);
    std::vector<uint16_t> theta16(W * S, 0x3F80);
    const int64_t off[3] = {0, 7, 63}, len[3] = {5, 33, 1};
    const int32_t members[6] = {5, 0, 3, 1, 4, 2}, offsets[3] = {0, 4, 6};
    CHECK(oracle_outer_step_f32(phi.data(), delta.data(), theta.data(), 0, S, W, off, len, 3, 0.9f, 0.7f, 1.0f,
                                members, offsets, 2) == 0);
    CHECK(oracle_outer_step_f32(phi.data(), delta.data(), theta16.data(), 1, S, W, off, len, 3, 0.9f, 0.7f, 1.0f,
                                members, offsets, 2) == 0);
    double out[4];
    CHECK(oracle_replica_spread(phi.data(), 0, S, W, off, len, 3, 0, out) == 0);
    CHECK(oracle_replica_spread(theta16.data(), 1, S, W, off, len, 3, 1, out) == 0);
  }
  std::printf("host sanitize driver: ok\n");
  return 0;
}
