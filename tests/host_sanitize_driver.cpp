// Host-only exercise of the library's host code and of the oracle under AddressSanitizer and
// UBSan (built and run by tests/test_host_sanitized.py; no GPU, no HIP runtime).  The C ABI's
// argument checking and launch splitting (api.cpp) run against stand-ins for the few HIP runtime
// calls they make and for the kernel launchers of kernels.hip, which record what would be launched.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "noloco.h"
#include "noloco_internal.h"

// ---- stand-ins: device memory is host memory, launches are recorded ----
extern "C" hipError_t hipGetDevice(int* device) { *device = 0; return hipSuccess; }
extern "C" hipError_t hipMalloc(void** ptr, size_t size) {
  *ptr = std::malloc(size ? size : 1);
  return *ptr ? hipSuccess : hipErrorOutOfMemory;
}
extern "C" hipError_t hipFree(void* ptr) { std::free(ptr); return hipSuccess; }
extern "C" hipError_t hipMemcpy(void* dst, const void* src, size_t size, hipMemcpyKind) {
  std::memcpy(dst, src, size);
  return hipSuccess;
}
namespace noloco {
struct Launch { StepArgs args; KernelChoice choice; };
static std::vector<Launch> launches;
static int fail_at_launch = -1;              // index of the launch the stand-in refuses
int launch_outer_step(const StepArgs& args, int32_t, const KernelChoice& choice, void*) {
  if (static_cast<int>(launches.size()) == fail_at_launch) return 1;
  launches.push_back(Launch{args, choice});
  return 0;
}
int launch_replica_spread(const SpreadArgs&, int32_t, const SegmentTiles*, int32_t, double*, void*) { return 0; }
int launch_stream_probe(int, void*, const void*, int64_t, float, void*) { return 0; }
int static_spread_scratch(double** out) { static double slot[4]; *out = slot; return 0; }
}  // namespace noloco

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
  // ---- the C ABI's host path: validation, bucketing by group size, launch splitting ----
  {
    using noloco::launches;
    float* const phi = reinterpret_cast<float*>(1ull << 40);       // never dereferenced on this path
    float* const delta = reinterpret_cast<float*>(2ull << 40);
    void* const theta = reinterpret_cast<void*>(3ull << 40);
    const noloco_hparams hp = {0.9f, 0.7f, 1.0f};
    auto make_plan = [&](int32_t W, int64_t stride, noloco_launch_plan** plan, noloco_arena* arena) {
      static noloco_segment seg;
      seg = noloco_segment{0, stride};
      *arena = noloco_arena{phi, delta, theta, stride, W, NOLOCO_F32, &seg, 1};
      return noloco_launch_plan_create(arena, plan);
    };
    noloco_launch_plan* plan = nullptr;
    noloco_arena arena;
    // (1) mixed group sizes, members unsorted, a worker left out, an empty group
    CHECK(make_plan(9, 1 << 24, &plan, &arena) == NOLOCO_OK);
    {
      const int32_t members[8] = {7, 2, 5, 0, 3, 1, 8, 6}, offsets[5] = {0, 2, 2, 6, 8};
      launches.clear();
      CHECK(noloco_outer_step(plan, &arena, &hp, members, offsets, 4, nullptr) == NOLOCO_OK);
      CHECK(launches.size() == 2);
      const noloco::StepArgs& a = launches[0].args;            // sizes ascending: the pairs first
      CHECK(a.n == 2 && a.num_groups == 2 && a.inv_n == 0.5f && a.tile_offset == 0);
      CHECK(a.rows[0] == 2 && a.rows[1] == 7 && a.rows[2] == 6 && a.rows[3] == 8);
      CHECK(a.num_tiles == (1 << 24) / 4096 && a.work_items == 2u * a.num_tiles);
      CHECK(launches[0].choice.vectors_per_thread == 4 && a.group_major == 1 && a.xcd_map == 0);
      const noloco::StepArgs& b = launches[1].args;
      CHECK(b.n == 4 && b.num_groups == 1 && b.inv_n == 0.25f);
      CHECK(b.rows[0] == 0 && b.rows[1] == 1 && b.rows[2] == 3 && b.rows[3] == 5);
      CHECK(b.num_tiles == (1 << 24) / 2048 && b.group_major == 0 && b.xcd_map == 1);
      // refused groupings launch nothing
      const int32_t dup[4] = {0, 1, 1, 2}, two[3] = {0, 2, 4}, range[4] = {0, 1, 2, 9};
      const int32_t bad_start[3] = {1, 2, 4}, decreasing[3] = {0, 3, 2};
      launches.clear();
      CHECK(noloco_outer_step(plan, &arena, &hp, dup, two, 2, nullptr) == NOLOCO_ERR_BAD_GROUPING);
      CHECK(noloco_outer_step(plan, &arena, &hp, range, two, 2, nullptr) == NOLOCO_ERR_BAD_GROUPING);
      CHECK(noloco_outer_step(plan, &arena, &hp, members, bad_start, 2, nullptr) == NOLOCO_ERR_BAD_GROUPING);
      CHECK(noloco_outer_step(plan, &arena, &hp, members, decreasing, 2, nullptr) == NOLOCO_ERR_BAD_GROUPING);
      CHECK(noloco_outer_step(plan, &arena, &hp, nullptr, two, 2, nullptr) == NOLOCO_ERR_NULL);
      noloco_arena other = arena;
      other.delta = phi + 64;                                  // aligned, but overlaps phi
      CHECK(noloco_outer_step(plan, &other, &hp, members, offsets, 4, nullptr) == NOLOCO_ERR_INVALID_ARG);
      CHECK(launches.empty());
      CHECK(noloco_outer_step(plan, &arena, &hp, nullptr, nullptr, 0, nullptr) == NOLOCO_OK && launches.empty());
      // the runtime refusing the second launch is reported
      noloco::fail_at_launch = 1;
      CHECK(noloco_outer_step(plan, &arena, &hp, members, offsets, 4, nullptr) == NOLOCO_ERR_DEVICE);
      CHECK(launches.size() == 1);
      noloco::fail_at_launch = -1;
    }
    CHECK(noloco_launch_plan_destroy(plan) == NOLOCO_OK);
    // (2) more groups than one member table holds: 300 pairs go out as 128 + 128 + 44; a group of
    //     257 is refused before anything is launched
    CHECK(make_plan(600, 1 << 20, &plan, &arena) == NOLOCO_OK);
    {
      std::vector<int32_t> members(600), offsets(301);
      for (int32_t w = 0; w < 600; ++w) members[w] = 599 - w;
      for (int32_t g = 0; g <= 300; ++g) offsets[g] = 2 * g;
      launches.clear();
      CHECK(noloco_outer_step(plan, &arena, &hp, members.data(), offsets.data(), 300, nullptr) == NOLOCO_OK);
      CHECK(launches.size() == 3 && launches[0].args.num_groups == 128 && launches[1].args.num_groups == 128 &&
            launches[2].args.num_groups == 44);
      CHECK(launches[2].args.rows[0] == 86 && launches[2].args.rows[1] == 87);   // group 256 = workers {87, 86}
      std::vector<int32_t> big_offsets = {0, 2, 259, 261};
      launches.clear();
      CHECK(noloco_outer_step(plan, &arena, &hp, members.data(), big_offsets.data(), 3, nullptr) == NOLOCO_ERR_UNSUPPORTED);
      CHECK(launches.empty());
    }
    CHECK(noloco_launch_plan_destroy(plan) == NOLOCO_OK);
    // (3) more workgroups than one grid holds: the launch is cut over tile ranges that tile the row
    CHECK(make_plan(2, 1ll << 35, &plan, &arena) == NOLOCO_OK);
    {
      const int32_t members[2] = {1, 0}, offsets[3] = {0, 1, 2};
      for (int32_t vpt : {-1, 1}) {
        const noloco_tuning tuning = {vpt, -1, -1, -1};
        CHECK(noloco_launch_plan_tune(plan, &tuning) == NOLOCO_OK);
        launches.clear();
        CHECK(noloco_outer_step(plan, &arena, &hp, members, offsets, 2, nullptr) == NOLOCO_OK);
        const int64_t tiles = (1ll << 35) / (vpt == 1 ? 1024 : 4096);
        CHECK(launches.size() == (vpt == 1 ? 5u : 2u));
        int64_t next = 0;
        for (const noloco::Launch& l : launches) {
          CHECK(l.args.n == 1 && l.args.num_groups == 2 && l.args.tile_offset == next);
          CHECK(l.args.work_items == static_cast<uint64_t>(l.args.num_tiles) * 2);
          CHECK(static_cast<int64_t>(l.args.work_items) <= noloco::kMaxGridWorkgroups);
          next += l.args.num_tiles;
        }
        CHECK(next == tiles);
      }
    }
    CHECK(noloco_launch_plan_destroy(plan) == NOLOCO_OK);
    // (4) a small arena takes small tiles; limits of plan creation
    CHECK(make_plan(4, 1 << 20, &plan, &arena) == NOLOCO_OK);
    {
      const int32_t members[4] = {0, 1, 2, 3}, offsets[3] = {0, 2, 4};
      launches.clear();
      CHECK(noloco_outer_step(plan, &arena, &hp, members, offsets, 2, nullptr) == NOLOCO_OK);
      CHECK(launches.size() == 1 && launches[0].choice.vectors_per_thread == 1 && launches[0].args.num_tiles == 1024);
    }
    CHECK(noloco_launch_plan_destroy(plan) == NOLOCO_OK);
    CHECK(make_plan(NOLOCO_MAX_WORKERS + 1, 64, &plan, &arena) == NOLOCO_ERR_UNSUPPORTED && plan == nullptr);
    CHECK(make_plan(4, 63, &plan, &arena) == NOLOCO_ERR_ALIGNMENT);
  }
  std::printf("host sanitize driver: ok\n");
  return 0;
}
