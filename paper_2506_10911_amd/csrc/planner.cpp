// Seeded subgroup sampling for the NoLoCo outer step (arxiv 2506.10911, section "Outer
// optimizer step with modified Nesterov momentum": each outer iteration draws fresh random
// subgroups of n workers; section "Inner optimizer step via dynamic pipeline routing":
// groups are formed from random permutations).
//
// Host only.  The draw sequence is counter based, so the plan for (seed, step) needs no
// state carried over from earlier steps.
#include <algorithm>
#include <cstdint>

#include "noloco.h"

namespace {

constexpr uint64_t kWeyl = 0x9E3779B97F4A7C15ull;  // 2^64 / golden ratio, SplitMix64's increment

// SplitMix64 finaliser (Steele, Lea, Flood 2014): two xor-shift-multiply rounds and a last xor-shift.
inline uint64_t finalise(uint64_t x) {
  x ^= x >> 30;
  x *= 0xBF58476D1CE4E5B9ull;
  x ^= x >> 27;
  x *= 0x94D049BB133111EBull;
  x ^= x >> 31;
  return x;
}

// In-place uniform shuffle of items[0..count): position i (from the top down) receives a
// uniformly chosen element of [0, i].  `state` is the SplitMix64 state, advanced per draw.
inline void shuffle(int32_t* items, int32_t count, uint64_t state) {
  for (int64_t i = static_cast<int64_t>(count) - 1; i > 0; --i) {
    const uint64_t range = static_cast<uint64_t>(i) + 1;
    // 2^64 = q*range + leftover; draws below `leftover` would make residues uneven.
    const uint64_t leftover = (~range + 1) % range;
    uint64_t draw;
    do {
      state += kWeyl;
      draw = finalise(state);
    } while (draw < leftover);
    const int64_t j = static_cast<int64_t>(draw % range);
    const int32_t tmp = items[i];
    items[i] = items[j];
    items[j] = tmp;
  }
}

}  // namespace

extern "C" noloco_status noloco_plan_routes(uint64_t seed, uint64_t step, uint64_t microbatch,
                                            int32_t num_stages, int32_t W, int32_t* send_to,
                                            int32_t* recv_from) {
  if (num_stages < 1 || W < 1) return NOLOCO_ERR_INVALID_ARG;
  if (num_stages > 1 && (send_to == nullptr || recv_from == nullptr)) return NOLOCO_ERR_NULL;
  // Key chain: step, then micro-batch, then stage boundary; each link is finalised so that
  // neighbouring counters give unrelated streams.
  uint64_t key = finalise(seed ^ finalise(step + kWeyl));
  key = finalise(key ^ finalise(microbatch + 2 * kWeyl));
  for (int32_t boundary = 0; boundary < num_stages - 1; ++boundary) {
    int32_t* forward = send_to + static_cast<int64_t>(boundary) * W;
    int32_t* backward = recv_from + static_cast<int64_t>(boundary) * W;
    for (int32_t r = 0; r < W; ++r) forward[r] = r;
    shuffle(forward, W, finalise(key ^ finalise(static_cast<uint64_t>(boundary) + 3 * kWeyl)));
    for (int32_t r = 0; r < W; ++r) backward[forward[r]] = r;   // the inverse permutation
  }
  return NOLOCO_OK;
}

extern "C" noloco_status noloco_plan_groups(uint64_t seed, uint64_t step, int32_t W, int32_t n,
                                            int32_t* members, int32_t* group_offsets) {
  if (members == nullptr || group_offsets == nullptr) return NOLOCO_ERR_NULL;
  if (W < 1) return NOLOCO_ERR_INVALID_ARG;
  if (n < 1 || n > W || W % n != 0) return NOLOCO_ERR_BAD_GROUPING;

  // Generator state for this step; every draw advances it by the Weyl constant.
  const uint64_t state = finalise(seed ^ finalise(step + kWeyl));

  for (int32_t w = 0; w < W; ++w) members[w] = w;

  shuffle(members, W, state);

  const int32_t groups = W / n;
  for (int32_t g = 0; g < groups; ++g) {
    int32_t* first = members + static_cast<int64_t>(g) * n;
    std::sort(first, first + n);
    group_offsets[g] = g * n;
  }
  group_offsets[groups] = W;
  return NOLOCO_OK;
}
