// Latency model of the paper (section "Latency results", appendix "Latency analysis"): Monte-Carlo
// estimates of (a) the time of a tree all-reduce against pairwise local averaging when every
// message takes a LogNormal(mu, sigma^2) time, and (b) the cost of a global barrier per outer step
// when inner steps take LogNormal times.  Host only; no GPU work.
//
// Random numbers: SplitMix64 (counter based, one stream per call) -> two uniforms in (0, 1) ->
// Box-Muller normal -> exp(mu + sigma z).
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <new>
#include <vector>

#include "noloco.h"

namespace {

constexpr uint64_t kWeyl = 0x9E3779B97F4A7C15ull;

struct Rng {
  uint64_t state;
  explicit Rng(uint64_t seed, uint64_t stream) {
    state = scramble(seed ^ scramble(stream + kWeyl));
  }
  static uint64_t scramble(uint64_t x) {
    x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27; x *= 0x94D049BB133111EBull;
    return x ^ (x >> 31);
  }
  uint64_t next() { state += kWeyl; return scramble(state); }
  double uniform() { return (static_cast<double>(next() >> 11) + 0.5) * (1.0 / 9007199254740992.0); }
  double normal() {
    const double u1 = uniform(), u2 = uniform();
    return std::sqrt(-2.0 * std::log(u1)) * std::cos(6.283185307179586476925 * u2);
  }
  double lognormal(double mu, double sigma) { return std::exp(mu + sigma * normal()); }
};

struct Moments {
  double sum = 0.0, sum_sq = 0.0;
  int64_t count = 0;
  void add(double x) { sum += x; sum_sq += x * x; ++count; }
  double mean() const { return sum / static_cast<double>(count); }
  double stderr_of_mean() const {
    if (count < 2) return 0.0;
    const double m = mean();
    const double var = std::max(0.0, (sum_sq - static_cast<double>(count) * m * m) / static_cast<double>(count - 1));
    return std::sqrt(var / static_cast<double>(count));
  }
};

noloco_status tree_vs_pair(uint64_t seed, int32_t W, double mu, double sigma, int32_t trials,
                           double* out) {
  if (out == nullptr) return NOLOCO_ERR_NULL;
  if (W < 2 || (W & (W - 1)) != 0 || trials < 1 || !(sigma >= 0.0)) return NOLOCO_ERR_INVALID_ARG;
  Rng rng(seed, 0x74726565);
  // Complete binary tree in heap order: node k has children 2k+1 and 2k+2; the last W nodes are
  // the workers.  A parent is ready when the later of its two children's messages has arrived;
  // the result then travels back down, one message per edge.
  const int64_t nodes = 2 * static_cast<int64_t>(W) - 1;
  std::vector<double> ready(static_cast<size_t>(nodes));
  Moments tree, pair;
  for (int32_t t = 0; t < trials; ++t) {
    for (int64_t k = nodes - 1; k >= 0; --k) {
      if (2 * k + 1 >= nodes) { ready[static_cast<size_t>(k)] = 0.0; continue; }
      const double left = ready[static_cast<size_t>(2 * k + 1)] + rng.lognormal(mu, sigma);
      const double right = ready[static_cast<size_t>(2 * k + 2)] + rng.lognormal(mu, sigma);
      ready[static_cast<size_t>(k)] = std::max(left, right);
    }
    double done = 0.0;
    for (int64_t k = 1; k < nodes; ++k) {
      ready[static_cast<size_t>(k)] = ready[static_cast<size_t>((k - 1) / 2)] + rng.lognormal(mu, sigma);
      if (2 * k + 1 >= nodes) done = std::max(done, ready[static_cast<size_t>(k)]);
    }
    tree.add(done);
    // Pairwise averaging: two exchanges, each as long as the slower of its two messages.
    const double first = std::max(rng.lognormal(mu, sigma), rng.lognormal(mu, sigma));
    const double second = std::max(rng.lognormal(mu, sigma), rng.lognormal(mu, sigma));
    pair.add(first + second);
  }
  out[0] = tree.mean();
  out[1] = tree.stderr_of_mean();
  out[2] = pair.mean();
  out[3] = pair.stderr_of_mean();
  return NOLOCO_OK;
}

noloco_status barrier_penalty(uint64_t seed, int32_t W, int32_t n, int32_t inner_steps,
                              int32_t outer_steps, double mu, double sigma, double* out) {
  if (out == nullptr) return NOLOCO_ERR_NULL;
  if (W < 1 || inner_steps < 1 || outer_steps < 1 || !(sigma >= 0.0)) return NOLOCO_ERR_INVALID_ARG;
  if (n < 1 || n > W || W % n != 0) return NOLOCO_ERR_BAD_GROUPING;
  Rng rng(seed, 0x62617272);
  std::vector<double> clock(static_cast<size_t>(W), 0.0);     // each worker's own time, subgroup sync only
  std::vector<int32_t> members(static_cast<size_t>(W)), offsets(static_cast<size_t>(W / n) + 1);
  double barrier_clock = 0.0;                                  // everybody waits for the slowest, every round
  for (int32_t round = 0; round < outer_steps; ++round) {
    double slowest = 0.0;
    for (int32_t w = 0; w < W; ++w) {
      double phase = 0.0;
      for (int32_t k = 0; k < inner_steps; ++k) phase += rng.lognormal(mu, sigma);
      clock[static_cast<size_t>(w)] += phase;
      slowest = std::max(slowest, phase);
    }
    barrier_clock += slowest;
    const noloco_status st = noloco_plan_groups(seed, static_cast<uint64_t>(round), W, n,
                                                members.data(), offsets.data());
    if (st != NOLOCO_OK) return st;
    for (int32_t g = 0; g < W / n; ++g) {
      double latest = 0.0;
      for (int32_t a = offsets[static_cast<size_t>(g)]; a < offsets[static_cast<size_t>(g) + 1]; ++a)
        latest = std::max(latest, clock[static_cast<size_t>(members[static_cast<size_t>(a)])]);
      for (int32_t a = offsets[static_cast<size_t>(g)]; a < offsets[static_cast<size_t>(g) + 1]; ++a)
        clock[static_cast<size_t>(members[static_cast<size_t>(a)])] = latest;
    }
  }
  out[0] = barrier_clock;
  out[1] = *std::max_element(clock.begin(), clock.end());
  return NOLOCO_OK;
}

// Runs `body` and turns a failed host allocation into a status: no exception leaves the C ABI.
template <typename Body> noloco_status guarded(Body body) {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    return NOLOCO_ERR_NO_MEMORY;
  } catch (...) {
    return NOLOCO_ERR_INVALID_ARG;
  }
}

}  // namespace

extern "C" noloco_status noloco_sim_tree_vs_pair(uint64_t seed, int32_t W, double mu, double sigma,
                                                 int32_t trials, double* out) {
  return guarded([&] { return tree_vs_pair(seed, W, mu, sigma, trials, out); });
}

extern "C" noloco_status noloco_sim_barrier_penalty(uint64_t seed, int32_t W, int32_t n,
                                                    int32_t inner_steps, int32_t outer_steps,
                                                    double mu, double sigma, double* out) {
  return guarded([&] { return barrier_penalty(seed, W, n, inner_steps, outer_steps, mu, sigma, out); });
}
