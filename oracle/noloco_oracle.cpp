// NoLoCo outer optimizer step: reference oracle (TEST INFRASTRUCTURE, not product).
//
// A plain, slow, single-threaded CPU evaluation of what the GPU library
// computes.  It exists so tests, the smoke check and the benchmark's
// cpu_baseline leg have something obviously correct to compare against.  It
// shares no code with the HIP path and the product never calls it.
//
// What it follows (arxiv 2506.10911, section "Outer optimizer step with
// modified Nesterov momentum"):
//   Eq. 1  outer gradient       Delta_i = phi_i - theta_i
//          (sign: outer weights minus local weights.  The printed Eq. 1 has
//          the opposite sign, which contradicts the mean dynamics of the
//          convergence appendix, E(delta_t) = alpha E(delta_{t-1}) + beta E(Delta_t)
//          with the contracting factor I + beta (B^m - I); with the sign used
//          here Eq. 2, inserted as printed, descends and reduces to DiLoCo.)
//   Eq. 2  momentum             delta'_i = alpha delta_i - (beta/n) sum_j Delta_j
//                                          - gamma (phi_i - (1/n) sum_j phi_j)
//          j runs over all n members of i's subgroup, i included; every phi on
//          the right-hand side is the value BEFORE this step.
//   Eq. 3  slow-weight update   phi'_i = phi_i + delta'_i
//   restart of the fast weights theta'_i = phi'_i   (convergence appendix:
//          the inner iteration of the next round starts from the slow weights)
//   subgroup sampling           a fresh random permutation of the workers every
//          outer step, cut into consecutive groups of n (section "Inner
//          optimizer step via dynamic pipeline routing" says groups come from
//          random permutations; section "Outer optimizer step ..." that they
//          are drawn afresh every iteration).  The paper names no generator;
//          the one below is this build's own choice, stated in full here.
//
// Pins (tests/test_oracle_*.py, run without a GPU): hand-worked dyadic
// examples of Eq. 1-3, the DiLoCo reduction for n = N against a textbook
// momentum loop, a literal per-worker evaluation over every partition of
// tiny worker sets, the group-mean / global-mean / spread identities that
// follow from Eq. 2-3, order invariance, the published SplitMix64
// known-answer vector, partition validity and uniformity of the planner,
// an exhaustive 16-bit analogue of the bounded draw, and planted mistakes in
// the step and in both planners that those pins must catch.
// Parity unpinned: the choice of generator and seed-mixing rule of the two
// planners (the paper fixes only that the draws are uniform and fresh), and
// the tree all-reduce time of the latency model for more than two workers
// with sigma > 0 (oracle/latency.py).
//
// Build: g++ -O2 -std=c++17 -ffp-contract=off -shared -fPIC (see build.py).
// -ffp-contract=off matters: the float instantiation is the bit-level target
// and every operation below is meant to round once, separately.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>
#include <algorithm>

namespace {

// ---------------------------------------------------------------------------
// Subgroup planner
// ---------------------------------------------------------------------------

constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;

// Output function of the published SplitMix64 generator.
uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// Rejection rule of the bounded draw for a word of type U (2^bits values):
// the lowest (2^bits mod m) values of r are thrown away so that the rest
// splits evenly over the m residues.  A template so that a 16-bit
// instantiation can be enumerated exhaustively by the tests.
template <typename U>
bool accepted(U r, U m) {
  U reject_below = static_cast<U>(static_cast<U>(U(0) - m) % m);  // == 2^bits mod m
  return r >= reject_below;
}

// One stream of draws per (seed, step).  Draw k is SplitMix64's (k+1)-th output
// when its state starts at `base`.
struct DrawStream {
  uint64_t base;
  uint64_t k = 0;
  DrawStream(uint64_t seed, uint64_t step) : base(mix64(seed ^ mix64(step + kGolden))) {}
  explicit DrawStream(uint64_t raw_base) : base(raw_base) {}
  uint64_t next() {
    uint64_t r = mix64(base + (k + 1) * kGolden);
    ++k;
    return r;
  }
  // Uniform integer in [0, m), m >= 1, by rejection.
  uint64_t bounded(uint64_t m) {
    for (;;) {
      uint64_t r = next();
      if (accepted<uint64_t>(r, m)) return r % m;
    }
  }
};

// ---------------------------------------------------------------------------
// bf16 <-> fp32 (bf16 = upper 16 bits of binary32; narrowing rounds to nearest,
// ties to even; NaN stays NaN)
// ---------------------------------------------------------------------------

float bf16_widen(uint16_t h) {
  uint32_t u = static_cast<uint32_t>(h) << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

uint16_t bf16_narrow(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) {          // NaN: keep sign, force quiet
    return static_cast<uint16_t>((u >> 16) | 0x0040u);
  }
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7FFFu + lsb;                              // carries into exponent -> Inf as IEEE asks
  return static_cast<uint16_t>(u >> 16);
}

// ---------------------------------------------------------------------------
// Outer step, one scalar type for all arithmetic.
//   T = float : every operation is one IEEE binary32 operation, in the order
//               written; this is what the GPU must reproduce.
//   T = double: the same formulas in binary64; bounds the fp32 rounding error.
// load_theta / store_theta hide the storage type of the fast weights.
// ---------------------------------------------------------------------------

template <typename T, typename LoadTheta, typename StoreTheta>
void outer_step_impl(T* phi, T* delta, int64_t stride,
                     const int64_t* seg_off, const int64_t* seg_len, int32_t num_segments,
                     T alpha, T beta, T gamma,
                     const int32_t* members, const int32_t* group_offsets, int32_t num_groups,
                     LoadTheta load_theta, StoreTheta store_theta) {
  std::vector<int32_t> g;       // members of the current group, ascending
  std::vector<T> phi_old;       // phi_j before the step, for this column
  for (int32_t gi = 0; gi < num_groups; ++gi) {
    g.assign(members + group_offsets[gi], members + group_offsets[gi + 1]);
    std::sort(g.begin(), g.end());
    const size_t n = g.size();
    if (n == 0) continue;
    const T inv_n = T(1) / T(static_cast<int64_t>(n));
    phi_old.resize(n);
    for (int32_t s = 0; s < num_segments; ++s) {
      for (int64_t k = seg_off[s]; k < seg_off[s] + seg_len[s]; ++k) {
        // Eq. 1 for every member, and the two subgroup sums of Eq. 2,
        // accumulated left to right in ascending worker order.
        T sum_Delta = T(0), sum_phi = T(0);
        for (size_t a = 0; a < n; ++a) {
          const int64_t at = static_cast<int64_t>(g[a]) * stride + k;
          const T p = phi[at];
          const T Delta = p - load_theta(at);
          phi_old[a] = p;
          if (a == 0) { sum_Delta = Delta; sum_phi = p; }
          else        { sum_Delta = sum_Delta + Delta; sum_phi = sum_phi + p; }
        }
        const T mean_Delta = sum_Delta * inv_n;
        const T mean_phi = sum_phi * inv_n;
        // Eq. 2, Eq. 3 and the restart, member by member.
        for (size_t a = 0; a < n; ++a) {
          const int64_t at = static_cast<int64_t>(g[a]) * stride + k;
          const T t1 = alpha * delta[at];
          const T t2 = beta * mean_Delta;
          const T t3 = gamma * (phi_old[a] - mean_phi);
          const T d_new = (t1 - t2) - t3;
          const T p_new = phi_old[a] + d_new;
          delta[at] = d_new;
          phi[at] = p_new;
          store_theta(at, p_new);
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Replica spread (results section, figure "standard deviation of the model
// weights across the data parallel world size"): how far the W replicas of one
// stage have drifted apart.  Per arena element k the population variance over
// the W workers, v_k = (1/W) sum_w (x_w[k] - m_k)^2 with m_k = (1/W) sum_w x_w[k];
// per tensor the pooled deviation sqrt(mean_k v_k); the same over all tensors.
// (The paper fixes neither the 1/W vs 1/(W-1) convention nor how elements are
// pooled into one number; these are this build's readings.)
//   T = double: the definition.  T = float: the per-element arithmetic in
//   binary32, in ascending worker order, as the GPU does it; pooling over
//   elements is in double either way.
// ---------------------------------------------------------------------------
template <typename T, typename Load>
void replica_spread_impl(Load load, int64_t stride, int32_t W,
                         const int64_t* seg_off, const int64_t* seg_len, int32_t num_segments,
                         double* out_std) {
  const T inv_W = T(1) / T(static_cast<int64_t>(W));
  double total = 0.0;
  int64_t total_count = 0;
  for (int32_t s = 0; s < num_segments; ++s) {
    double pooled = 0.0;
    for (int64_t k = seg_off[s]; k < seg_off[s] + seg_len[s]; ++k) {
      T sum = load(k);
      for (int32_t w = 1; w < W; ++w) sum = sum + load(static_cast<int64_t>(w) * stride + k);
      const T mean = sum * inv_W;
      T q = T(0);
      for (int32_t w = 0; w < W; ++w) {
        const T dev = load(static_cast<int64_t>(w) * stride + k) - mean;
        const T sq = dev * dev;
        q = (w == 0) ? sq : q + sq;
      }
      pooled += static_cast<double>(q * inv_W);
    }
    out_std[s] = seg_len[s] > 0 ? std::sqrt(pooled / static_cast<double>(seg_len[s])) : 0.0;
    total += pooled;
    total_count += seg_len[s];
  }
  out_std[num_segments] = total_count > 0 ? std::sqrt(total / static_cast<double>(total_count)) : 0.0;
}

bool groups_ok(const int32_t* members, const int32_t* group_offsets, int32_t num_groups, int32_t W) {
  if (num_groups < 0 || W < 1) return false;
  if (num_groups > 0 && (!members || !group_offsets)) return false;
  if (num_groups > 0 && group_offsets[0] != 0) return false;
  std::vector<char> seen(static_cast<size_t>(W), 0);
  for (int32_t gi = 0; gi < num_groups; ++gi) {
    if (group_offsets[gi + 1] < group_offsets[gi]) return false;
    for (int32_t a = group_offsets[gi]; a < group_offsets[gi + 1]; ++a) {
      int32_t w = members[a];
      if (w < 0 || w >= W || seen[static_cast<size_t>(w)]) return false;
      seen[static_cast<size_t>(w)] = 1;
    }
  }
  return true;
}

}  // namespace

extern "C" {

uint64_t oracle_mix64(uint64_t z) { return mix64(z); }

// The bounded draw's accept/reduce rule on a 16-bit word: r mod m, or -1 when
// r is rejected.  Same template as the 64-bit draw uses.
int32_t oracle_bounded16(uint16_t r, uint16_t m) {
  return accepted<uint16_t>(r, m) ? static_cast<int32_t>(r % m) : -1;
}

// Draw k (k = 0, 1, ...) of the stream for (seed, step).
uint64_t oracle_draw(uint64_t seed, uint64_t step, uint64_t k) {
  DrawStream s(seed, step);
  s.k = k;
  return s.next();
}

// Random partition of {0..W-1} into W/n groups of n for outer step `step`.
// Fisher-Yates from the top index down, then consecutive chunks of n, each
// chunk listed in ascending worker id.  Returns 0, or 1 if the arguments do
// not describe a partition into equal groups.
int oracle_plan_groups(uint64_t seed, uint64_t step, int32_t W, int32_t n,
                       int32_t* members, int32_t* group_offsets) {
  if (W < 1 || n < 1 || n > W || W % n != 0 || !members || !group_offsets) return 1;
  DrawStream s(seed, step);
  for (int32_t i = 0; i < W; ++i) members[i] = i;
  for (int32_t i = W - 1; i >= 1; --i) {
    int32_t j = static_cast<int32_t>(s.bounded(static_cast<uint64_t>(i) + 1));
    std::swap(members[i], members[j]);
  }
  const int32_t G = W / n;
  for (int32_t g = 0; g < G; ++g) {
    std::sort(members + g * n, members + (g + 1) * n);
    group_offsets[g] = g * n;
  }
  group_offsets[G] = W;
  return 0;
}

// Random pipeline routing (section "Inner optimizer step via dynamic pipeline routing" and the
// appendix algorithm "Random pipeline routing"): for every micro-batch of every step, and for
// every boundary b between pipeline stage b and stage b+1, a fresh random permutation pairs the
// W replicas of stage b with the W replicas of stage b+1, so every replica sends to exactly one
// and receives from exactly one (balanced load), and the backward pass can retrace the path.
//   send_to[b*W + r]   = replica of stage b+1 that replica r of stage b sends its outputs to
//   recv_from[b*W + q] = replica of stage b that replica q of stage b+1 receives its inputs from
// Every worker evaluates this from (seed, step, microbatch) alone; nothing is exchanged.
// The draw stream of boundary b starts at
//   mix64( mix64( mix64(seed ^ mix64(step + G)) ^ mix64(microbatch + 2G) ) ^ mix64(b + 3G) )
// and drives the same top-down Fisher-Yates shuffle as the subgroup planner.
int oracle_plan_routes(uint64_t seed, uint64_t step, uint64_t microbatch, int32_t num_stages,
                       int32_t W, int32_t* send_to, int32_t* recv_from) {
  if (num_stages < 1 || W < 1) return 1;
  if (num_stages > 1 && (!send_to || !recv_from)) return 1;
  const uint64_t step_key = mix64(seed ^ mix64(step + kGolden));
  const uint64_t batch_key = mix64(step_key ^ mix64(microbatch + 2 * kGolden));
  for (int32_t b = 0; b + 1 < num_stages; ++b) {
    DrawStream s(mix64(batch_key ^ mix64(static_cast<uint64_t>(b) + 3 * kGolden)));
    int32_t* to = send_to + static_cast<int64_t>(b) * W;
    int32_t* from = recv_from + static_cast<int64_t>(b) * W;
    for (int32_t r = 0; r < W; ++r) to[r] = r;
    for (int32_t i = W - 1; i >= 1; --i) {
      int32_t j = static_cast<int32_t>(s.bounded(static_cast<uint64_t>(i) + 1));
      std::swap(to[i], to[j]);
    }
    for (int32_t r = 0; r < W; ++r) from[to[r]] = r;
  }
  return 0;
}

void oracle_bf16_narrow(const float* x, uint16_t* out, int64_t count) {
  for (int64_t i = 0; i < count; ++i) out[i] = bf16_narrow(x[i]);
}
void oracle_bf16_widen(const uint16_t* h, float* out, int64_t count) {
  for (int64_t i = 0; i < count; ++i) out[i] = bf16_widen(h[i]);
}

// One outer step in binary32.  phi, delta: [W][stride] float, updated in place.
// theta: [W][stride] of float (theta_is_bf16 == 0) or bf16 bit patterns
// (theta_is_bf16 == 1), read as the fast weights and overwritten with the
// restarted ones.  Segments are element ranges inside one worker's row.
// Groups: any partition of a subset of the workers; workers in no group and
// elements in no segment are left untouched.  Returns 0, or 1 on bad groups.
int oracle_outer_step_f32(float* phi, float* delta, void* theta, int32_t theta_is_bf16,
                          int64_t stride, int32_t W,
                          const int64_t* seg_off, const int64_t* seg_len, int32_t num_segments,
                          float alpha, float beta, float gamma,
                          const int32_t* members, const int32_t* group_offsets, int32_t num_groups) {
  if (!groups_ok(members, group_offsets, num_groups, W)) return 1;
  if (theta_is_bf16) {
    uint16_t* th = static_cast<uint16_t*>(theta);
    outer_step_impl<float>(phi, delta, stride, seg_off, seg_len, num_segments, alpha, beta, gamma,
                           members, group_offsets, num_groups,
                           [th](int64_t at) { return bf16_widen(th[at]); },
                           [th](int64_t at, float v) { th[at] = bf16_narrow(v); });
  } else {
    float* th = static_cast<float*>(theta);
    outer_step_impl<float>(phi, delta, stride, seg_off, seg_len, num_segments, alpha, beta, gamma,
                           members, group_offsets, num_groups,
                           [th](int64_t at) { return th[at]; },
                           [th](int64_t at, float v) { th[at] = v; });
  }
  return 0;
}

// The same step in binary64 (theta held as double; the restart copies phi').
int oracle_outer_step_f64(double* phi, double* delta, double* theta,
                          int64_t stride, int32_t W,
                          const int64_t* seg_off, const int64_t* seg_len, int32_t num_segments,
                          double alpha, double beta, double gamma,
                          const int32_t* members, const int32_t* group_offsets, int32_t num_groups) {
  if (!groups_ok(members, group_offsets, num_groups, W)) return 1;
  outer_step_impl<double>(phi, delta, stride, seg_off, seg_len, num_segments, alpha, beta, gamma,
                          members, group_offsets, num_groups,
                          [theta](int64_t at) { return theta[at]; },
                          [theta](int64_t at, double v) { theta[at] = v; });
  return 0;
}

// Replica spread of x ([W][stride] float, or bf16 bit patterns if x_is_bf16).
// out_std: double[num_segments + 1]: pooled deviation per segment, then over all
// segments.  arithmetic: 0 = binary64 definition, 1 = binary32 per element.
int oracle_replica_spread(const void* x, int32_t x_is_bf16, int64_t stride, int32_t W,
                          const int64_t* seg_off, const int64_t* seg_len, int32_t num_segments,
                          int32_t arithmetic, double* out_std) {
  if (!x || W < 1 || num_segments < 0 || !out_std) return 1;
  const float* xf = static_cast<const float*>(x);
  const uint16_t* xh = static_cast<const uint16_t*>(x);
  if (arithmetic == 0) {
    if (x_is_bf16)
      replica_spread_impl<double>([xh](int64_t at) { return static_cast<double>(bf16_widen(xh[at])); },
                                  stride, W, seg_off, seg_len, num_segments, out_std);
    else
      replica_spread_impl<double>([xf](int64_t at) { return static_cast<double>(xf[at]); },
                                  stride, W, seg_off, seg_len, num_segments, out_std);
  } else {
    if (x_is_bf16)
      replica_spread_impl<float>([xh](int64_t at) { return bf16_widen(xh[at]); },
                                 stride, W, seg_off, seg_len, num_segments, out_std);
    else
      replica_spread_impl<float>([xf](int64_t at) { return xf[at]; },
                                 stride, W, seg_off, seg_len, num_segments, out_std);
  }
  return 0;
}

}  // extern "C"
