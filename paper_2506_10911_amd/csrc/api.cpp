// C ABI of the NoLoCo outer step: argument checking, the launch plan, and the split of one
// outer step into kernel launches.  All arithmetic of the method is in kernels.hip.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <memory>
#include <new>
#include <vector>

#include "noloco_internal.h"

namespace {

using noloco::Span;

constexpr int32_t kTileSizes[3] = {1024, 2048, 4096};  // kBlockThreads * kVecElems * {1, 2, 4}

// Launch shape for subgroup size n: the caller's explicit choices, else the measured best on
// MI355X.  Pairs stream best with big tiles walked group by group; larger subgroups have
// smaller tiles, which want each XCD on a contiguous range (all 16 of its L2 channels busy)
// and all groups in flight at once.
noloco::KernelChoice resolve(const noloco::KernelChoice& asked, int32_t n, int64_t big_tiles) {
  noloco::KernelChoice c = asked;
  if (c.vectors_per_thread == -1) {
    // `big_tiles` = workgroups the launch would have with 4096-column tiles.  An arena too small
    // to give every CU eight of them is latency-bound, not bandwidth-bound: smaller tiles put
    // more workgroups in flight.
    constexpr int64_t kFill = 256 * 8;
    c.vectors_per_thread = big_tiles >= kFill ? 4 : (2 * big_tiles >= kFill ? 2 : 1);
  }
  if (c.nontemporal == -1) c.nontemporal = 1;
  if (c.group_major == -1) c.group_major = n <= 2 ? 1 : 0;
  if (c.xcd_map == -1) c.xcd_map = n <= 2 ? 0 : 1;
  return c;
}

bool aligned(const void* p, uintptr_t bytes) {
  return (reinterpret_cast<uintptr_t>(p) % bytes) == 0;
}

// Do the byte ranges [a, a + a_bytes) and [b, b + b_bytes) share a byte?
bool overlap(const void* a, uint64_t a_bytes, const void* b, uint64_t b_bytes) {
  const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
  return a0 < b0 + b_bytes && b0 < a0 + a_bytes;
}

}  // namespace

struct noloco_launch_plan {
  int device = -1;
  int32_t W = 0;
  int32_t theta_dtype = 0;
  int64_t stride = 0;
  int64_t elements = 0;                      // real elements per worker
  std::vector<noloco_segment> runs;          // host copy, sorted and merged
  Span* dev_spans = nullptr;                 // one allocation holding the three tables
  int64_t table_offset[3] = {0, 0, 0};       // entry index of each table inside dev_spans
  int64_t tiles[3] = {0, 0, 0};              // tiles per group for each tile size
  noloco::KernelChoice choice{-1, -1, -1, -1};   // -1 = chosen per launch, see resolve()
  // replica-spread pass: per-tensor tiles (unmerged segments), their partial sums
  int32_t num_segments = 0;                  // as given by the caller, empty ones included
  int64_t seg_tiles_total = 0;
  Span* dev_seg_spans = nullptr;             // points into dev_spans
  noloco::SegmentTiles* dev_seg_tiles = nullptr;
  double* dev_partials = nullptr;            // [seg_tiles_total + num_segments]
  int32_t num_seg_spans = 0;

  noloco_launch_plan() = default;
  noloco_launch_plan(const noloco_launch_plan&) = delete;
  noloco_launch_plan& operator=(const noloco_launch_plan&) = delete;
  ~noloco_launch_plan() {
    if (dev_spans != nullptr) (void)hipFree(dev_spans);   // the one device allocation of a plan
  }
};

namespace {

// Builds a plan; may throw std::bad_alloc from the host containers (caught by the C entry point).
noloco_status create_plan(const noloco_arena* arena, noloco_launch_plan** out) {
  std::unique_ptr<noloco_launch_plan> plan(new noloco_launch_plan);
  noloco_status st = noloco::merge_segments(arena->segments, arena->num_segments,
                                            arena->worker_stride, &plan->runs);
  if (st != NOLOCO_OK) return st;
  plan->W = arena->W;
  plan->theta_dtype = arena->theta_dtype;
  plan->stride = arena->worker_stride;
  for (const noloco_segment& r : plan->runs) plan->elements += r.numel;

  std::vector<Span> all, one;
  for (int t = 0; t < 3; ++t) {
    plan->table_offset[t] = static_cast<int64_t>(all.size());
    plan->tiles[t] = noloco::build_spans(plan->runs, kTileSizes[t], &one);
    all.insert(all.end(), one.begin(), one.end());
  }
  // Table for the replica-spread pass: one span per non-empty segment in the caller's order,
  // cut into tiles of its own, so that every tile lies inside one tensor.
  plan->num_segments = arena->num_segments;
  std::vector<noloco_segment> nonempty;
  std::vector<noloco::SegmentTiles> seg_tiles(static_cast<size_t>(arena->num_segments));
  for (int32_t i = 0; i < arena->num_segments; ++i)
    if (arena->segments[i].numel > 0) nonempty.push_back(arena->segments[i]);
  const int64_t seg_span_offset = static_cast<int64_t>(all.size());
  plan->seg_tiles_total = noloco::build_spans(nonempty, noloco::spread_tile_elems_for(arena->W), &one);
  plan->num_seg_spans = static_cast<int32_t>(nonempty.size());
  all.insert(all.end(), one.begin(), one.end());
  for (int32_t i = 0, k = 0; i < arena->num_segments; ++i) {
    noloco::SegmentTiles& tiles = seg_tiles[static_cast<size_t>(i)];
    tiles.numel = arena->segments[i].numel;
    if (tiles.numel > 0) {
      tiles.first_tile = one[static_cast<size_t>(k)].tile_prefix;
      tiles.num_tiles = one[static_cast<size_t>(k) + 1].tile_prefix - tiles.first_tile;
      ++k;
    } else {
      tiles.first_tile = tiles.num_tiles = 0;
    }
  }
  if (plan->seg_tiles_total > noloco::kMaxGridWorkgroups) return NOLOCO_ERR_UNSUPPORTED;

  // One device allocation: span tables, per-segment tile ranges, partial sums.
  const size_t spans_bytes = (all.size() * sizeof(Span) + 255) / 256 * 256;
  const size_t segs_bytes = (seg_tiles.size() * sizeof(noloco::SegmentTiles) + 255) / 256 * 256;
  const size_t partial_bytes =
      static_cast<size_t>(plan->seg_tiles_total + plan->num_segments + 1) * sizeof(double);
  char* block = nullptr;
  if (hipGetDevice(&plan->device) != hipSuccess ||
      hipMalloc(reinterpret_cast<void**>(&block), spans_bytes + segs_bytes + partial_bytes) != hipSuccess)
    return NOLOCO_ERR_DEVICE;
  plan->dev_spans = reinterpret_cast<Span*>(block);        // owned from here on (freed by ~noloco_launch_plan)
  plan->dev_seg_spans = plan->dev_spans + seg_span_offset;
  plan->dev_seg_tiles = reinterpret_cast<noloco::SegmentTiles*>(block + spans_bytes);
  plan->dev_partials = reinterpret_cast<double*>(block + spans_bytes + segs_bytes);
  // Synchronous copies from pageable memory: the tables are final when create returns.
  if (hipMemcpy(plan->dev_spans, all.data(), all.size() * sizeof(Span), hipMemcpyHostToDevice) != hipSuccess ||
      (!seg_tiles.empty() &&
       hipMemcpy(plan->dev_seg_tiles, seg_tiles.data(), seg_tiles.size() * sizeof(noloco::SegmentTiles),
                 hipMemcpyHostToDevice) != hipSuccess))
    return NOLOCO_ERR_DEVICE;
  // Resolve this GPU's static scratch array now, at set-up, so that noloco_replica_spread_noalloc
  // finds the address cached.  A failure here only matters to that entry point, which reports it.
  double* unused = nullptr;
  (void)noloco::static_spread_scratch(&unused);
  *out = plan.release();
  return NOLOCO_OK;
}

}  // namespace

extern "C" noloco_status noloco_launch_plan_create(const noloco_arena* arena,
                                                   noloco_launch_plan** out) {
  if (out == nullptr) return NOLOCO_ERR_NULL;
  *out = nullptr;
  if (arena == nullptr) return NOLOCO_ERR_NULL;
  if (arena->phi == nullptr || arena->delta == nullptr || arena->theta == nullptr)
    return NOLOCO_ERR_NULL;
  if (arena->W < 1 || arena->worker_stride < 0 || arena->num_segments < 0)
    return NOLOCO_ERR_INVALID_ARG;
  if (arena->W > NOLOCO_MAX_WORKERS) return NOLOCO_ERR_UNSUPPORTED;
  if (arena->theta_dtype != NOLOCO_F32 && arena->theta_dtype != NOLOCO_BF16)
    return NOLOCO_ERR_INVALID_ARG;
  if (!aligned(arena->phi, NOLOCO_BASE_ALIGN_BYTES) || !aligned(arena->delta, NOLOCO_BASE_ALIGN_BYTES) ||
      !aligned(arena->theta, NOLOCO_BASE_ALIGN_BYTES) ||
      arena->worker_stride % NOLOCO_STRIDE_ALIGN_ELEMS != 0)
    return NOLOCO_ERR_ALIGNMENT;
  try {
    return create_plan(arena, out);
  } catch (const std::bad_alloc&) {
    return NOLOCO_ERR_NO_MEMORY;
  } catch (...) {
    return NOLOCO_ERR_INVALID_ARG;
  }
}

extern "C" noloco_status noloco_launch_plan_destroy(noloco_launch_plan* plan) {
  if (plan == nullptr) return NOLOCO_OK;
  noloco_status st = NOLOCO_OK;
  if (plan->dev_spans != nullptr) {
    if (hipFree(plan->dev_spans) != hipSuccess) st = NOLOCO_ERR_DEVICE;
    plan->dev_spans = nullptr;
  }
  delete plan;
  return st;
}

extern "C" noloco_status noloco_launch_plan_tune(noloco_launch_plan* plan,
                                                 const noloco_tuning* tuning) {
  if (plan == nullptr || tuning == nullptr) return NOLOCO_ERR_NULL;
  const int32_t v = tuning->vectors_per_thread;
  if (v != -1 && v != 1 && v != 2 && v != 4) return NOLOCO_ERR_INVALID_ARG;
  if (tuning->nontemporal < -1 || tuning->nontemporal > 1) return NOLOCO_ERR_INVALID_ARG;
  if (tuning->group_major < -1 || tuning->group_major > 1) return NOLOCO_ERR_INVALID_ARG;
  if (tuning->xcd_map < -1 || tuning->xcd_map > 4096) return NOLOCO_ERR_INVALID_ARG;
  plan->choice = noloco::KernelChoice{v, tuning->nontemporal, tuning->group_major, tuning->xcd_map};
  return NOLOCO_OK;
}

extern "C" noloco_status noloco_launch_plan_info(const noloco_launch_plan* plan,
                                                 int64_t* elements_per_worker, int32_t* num_runs,
                                                 int64_t* num_tiles, int32_t* tile_elems) {
  if (plan == nullptr) return NOLOCO_ERR_NULL;
  const int32_t te = noloco::tile_elems_for(2, resolve(plan->choice, 2, plan->tiles[2] * (plan->W / 2)).vectors_per_thread);
  int t = 0;
  while (kTileSizes[t] != te) ++t;
  if (elements_per_worker) *elements_per_worker = plan->elements;
  if (num_runs) *num_runs = static_cast<int32_t>(plan->runs.size());
  if (num_tiles) *num_tiles = plan->tiles[t];
  if (tile_elems) *tile_elems = te;
  return NOLOCO_OK;
}

namespace {

// Sorted member lists of the groups of one size, gathered into the member table of a launch and
// flushed (one kernel launch per tile range) whenever the table or the grid is full.
struct LaunchBatch {
  noloco::StepArgs args;
  noloco::KernelChoice choice;
  int32_t theta_dtype;
  void* stream;
  int64_t tiles_total;       // tiles per group for this tile size
  int32_t groups = 0;        // groups gathered so far
  int32_t capacity = 0;      // groups one launch may hold

  noloco_status flush() {
    if (groups == 0) return NOLOCO_OK;
    // A launch holds at most kMaxGridWorkgroups work items: all tiles of `groups` groups if they
    // fit, else a range of tiles at a time.
    const int64_t tiles_per_launch = std::min<int64_t>(tiles_total, noloco::kMaxGridWorkgroups / groups);
    args.num_groups = groups;
    for (int64_t t0 = 0; t0 < tiles_total; t0 += tiles_per_launch) {
      args.tile_offset = t0;
      args.num_tiles = std::min(tiles_per_launch, tiles_total - t0);
      args.work_items = static_cast<uint32_t>(args.num_tiles * groups);
      if (noloco::launch_outer_step(args, theta_dtype, choice, stream) != 0) return NOLOCO_ERR_DEVICE;
    }
    groups = 0;
    return NOLOCO_OK;
  }
};

}  // namespace

extern "C" noloco_status noloco_outer_step(const noloco_launch_plan* plan, const noloco_arena* arena,
                                           const noloco_hparams* hparams, const int32_t* members,
                                           const int32_t* group_offsets, int32_t num_groups,
                                           void* hip_stream) {
  // No heap allocation and nothing that can throw on this path: all scratch is on the stack.
  if (plan == nullptr || arena == nullptr || hparams == nullptr) return NOLOCO_ERR_NULL;
  if (arena->phi == nullptr || arena->delta == nullptr || arena->theta == nullptr)
    return NOLOCO_ERR_NULL;
  if (num_groups < 0) return NOLOCO_ERR_INVALID_ARG;
  if (num_groups > 0 && (members == nullptr || group_offsets == nullptr)) return NOLOCO_ERR_NULL;
  if (arena->W != plan->W || arena->worker_stride != plan->stride ||
      arena->theta_dtype != plan->theta_dtype)
    return NOLOCO_ERR_INVALID_ARG;
  if (!aligned(arena->phi, NOLOCO_BASE_ALIGN_BYTES) || !aligned(arena->delta, NOLOCO_BASE_ALIGN_BYTES) ||
      !aligned(arena->theta, NOLOCO_BASE_ALIGN_BYTES))
    return NOLOCO_ERR_ALIGNMENT;
  {
    // The step is in place and every array is both read and written: the three must be disjoint.
    const uint64_t elems = static_cast<uint64_t>(plan->W) * static_cast<uint64_t>(plan->stride);
    const uint64_t f32_bytes = elems * 4, theta_bytes = elems * (plan->theta_dtype == NOLOCO_BF16 ? 2 : 4);
    if (overlap(arena->phi, f32_bytes, arena->delta, f32_bytes) ||
        overlap(arena->phi, f32_bytes, arena->theta, theta_bytes) ||
        overlap(arena->delta, f32_bytes, arena->theta, theta_bytes))
      return NOLOCO_ERR_INVALID_ARG;
  }

  // Validate the grouping completely before anything is launched.  `seen` is a bitmap over the
  // workers (plan creation bounds W by NOLOCO_MAX_WORKERS); `count_of_size[n]` counts groups of size n.
  if (num_groups > 0 && group_offsets[0] != 0) return NOLOCO_ERR_BAD_GROUPING;
  uint64_t seen[NOLOCO_MAX_WORKERS / 64];
  std::memset(seen, 0, (static_cast<size_t>(plan->W) + 63) / 64 * sizeof(uint64_t));
  int32_t count_of_size[NOLOCO_MAX_GROUP + 1];
  std::memset(count_of_size, 0, sizeof(count_of_size));
  bool too_large = false, any = false;
  for (int32_t g = 0; g < num_groups; ++g) {
    const int32_t lo = group_offsets[g], hi = group_offsets[g + 1];
    if (hi < lo) return NOLOCO_ERR_BAD_GROUPING;
    for (int32_t a = lo; a < hi; ++a) {
      const int32_t w = members[a];
      if (w < 0 || w >= plan->W) return NOLOCO_ERR_BAD_GROUPING;
      const uint64_t bit = 1ull << (w & 63);
      if (seen[w >> 6] & bit) return NOLOCO_ERR_BAD_GROUPING;
      seen[w >> 6] |= bit;
    }
    const int32_t n = hi - lo;
    if (n > NOLOCO_MAX_GROUP) too_large = true;
    else if (n > 0) { ++count_of_size[n]; any = true; }
  }
  if (too_large) return NOLOCO_ERR_UNSUPPORTED;
  if (plan->elements == 0 || !any) return NOLOCO_OK;

  int device = -1;
  if (hipGetDevice(&device) != hipSuccess) return NOLOCO_ERR_DEVICE;
  if (device != plan->device) return NOLOCO_ERR_INVALID_ARG;

  LaunchBatch batch;
  std::memset(&batch.args, 0, sizeof(batch.args));
  batch.theta_dtype = plan->theta_dtype;
  batch.stream = hip_stream;
  noloco::StepArgs& args = batch.args;
  args.phi = arena->phi;
  args.delta = arena->delta;
  args.theta = arena->theta;
  args.stride = plan->stride;
  args.num_spans = static_cast<int32_t>(plan->runs.size());
  args.alpha = hparams->alpha;
  args.beta = hparams->beta;
  args.gamma = hparams->gamma;

  // One pass over the groups per distinct size, sizes ascending; a launch takes as many groups
  // as its member table (NOLOCO_MAX_GROUP rows) holds.
  for (int32_t n = 1; n <= NOLOCO_MAX_GROUP; ++n) {
    if (count_of_size[n] == 0) continue;
    batch.choice = resolve(plan->choice, n, plan->tiles[2] * count_of_size[n]);
    args.group_major = batch.choice.group_major;
    args.xcd_map = batch.choice.xcd_map;
    const int32_t te = noloco::tile_elems_for(n, batch.choice.vectors_per_thread);
    int t = 0;
    while (kTileSizes[t] != te) ++t;
    args.spans = plan->dev_spans + plan->table_offset[t];
    batch.tiles_total = plan->tiles[t];
    args.n = n;
    args.inv_n = 1.0f / static_cast<float>(n);
    batch.capacity = NOLOCO_MAX_GROUP / n;
    int32_t left = count_of_size[n];
    for (int32_t g = 0; g < num_groups && left > 0; ++g) {
      const int32_t lo = group_offsets[g];
      if (group_offsets[g + 1] - lo != n) continue;
      int32_t* rows = args.rows + static_cast<size_t>(batch.groups) * n;
      std::memcpy(rows, members + lo, static_cast<size_t>(n) * sizeof(int32_t));
      std::sort(rows, rows + n);                       // sums run in ascending worker id
      --left;
      if (++batch.groups == batch.capacity) {
        const noloco_status st = batch.flush();
        if (st != NOLOCO_OK) return st;
      }
    }
    const noloco_status st = batch.flush();
    if (st != NOLOCO_OK) return st;
  }
  return NOLOCO_OK;
}

namespace {

// Common body of the two replica-spread entry points: `partials` is where the per-tile and
// per-segment sums are staged (the plan's own buffer, or the static per-GPU array).
noloco_status spread_into(const noloco_launch_plan* plan, const void* x_device, int32_t x_dtype,
                          double* out_std_device, double* partials, void* hip_stream) {
  noloco::SpreadArgs args;
  args.x = x_device;
  args.stride = plan->stride;
  args.spans = plan->dev_seg_spans;
  args.num_spans = plan->num_seg_spans;
  args.W = plan->W;
  args.inv_W = 1.0f / static_cast<float>(plan->W);
  args.tiles = static_cast<uint32_t>(plan->seg_tiles_total);
  args.partials = partials;
  args.xcd_map = plan->choice.xcd_map == 0 ? 0 : 1;   // automatic (-1) = contiguous per XCD
  return noloco::launch_replica_spread(args, x_dtype, plan->dev_seg_tiles, plan->num_segments,
                                       out_std_device, hip_stream) == 0
             ? NOLOCO_OK : NOLOCO_ERR_DEVICE;
}

noloco_status check_spread_args(const noloco_launch_plan* plan, const void* x_device, int32_t x_dtype,
                                const double* out_std_device) {
  if (plan == nullptr || x_device == nullptr || out_std_device == nullptr) return NOLOCO_ERR_NULL;
  if (x_dtype != NOLOCO_F32 && x_dtype != NOLOCO_BF16) return NOLOCO_ERR_INVALID_ARG;
  if (!aligned(x_device, NOLOCO_BASE_ALIGN_BYTES) || !aligned(out_std_device, 8))
    return NOLOCO_ERR_ALIGNMENT;
  int device = -1;
  if (hipGetDevice(&device) != hipSuccess) return NOLOCO_ERR_DEVICE;
  if (device != plan->device) return NOLOCO_ERR_INVALID_ARG;
  return NOLOCO_OK;
}

}  // namespace

extern "C" noloco_status noloco_replica_spread(const noloco_launch_plan* plan, const void* x_device,
                                               int32_t x_dtype, double* out_std_device,
                                               void* hip_stream) {
  const noloco_status st = check_spread_args(plan, x_device, x_dtype, out_std_device);
  if (st != NOLOCO_OK) return st;
  return spread_into(plan, x_device, x_dtype, out_std_device, plan->dev_partials, hip_stream);
}

extern "C" noloco_status noloco_replica_spread_noalloc(const noloco_launch_plan* plan,
                                                       const void* x_device, int32_t x_dtype,
                                                       double* out_std_device, void* hip_stream) {
  const noloco_status st = check_spread_args(plan, x_device, x_dtype, out_std_device);
  if (st != NOLOCO_OK) return st;
  // tile sums, then per-segment sums, then one spare slot: same staging as the plan's buffer
  if (plan->seg_tiles_total + plan->num_segments + 1 > noloco::kSpreadScratchDoubles)
    return NOLOCO_ERR_UNSUPPORTED;
  double* scratch = nullptr;
  if (noloco::static_spread_scratch(&scratch) != 0 || scratch == nullptr) return NOLOCO_ERR_DEVICE;
  // Nothing has to start at zero: every slot that is read is written first by this call's kernels.
  return spread_into(plan, x_device, x_dtype, out_std_device, scratch, hip_stream);
}

extern "C" noloco_status noloco_copy_probe(void* dst_device, const void* src_device, int64_t bytes,
                                           void* hip_stream) {
  if (dst_device == nullptr || src_device == nullptr) return NOLOCO_ERR_NULL;
  if (bytes < 0 || bytes % 16 != 0) return NOLOCO_ERR_INVALID_ARG;
  if (!aligned(dst_device, 16) || !aligned(src_device, 16)) return NOLOCO_ERR_ALIGNMENT;
  if (bytes == 0) return NOLOCO_OK;
  return noloco::launch_stream_probe(0, dst_device, src_device, bytes, 0.f, hip_stream) == 0
             ? NOLOCO_OK : NOLOCO_ERR_DEVICE;
}

extern "C" noloco_status noloco_read_probe(const void* src_device, int64_t bytes, void* sink_device,
                                           void* hip_stream) {
  if (src_device == nullptr || sink_device == nullptr) return NOLOCO_ERR_NULL;
  if (bytes < 0 || bytes % 16 != 0) return NOLOCO_ERR_INVALID_ARG;
  if (!aligned(src_device, 16) || !aligned(sink_device, 4)) return NOLOCO_ERR_ALIGNMENT;
  if (bytes == 0) return NOLOCO_OK;
  return noloco::launch_stream_probe(1, sink_device, src_device, bytes, 0.f, hip_stream) == 0
             ? NOLOCO_OK : NOLOCO_ERR_DEVICE;
}

extern "C" noloco_status noloco_fill_probe(void* dst_device, int64_t bytes, float value,
                                           void* hip_stream) {
  if (dst_device == nullptr) return NOLOCO_ERR_NULL;
  if (bytes < 0 || bytes % 16 != 0) return NOLOCO_ERR_INVALID_ARG;
  if (!aligned(dst_device, 16)) return NOLOCO_ERR_ALIGNMENT;
  if (bytes == 0) return NOLOCO_OK;
  return noloco::launch_stream_probe(2, dst_device, nullptr, bytes, value, hip_stream) == 0
             ? NOLOCO_OK : NOLOCO_ERR_DEVICE;
}

extern "C" const char* noloco_strerror(noloco_status status) {
  switch (status) {
    case NOLOCO_OK: return "ok";
    case NOLOCO_ERR_NULL: return "a required pointer is null";
    case NOLOCO_ERR_INVALID_ARG: return "invalid argument";
    case NOLOCO_ERR_BAD_GROUPING: return "groups are not a valid partition";
    case NOLOCO_ERR_SEGMENT_OVERLAP: return "segments overlap or leave the row";
    case NOLOCO_ERR_ALIGNMENT: return "base pointer or worker stride misaligned";
    case NOLOCO_ERR_DEVICE: return "HIP runtime error";
    case NOLOCO_ERR_UNSUPPORTED: return "documented limit exceeded";
    case NOLOCO_ERR_NO_MEMORY: return "host memory allocation failed";
  }
  return "unknown status";
}
