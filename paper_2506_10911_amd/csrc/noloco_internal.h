// Types shared by the host side of the library and its kernels (not part of the C ABI).
#pragma once

#include <cstdint>
#include <vector>

#include "noloco.h"

namespace noloco {

constexpr int kBlockThreads = 256;   // four wave64 per workgroup
constexpr int kVecElems = 4;         // one 16-byte fp32 vector per lane and load

// A maximal contiguous run of arena elements, cut into tiles of `tile_elems` columns whose
// boundaries sit at multiples of tile_elems in row coordinates.  The run's first and last
// tile may be partial; all others are whole.
struct Span {
  int64_t col_begin;     // first element of the run (inclusive)
  int64_t col_end;       // one past its last element
  int64_t first_block;   // col_begin / tile_elems
  int64_t tile_prefix;   // number of tiles in all earlier spans
};

// Kernel arguments of one launch: all groups in it have the same size n.
struct StepArgs {
  float* phi;
  float* delta;
  void* theta;
  int64_t stride;          // elements between rows
  const Span* spans;       // device, num_spans + 1 entries (last is a sentinel holding the tile total)
  int32_t num_spans;
  int32_t num_groups;      // groups in this launch
  int64_t num_tiles;       // tiles per group taken by this launch
  int64_t tile_offset;     // first of them: the launch covers tiles [tile_offset, tile_offset + num_tiles)
  float alpha, beta, gamma, inv_n;
  int32_t n;               // group size
  int32_t group_major;     // work item -> (tile, group) order
  int32_t xcd_map;         // workgroup -> work item permutation, see noloco_tuning
  uint32_t work_items;     // num_tiles * num_groups
  int32_t rows[NOLOCO_MAX_GROUP];  // group g = rows[g*n .. g*n+n), ascending worker ids
};

// Kernel arguments of the replica-spread pass (one tile = spread_tile_elems_for(W) columns of ONE tensor).
struct SpreadArgs {
  const void* x;           // [W][stride] float or bf16
  int64_t stride;
  const Span* spans;       // one span per non-empty segment, caller's order, + sentinel
  int32_t num_spans;
  int32_t W;
  float inv_W;
  uint32_t tiles;
  int32_t xcd_map;         // 0 = workgroup i takes tile i, 1 = one contiguous eighth of the tiles per XCD
  double* partials;        // [tiles] sum over the tile's owned columns of the per-column variance
};

// One entry per segment in the caller's order (empty ones included): where its tiles' partial
// sums sit and how many elements it has.
struct SegmentTiles {
  int64_t first_tile;
  int64_t num_tiles;
  int64_t numel;
};

struct KernelChoice {
  int32_t vectors_per_thread;
  int32_t nontemporal;
  int32_t group_major;
  int32_t xcd_map;
};

constexpr uint32_t kXcds = 8;        // MI355X: 8 accelerator dies, workgroups are dealt to them round-robin

// The HIP runtime refuses a launch whose grid.x * block.x exceeds 2^32 - 1.  Launches are cut
// (over groups and over tile ranges) so that a grid stays at or below this many workgroups;
// the margin leaves room for the rounding the XCD maps add.
constexpr int64_t kMaxGridWorkgroups = (0xFFFFFFFFll / kBlockThreads) - 8 * 4096;

// Capacity, in doubles, of the file-scope device array that noloco_replica_spread_noalloc uses
// in place of the plan's own partial-sum buffer (16 MiB per GPU).
constexpr int64_t kSpreadScratchDoubles = 2 * 1024 * 1024;

// host: segment table -> runs (sorted, merged); see noloco_merge_segments
noloco_status merge_segments(const noloco_segment* segments, int32_t num_segments,
                             int64_t worker_stride, std::vector<noloco_segment>* runs);

// host: runs -> spans for a tile size; returns the tile total
int64_t build_spans(const std::vector<noloco_segment>& runs, int32_t tile_elems,
                    std::vector<Span>* spans);

// kernels.hip: enqueue one launch.  Returns hipError_t as int.
int launch_outer_step(const StepArgs& args, int32_t theta_dtype, const KernelChoice& choice,
                      void* stream);
// mode 0 copy, 1 read only (dst = 4-byte sink), 2 fill
int launch_stream_probe(int mode, void* dst, const void* src, int64_t bytes, float value, void* stream);

int launch_replica_spread(const SpreadArgs& args, int32_t x_dtype, const SegmentTiles* seg_tiles,
                          int32_t num_segments, double* out_std, void* stream);

// kernels.hip: address of the current device's copy of the static scratch array (resolved once
// per device and cached).  Returns hipError_t as int; performs no allocation of its own.
int static_spread_scratch(double** out);

// tile size in elements for a kernel choice and group size
int32_t tile_elems_for(int32_t n, int32_t vectors_per_thread);
// tile size of the replica-spread pass for W rows
int32_t spread_tile_elems_for(int32_t W);
bool has_fixed_kernel(int32_t n);

}  // namespace noloco
