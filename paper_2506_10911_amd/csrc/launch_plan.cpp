// Multi-tensor dispatch, host side: segment table -> contiguous runs -> tile spans.
//
// The arena of one worker is a row of `worker_stride` elements in which the tensors occupy
// arbitrary, possibly odd-sized and odd-placed ranges.  Touching ranges are merged into runs so
// that a tight-packed arena of thousands of tensors becomes a single stream; every run is
// then cut at multiples of the tile size (in row coordinates, so interior tiles start on
// 16-byte vector boundaries whatever the run's own start is).
#include <algorithm>
#include <new>

#include "noloco_internal.h"

namespace noloco {

noloco_status merge_segments(const noloco_segment* segments, int32_t num_segments,
                             int64_t worker_stride, std::vector<noloco_segment>* runs) {
  runs->clear();
  if (num_segments < 0 || worker_stride < 0) return NOLOCO_ERR_INVALID_ARG;
  if (num_segments > 0 && segments == nullptr) return NOLOCO_ERR_NULL;

  std::vector<noloco_segment> sorted;
  sorted.reserve(static_cast<size_t>(num_segments));
  for (int32_t s = 0; s < num_segments; ++s) {
    const noloco_segment& seg = segments[s];
    if (seg.offset < 0 || seg.numel < 0) return NOLOCO_ERR_INVALID_ARG;
    if (seg.numel > worker_stride || seg.offset > worker_stride - seg.numel)
      return NOLOCO_ERR_SEGMENT_OVERLAP;  // leaves the row
    if (seg.numel > 0) sorted.push_back(seg);
  }
  std::sort(sorted.begin(), sorted.end(), [](const noloco_segment& a, const noloco_segment& b) {
    return a.offset < b.offset;
  });
  for (const noloco_segment& seg : sorted) {
    if (!runs->empty()) {
      noloco_segment& last = runs->back();
      const int64_t last_end = last.offset + last.numel;
      if (seg.offset < last_end) return NOLOCO_ERR_SEGMENT_OVERLAP;
      if (seg.offset == last_end) {
        last.numel += seg.numel;
        continue;
      }
    }
    runs->push_back(seg);
  }
  return NOLOCO_OK;
}

int64_t build_spans(const std::vector<noloco_segment>& runs, int32_t tile_elems,
                    std::vector<Span>* spans) {
  spans->clear();
  int64_t tiles = 0;
  for (const noloco_segment& run : runs) {
    Span sp;
    sp.col_begin = run.offset;
    sp.col_end = run.offset + run.numel;
    sp.first_block = sp.col_begin / tile_elems;
    sp.tile_prefix = tiles;
    const int64_t last_block = (sp.col_end - 1) / tile_elems;
    tiles += last_block - sp.first_block + 1;
    spans->push_back(sp);
  }
  Span sentinel;
  sentinel.col_begin = sentinel.col_end = sentinel.first_block = 0;
  sentinel.tile_prefix = tiles;
  spans->push_back(sentinel);
  return tiles;
}

// Tile shapes of the kernels (kernels.hip instantiates exactly these).
int32_t spread_tile_elems_for(int32_t W) {
  const int32_t u = (W == 2 || W == 4 || W == 8) ? 4 : 1;   // W = 16 measured faster with 1 than with 2
  return kBlockThreads * kVecElems * u;
}

bool has_fixed_kernel(int32_t n) { return n == 1 || n == 2 || n == 4 || n == 8 || n == 16; }

int32_t tile_elems_for(int32_t n, int32_t vectors_per_thread) {
  int32_t u = 1;
  if (has_fixed_kernel(n)) {
    const int32_t max_u = n <= 2 ? 4 : (n == 4 ? 2 : 1);
    u = vectors_per_thread < max_u ? vectors_per_thread : max_u;
  }
  return kBlockThreads * kVecElems * u;
}

}  // namespace noloco

extern "C" noloco_status noloco_merge_segments(const noloco_segment* segments, int32_t num_segments,
                                               int64_t worker_stride, noloco_segment* runs_out,
                                               int32_t* num_runs) {
  if (num_runs == nullptr) return NOLOCO_ERR_NULL;
  *num_runs = 0;
  try {
    std::vector<noloco_segment> runs;
    noloco_status st = noloco::merge_segments(segments, num_segments, worker_stride, &runs);
    if (st != NOLOCO_OK) return st;
    *num_runs = static_cast<int32_t>(runs.size());
    if (runs_out != nullptr) std::copy(runs.begin(), runs.end(), runs_out);
    return NOLOCO_OK;
  } catch (const std::bad_alloc&) {      // no exception leaves the C ABI
    return NOLOCO_ERR_NO_MEMORY;
  } catch (...) {
    return NOLOCO_ERR_INVALID_ARG;
  }
}
