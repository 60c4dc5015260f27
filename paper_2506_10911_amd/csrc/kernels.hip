// Fused NoLoCo outer step for gfx950 (arxiv 2506.10911, section "Outer optimizer step with
// modified Nesterov momentum", Eq. 1-3, plus the restart of the fast weights).
//
// The operation is a pure stream: per worker-parameter it reads phi, delta, theta once and
// writes them once, with about ten flops in between, so HBM bandwidth is the only roofline
// that matters.  The kernels are therefore organised around memory access:
//   * one thread owns one 16-byte vector of four consecutive columns of ONE subgroup and
//     does the whole step for all n members of it, so every byte is moved exactly once and
//     the subgroup reduction never leaves registers;
//   * a wave's load instruction covers 1 KiB of consecutive addresses of one row
//     (global_load_dwordx4; 8 bytes per lane for bf16 theta);
//   * all 3*n*U loads of a thread are issued before the first use, to keep enough bytes in
//     flight per CU to cover HBM latency;
//   * a workgroup is one tile (1024*U columns) of one subgroup; tiles whose column range
//     is whole take a branch-free path, the first/last tile of a run takes a path that
//     handles partially owned vectors element by element.
//
// Arithmetic contract (binary32, one rounding per operation, no contraction; this file is
// compiled with -ffp-contract=off), members a = 0..n-1 in ascending worker id:
//   D_a = phi_a - widen(theta_a);  SD = D_0 (+ D_a ...);  SP = phi_0 (+ phi_a ...)
//   mD = SD * inv_n;  mP = SP * inv_n
//   delta'_a = (alpha*delta_a - beta*mD) - gamma*(phi_a - mP)
//   phi'_a = phi_a + delta'_a;  theta'_a = narrow(phi'_a)
#include <hip/hip_runtime.h>

#include <atomic>

#include "noloco_internal.h"

namespace noloco {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned short h4 __attribute__((ext_vector_type(4)));  // four bf16 bit patterns
typedef unsigned int u4 __attribute__((ext_vector_type(4)));

struct Bf16Tag {};  // theta stored as bf16; `float` doubles as the tag for fp32 theta

// bf16 is the upper half of binary32.  Narrowing rounds to nearest, ties to even, by adding
// 0x7FFF plus the lowest kept bit and dropping 16 bits; NaN is kept as a quiet NaN.
__device__ __forceinline__ unsigned int narrow_bits(unsigned int u) {
  const unsigned int r = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
  const unsigned int q = (u >> 16) | 0x0040u;
  return ((u & 0x7FFFFFFFu) > 0x7F800000u) ? q : r;
}

// How `theta` is held in memory for a lane that works on V (f4 = four columns, float = one).
template <typename Tag, typename V> struct ThetaMem;
template <> struct ThetaMem<float, f4> {
  typedef float elem; typedef f4 mem;
  static __device__ __forceinline__ f4 widen(f4 m) { return m; }
  static __device__ __forceinline__ f4 narrow(f4 v) { return v; }
};
template <> struct ThetaMem<float, float> {
  typedef float elem; typedef float mem;
  static __device__ __forceinline__ float widen(float m) { return m; }
  static __device__ __forceinline__ float narrow(float v) { return v; }
};
template <> struct ThetaMem<Bf16Tag, f4> {
  typedef unsigned short elem; typedef h4 mem;
  static __device__ __forceinline__ f4 widen(h4 m) {
    u4 w = __builtin_convertvector(m, u4) << 16;
    return __builtin_bit_cast(f4, w);
  }
  static __device__ __forceinline__ h4 narrow(f4 v) {
    u4 u = __builtin_bit_cast(u4, v);
    u4 r;
    r.x = narrow_bits(u.x); r.y = narrow_bits(u.y); r.z = narrow_bits(u.z); r.w = narrow_bits(u.w);
    return __builtin_convertvector(r, h4);
  }
};
template <> struct ThetaMem<Bf16Tag, float> {
  typedef unsigned short elem; typedef unsigned short mem;
  static __device__ __forceinline__ float widen(unsigned short m) {
    return __uint_as_float(static_cast<unsigned int>(m) << 16);
  }
  static __device__ __forceinline__ unsigned short narrow(float v) {
    return static_cast<unsigned short>(narrow_bits(__float_as_uint(v)));
  }
};

template <bool NT, typename T> __device__ __forceinline__ T ld(const T* p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}
template <bool NT, typename T> __device__ __forceinline__ void st(T* p, T v) {
  if constexpr (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
}

// Enqueue a kernel and return the launch status itself (hipLaunchKernel), so that an error some
// earlier, unrelated call left behind on this thread is neither reported as ours nor cleared.
template <typename T> struct same { typedef T type; };
template <typename... KArgs>
hipError_t enqueue(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t s,
                   typename same<KArgs>::type... args) {
  void* argv[] = {static_cast<void*>(&args)...};
  return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, argv, 0, s);
}

// Which tile of which group this workgroup owns, and that tile's column range.
struct TileRef {
  uint32_t group;
  int64_t base;   // first column of the tile's aligned block
  int64_t c0;     // owned columns are [c0, c1)
  int64_t c1;
};

__device__ __forceinline__ bool locate_tile(const StepArgs& a, int tile_elems, TileRef& r) {
  const uint32_t tiles = static_cast<uint32_t>(a.num_tiles);   // host keeps tiles*groups below the grid limit
  // Workgroup -> work item.  The hardware deals consecutive workgroups to the 8 XCDs in turn,
  // and each XCD's L2 interleaves its 16 channels at 4 KiB; handing an XCD every 8th tile
  // would confine it to a few of its channels, so the map below gives each XCD runs of
  // consecutive tiles instead.
  uint32_t item = blockIdx.x;
  if (a.xcd_map != 0) {
    const uint32_t xcd = item % kXcds, slot = item / kXcds;
    if (a.xcd_map == 1) {
      const uint32_t per_xcd = (a.work_items + kXcds - 1) / kXcds;
      item = xcd * per_xcd + slot;                            // one contiguous range per XCD
    } else {
      const uint32_t c = static_cast<uint32_t>(a.xcd_map);    // runs of c tiles per XCD
      const uint32_t blk = slot / c;
      item = (blk * kXcds + xcd) * c + (slot - blk * c);
    }
    if (item >= a.work_items) return false;
  }
  uint32_t local;
  if (a.group_major) {
    r.group = item / tiles;
    local = item - r.group * tiles;
  } else {
    const uint32_t groups = static_cast<uint32_t>(a.num_groups);
    local = item / groups;
    r.group = item - local * groups;
  }
  const int64_t tile = a.tile_offset + static_cast<int64_t>(local);
  int lo = 0, hi = a.num_spans;             // spans[hi] is the sentinel: its prefix is the tile total
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (a.spans[mid].tile_prefix <= tile) lo = mid; else hi = mid;
  }
  const Span s = a.spans[lo];
  r.base = (s.first_block + (tile - s.tile_prefix)) * tile_elems;
  r.c0 = r.base > s.col_begin ? r.base : s.col_begin;
  const int64_t end = r.base + tile_elems;
  r.c1 = end < s.col_end ? end : s.col_end;
  return true;
}

// Eq. 1-3 and the restart for N members held in registers.  V is f4 or float.
template <int N, typename Tag, typename V>
__device__ __forceinline__ void update_members(V (&p)[N], V (&d)[N],
                                               typename ThetaMem<Tag, V>::mem (&t)[N],
                                               float alpha, float beta, float gamma, float inv_n) {
  typedef ThetaMem<Tag, V> TM;
  V sum_D = p[0] - TM::widen(t[0]);          // Eq. 1, and the two sums of Eq. 2
  V sum_P = p[0];
#pragma unroll
  for (int j = 1; j < N; ++j) {
    const V D = p[j] - TM::widen(t[j]);
    sum_D = sum_D + D;
    sum_P = sum_P + p[j];
  }
  const V mean_P = sum_P * inv_n;
  const V t2 = beta * (sum_D * inv_n);
#pragma unroll
  for (int j = 0; j < N; ++j) {
    const V t1 = alpha * d[j];
    const V t3 = gamma * (p[j] - mean_P);
    const V d_new = (t1 - t2) - t3;          // Eq. 2
    const V p_new = p[j] + d_new;            // Eq. 3
    d[j] = d_new;
    p[j] = p_new;
    t[j] = TM::narrow(p_new);                // restart of the fast weights
  }
}

// One lane's whole step at column `c` for a compile-time group size: load all, update, store all.
template <int N, typename Tag, typename V, bool NT>
__device__ __forceinline__ void step_at(float* const (&P)[N], float* const (&D)[N],
                                        typename ThetaMem<Tag, V>::elem* const (&T)[N], int64_t c,
                                        const StepArgs& a) {
  typedef ThetaMem<Tag, V> TM;
  typedef typename TM::mem TMem;
  V p[N], d[N];
  TMem t[N];
#pragma unroll
  for (int j = 0; j < N; ++j) {
    p[j] = ld<NT>(reinterpret_cast<const V*>(P[j] + c));
    t[j] = ld<NT>(reinterpret_cast<const TMem*>(T[j] + c));
    d[j] = ld<NT>(reinterpret_cast<const V*>(D[j] + c));
  }
  update_members<N, Tag, V>(p, d, t, a.alpha, a.beta, a.gamma, a.inv_n);
#pragma unroll
  for (int j = 0; j < N; ++j) {
    st<NT>(reinterpret_cast<V*>(P[j] + c), p[j]);
    st<NT>(reinterpret_cast<V*>(D[j] + c), d[j]);
    st<NT>(reinterpret_cast<TMem*>(T[j] + c), t[j]);
  }
}

// Register-resident kernel: group size N known at compile time, U vectors per thread.
template <int N, typename Tag, int U, bool NT>
__global__ void __launch_bounds__(kBlockThreads) outer_step_fixed(const StepArgs a) {
  constexpr int kTile = kBlockThreads * kVecElems * U;
  typedef ThetaMem<Tag, f4> TM;
  typedef typename TM::elem TElem;
  typedef typename TM::mem TMem;

  TileRef tr;
  if (!locate_tile(a, kTile, tr)) return;
  float* P[N];
  float* D[N];
  TElem* T[N];
#pragma unroll
  for (int j = 0; j < N; ++j) {
    const int64_t off = static_cast<int64_t>(a.rows[tr.group * N + j]) * a.stride;
    P[j] = a.phi + off;
    D[j] = a.delta + off;
    T[j] = static_cast<TElem*>(a.theta) + off;
  }
  const int64_t lane_col = tr.base + static_cast<int64_t>(threadIdx.x) * kVecElems;

  if (tr.c0 == tr.base && tr.c1 == tr.base + kTile) {
    // Whole tile: every vector is owned entirely.  Loads first, all of them.
    f4 p[U][N], d[U][N];
    TMem t[U][N];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t c = lane_col + u * (kBlockThreads * kVecElems);
#pragma unroll
      for (int j = 0; j < N; ++j) {
        p[u][j] = ld<NT>(reinterpret_cast<const f4*>(P[j] + c));
        t[u][j] = ld<NT>(reinterpret_cast<const TMem*>(T[j] + c));
        d[u][j] = ld<NT>(reinterpret_cast<const f4*>(D[j] + c));
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      update_members<N, Tag, f4>(p[u], d[u], t[u], a.alpha, a.beta, a.gamma, a.inv_n);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t c = lane_col + u * (kBlockThreads * kVecElems);
#pragma unroll
      for (int j = 0; j < N; ++j) {
        st<NT>(reinterpret_cast<f4*>(P[j] + c), p[u][j]);
        st<NT>(reinterpret_cast<f4*>(D[j] + c), d[u][j]);
        st<NT>(reinterpret_cast<TMem*>(T[j] + c), t[u][j]);
      }
    }
    return;
  }

  // First or last tile of a run: a vector may be owned whole, in part, or not at all.
  float* const (&Pc)[N] = P;
  float* const (&Dc)[N] = D;
  TElem* const (&Tc)[N] = T;
  for (int u = 0; u < U; ++u) {
    const int64_t c = lane_col + u * (kBlockThreads * kVecElems);
    if (c >= tr.c0 && c + kVecElems <= tr.c1) {
      step_at<N, Tag, f4, NT>(Pc, Dc, Tc, c, a);
    } else {
      for (int e = 0; e < kVecElems; ++e)
        if (c + e >= tr.c0 && c + e < tr.c1) step_at<N, Tag, float, false>(Pc, Dc, Tc, c + e, a);
    }
  }
}

// Two passes over the members for a group size only known at run time: the first forms the
// two sums, the second re-reads phi, reads delta and writes.  V is f4 or float.  Members are
// taken four at a time with their loads issued together; the sums still run strictly in
// ascending member order.
template <typename Tag, typename V, bool NT>
__device__ __forceinline__ void two_pass_at(const StepArgs& a, const int32_t* rows, int64_t c) {
  typedef ThetaMem<Tag, V> TM;
  typedef typename TM::elem TElem;
  typedef typename TM::mem TMem;
  constexpr int kChunk = 4;
  const int n = a.n;
  TElem* const theta = static_cast<TElem*>(a.theta);
  int64_t at = static_cast<int64_t>(rows[0]) * a.stride + c;
  V sum_P = *reinterpret_cast<const V*>(a.phi + at);              // ordinary loads of phi: read again below
  V sum_D = sum_P - TM::widen(ld<NT>(reinterpret_cast<const TMem*>(theta + at)));
  int j = 1;
  for (; j + kChunk <= n; j += kChunk) {
    V p[kChunk];
    TMem t[kChunk];
#pragma unroll
    for (int k = 0; k < kChunk; ++k) {
      at = static_cast<int64_t>(rows[j + k]) * a.stride + c;
      p[k] = *reinterpret_cast<const V*>(a.phi + at);
      t[k] = ld<NT>(reinterpret_cast<const TMem*>(theta + at));
    }
#pragma unroll
    for (int k = 0; k < kChunk; ++k) {
      sum_D = sum_D + (p[k] - TM::widen(t[k]));
      sum_P = sum_P + p[k];
    }
  }
  for (; j < n; ++j) {
    at = static_cast<int64_t>(rows[j]) * a.stride + c;
    const V p = *reinterpret_cast<const V*>(a.phi + at);
    sum_D = sum_D + (p - TM::widen(ld<NT>(reinterpret_cast<const TMem*>(theta + at))));
    sum_P = sum_P + p;
  }
  const V mean_P = sum_P * a.inv_n;
  const V t2 = a.beta * (sum_D * a.inv_n);
  auto finish = [&](int64_t where, V p, V d) {
    const V t1 = a.alpha * d;
    const V t3 = a.gamma * (p - mean_P);
    const V d_new = (t1 - t2) - t3;
    const V p_new = p + d_new;
    st<NT>(reinterpret_cast<V*>(a.delta + where), d_new);
    st<NT>(reinterpret_cast<V*>(a.phi + where), p_new);
    st<NT>(reinterpret_cast<TMem*>(theta + where), TM::narrow(p_new));
  };
  j = 0;
  for (; j + kChunk <= n; j += kChunk) {
    V p[kChunk], d[kChunk];
    int64_t where[kChunk];
#pragma unroll
    for (int k = 0; k < kChunk; ++k) {
      where[k] = static_cast<int64_t>(rows[j + k]) * a.stride + c;
      p[k] = ld<NT>(reinterpret_cast<const V*>(a.phi + where[k]));
      d[k] = ld<NT>(reinterpret_cast<const V*>(a.delta + where[k]));
    }
#pragma unroll
    for (int k = 0; k < kChunk; ++k) finish(where[k], p[k], d[k]);
  }
  for (; j < n; ++j) {
    at = static_cast<int64_t>(rows[j]) * a.stride + c;
    finish(at, ld<NT>(reinterpret_cast<const V*>(a.phi + at)),
           ld<NT>(reinterpret_cast<const V*>(a.delta + at)));
  }
}

// Subgroups of 32 or 64: too many members to keep phi, delta and theta of all of them in
// registers, but phi alone fits (4 VGPRs per member).  First sweep: load phi and theta of every
// member, keep phi, fold both sums.  Second sweep: load delta, finish, store.  Every byte is
// still moved once.  Partial tiles fall back to the two-pass routine.
template <int N, typename Tag, bool NT>
__global__ void __launch_bounds__(kBlockThreads) outer_step_phi_resident(const StepArgs a) {
  constexpr int kTile = kBlockThreads * kVecElems;
  constexpr int kChunk = 8;
  typedef ThetaMem<Tag, f4> TM;
  typedef typename TM::elem TElem;
  typedef typename TM::mem TMem;
  TileRef tr;
  if (!locate_tile(a, kTile, tr)) return;
  const int32_t* rows = a.rows + tr.group * N;
  const int64_t c = tr.base + static_cast<int64_t>(threadIdx.x) * kVecElems;
  if (tr.c0 == tr.base && tr.c1 == tr.base + kTile) {
    TElem* const theta = static_cast<TElem*>(a.theta);
    f4 p[N];
    f4 sum_D, sum_P;
#pragma unroll
    for (int j0 = 0; j0 < N; j0 += kChunk) {
      TMem t[kChunk];
#pragma unroll
      for (int k = 0; k < kChunk; ++k) {
        const int64_t at = static_cast<int64_t>(rows[j0 + k]) * a.stride + c;
        p[j0 + k] = ld<NT>(reinterpret_cast<const f4*>(a.phi + at));
        t[k] = ld<NT>(reinterpret_cast<const TMem*>(theta + at));
      }
#pragma unroll
      for (int k = 0; k < kChunk; ++k) {
        const f4 D = p[j0 + k] - TM::widen(t[k]);
        if (j0 + k == 0) { sum_D = D; sum_P = p[0]; }
        else { sum_D = sum_D + D; sum_P = sum_P + p[j0 + k]; }
      }
    }
    const f4 mean_P = sum_P * a.inv_n;
    const f4 t2 = a.beta * (sum_D * a.inv_n);
#pragma unroll
    for (int j0 = 0; j0 < N; j0 += kChunk) {
      f4 d[kChunk];
#pragma unroll
      for (int k = 0; k < kChunk; ++k) {
        const int64_t at = static_cast<int64_t>(rows[j0 + k]) * a.stride + c;
        d[k] = ld<NT>(reinterpret_cast<const f4*>(a.delta + at));
      }
#pragma unroll
      for (int k = 0; k < kChunk; ++k) {
        const int64_t at = static_cast<int64_t>(rows[j0 + k]) * a.stride + c;
        const f4 t1 = a.alpha * d[k];
        const f4 t3 = a.gamma * (p[j0 + k] - mean_P);
        const f4 d_new = (t1 - t2) - t3;
        const f4 p_new = p[j0 + k] + d_new;
        st<NT>(reinterpret_cast<f4*>(a.delta + at), d_new);
        st<NT>(reinterpret_cast<f4*>(a.phi + at), p_new);
        st<NT>(reinterpret_cast<TMem*>(theta + at), TM::narrow(p_new));
      }
    }
    return;
  }
  if (c >= tr.c0 && c + kVecElems <= tr.c1) {
    two_pass_at<Tag, f4, NT>(a, rows, c);
  } else {
    for (int e = 0; e < kVecElems; ++e)
      if (c + e >= tr.c0 && c + e < tr.c1) two_pass_at<Tag, float, false>(a, rows, c + e);
  }
}

template <typename Tag, bool NT>
__global__ void __launch_bounds__(kBlockThreads) outer_step_generic(const StepArgs a) {
  constexpr int kTile = kBlockThreads * kVecElems;
  TileRef tr;
  if (!locate_tile(a, kTile, tr)) return;
  const int32_t* rows = a.rows + tr.group * a.n;
  const int64_t c = tr.base + static_cast<int64_t>(threadIdx.x) * kVecElems;
  if (c >= tr.c0 && c + kVecElems <= tr.c1) {
    two_pass_at<Tag, f4, NT>(a, rows, c);
  } else {
    for (int e = 0; e < kVecElems; ++e)
      if (c + e >= tr.c0 && c + e < tr.c1) two_pass_at<Tag, float, false>(a, rows, c + e);
  }
}

// Plain streaming copy: 4 vectors per thread, loads before stores.
__global__ void __launch_bounds__(kBlockThreads) copy_probe_kernel(f4* __restrict__ dst,
                                                                   const f4* __restrict__ src,
                                                                   int64_t vectors) {
  const int64_t first = static_cast<int64_t>(blockIdx.x) * (kBlockThreads * 4) + threadIdx.x;
  f4 v[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int64_t i = first + u * kBlockThreads;
    if (i < vectors) v[u] = __builtin_nontemporal_load(src + i);
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int64_t i = first + u * kBlockThreads;
    if (i < vectors) __builtin_nontemporal_store(v[u], dst + i);
  }
}

// Read-only and write-only counterparts of the copy probe (same grid shape).  The read probe
// folds what it loads into a value that is stored only if it equals a pattern the data never
// produces, so the loads cannot be optimised away and nothing is written.
__global__ void __launch_bounds__(kBlockThreads) read_probe_kernel(const f4* __restrict__ src,
                                                                   int64_t vectors, float* sink) {
  const int64_t first = static_cast<int64_t>(blockIdx.x) * (kBlockThreads * 4) + threadIdx.x;
  f4 acc = {0.f, 0.f, 0.f, 0.f};
  f4 v[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int64_t i = first + u * kBlockThreads;
    v[u] = i < vectors ? __builtin_nontemporal_load(src + i) : acc;
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) acc = acc + v[u];
  if (acc.x == 1.2345e-30f && acc.y == -5.4321e-30f) *sink = acc.z;
}

__global__ void __launch_bounds__(kBlockThreads) fill_probe_kernel(f4* __restrict__ dst,
                                                                   int64_t vectors, float value) {
  const int64_t first = static_cast<int64_t>(blockIdx.x) * (kBlockThreads * 4) + threadIdx.x;
  const f4 v = {value, value, value, value};
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int64_t i = first + u * kBlockThreads;
    if (i < vectors) __builtin_nontemporal_store(v, dst + i);
  }
}

// ---------------------------------------------------------------------------------------
// Replica spread (results section of the paper: standard deviation of the weights across the
// data-parallel replicas).  Read-only pass: per column the population variance over the W
// rows in binary32 (sum in ascending row order, mean = sum * inv_W, then the squared
// deviations summed in the same order, times inv_W), pooled in binary64 per tile in a fixed
// order; two small kernels then pool tiles per tensor and tensors overall and take the roots.
// ---------------------------------------------------------------------------------------

__device__ __forceinline__ double wave_sum_fixed(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_down(v, off, 64);
  return v;                                   // lane 0 holds the total
}

__device__ __forceinline__ double block_sum_fixed(double v, double* wave_part) {
  const double w = wave_sum_fixed(v);
  if ((threadIdx.x & 63) == 0) wave_part[threadIdx.x >> 6] = w;
  __syncthreads();
  return ((wave_part[0] + wave_part[1]) + wave_part[2]) + wave_part[3];   // same value in every thread
}

// Column variance of a lane's four columns from WT rows held in registers.
template <int WT, typename Tag>
__device__ __forceinline__ f4 column_variance_regs(const SpreadArgs& a, int64_t c) {
  typedef ThetaMem<Tag, f4> TM;
  typedef typename TM::elem TElem;
  typedef typename TM::mem TMem;
  const TElem* x = static_cast<const TElem*>(a.x);
  f4 v[WT];
#pragma unroll
  for (int w = 0; w < WT; ++w)
    v[w] = TM::widen(__builtin_nontemporal_load(reinterpret_cast<const TMem*>(x + w * a.stride + c)));
  f4 sum = v[0];
#pragma unroll
  for (int w = 1; w < WT; ++w) sum = sum + v[w];
  const f4 mean = sum * a.inv_W;
  f4 q = (v[0] - mean) * (v[0] - mean);
#pragma unroll
  for (int w = 1; w < WT; ++w) {
    const f4 dev = v[w] - mean;
    q = q + dev * dev;
  }
  return q * a.inv_W;
}

// Any W: two sweeps over memory, four rows at a time.
template <typename Tag>
__device__ __forceinline__ f4 column_variance_mem(const SpreadArgs& a, int64_t c) {
  typedef ThetaMem<Tag, f4> TM;
  typedef typename TM::elem TElem;
  typedef typename TM::mem TMem;
  const TElem* x = static_cast<const TElem*>(a.x);
  auto row = [&](int w) { return TM::widen(*reinterpret_cast<const TMem*>(x + w * a.stride + c)); };
  f4 sum = row(0);
  int w = 1;
  for (; w + 4 <= a.W; w += 4) {
    const f4 r0 = row(w), r1 = row(w + 1), r2 = row(w + 2), r3 = row(w + 3);
    sum = sum + r0; sum = sum + r1; sum = sum + r2; sum = sum + r3;
  }
  for (; w < a.W; ++w) sum = sum + row(w);
  const f4 mean = sum * a.inv_W;
  const f4 d0 = row(0) - mean;
  f4 q = d0 * d0;
  w = 1;
  for (; w + 4 <= a.W; w += 4) {
    const f4 r0 = row(w) - mean, r1 = row(w + 1) - mean, r2 = row(w + 2) - mean, r3 = row(w + 3) - mean;
    q = q + r0 * r0; q = q + r1 * r1; q = q + r2 * r2; q = q + r3 * r3;
  }
  for (; w < a.W; ++w) {
    const f4 dev = row(w) - mean;
    q = q + dev * dev;
  }
  return q * a.inv_W;
}

// WT = 0 selects the any-W routine.  U = 16-byte vectors per thread: a tile is 1024*U columns.
template <int WT, int U, typename Tag>
__global__ void __launch_bounds__(kBlockThreads) replica_spread_tiles(const SpreadArgs a) {
  constexpr int kTile = kBlockThreads * kVecElems * U;
  __shared__ double wave_part[kBlockThreads / 64];
  // Each XCD (workgroups are dealt to the 8 of them in turn) walks one contiguous eighth of the
  // tiles, so that its consecutive row pieces spread over all 16 channels of its L2.
  uint32_t tile = blockIdx.x;
  if (a.xcd_map == 1) {
    const uint32_t per_xcd = (a.tiles + kXcds - 1) / kXcds;
    tile = (tile % kXcds) * per_xcd + tile / kXcds;
    if (tile >= a.tiles) return;
  }
  int lo = 0, hi = a.num_spans;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (a.spans[mid].tile_prefix <= static_cast<int64_t>(tile)) lo = mid; else hi = mid;
  }
  const Span s = a.spans[lo];
  const int64_t base = (s.first_block + (static_cast<int64_t>(tile) - s.tile_prefix)) * kTile;
  const int64_t c0 = base > s.col_begin ? base : s.col_begin;
  const int64_t c1 = base + kTile < s.col_end ? base + kTile : s.col_end;
  double mine = 0.0;
  if (c0 == base && c1 == base + kTile) {     // whole tile: all U vectors' loads can be in flight together
    f4 var[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t c = base + (u * kBlockThreads + static_cast<int64_t>(threadIdx.x)) * kVecElems;
      if constexpr (WT > 0) var[u] = column_variance_regs<WT, Tag>(a, c);
      else var[u] = column_variance_mem<Tag>(a, c);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      mine += ((static_cast<double>(var[u].x) + static_cast<double>(var[u].y)) +
               static_cast<double>(var[u].z)) + static_cast<double>(var[u].w);
  } else {
    for (int u = 0; u < U; ++u) {
      const int64_t c = base + (u * kBlockThreads + static_cast<int64_t>(threadIdx.x)) * kVecElems;
      if (c + kVecElems > c0 && c < c1) {     // the vector overlaps the tensor: load it whole, keep owned lanes
        f4 var;
        if constexpr (WT > 0) var = column_variance_regs<WT, Tag>(a, c);
        else var = column_variance_mem<Tag>(a, c);
        const float e0 = (c + 0 >= c0 && c + 0 < c1) ? var.x : 0.f;
        const float e1 = (c + 1 >= c0 && c + 1 < c1) ? var.y : 0.f;
        const float e2 = (c + 2 >= c0 && c + 2 < c1) ? var.z : 0.f;
        const float e3 = (c + 3 >= c0 && c + 3 < c1) ? var.w : 0.f;
        mine += ((static_cast<double>(e0) + static_cast<double>(e1)) + static_cast<double>(e2)) +
                static_cast<double>(e3);
      }
    }
  }
  const double total = block_sum_fixed(mine, wave_part);
  if (threadIdx.x == 0) a.partials[tile] = total;
}

// Workgroup s pools the tile sums of segment s (thread t takes tiles t, t+256, ...; then a fixed
// tree) and writes that tensor's figure.
__global__ void __launch_bounds__(kBlockThreads) replica_spread_segments(const double* partials,
                                                                         const SegmentTiles* seg,
                                                                         double* out_std, double* seg_sums) {
  __shared__ double wave_part[kBlockThreads / 64];
  const SegmentTiles st = seg[blockIdx.x];
  double acc = 0.0;
  for (int64_t t = threadIdx.x; t < st.num_tiles; t += kBlockThreads) acc += partials[st.first_tile + t];
  const double total = block_sum_fixed(acc, wave_part);
  if (threadIdx.x == 0) {
    seg_sums[blockIdx.x] = total;
    out_std[blockIdx.x] = st.numel > 0 ? sqrt(total / static_cast<double>(st.numel)) : 0.0;
  }
}

// One workgroup pools the per-segment sums (same fixed scheme) for the overall figure.
__global__ void __launch_bounds__(kBlockThreads) replica_spread_total(const SegmentTiles* seg,
                                                                      int32_t num_segments,
                                                                      const double* seg_sums, double* out_std) {
  __shared__ double wave_part[kBlockThreads / 64];
  __shared__ double count_part[kBlockThreads / 64];
  double acc = 0.0, count = 0.0;            // element counts are below 2^53: exact in binary64
  for (int s = threadIdx.x; s < num_segments; s += kBlockThreads) {
    acc += seg_sums[s];
    count += static_cast<double>(seg[s].numel);
  }
  const double total = block_sum_fixed(acc, wave_part);
  const double n = block_sum_fixed(count, count_part);
  if (threadIdx.x == 0) out_std[num_segments] = n > 0.0 ? sqrt(total / n) : 0.0;
}

template <typename Tag>
hipError_t launch_spread_for_dtype(const SpreadArgs& a, hipStream_t s) {
  const dim3 grid(a.xcd_map == 1 ? (a.tiles + kXcds - 1) / kXcds * kXcds : a.tiles), block(kBlockThreads);
  switch (a.W) {   // vectors per thread as in spread_tile_elems_for()
    case 2: return enqueue(replica_spread_tiles<2, 4, Tag>, grid, block, s, a);
    case 4: return enqueue(replica_spread_tiles<4, 4, Tag>, grid, block, s, a);
    case 8: return enqueue(replica_spread_tiles<8, 4, Tag>, grid, block, s, a);
    case 16: return enqueue(replica_spread_tiles<16, 1, Tag>, grid, block, s, a);
    case 32: return enqueue(replica_spread_tiles<32, 1, Tag>, grid, block, s, a);
    case 64: return enqueue(replica_spread_tiles<64, 1, Tag>, grid, block, s, a);
    default: return enqueue(replica_spread_tiles<0, 1, Tag>, grid, block, s, a);
  }
}

template <int N, typename Tag, int U>
hipError_t launch_fixed_nt(const StepArgs& args, bool nt, dim3 grid, hipStream_t s) {
  const dim3 block(kBlockThreads);
  return nt ? enqueue(outer_step_fixed<N, Tag, U, true>, grid, block, s, args)
            : enqueue(outer_step_fixed<N, Tag, U, false>, grid, block, s, args);
}

template <int N, typename Tag>
hipError_t launch_fixed(const StepArgs& args, int u, bool nt, dim3 grid, hipStream_t s) {
  constexpr int kMaxU = N <= 2 ? 4 : (N == 4 ? 2 : 1);
  if constexpr (kMaxU >= 4) if (u == 4) return launch_fixed_nt<N, Tag, 4>(args, nt, grid, s);
  if constexpr (kMaxU >= 2) if (u == 2) return launch_fixed_nt<N, Tag, 2>(args, nt, grid, s);
  return launch_fixed_nt<N, Tag, 1>(args, nt, grid, s);
}

template <typename Tag>
hipError_t launch_for_dtype(const StepArgs& args, const KernelChoice& choice, hipStream_t s) {
  const bool nt = choice.nontemporal != 0;
  const int u = tile_elems_for(args.n, choice.vectors_per_thread) / (kBlockThreads * kVecElems);
  uint32_t wgs = args.work_items;
  if (args.xcd_map == 1) wgs = (wgs + kXcds - 1) / kXcds * kXcds;
  else if (args.xcd_map > 1) {
    const uint32_t round = kXcds * static_cast<uint32_t>(args.xcd_map);
    wgs = (wgs + round - 1) / round * round;
  }
  const dim3 grid(wgs), block(kBlockThreads);
  switch (args.n) {
    case 1: return launch_fixed<1, Tag>(args, u, nt, grid, s);
    case 2: return launch_fixed<2, Tag>(args, u, nt, grid, s);
    case 4: return launch_fixed<4, Tag>(args, u, nt, grid, s);
    case 8: return launch_fixed<8, Tag>(args, u, nt, grid, s);
    case 16: return launch_fixed<16, Tag>(args, u, nt, grid, s);
    case 32:
      return nt ? enqueue(outer_step_phi_resident<32, Tag, true>, grid, block, s, args)
                : enqueue(outer_step_phi_resident<32, Tag, false>, grid, block, s, args);
    case 64:
      return nt ? enqueue(outer_step_phi_resident<64, Tag, true>, grid, block, s, args)
                : enqueue(outer_step_phi_resident<64, Tag, false>, grid, block, s, args);
    default: break;
  }
  return nt ? enqueue(outer_step_generic<Tag, true>, grid, block, s, args)
            : enqueue(outer_step_generic<Tag, false>, grid, block, s, args);
}

// Scratch of noloco_replica_spread_noalloc: tile partial sums, then per-segment sums.  One copy
// per GPU, allocated with the code object and kept until the process ends.  In host code this
// name is only a handle for hipGetSymbolAddress; kernels receive the resolved device address.
static __device__ __align__(256) double spread_scratch[kSpreadScratchDoubles];

constexpr int kMaxDevices = 64;
double* scratch_of_device[kMaxDevices];          // resolved addresses, filled on first use per device
std::atomic<bool> scratch_known[kMaxDevices];

}  // namespace

int launch_outer_step(const StepArgs& args, int32_t theta_dtype, const KernelChoice& choice,
                      void* stream) {
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (args.num_tiles <= 0 || args.num_groups <= 0) return 0;
  const hipError_t e = theta_dtype == NOLOCO_BF16 ? launch_for_dtype<Bf16Tag>(args, choice, s)
                                                  : launch_for_dtype<float>(args, choice, s);
  return static_cast<int>(e);
}

int launch_replica_spread(const SpreadArgs& args, int32_t x_dtype, const SegmentTiles* seg_tiles,
                          int32_t num_segments, double* out_std, void* stream) {
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (args.tiles > 0) {
    const hipError_t e = x_dtype == NOLOCO_BF16 ? launch_spread_for_dtype<Bf16Tag>(args, s)
                                                : launch_spread_for_dtype<float>(args, s);
    if (e != hipSuccess) return static_cast<int>(e);
  }
  double* seg_sums = args.partials + args.tiles;   // per-segment sums are staged behind the tile partials
  if (num_segments > 0) {
    const hipError_t e = enqueue(replica_spread_segments, dim3(static_cast<uint32_t>(num_segments)),
                                 dim3(kBlockThreads), s, static_cast<const double*>(args.partials),
                                 seg_tiles, out_std, seg_sums);
    if (e != hipSuccess) return static_cast<int>(e);
  }
  return static_cast<int>(enqueue(replica_spread_total, dim3(1), dim3(kBlockThreads), s, seg_tiles,
                                  num_segments, static_cast<const double*>(seg_sums), out_std));
}

int static_spread_scratch(double** out) {
  int device = -1;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) return static_cast<int>(e);
  if (device < 0 || device >= kMaxDevices) return static_cast<int>(hipErrorInvalidDevice);
  if (!scratch_known[device].load(std::memory_order_acquire)) {
    // Every GPU holds its own copy of the array at its own address: resolve with that GPU current.
    // Two threads racing here resolve the same address twice, which is harmless.
    void* address = nullptr;
    e = hipGetSymbolAddress(&address, HIP_SYMBOL(spread_scratch));
    if (e != hipSuccess) return static_cast<int>(e);
    if (address == nullptr) return static_cast<int>(hipErrorInvalidSymbol);
    scratch_of_device[device] = static_cast<double*>(address);
    scratch_known[device].store(true, std::memory_order_release);
  }
  *out = scratch_of_device[device];
  return 0;
}

int launch_stream_probe(int mode, void* dst, const void* src, int64_t bytes, float value,
                        void* stream) {
  const int64_t vectors = bytes / 16;
  const int64_t per_block = kBlockThreads * 4;
  const int64_t blocks = (vectors + per_block - 1) / per_block;
  if (blocks > kMaxGridWorkgroups) return static_cast<int>(hipErrorInvalidValue);
  const dim3 grid(static_cast<uint32_t>(blocks)), block(kBlockThreads);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (mode == 0)
    return static_cast<int>(enqueue(copy_probe_kernel, grid, block, s, static_cast<f4*>(dst),
                                    static_cast<const f4*>(src), vectors));
  if (mode == 1)
    return static_cast<int>(enqueue(read_probe_kernel, grid, block, s, static_cast<const f4*>(src),
                                    vectors, static_cast<float*>(dst)));
  return static_cast<int>(enqueue(fill_probe_kernel, grid, block, s, static_cast<f4*>(dst), vectors, value));
}

}  // namespace noloco
