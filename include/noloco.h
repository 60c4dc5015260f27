/*
 * noloco.h - C ABI of the NoLoCo outer optimizer step for AMD MI355X (gfx950).
 *
 * Method: arxiv 2506.10911, section "Outer optimizer step with modified Nesterov
 * momentum".  W worker replicas of one pipeline stage's parameters live stacked in one
 * GPU's HBM; an outer step partitions the workers into random subgroups and applies,
 * per subgroup G of size n and per parameter k,
 *
 *   Eq. 1   Delta_j  = phi_j - theta_j                       (j in G; outer weights minus
 *                                                             local weights after the inner steps)
 *           The paper prints Eq. 1 with the opposite sign and then subtracts the term in Eq. 2;
 *           taken literally that moves phi away from theta.  The sign used here ("outer minus
 *           local", DiLoCo's convention) is the one under which Eq. 2 descends, reduces to
 *           DiLoCo's outer step when the subgroup is all workers, and reproduces the
 *           contraction factor of the paper's own convergence analysis.
 *   Eq. 2   delta'_i = alpha*delta_i - (beta/n)*sum_j Delta_j
 *                      - gamma*(phi_i - (1/n)*sum_j phi_j)   (i in G, j over all of G, i included)
 *   Eq. 3   phi'_i   = phi_i + delta'_i
 *   restart theta'_i = phi'_i   (the next inner phase starts from the slow weights;
 *                                rounded to nearest-even when theta is stored as bf16)
 *
 * in place, in IEEE binary32 with one rounding per operation (no fused multiply-add),
 * sums taken in ascending worker order.
 *
 * Conventions for every entry point
 *   - returns a noloco_status; never throws (no C++ exception crosses this boundary: a failed
 *     host allocation comes back as NOLOCO_ERR_NO_MEMORY), never aborts, never prints;
 *   - all pointers are borrowed: the caller owns every host array and every device
 *     buffer; host arrays may be freed as soon as the call returns;
 *   - "device" pointers are HIP device memory of the GPU that is current when the
 *     launch plan is created; "host" pointers are ordinary process memory;
 *   - GPU work is enqueued on the caller's stream and is NOT synchronised;
 *   - the library keeps no global state; a launch plan is immutable after creation
 *     (except through noloco_launch_plan_tune) and noloco_outer_step may use one plan from
 *     several threads.
 */
#ifndef NOLOCO_H_
#define NOLOCO_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum noloco_status {
  NOLOCO_OK = 0,
  NOLOCO_ERR_NULL = 1,            /* a required pointer is null */
  NOLOCO_ERR_INVALID_ARG = 2,     /* a size, dtype or layout field is out of range, or does not match the plan */
  NOLOCO_ERR_BAD_GROUPING = 3,    /* groups are not a partition of a subset of the workers / W not divisible by n */
  NOLOCO_ERR_SEGMENT_OVERLAP = 4, /* two segments share an element, or a segment leaves the row */
  NOLOCO_ERR_ALIGNMENT = 5,       /* a base pointer or the worker stride is not aligned as required */
  NOLOCO_ERR_DEVICE = 6,          /* the HIP runtime reported an error */
  NOLOCO_ERR_UNSUPPORTED = 7,     /* a documented limit is exceeded (e.g. a group larger than NOLOCO_MAX_GROUP) */
  NOLOCO_ERR_NO_MEMORY = 8        /* a host-side allocation failed while building a plan or a simulation */
} noloco_status;

typedef enum noloco_dtype { NOLOCO_F32 = 0, NOLOCO_BF16 = 1 } noloco_dtype;

/* Largest subgroup one call can handle (its member list travels in the kernel arguments). */
#define NOLOCO_MAX_GROUP 256
/* Largest number of worker rows a launch plan accepts (NOLOCO_ERR_UNSUPPORTED beyond it). */
#define NOLOCO_MAX_WORKERS 65536
/* Required alignment of phi/delta/theta base addresses, in bytes, and of worker_stride, in elements. */
#define NOLOCO_BASE_ALIGN_BYTES 256
#define NOLOCO_STRIDE_ALIGN_ELEMS 64

/*
 * Subgroup sampling (section "Outer optimizer step ...": a random subgroup of n of the
 * N instances, re-sampled every iteration; section "Inner optimizer step ...": groups
 * come from random permutations).  Host only, integers only, a pure function of its
 * arguments, so a resumed run replays the same groups.
 *
 * The permutation is a Fisher-Yates shuffle (index W-1 down to 1, partner drawn from
 * [0, i]) driven by SplitMix64 started at mix64(seed ^ mix64(step + 0x9E3779B97F4A7C15)),
 * with rejection of the lowest (2^64 mod m) draws for an unbiased partner; the shuffled
 * list is cut into consecutive chunks of n and every chunk is sorted ascending.
 *
 *   seed, step     any 64-bit values (step = outer iteration counter t)
 *   W              number of workers, >= 1
 *   n              subgroup size, 1 <= n <= W, must divide W (else NOLOCO_ERR_BAD_GROUPING)
 *   members        host, out, int32[W]: worker ids, group g is members[g*n .. g*n+n)
 *   group_offsets  host, out, int32[W/n + 1]: group_offsets[g] = g*n
 */
noloco_status noloco_plan_groups(uint64_t seed, uint64_t step, int32_t W, int32_t n,
                                 int32_t* members, int32_t* group_offsets);

/*
 * Random pipeline routing plan (section "Inner optimizer step via dynamic pipeline routing";
 * appendix algorithm "Random pipeline routing", its RandomRank): for one micro-batch of one
 * step, and for every boundary b between pipeline stage b and stage b+1, a fresh uniformly
 * random permutation pairs the W data-parallel replicas of stage b with those of stage b+1.
 * Every replica sends to exactly one and receives from exactly one replica, so load is
 * balanced, and the backward pass retraces the same path through recv_from.  Host only,
 * integers only, a pure function of its arguments: every worker computes the same plan
 * from the shared seed without communicating.
 *
 * Boundary b uses the subgroup planner's shuffle with a SplitMix64 stream started at
 * mix64( mix64( mix64(seed ^ mix64(step + G)) ^ mix64(microbatch + 2G) ) ^ mix64(b + 3G) ),
 * G = 0x9E3779B97F4A7C15.
 *
 *   num_stages   pipeline stages, >= 1 (one stage: nothing to route, nothing is written)
 *   W            replicas per stage, >= 1
 *   send_to      host, out, int32[(num_stages-1) * W]: send_to[b*W + r] = replica of stage
 *                b+1 that replica r of stage b sends its outputs to
 *   recv_from    host, out, int32[(num_stages-1) * W]: recv_from[b*W + q] = replica of stage b
 *                that replica q of stage b+1 receives its inputs from (inverse of send_to)
 */
noloco_status noloco_plan_routes(uint64_t seed, uint64_t step, uint64_t microbatch,
                                 int32_t num_stages, int32_t W, int32_t* send_to,
                                 int32_t* recv_from);

/* One tensor of the arena: `numel` consecutive elements starting `offset` elements into
 * every worker's row. */
typedef struct noloco_segment {
  int64_t offset;
  int64_t numel;
} noloco_segment;

/*
 * The parameter arena: three device arrays of W rows, row w starting at
 * base + w * worker_stride elements.  phi (slow / outer weights) and delta (outer
 * momentum) are float; theta (fast / local weights) is float or bf16 (theta_dtype).
 * Only elements inside a segment belong to the method; everything else in a row
 * (gaps, padding up to worker_stride) is never read for its value and never written.
 * Bases must be NOLOCO_BASE_ALIGN_BYTES-aligned and worker_stride a multiple of
 * NOLOCO_STRIDE_ALIGN_ELEMS; segment offsets and lengths are arbitrary (odd is fine).
 * Segments (host array) may come in any order, may leave gaps, must not overlap and
 * must end at or before worker_stride; empty segments are ignored.
 * Speed note (results never depend on it): on MI355X the three arrays stream about 15 % faster
 * when they lie in different 96 GiB thirds of the GPU's memory than when they are neighbours
 * inside one third.  An arena that fills most of the memory is spread by itself; a small one
 * gains from being allocated with two temporary spacer allocations in between.
 */
typedef struct noloco_arena {
  float* phi;              /* device, in/out */
  float* delta;            /* device, in/out */
  void* theta;             /* device, in/out, float or bf16 */
  int64_t worker_stride;   /* elements between consecutive workers' rows, same for all three arrays */
  int32_t W;               /* number of worker rows */
  int32_t theta_dtype;     /* noloco_dtype */
  const noloco_segment* segments; /* host, [num_segments] */
  int32_t num_segments;
} noloco_arena;

/* Eq. 2's coefficients: alpha = outer momentum, beta = outer learning rate,
 * gamma = pull towards the subgroup mean of the slow weights. */
typedef struct noloco_hparams {
  float alpha;
  float beta;
  float gamma;
} noloco_hparams;

/*
 * Pure host helper behind the multi-tensor dispatch: validates a segment list against a
 * row of `worker_stride` elements, sorts it and merges touching segments into maximal
 * contiguous runs.
 *   runs_out   host, out, capacity num_segments entries (may be null to only validate/count)
 *   num_runs   host, out
 * Errors: NOLOCO_ERR_SEGMENT_OVERLAP (overlap or out of row), NOLOCO_ERR_INVALID_ARG
 * (negative offset/numel/count).
 */
noloco_status noloco_merge_segments(const noloco_segment* segments, int32_t num_segments,
                                    int64_t worker_stride, noloco_segment* runs_out,
                                    int32_t* num_runs);

/*
 * Multi-tensor launch table.  Validates the arena layout (W, worker_stride, theta_dtype,
 * segments, alignment of the three base pointers), merges segments into runs, cuts runs
 * into tiles and uploads the tables to the current device (one hipMalloc that also holds the
 * scratch of noloco_replica_spread, 8 bytes per 1024 arena elements; freed by
 * noloco_launch_plan_destroy).  The plan depends on the layout only: the same plan serves
 * any three base pointers with the same layout.  Build once per arena, reuse every step.
 * On error *out is null.
 */
typedef struct noloco_launch_plan noloco_launch_plan;
noloco_status noloco_launch_plan_create(const noloco_arena* arena, noloco_launch_plan** out);
noloco_status noloco_launch_plan_destroy(noloco_launch_plan* plan);

/* Facts about a plan, for harnesses and tests.  Any out pointer may be null. */
noloco_status noloco_launch_plan_info(const noloco_launch_plan* plan, int64_t* elements_per_worker,
                                      int32_t* num_runs, int64_t* num_tiles, int32_t* tile_elems);

/*
 * Launch-shape knobs: an aid for measurement harnesses, not part of the method's interface.
 * Results never depend on them, only speed does.  Every field set to
 * -1 means "automatic": the library picks the measured best for MI355X per subgroup size
 * (the state of a new plan).  The call replaces all four fields.
 *   vectors_per_thread  16-byte vectors each thread handles per tile: 1, 2 or 4 (subgroups of
 *                       4 use at most 2, larger ones 1, to stay within the register file)
 *   nontemporal         1 = streaming (non-temporal) loads and stores, 0 = ordinary
 *   group_major         1 = consecutive work items walk the tiles of one group,
 *                       0 = consecutive work items take the same tile of successive groups
 *   xcd_map             how workgroups (dealt round-robin to the 8 XCDs by the hardware) pick
 *                       work items: 0 = workgroup i takes item i; 1 = each XCD takes one
 *                       contiguous eighth of the items; c in [2, 4096] = each XCD takes runs
 *                       of c consecutive items
 */
typedef struct noloco_tuning {
  int32_t vectors_per_thread;
  int32_t nontemporal;
  int32_t group_major;
  int32_t xcd_map;
} noloco_tuning;
noloco_status noloco_launch_plan_tune(noloco_launch_plan* plan, const noloco_tuning* tuning);

/*
 * One outer step (Eq. 1-3 and the restart of the fast weights), fused, in place, enqueued
 * on `hip_stream` (a hipStream_t; null = the default stream).  Returns after the launch.
 * The call allocates, copies and synchronises nothing on the device (the member table
 * travels in the kernel arguments), so it may be recorded into a HIP graph by stream capture;
 * the grouping is then fixed at capture time.
 *
 *   plan           from noloco_launch_plan_create for this layout
 *   arena          base pointers for this step; W, worker_stride and theta_dtype must match
 *                  the plan (arena->segments is not read again); the three arrays must not
 *                  overlap (NOLOCO_ERR_INVALID_ARG)
 *   hparams        alpha, beta, gamma of Eq. 2
 *   members        host, int32[group_offsets[num_groups]]: worker ids, any order inside a group
 *   group_offsets  host, int32[num_groups + 1], group_offsets[0] = 0, non-decreasing;
 *                  group g is members[group_offsets[g] .. group_offsets[g+1])
 *   num_groups     >= 0
 *
 * The call makes no heap allocation on the host either: the grouping is validated and bucketed
 * by size in fixed stack storage.  Groups of each size go out in one kernel launch per
 * NOLOCO_MAX_GROUP member rows (and per 2^32 threads of grid), sizes ascending.  Every argument
 * and every limit is checked before the first launch; if the HIP runtime then refuses a launch
 * (NOLOCO_ERR_DEVICE) earlier launches of the same call may already have updated their groups'
 * rows, so after NOLOCO_ERR_DEVICE the arena's contents are undefined.
 * The groups must be disjoint and hold valid worker ids (NOLOCO_ERR_BAD_GROUPING
 * otherwise, nothing is launched).  They need not cover all workers: rows of workers in
 * no group are left untouched (a peer that dropped out of this round).  Groups may differ
 * in size; each uses its own n in Eq. 2; a group of one has a zero third term; empty
 * groups are ignored; a group larger than NOLOCO_MAX_GROUP gives NOLOCO_ERR_UNSUPPORTED.
 * The result does not depend on the order of members inside a group nor on the order of
 * the groups (sums run in ascending worker id), and is bit-identical from run to run.
 * Subgroup sizes 1, 2, 4, 8, 16 (everything in registers) and 32, 64 (phi in registers) move
 * each byte once; other sizes take a two-pass kernel that reads phi twice (the second read
 * normally hits in cache).
 */
noloco_status noloco_outer_step(const noloco_launch_plan* plan, const noloco_arena* arena,
                                const noloco_hparams* hparams, const int32_t* members,
                                const int32_t* group_offsets, int32_t num_groups,
                                void* hip_stream);

/*
 * Replica spread: how far the W replicas have drifted apart (results section of the paper,
 * the figure plotting the standard deviation of the model weights across the data-parallel
 * replicas, which the pull term of Eq. 2 is there to contain).  Read-only pass over one
 * arena array x (phi, or theta):
 *   per element k  v_k = (1/W) sum_w (x_w[k] - m_k)^2,  m_k = (1/W) sum_w x_w[k]   (all W rows)
 *   per tensor s   out[s] = sqrt( mean over k in segment s of v_k )
 *   overall        out[num_segments] = sqrt( mean over all segment elements of v_k )
 * v_k is evaluated in binary32 (rows in ascending order: sum, mean = sum * (1/W), then the
 * squared deviations summed in the same order, times 1/W); pooling over elements is in
 * binary64 in a fixed order, so the result is bit-identical from run to run.
 *   plan            launch plan of this layout (its W, worker_stride and segments are used)
 *   x_device        device, [W][worker_stride] float or bf16 (x_dtype), NOLOCO_BASE_ALIGN_BYTES-aligned
 *   out_std_device  device, out, double[num_segments + 1] in the order the segments were given
 *                   at plan creation; an empty segment gives 0
 * Enqueued on hip_stream, not synchronised.  The plan owns the scratch for the per-tile
 * partial sums, so calls sharing one plan must not overlap in time.
 */
noloco_status noloco_replica_spread(const noloco_launch_plan* plan, const void* x_device,
                                    int32_t x_dtype, double* out_std_device, void* hip_stream);

/*
 * noloco_replica_spread for callers that cannot allocate: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same result bit
 * for bit as noloco_replica_spread; the difference is where the per-tile and per-tensor partial
 * sums are staged: not in the plan's own buffer but in one file-scope device array of the library,
 * 16 MiB (2 097 152 doubles) per GPU, which every GPU the library runs on holds until the process
 * ends.  The call performs no device or host allocation and no free, directly or through a
 * library routine (the array's device address is looked up once per GPU, normally already at
 * noloco_launch_plan_create, otherwise on the first call on that GPU).
 *   Limit: the plan's spread tiles (arena elements / 1024 for W = 16, 32, 64 or any other W;
 *   / 4096 for W = 2, 4, 8) plus num_segments plus one must not exceed 2 097 152, else
 *   NOLOCO_ERR_UNSUPPORTED and nothing is launched.
 *   All calls on one GPU share that GPU's array, whichever plan or stream they use: calls that
 *   overlap in time on one GPU race with each other.  Every slot a call reads it has written
 *   first, so what an earlier call left behind is harmless and nothing needs clearing.
 */
noloco_status noloco_replica_spread_noalloc(const noloco_launch_plan* plan, const void* x_device,
                                            int32_t x_dtype, double* out_std_device,
                                            void* hip_stream);

/*
 * Latency model (section "Latency results", appendix "Latency analysis").  Host only, seeded
 * Monte-Carlo; no GPU work.  Message and step times are LogNormal(mu, sigma^2), sigma >= 0.
 *
 * noloco_sim_tree_vs_pair: W workers (a power of two >= 2) at the leaves of a complete binary
 * tree.  Reduce: a parent is ready when the later of its two children's messages has arrived
 * (max(t1, t2), whose mean is (1 + erf(sigma/2)) exp(mu + sigma^2/2)); broadcast: the result
 * travels back down one message per edge; the all-reduce ends when the last worker has it
 * (2 t_c log2 W when sigma = 0).  Pairwise local averaging: two exchanges, each max(t1, t2).
 *   out   host, double[4]: mean tree time, its standard error, mean pair time, its standard error
 *
 * noloco_sim_barrier_penalty: W workers run outer_steps rounds of inner_steps inner steps each
 * (communication time ignored).  With a global barrier every round lasts as long as its slowest
 * worker; with subgroup synchronisation a worker only waits for the n-1 partners
 * noloco_plan_groups(seed, round, W, n) gives it.  Both clocks see the same step times.
 *   out   host, double[2]: finishing time with the global barrier, finishing time (of the last
 *         worker) with subgroup synchronisation
 * Errors: NOLOCO_ERR_INVALID_ARG (sizes, sigma < 0, W not a power of two for the tree),
 * NOLOCO_ERR_BAD_GROUPING (n does not divide W).
 */
noloco_status noloco_sim_tree_vs_pair(uint64_t seed, int32_t W, double mu, double sigma,
                                      int32_t trials, double* out);
noloco_status noloco_sim_barrier_penalty(uint64_t seed, int32_t W, int32_t n, int32_t inner_steps,
                                         int32_t outer_steps, double mu, double sigma, double* out);

/*
 * Measurement aids for harnesses, not part of the method and outside the interface the method
 * needs (noloco_plan_groups, the launch plan, noloco_outer_step): plain streaming kernels over `bytes` bytes (a
 * multiple of 16; pointers 16-byte aligned) on `hip_stream`, with the same non-temporal
 * 16-byte accesses as the outer step.  Harnesses use them as yardsticks for what the chip's
 * HBM delivers to pure reads, pure writes and a 1:1 copy, and to calibrate the profiler's
 * HBM byte counters against a transfer of known size.
 *   noloco_copy_probe  dst[i] = src[i]
 *   noloco_read_probe  reads src and writes nothing (sink_device: 4 writable bytes that are
 *                      only written if the data folds to a pattern no real data produces)
 *   noloco_fill_probe  dst[i] = value
 */
noloco_status noloco_copy_probe(void* dst_device, const void* src_device, int64_t bytes,
                                void* hip_stream);
noloco_status noloco_read_probe(const void* src_device, int64_t bytes, void* sink_device,
                                void* hip_stream);
noloco_status noloco_fill_probe(void* dst_device, int64_t bytes, float value, void* hip_stream);

/* Static, human-readable name of a status code. */
const char* noloco_strerror(noloco_status status);

#ifdef __cplusplus
}
#endif
#endif /* NOLOCO_H_ */
