/* g10.h - C ABI of the MI355X (gfx950) implementation of G10's compile-time
 * hot path: tensor vitality analysis and smart tensor eviction planning
 * (G10, MICRO'23, Sections 4.2-4.4 and Algorithm 1).
 *
 * A DNN training step's kernel trace goes in; an eviction / prefetch schedule
 * over GPU memory, host memory and flash comes out.  All work runs in HIP
 * kernels on the device of the caller's stream; the library never falls back
 * to the CPU.  Times are integer nanoseconds, sizes integer bytes, bandwidths
 * bytes per microsecond (6 GB/s = 6000).
 *
 * Conventions
 *   - plain C, no exceptions; the only state outside the handles is the cache
 *     of released memory (g10_trim) and the array of g10_vitality_static;
 *     every call but g10_plan_free and g10_trim returns an int:
 *     G10_OK or a negative error.  On error output arguments are left
 *     untouched (handles) or zeroed (result structs).
 *   - pointers inside g10_trace are DEVICE pointers owned by the caller; the
 *     library copies what it needs, so they may be freed once g10_vitality
 *     returns.  Everything a result struct points to is HOST memory owned by
 *     the handle, valid until the next g10_plan on that handle or
 *     g10_plan_free.
 *   - a handle is bound to the device and stream given to g10_vitality and is
 *     not thread-safe; distinct handles are independent.
 */
#ifndef G10_H
#define G10_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  G10_OK = 0,
  G10_EINVAL = -1,    /* NULL argument, K = 0, N = 0, K >= 2^31, P >= 2^32, an index out of
                         range, a zero duration / size / bandwidth                     */
  G10_EOVERFLOW = -2, /* sum of durations >= 2^62, sum of used sizes >= 2^64,
                         or a size * 1000 >= 2^64                                      */
  G10_ENOMEM = -3,    /* host or device allocation failed                              */
  G10_EDEVICE = -4,   /* a HIP call failed                                             */
  G10_ELIMIT = -5     /* g10_vitality_static only: the trace is larger than the fixed
                         device memory of that call can take                           */
};

enum { G10_FLASH = 0, G10_HOST = 1 };          /* migration destinations               */
enum { G10_FITS = 0, G10_RESIDUAL = 1, G10_TRUNCATED = 2 };

#define G10_NO_WRAP 1u  /* g10_trace.flags: ignore the cross-iteration inactive
                           period of global tensors                                    */

/* One training iteration as profiled offline (Section 4.2): kernels in
 * execution order with their durations, the tensors each kernel touches, tensor
 * sizes, and which tensors are global (weights: alive across iterations) rather
 * than intermediate (born at first use, dead after last use).  The (kernel,
 * tensor) pairs are a COO list in any order; duplicates are legal (Figure 6
 * passes one tensor twice to a kernel) and collapse. */
typedef struct {
  uint32_t K, N;               /* kernels, tensors                                     */
  uint64_t P;                  /* use pairs (may be 0; fewer than 2^32)                */
  const uint64_t *dur_ns;      /* device [K], each > 0                                 */
  const uint64_t *size_bytes;  /* device [N], each > 0                                 */
  const uint8_t *is_global;    /* device [N], 1 = global                               */
  const uint32_t *use_kernel;  /* device [P], each < K                                 */
  const uint32_t *use_tensor;  /* device [P], each < N                                 */
  uint32_t flags;              /* G10_NO_WRAP or 0                                     */
} g10_trace;

typedef struct {
  uint64_t n_uses;      /* distinct (tensor, kernel) pairs                             */
  uint64_t n_periods;   /* inactive periods = eviction candidates                      */
  uint64_t peak_bytes;  /* maximum of the memory-pressure timeline                     */
  uint64_t iter_ns;     /* duration of the iteration                                   */
} g10_vitality_stats;

enum { G10_RANK_BENEFIT = 0, G10_RANK_RATIO = 1 };
enum { G10_AREA_BAND = 0, G10_AREA_CLIPPED = 1 };

/* Inputs of Algorithm 1 beyond the periods: the GPU memory capacity, the host
 * memory that may hold evicted tensors, and the bandwidths from which eviction
 * and prefetch times are estimated (Section 4.2; Table 2 has asymmetric flash
 * read / write bandwidth, hence separate directions). */
typedef struct {
  uint64_t gpu_cap_bytes;
  uint64_t host_cap_bytes;
  uint64_t bw_out_Bpus[2];   /* GPU -> [G10_FLASH, G10_HOST], bytes per microsecond    */
  uint64_t bw_in_Bpus[2];    /* [G10_FLASH, G10_HOST] -> GPU                           */
  uint64_t max_iterations;   /* stop after this many ranking passes (of Algorithm 1: one migration or
                                one dropped candidate each); 0 = no limit                              */
  const uint64_t *dur_ns;    /* NULL, or device [K]: kernel durations that replace the analysed trace's
                                for this plan, each > 0 (re-planning under profiling errors, the study of
                                the evaluation's "Impact of Profiling Errors").  Which tensors are used
                                where does not change, so the periods and the pressure per slot are the
                                analysed ones; slot start times, the iteration time, transfer windows,
                                channel capacities and over-capacity times follow the new durations: the
                                plan is the one an analysis of the trace with these durations gives.
                                Caller-owned; read during the planning call only.                        */
  uint32_t rank;             /* G10_RANK_BENEFIT (0, Algorithm 1: by the benefit alone) or G10_RANK_RATIO:
                                periods are ranked by benefit / (eviction time + prefetch time) of the
                                destination the policy picks, the benefit-cost ratio of Section 4.3's
                                example, compared exactly as fractions; ties to the lowest period index   */
  uint32_t area;             /* G10_AREA_BAND (0): the benefit is size x time over capacity inside the
                                absent window, the tensor's whole band; G10_AREA_CLIPPED: the area between
                                the pressure curve and the capacity line that the eviction removes, per
                                slot duration x min(size, pressure - capacity).  The clipped area is
                                evaluated lazily: candidates are ranked by bounds (the band, or an area
                                computed in an earlier pass) and only the best by bound is summed exactly,
                                so the plan is exact and the cost stays near the default's while the
                                pressure is far above the capacity                                        */
} g10_params;

/* One migration, i.e. one g10_pre_evict / g10_prefetch pair of Section 4.4's
 * instruction set: evict `tensor` to `dest` right after kernel `evict_after`
 * finished; its memory is free during kernels absent_first..absent_last
 * (cyclically when `wraps`); the prefetch must have completed before kernel
 * `next_use` starts (of the next iteration when `wraps`). */
typedef struct {
  uint32_t cand;          /* index of the inactive period (tensor-major, by start)     */
  uint32_t tensor;
  uint32_t evict_after;   /* last kernel using the tensor before the period            */
  uint32_t absent_first;  /* first kernel slot in which the memory is free             */
  uint32_t absent_last;   /* last such slot; the prefetch is issued after it           */
  uint32_t next_use;      /* first kernel using the tensor after the period            */
  uint32_t dest;          /* G10_FLASH or G10_HOST                                     */
  uint32_t wraps;         /* 1: the period runs into the next iteration                */
  uint64_t size_bytes;
  uint64_t t_out_ns;      /* eviction time  = ceil(size * 1000 / bw_out[dest])         */
  uint64_t t_in_ns;       /* prefetch time  = ceil(size * 1000 / bw_in[dest])          */
  uint64_t benefit_lo;    /* size x over-capacity time removed, byte*ns, 128 bit       */
  uint64_t benefit_hi;
} g10_migration;

/* A candidate that won a ranking pass but was dropped: flash could not carry
 * it and host memory had no room during its period. */
typedef struct {
  uint64_t iteration;     /* 0-based ranking pass                                      */
  uint32_t cand;
  uint32_t reserved;
} g10_dropped;

typedef struct {
  int32_t status;         /* G10_FITS: pressure <= capacity everywhere; G10_RESIDUAL:
                             no beneficial candidate left; G10_TRUNCATED: max_iterations */
  uint64_t n_migrations, n_iterations, n_dropped;
  uint64_t n_cand_evals;  /* sum over ranking passes of the live candidates            */
  uint64_t peak_before, peak_after;          /* bytes                                  */
  uint64_t overtime_before_ns, overtime_after_ns; /* time spent over capacity          */
  const g10_migration *migrations;           /* host [n_migrations], commit order      */
  const g10_dropped *dropped;                /* host [n_dropped]                       */
  const uint64_t *pressure_after;            /* host [K]                               */
  double plan_ms;         /* device time of the whole call (events on the stream); for the
                             plans of a batch, of the whole batch                      */
} g10_result;

/* How the last planning call on a handle did its work: device times and work counters of one
 * of its plans (g10_plan_counters).  For measurements and tests; no part of the plan. */
typedef struct {
  double score_full_ms;        /* the one streaming scoring pass over all candidates   */
                               /* (not timed for the plans of a batch of several: 0)   */
  uint64_t score_full_cands;   /* candidates it streamed (those with a valid window)   */
  double loop_ms;              /* the greedy loop (of a batch: all loops)              */
  uint64_t loop_launches;      /* launches of the loop kernel                          */
  uint64_t loop_passes;        /* ranking passes the kernel made: a pass commits one migration or,
                                  where that is provably what Algorithm 1 would do next, several  */
  uint64_t loop_more_rounds;   /* further rounds of commits made from the list of a ranking pass
                                  (its entries scored again) instead of a new ranking pass        */
  uint64_t loop_retiles;       /* times the candidate list was put back into score order */
  uint64_t retile_cands;       /* candidates scored again by those re-orderings        */
  uint64_t loop_cands_scored;  /* candidates re-scored inside the loop (tiles * 256, and the list
                                  entries scored again for loop_more_rounds)              */
  uint64_t loop_second_rounds; /* passes that needed a second scoring round            */
  uint64_t loop_chunk_jobs;    /* timeline chunks rewritten slot by slot               */
  uint64_t loop_area_evals;    /* G10_AREA_CLIPPED: clipped areas summed exactly       */
  uint64_t loop_area_refused;  /* ... of which came out below the bound (ranked again) */
  uint64_t loop_wide_rounds;   /* G10_RANK_RATIO, one plan: scoring rounds of a pass left to the scoring
                                  kernel on all compute units (their candidates count in loop_cands_scored) */
  /* g10_plan_batch with more than one plan: host wall clock of the phases of the call (0 otherwise) */
  double batch_prepare_ms;     /* timelines, candidate windows, first scoring and ordering of all plans */
  double batch_loops_ms;       /* the launches of the greedy loops (all plans side by side) and the read-back of their progress */
  double batch_retile_ms;      /* putting the candidate lists back into score order between launches */
  double batch_results_ms;     /* final pressure, copies of the plans to the host              */
} g10_counters;

typedef struct g10_plan_s g10_plan_t;   /* opaque: device copy of the analysis + workspaces */

/* Tensor vitality analysis (Section 4.2): per-tensor use lists (sorted,
 * duplicates dropped), birth / death, inactive periods (gaps of at least one
 * whole kernel between consecutive uses, plus the cross-iteration gap of
 * global tensors), and the memory-pressure timeline (bytes resident per
 * kernel slot) with its peak.  Enqueues on `hip_stream` (a hipStream_t, NULL =
 * default stream) and synchronises it before returning.
 * Errors: G10_EINVAL / G10_EOVERFLOW as listed above (array contents are
 * validated on the device before any other work), G10_ENOMEM, G10_EDEVICE. */
int g10_vitality(const g10_trace *trace, void *hip_stream, g10_plan_t **out_handle);

/* Counts and peak of a finished analysis (Section 4.2: the uses, the inactive periods that are
 * Algorithm 1's input, the peak of the memory-pressure curve of Section 4.3). */
int g10_vitality_info(const g10_plan_t *handle, g10_vitality_stats *out);

/* Read-back of the analysis of Section 4.2 (with g10_vitality_info: what the planner works on),
 * for tests and tools: copies one analysis array to HOST memory `dst` of `bytes` bytes (must
 * match the array's size exactly, else G10_EINVAL).  `which`:
 *   0 use_off  u64[N+1]   CSR offsets into use_k
 *   1 use_k    u32[n_uses]
 *   2 per_tensor u32[n_periods]   3 per_L u32[n_periods]   4 per_R u32[n_periods]
 *     (L = last use before the period, R = next use; R >= K for the
 *      cross-iteration period: R - K is the kernel of the next iteration)
 *   5 start    u64[K+1]  start time of every kernel slot
 *   6 pressure u64[K] */
int g10_vitality_read(const g10_plan_t *handle, int which, void *dst, uint64_t bytes);

/* Device buffers for the results of g10_vitality_static, owned by the caller. */
typedef struct {
  uint64_t *use_off;     /* device [N+1]  CSR offsets into use_k                              */
  uint32_t *use_k;       /* device [P]    the first n_uses entries are written                */
  uint32_t *per_tensor;  /* device [P]    the first n_periods entries of these three are      */
  uint32_t *per_L;       /* device [P]    written (L = last use before the period, R = next   */
  uint32_t *per_R;       /* device [P]    use; R >= K for the cross-iteration period)         */
  uint64_t *start;       /* device [K+1]  start time of every kernel slot                     */
  uint64_t *pressure;    /* device [K]    bytes resident per kernel slot                      */
} g10_vitality_buffers;

#define G10_STATIC_MAX_K 131072u            /* limits of g10_vitality_static ...              */
#define G10_STATIC_MAX_N 262144u
#define G10_STATIC_MAX_P 262144u
#define G10_STATIC_SCRATCH_BYTES (24u << 20) /* ... and the device memory it works in, per GPU */

/* g10_vitality for callers that cannot allocate: code under HIP graph capture or between
 * captures, tight serving loops, harnesses that forbid hipMalloc.  The same analysis, the same
 * results bit for bit, but no handle: the results are written into the caller's device buffers
 * (`out`, sized as listed above) and the counts into `stats` (host).  The call allocates
 * nothing, on the device or through any library: every intermediate lives in one fixed array
 * of G10_STATIC_SCRATCH_BYTES bytes that the library holds on each GPU it runs on until the
 * process ends.  The trace's arrays are read in place during the call.  Traces beyond
 * G10_STATIC_MAX_K kernels, G10_STATIC_MAX_N tensors or G10_STATIC_MAX_P pairs (or whose
 * intermediates would not fit the array) are refused with G10_ELIMIT before any work.  All calls
 * on one GPU share that array, which keeps the last call's contents (the call clears what it
 * needs cleared): calls that overlap in time on one GPU race and must be serialised by the
 * caller.  Enqueues on `hip_stream` and synchronises it before returning.  No planning can follow
 * (use g10_vitality for that).
 * Errors: G10_EINVAL / G10_EOVERFLOW as g10_vitality, G10_ELIMIT, G10_EDEVICE. */
int g10_vitality_static(const g10_trace *trace, void *hip_stream, const g10_vitality_buffers *out,
                        g10_vitality_stats *stats);

/* Smart tensor eviction (Algorithm 1, Section 4.3) on an analysed trace: the
 * whole greedy loop - scoring of the live candidates against the pressure and
 * channel timelines, arg-max with lowest-index tie-break, commit and range
 * updates - runs on the device.  May be called repeatedly with different
 * parameters; the analysis is never modified.  Synchronises the stream.
 * Errors: G10_EINVAL (NULL, zero bandwidth, a zero in dur_ns, unknown rank or area), G10_EOVERFLOW (sum of dur_ns
 * >= 2^62), G10_ENOMEM, G10_EDEVICE.  Not
 * getting under capacity is not an error: status = G10_RESIDUAL. */
int g10_plan(g10_plan_t *handle, const g10_params *params, g10_result *out);

/* Counters of plan `plan_index` (0 for g10_plan; 0 .. count-1 after g10_plan_batch) of the last
 * planning call on the handle.  Errors: G10_EINVAL (NULL, no such plan). */
int g10_plan_counters(const g10_plan_t *handle, uint32_t plan_index, g10_counters *out);

/* Bounds of the two on-chip structures of the greedy loop for the planning calls that follow on
 * this handle; 0 = the library's default, which is also the maximum.  max_tiles: candidates are
 * ranked in tiles of 256 << k, k the smallest with at most this many tiles (8192).  max_chunks:
 * the kernel timeline is split into chunks of 256 << k slots, k the smallest with at most this
 * many chunks (512).  Both only trade speed against on-chip memory; no plan depends on them.
 * They exist so that tests reach the code paths of very long traces with small ones.
 * Errors: G10_EINVAL (NULL). */
int g10_plan_limits(g10_plan_t *handle, uint32_t max_tiles, uint32_t max_chunks);

/* `count` plans on one analysed trace in one call.  The sensitivity studies of the paper's
 * evaluation (Section 7: host memory capacity, SSD bandwidth, profiling errors) plan one trace
 * many times with other capacities, bandwidths or kernel times; this is that sweep as one call:
 * outs[i] is what g10_plan(handle, &params[i], &outs[i]) would return, bit for bit.
 * The greedy loop of a plan is a serial chain that occupies one workgroup; a batch runs the
 * loops of all its plans side by side (one workgroup each), so up to a few hundred plans take
 * about as long as the slowest one plus their streaming passes.  Every plan keeps its own
 * workspaces in the handle (about 350 bytes per inactive period): the result arrays of all
 * `count` plans stay valid until the next planning call on the handle.  plan_ms of every
 * result is that of the whole batch.  g10_prefetch afterwards refers to params[0]'s plan.
 * Errors: as g10_plan; also G10_EINVAL for count = 0 or count > 4096.  On G10_ENOMEM the workspaces
 * of the plans after the first are released again and the handle stays usable. */
int g10_plan_batch(g10_plan_t *handle, const g10_params *params, uint32_t count, g10_result *outs);

/* Result of g10_prefetch; the arrays are host memory owned by the handle, valid until the
 * next g10_plan / g10_prefetch on it or g10_plan_free. */
typedef struct {
  uint64_t n_migrations;        /* records of the plan                                  */
  uint64_t n_moved;             /* prefetches that moved back                           */
  uint64_t slots_gained;        /* kernel slots gained, summed over the records         */
  uint64_t peak_bytes;          /* maximum of the pressure with the earlier prefetches  */
  const uint32_t *order;        /* [n_migrations] records in the order they were visited */
  const uint32_t *gained;       /* [n_migrations] slots by which each prefetch moved back */
  const uint32_t *absent_last;  /* [n_migrations] last kernel slot in which the memory is still free
                                   (the prefetch is issued after it); one before absent_first if
                                   none is left                                          */
  const uint64_t *pressure;     /* [K] bytes resident per kernel slot                   */
  double ms;                    /* device time of the call                              */
} g10_prefetch_result;

/* Smart tensor prefetching (Section 4.4) on the plan the last g10_plan made on this handle.
 * Algorithm 1 assumes every prefetch at its latest safe time (so that it ends exactly when
 * the tensor is used again).  Here the evicted periods are visited in the order of that
 * time (equal times in plan order); each prefetch is moved back, in whole kernel slots and
 * not past the first slot in which the memory was free, as far as every slot up to the old
 * prefetch can hold the whole tensor within the capacity the plan was made for, and the
 * pressure of the slots gained rises by the tensor's size.  The channel reservations are
 * left as the plan made them.  Runs on the handle's stream and synchronises it.
 * Errors: G10_EINVAL (NULL, no plan on the handle), G10_ENOMEM, G10_EDEVICE. */
int g10_prefetch(g10_plan_t *handle, g10_prefetch_result *out);

/* Result of g10_replay; late_ns is host memory owned by the handle, valid until the next
 * g10_plan / g10_replay on it or g10_plan_free. */
typedef struct {
  uint64_t iter_ns;             /* duration of the steady-state iteration               */
  uint64_t planned_ns;          /* sum of the replayed kernel durations (no stall)      */
  uint64_t stall_ns;            /* iter_ns - planned_ns: time kernels waited for prefetches */
  uint64_t n_stalled;           /* kernels that waited                                  */
  uint64_t bytes[2];            /* evicted (= prefetched) bytes per destination and iteration */
  uint64_t busy_out_ns[2];      /* eviction time per destination                        */
  uint64_t busy_in_ns[2];       /* prefetch time per destination                        */
  uint64_t n_migrations;
  const uint64_t *late_ns;      /* [n_migrations] how long the next use of each migration's tensor
                                   waited for its prefetch beyond the end of the kernel before it */
  double ms;                    /* device time of the call                              */
} g10_replay_result;

/* Slot-level replay of the plan the last g10_plan made on this handle: what would the
 * iteration take if the kernels ran `dur_ns` long (device [K], each > 0; NULL = the durations
 * the plan was made for) and the plan's transfers went through one first-in-first-out channel
 * per destination and direction?  A stand-in for the time and traffic breakdown of the paper's
 * simulator (evaluation, "End-to-end Performance" and "Impact of Profiling Errors"); not a step
 * of the planner.  The eviction of a migration is issued when kernel evict_after has finished,
 * its prefetch when kernel absent_last has finished - with `eager` != 0 at the slot g10_prefetch
 * moved it to (g10_prefetch must have run on this plan) - and not before the eviction is done; a
 * kernel waits until every prefetch of a tensor it uses is done.  Two iterations are replayed
 * end to end; the figures are those of the second.  Synchronises the stream.
 * Errors: G10_EINVAL (NULL, no plan, eager without g10_prefetch, a zero duration),
 * G10_EOVERFLOW (durations sum to >= 2^62), G10_ENOMEM, G10_EDEVICE. */
int g10_replay(g10_plan_t *handle, const uint64_t *dur_ns, uint32_t eager, g10_replay_result *out);

/* Releases everything the library allocated for the handle (the analysis of g10_vitality and the
 * workspaces of the planning calls), after waiting for the handle's stream.  NULL is allowed.
 * The profiling -> analysis -> plan cycle of Section 4.1 repeats with every new trace, and
 * allocating and freeing device memory costs about as much host time as the analysis' kernels
 * take: the blocks (device memory, pinned host memory, events) go to a cache inside the library,
 * at most 4 GiB and 96 blocks per process, oldest out first, and the next g10_vitality / g10_plan
 * takes a block of a fitting size from there before it asks the driver.  When the driver has no
 * memory left the cache is emptied and the request made once more. */
void g10_plan_free(g10_plan_t *handle);

/* Hands every block of that cache back to the driver (for a caller that is done with the library
 * for a while, or needs the memory).  Handles in use are not affected. */
void g10_trim(void);

#ifdef __cplusplus
}
#endif
#endif /* G10_H */
