// Internal declarations shared by the library's translation units (gfx950).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "g10.h"

typedef uint64_t u64;
typedef uint32_t u32;

#define G10_WAVE 64
#define G10_AUX_STREAMS 8
#define G10_BLOCK 256               // 4 wavefronts per workgroup everywhere
#define G10_WAVES (G10_BLOCK / G10_WAVE)

#define G10_HIP(call)                                   \
  do {                                                  \
    hipError_t e_ = (call);                             \
    if (e_ != hipSuccess) return g10_hip_fail(e_, __FILE__, __LINE__); \
  } while (0)

int g10_hip_fail(hipError_t e, const char* file, int line);
#define G10_TRY(x) do { int rc_ = (x); if (rc_) return rc_; } while (0)

// Device memory, pinned host memory and events that outlive the call that released them (kept up
// to a limit and handed to the next request of a fitting size; g10_trim gives them back to the
// driver).  A block is released only after the work that used it has been waited for.
#define G10_MEM_MAX_DEVICES 64
int mem_dev_alloc(void** out, size_t bytes);      // on the current device
void mem_dev_free(void* p);
int mem_host_alloc(void** out, size_t bytes);     // pinned
void mem_host_free(void* p);
int mem_event_get(hipEvent_t* out);               // of the current device
void mem_event_put(hipEvent_t e, int device);
void mem_trim();

// ---------------------------------------------------------------------------
// wavefront / workgroup primitives (64-wide)
// ---------------------------------------------------------------------------
__device__ __forceinline__ u32 lane_id() { return threadIdx.x & (G10_WAVE - 1); }
__device__ __forceinline__ u32 wave_id() { return threadIdx.x / G10_WAVE; }

// Cross-lane steps run on the DPP path of the vector ALU (row shifts inside
// rows of 16 lanes, then the row broadcasts 15 and 31 of the 64-wide wavefront)
// instead of ds_bpermute: a few cycles per step, no LDS crossbar.  Lanes a step
// does not write take the operation's identity.
template <int CTRL, int ROW_MASK, int BANK_MASK>
__device__ __forceinline__ u32 dpp_move32(u32 identity, u32 v) {
  return (u32)__builtin_amdgcn_update_dpp((int)identity, (int)v, CTRL, ROW_MASK, BANK_MASK, false);
}
template <int CTRL, int ROW_MASK, int BANK_MASK, class T>
__device__ __forceinline__ T dpp_move(T identity, T v) {
  static_assert(sizeof(T) == 4 || sizeof(T) == 8, "32- or 64-bit integers");
  if constexpr (sizeof(T) == 4) {
    return (T)dpp_move32<CTRL, ROW_MASK, BANK_MASK>((u32)identity, (u32)v);
  } else {
    const u32 lo = dpp_move32<CTRL, ROW_MASK, BANK_MASK>((u32)identity, (u32)v);
    const u32 hi = dpp_move32<CTRL, ROW_MASK, BANK_MASK>((u32)((u64)identity >> 32), (u32)((u64)v >> 32));
    return (T)(((u64)hi << 32) | lo);
  }
}

struct OpAdd { template <class T> static __device__ __forceinline__ T f(T a, T b) { return a + b; } };
struct OpMax { template <class T> static __device__ __forceinline__ T f(T a, T b) { return a > b ? a : b; } };
struct OpMin { template <class T> static __device__ __forceinline__ T f(T a, T b) { return a < b ? a : b; } };

// inclusive scan inside a wavefront (all 64 lanes must be active); lane 63 ends with the total
template <class Op, class T>
__device__ __forceinline__ T wave_scan_dpp(T x, T identity) {
  T v = x;
  v = Op::f(v, dpp_move<0x111, 0xf, 0xf>(identity, x));      // row_shr:1
  v = Op::f(v, dpp_move<0x112, 0xf, 0xf>(identity, x));      // row_shr:2
  v = Op::f(v, dpp_move<0x113, 0xf, 0xf>(identity, x));      // row_shr:3
  v = Op::f(v, dpp_move<0x114, 0xf, 0xe>(identity, v));      // row_shr:4, lanes 4..15 of a row
  v = Op::f(v, dpp_move<0x118, 0xf, 0xc>(identity, v));      // row_shr:8, lanes 8..15 of a row
  v = Op::f(v, dpp_move<0x142, 0xa, 0xf>(identity, v));      // lane 15 of rows 0 and 2 into rows 1 and 3
  v = Op::f(v, dpp_move<0x143, 0xc, 0xf>(identity, v));      // lane 31 into rows 2 and 3
  return v;
}

template <class T>
__device__ __forceinline__ T wave_last(T v) {                 // the value of lane 63, in every lane
  if constexpr (sizeof(T) == 4) {
    return (T)__builtin_amdgcn_readlane((int)v, G10_WAVE - 1);
  } else {
    const u32 lo = (u32)__builtin_amdgcn_readlane((int)(u32)v, G10_WAVE - 1);
    const u32 hi = (u32)__builtin_amdgcn_readlane((int)(u32)((u64)v >> 32), G10_WAVE - 1);
    return (T)(((u64)hi << 32) | lo);
  }
}

template <class T>
__device__ __forceinline__ T wave_sum(T v) { return wave_last(wave_scan_dpp<OpAdd>(v, (T)0)); }

template <class T>
__device__ __forceinline__ T wave_max(T v) { return wave_last(wave_scan_dpp<OpMax>(v, (T)0)); }

template <class T>
__device__ __forceinline__ T wave_min(T v) { return wave_last(wave_scan_dpp<OpMin>(v, (T)~(T)0)); }

// inclusive scan inside a wavefront
template <class T>
__device__ __forceinline__ T wave_scan_incl(T v) { return wave_scan_dpp<OpAdd>(v, (T)0); }

// Exclusive scan over the workgroup; `total` receives the sum on every thread.
// `tmp` is LDS of G10_WAVES + 1 elements.  Contains two barriers.
template <class T>
__device__ __forceinline__ T block_scan_excl(T v, T* tmp, T& total) {
  T inc = wave_scan_incl(v);
  if (lane_id() == G10_WAVE - 1) tmp[wave_id()] = inc;
  __syncthreads();
  T base = 0, tot = 0;
#pragma unroll
  for (u32 w = 0; w < G10_WAVES; ++w) {
    T x = tmp[w];
    if (w < wave_id()) base += x;
    tot += x;
  }
  __syncthreads();
  total = tot;
  return base + inc - v;
}

// The same for N values at once (two barriers in total).  tmp: LDS of N * G10_WAVES.
template <int N>
__device__ __forceinline__ void block_scan_excl_n(u64 (&v)[N], u64* tmp, u64 (&total)[N]) {
  u64 inc[N];
#pragma unroll
  for (int n = 0; n < N; ++n) inc[n] = wave_scan_incl(v[n]);
  if (lane_id() == G10_WAVE - 1) {
#pragma unroll
    for (int n = 0; n < N; ++n) tmp[n * G10_WAVES + wave_id()] = inc[n];
  }
  __syncthreads();
#pragma unroll
  for (int n = 0; n < N; ++n) {
    u64 base = 0, tot = 0;
#pragma unroll
    for (u32 w = 0; w < G10_WAVES; ++w) {
      const u64 x = tmp[n * G10_WAVES + w];
      if (w < wave_id()) base += x;
      tot += x;
    }
    v[n] = base + inc[n] - v[n];
    total[n] = tot;
  }
  __syncthreads();
}

template <class T>
__device__ __forceinline__ T block_sum(T v, T* tmp) {
  v = wave_sum(v);
  if (lane_id() == 0) tmp[wave_id()] = v;
  __syncthreads();
  T tot = 0;
#pragma unroll
  for (u32 w = 0; w < G10_WAVES; ++w) tot += tmp[w];
  __syncthreads();
  return tot;
}

template <class T>
__device__ __forceinline__ T block_max(T v, T* tmp) {
  v = wave_max(v);
  if (lane_id() == 0) tmp[wave_id()] = v;
  __syncthreads();
  T m = tmp[0];
#pragma unroll
  for (u32 w = 1; w < G10_WAVES; ++w) m = tmp[w] > m ? tmp[w] : m;
  __syncthreads();
  return m;
}

// ---------------------------------------------------------------------------
// device-wide exclusive scan: out[i] = sum of in[0..i), i in [0, n]; out has
// n + 1 elements (out[n] = total).  in == out is allowed.  `scratch` must
// hold scan_scratch_elems(n) elements of T.
// ---------------------------------------------------------------------------
size_t scan_scratch_elems(u64 n);
int scan_excl_u32(const u32* in, u32* out, u64 n, u32* scratch, hipStream_t s);
int scan_excl_u64(const u64* in, u64* out, u64 n, u64* scratch, hipStream_t s);

// stable LSD radix sort of the low `bits` bits of 64-bit keys (see g10_vitality.hip)
size_t radix_hist_elems(u64 n);
int radix_sort_u64(u64** keys, u64** alt, u64 n, u32 bits, u32* hist, u32* scratch, hipStream_t s);
int radix_sort_u32_pairs(u32** keys, u32** alt, u32** vals, u32** valt, u64 n, u32 bits, u32* hist, u32* scratch,
                         hipStream_t s, bool iota = false);
// Many such sorts in the same launches.  One job: n > 0 pairs in (keys, vals), buffers (alt, valt) of the same
// size, hist of radix_hist_elems(n) words, nb = radix_blocks(n).
struct SortJob { u32 *keys, *alt, *vals, *valt, *hist; u32 n, nb; };
u32 radix_blocks(u64 n);
int radix_sort_u32_pairs_jobs(const SortJob* jobs_dev, u32 njobs, u32 max_nb, u32 bits, bool iota, hipStream_t s);
int radix_sort_u64_pairs(u64** keys, u64** alt, u32** vals, u32** valt, u64 n, u32 bits, u32* hist, u32* scratch,
                         hipStream_t s, bool iota = false);

// ---------------------------------------------------------------------------
// handle
// ---------------------------------------------------------------------------
struct PlanWork;   // planning workspaces, defined in g10_plan.hip

struct g10_plan_s {
  int device = 0;
  hipStream_t stream = nullptr;
  u32 K = 0, N = 0, flags = 0;
  u64 P = 0;
  u32 kbits = 0;                 // bits of the kernel index inside a sort key
  // counts known after the analysis
  u64 n_uses = 0, n_periods = 0, peak = 0, T = 0;
  // device arrays (owned)
  u64* dur = nullptr;            // [K]
  u64* size = nullptr;           // [N]
  uint8_t* glob = nullptr;       // [N]
  u64* start = nullptr;          // [K+1]
  u64* ukeys = nullptr;          // [n_uses] sorted distinct (tensor << kbits | kernel)
  u64* use_off = nullptr;        // [N+1]
  u32* use_k = nullptr;          // [n_uses]
  u32* per_t = nullptr;          // [n_periods]
  u32* per_L = nullptr;
  u32* per_R = nullptr;
  uint4* per_by_start = nullptr; // [n_periods] {L, R, tensor, period index}, ordered by L (then index)
  u64* per_size = nullptr;       // [n_periods] size of the period's tensor, same order
  u64* pressure_buf = nullptr;   // [K+1]; pressure = pressure_buf + 1
  PlanWork* work = nullptr;      // workspaces of the first plan of a batch (the only one of g10_plan)
  PlanWork** more = nullptr;     // ... of the further plans of a batch
  u32 n_more = 0;
  u64 max_size = 0;              // the largest tensor
  u32 max_tiles = 0, max_chunks = 0;   // g10_plan_limits (0 = the defaults)
  g10_counters* counters = nullptr;    // of the plans of the last planning call
  u32 n_counters = 0;
  bool big_size = false;         // some tensor has 2^43 bytes or more (the planner's 16-byte candidate copies hold 43 bits)
  void* loop_args = nullptr;     // device array of per-plan arguments of the loop kernel
  u32 loop_args_cap = 0;
  bool lds_opt_in = false;       // the loop kernel was allowed more than 64 KB of LDS
  void* arena = nullptr;         // the one device allocation the analysis arrays above point into
  void* tmp_arena = nullptr;     // the analysis' temporaries, until the stream has next been waited for
  hipStream_t aux[8] = {};       // streams for the streaming kernels of the plans of a batch (made at the first batch)
  u32 n_aux = 0;
};

int vitality_run(g10_plan_s* h, const g10_trace* tr);
// durations of one plan that replace the trace's (g10_vitality.hip): copy, checks, start times
int slot_times_begin(const u64* src, u32 K, u64* dur, u64* start, u64* scratch64, void* stats_dev, void* check,
                     hipStream_t s);
int slot_times_end(const void* check, u64* T_out);
int plan_run(g10_plan_s* h, const g10_params* p, g10_result* out);
int plan_batch_run(g10_plan_s* h, const g10_params* params, u32 count, g10_result* outs);
int prefetch_run(g10_plan_s* h, g10_prefetch_result* out);
int replay_run(g10_plan_s* h, const u64* dur_ns, u32 eager, g10_replay_result* out);
void plan_work_free(PlanWork* w);
