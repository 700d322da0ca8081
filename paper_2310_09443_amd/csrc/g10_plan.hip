// Smart tensor eviction on the device (G10, Section 4.3, Algorithm 1).
//
// State on the device (u64 unless noted, K = kernel slots):
//   pressure[K]                 bytes resident per slot
//   busy[4][K]                  channel time already reserved per slot;
//                               channel = 2 * direction + destination
//                               (0 flash-out, 1 host-out, 2 flash-in, 3 host-in)
//   host_used[K]                bytes parked in host memory per slot
//   two-level prefix sums of five per-slot quantities, rebuilt where they
//   change after every commit:
//     array 0        over-capacity time   dur[k] * [pressure[k] > cap]
//     array 1 + ch   free channel time    dur[k] - busy[ch][k]
//   level 0 = exclusive prefix inside a chunk of CH slots, interleaved per
//             slot (px[K][8], one 64-byte record per slot, so that the words a
//             candidate needs at one slot share a cache line);
//   level 1 = exclusive prefix of the chunk totals (bases[5][nch + 1]), small
//             enough to sit in LDS while candidates are scored.
//   A prefix up to slot j is bases[j / CH] + px[j].
//
// Candidates (inactive periods with at least one valid window) are kept as
// packed 16-byte vectors, sorted by period start so that neighbouring lanes
// gather neighbouring timeline records, and are compacted between batches of
// passes: a candidate whose both destinations are invalid, can no longer be
// carried, or remove no over-capacity time can never score again (pressure
// only falls, reservations only grow), so dropping it changes nothing.
//
// One ranking pass = two launches:
//   k_score   streams the candidate vectors (32 B per candidate), gathers the
//             prefix words, reduces to the best (benefit, lowest index) per
//             workgroup; the last workgroup to finish reduces the partials,
//             decides (stop / drop / commit) and appends the migration record.
//   k_commit  one workgroup per chunk applies the winner's range updates
//             (pressure, channel reservations, host memory) to its slots and
//             rebuilds its chunk's prefixes; the last workgroup rebuilds
//             level 1 and tests the "fits" stop rule.
// The host only enqueues batches of passes and polls a done flag per batch.

#include "g10_internal.h"

#include <new>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

namespace {

enum { A_OT = 0, A_FO = 1, A_FI = 3, N_ARR = 5, PX = 8 };   // FO + dest, FI + dest; PX = words per slot record
enum { ACT_NONE = 0, ACT_COMMIT = 1, ACT_DROP = 2 };

struct Ctl {
  // parameters
  u64 gpu_cap, host_cap, bw_out[2], bw_in[2], max_iter;
  u64 C;                      // all inactive periods (live before any removal)
  // progress
  u32 done, status;
  u64 n_iter, n_mig, n_drop, n_evals;
  // decision of the current pass, consumed by k_commit
  u32 action, dest, pos, cand;
  u32 L1, R, a, b;            // doubled slot coordinates: period interior [L1, R-1], absent [a, b]
  u64 s, tau_o, tau_i;
  u64 fo_base, fi_end;        // free out-channel time before L1 / free in-channel time before R
  // last-workgroup-done counters
  u32 score_done, commit_done;
  u64 overtime_before;
};

struct Partial {
  u64 hi, lo;                 // benefit
  u32 cand, pos, dest, pad;
};

struct Cands {                // live candidates, sorted by L1
  uint4* A;                   // {L1, R, a0, b0}     a > b: no valid window for that destination
  uint4* B;                   // {a1, b1, size lo, size hi}
  u32* idx;                   // index of the period in the analysis order (the tie-break)
};

struct Timelines {
  const u64* dur;
  u64* pressure;
  u64* busy;                  // [4][K]
  u64* host_used;
  u64* px;                    // [K][PX]
  u64* tot;                   // [5][nch]
  u64* bases;                 // [5][nch + 1]
  u64* hostmax;               // [nch]
  u32 K, nch, spt, shift_ch;  // chunk = 256 * spt = 1 << shift_ch slots
};

// ---------------------------------------------------------------------------
// prefix queries on the doubled timeline (two iterations end to end)
// ---------------------------------------------------------------------------
struct Slot {                 // a doubled coordinate j in [0, 2K) resolved once
  const u64* rec;             // its 64-byte record
  u32 chunk;
  bool second;                // j >= K: add one whole iteration
};

struct Prefix {
  const u64* px;
  const u64* base;            // [5][nb1], LDS in k_score
  u32 K, nb1, shift_ch;
  __device__ __forceinline__ Slot slot(u32 j) const {
    Slot s;
    s.second = j >= K;
    const u32 jj = s.second ? j - K : j;
    s.rec = px + (u64)jj * PX;
    s.chunk = jj >> shift_ch;
    return s;
  }
  // sum of array `arr` over the slots before the slot
  __device__ __forceinline__ u64 at(u32 arr, const Slot& s) const {
    const u64* b = base + arr * nb1;
    return (s.second ? b[nb1 - 1] : 0ull) + b[s.chunk] + s.rec[arr];
  }
};

__device__ __forceinline__ bool carries(u64 free_ns, u64 bw, u64 bytes_x1000) {
  // free_ns >= ceil(bytes_x1000 / bw)  <=>  free_ns * bw >= bytes_x1000
  return __umul64hi(free_ns, bw) != 0 || free_ns * bw >= bytes_x1000;
}

struct Machine { u64 bwo[2], bwi[2]; };

// Policy destination and over-capacity time of one candidate: flash unless
// flash has no valid window or cannot carry the transfer, then host.
// Returns false if no destination can take it now.
__device__ __forceinline__ bool policy(const Prefix& pf, const Machine& m, const uint4 A, const uint4 B, u64 s,
                                       u32& dest, u64& ot) {
  const u64 x1000 = s * 1000ull;
  const Slot sL = pf.slot(A.x), sR = pf.slot(A.y);
#pragma unroll
  for (u32 d = 0; d < 2; ++d) {
    const u32 a = d ? B.x : A.z, b = d ? B.y : A.w;
    if (a > b) continue;
    const Slot sa = pf.slot(a);
    if (!carries(pf.at(A_FO + d, sa) - pf.at(A_FO + d, sL), m.bwo[d], x1000)) continue;   // eviction in [L1, a-1]
    const Slot sb = pf.slot(b + 1);
    if (!carries(pf.at(A_FI + d, sR) - pf.at(A_FI + d, sb), m.bwi[d], x1000)) continue;   // prefetch in [b+1, R-1]
    ot = pf.at(A_OT, sb) - pf.at(A_OT, sa);                                               // over capacity while absent
    dest = d;
    return true;
  }
  return false;
}

// Can the candidate ever score again?  (either destination still possible and useful)
__device__ __forceinline__ bool alive(const Prefix& pf, const Machine& m, const uint4 A, const uint4 B, u64 s) {
  const u64 x1000 = s * 1000ull;
  const Slot sL = pf.slot(A.x), sR = pf.slot(A.y);
#pragma unroll
  for (u32 d = 0; d < 2; ++d) {
    const u32 a = d ? B.x : A.z, b = d ? B.y : A.w;
    if (a > b) continue;
    const Slot sa = pf.slot(a), sb = pf.slot(b + 1);
    if (pf.at(A_OT, sb) == pf.at(A_OT, sa)) continue;
    if (!carries(pf.at(A_FO + d, sa) - pf.at(A_FO + d, sL), m.bwo[d], x1000)) continue;
    if (!carries(pf.at(A_FI + d, sR) - pf.at(A_FI + d, sb), m.bwi[d], x1000)) continue;
    return true;
  }
  return false;
}

__device__ __forceinline__ bool better(u64 hi, u64 lo, u32 cand, u64 bhi, u64 blo, u32 bcand) {
  if (hi != bhi) return hi > bhi;
  if (lo != blo) return lo > blo;
  return cand < bcand;
}

// ---------------------------------------------------------------------------
// candidate preparation: transfer times and absent windows per destination
// ---------------------------------------------------------------------------
__device__ __forceinline__ u64 start2(const u64* start, u32 K, u64 T, u32 j) { return j < K ? start[j] : start[j - K] + T; }

__device__ __forceinline__ u64 ceil_div_x1000(u64 s, u64 bw) {
  const u64 x = s * 1000ull;              // validated: no overflow
  return x / bw + (x % bw != 0);
}

__global__ __launch_bounds__(G10_BLOCK) void k_prep(const u32* __restrict__ per_t, const u32* __restrict__ per_L,
                                                   const u32* __restrict__ per_R, const u64* __restrict__ size,
                                                   const u64* __restrict__ start, u32 K, u64 T, u32 C, const Ctl* ctl,
                                                   uint4* __restrict__ win, u32* __restrict__ keep) {
  const u32 c = blockIdx.x * G10_BLOCK + threadIdx.x;
  if (c >= C) return;
  const u32 L = per_L[c], R = per_R[c];
  const u64 s = size[per_t[c]];
  const u64 t_r = start2(start, K, T, L + 1), t_use = start2(start, K, T, R), len = t_use - t_r;
  u32 any = 0;
  u32 w[4];
#pragma unroll
  for (int d = 0; d < 2; ++d) {
    const u64 tau_o = ceil_div_x1000(s, ctl->bw_out[d]), tau_i = ceil_div_x1000(s, ctl->bw_in[d]);
    u32 a = 1, b = 0;
    if (tau_o <= len && tau_i <= len) {
      u32 lo = L + 1, hi = R;               // first slot boundary at or after the end of the eviction
      const u64 want = t_r + tau_o;
      while (lo < hi) { u32 mid = lo + ((hi - lo) >> 1); if (start2(start, K, T, mid) >= want) hi = mid; else lo = mid + 1; }
      const u32 aa = lo;
      lo = L; hi = R - 1;                   // last slot ending at or before the start of the prefetch
      const u64 lim = t_use - tau_i;
      while (lo < hi) { u32 mid = lo + ((hi - lo + 1) >> 1); if (start2(start, K, T, mid + 1) <= lim) lo = mid; else hi = mid - 1; }
      if (aa <= lo) { a = aa; b = lo; any = 1; }
    }
    w[2 * d] = a; w[2 * d + 1] = b;
  }
  win[c] = make_uint4(w[0], w[1], w[2], w[3]);
  keep[c] = any;
}

// sort keys of the kept candidates: (L + 1) in the high bits, period index below
__global__ __launch_bounds__(G10_BLOCK) void k_sort_keys(const u32* __restrict__ per_L, const u32* __restrict__ pos, u32 C,
                                                        u32 cbits, u64* __restrict__ keys) {
  const u32 c = blockIdx.x * G10_BLOCK + threadIdx.x;
  if (c >= C || pos[c + 1] == pos[c]) return;
  keys[pos[c]] = ((u64)(per_L[c] + 1) << cbits) | c;
}

__global__ __launch_bounds__(G10_BLOCK) void k_gather_sorted(const u64* __restrict__ keys, u32 n, u32 cbits,
                                                            const u32* __restrict__ per_t, const u32* __restrict__ per_R,
                                                            const u64* __restrict__ size, const uint4* __restrict__ win,
                                                            Cands out) {
  const u32 o = blockIdx.x * G10_BLOCK + threadIdx.x;
  if (o >= n) return;
  const u64 key = keys[o];
  const u32 c = (u32)(key & ((1ull << cbits) - 1ull));
  const uint4 w = win[c];
  const u64 s = size[per_t[c]];
  out.A[o] = make_uint4((u32)(key >> cbits), per_R[c], w.x, w.y);
  out.B[o] = make_uint4(w.z, w.w, (u32)s, (u32)(s >> 32));
  out.idx[o] = c;
}

// ---------------------------------------------------------------------------
// chunk-local rebuild of the prefix arrays (also used to initialise them)
// ---------------------------------------------------------------------------
template <class F>
__device__ __forceinline__ void rebuild_chunk(const Timelines& tl, u32 arr, u64* lds_tmp, F val) {
  const u32 chunk = blockIdx.x, ch = G10_BLOCK * tl.spt;
  const u32 j0 = chunk * ch + threadIdx.x * tl.spt;
  u64 acc = 0;
  for (u32 i = 0; i < tl.spt; ++i) { const u32 j = j0 + i; if (j < tl.K) acc += val(j); }
  u64 total;
  u64 run = block_scan_excl(acc, lds_tmp, total);
  for (u32 i = 0; i < tl.spt; ++i) {
    const u32 j = j0 + i;
    if (j < tl.K) { tl.px[(u64)j * PX + arr] = run; run += val(j); }
  }
  if (threadIdx.x == 0) tl.tot[(u64)arr * tl.nch + chunk] = total;
}

// Level 1: exclusive scan of the chunk totals of array `arr` by one workgroup.
__device__ __forceinline__ void rebuild_bases(const Timelines& tl, u32 arr, u64* lds_tmp) {
  const u32 per = (tl.nch + G10_BLOCK - 1) / G10_BLOCK;
  const u64* tot = tl.tot + (u64)arr * tl.nch;
  u64* base = tl.bases + (u64)arr * (tl.nch + 1);
  const u32 c0 = threadIdx.x * per;
  u64 acc = 0;
  for (u32 i = 0; i < per; ++i) if (c0 + i < tl.nch) acc += tot[c0 + i];
  u64 total;
  u64 run = block_scan_excl(acc, lds_tmp, total);
  for (u32 i = 0; i < per; ++i) if (c0 + i < tl.nch) { base[c0 + i] = run; run += tot[c0 + i]; }
  if (threadIdx.x == 0) base[tl.nch] = total;
}

// true on exactly the last workgroup to arrive; makes the other workgroups'
// global writes visible to it.  One release per workgroup (thread 0, after the
// barrier has ordered the other threads' writes before it) and one acquire in
// the last workgroup only: agent-scope fences write back / invalidate L2 on
// this multi-die part, so they are kept off the other waves.
__device__ __forceinline__ bool last_workgroup(u32* counter, u32* lds_flag) {
  __syncthreads();
  if (threadIdx.x == 0) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    const u32 t = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *lds_flag = (t == gridDim.x - 1);
  }
  __syncthreads();
  const bool last = *lds_flag != 0;
  if (last) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  return last;
}

__global__ __launch_bounds__(G10_BLOCK) void k_init_timelines(Timelines tl, Ctl* ctl) {
  __shared__ u64 tmp[G10_WAVES + 1];
  __shared__ u32 flag;
  const u64 cap = ctl->gpu_cap;
  rebuild_chunk(tl, A_OT, tmp, [&](u32 j) { return tl.pressure[j] > cap ? tl.dur[j] : 0ull; });
  for (u32 ch = 0; ch < 4; ++ch)
    rebuild_chunk(tl, A_FO + ch, tmp, [&](u32 j) { return tl.dur[j]; });       // nothing reserved yet
  if (threadIdx.x == 0) tl.hostmax[blockIdx.x] = 0;
  if (!last_workgroup(&ctl->commit_done, &flag)) return;
  for (u32 arr = 0; arr < N_ARR; ++arr) rebuild_bases(tl, arr, tmp);
  if (threadIdx.x == 0) {
    const u64 ot = tl.bases[(u64)A_OT * (tl.nch + 1) + tl.nch];
    ctl->overtime_before = ot;
    ctl->commit_done = 0;
    if (ot == 0) { ctl->done = 1; ctl->status = G10_FITS; }
  }
}

// ---------------------------------------------------------------------------
// scoring pass + arg-max + decision
// ---------------------------------------------------------------------------
struct Best {
  u64 hi, lo;
  u32 cand, pos, dest;
};

__device__ __forceinline__ void best_merge(Best& x, const Best& y) {
  if (better(y.hi, y.lo, y.cand, x.hi, x.lo, x.cand)) x = y;
}

__device__ __forceinline__ Best wave_best(Best x) {
#pragma unroll
  for (int o = G10_WAVE / 2; o > 0; o >>= 1) {
    Best y;
    y.hi = __shfl_xor(x.hi, o, G10_WAVE);
    y.lo = __shfl_xor(x.lo, o, G10_WAVE);
    y.cand = __shfl_xor(x.cand, o, G10_WAVE);
    y.pos = __shfl_xor(x.pos, o, G10_WAVE);
    y.dest = __shfl_xor(x.dest, o, G10_WAVE);
    best_merge(x, y);
  }
  return x;
}

__device__ __forceinline__ Best block_best(Best x, Best* lds) {
  x = wave_best(x);
  if (lane_id() == 0) lds[wave_id()] = x;
  __syncthreads();
  Best r = lds[0];
#pragma unroll
  for (u32 w = 1; w < G10_WAVES; ++w) best_merge(r, lds[w]);
  __syncthreads();
  return r;
}

// max of host_used over the slots [x, y] (plain coordinates, x <= y < K)
__device__ __forceinline__ u64 host_max_segment(const Timelines& tl, u32 x, u32 y) {
  const u32 ch = G10_BLOCK * tl.spt;
  const u32 c_lo = x / ch, c_hi = y / ch;
  u64 m = 0;
  for (u32 c = c_lo + threadIdx.x; c <= c_hi; c += G10_BLOCK) {
    const u32 s0 = c * ch, s1 = s0 + ch - 1;
    if (s0 >= x && s1 <= y) { const u64 v = tl.hostmax[c]; m = v > m ? v : m; }
  }
  // the (at most two) chunks cut by the segment ends: slot by slot
  for (int e = 0; e < 2; ++e) {
    const u32 c = e ? c_hi : c_lo;
    if (e && c_hi == c_lo) break;
    const u32 s0 = c * ch, s1 = s0 + ch - 1;
    if (s0 >= x && s1 <= y) continue;
    const u32 lo = s0 > x ? s0 : x, hi = s1 < y ? s1 : y;
    for (u32 j = lo + threadIdx.x; j <= hi; j += G10_BLOCK) { const u64 v = tl.host_used[j]; m = v > m ? v : m; }
  }
  return m;
}

// Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous
// run of candidate blocks so that its L2 sees one region of the timeline.
__device__ __forceinline__ u32 logical_block() {
  const u32 g = gridDim.x;
  return (g & 7u) ? blockIdx.x : (blockIdx.x & 7u) * (g >> 3) + (blockIdx.x >> 3);
}

__device__ __forceinline__ void load_bases(const Timelines& tl, u64* lds_base) {
  const u32 nb1 = tl.nch + 1;
  for (u32 i = threadIdx.x; i < N_ARR * nb1; i += G10_BLOCK) lds_base[i] = tl.bases[i];
  __syncthreads();
}

__global__ __launch_bounds__(G10_BLOCK) void k_score(Cands cd, u32 n_act, u32 per_block, Timelines tl, Ctl* ctl,
                                                    Partial* partials, const u32* __restrict__ per_t,
                                                    g10_migration* records, g10_dropped* dropped) {
  extern __shared__ u64 lds_base[];            // [5][nch + 1]
  __shared__ Best lds_best[G10_WAVES];
  __shared__ u64 lds_tmp[G10_WAVES + 1];
  __shared__ u32 lds_flag;
  if (ctl->done) return;
  load_bases(tl, lds_base);
  Prefix pf;
  pf.px = tl.px; pf.base = lds_base; pf.K = tl.K; pf.nb1 = tl.nch + 1; pf.shift_ch = tl.shift_ch;
  Machine m;
  m.bwo[0] = ctl->bw_out[0]; m.bwo[1] = ctl->bw_out[1]; m.bwi[0] = ctl->bw_in[0]; m.bwi[1] = ctl->bw_in[1];

  Best best;
  best.hi = 0; best.lo = 0; best.cand = 0xffffffffu; best.pos = 0; best.dest = 0;
  const u32 p0 = logical_block() * per_block;
  const u32 p1 = p0 + per_block < n_act ? p0 + per_block : n_act;
  for (u32 p = p0 + threadIdx.x; p < p1; p += G10_BLOCK) {
    const uint4 A = cd.A[p], B = cd.B[p];
    const u64 s = ((u64)B.w << 32) | B.z;
    u32 d;
    u64 ot;
    if (!policy(pf, m, A, B, s, d, ot)) continue;
    const u64 hi = __umul64hi(s, ot), lo = s * ot;
    if ((hi | lo) == 0) continue;
    if (hi > best.hi || (hi == best.hi && lo >= best.lo)) {           // the index is needed on ties only
      const u32 c = cd.idx[p];
      if (better(hi, lo, c, best.hi, best.lo, best.cand)) { best.hi = hi; best.lo = lo; best.cand = c; best.pos = p; best.dest = d; }
    }
  }
  best = block_best(best, lds_best);
  if (threadIdx.x == 0) {
    Partial q;
    q.hi = best.hi; q.lo = best.lo; q.cand = best.cand; q.pos = best.pos; q.dest = best.dest; q.pad = 0;
    partials[blockIdx.x] = q;
  }
  if (!last_workgroup(&ctl->score_done, &lds_flag)) return;

  // ---- last workgroup: reduce the partials and decide -------------------------------
  best.hi = 0; best.lo = 0; best.cand = 0xffffffffu; best.pos = 0; best.dest = 0;
  for (u32 i = threadIdx.x; i < gridDim.x; i += G10_BLOCK) {
    const Partial q = partials[i];
    Best y; y.hi = q.hi; y.lo = q.lo; y.cand = q.cand; y.pos = q.pos; y.dest = q.dest;
    best_merge(best, y);
  }
  best = block_best(best, lds_best);
  if (threadIdx.x == 0) lds_flag = ctl->max_iter && ctl->n_iter >= ctl->max_iter;
  __syncthreads();
  const bool limit = lds_flag != 0;                // read once: thread 0 advances n_iter below
  const bool none = (best.hi | best.lo) == 0;
  if (limit || none) {
    if (threadIdx.x == 0) {
      if (!limit) { ctl->n_iter += 1; ctl->n_evals += ctl->C - ctl->n_mig - ctl->n_drop; }
      ctl->done = 1;
      ctl->status = limit ? G10_TRUNCATED : G10_RESIDUAL;
      ctl->action = ACT_NONE;
      ctl->score_done = 0;
    }
    return;
  }
  const u32 p = best.pos, d = best.dest;
  const uint4 A = cd.A[p], B = cd.B[p];
  const u32 L1 = A.x, R = A.y;
  const u64 s = ((u64)B.w << 32) | B.z;
  bool room = true;
  if (d == G10_HOST) {                          // host memory must hold it during the whole period
    u64 mx = 0;
    const u32 x = L1, y = R - 1;                // doubled coordinates, y - x < K
    if (y < tl.K) mx = host_max_segment(tl, x, y);
    else if (x >= tl.K) mx = host_max_segment(tl, x - tl.K, y - tl.K);
    else {
      const u64 m1 = host_max_segment(tl, x, tl.K - 1), m2 = host_max_segment(tl, 0, y - tl.K);
      mx = m1 > m2 ? m1 : m2;
    }
    mx = block_max(mx, lds_tmp);
    room = s <= ctl->host_cap && mx <= ctl->host_cap - s;
  }
  __syncthreads();                              // every thread has read the candidate before it is retired
  if (threadIdx.x == 0) {
    const u32 a = d ? B.x : A.z, b = d ? B.y : A.w;
    const u64 it = ctl->n_iter;
    ctl->n_iter = it + 1;
    ctl->n_evals += ctl->C - ctl->n_mig - ctl->n_drop;
    cd.A[p] = make_uint4(L1, R, 1u, 0u);                             // the candidate leaves the live set
    cd.B[p] = make_uint4(1u, 0u, B.z, B.w);
    if (!room) {
      g10_dropped dr; dr.iteration = it; dr.cand = best.cand; dr.reserved = 0;
      dropped[ctl->n_drop] = dr;
      ctl->n_drop += 1;
      ctl->action = ACT_DROP;
    } else {
      const u64 tau_o = ceil_div_x1000(s, ctl->bw_out[d]), tau_i = ceil_div_x1000(s, ctl->bw_in[d]);
      g10_migration mg;
      mg.cand = best.cand; mg.tensor = per_t[best.cand];
      mg.evict_after = L1 - 1; mg.absent_first = a % tl.K; mg.absent_last = b % tl.K; mg.next_use = R % tl.K;
      mg.dest = d; mg.wraps = R >= tl.K ? 1u : 0u;
      mg.size_bytes = s; mg.t_out_ns = tau_o; mg.t_in_ns = tau_i; mg.benefit_lo = best.lo; mg.benefit_hi = best.hi;
      records[ctl->n_mig] = mg;
      ctl->n_mig += 1;
      ctl->action = ACT_COMMIT;
      ctl->dest = d; ctl->pos = p; ctl->cand = best.cand;
      ctl->L1 = L1; ctl->R = R; ctl->a = a; ctl->b = b;
      ctl->s = s; ctl->tau_o = tau_o; ctl->tau_i = tau_i;
      ctl->fo_base = pf.at(A_FO + d, pf.slot(L1));
      ctl->fi_end = pf.at(A_FI + d, pf.slot(R));
    }
    ctl->score_done = 0;
  }
}

// ---------------------------------------------------------------------------
// compaction of candidates that can never score again
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(G10_BLOCK) void k_alive(Cands cd, u32 n_act, Timelines tl, const Ctl* ctl, u32* __restrict__ flag) {
  extern __shared__ u64 lds_base[];
  load_bases(tl, lds_base);
  Prefix pf;
  pf.px = tl.px; pf.base = lds_base; pf.K = tl.K; pf.nb1 = tl.nch + 1; pf.shift_ch = tl.shift_ch;
  Machine m;
  m.bwo[0] = ctl->bw_out[0]; m.bwo[1] = ctl->bw_out[1]; m.bwi[0] = ctl->bw_in[0]; m.bwi[1] = ctl->bw_in[1];
  for (u32 p = blockIdx.x * G10_BLOCK + threadIdx.x; p < n_act; p += gridDim.x * G10_BLOCK) {
    const uint4 A = cd.A[p], B = cd.B[p];
    flag[p] = alive(pf, m, A, B, ((u64)B.w << 32) | B.z) ? 1u : 0u;
  }
}

__global__ __launch_bounds__(G10_BLOCK) void k_compact(Cands src, Cands dst, const u32* __restrict__ pos, u32 n_act) {
  const u32 p = blockIdx.x * G10_BLOCK + threadIdx.x;
  if (p >= n_act || pos[p + 1] == pos[p]) return;
  const u32 o = pos[p];
  dst.A[o] = src.A[p];
  dst.B[o] = src.B[p];
  dst.idx[o] = src.idx[p];
}

// ---------------------------------------------------------------------------
// commit: range updates + chunk rebuild
// ---------------------------------------------------------------------------
// position of plain slot j inside the doubled range [x, y] (y - x < K), or ~0u
__device__ __forceinline__ u32 in_doubled(u32 j, u32 K, u32 x, u32 y) {
  if (j >= x && j <= y) return j;
  const u32 jj = j + K;
  if (jj >= x && jj <= y) return jj;
  return 0xffffffffu;
}

__global__ __launch_bounds__(G10_BLOCK) void k_commit(Timelines tl, Ctl* ctl) {
  __shared__ u64 tmp[G10_WAVES + 1];
  __shared__ u32 flag;
  if (ctl->done || ctl->action != ACT_COMMIT) return;
  const u32 K = tl.K, ch = G10_BLOCK * tl.spt, chunk = blockIdx.x;
  const u32 d = ctl->dest, L1 = ctl->L1, R = ctl->R, a = ctl->a, b = ctl->b;
  const u64 s = ctl->s, tau_o = ctl->tau_o, tau_i = ctl->tau_i, cap = ctl->gpu_cap;
  const u32 s0 = chunk * ch, s1 = (s0 + ch - 1 < K - 1) ? s0 + ch - 1 : K - 1;
  // does the chunk meet the period interior [L1, R-1]?  (the only slots that change)
  const u32 x = L1, y = R - 1;
  bool touched;
  if (y < K) touched = !(s1 < x || s0 > y);
  else if (x >= K) touched = !(s1 < x - K || s0 > y - K);
  else touched = !(s1 < x) || !(s0 > y - K);
  if (touched) {
    u64* busy_o = tl.busy + (u64)(0 + d) * K;
    u64* busy_i = tl.busy + (u64)(2 + d) * K;
    const u64* base_o = tl.bases + (u64)(A_FO + d) * (tl.nch + 1);
    const u64* base_i = tl.bases + (u64)(A_FI + d) * (tl.nch + 1);
    const u64 bo = base_o[chunk], bi = base_i[chunk], tot_o = base_o[tl.nch], tot_i = base_i[tl.nch];
    const u64 fo_base = ctl->fo_base, fi_end = ctl->fi_end;
    for (u32 i = 0; i < tl.spt; ++i) {
      const u32 j = s0 + threadIdx.x * tl.spt + i;
      if (j >= K) break;
      if (in_doubled(j, K, a, b) != 0xffffffffu) tl.pressure[j] -= s;
      u32 jj = in_doubled(j, K, L1, a - 1);                 // eviction window: earliest free time first
      if (jj != 0xffffffffu) {
        const u64 fr = tl.dur[j] - busy_o[j];
        const u64 before = (jj >= K ? tot_o : 0) + bo + tl.px[(u64)j * PX + A_FO + d] - fo_base;
        const u64 used = before < tau_o ? before : tau_o;
        const u64 take = fr < tau_o - used ? fr : tau_o - used;
        busy_o[j] += take;
      }
      jj = in_doubled(j, K, b + 1, R - 1);                  // prefetch window: latest free time first
      if (jj != 0xffffffffu) {
        const u64 fr = tl.dur[j] - busy_i[j];
        const u64 upto = (jj >= K ? tot_i : 0) + bi + tl.px[(u64)j * PX + A_FI + d] + fr;   // free time before slot jj + 1
        const u64 after = fi_end - upto;
        const u64 used = after < tau_i ? after : tau_i;
        const u64 take = fr < tau_i - used ? fr : tau_i - used;
        busy_i[j] += take;
      }
      if (d == G10_HOST && in_doubled(j, K, L1, R - 1) != 0xffffffffu) tl.host_used[j] += s;
    }
    __syncthreads();                                         // slot values final before the rebuild reads them
    rebuild_chunk(tl, A_OT, tmp, [&](u32 j) { return tl.pressure[j] > cap ? tl.dur[j] : 0ull; });
    rebuild_chunk(tl, A_FO + d, tmp, [&](u32 j) { return tl.dur[j] - busy_o[j]; });
    rebuild_chunk(tl, A_FI + d, tmp, [&](u32 j) { return tl.dur[j] - busy_i[j]; });
    if (d == G10_HOST) {
      u64 m = 0;
      for (u32 i = 0; i < tl.spt; ++i) {
        const u32 j = s0 + threadIdx.x * tl.spt + i;
        if (j < K) { const u64 v = tl.host_used[j]; m = v > m ? v : m; }
      }
      m = block_max(m, tmp);
      if (threadIdx.x == 0) tl.hostmax[chunk] = m;
    }
  }
  if (!last_workgroup(&ctl->commit_done, &flag)) return;
  rebuild_bases(tl, A_OT, tmp);
  rebuild_bases(tl, A_FO + d, tmp);
  rebuild_bases(tl, A_FI + d, tmp);
  if (threadIdx.x == 0) {
    ctl->commit_done = 0;
    ctl->action = ACT_NONE;
    if (tl.bases[(u64)A_OT * (tl.nch + 1) + tl.nch] == 0) { ctl->done = 1; ctl->status = G10_FITS; }
  }
}

__global__ __launch_bounds__(G10_BLOCK) void k_max_u64p(const u64* __restrict__ v, u64 n, u64* out) {
  __shared__ u64 tmp[G10_WAVES + 1];
  u64 m = 0;
  for (u64 i = (u64)blockIdx.x * G10_BLOCK + threadIdx.x; i < n; i += (u64)gridDim.x * G10_BLOCK) m = v[i] > m ? v[i] : m;
  m = block_max(m, tmp);
  if (threadIdx.x == 0) atomicMax((unsigned long long*)out, (unsigned long long)m);
}

template <class T>
int dalloc(T** out, u64 elems) {
  void* q = nullptr;
  if (hipMalloc(&q, (elems ? elems : 1) * sizeof(T)) != hipSuccess) { (void)hipGetLastError(); return G10_ENOMEM; }
  *out = (T*)q;
  return G10_OK;
}

inline u32 bits_for(u64 max_value) {
  u32 b = 1;
  while (b < 64 && (max_value >> b)) ++b;
  return b;
}

}  // namespace

#define G10_TRY(x) do { int rc_ = (x); if (rc_) return rc_; } while (0)

struct PlanWork {
  u32 K = 0, nch = 0, spt = 1, shift_ch = 8;
  u64 C = 0;
  uint4* win = nullptr;
  u32 *keep = nullptr, *scratch32 = nullptr, *hist = nullptr;
  u64 *keys = nullptr, *keys_alt = nullptr;
  Cands cd[2] = {};
  u64 *pressure = nullptr, *busy = nullptr, *host_used = nullptr, *px = nullptr, *tot = nullptr, *bases = nullptr,
      *hostmax = nullptr, *peak_after = nullptr;
  Ctl* ctl = nullptr;
  Partial* partials = nullptr;
  g10_migration* records = nullptr;
  g10_dropped* dropped = nullptr;
  // host copies handed out through g10_result
  g10_migration* h_records = nullptr;
  g10_dropped* h_dropped = nullptr;
  u64* h_pressure = nullptr;
  hipEvent_t ev[2] = {nullptr, nullptr};
  hipEvent_t* prof = nullptr;
  u32 n_prof = 0;
};

void plan_work_free(PlanWork* w) {
  if (!w) return;
  void* dev[] = {w->win, w->keep, w->scratch32, w->hist, w->keys, w->keys_alt, w->cd[0].A, w->cd[0].B, w->cd[0].idx,
                 w->cd[1].A, w->cd[1].B, w->cd[1].idx, w->pressure, w->busy, w->host_used, w->px, w->tot, w->bases,
                 w->hostmax, w->peak_after, w->ctl, w->partials, w->records, w->dropped};
  for (void* p : dev) if (p) (void)hipFree(p);
  free(w->h_records);
  free(w->h_dropped);
  free(w->h_pressure);
  for (int i = 0; i < 2; ++i) if (w->ev[i]) (void)hipEventDestroy(w->ev[i]);
  for (u32 i = 0; i < w->n_prof; ++i) (void)hipEventDestroy(w->prof[i]);
  free(w->prof);
  delete w;
}

static const u32 MAX_SCORE_BLOCKS = 2048;
static const u32 BATCH = 32;                     // ranking passes enqueued between two polls of the done flag

static int work_alloc(g10_plan_s* h) {
  PlanWork* w = new (std::nothrow) PlanWork();
  if (!w) return G10_ENOMEM;
  h->work = w;
  const u32 K = h->K;
  const u64 C = h->n_periods;
  w->K = K; w->C = C;
  w->spt = 1; w->shift_ch = 8;
  while ((u64)G10_BLOCK * w->spt * 1024 < K) { w->spt *= 2; w->shift_ch += 1; }   // at most 1024 chunks
  const u32 ch = G10_BLOCK * w->spt;
  w->nch = (K + ch - 1) / ch;
  G10_TRY(dalloc(&w->win, C));
  G10_TRY(dalloc(&w->keep, C + 1));
  const u64 he = radix_hist_elems(C);
  G10_TRY(dalloc(&w->hist, he));
  G10_TRY(dalloc(&w->scratch32, scan_scratch_elems(he > C ? he : C)));
  G10_TRY(dalloc(&w->keys, C)); G10_TRY(dalloc(&w->keys_alt, C));
  for (int i = 0; i < 2; ++i) {
    G10_TRY(dalloc(&w->cd[i].A, C)); G10_TRY(dalloc(&w->cd[i].B, C)); G10_TRY(dalloc(&w->cd[i].idx, C));
  }
  G10_TRY(dalloc(&w->pressure, K)); G10_TRY(dalloc(&w->busy, (u64)4 * K)); G10_TRY(dalloc(&w->host_used, K));
  G10_TRY(dalloc(&w->px, (u64)PX * K));
  G10_TRY(dalloc(&w->tot, (u64)N_ARR * w->nch));
  G10_TRY(dalloc(&w->bases, (u64)N_ARR * (w->nch + 1)));
  G10_TRY(dalloc(&w->hostmax, w->nch));
  G10_TRY(dalloc(&w->peak_after, 1));
  G10_TRY(dalloc(&w->ctl, 1));
  G10_TRY(dalloc(&w->partials, MAX_SCORE_BLOCKS));
  G10_TRY(dalloc(&w->records, C));
  G10_TRY(dalloc(&w->dropped, C));
  w->h_records = (g10_migration*)malloc((C ? C : 1) * sizeof(g10_migration));
  w->h_dropped = (g10_dropped*)malloc((C ? C : 1) * sizeof(g10_dropped));
  w->h_pressure = (u64*)malloc((u64)K * sizeof(u64));
  if (!w->h_records || !w->h_dropped || !w->h_pressure) return G10_ENOMEM;
  for (int i = 0; i < 2; ++i) G10_HIP(hipEventCreate(&w->ev[i]));
  return G10_OK;
}

// launch shape of the scoring pass for n live candidates
static void score_shape(u32 n, u32& grid, u32& per_block) {
  grid = (n + 2 * G10_BLOCK - 1) / (2 * G10_BLOCK);            // about two candidates per thread
  if (grid < 1) grid = 1;
  if (grid >= 8) grid = (grid + 7u) & ~7u;                     // a multiple of the XCD count
  u32 cap = 512;                                               // two workgroups per CU: more only adds fences
  if (const char* e = getenv("G10_SCORE_BLOCKS")) { u32 v = (u32)atoi(e); if (v >= 8 && v <= MAX_SCORE_BLOCKS) cap = v & ~7u; }
  if (grid > cap) grid = cap;
  per_block = (n + grid - 1) / grid;
  per_block = (per_block + G10_BLOCK - 1) / G10_BLOCK * G10_BLOCK;
  if (per_block < G10_BLOCK) per_block = G10_BLOCK;
}

int plan_run(g10_plan_s* h, const g10_params* p, g10_result* out) {
  if (!h->work) {
    int rc = work_alloc(h);
    if (rc) { plan_work_free(h->work); h->work = nullptr; return rc; }
  }
  PlanWork* w = h->work;
  hipStream_t s = h->stream;
  const u32 K = h->K;
  const u32 C = (u32)h->n_periods;
  if (p->profile && !w->prof) {
    w->prof = (hipEvent_t*)calloc(2 * BATCH, sizeof(hipEvent_t));
    if (!w->prof) return G10_ENOMEM;
    for (u32 i = 0; i < 2 * BATCH; ++i) { G10_HIP(hipEventCreate(&w->prof[i])); w->n_prof = i + 1; }
  }

  G10_HIP(hipEventRecord(w->ev[0], s));
  Ctl hc;
  memset(&hc, 0, sizeof hc);
  hc.gpu_cap = p->gpu_cap_bytes; hc.host_cap = p->host_cap_bytes;
  for (int d = 0; d < 2; ++d) { hc.bw_out[d] = p->bw_out_Bpus[d]; hc.bw_in[d] = p->bw_in_Bpus[d]; }
  hc.max_iter = p->max_iterations;
  hc.C = C;
  G10_HIP(hipMemcpyAsync(w->ctl, &hc, sizeof hc, hipMemcpyHostToDevice, s));

  Timelines tl;
  tl.dur = h->dur; tl.pressure = w->pressure; tl.busy = w->busy; tl.host_used = w->host_used; tl.px = w->px;
  tl.tot = w->tot; tl.bases = w->bases; tl.hostmax = w->hostmax; tl.K = K; tl.nch = w->nch; tl.spt = w->spt;
  tl.shift_ch = w->shift_ch;

  G10_HIP(hipMemcpyAsync(w->pressure, h->pressure_buf + 1, (u64)K * 8, hipMemcpyDeviceToDevice, s));
  G10_HIP(hipMemsetAsync(w->busy, 0, (u64)4 * K * 8, s));
  G10_HIP(hipMemsetAsync(w->host_used, 0, (u64)K * 8, s));
  G10_HIP(hipMemsetAsync(w->peak_after, 0, 8, s));
  hipLaunchKernelGGL(k_init_timelines, dim3(w->nch), dim3(G10_BLOCK), 0, s, tl, w->ctl);
  G10_HIP(hipGetLastError());

  // candidates: windows per destination; keep those with at least one valid window; sort by period start
  u32 n_act = 0;
  const u32 cbits = bits_for(C ? C - 1 : 0);
  const u32 gC = (C + G10_BLOCK - 1) / G10_BLOCK;
  if (C) {
    hipLaunchKernelGGL(k_prep, dim3(gC), dim3(G10_BLOCK), 0, s, h->per_t, h->per_L, h->per_R, h->size, h->start, K, h->T, C,
                       w->ctl, w->win, w->keep);
    G10_HIP(hipGetLastError());
    G10_TRY(scan_excl_u32(w->keep, w->keep, C, w->scratch32, s));
    G10_HIP(hipMemcpyAsync(&n_act, w->keep + C, sizeof(u32), hipMemcpyDeviceToHost, s));
  }
  G10_HIP(hipMemcpyAsync(&hc, w->ctl, sizeof hc, hipMemcpyDeviceToHost, s));
  G10_HIP(hipStreamSynchronize(s));
  const u64 overtime_before = hc.overtime_before;
  int cur = 0;
  if (n_act && !hc.done) {
    hipLaunchKernelGGL(k_sort_keys, dim3(gC), dim3(G10_BLOCK), 0, s, h->per_L, w->keep, C, cbits, w->keys);
    u64 *keys = w->keys, *alt = w->keys_alt;
    G10_TRY(radix_sort_u64(&keys, &alt, n_act, cbits + bits_for(2ull * K), w->hist, w->scratch32, s));
    hipLaunchKernelGGL(k_gather_sorted, dim3((n_act + G10_BLOCK - 1) / G10_BLOCK), dim3(G10_BLOCK), 0, s, keys, n_act, cbits,
                       h->per_t, h->per_R, h->size, w->win, w->cd[cur]);
    G10_HIP(hipGetLastError());
  }

  // the greedy loop
  const size_t lds = (size_t)N_ARR * (w->nch + 1) * sizeof(u64);
  u64 launches = 0, streamed = 0, enqueued = 0;
  double score_ms = 0.0, full_ms = 0.0;
  u64 full_launches = 0;
  const u32 n_full = n_act;
  const u64 max_passes = (u64)n_act + 2;
  while (!hc.done) {
    if (enqueued > max_passes) return G10_EDEVICE;           // every pass removes a candidate or stops: cannot happen
    enqueued += BATCH;
    u32 grid, per_block;
    score_shape(n_act, grid, per_block);
    for (u32 i = 0; i < BATCH; ++i) {
      if (p->profile) G10_HIP(hipEventRecord(w->prof[2 * i], s));
      hipLaunchKernelGGL(k_score, dim3(grid), dim3(G10_BLOCK), lds, s, w->cd[cur], n_act, per_block, tl, w->ctl, w->partials,
                         h->per_t, w->records, w->dropped);
      if (p->profile) G10_HIP(hipEventRecord(w->prof[2 * i + 1], s));
      hipLaunchKernelGGL(k_commit, dim3(w->nch), dim3(G10_BLOCK), 0, s, tl, w->ctl);
    }
    // which candidates can still score?  (flags + positions; compacted below if it pays)
    u32 n_alive = n_act;
    const bool sweep = n_act > 4096;
    if (sweep) {
      u32 ga = (n_act + G10_BLOCK - 1) / G10_BLOCK;
      if (ga > MAX_SCORE_BLOCKS) ga = MAX_SCORE_BLOCKS;
      hipLaunchKernelGGL(k_alive, dim3(ga), dim3(G10_BLOCK), lds, s, w->cd[cur], n_act, tl, w->ctl, w->keep);
      G10_TRY(scan_excl_u32(w->keep, w->keep, n_act, w->scratch32, s));
      G10_HIP(hipMemcpyAsync(&n_alive, w->keep + n_act, sizeof(u32), hipMemcpyDeviceToHost, s));
    }
    G10_HIP(hipGetLastError());
    G10_HIP(hipMemcpyAsync(&hc, w->ctl, sizeof hc, hipMemcpyDeviceToHost, s));
    G10_HIP(hipStreamSynchronize(s));
    // scoring launches that did work: one per counted pass, plus the one that hit the pass limit
    const u64 ran = hc.n_iter + (hc.done && hc.status == G10_TRUNCATED ? 1 : 0) - launches;
    const u32 cnt = (u32)(ran < BATCH ? ran : BATCH);
    if (p->profile)
      for (u32 i = 0; i < cnt; ++i) {
        float ms = 0.f;
        G10_HIP(hipEventElapsedTime(&ms, w->prof[2 * i], w->prof[2 * i + 1]));
        score_ms += ms;
      }
    launches += cnt;
    streamed += (u64)cnt * n_act;
    if (p->profile && n_act == n_full) {                    // launches over the full candidate list
      full_launches += cnt;
      for (u32 i = 0; i < cnt; ++i) {
        float ms = 0.f;
        G10_HIP(hipEventElapsedTime(&ms, w->prof[2 * i], w->prof[2 * i + 1]));
        full_ms += ms;
      }
    }
    if (p->profile && getenv("G10_LOG") && cnt) {
      double b = 0.0;
      for (u32 i = 0; i < cnt; ++i) { float ms = 0.f; (void)hipEventElapsedTime(&ms, w->prof[2 * i], w->prof[2 * i + 1]); b += ms; }
      fprintf(stderr, "g10: passes %llu..%llu  live %u  score %.2f us/launch\n", (unsigned long long)(launches - cnt),
              (unsigned long long)launches, n_act, 1e3 * b / cnt);
    }
    if (!hc.done && sweep && (u64)n_alive * 8 < (u64)n_act * 7) {
      hipLaunchKernelGGL(k_compact, dim3((n_act + G10_BLOCK - 1) / G10_BLOCK), dim3(G10_BLOCK), 0, s, w->cd[cur], w->cd[cur ^ 1],
                         w->keep, n_act);
      G10_HIP(hipGetLastError());
      cur ^= 1;
      n_act = n_alive;
    }
  }

  hipLaunchKernelGGL(k_max_u64p, dim3(K / G10_BLOCK / 4 + 1), dim3(G10_BLOCK), 0, s, w->pressure, (u64)K, w->peak_after);
  G10_HIP(hipGetLastError());
  u64 peak_after = 0, overtime_after = 0;
  G10_HIP(hipMemcpyAsync(&peak_after, w->peak_after, 8, hipMemcpyDeviceToHost, s));
  G10_HIP(hipMemcpyAsync(&overtime_after, w->bases + (u64)A_OT * (w->nch + 1) + w->nch, 8, hipMemcpyDeviceToHost, s));
  if (hc.n_mig) G10_HIP(hipMemcpyAsync(w->h_records, w->records, hc.n_mig * sizeof(g10_migration), hipMemcpyDeviceToHost, s));
  if (hc.n_drop) G10_HIP(hipMemcpyAsync(w->h_dropped, w->dropped, hc.n_drop * sizeof(g10_dropped), hipMemcpyDeviceToHost, s));
  G10_HIP(hipMemcpyAsync(w->h_pressure, w->pressure, (u64)K * 8, hipMemcpyDeviceToHost, s));
  G10_HIP(hipEventRecord(w->ev[1], s));
  G10_HIP(hipStreamSynchronize(s));
  float ms = 0.f;
  G10_HIP(hipEventElapsedTime(&ms, w->ev[0], w->ev[1]));

  memset(out, 0, sizeof *out);
  out->status = (int32_t)hc.status;
  out->n_migrations = hc.n_mig; out->n_iterations = hc.n_iter; out->n_dropped = hc.n_drop; out->n_cand_evals = hc.n_evals;
  out->peak_before = h->peak; out->peak_after = peak_after;
  out->overtime_before_ns = overtime_before; out->overtime_after_ns = overtime_after;
  out->migrations = w->h_records; out->dropped = w->h_dropped; out->pressure_after = w->h_pressure;
  out->score_launches = launches; out->score_cands_streamed = streamed;
  out->score_ms = score_ms; out->plan_ms = ms;
  out->full_launches = full_launches; out->full_cands = n_full; out->full_ms = full_ms;
  return G10_OK;
}
