// Smart tensor eviction on the device (G10, Section 4.3, Algorithm 1).
//
// State on the device (all u64 unless noted, K = kernel slots):
//   pressure[K]                 bytes resident per slot
//   busy[4][K]                  channel time already reserved per slot;
//                               channel = 2 * direction + destination
//                               (0 flash-out, 1 host-out, 2 flash-in, 3 host-in)
//   host_used[K]                bytes parked in host memory per slot
//   two-level prefix sums of five per-slot quantities, rebuilt where they
//   change after every commit:
//     array 0        over-capacity time   dur[k] * [pressure[k] > cap]
//     array 1 + ch   free channel time    dur[k] - busy[ch][k]
//   level 0 = exclusive prefix inside a chunk of CH slots (inch[5][K]),
//   level 1 = exclusive prefix of the chunk totals (bases[5][nch + 1]); a
//   prefix up to slot j is bases[j / CH] + inch[j].  Level 1 is small enough to
//   sit in LDS while candidates are scored.
//
// One ranking pass = two launches:
//   k_score   streams the candidate SoA (36 B per candidate), gathers the few
//             prefix words each candidate needs, reduces to the best
//             (benefit, lowest index) per workgroup; the last workgroup to
//             finish reduces the partials, decides (stop / drop / commit),
//             appends the migration record.
//   k_commit  one workgroup per chunk applies the range updates of the winner
//             (pressure, channel reservations, host memory) to its slots and
//             rebuilds its chunk's prefixes; the last workgroup rebuilds
//             level 1 and tests the "fits" stop rule.
// The host only enqueues batches of passes and polls a done flag per batch.

#include "g10_internal.h"

#include <new>
#include <stdlib.h>
#include <string.h>

namespace {

enum { A_OT = 0, A_FO = 1, A_FI = 3, N_ARR = 5 };   // FO + dest, FI + dest
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

struct Cands {                // active candidates, SoA
  u32 *idx, *L1, *R, *a0, *b0, *a1, *b1;
  u64* s;
};

struct Timelines {
  const u64* dur;
  u64* pressure;
  u64* busy;                  // [4][K]
  u64* host_used;
  u64* inch;                  // [5][K]
  u64* tot;                   // [5][nch]
  u64* bases;                 // [5][nch + 1]
  u64* hostmax;               // [nch]
  u32 K, nch, spt;            // chunk = 256 * spt slots
};

// ---------------------------------------------------------------------------
// prefix queries on the doubled timeline (two iterations end to end)
// ---------------------------------------------------------------------------
struct PrefixView {
  const u64* inch;            // global, [K]
  const u64* base;            // LDS or global, [nch + 1]
  u32 K, nch, shift_ch;       // chunk = 1 << shift_ch slots
  __device__ __forceinline__ u64 total() const { return base[nch]; }
  // sum over slots [0, j) of the doubled timeline, j in [0, 2K]
  __device__ __forceinline__ u64 at(u32 j) const {
    u64 add = 0;
    if (j >= K) { j -= K; add = base[nch]; }
    if (j == K) return add + base[nch];
    return add + base[j >> shift_ch] + inch[j];
  }
};

__device__ __forceinline__ bool carries(u64 free_ns, u64 bw, u64 bytes_x1000) {
  // free_ns >= ceil(bytes_x1000 / bw)  <=>  free_ns * bw >= bytes_x1000
  const u64 hi = __umul64hi(free_ns, bw);
  return hi != 0 || free_ns * bw >= bytes_x1000;
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
                                                   u32* __restrict__ a0, u32* __restrict__ b0, u32* __restrict__ a1,
                                                   u32* __restrict__ b1, u32* __restrict__ keep) {
  const u32 c = blockIdx.x * G10_BLOCK + threadIdx.x;
  if (c >= C) return;
  const u32 L = per_L[c], R = per_R[c];
  const u64 s = size[per_t[c]];
  const u64 t_r = start2(start, K, T, L + 1), t_use = start2(start, K, T, R), len = t_use - t_r;
  u32 any = 0;
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
    if (d == 0) { a0[c] = a; b0[c] = b; } else { a1[c] = a; b1[c] = b; }
  }
  keep[c] = any;
}

__global__ __launch_bounds__(G10_BLOCK) void k_gather_active(const u32* __restrict__ per_t, const u32* __restrict__ per_L,
                                                            const u32* __restrict__ per_R, const u64* __restrict__ size,
                                                            const u32* __restrict__ a0, const u32* __restrict__ b0,
                                                            const u32* __restrict__ a1, const u32* __restrict__ b1,
                                                            const u32* __restrict__ pos, u32 C, Cands out) {
  const u32 c = blockIdx.x * G10_BLOCK + threadIdx.x;
  if (c >= C || pos[c + 1] == pos[c]) return;
  const u32 o = pos[c];
  out.idx[o] = c;
  out.L1[o] = per_L[c] + 1;
  out.R[o] = per_R[c];
  out.a0[o] = a0[c]; out.b0[o] = b0[c];
  out.a1[o] = a1[c]; out.b1[o] = b1[c];
  out.s[o] = size[per_t[c]];
}

// ---------------------------------------------------------------------------
// chunk-local rebuild of the prefix arrays (also used to initialise them)
// ---------------------------------------------------------------------------
// Rebuilds array `arr` for the calling workgroup's chunk from per-slot values
// supplied by `val(slot)`.
template <class F>
__device__ __forceinline__ void rebuild_chunk(const Timelines& tl, u32 arr, u64* lds_tmp, F val) {
  const u32 chunk = blockIdx.x, ch = G10_BLOCK * tl.spt;
  const u32 j0 = chunk * ch + threadIdx.x * tl.spt;
  u64 acc = 0;
  for (u32 i = 0; i < tl.spt; ++i) { const u32 j = j0 + i; if (j < tl.K) acc += val(j); }
  u64 total;
  u64 run = block_scan_excl(acc, lds_tmp, total);
  u64* inch = tl.inch + (u64)arr * tl.K;
  for (u32 i = 0; i < tl.spt; ++i) {
    const u32 j = j0 + i;
    if (j < tl.K) { inch[j] = run; run += val(j); }
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
// global writes visible to it
__device__ __forceinline__ bool last_workgroup(u32* counter, u32* lds_flag) {
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) {
    const u32 t = atomicAdd(counter, 1u);
    *lds_flag = (t == gridDim.x - 1);
  }
  __syncthreads();
  const bool last = *lds_flag != 0;
  if (last) __threadfence();
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

__global__ __launch_bounds__(G10_BLOCK) void k_score(Cands cd, u32 n_act, Timelines tl, Ctl* ctl, Partial* partials,
                                                    const u32* __restrict__ per_t, g10_migration* records,
                                                    g10_dropped* dropped) {
  extern __shared__ u64 lds_base[];            // [5][nch + 1]
  __shared__ Best lds_best[G10_WAVES];
  __shared__ u64 lds_tmp[G10_WAVES + 1];
  __shared__ u32 lds_flag;
  if (ctl->done) return;

  const u32 nb1 = tl.nch + 1;
  for (u32 i = threadIdx.x; i < N_ARR * nb1; i += G10_BLOCK) lds_base[i] = tl.bases[i];
  __syncthreads();
  u32 shift_ch = 0;
  while ((1u << shift_ch) < G10_BLOCK * tl.spt) ++shift_ch;
  PrefixView pv[N_ARR];
#pragma unroll
  for (u32 arr = 0; arr < N_ARR; ++arr) {
    pv[arr].inch = tl.inch + (u64)arr * tl.K;
    pv[arr].base = lds_base + arr * nb1;
    pv[arr].K = tl.K; pv[arr].nch = tl.nch; pv[arr].shift_ch = shift_ch;
  }
  const u64 bwo0 = ctl->bw_out[0], bwo1 = ctl->bw_out[1], bwi0 = ctl->bw_in[0], bwi1 = ctl->bw_in[1];

  Best best;
  best.hi = 0; best.lo = 0; best.cand = 0xffffffffu; best.pos = 0; best.dest = 0;
  for (u32 p = blockIdx.x * G10_BLOCK + threadIdx.x; p < n_act; p += gridDim.x * G10_BLOCK) {
    const u32 L1 = cd.L1[p], R = cd.R[p];
    const u64 s = cd.s[p];
    const u64 x1000 = s * 1000ull;
#pragma unroll
    for (u32 d = 0; d < 2; ++d) {
      const u32 a = d ? cd.a1[p] : cd.a0[p], b = d ? cd.b1[p] : cd.b0[p];
      if (a > b) continue;                                            // no valid window for this destination
      const PrefixView& fo = pv[A_FO + d];
      if (!carries(fo.at(a) - fo.at(L1), d ? bwo1 : bwo0, x1000)) continue;      // eviction: slots [L1, a-1]
      const PrefixView& fi = pv[A_FI + d];
      if (!carries(fi.at(R) - fi.at(b + 1), d ? bwi1 : bwi0, x1000)) continue;   // prefetch: slots [b+1, R-1]
      const u64 ot = pv[A_OT].at(b + 1) - pv[A_OT].at(a);                        // over-capacity time while absent
      Best me;
      me.hi = __umul64hi(s, ot); me.lo = s * ot; me.cand = cd.idx[p]; me.pos = p; me.dest = d;
      if ((me.hi | me.lo) != 0) best_merge(best, me);
      break;                                                          // flash first: host only if flash cannot
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
  const u32 L1 = cd.L1[p], R = cd.R[p];
  const u64 s = cd.s[p];
  bool room = true;
  if (d == G10_HOST) {                          // host memory must hold it during the whole period
    u64 m = 0;
    const u32 x = L1, y = R - 1;                // doubled coordinates, y - x < K
    if (y < tl.K) m = host_max_segment(tl, x, y);
    else if (x >= tl.K) m = host_max_segment(tl, x - tl.K, y - tl.K);
    else {
      const u64 m1 = host_max_segment(tl, x, tl.K - 1), m2 = host_max_segment(tl, 0, y - tl.K);
      m = m1 > m2 ? m1 : m2;
    }
    m = block_max(m, lds_tmp);
    room = s <= ctl->host_cap && m <= ctl->host_cap - s;
  }
  if (threadIdx.x == 0) {
    const u32 a = d ? cd.a1[p] : cd.a0[p], b = d ? cd.b1[p] : cd.b0[p];
    const u64 it = ctl->n_iter;
    ctl->n_iter = it + 1;
    ctl->n_evals += ctl->C - ctl->n_mig - ctl->n_drop;
    cd.a0[p] = 1; cd.b0[p] = 0; cd.a1[p] = 1; cd.b1[p] = 0;        // the candidate leaves the live set
    if (!room) {
      g10_dropped dr; dr.iteration = it; dr.cand = best.cand; dr.reserved = 0;
      dropped[ctl->n_drop] = dr;
      ctl->n_drop += 1;
      ctl->action = ACT_DROP;
    } else {
      const u64 tau_o = ceil_div_x1000(s, ctl->bw_out[d]), tau_i = ceil_div_x1000(s, ctl->bw_in[d]);
      g10_migration m;
      m.cand = best.cand; m.tensor = per_t[best.cand];
      m.evict_after = L1 - 1; m.absent_first = a % tl.K; m.absent_last = b % tl.K; m.next_use = R % tl.K;
      m.dest = d; m.wraps = R >= tl.K ? 1u : 0u;
      m.size_bytes = s; m.t_out_ns = tau_o; m.t_in_ns = tau_i; m.benefit_lo = best.lo; m.benefit_hi = best.hi;
      records[ctl->n_mig] = m;
      ctl->n_mig += 1;
      ctl->action = ACT_COMMIT;
      ctl->dest = d; ctl->pos = p; ctl->cand = best.cand;
      ctl->L1 = L1; ctl->R = R; ctl->a = a; ctl->b = b;
      ctl->s = s; ctl->tau_o = tau_o; ctl->tau_i = tau_i;
      ctl->fo_base = pv[A_FO + d].at(L1);
      ctl->fi_end = pv[A_FI + d].at(R);
    }
    ctl->score_done = 0;
  }
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
    const u64* inch_o = tl.inch + (u64)(A_FO + d) * K;
    const u64* inch_i = tl.inch + (u64)(A_FI + d) * K;
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
        const u64 before = (jj >= K ? tot_o : 0) + bo + inch_o[j] - fo_base;
        const u64 used = before < tau_o ? before : tau_o;
        const u64 take = fr < tau_o - used ? fr : tau_o - used;
        busy_o[j] += take;
      }
      jj = in_doubled(j, K, b + 1, R - 1);                  // prefetch window: latest free time first
      if (jj != 0xffffffffu) {
        const u64 fr = tl.dur[j] - busy_i[j];
        const u64 upto = (jj >= K ? tot_i : 0) + bi + inch_i[j] + fr;   // free time before slot jj + 1
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

}  // namespace

#define G10_TRY(x) do { int rc_ = (x); if (rc_) return rc_; } while (0)

struct PlanWork {
  // sized by the trace
  u32 K = 0, nch = 0, spt = 1;
  u64 C = 0;
  u32 *a0 = nullptr, *b0 = nullptr, *a1 = nullptr, *b1 = nullptr, *keep = nullptr, *scratch32 = nullptr;
  Cands cd = {};
  u64 *pressure = nullptr, *busy = nullptr, *host_used = nullptr, *inch = nullptr, *tot = nullptr, *bases = nullptr,
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
  void* dev[] = {w->a0, w->b0, w->a1, w->b1, w->keep, w->scratch32, w->cd.idx, w->cd.L1, w->cd.R, w->cd.a0, w->cd.b0,
                 w->cd.a1, w->cd.b1, w->cd.s, w->pressure, w->busy, w->host_used, w->inch, w->tot, w->bases, w->hostmax,
                 w->peak_after, w->ctl, w->partials, w->records, w->dropped};
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
static const u32 BATCH = 64;                     // ranking passes enqueued between two polls of the done flag

static int work_alloc(g10_plan_s* h) {
  PlanWork* w = new (std::nothrow) PlanWork();
  if (!w) return G10_ENOMEM;
  h->work = w;
  const u32 K = h->K;
  const u64 C = h->n_periods;
  w->K = K; w->C = C;
  w->spt = 1;
  while ((u64)G10_BLOCK * w->spt * 1024 < K) w->spt *= 2;      // at most 1024 chunks; chunk size a power of two
  const u32 ch = G10_BLOCK * w->spt;
  w->nch = (K + ch - 1) / ch;
  G10_TRY(dalloc(&w->a0, C)); G10_TRY(dalloc(&w->b0, C)); G10_TRY(dalloc(&w->a1, C)); G10_TRY(dalloc(&w->b1, C));
  G10_TRY(dalloc(&w->keep, C + 1));
  G10_TRY(dalloc(&w->scratch32, scan_scratch_elems(C)));
  G10_TRY(dalloc(&w->cd.idx, C)); G10_TRY(dalloc(&w->cd.L1, C)); G10_TRY(dalloc(&w->cd.R, C));
  G10_TRY(dalloc(&w->cd.a0, C)); G10_TRY(dalloc(&w->cd.b0, C)); G10_TRY(dalloc(&w->cd.a1, C)); G10_TRY(dalloc(&w->cd.b1, C));
  G10_TRY(dalloc(&w->cd.s, C));
  G10_TRY(dalloc(&w->pressure, K)); G10_TRY(dalloc(&w->busy, (u64)4 * K)); G10_TRY(dalloc(&w->host_used, K));
  G10_TRY(dalloc(&w->inch, (u64)N_ARR * K));
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
  tl.dur = h->dur; tl.pressure = w->pressure; tl.busy = w->busy; tl.host_used = w->host_used; tl.inch = w->inch;
  tl.tot = w->tot; tl.bases = w->bases; tl.hostmax = w->hostmax; tl.K = K; tl.nch = w->nch; tl.spt = w->spt;

  G10_HIP(hipMemcpyAsync(w->pressure, h->pressure_buf + 1, (u64)K * 8, hipMemcpyDeviceToDevice, s));
  G10_HIP(hipMemsetAsync(w->busy, 0, (u64)4 * K * 8, s));
  G10_HIP(hipMemsetAsync(w->host_used, 0, (u64)K * 8, s));
  G10_HIP(hipMemsetAsync(w->peak_after, 0, 8, s));
  hipLaunchKernelGGL(k_init_timelines, dim3(w->nch), dim3(G10_BLOCK), 0, s, tl, w->ctl);
  G10_HIP(hipGetLastError());

  // candidates: windows per destination, then keep those with at least one valid window
  u32 n_act = 0;
  if (C) {
    const u32 g = (C + G10_BLOCK - 1) / G10_BLOCK;
    hipLaunchKernelGGL(k_prep, dim3(g), dim3(G10_BLOCK), 0, s, h->per_t, h->per_L, h->per_R, h->size, h->start, K, h->T, C,
                       w->ctl, w->a0, w->b0, w->a1, w->b1, w->keep);
    G10_HIP(hipGetLastError());
    G10_TRY(scan_excl_u32(w->keep, w->keep, C, w->scratch32, s));
    hipLaunchKernelGGL(k_gather_active, dim3(g), dim3(G10_BLOCK), 0, s, h->per_t, h->per_L, h->per_R, h->size, w->a0, w->b0,
                       w->a1, w->b1, w->keep, C, w->cd);
    G10_HIP(hipGetLastError());
    G10_HIP(hipMemcpyAsync(&n_act, w->keep + C, sizeof(u32), hipMemcpyDeviceToHost, s));
  }
  G10_HIP(hipMemcpyAsync(&hc, w->ctl, sizeof hc, hipMemcpyDeviceToHost, s));
  G10_HIP(hipStreamSynchronize(s));
  const u64 overtime_before = hc.overtime_before;

  // the greedy loop
  u32 grid = (n_act + G10_BLOCK - 1) / G10_BLOCK;
  if (grid < 1) grid = 1;
  if (grid > MAX_SCORE_BLOCKS) grid = MAX_SCORE_BLOCKS;
  const size_t lds = (size_t)N_ARR * (w->nch + 1) * sizeof(u64);
  u64 launches = 0;
  double score_ms = 0.0;
  u64 enqueued = 0;
  while (!hc.done) {
    if (enqueued > (u64)n_act + 2) return G10_EDEVICE;      // every pass removes a candidate or stops: cannot happen
    enqueued += BATCH;
    for (u32 i = 0; i < BATCH; ++i) {
      if (p->profile) G10_HIP(hipEventRecord(w->prof[2 * i], s));
      hipLaunchKernelGGL(k_score, dim3(grid), dim3(G10_BLOCK), lds, s, w->cd, n_act, tl, w->ctl, w->partials, h->per_t,
                         w->records, w->dropped);
      if (p->profile) G10_HIP(hipEventRecord(w->prof[2 * i + 1], s));
      hipLaunchKernelGGL(k_commit, dim3(w->nch), dim3(G10_BLOCK), 0, s, tl, w->ctl);
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
  out->score_launches = launches; out->score_cands_streamed = launches * (u64)n_act;
  out->score_ms = score_ms; out->plan_ms = ms;
  return G10_OK;
}
