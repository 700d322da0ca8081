// Smart tensor eviction on the device (G10, Section 4.3, Algorithm 1).
//
// Algorithm 1 ranks every inactive period again after every eviction.  Two
// facts make most of that work unnecessary without changing any decision:
//   * memory pressure only falls and channel reservations only grow, so for a
//     fixed (period, destination) the benefit never rises and a transfer that
//     no longer fits never fits again.  U(c) = the larger of the two
//     destinations' benefits (0 for a destination that cannot carry the
//     transfer) therefore only falls, and is an upper bound on the benefit
//     B(c) of the policy's destination at every later pass;
//   * only the maximum of the ranking is used.
// So the candidates are scored once in one streaming pass over the whole
// list (k_score_full, HBM-bound), sorted by that score into tiles of 256, and
// each tile keeps the largest U seen at its last evaluation.  A ranking pass
// re-scores only the tiles whose bound reaches the best benefit found so far;
// every tile left out holds no candidate that could win or tie.
//
// The greedy loop itself is a serial chain of small dependent steps (rank,
// decide, range updates, prefix rebuild), bound by latency, not bandwidth.  It
// runs in ONE persistent workgroup of 1024 threads (k_loop): no grid barrier
// and no kernel boundary per pass, the level-1 state in LDS, the slot arrays
// in L2.  Range updates over a period are chunked: whole chunks take a lazy
// add in LDS (pressure, host occupancy), only chunks cut by the period ends,
// chunks holding the transfer windows and chunks in which a slot drops under
// the capacity are rewritten slot by slot, one wavefront per chunk.
//
// State (u64 unless noted, K = kernel slots, chunk = CH slots, nch chunks):
//   P[K], lazyP[nch]      pressure of slot j = P[j] - lazyP[chunk(j)]
//   minOver[nch]          smallest pressure above the capacity in the chunk
//   fre[4][K]             unreserved channel time per slot; channel =
//                         2 * direction + destination (0 flash-out, 1 host-out,
//                         2 flash-in, 3 host-in)
//   H[K], lazyH[nch]      host bytes parked in slot j = H[j] + lazyH[chunk(j)]
//   hmax[nch]             maximum of that over the chunk
//   px[K][8]              chunk-local exclusive prefix sums, one 64-byte record
//                         per slot: {FO0, OT, FO1, OT, FI0, OT, FI1, OT} with
//                         OT over-capacity time dur*[pressure > cap], FOd / FId
//                         free out / in channel time of destination d.  The
//                         pairs a candidate needs at one slot are 16-byte
//                         aligned neighbours.
//   tot[5][nch], base[5][nch+1]   chunk totals and their exclusive prefix
//                         (arrays: 0 OT, 1+d FOd, 3+d FId); a prefix up to
//                         slot j is base[chunk(j)] + px[j].
// Cross-iteration periods use doubled slot coordinates j in [0, 2K).

#include "g10_internal.h"

#include <new>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

namespace {

enum { A_OT = 0, A_FO = 1, A_FI = 3, N_ARR = 5, PX = 8 };
enum { J_FO = 0, J_FI = 1, J_P_PART = 2, J_P_FULL = 3, J_H = 4, J_HQ = 5 };

constexpr u32 LB = 1024;               // threads of the loop workgroup
constexpr u32 LW = LB / G10_WAVE;      // its wavefronts
constexpr u32 UNIT = 256;              // candidates scored by four wavefronts at a time
constexpr u32 NCH_MAX = 512;           // chunks (level-1 arrays live in LDS)
constexpr u32 NT_MAX = 8192;           // tiles  (their bounds live in LDS)
constexpr u32 GUESS_SHIFT = 5;         // first threshold of a pass: last benefit * (1 - 2^-5)
constexpr u64 NONE64 = ~0ull;
constexpr u32 NONE32 = 0xffffffffu;

__device__ __forceinline__ u32 w_fo(u32 d) { return 2 * d; }          // word of FOd in a slot record (OT follows)
__device__ __forceinline__ u32 w_fi(u32 d) { return 4 + 2 * d; }      // word of FId (OT follows)

struct Ctl {
  // parameters
  u64 gpu_cap, host_cap, bw_out[2], bw_in[2], max_iter;
  u64 C;                      // all inactive periods (live before any removal)
  // progress
  u32 done, status;
  u64 n_iter, n_mig, n_drop, n_evals;
  u64 overtime_before, overtime_after;
  u32 thr_key, pad0;          // first threshold of the next pass (0: use the largest tile bound)
  // statistics
  u64 units_scored, second_rounds, jobs_run, launches;
};

struct Cands {
  uint4* A;                   // {L1, R, a0, b0}     a > b: no valid window for that destination
  uint4* B;                   // {a1, b1, size lo, size hi}
  uint2* id;                  // {index of the period in the analysis order (the tie-break), tensor}
};

struct Timelines {
  const u64* dur;
  u64* P;
  u64* fre;                   // [4][Kp]
  u64* H;
  u64* px;                    // [K][PX]
  u64* otc;                   // [K] chunk-local prefix of the over-capacity time before any eviction
  u32 K, Kp, nch, spt, shift_ch;   // chunk = 256 * spt = 1 << shift_ch slots
};

// ---------------------------------------------------------------------------
// 128-bit helpers and the 32-bit order-preserving upper key
// ---------------------------------------------------------------------------
__device__ __forceinline__ bool gt128(u64 ahi, u64 alo, u64 bhi, u64 blo) { return ahi != bhi ? ahi > bhi : alo > blo; }

// Monotone non-decreasing map of a 128-bit value to 31 bits that rounds up:
// x <= y  =>  key(x) <= key(y), and key(x) < key(y)  =>  x < y.  Values below
// 2^24 map to themselves; above, 24 significant bits (rounded up) and a shift.
__device__ __forceinline__ u32 upkey(u64 hi, u64 lo) {
  if (hi == 0 && lo < (1ull << 24)) return (u32)lo;
  const int n = hi ? 128 - __clzll((long long)hi) : 64 - __clzll((long long)lo);
  int sh = n - 24;                                   // >= 1
  u64 m;
  bool sticky;
  if (sh >= 64) {
    const int r = sh - 64;
    m = hi >> r;
    sticky = lo != 0 || (r && (hi & ((1ull << r) - 1ull)) != 0);
  } else {
    m = (lo >> sh) | (hi ? hi << (64 - sh) : 0ull);
    sticky = (lo & ((1ull << sh) - 1ull)) != 0;
  }
  m += sticky ? 1u : 0u;
  if (m == (1ull << 24)) { m = 1ull << 23; sh += 1; }
  return ((u32)sh << 24) + (u32)m;
}

__device__ __forceinline__ bool carries(u64 free_ns, u64 bw, u64 bytes_x1000) {
  // free_ns >= ceil(bytes_x1000 / bw)  <=>  free_ns * bw >= bytes_x1000
  return __umul64hi(free_ns, bw) != 0 || free_ns * bw >= bytes_x1000;
}

__device__ __forceinline__ u64 ceil_div_x1000(u64 s, u64 bw) {
  const u64 x = s * 1000ull;              // validated: no overflow
  return x / bw + (x % bw != 0);
}

// ---------------------------------------------------------------------------
// candidate preparation: transfer times and absent windows per destination
// ---------------------------------------------------------------------------
__device__ __forceinline__ u64 start2(const u64* start, u32 K, u64 T, u32 j) { return j < K ? start[j] : start[j - K] + T; }

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

// candidates with at least one valid window, packed in the analysis order
__global__ __launch_bounds__(G10_BLOCK) void k_pack(const u32* __restrict__ per_t, const u32* __restrict__ per_L,
                                                   const u32* __restrict__ per_R, const u64* __restrict__ size,
                                                   const uint4* __restrict__ win, const u32* __restrict__ pos, u32 C,
                                                   Cands out) {
  const u32 c = blockIdx.x * G10_BLOCK + threadIdx.x;
  if (c >= C || pos[c + 1] == pos[c]) return;
  const u32 o = pos[c], t = per_t[c];
  const uint4 w = win[c];
  const u64 s = size[t];
  out.A[o] = make_uint4(per_L[c] + 1, per_R[c], w.x, w.y);
  out.B[o] = make_uint4(w.z, w.w, (u32)s, (u32)(s >> 32));
  out.id[o] = make_uint2(c, t);
}

// ---------------------------------------------------------------------------
// timelines before any eviction: slot arrays, chunk-local prefixes, chunk totals
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(G10_BLOCK) void k_init_timelines(Timelines tl, const u64* __restrict__ pressure0, const Ctl* ctl,
                                                             u64* __restrict__ g_tot, u64* __restrict__ g_lazyP,
                                                             u64* __restrict__ g_minOver, u64* __restrict__ g_lazyH,
                                                             u64* __restrict__ g_hmax) {
  __shared__ u64 tmp[2 * G10_WAVES];
  __shared__ u64 mins[G10_WAVES];
  const u64 cap = ctl->gpu_cap;
  const u32 chunk = blockIdx.x, ch = G10_BLOCK * tl.spt, K = tl.K;
  const u32 j0 = chunk * ch + threadIdx.x * tl.spt;
  u64 v[2] = {0, 0};
  u64 mn = NONE64;
  for (u32 i = 0; i < tl.spt; ++i) {
    const u32 j = j0 + i;
    if (j >= K) break;
    const u64 d = tl.dur[j], p = pressure0[j];
    v[0] += d;
    if (p > cap) { v[1] += d; mn = p < mn ? p : mn; }
    tl.P[j] = p;
    tl.H[j] = 0;
    for (u32 c = 0; c < 4; ++c) tl.fre[(u64)c * tl.Kp + j] = d;
  }
  u64 total[2];
  block_scan_excl_n<2>(v, tmp, total);
  u64 run_d = v[0], run_o = v[1];
  for (u32 i = 0; i < tl.spt; ++i) {
    const u32 j = j0 + i;
    if (j >= K) break;
    u64* rec = tl.px + (u64)j * PX;
    rec[0] = run_d; rec[2] = run_d; rec[4] = run_d; rec[6] = run_d;
    rec[1] = run_o; rec[3] = run_o; rec[5] = run_o; rec[7] = run_o;
    tl.otc[j] = run_o;
    const u64 d = tl.dur[j];
    run_d += d;
    if (pressure0[j] > cap) run_o += d;
  }
  // smallest pressure above the capacity
  u64 m = mn;
#pragma unroll
  for (int o = G10_WAVE / 2; o > 0; o >>= 1) { const u64 w = __shfl_xor(m, o, G10_WAVE); m = w < m ? w : m; }
  if (lane_id() == 0) mins[wave_id()] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (u32 w = 1; w < G10_WAVES; ++w) m = mins[w] < m ? mins[w] : m;
    g_tot[(u64)A_OT * tl.nch + chunk] = total[1];
    for (u32 c = 0; c < 4; ++c) g_tot[(u64)(A_FO + c) * tl.nch + chunk] = total[0];
    g_lazyP[chunk] = 0; g_minOver[chunk] = m; g_lazyH[chunk] = 0; g_hmax[chunk] = 0;
  }
}

// level 1 of the over-capacity time before any eviction, for the full scoring
// pass; also the "fits already" test
__global__ __launch_bounds__(LB) void k_level1_init(const u64* __restrict__ g_tot, u32 nch, u64* __restrict__ base0, Ctl* ctl) {
  __shared__ u64 scr[LW];
  const u32 tid = threadIdx.x;
  const u64 v = tid < nch ? g_tot[(u64)A_OT * nch + tid] : 0ull;
  const u64 inc = wave_scan_incl(v);
  if (lane_id() == G10_WAVE - 1) scr[wave_id()] = inc;
  __syncthreads();
  u64 b = 0, t = 0;
  for (u32 w = 0; w < LW; ++w) { const u64 x = scr[w]; if (w < wave_id()) b += x; t += x; }
  if (tid < nch) base0[tid] = b + inc - v;
  if (tid == 0) {
    base0[nch] = t;
    ctl->overtime_before = t;
    ctl->overtime_after = t;
    if (t == 0) { ctl->done = 1; ctl->status = G10_FITS; }
  }
}

// ---------------------------------------------------------------------------
// the streaming scoring pass over every candidate, before any eviction: all
// channels are still free, so every valid window can be carried and
// U = size * (largest over-capacity time of the valid windows).  Reads the 32
// bytes of the candidate, gathers four prefix words from a table that fits
// L2, writes the 4-byte key and the sort key.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(G10_BLOCK) void k_score_full(Cands cd, u32 n, const u64* __restrict__ otc,
                                                         const u64* __restrict__ base0, u32 K, u32 nch, u32 shift_ch,
                                                         u32 posbits, u32* __restrict__ key32, u64* __restrict__ sortkeys) {
  extern __shared__ u64 lb[];                  // [nch + 1]
  for (u32 i = threadIdx.x; i <= nch; i += G10_BLOCK) lb[i] = base0[i];
  __syncthreads();
  const u32 p = blockIdx.x * G10_BLOCK + threadIdx.x;
  if (p >= n) return;
  const uint4 A = cd.A[p], B = cd.B[p];
  const u64 s = ((u64)B.w << 32) | B.z;
  const u64 total = lb[nch];
  auto ot2 = [&](u32 j) -> u64 {               // over-capacity time before doubled slot j
    const bool second = j >= K;
    const u32 jj = second ? j - K : j;
    return (second ? total : 0ull) + lb[jj >> shift_ch] + otc[jj];
  };
  u64 ot = 0;
  if (A.z <= A.w) ot = ot2(A.w + 1) - ot2(A.z);
  if (B.x <= B.y) { const u64 o1 = ot2(B.y + 1) - ot2(B.x); ot = o1 > ot ? o1 : ot; }
  const u32 k = upkey(__umul64hi(s, ot), s * ot);
  key32[p] = k;
  sortkeys[p] = ((u64)(0x7fffffu - (k >> 8)) << posbits) | p;      // descending score, then analysis order
}

// candidates into score order; the tile bound is the largest key of its members
__global__ __launch_bounds__(G10_BLOCK) void k_tile_gather(const u64* __restrict__ sorted, u32 n, u32 n_pad, u32 posbits,
                                                          Cands src, const u32* __restrict__ key32, Cands dst,
                                                          u32 tile_shift, u32* __restrict__ tkeys) {
  const u32 r = blockIdx.x * G10_BLOCK + threadIdx.x;
  if (r >= n_pad) return;
  u32 k = 0;
  if (r < n) {
    const u32 p = (u32)(sorted[r] & ((1ull << posbits) - 1ull));
    dst.A[r] = src.A[p];
    dst.B[r] = src.B[p];
    dst.id[r] = src.id[p];
    k = key32[p];
  } else {                                       // padding of the last tile: no valid window
    dst.A[r] = make_uint4(0u, 0u, 1u, 0u);
    dst.B[r] = make_uint4(1u, 0u, 0u, 0u);
    dst.id[r] = make_uint2(NONE32, 0u);
  }
  k = wave_max(k);
  if (lane_id() == 0 && k) atomicMax(&tkeys[r >> tile_shift], k);
}

// ---------------------------------------------------------------------------
// the greedy loop
// ---------------------------------------------------------------------------
struct LoopArgs {
  Cands cd;
  u32 n_pad, nt, tshift;      // tile = UNIT << tshift candidates
  Timelines tl;
  u64 *g_tot, *g_lazyP, *g_minOver, *g_lazyH, *g_hmax;
  u32* g_keys;
  Ctl* ctl;
  g10_migration* records;
  g10_dropped* dropped;
  u32 pass_budget;
};

struct Best {
  u64 hi, lo;
  u32 cand;
};

__device__ __forceinline__ bool better(u64 hi, u64 lo, u32 cand, u64 bhi, u64 blo, u32 bcand) {
  if (hi != bhi) return hi > bhi;
  if (lo != blo) return lo > blo;
  return cand < bcand;
}

struct Shared {               // small per-pass state of the loop workgroup
  u64 whi, wlo;               // winner: benefit
  u64 s, tau_o, tau_i, fo_base, fi_end;
  u32 cand, tensor, pos, dest, L1, R, a, b;
  u64 hq;                     // host-capacity query: maximum over the period
  u32 ntl, restmax, njobs, ot_changed;
  u64 wave_hi[LW], wave_lo[LW];
  u32 wave_cand[LW];
  // progress (mirrors Ctl)
  u64 n_iter, n_mig, n_drop, n_evals, units, second, jobs;
  u32 thr_key, status, done, room;
};

// covered slots of chunk c by the doubled range [x, y] (x <= y, y - x < K)
__device__ __forceinline__ u32 cover(u32 c, u32 ch, u32 K, u32 x, u32 y, u32& len) {
  const u32 s0 = c * ch, s1 = (s0 + ch - 1 < K - 1) ? s0 + ch - 1 : K - 1;
  len = s1 - s0 + 1;
  u32 cnt = 0;
  if (x < K) {
    const u32 lo = s0 > x ? s0 : x, hi0 = y < K - 1 ? y : K - 1, hi = s1 < hi0 ? s1 : hi0;
    if (lo <= hi) cnt += hi - lo + 1;
  }
  if (y >= K) {
    const u32 x2 = x >= K ? x - K : 0u, y2 = y - K;
    const u32 lo = s0 > x2 ? s0 : x2, hi = s1 < y2 ? s1 : y2;
    if (lo <= hi) cnt += hi - lo + 1;
  }
  return cnt;
}

// position of plain slot j inside the doubled range [x, y] (y - x < K), or NONE32
__device__ __forceinline__ u32 in_doubled(u32 j, u32 K, u32 x, u32 y) {
  if (j >= x && j <= y) return j;
  const u32 jj = j + K;
  if (jj >= x && jj <= y) return jj;
  return NONE32;
}

__device__ __forceinline__ u64 wave_min64(u64 v) {
#pragma unroll
  for (int o = G10_WAVE / 2; o > 0; o >>= 1) { const u64 w = __shfl_xor(v, o, G10_WAVE); v = w < v ? w : v; }
  return v;
}

__global__ __launch_bounds__(LB) void k_loop(LoopArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  const Timelines tl = a.tl;
  const u32 nch = tl.nch, nb1 = nch + 1, K = tl.K, CH = 1u << tl.shift_ch, nt = a.nt;
  u64* base = (u64*)smem;                               // [5][nch + 1]
  u64* tot = base + (u64)N_ARR * nb1;                   // [5][nch]
  u64* lazyP = tot + (u64)N_ARR * nch;
  u64* minOver = lazyP + nch;
  u64* lazyH = minOver + nch;
  u64* hmax = lazyH + nch;
  u64* scr = hmax + nch;                                // [3 * LW]
  Shared* S = (Shared*)(scr + 3 * LW);
  u32* keys = (u32*)(S + 1);                            // [nt]
  u32* jobs = keys + nt;                                // [4 * nch + 8]
  u32* mark = jobs + 4 * nch + 8;                       // [(nt + 31) / 32]
  unsigned short* tlist = (unsigned short*)(mark + (nt + 31) / 32);   // [nt]

  const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  Ctl* ctl = a.ctl;
  const u64 cap = ctl->gpu_cap, host_cap = ctl->host_cap, max_iter = ctl->max_iter, C = ctl->C;
  const u64 bwo[2] = {ctl->bw_out[0], ctl->bw_out[1]}, bwi[2] = {ctl->bw_in[0], ctl->bw_in[1]};

  // ---- state in ----------------------------------------------------------------------
  for (u32 i = tid; i < N_ARR * nch; i += LB) tot[i] = a.g_tot[i];
  for (u32 i = tid; i < nch; i += LB) { lazyP[i] = a.g_lazyP[i]; minOver[i] = a.g_minOver[i]; lazyH[i] = a.g_lazyH[i]; hmax[i] = a.g_hmax[i]; }
  for (u32 i = tid; i < nt; i += LB) keys[i] = a.g_keys[i];
  for (u32 i = tid; i < (nt + 31) / 32; i += LB) mark[i] = 0;
  if (tid == 0) {
    S->n_iter = ctl->n_iter; S->n_mig = ctl->n_mig; S->n_drop = ctl->n_drop; S->n_evals = ctl->n_evals;
    S->units = 0; S->second = 0; S->jobs = 0;
    S->thr_key = ctl->thr_key; S->status = ctl->status; S->done = ctl->done;
  }
  __syncthreads();

  // exclusive scan of the chunk totals of NA arrays into base
  auto scan_bases = [&](const u32* arrs, u32 na) {
    u64 v[3], inc[3];
    for (u32 q = 0; q < na; ++q) {
      v[q] = tid < nch ? tot[(u64)arrs[q] * nch + tid] : 0ull;
      inc[q] = wave_scan_incl(v[q]);
      if (lane == G10_WAVE - 1) scr[q * LW + wave] = inc[q];
    }
    __syncthreads();
    for (u32 q = 0; q < na; ++q) {
      u64 b = 0, t = 0;
      for (u32 w = 0; w < LW; ++w) { const u64 x = scr[q * LW + w]; if (w < wave) b += x; t += x; }
      if (tid < nch) base[(u64)arrs[q] * nb1 + tid] = b + inc[q] - v[q];
      if (tid == 0) base[(u64)arrs[q] * nb1 + nch] = t;
    }
    __syncthreads();
  };
  { const u32 a3[3] = {0, 1, 2}; scan_bases(a3, 3); const u32 a2[2] = {3, 4}; scan_bases(a2, 2); }

  // full prefix of record word `w` (array arr) before doubled slot j
  auto pref = [&](u32 arr, u32 w, u32 j) -> u64 {
    const bool second = j >= K;
    const u32 jj = second ? j - K : j;
    const u64* b = base + (u64)arr * nb1;
    return (second ? b[nch] : 0ull) + b[jj >> tl.shift_ch] + tl.px[(u64)jj * PX + w];
  };

  // tiles whose bound reaches `thr` and that were not scored in this pass -> tlist;
  // the largest bound among the tiles left out -> restmax
  auto build_list = [&](u32 thr) {
    if (tid == 0) { S->ntl = 0; S->restmax = 0; }
    __syncthreads();
    u32 rm = 0;
    for (u32 t0 = 0; t0 < nt; t0 += LB) {
      const u32 t = t0 + tid;
      const u32 k = t < nt ? keys[t] : 0u;
      const bool marked = t < nt && ((mark[t >> 5] >> (t & 31u)) & 1u);
      const bool sel = k != 0 && k >= thr && !marked;
      if (!sel && !marked && k > rm) rm = k;
      const u64 m = __ballot(sel);
      if (m) {
        u32 off = 0;
        if (lane == 0) off = atomicAdd(&S->ntl, (u32)__popcll(m));
        off = __shfl(off, 0, G10_WAVE);
        if (sel) {
          tlist[off + __popcll(m & ((1ull << lane) - 1ull))] = (unsigned short)t;
          atomicOr(&mark[t >> 5], 1u << (t & 31u));
          keys[t] = 0;                           // rebuilt by the scoring below
        }
      }
    }
    rm = wave_max(rm);
    if (lane == 0 && rm) atomicMax(&S->restmax, rm);
    __syncthreads();
  };

  // this thread's best candidate of the pass, with what a commit needs
  u64 m_hi = 0, m_lo = 0, m_s = 0, m_fo = 0, m_fi = 0;
  u32 m_cand = NONE32, m_tensor = 0, m_pos = 0, m_dest = 0, m_L1 = 0, m_R = 0, m_a = 0, m_b = 0;

  auto score_list = [&]() {
    const u32 nunits = S->ntl << a.tshift;
    for (u32 u = tid >> 8; u < nunits; u += LB / UNIT) {
      const u32 t = tlist[u >> a.tshift], sub = u & ((1u << a.tshift) - 1u);
      const u32 p = (((t << a.tshift) + sub) << 8) + (tid & 255u);
      const uint4 A = a.cd.A[p], B = a.cd.B[p];
      const uint2 id = a.cd.id[p];
      const u64 s = ((u64)B.w << 32) | B.z, x1000 = s * 1000ull;
      const u32 L1 = A.x, R = A.y;
      u64 uhi = 0, ulo = 0;
      bool have = false;                        // the policy's destination found
#pragma unroll
      for (u32 d = 0; d < 2; ++d) {
        const u32 wa = d ? B.x : A.z, wb = d ? B.y : A.w;
        if (wa > wb) continue;
        const u64 fo_L = pref(A_FO + d, w_fo(d), L1), fo_a = pref(A_FO + d, w_fo(d), wa);
        const u64 fi_R = pref(A_FI + d, w_fi(d), R), fi_b = pref(A_FI + d, w_fi(d), wb + 1);
        const u64 ot = pref(A_OT, w_fi(d) + 1, wb + 1) - pref(A_OT, w_fo(d) + 1, wa);
        if (!carries(fo_a - fo_L, bwo[d], x1000) || !carries(fi_R - fi_b, bwi[d], x1000)) continue;
        const u64 hi = __umul64hi(s, ot), lo = s * ot;
        if (gt128(hi, lo, uhi, ulo)) { uhi = hi; ulo = lo; }
        if (!have) {                            // flash first; host only if flash cannot take it
          have = true;
          if ((hi | lo) != 0 && better(hi, lo, id.x, m_hi, m_lo, m_cand)) {
            m_hi = hi; m_lo = lo; m_cand = id.x; m_tensor = id.y; m_pos = p; m_dest = d;
            m_L1 = L1; m_R = R; m_a = wa; m_b = wb; m_s = s; m_fo = fo_L; m_fi = fi_R;
          }
        }
      }
      const u32 k = wave_max(upkey(uhi, ulo));
      if (lane == 0 && k) atomicMax(&keys[t], k);
    }
    if (tid == 0) S->units += nunits;
  };

  // block-wide arg-max of the threads' best; the owner publishes the winner
  auto reduce_best = [&]() {
    Best x; x.hi = m_hi; x.lo = m_lo; x.cand = m_cand;
#pragma unroll
    for (int o = G10_WAVE / 2; o > 0; o >>= 1) {
      const u64 yh = __shfl_xor(x.hi, o, G10_WAVE), yl = __shfl_xor(x.lo, o, G10_WAVE);
      const u32 yc = __shfl_xor(x.cand, o, G10_WAVE);
      if (better(yh, yl, yc, x.hi, x.lo, x.cand)) { x.hi = yh; x.lo = yl; x.cand = yc; }
    }
    if (lane == 0) { S->wave_hi[wave] = x.hi; S->wave_lo[wave] = x.lo; S->wave_cand[wave] = x.cand; }
    __syncthreads();
    x.hi = S->wave_hi[0]; x.lo = S->wave_lo[0]; x.cand = S->wave_cand[0];
    for (u32 w = 1; w < LW; ++w)
      if (better(S->wave_hi[w], S->wave_lo[w], S->wave_cand[w], x.hi, x.lo, x.cand)) { x.hi = S->wave_hi[w]; x.lo = S->wave_lo[w]; x.cand = S->wave_cand[w]; }
    if ((x.hi | x.lo) != 0 && m_cand == x.cand && m_hi == x.hi && m_lo == x.lo) {
      S->whi = m_hi; S->wlo = m_lo; S->cand = m_cand; S->tensor = m_tensor; S->pos = m_pos; S->dest = m_dest;
      S->L1 = m_L1; S->R = m_R; S->a = m_a; S->b = m_b; S->s = m_s; S->fo_base = m_fo; S->fi_end = m_fi;
      S->tau_o = ceil_div_x1000(m_s, m_dest ? bwo[1] : bwo[0]); S->tau_i = ceil_div_x1000(m_s, m_dest ? bwi[1] : bwi[0]);
    }
    if (tid == 0 && (x.hi | x.lo) == 0) { S->whi = 0; S->wlo = 0; }
    __syncthreads();
  };

  // ---- chunk jobs: one wavefront rewrites one chunk of one array ------------------------
  auto run_jobs = [&]() {
    const u32 nj = S->njobs;
    const u32 d = S->dest, L1 = S->L1, R = S->R, wa = S->a, wb = S->b;
    const u64 s = S->s, tau_o = S->tau_o, tau_i = S->tau_i, fo_base = S->fo_base, fi_end = S->fi_end;
    for (u32 jb = wave; jb < nj; jb += LW) {
      const u32 type = jobs[jb] >> 16, c = jobs[jb] & 0xffffu;
      const u32 s0 = c * CH;
      if (type == J_FO || type == J_FI) {
        const bool out = type == J_FO;
        const u32 arr = (out ? A_FO : A_FI) + d, w = out ? w_fo(d) : w_fi(d);
        u64* fr = tl.fre + (u64)((out ? 0u : 2u) + d) * tl.Kp;
        const u64 bc = base[(u64)arr * nb1 + c], ball = base[(u64)arr * nb1 + nch];
        const u32 x = out ? L1 : wb + 1, y = out ? wa - 1 : R - 1;
        u64 carry = 0;
        for (u32 st = 0; st < tl.spt; ++st) {
          const u32 j0 = s0 + st * 256u + lane * 4u;
          u64 f[4];
          u64 lsum = 0;
#pragma unroll
          for (u32 i = 0; i < 4; ++i) {
            const u32 j = j0 + i;
            f[i] = 0;
            if (j < K) {
              f[i] = fr[j];
              const u32 jj = in_doubled(j, K, x, y);
              if (jj != NONE32) {
                const u64 before_slot = (jj >= K ? ball : 0ull) + bc + tl.px[(u64)j * PX + w];   // free time before slot jj
                u64 take;
                if (out) {                         // eviction: earliest free time of the window first
                  const u64 before = before_slot - fo_base;
                  const u64 used = before < tau_o ? before : tau_o;
                  take = f[i] < tau_o - used ? f[i] : tau_o - used;
                } else {                           // prefetch: latest free time first
                  const u64 after = fi_end - (before_slot + f[i]);
                  const u64 used = after < tau_i ? after : tau_i;
                  take = f[i] < tau_i - used ? f[i] : tau_i - used;
                }
                if (take) { f[i] -= take; fr[j] = f[i]; }
              }
            }
            lsum += f[i];
          }
          const u64 inc = wave_scan_incl(lsum);
          u64 run = carry + inc - lsum;
#pragma unroll
          for (u32 i = 0; i < 4; ++i) {
            const u32 j = j0 + i;
            if (j < K) { tl.px[(u64)j * PX + w] = run; run += f[i]; }
          }
          carry += __shfl(inc, G10_WAVE - 1, G10_WAVE);
        }
        if (lane == 0) tot[(u64)arr * nch + c] = carry;
      } else if (type == J_P_PART || type == J_P_FULL) {
        const u64 lz = lazyP[c];
        u64 carry = 0, mn = NONE64;
        for (u32 st = 0; st < tl.spt; ++st) {
          const u32 j0 = s0 + st * 256u + lane * 4u;
          u64 v[4];
          u64 lsum = 0;
#pragma unroll
          for (u32 i = 0; i < 4; ++i) {
            const u32 j = j0 + i;
            v[i] = 0;
            if (j < K) {
              u64 p = tl.P[j];
              if (type == J_P_PART && in_doubled(j, K, wa, wb) != NONE32) { p -= s; tl.P[j] = p; }
              const u64 act = p - lz;
              if (act > cap) { v[i] = tl.dur[j]; mn = act < mn ? act : mn; }
            }
            lsum += v[i];
          }
          const u64 inc = wave_scan_incl(lsum);
          u64 run = carry + inc - lsum;
#pragma unroll
          for (u32 i = 0; i < 4; ++i) {
            const u32 j = j0 + i;
            if (j < K) {
              u64* rec = tl.px + (u64)j * PX;
              rec[1] = run; rec[3] = run; rec[5] = run; rec[7] = run;
              run += v[i];
            }
          }
          carry += __shfl(inc, G10_WAVE - 1, G10_WAVE);
        }
        mn = wave_min64(mn);
        if (lane == 0) { tot[(u64)A_OT * nch + c] = carry; minOver[c] = mn; S->ot_changed = 1; }
      } else {                                     // J_H: add the tensor; J_HQ: only ask for the maximum
        const u64 lz = lazyH[c];
        u64 m_all = 0, m_cov = 0;
        for (u32 st = 0; st < tl.spt; ++st) {
          const u32 j0 = s0 + st * 256u + lane * 4u;
#pragma unroll
          for (u32 i = 0; i < 4; ++i) {
            const u32 j = j0 + i;
            if (j < K) {
              u64 h = tl.H[j];
              const bool cov = in_doubled(j, K, L1, R - 1) != NONE32;
              if (type == J_H && cov) { h += s; tl.H[j] = h; }
              const u64 act = h + lz;
              m_all = act > m_all ? act : m_all;
              if (cov) m_cov = act > m_cov ? act : m_cov;
            }
          }
        }
        if (type == J_H) { m_all = wave_max(m_all); if (lane == 0) hmax[c] = m_all; }
        else { m_cov = wave_max(m_cov); if (lane == 0) atomicMax((unsigned long long*)&S->hq, (unsigned long long)m_cov); }
      }
    }
    if (tid == 0) S->jobs += nj;
  };

  // ---- passes ------------------------------------------------------------------------
  u32 passes = 0;
  while (true) {
    if (S->done) break;
    if (base[(u64)A_OT * nb1 + nch] == 0) { if (tid == 0) { S->done = 1; S->status = G10_FITS; } break; }
    if (max_iter && S->n_iter >= max_iter) { if (tid == 0) { S->done = 1; S->status = G10_TRUNCATED; } break; }
    if (passes >= a.pass_budget) break;
    ++passes;
    m_hi = 0; m_lo = 0; m_cand = NONE32;

    // rank: tiles that can hold the winner, first against a guess, then against the best found
    u32 thr = S->thr_key;
    __syncthreads();                               // everyone has read the loop conditions and thr
    build_list(thr ? thr : 1u);
    if (S->ntl == 0 && S->restmax != 0) {          // the guess was too high: start from the largest bound
      thr = S->restmax;
      __syncthreads();
      build_list(thr);
    }
    const u32 n1 = S->ntl;
    score_list();
    reduce_best();
    {
      const u32 kb = upkey(S->whi, S->wlo);
      const u32 need = kb ? kb : 1u;
      if (S->restmax >= need) {                    // a tile left out may hold an equal or better one
        __syncthreads();
        build_list(need);
        if (tid == 0) S->second += 1;
        score_list();
        reduce_best();
      }
    }
    // forget which tiles were scored in this pass
    for (u32 i = tid; i < (nt + 31) / 32; i += LB) mark[i] = 0;
    (void)n1;

    const bool none = (S->whi | S->wlo) == 0;
    if (tid == 0) { S->n_iter += 1; S->n_evals += C - S->n_mig - S->n_drop; S->hq = 0; S->njobs = 0; S->ot_changed = 0; }
    __syncthreads();
    if (none) { if (tid == 0) { S->done = 1; S->status = G10_RESIDUAL; } break; }

    const u32 d = S->dest, L1 = S->L1, R = S->R, wa = S->a, wb = S->b;
    const u64 s = S->s;
    // host memory must hold the tensor during the whole period
    bool room = true;
    if (d == G10_HOST) {
      if (tid < nch) {
        u32 len;
        const u32 cv = cover(tid, CH, K, L1, R - 1, len);
        if (cv == len) atomicMax((unsigned long long*)&S->hq, (unsigned long long)hmax[tid]);
        else if (cv) jobs[atomicAdd(&S->njobs, 1u)] = ((u32)J_HQ << 16) | tid;
      }
      __syncthreads();
      run_jobs();
      __syncthreads();
      room = s <= host_cap && S->hq <= host_cap - s;
      __syncthreads();
      if (tid == 0) S->njobs = 0;
    }
    if (tid == 0) {
      const u32 p = S->pos;
      a.cd.A[p] = make_uint4(L1, R, 1u, 0u);       // the candidate leaves the live set
      a.cd.B[p] = make_uint4(1u, 0u, (u32)s, (u32)(s >> 32));
      // first threshold of the next pass: a little under this benefit
      u64 ghi = S->whi, glo = S->wlo;
      const u64 dlo = (glo >> GUESS_SHIFT) | (ghi << (64 - GUESS_SHIFT)), dhi = ghi >> GUESS_SHIFT;
      const u64 nlo = glo - dlo;
      ghi = ghi - dhi - (glo < dlo ? 1ull : 0ull);
      S->thr_key = upkey(ghi, nlo);
      if (!room) {
        g10_dropped dr; dr.iteration = S->n_iter - 1; dr.cand = S->cand; dr.reserved = 0;
        a.dropped[S->n_drop] = dr;
        S->n_drop += 1;
      } else {
        g10_migration mg;
        mg.cand = S->cand; mg.tensor = S->tensor;
        mg.evict_after = L1 - 1; mg.absent_first = wa % K; mg.absent_last = wb % K; mg.next_use = R % K;
        mg.dest = d; mg.wraps = R >= K ? 1u : 0u;
        mg.size_bytes = s; mg.t_out_ns = S->tau_o; mg.t_in_ns = S->tau_i; mg.benefit_lo = S->wlo; mg.benefit_hi = S->whi;
        a.records[S->n_mig] = mg;
        S->n_mig += 1;
      }
    }
    __syncthreads();
    if (!room) continue;

    // commit: which chunks change, and how
    if (tid < nch) {
      const u32 c = tid;
      u32 len;
      if (cover(c, CH, K, L1, wa - 1, len)) jobs[atomicAdd(&S->njobs, 1u)] = ((u32)J_FO << 16) | c;
      if (cover(c, CH, K, wb + 1, R - 1, len)) jobs[atomicAdd(&S->njobs, 1u)] = ((u32)J_FI << 16) | c;
      u32 cv = cover(c, CH, K, wa, wb, len);
      if (cv == len) {                             // the whole chunk loses the tensor
        lazyP[c] += s;
        u64 mo = minOver[c];
        if (mo != NONE64) {
          mo -= s;
          minOver[c] = mo;
          if (mo <= cap) jobs[atomicAdd(&S->njobs, 1u)] = ((u32)J_P_FULL << 16) | c;   // a slot drops under the capacity
        }
      } else if (cv) {
        jobs[atomicAdd(&S->njobs, 1u)] = ((u32)J_P_PART << 16) | c;
      }
      if (d == G10_HOST) {
        cv = cover(c, CH, K, L1, R - 1, len);
        if (cv == len) { lazyH[c] += s; hmax[c] += s; }
        else if (cv) jobs[atomicAdd(&S->njobs, 1u)] = ((u32)J_H << 16) | c;
      }
    }
    __syncthreads();
    run_jobs();
    __syncthreads();
    if (S->ot_changed) { const u32 a3[3] = {A_OT, A_FO + d, A_FI + d}; scan_bases(a3, 3); }
    else { const u32 a2[2] = {A_FO + d, A_FI + d}; scan_bases(a2, 2); }
  }
  __syncthreads();

  // ---- state out ---------------------------------------------------------------------
  for (u32 i = tid; i < N_ARR * nch; i += LB) a.g_tot[i] = tot[i];
  for (u32 i = tid; i < nch; i += LB) { a.g_lazyP[i] = lazyP[i]; a.g_minOver[i] = minOver[i]; a.g_lazyH[i] = lazyH[i]; a.g_hmax[i] = hmax[i]; }
  for (u32 i = tid; i < nt; i += LB) a.g_keys[i] = keys[i];
  if (tid == 0) {
    ctl->n_iter = S->n_iter; ctl->n_mig = S->n_mig; ctl->n_drop = S->n_drop; ctl->n_evals = S->n_evals;
    ctl->thr_key = S->thr_key; ctl->status = S->status; ctl->done = S->done;
    ctl->overtime_after = base[(u64)A_OT * nb1 + nch];
    ctl->units_scored += S->units; ctl->second_rounds += S->second; ctl->jobs_run += S->jobs; ctl->launches += 1;
  }
}

// pressure after the plan (lazy adds applied) and its maximum
__global__ __launch_bounds__(G10_BLOCK) void k_finish(Timelines tl, const u64* __restrict__ g_lazyP, u64* __restrict__ out,
                                                     u64* peak) {
  __shared__ u64 tmp[G10_WAVES + 1];
  u64 m = 0;
  for (u32 j = blockIdx.x * G10_BLOCK + threadIdx.x; j < tl.K; j += gridDim.x * G10_BLOCK) {
    const u64 p = tl.P[j] - g_lazyP[j >> tl.shift_ch];
    out[j] = p;
    m = p > m ? p : m;
  }
  m = block_max(m, tmp);
  if (threadIdx.x == 0) atomicMax((unsigned long long*)peak, (unsigned long long)m);
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
  u32 K = 0, Kp = 0, nch = 0, spt = 1, shift_ch = 8;
  u64 C = 0, cap_pad = 0;
  uint4* win = nullptr;
  u32 *keep = nullptr, *scratch32 = nullptr, *hist = nullptr, *key32 = nullptr, *tkeys = nullptr;
  u64 *keys = nullptr, *keys_alt = nullptr;
  Cands cd[2] = {};
  u64 *P = nullptr, *fre = nullptr, *H = nullptr, *px = nullptr, *otc = nullptr, *base0 = nullptr, *g_tot = nullptr,
      *g_lazyP = nullptr, *g_minOver = nullptr, *g_lazyH = nullptr, *g_hmax = nullptr, *pressure_after = nullptr,
      *peak_after = nullptr;
  Ctl* ctl = nullptr;
  g10_migration* records = nullptr;
  g10_dropped* dropped = nullptr;
  // host copies handed out through g10_result
  g10_migration* h_records = nullptr;
  g10_dropped* h_dropped = nullptr;
  u64* h_pressure = nullptr;
  hipEvent_t ev[6] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
  bool lds_opt_in = false;
};

void plan_work_free(PlanWork* w) {
  if (!w) return;
  void* dev[] = {w->win, w->keep, w->scratch32, w->hist, w->key32, w->tkeys, w->keys, w->keys_alt, w->cd[0].A, w->cd[0].B,
                 w->cd[0].id, w->cd[1].A, w->cd[1].B, w->cd[1].id, w->P, w->fre, w->H, w->px, w->otc, w->base0, w->g_tot,
                 w->g_lazyP, w->g_minOver, w->g_lazyH, w->g_hmax, w->pressure_after, w->peak_after, w->ctl, w->records,
                 w->dropped};
  for (void* p : dev) if (p) (void)hipFree(p);
  free(w->h_records);
  free(w->h_dropped);
  free(w->h_pressure);
  for (hipEvent_t e : w->ev) if (e) (void)hipEventDestroy(e);
  delete w;
}

static const u32 PASS_BUDGET = 4096;             // ranking passes per launch of the loop kernel

static u32 tile_shift_for(u64 n) {               // smallest tile (256 << shift) with at most NT_MAX tiles
  u32 sh = 0;
  while ((((n + UNIT - 1) / UNIT) + (1ull << sh) - 1) >> sh > NT_MAX) ++sh;
  return sh;
}

static int work_alloc(g10_plan_s* h) {
  PlanWork* w = new (std::nothrow) PlanWork();
  if (!w) return G10_ENOMEM;
  h->work = w;
  const u32 K = h->K;
  const u64 C = h->n_periods;
  w->K = K; w->C = C;
  w->Kp = (K + 3u) & ~3u;
  w->spt = 1; w->shift_ch = 8;
  while ((u64)G10_BLOCK * w->spt * NCH_MAX < K) { w->spt *= 2; w->shift_ch += 1; }
  const u32 ch = G10_BLOCK * w->spt;
  w->nch = (K + ch - 1) / ch;
  const u32 tsh = tile_shift_for(C);
  w->cap_pad = ((C + ((u64)UNIT << tsh) - 1) >> (8 + tsh)) << (8 + tsh);
  if (!w->cap_pad) w->cap_pad = UNIT;
  G10_TRY(dalloc(&w->win, C));
  G10_TRY(dalloc(&w->keep, C + 1));
  const u64 he = radix_hist_elems(C);
  G10_TRY(dalloc(&w->hist, he));
  G10_TRY(dalloc(&w->scratch32, scan_scratch_elems(he > C ? he : C)));
  G10_TRY(dalloc(&w->keys, C)); G10_TRY(dalloc(&w->keys_alt, C));
  G10_TRY(dalloc(&w->key32, C));
  G10_TRY(dalloc(&w->tkeys, (u64)NT_MAX));
  for (int i = 0; i < 2; ++i) {
    const u64 n = i ? w->cap_pad : C;
    G10_TRY(dalloc(&w->cd[i].A, n)); G10_TRY(dalloc(&w->cd[i].B, n)); G10_TRY(dalloc(&w->cd[i].id, n));
  }
  G10_TRY(dalloc(&w->P, K)); G10_TRY(dalloc(&w->fre, (u64)4 * w->Kp)); G10_TRY(dalloc(&w->H, K));
  G10_TRY(dalloc(&w->px, (u64)PX * K)); G10_TRY(dalloc(&w->otc, K));
  G10_TRY(dalloc(&w->base0, (u64)w->nch + 1));
  G10_TRY(dalloc(&w->g_tot, (u64)N_ARR * w->nch));
  G10_TRY(dalloc(&w->g_lazyP, w->nch)); G10_TRY(dalloc(&w->g_minOver, w->nch));
  G10_TRY(dalloc(&w->g_lazyH, w->nch)); G10_TRY(dalloc(&w->g_hmax, w->nch));
  G10_TRY(dalloc(&w->pressure_after, K));
  G10_TRY(dalloc(&w->peak_after, 1));
  G10_TRY(dalloc(&w->ctl, 1));
  G10_TRY(dalloc(&w->records, C));
  G10_TRY(dalloc(&w->dropped, C));
  w->h_records = (g10_migration*)malloc((C ? C : 1) * sizeof(g10_migration));
  w->h_dropped = (g10_dropped*)malloc((C ? C : 1) * sizeof(g10_dropped));
  w->h_pressure = (u64*)malloc((u64)K * sizeof(u64));
  if (!w->h_records || !w->h_dropped || !w->h_pressure) return G10_ENOMEM;
  for (hipEvent_t& e : w->ev) G10_HIP(hipEventCreate(&e));
  return G10_OK;
}

static size_t loop_lds_bytes(u32 nch, u32 nt) {
  size_t b = 0;
  b += (size_t)N_ARR * (nch + 1) * 8 + (size_t)N_ARR * nch * 8 + (size_t)4 * nch * 8 + (size_t)3 * LW * 8;
  b += sizeof(Shared);
  b += (size_t)nt * 4 + ((size_t)4 * nch + 8) * 4 + (size_t)((nt + 31) / 32) * 4 + (size_t)nt * 2;
  return (b + 15) & ~(size_t)15;
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

  G10_HIP(hipEventRecord(w->ev[0], s));
  Ctl hc;
  memset(&hc, 0, sizeof hc);
  hc.gpu_cap = p->gpu_cap_bytes; hc.host_cap = p->host_cap_bytes;
  for (int d = 0; d < 2; ++d) { hc.bw_out[d] = p->bw_out_Bpus[d]; hc.bw_in[d] = p->bw_in_Bpus[d]; }
  hc.max_iter = p->max_iterations;
  hc.C = C;
  G10_HIP(hipMemcpyAsync(w->ctl, &hc, sizeof hc, hipMemcpyHostToDevice, s));

  Timelines tl;
  tl.dur = h->dur; tl.P = w->P; tl.fre = w->fre; tl.H = w->H; tl.px = w->px; tl.otc = w->otc;
  tl.K = K; tl.Kp = w->Kp; tl.nch = w->nch; tl.spt = w->spt; tl.shift_ch = w->shift_ch;

  G10_HIP(hipMemsetAsync(w->peak_after, 0, 8, s));
  hipLaunchKernelGGL(k_init_timelines, dim3(w->nch), dim3(G10_BLOCK), 0, s, tl, (const u64*)(h->pressure_buf + 1),
                     (const Ctl*)w->ctl, w->g_tot, w->g_lazyP, w->g_minOver, w->g_lazyH, w->g_hmax);
  hipLaunchKernelGGL(k_level1_init, dim3(1), dim3(LB), 0, s, (const u64*)w->g_tot, w->nch, w->base0, w->ctl);
  G10_HIP(hipGetLastError());

  // candidates: windows per destination; keep those with at least one valid window
  u32 n = 0;
  const u32 gC = (C + G10_BLOCK - 1) / G10_BLOCK;
  if (C) {
    hipLaunchKernelGGL(k_prep, dim3(gC), dim3(G10_BLOCK), 0, s, h->per_t, h->per_L, h->per_R, h->size, h->start, K, h->T, C,
                       (const Ctl*)w->ctl, w->win, w->keep);
    G10_HIP(hipGetLastError());
    G10_TRY(scan_excl_u32(w->keep, w->keep, C, w->scratch32, s));
    G10_HIP(hipMemcpyAsync(&n, w->keep + C, sizeof(u32), hipMemcpyDeviceToHost, s));
  }
  G10_HIP(hipMemcpyAsync(&hc, w->ctl, sizeof hc, hipMemcpyDeviceToHost, s));
  G10_HIP(hipStreamSynchronize(s));
  const u64 overtime_before = hc.overtime_before;

  const u32 tsh = tile_shift_for(n);
  const u32 tile = UNIT << tsh;
  const u32 nt = (u32)(((u64)n + tile - 1) / tile);
  const u32 n_pad = nt * tile;
  float full_ms = 0.f, loop_ms = 0.f;
  bool timed_full = false, timed_loop = false;
  if (!hc.done) {
    if (n) {
      const u32 posbits = bits_for(n - 1);
      const u32 gn = (n + G10_BLOCK - 1) / G10_BLOCK;
      hipLaunchKernelGGL(k_pack, dim3(gC), dim3(G10_BLOCK), 0, s, h->per_t, h->per_L, h->per_R, h->size, (const uint4*)w->win,
                         (const u32*)w->keep, C, w->cd[0]);
      G10_HIP(hipEventRecord(w->ev[2], s));
      hipLaunchKernelGGL(k_score_full, dim3(gn), dim3(G10_BLOCK), (size_t)(w->nch + 1) * 8, s, w->cd[0], n, (const u64*)w->otc,
                         (const u64*)w->base0, K, w->nch, w->shift_ch, posbits, w->key32, w->keys);
      G10_HIP(hipEventRecord(w->ev[3], s));
      timed_full = true;
      G10_HIP(hipGetLastError());
      u64 *keys = w->keys, *alt = w->keys_alt;
      G10_TRY(radix_sort_u64(&keys, &alt, n, posbits + 23, w->hist, w->scratch32, s));
      G10_HIP(hipMemsetAsync(w->tkeys, 0, (u64)NT_MAX * 4, s));
      hipLaunchKernelGGL(k_tile_gather, dim3(n_pad / G10_BLOCK), dim3(G10_BLOCK), 0, s, (const u64*)keys, n, n_pad, posbits,
                         w->cd[0], (const u32*)w->key32, w->cd[1], 8 + tsh, w->tkeys);
      G10_HIP(hipGetLastError());
    }
    LoopArgs la;
    la.cd = w->cd[1]; la.n_pad = n_pad; la.nt = nt; la.tshift = tsh; la.tl = tl;
    la.g_tot = w->g_tot; la.g_lazyP = w->g_lazyP; la.g_minOver = w->g_minOver; la.g_lazyH = w->g_lazyH; la.g_hmax = w->g_hmax;
    la.g_keys = w->tkeys; la.ctl = w->ctl; la.records = w->records; la.dropped = w->dropped; la.pass_budget = PASS_BUDGET;
    const size_t lds = loop_lds_bytes(w->nch, nt);
    if (lds > 64 * 1024 && !w->lds_opt_in) {
      G10_HIP(hipFuncSetAttribute((const void*)k_loop, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
      w->lds_opt_in = true;
    }
    G10_HIP(hipEventRecord(w->ev[4], s));
    const u64 max_launches = (u64)n / PASS_BUDGET + 3;          // every pass removes a candidate or stops
    u64 launches = 0;
    while (!hc.done) {
      if (launches++ > max_launches) return G10_EDEVICE;
      hipLaunchKernelGGL(k_loop, dim3(1), dim3(LB), lds, s, la);
      G10_HIP(hipGetLastError());
      G10_HIP(hipMemcpyAsync(&hc, w->ctl, sizeof hc, hipMemcpyDeviceToHost, s));
      G10_HIP(hipStreamSynchronize(s));
    }
    G10_HIP(hipEventRecord(w->ev[5], s));
    timed_loop = true;
  }

  hipLaunchKernelGGL(k_finish, dim3(K / G10_BLOCK / 4 + 1), dim3(G10_BLOCK), 0, s, tl, (const u64*)w->g_lazyP, w->pressure_after,
                     w->peak_after);
  G10_HIP(hipGetLastError());
  u64 peak_after = 0;
  G10_HIP(hipMemcpyAsync(&peak_after, w->peak_after, 8, hipMemcpyDeviceToHost, s));
  if (hc.n_mig) G10_HIP(hipMemcpyAsync(w->h_records, w->records, hc.n_mig * sizeof(g10_migration), hipMemcpyDeviceToHost, s));
  if (hc.n_drop) G10_HIP(hipMemcpyAsync(w->h_dropped, w->dropped, hc.n_drop * sizeof(g10_dropped), hipMemcpyDeviceToHost, s));
  G10_HIP(hipMemcpyAsync(w->h_pressure, w->pressure_after, (u64)K * 8, hipMemcpyDeviceToHost, s));
  G10_HIP(hipEventRecord(w->ev[1], s));
  G10_HIP(hipStreamSynchronize(s));
  float ms = 0.f;
  G10_HIP(hipEventElapsedTime(&ms, w->ev[0], w->ev[1]));
  if (timed_full) G10_HIP(hipEventElapsedTime(&full_ms, w->ev[2], w->ev[3]));
  if (timed_loop) G10_HIP(hipEventElapsedTime(&loop_ms, w->ev[4], w->ev[5]));

  memset(out, 0, sizeof *out);
  out->status = (int32_t)hc.status;
  out->n_migrations = hc.n_mig; out->n_iterations = hc.n_iter; out->n_dropped = hc.n_drop; out->n_cand_evals = hc.n_evals;
  out->peak_before = h->peak; out->peak_after = peak_after;
  out->overtime_before_ns = overtime_before; out->overtime_after_ns = hc.overtime_after;
  out->migrations = w->h_records; out->dropped = w->h_dropped; out->pressure_after = w->h_pressure;
  out->plan_ms = ms;
  out->score_full_ms = full_ms; out->score_full_cands = n;
  out->loop_ms = loop_ms; out->loop_launches = hc.launches;
  out->loop_cands_scored = hc.units_scored * UNIT; out->loop_second_rounds = hc.second_rounds; out->loop_chunk_jobs = hc.jobs_run;
  return G10_OK;
}
