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

#include <hip/hip_ext.h>
#include <new>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

namespace {

enum { A_OT = 0, A_FO = 1, A_FI = 3, N_ARR = 5, PX = 8 };
enum { J_FO = 0, J_FI = 1, J_P_PART = 2, J_P_FULL = 3, J_H = 4, J_HQ = 5 };

#ifndef G10_LOOP_THREADS
#define G10_LOOP_THREADS 512
#endif
constexpr u32 LB = G10_LOOP_THREADS;   // threads of the loop workgroup (at least NCH_MAX)
constexpr u32 LW = LB / G10_WAVE;      // its wavefronts
constexpr u32 UNIT = 256;              // candidates scored by four wavefronts at a time
constexpr u32 NCH_MAX = 512;           // chunks (level-1 arrays live in LDS)
constexpr u32 NT_MAX = 8192;           // tiles  (their bounds live in LDS)
#ifndef G10_GUESS_SHIFT
#define G10_GUESS_SHIFT 7
#endif
constexpr u32 GUESS_SHIFT = G10_GUESS_SHIFT;   // first threshold of a pass: last benefit * (1 - 2^-shift)
constexpr u64 NONE64 = ~0ull;
constexpr u32 NONE32 = 0xffffffffu;

__device__ __forceinline__ u32 w_fo(u32 d) { return 2 * d; }          // word of FOd in a slot record (OT follows)
__device__ __forceinline__ u32 w_fi(u32 d) { return 4 + 2 * d; }      // word of FId (OT follows)

struct Ctl {
  // parameters
  u64 gpu_cap, host_cap, bw_out[2], bw_in[2], max_iter;
  u64 inv_out[2], inv_in[2];  // floor(2^64 / bandwidth), 0 for bandwidth 1
  u64 C;                      // all inactive periods (live before any removal)
  // progress
  u32 done, status;
  u64 n_iter, n_mig, n_drop, n_evals;
  u64 overtime_before, overtime_after;
  u32 thr_key;                // first threshold of the next pass (0: use the largest tile bound)
  u32 n_live;                 // candidates that could still score at the last re-scoring
  // statistics
  u64 units_scored, second_rounds, jobs_run, launches;
  u64 phase[12];              // wall-clock ticks per phase of the loop (only with G10_PHASE_TIMERS)
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
  u64* otc;                   // [K + 1] over-capacity time before every slot, before any eviction
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
  if (((free_ns | bw) >> 32) == 0) return (u64)(u32)free_ns * (u32)bw >= bytes_x1000;   // the usual case: one 32 x 32 multiply
  return __umul64hi(free_ns, bw) != 0 || free_ns * bw >= bytes_x1000;
}

// ceil(s * 1000 / bw) with the reciprocal inv = floor(2^64 / bw) (bw >= 2; inv = 0 stands for
// bw = 1): the high half of x * inv is the quotient or up to 2 below it.
__device__ __forceinline__ u64 ceil_div_x1000(u64 s, u64 bw, u64 inv) {
  const u64 x = s * 1000ull;              // validated: no overflow
  if (inv == 0) return x;
  u64 q = __umul64hi(x, inv), r = x - q * bw;
  while (r >= bw) { r -= bw; ++q; }
  return q + (r != 0);
}

// ---------------------------------------------------------------------------
// candidate preparation: transfer times and absent windows per destination
// ---------------------------------------------------------------------------
__device__ __forceinline__ u64 start2(const u64* start, u32 K, u64 T, u32 j) { return j < K ? start[j] : start[j - K] + T; }

// (one thread per period, the periods in the order of their start: neighbouring threads search
// neighbouring parts of the start-time array)
__global__ __launch_bounds__(G10_BLOCK) void k_prep(const uint4* __restrict__ per, const u64* __restrict__ size,
                                                   const u64* __restrict__ start, u32 K, u64 T, u32 C, const Ctl* ctl,
                                                   uint4* __restrict__ win, u32* __restrict__ keep) {
  const u32 c = blockIdx.x * G10_BLOCK + threadIdx.x;
  if (c >= C) return;
  const uint4 pd = per[c];                  // {L, R, tensor, period index}
  const u32 L = pd.x, R = pd.y;
  const u64 s = size[c];                    // sizes in the same order
  const u64 t_r = start2(start, K, T, L + 1), t_use = start2(start, K, T, R), len = t_use - t_r;
  u32 any = 0;
  u32 w[4];
#pragma unroll
  for (int d = 0; d < 2; ++d) {
    const u64 tau_o = ceil_div_x1000(s, ctl->bw_out[d], ctl->inv_out[d]), tau_i = ceil_div_x1000(s, ctl->bw_in[d], ctl->inv_in[d]);
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

// candidates with at least one valid window, packed in the order of their start
__global__ __launch_bounds__(G10_BLOCK) void k_pack(const uint4* __restrict__ per, const u64* __restrict__ size,
                                                   const uint4* __restrict__ win, const u32* __restrict__ pos, u32 C,
                                                   Cands out) {
  const u32 c = blockIdx.x * G10_BLOCK + threadIdx.x;
  if (c >= C || pos[c + 1] == pos[c]) return;
  const uint4 pd = per[c];                  // {L, R, tensor, period index}
  const u32 o = pos[c];
  const uint4 w = win[c];
  const u64 s = size[c];                    // sizes in the same order
  out.A[o] = make_uint4(pd.x + 1, pd.y, w.x, w.y);
  out.B[o] = make_uint4(w.z, w.w, (u32)s, (u32)(s >> 32));
  out.id[o] = make_uint2(pd.w, pd.z);
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
  u64 m = wave_min(mn);
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

// over-capacity time before every slot, before any eviction: ot[j] for j in [0, K], chunk-local
// prefix + chunk base, in place
__global__ __launch_bounds__(G10_BLOCK) void k_ot_full(u64* __restrict__ ot, const u64* __restrict__ base0, u32 K, u32 nch,
                                                      u32 shift_ch) {
  const u32 j = blockIdx.x * G10_BLOCK + threadIdx.x;
  if (j < K) ot[j] += base0[j >> shift_ch];
  else if (j == K) ot[K] = base0[nch];
}

// ---------------------------------------------------------------------------
// the streaming scoring pass over every candidate, before any eviction: all
// channels are still free, so every valid window can be carried and
// U = size * (largest over-capacity time of the valid windows).  Reads the 32
// bytes of the candidate, gathers two words per window of a prefix table that
// fits L2 (8 bytes per slot; a window inside the other one is skipped), writes
// the 8-byte sort key: the 31-bit score key rounded up to its top 23 bits
// (descending), then the position.
// ---------------------------------------------------------------------------
__device__ __forceinline__ u64 sort_key(u32 key31, u32 posbits, u32 p) {
  return ((u64)(0x7fffffu - ((key31 + 255u) >> 8)) << posbits) | p;
}
// the bound a sort key stands for: at least the score key it was made from, 0 only for 0
__device__ __forceinline__ u32 bound_of_sort_key(u64 sk, u32 posbits) { return (0x7fffffu - (u32)(sk >> posbits)) << 8; }

__global__ __launch_bounds__(G10_BLOCK) void k_score_full(const uint4* __restrict__ cA, const uint4* __restrict__ cB, u32 n,
                                                         const u64* __restrict__ ot, u32 K, u32 posbits,
                                                         u64* __restrict__ sortkeys) {
  const u32 p = blockIdx.x * G10_BLOCK + threadIdx.x;
  if (p >= n) return;
  const uint4 A = cA[p], B = cB[p];
  const u64 s = ((u64)B.w << 32) | B.z;
  const u64 total = ot[K];
  bool v0 = A.z <= A.w, v1 = B.x <= B.y;
  // the prefix is monotone: a window inside the other one cannot hold more over-capacity time
  if (v0 && v1) {
    if (B.x <= A.z && B.y >= A.w) v0 = false;
    else if (A.z <= B.x && A.w >= B.y) v1 = false;
  }
  u64 t0 = 0, t1 = 0;
  if (v0) {
    const u32 a = A.z, b = A.w + 1;
    const u64 oa = ot[a >= K ? a - K : a], ob = ot[b >= K ? b - K : b];
    t0 = (ob + (b >= K ? total : 0ull)) - (oa + (a >= K ? total : 0ull));
  }
  if (v1) {
    const u32 a = B.x, b = B.y + 1;
    const u64 oa = ot[a >= K ? a - K : a], ob = ot[b >= K ? b - K : b];
    t1 = (ob + (b >= K ? total : 0ull)) - (oa + (a >= K ? total : 0ull));
  }
  const u64 t = t1 > t0 ? t1 : t0;
  sortkeys[p] = sort_key(upkey(__umul64hi(s, t), s * t), posbits, p);
}

// ---------------------------------------------------------------------------
// score of one candidate against the current timelines
// ---------------------------------------------------------------------------
struct Machine { u64 bwo0, bwo1, bwi0, bwi1; };

struct PrefixView {           // slot records in HBM / L2, level 1 in LDS
  const u64* px;
  const u64* base;            // [5][nch + 1]
  u32 K, nch, shift_ch;
};

struct Score {
  u64 h0, l0, h1, l1;         // benefit per destination (0 if it cannot be used now)
  u64 fo_L, fi_R;             // of the policy's destination: free out-channel time before L1, in-channel before R
  bool ok0, ok1;              // the destination's channels can carry the transfer now
  bool strike0, strike1;      // the destination can never count again
};

__device__ __forceinline__ ulonglong2 ld2(const u64* p) { return *reinterpret_cast<const ulonglong2*>(p); }

// Both destinations' record pairs are gathered before anything is used.  A
// destination is struck when its channel cannot carry the transfer any more
// (reservations only grow); host also when no over-capacity time is left in
// its window (pressure only falls), flash then too if host is gone: while
// host could still score, a feasible flash window keeps the policy on flash.
__device__ __forceinline__ Score score_candidate(const PrefixView& pv, const Machine& mc, const uint4 A, const uint4 B) {
  Score r;
  r.h0 = r.l0 = r.h1 = r.l1 = r.fo_L = r.fi_R = 0;
  r.ok0 = r.ok1 = r.strike0 = r.strike1 = false;
  const bool v0 = A.z <= A.w, v1 = B.x <= B.y;
  if (!(v0 || v1)) return r;
  const u32 K = pv.K, nb1 = pv.nch + 1;
  const u64 s = ((u64)B.w << 32) | B.z, x1000 = s * 1000ull;
  const u32 L1 = A.x, R = A.y;
  const bool sL = L1 >= K, sR = R >= K;
  const u32 jL = sL ? L1 - K : L1, jR = sR ? R - K : R;
  const u32 cL = jL >> pv.shift_ch, cR = jR >> pv.shift_ch;
  const u64* bOT = pv.base + (u64)A_OT * nb1;
  bool sa0 = false, sb0 = false, sa1 = false, sb1 = false;
  u32 ca0 = 0, cb0 = 0, ca1 = 0, cb1 = 0;
  ulonglong2 qa0 = {0, 0}, qb0 = {0, 0}, qL0 = {0, 0}, qR0 = {0, 0}, qa1 = {0, 0}, qb1 = {0, 0}, qL1 = {0, 0}, qR1 = {0, 0};
  if (v0) {
    sa0 = A.z >= K; sb0 = A.w + 1 >= K;
    const u32 ja = sa0 ? A.z - K : A.z, jb = sb0 ? A.w + 1 - K : A.w + 1;
    ca0 = ja >> pv.shift_ch; cb0 = jb >> pv.shift_ch;
    qL0 = ld2(pv.px + (u64)jL * PX + 0); qR0 = ld2(pv.px + (u64)jR * PX + 4);      // {FO0, OT} {FI0, OT}
    qa0 = ld2(pv.px + (u64)ja * PX + 0); qb0 = ld2(pv.px + (u64)jb * PX + 4);
  }
  if (v1) {
    sa1 = B.x >= K; sb1 = B.y + 1 >= K;
    const u32 ja = sa1 ? B.x - K : B.x, jb = sb1 ? B.y + 1 - K : B.y + 1;
    ca1 = ja >> pv.shift_ch; cb1 = jb >> pv.shift_ch;
    qL1 = ld2(pv.px + (u64)jL * PX + 2); qR1 = ld2(pv.px + (u64)jR * PX + 6);      // {FO1, OT} {FI1, OT}
    qa1 = ld2(pv.px + (u64)ja * PX + 2); qb1 = ld2(pv.px + (u64)jb * PX + 6);
  }
  u64 fo0_L = 0, fi0_R = 0, fo1_L = 0, fi1_R = 0;
  if (v0) {
    const u64 *bFO = pv.base + (u64)(A_FO + 0) * nb1, *bFI = pv.base + (u64)(A_FI + 0) * nb1;
    const u64 allFO = bFO[pv.nch], allFI = bFI[pv.nch], allOT = bOT[pv.nch];
    fo0_L = (sL ? allFO : 0ull) + bFO[cL] + qL0.x; fi0_R = (sR ? allFI : 0ull) + bFI[cR] + qR0.x;
    const u64 fo_a = (sa0 ? allFO : 0ull) + bFO[ca0] + qa0.x, fi_b = (sb0 ? allFI : 0ull) + bFI[cb0] + qb0.x;
    r.ok0 = carries(fo_a - fo0_L, mc.bwo0, x1000) && carries(fi0_R - fi_b, mc.bwi0, x1000);
    if (r.ok0) {
      const u64 ot = ((sb0 ? allOT : 0ull) + bOT[cb0] + qb0.y) - ((sa0 ? allOT : 0ull) + bOT[ca0] + qa0.y);
      r.h0 = __umul64hi(s, ot); r.l0 = s * ot;
    }
  }
  if (v1) {
    const u64 *bFO = pv.base + (u64)(A_FO + 1) * nb1, *bFI = pv.base + (u64)(A_FI + 1) * nb1;
    const u64 allFO = bFO[pv.nch], allFI = bFI[pv.nch], allOT = bOT[pv.nch];
    fo1_L = (sL ? allFO : 0ull) + bFO[cL] + qL1.x; fi1_R = (sR ? allFI : 0ull) + bFI[cR] + qR1.x;
    const u64 fo_a = (sa1 ? allFO : 0ull) + bFO[ca1] + qa1.x, fi_b = (sb1 ? allFI : 0ull) + bFI[cb1] + qb1.x;
    r.ok1 = carries(fo_a - fo1_L, mc.bwo1, x1000) && carries(fi1_R - fi_b, mc.bwi1, x1000);
    if (r.ok1) {
      const u64 ot = ((sb1 ? allOT : 0ull) + bOT[cb1] + qb1.y) - ((sa1 ? allOT : 0ull) + bOT[ca1] + qa1.y);
      r.h1 = __umul64hi(s, ot); r.l1 = s * ot;
    }
  }
  const bool keep1 = r.ok1 && (r.h1 | r.l1) != 0;
  const bool keep0 = r.ok0 && (keep1 || (r.h0 | r.l0) != 0);
  r.strike0 = v0 && !keep0;
  r.strike1 = v1 && !keep1;
  r.fo_L = r.ok0 ? fo0_L : fo1_L; r.fi_R = r.ok0 ? fi0_R : fi1_R;
  return r;
}

// candidates into score order; the tile bound is the largest bound of its members
__global__ __launch_bounds__(G10_BLOCK) void k_tile_gather(const u64* __restrict__ sorted, u32 n, u32 n_pad, u32 posbits,
                                                          Cands src, Cands dst, u32 tile_shift, u32* __restrict__ tkeys) {
  const u32 r = blockIdx.x * G10_BLOCK + threadIdx.x;
  if (r >= n_pad) return;
  u32 k = 0;
  if (r < n) {
    const u64 sk = sorted[r];
    const u32 p = (u32)(sk & ((1ull << posbits) - 1ull));
    dst.A[r] = src.A[p];
    dst.B[r] = src.B[p];
    dst.id[r] = src.id[p];
    k = bound_of_sort_key(sk, posbits);
  } else {                                       // padding of the last tile: no valid window
    dst.A[r] = make_uint4(0u, 0u, 1u, 0u);
    dst.B[r] = make_uint4(1u, 0u, 0u, 0u);
    dst.id[r] = make_uint2(NONE32, 0u);
  }
  k = wave_max(k);
  if (lane_id() == 0 && k) atomicMax(&tkeys[r >> tile_shift], k);
}

// Re-scores every candidate of the list against the current timelines (all
// workgroups of the chip; used between launches of the loop kernel to put the
// candidates back into score order).  Writes the sort key;
// strikes dead destinations; counts the candidates that can still score.
__global__ __launch_bounds__(G10_BLOCK) void k_rescore(Cands cd, u32 n, const u64* __restrict__ px, const u64* __restrict__ g_base,
                                                      u32 K, u32 nch, u32 shift_ch, const Ctl* ctl, u32 posbits,
                                                      u64* __restrict__ sortkeys, u32* __restrict__ n_live) {
  extern __shared__ u64 lb[];                  // [5][nch + 1]
  for (u32 i = threadIdx.x; i < N_ARR * (nch + 1); i += G10_BLOCK) lb[i] = g_base[i];
  __syncthreads();
  PrefixView pv; pv.px = px; pv.base = lb; pv.K = K; pv.nch = nch; pv.shift_ch = shift_ch;
  Machine mc; mc.bwo0 = ctl->bw_out[0]; mc.bwo1 = ctl->bw_out[1]; mc.bwi0 = ctl->bw_in[0]; mc.bwi1 = ctl->bw_in[1];
  u32 live = 0;
  for (u32 p = blockIdx.x * G10_BLOCK + threadIdx.x; p < n; p += gridDim.x * G10_BLOCK) {
    const uint4 A = cd.A[p], B = cd.B[p];
    const Score r = score_candidate(pv, mc, A, B);
    if (r.strike0) cd.A[p] = make_uint4(A.x, A.y, 1u, 0u);
    if (r.strike1) cd.B[p] = make_uint4(1u, 0u, B.z, B.w);
    const bool one = gt128(r.h1, r.l1, r.h0, r.l0);
    const u32 k = upkey(one ? r.h1 : r.h0, one ? r.l1 : r.l0);
    sortkeys[p] = sort_key(k, posbits, p);
    live += k != 0;
  }
  __shared__ u32 tmp[G10_WAVES + 1];
  live = block_sum(live, tmp);
  if (threadIdx.x == 0 && live) atomicAdd(n_live, live);
}

// ---------------------------------------------------------------------------
// the greedy loop
// ---------------------------------------------------------------------------
struct LoopArgs {
  Cands cd;
  u32 n_pad, nt, tshift;      // tile = UNIT << tshift candidates
  Timelines tl;
  u64 *g_tot, *g_lazyP, *g_minOver, *g_lazyH, *g_hmax, *g_base;
  u32* g_keys;
  Ctl* ctl;
  g10_migration* records;
  uint2* rec_ab;              // absent window [a, b] of every migration in doubled coordinates
  g10_dropped* dropped;
  u32 pass_budget;            // the launch ends after this many passes,
  u64 tick_budget;            // or (if not 0) after this many ticks of the 100 MHz wall clock
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

#ifdef G10_PHASE_TIMERS
#define PHASE(i) do { if (tid == 0) { const u64 now_ = wall_clock64(); S->phase[i] += now_ - S->t_last; S->t_last = now_; } } while (0)
#else
#define PHASE(i) do { } while (0)
#endif

struct Winner {               // what a commit needs of the winning candidate
  u64 hi, lo;                 // benefit
  u64 s, fo_base, fi_end;     // size; free out-channel time before L1; free in-channel time before R
  u32 cand, tensor, pos, dest, L1, R, a, b;
};

struct Shared {               // small per-pass state of the loop workgroup
  Winner win;                 // winner of the pass (hi = lo = 0: none)
  Winner wave_win[LW];        // best of every wavefront
  u64 tau_o, tau_i;
  u64 hq;                     // host-capacity query: maximum over the period
  u32 nl, restL;              // hot list: length; bound of the tiles outside it
  u32 ntl, filt;              // current round: tiles to score; bound of the hot tiles left out
  u32 njobs, ot_changed, stale_hot, pad1;
  // progress (mirrors Ctl)
  u64 n_iter, n_mig, n_drop, n_evals, units, second, jobs;
  u32 thr_key, status, done, stop;
  u64 t_start;
  u64 phase[12], t_last;
};

// covered slots of chunk c by the doubled range [x, y] (x <= y, y - x < K): the chunk's slots
// appear at [s0, s1] and at [s0 + K, s1 + K] in doubled coordinates
__device__ __forceinline__ u32 cover(u32 c, u32 ch, u32 K, u32 x, u32 y, u32& len) {
  const long long s0 = (long long)c * ch, s1 = (s0 + ch - 1 < (long long)K - 1) ? s0 + ch - 1 : (long long)K - 1;
  len = (u32)(s1 - s0 + 1);
  const long long X = x, Y = y;
  long long n1 = (s1 < Y ? s1 : Y) - (s0 > X ? s0 : X) + 1;
  long long n2 = (s1 + K < Y ? s1 + K : Y) - (s0 + K > X ? s0 + K : X) + 1;
  if (n1 < 0) n1 = 0;
  if (n2 < 0) n2 = 0;
  return (u32)(n1 + n2);
}

// first plain slot of [s0, s1] inside the doubled range [x, y] (y - x < K), or NONE32
__device__ __forceinline__ u32 first_covered(u32 s0, u32 s1, u32 K, u32 x, u32 y) {
  u32 first = NONE32;
  if (y >= K) {                                   // the part in the second iteration: plain [max(x, K) - K, y - K]
    const u32 x2 = x >= K ? x - K : 0u, lo = s0 > x2 ? s0 : x2, hi = s1 < y - K ? s1 : y - K;
    if (lo <= hi) first = lo;
  }
  if (x < K) {                                    // the part in the first iteration: plain [x, min(y, K - 1)]
    const u32 y1 = y < K - 1 ? y : K - 1, lo = s0 > x ? s0 : x, hi = s1 < y1 ? s1 : y1;
    if (lo <= hi && lo < first) first = lo;
  }
  return first;
}

// position of plain slot j inside the doubled range [x, y] (y - x < K), or NONE32
__device__ __forceinline__ u32 in_doubled(u32 j, u32 K, u32 x, u32 y) {
  if (j >= x && j <= y) return j;
  const u32 jj = j + K;
  if (jj >= x && jj <= y) return jj;
  return NONE32;
}

// The lane of the wavefront holding the best (benefit, lowest index), or NONE32
// if every benefit is 0.  The 31-bit key decides unless several lanes share the
// largest key (equal or nearly equal benefits: common where a model repeats one
// layer); those are settled by three more reductions: high word, low word, index.
__device__ __forceinline__ u32 wave_best_lane(u64 hi, u64 lo, u32 cand) {
  const u32 k = upkey(hi, lo);
  const u32 kmax = wave_max(k);
  if (kmax == 0) return NONE32;
  u64 m = __ballot(k == kmax);
  if (m & (m - 1)) {
    const bool in1 = k == kmax;
    const u64 hmax = wave_max(in1 ? hi : 0ull);
    const bool in2 = in1 && hi == hmax;
    const u64 lmax = wave_max(in2 ? lo : 0ull);
    const bool in3 = in2 && lo == lmax;
    const u32 cmin = wave_min(in3 ? cand : NONE32);
    m = __ballot(in3 && cand == cmin);
  }
  return (u32)__builtin_ctzll(m);
}

__global__ __launch_bounds__(LB) void k_loop(const LoopArgs* __restrict__ plans) {
  extern __shared__ __align__(16) unsigned char smem[];
  const LoopArgs a = plans[blockIdx.x];        // one workgroup per plan
  const Timelines tl = a.tl;
  const u32 nch = tl.nch, nb1 = nch + 1, K = tl.K, CH = 1u << tl.shift_ch, nt = a.nt, ns = (nt + 63) / 64;
  u64* base = (u64*)smem;                               // [5][nch + 1]
  u64* tot = base + (u64)N_ARR * nb1;                   // [5][nch]
  u64* lazyP = tot + (u64)N_ARR * nch;
  u64* minOver = lazyP + nch;
  u64* lazyH = minOver + nch;
  u64* hmax = lazyH + nch;
  u64* smark = hmax + nch;                              // [ns] tiles of a group of 64 scored in this pass
  u64* scr = smark + ns;                                // [4 * LW]
  Shared* S = (Shared*)(scr + 4 * LW);
  u32* keys = (u32*)(S + 1);                            // [nt]  bound of every tile
  u32* skeys = keys + nt;                               // [ns]  largest bound of every group of 64 tiles
  u32* jobs = skeys + ns;                               // [4 * nch + 8]
  unsigned short* tlist = (unsigned short*)(jobs + 4 * nch + 8);   // [nt]  the hot list
  unsigned short* alist = tlist + nt;                            // [nt]  tiles scored in the current round

  const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  Ctl* ctl = a.ctl;
  const u64 cap = ctl->gpu_cap, host_cap = ctl->host_cap, max_iter = ctl->max_iter, C = ctl->C;
  const u64 bwo0 = ctl->bw_out[0], bwo1 = ctl->bw_out[1], bwi0 = ctl->bw_in[0], bwi1 = ctl->bw_in[1];
  const u64 ivo0 = ctl->inv_out[0], ivo1 = ctl->inv_out[1], ivi0 = ctl->inv_in[0], ivi1 = ctl->inv_in[1];

  // ---- state in ----------------------------------------------------------------------
  for (u32 i = tid; i < N_ARR * nch; i += LB) tot[i] = a.g_tot[i];
  for (u32 i = tid; i < nch; i += LB) { lazyP[i] = a.g_lazyP[i]; minOver[i] = a.g_minOver[i]; lazyH[i] = a.g_lazyH[i]; hmax[i] = a.g_hmax[i]; }
  for (u32 i = tid; i < nt; i += LB) keys[i] = a.g_keys[i];
  for (u32 i = tid; i < ns; i += LB) smark[i] = 0;
  if (tid == 0) {
    S->n_iter = ctl->n_iter; S->n_mig = ctl->n_mig; S->n_drop = ctl->n_drop; S->n_evals = ctl->n_evals;
    S->units = 0; S->second = 0; S->jobs = 0;
    S->thr_key = ctl->thr_key; S->status = ctl->status; S->done = ctl->done;
    S->nl = 0; S->restL = NONE32; S->stale_hot = 0;
    S->stop = 0; S->t_start = wall_clock64();
    S->win.hi = 0; S->win.lo = 0;
    for (u32 i = 0; i < 12; ++i) S->phase[i] = 0;
    S->t_last = wall_clock64();
  }
  __syncthreads();
  for (u32 g = wave; g < ns; g += LW) {                 // group bounds
    const u32 t = g * 64 + lane;
    const u32 k = wave_max(t < nt ? keys[t] : 0u);
    if (lane == 0) skeys[g] = k;
  }

  // exclusive scan of the chunk totals of `na` arrays into base (three barriers)
  auto scan_bases = [&](u32 arr0, u32 arr1, u32 arr2, u32 na) {
    const u32 arrs[3] = {arr0, arr1, arr2};
    const bool act = tid < ((nch + 63u) & ~63u);
    u64 v[3] = {0, 0, 0}, inc[3] = {0, 0, 0};
    if (act) {
      for (u32 q = 0; q < na; ++q) {
        v[q] = tid < nch ? tot[(u64)arrs[q] * nch + tid] : 0ull;
        inc[q] = wave_scan_incl(v[q]);
        if (lane == G10_WAVE - 1) scr[q * LW + wave] = inc[q];
      }
    }
    __syncthreads();
    if (wave == 0) {                                    // the wavefront totals: one small scan
      const u32 nw = (nch + 63) / 64;
      for (u32 q = 0; q < na; ++q) {
        const u64 x = lane < nw ? scr[q * LW + lane] : 0ull;
        const u64 xi = wave_scan_incl(x);
        if (lane < nw) scr[q * LW + lane] = xi - x;
        if (lane == G10_WAVE - 1) base[(u64)arrs[q] * nb1 + nch] = xi;
      }
    }
    __syncthreads();
    if (act && tid < nch)
      for (u32 q = 0; q < na; ++q) base[(u64)arrs[q] * nb1 + tid] = scr[q * LW + wave] + inc[q] - v[q];
    __syncthreads();
  };
  scan_bases(0, 1, 2, 3);
  scan_bases(3, 4, 0, 2);

  // The hot list: every tile not scored in this pass whose bound reaches `thr`; restL bounds
  // the tiles left out.  Bounds only fall and only scored tiles change, so the list stays
  // complete for any later threshold above restL and is kept across passes.
  auto build_hot = [&](u32 thr) {
    if (tid == 0) { S->nl = 0; S->restL = 0; }
    __syncthreads();
    u32 rm = 0;
    for (u32 g0 = 0; g0 < ns; g0 += 64) {          // 64 groups at a time, one per lane, in every wavefront alike
      const u32 sk = g0 + lane < ns ? skeys[g0 + lane] : 0u;
      const bool q = sk != 0 && sk >= thr;
      if (!q && sk > rm) rm = sk;
      u64 qm = __ballot(q);
      for (u32 turn = 0; qm; ++turn) {             // the wavefronts share the groups that qualify
        const u32 g = g0 + (u32)__builtin_ctzll(qm);
        qm &= qm - 1;
        if (turn % LW != wave) continue;
        const u32 t = g * 64 + lane;
        const u32 k = t < nt ? keys[t] : 0u;
        const bool marked = (smark[g] >> lane) & 1ull;
        const bool sel = k != 0 && k >= thr && !marked;
        if (!sel && !marked && k > rm) rm = k;
        const u64 m = __ballot(sel);
        if (m) {
          u32 off = 0;
          if (lane == 0) off = atomicAdd(&S->nl, (u32)__popcll(m));
          off = (u32)__builtin_amdgcn_readfirstlane((int)off);
          if (sel) tlist[off + __popcll(m & ((1ull << lane) - 1ull))] = (unsigned short)t;
        }
      }
    }
    rm = wave_max(rm);
    if (lane == 0 && rm) atomicMax(&S->restL, rm);
    __syncthreads();
  };

  // The tiles of the hot list whose bound reaches `thr` and that were not scored in this pass
  // -> alist (marked, bound cleared: the scoring rebuilds it); filt bounds the others.
  auto activate = [&](u32 thr) {
    if (tid == 0) { S->ntl = 0; S->filt = 0; }
    __syncthreads();
    const u32 nl = S->nl;
    u32 fm = 0;
    for (u32 i0 = 0; i0 < nl; i0 += LB) {
      const u32 i = i0 + tid;
      const u32 t = i < nl ? tlist[i] : 0u;
      const u32 k = i < nl ? keys[t] : 0u;
      const bool marked = i < nl && ((smark[t >> 6] >> (t & 63u)) & 1ull);
      const bool sel = k != 0 && k >= thr && !marked;
      if (!sel && !marked && k > fm) fm = k;
      const u64 m = __ballot(sel);
      if (m) {
        u32 off = 0;
        if (lane == 0) off = atomicAdd(&S->ntl, (u32)__popcll(m));
        off = (u32)__builtin_amdgcn_readfirstlane((int)off);
        if (sel) {
          alist[off + __popcll(m & ((1ull << lane) - 1ull))] = (unsigned short)t;
          keys[t] = 0;
          atomicOr((unsigned long long*)&smark[t >> 6], 1ull << (t & 63u));
        }
      }
      if (i0 + LB >= nl) break;
    }
    fm = wave_max(fm);
    if (lane == 0 && fm) atomicMax(&S->filt, fm);
    __syncthreads();
  };

  // this thread's best candidate of the pass
  Winner mine;
  mine.hi = 0; mine.lo = 0; mine.cand = NONE32;

  struct CandV { uint4 A, B; uint2 id; u32 p, t; };
  auto load_cand = [&](u32 u) -> CandV {
    CandV c;
    c.t = alist[u >> a.tshift];
    c.p = (((c.t << a.tshift) + (u & ((1u << a.tshift) - 1u))) << 8) + (tid & 255u);
    c.A = a.cd.A[c.p]; c.B = a.cd.B[c.p]; c.id = a.cd.id[c.p];
    return c;
  };

  // Scores the listed tiles: four wavefronts per 256 candidates, the next
  // candidate's record already in flight.  One workgroup has one texture
  // unit, about one cache line per clock: lanes whose candidate is dead load
  // nothing, and struck destinations are written back so later passes skip them.
  auto score_list = [&]() {
    const u32 nunits = S->ntl << a.tshift;
    PrefixView pv; pv.px = tl.px; pv.base = base; pv.K = K; pv.nch = nch; pv.shift_ch = tl.shift_ch;
    Machine mc; mc.bwo0 = bwo0; mc.bwo1 = bwo1; mc.bwi0 = bwi0; mc.bwi1 = bwi1;
    u32 u = tid >> 8;
    CandV cur;
    if (u < nunits) cur = load_cand(u);
    while (u < nunits) {
      const u32 un = u + LB / UNIT;
      CandV nxt;
      if (un < nunits) nxt = load_cand(un);
      const uint4 A = cur.A, B = cur.B;
      const Score r = score_candidate(pv, mc, A, B);
      if (r.strike0) a.cd.A[cur.p] = make_uint4(A.x, A.y, 1u, 0u);
      if (r.strike1) a.cd.B[cur.p] = make_uint4(1u, 0u, B.z, B.w);
#ifdef G10_PHASE_TIMERS
      {                                          // live candidates and destinations looked at
        const bool v0 = A.z <= A.w, v1 = B.x <= B.y;
        const u32 nl = (u32)__popcll(__ballot(v0 || v1)), nd = (u32)(__popcll(__ballot(v0)) + __popcll(__ballot(v1)));
        if (lane == 0) { atomicAdd((unsigned long long*)&S->phase[9], (unsigned long long)nl); atomicAdd((unsigned long long*)&S->phase[10], (unsigned long long)nd); }
      }
#endif
      const bool one = gt128(r.h1, r.l1, r.h0, r.l0);
      const u32 k = wave_max(upkey(one ? r.h1 : r.h0, one ? r.l1 : r.l0));
      if (lane == 0 && k) atomicMax(&keys[cur.t], k);
      if (r.ok0 || r.ok1) {                      // flash first; host only if flash cannot take it
        const u32 d = r.ok0 ? 0u : 1u;
        const u64 hi = d ? r.h1 : r.h0, lo = d ? r.l1 : r.l0;
        if ((hi | lo) != 0 && better(hi, lo, cur.id.x, mine.hi, mine.lo, mine.cand)) {
          mine.hi = hi; mine.lo = lo; mine.cand = cur.id.x; mine.tensor = cur.id.y; mine.pos = cur.p; mine.dest = d;
          mine.L1 = A.x; mine.R = A.y; mine.a = d ? B.x : A.z; mine.b = d ? B.y : A.w; mine.s = ((u64)B.w << 32) | B.z;
          mine.fo_base = r.fo_L; mine.fi_end = r.fi_R;
        }
      }
      u = un;
      cur = nxt;
    }
    if (tid == 0) S->units += nunits;
  };

  // block-wide arg-max of the threads' best (two barriers); refreshes the group bounds in between
  auto reduce_best = [&]() {
    const u32 bl = wave_best_lane(mine.hi, mine.lo, mine.cand);
    if (bl == NONE32) { if (lane == 0) { S->wave_win[wave].hi = 0; S->wave_win[wave].lo = 0; S->wave_win[wave].cand = NONE32; } }
    else if (lane == bl) S->wave_win[wave] = mine;
    __syncthreads();                               // all tile bounds and wavefront winners are in LDS
    const u32 ntl = S->ntl;
    for (u32 i = wave - 1; wave && i < ntl; i += LW - 1) {   // bounds of the groups that hold re-scored tiles
      const u32 g = alist[i] >> 6, t = g * 64 + lane;
      const u32 k = wave_max(t < nt ? keys[t] : 0u);
      if (lane == 0) skeys[g] = k;
    }
    if (wave == 0) {
      u64 h = 0, l = 0;
      u32 c = NONE32;
      if (lane < LW) { h = S->wave_win[lane].hi; l = S->wave_win[lane].lo; c = S->wave_win[lane].cand; }
      const u32 w = wave_best_lane(h, l, c);
      if (w == NONE32) { if (lane == 0) { S->win.hi = 0; S->win.lo = 0; } }
      else {
        if (lane == 0) {
          S->win = S->wave_win[w];
          S->tau_o = ceil_div_x1000(S->wave_win[w].s, S->wave_win[w].dest ? bwo1 : bwo0, S->wave_win[w].dest ? ivo1 : ivo0);
        }
        if (lane == 1) S->tau_i = ceil_div_x1000(S->wave_win[w].s, S->wave_win[w].dest ? bwi1 : bwi0, S->wave_win[w].dest ? ivi1 : ivi0);
      }
    }
    __syncthreads();
  };

  // ---- chunk jobs: one wavefront rewrites one chunk of one array ------------------------
  auto run_jobs = [&]() {
    const u32 nj = S->njobs;
    const u32 d = S->win.dest, L1 = S->win.L1, R = S->win.R, wa = S->win.a, wb = S->win.b;
    const u64 s = S->win.s, tau_o = S->tau_o, tau_i = S->tau_i, fo_base = S->win.fo_base, fi_end = S->win.fi_end;
    for (u32 jb = wave; jb < nj; jb += LW) {
      const u32 type = jobs[jb] >> 16, c = jobs[jb] & 0xffffu;
      const u32 s0 = c * CH;
      if (type == J_FO || type == J_FI) {
        // channel time of the window is taken from this chunk's slots; the free-time prefix
        // of the slots after the first window slot is rewritten from a scan of the new values
        const bool out = type == J_FO;
        const u32 arr = (out ? A_FO : A_FI) + d, w = out ? w_fo(d) : w_fi(d);
        u64* fr = tl.fre + (u64)((out ? 0u : 2u) + d) * tl.Kp;
        const u64 bc = base[(u64)arr * nb1 + c], ball = base[(u64)arr * nb1 + nch];
        const u32 x = out ? L1 : wb + 1, y = out ? wa - 1 : R - 1;
        const u32 first = first_covered(s0, (s0 + CH - 1 < K - 1) ? s0 + CH - 1 : K - 1, K, x, y);
        u64 carry = 0;
        for (u32 st = 0; st < tl.spt; ++st) {
          const u32 j0 = s0 + st * 256u + lane * 4u;
          u64 f[4], old[4];
          u32 jj[4];
#pragma unroll
          for (u32 i = 0; i < 4; ++i) {
            const u32 j = j0 + i;
            f[i] = j < K ? fr[j] : 0ull;
            jj[i] = j < K ? in_doubled(j, K, x, y) : NONE32;
            old[i] = jj[i] != NONE32 ? tl.px[(u64)j * PX + w] : 0ull;       // free time of the chunk before the slot
          }
          u64 lsum = 0;
#pragma unroll
          for (u32 i = 0; i < 4; ++i) {
            if (jj[i] != NONE32) {
              const u64 before_slot = (jj[i] >= K ? ball : 0ull) + bc + old[i];  // free time before slot jj
              u64 take;
              if (out) {                           // eviction: earliest free time of the window first
                const u64 before = before_slot - fo_base;
                const u64 used = before < tau_o ? before : tau_o;
                take = f[i] < tau_o - used ? f[i] : tau_o - used;
              } else {                             // prefetch: latest free time first
                const u64 after = fi_end - (before_slot + f[i]);
                const u64 used = after < tau_i ? after : tau_i;
                take = f[i] < tau_i - used ? f[i] : tau_i - used;
              }
              if (take) { f[i] -= take; fr[j0 + i] = f[i]; }
            }
            lsum += f[i];
          }
          const u64 inc = wave_scan_incl(lsum);
          u64 run = carry + inc - lsum;
#pragma unroll
          for (u32 i = 0; i < 4; ++i) {
            const u32 j = j0 + i;
            if (j < K && j > first) tl.px[(u64)j * PX + w] = run;
            run += f[i];
          }
          carry += wave_last(inc);
        }
        if (lane == 0) tot[(u64)arr * nch + c] = carry;
      } else if (type == J_P_PART || type == J_P_FULL) {
        // pressure of the chunk's slots; where a slot drops under the capacity the
        // over-capacity prefix after it is rewritten
        const u64 lz = lazyP[c];
        u64 mn = NONE64;
        u32 first = NONE32;                              // first slot that dropped under the capacity
        for (u32 st = 0; st < tl.spt; ++st) {
          const u32 j0 = s0 + st * 256u + lane * 4u;
          u32 myfirst = NONE32;
#pragma unroll
          for (u32 i = 0; i < 4; ++i) {
            const u32 j = j0 + i;
            if (j < K) {
              u64 p = tl.P[j];
              const bool hit = type == J_P_PART && in_doubled(j, K, wa, wb) != NONE32;
              const u64 before = p - lz + (type == J_P_FULL ? s : 0ull);     // pressure before this eviction
              if (hit) { p -= s; tl.P[j] = p; }
              const u64 act = p - lz;
              if (act > cap) mn = act < mn ? act : mn;
              else if (before > cap && myfirst == NONE32) myfirst = j;
            }
          }
          const u32 stfirst = wave_min(myfirst);
          if (first == NONE32) first = stfirst;
        }
        mn = wave_min(mn);
        if (lane == 0) minOver[c] = mn;
        if (first != NONE32) {                           // rewrite the prefix of the slots after it
          u64 carry = 0;
          for (u32 st = 0; st < tl.spt; ++st) {
            const u32 j0 = s0 + st * 256u + lane * 4u;
            u64 v[4];
            u64 lsum = 0;
#pragma unroll
            for (u32 i = 0; i < 4; ++i) {
              const u32 j = j0 + i;
              v[i] = 0;
              if (j < K && tl.P[j] - lz > cap) v[i] = tl.dur[j];
              lsum += v[i];
            }
            const u64 inc = wave_scan_incl(lsum);
            u64 run = carry + inc - lsum;
#pragma unroll
            for (u32 i = 0; i < 4; ++i) {
              const u32 j = j0 + i;
              if (j < K && j > first) {
                ulonglong2* rec = reinterpret_cast<ulonglong2*>(tl.px + (u64)j * PX);
                rec[0].y = run; rec[1].y = run; rec[2].y = run; rec[3].y = run;   // the four copies of OT
              }
              run += v[i];
            }
            carry += wave_last(inc);
          }
          if (lane == 0) { tot[(u64)A_OT * nch + c] = carry; S->ot_changed = 1; }
        }
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

  __syncthreads();
  // ---- passes ------------------------------------------------------------------------
  u32 passes = 0;
  while (true) {
    if (S->done) break;
    if (base[(u64)A_OT * nb1 + nch] == 0) { if (tid == 0) { S->done = 1; S->status = G10_FITS; } break; }
    if (max_iter && S->n_iter >= max_iter) { if (tid == 0) { S->done = 1; S->status = G10_TRUNCATED; } break; }
    if (passes >= a.pass_budget || S->stop) break;
    ++passes;
    mine.hi = 0; mine.lo = 0; mine.cand = NONE32;
    u32 thr = S->thr_key ? S->thr_key : NONE32;
    __syncthreads();                               // the loop conditions and thr are read
    for (u32 i = tid; i < ns; i += LB) smark[i] = 0;     // no tile scored in this pass yet
    if (tid == 0) {
      S->n_iter += 1; S->n_evals += C - S->n_mig - S->n_drop;
      S->hq = 0; S->njobs = 0; S->ot_changed = 0;
      S->win.hi = 0; S->win.lo = 0;
      if (S->stale_hot) { S->restL = NONE32; S->stale_hot = 0; }
      if (a.tick_budget && wall_clock64() - S->t_start > a.tick_budget) S->stop = 1;
    }
    __syncthreads();

    // rank: score the hot tiles whose bound reaches a threshold (first a guess a little under
    // the last benefit), lower the threshold to the best benefit found, repeat until no tile
    // left out could hold an equal or better candidate
    u32 rounds = 0;
    while (true) {
      if (S->restL >= thr) {                       // the hot list may miss a tile that reaches thr: build it anew,
        const u32 low = thr == NONE32 ? thr : (thr > (1u << 19) ? thr - (1u << 19) : 1u);   // a few percent lower to last a while
        __syncthreads();
        build_hot(low);
        if (rounds && tid == 0) S->stale_hot = 1;  // built without the tiles already scored: not kept for the next pass
      }
      activate(thr);
      const u32 ntl = S->ntl, rest = S->restL > S->filt ? S->restL : S->filt;
      if (ntl == 0) {
        if ((rounds && (S->win.hi | S->win.lo) != 0) || rest == 0) break;      // nothing left that could win
        thr = rest;                                      // strictly lower than before: start from the largest bound left
        __syncthreads();
        continue;
      }
      PHASE(0);
      score_list();
      PHASE(1);
      reduce_best();
      PHASE(2);
      ++rounds;
      const u32 kb = upkey(S->win.hi, S->win.lo);
      const u32 need = kb ? kb : 1u;
      if (rest < need) break;                            // every tile left out is below the best found
      // a tile left out may hold an equal or better one; with nothing found yet, step down a few percent
      thr = kb ? kb : (rest > (1u << 19) ? rest - (1u << 19) : 1u);
      if (tid == 0) S->second += 1;
      __syncthreads();
    }
    PHASE(3);

    const bool none = (S->win.hi | S->win.lo) == 0;
    const u32 d = S->win.dest, L1 = S->win.L1, R = S->win.R, wa = S->win.a, wb = S->win.b;
    const u64 s = S->win.s;
    if (none) { __syncthreads(); if (tid == 0) { S->done = 1; S->status = G10_RESIDUAL; } break; }

    // which chunks the period, its absent window and its transfer windows cover
    u32 cvE = 0, cvW = 0, cvA = 0, cvP = 0, len = 0;
    if (tid < nch) {
      cvE = cover(tid, CH, K, L1, wa - 1, len);
      cvW = cover(tid, CH, K, wb + 1, R - 1, len);
      cvA = cover(tid, CH, K, wa, wb, len);
      cvP = cvE + cvA + cvW;                             // the period interior [L1, R - 1]
    }
    // host memory must hold the tensor during the whole period
    bool room = true;
    if (d == G10_HOST) {
      if (tid < ((nch + 63u) & ~63u)) {                  // bound: the maxima of all chunks the period touches
        const u64 m = wave_max(cvP ? hmax[tid] : 0ull);
        if (lane == 0 && m) atomicMax((unsigned long long*)&S->hq, (unsigned long long)m);
      }
      __syncthreads();
      room = s <= host_cap && S->hq <= host_cap - s;
      if (!room) {                                       // exact: chunks cut by the period ends slot by slot
        __syncthreads();
        if (tid == 0) S->hq = 0;
        __syncthreads();
        if (cvP == len && cvP) atomicMax((unsigned long long*)&S->hq, (unsigned long long)hmax[tid]);
        else if (cvP) jobs[atomicAdd(&S->njobs, 1u)] = ((u32)J_HQ << 16) | tid;
        __syncthreads();
        run_jobs();
        __syncthreads();
        room = s <= host_cap && S->hq <= host_cap - s;
        __syncthreads();
        if (tid == 0) S->njobs = 0;
        __syncthreads();
      }
    }
    PHASE(4);
    if (tid == 0) {
      const u32 p = S->win.pos;
      a.cd.A[p] = make_uint4(L1, R, 1u, 0u);             // the candidate leaves the live set
      a.cd.B[p] = make_uint4(1u, 0u, (u32)s, (u32)(s >> 32));
      // first threshold of the next pass: a little under this benefit
      u64 ghi = S->win.hi, glo = S->win.lo;
      const u64 dlo = (glo >> GUESS_SHIFT) | (ghi << (64 - GUESS_SHIFT)), dhi = ghi >> GUESS_SHIFT;
      const u64 nlo = glo - dlo;
      ghi = ghi - dhi - (glo < dlo ? 1ull : 0ull);
      S->thr_key = upkey(ghi, nlo);
      if (!room) {
        g10_dropped dr; dr.iteration = S->n_iter - 1; dr.cand = S->win.cand; dr.reserved = 0;
        a.dropped[S->n_drop] = dr;
        S->n_drop += 1;
      } else {
        g10_migration mg;
        mg.cand = S->win.cand; mg.tensor = S->win.tensor;
        mg.evict_after = L1 - 1; mg.absent_first = wa >= K ? wa - K : wa; mg.absent_last = wb >= K ? wb - K : wb;
        mg.next_use = R >= K ? R - K : R;
        mg.dest = d; mg.wraps = R >= K ? 1u : 0u;
        mg.size_bytes = s; mg.t_out_ns = S->tau_o; mg.t_in_ns = S->tau_i; mg.benefit_lo = S->win.lo; mg.benefit_hi = S->win.hi;
        a.records[S->n_mig] = mg;
        a.rec_ab[S->n_mig] = make_uint2(wa, wb);
        S->n_mig += 1;
      }
    }
    if (!room) { __syncthreads(); continue; }

    // commit: whole chunks take a lazy add, the others a job
    if (tid < nch) {
      const u32 c = tid;
      if (cvE) jobs[atomicAdd(&S->njobs, 1u)] = ((u32)J_FO << 16) | c;
      if (cvW) jobs[atomicAdd(&S->njobs, 1u)] = ((u32)J_FI << 16) | c;
      if (cvA == len) {                                  // the whole chunk loses the tensor
        lazyP[c] += s;
        u64 mo = minOver[c];
        if (mo != NONE64) {
          mo -= s;
          minOver[c] = mo;
          if (mo <= cap) jobs[atomicAdd(&S->njobs, 1u)] = ((u32)J_P_FULL << 16) | c;   // a slot drops under the capacity
        }
      } else if (cvA) {
        jobs[atomicAdd(&S->njobs, 1u)] = ((u32)J_P_PART << 16) | c;
      }
      if (d == G10_HOST) {
        if (cvP == len) { lazyH[c] += s; hmax[c] += s; }
        else if (cvP) jobs[atomicAdd(&S->njobs, 1u)] = ((u32)J_H << 16) | c;
      }
    }
    __syncthreads();
    PHASE(6);
    run_jobs();
    __syncthreads();
    PHASE(7);
    // level 1: a transfer window inside one chunk lowers every later chunk's base by the
    // transfer time; otherwise (and for the over-capacity time, if it changed) scan again
    {
      const u32 eA = (L1 >= K ? L1 - K : L1) >> tl.shift_ch, eB = (wa - 1 >= K ? wa - 1 - K : wa - 1) >> tl.shift_ch;
      const u32 pA = (wb + 1 >= K ? wb + 1 - K : wb + 1) >> tl.shift_ch, pB = (R - 1 >= K ? R - 1 - K : R - 1) >> tl.shift_ch;
      const bool oneE = eA == eB && !(L1 < K && wa - 1 >= K), oneP = pA == pB && !(wb + 1 < K && R - 1 >= K);
      const bool ot = S->ot_changed != 0;
      if (oneE && oneP && !ot) {
        if (tid < nch) {
          if (tid > eA) base[(u64)(A_FO + d) * nb1 + tid] -= S->tau_o;
          if (tid > pA) base[(u64)(A_FI + d) * nb1 + tid] -= S->tau_i;
        }
        if (tid == 0) { base[(u64)(A_FO + d) * nb1 + nch] -= S->tau_o; base[(u64)(A_FI + d) * nb1 + nch] -= S->tau_i; }
        __syncthreads();
      } else if (ot) scan_bases(A_OT, A_FO + d, A_FI + d, 3);
      else scan_bases(A_FO + d, A_FI + d, 0, 2);
    }
    PHASE(8);
  }
  __syncthreads();

  // ---- state out ---------------------------------------------------------------------
  for (u32 i = tid; i < N_ARR * nch; i += LB) a.g_tot[i] = tot[i];
  for (u32 i = tid; i < nch; i += LB) { a.g_lazyP[i] = lazyP[i]; a.g_minOver[i] = minOver[i]; a.g_lazyH[i] = lazyH[i]; a.g_hmax[i] = hmax[i]; }
  for (u32 i = tid; i < nt; i += LB) a.g_keys[i] = keys[i];
  for (u32 i = tid; i < N_ARR * nb1; i += LB) a.g_base[i] = base[i];
  if (tid == 0) {
    ctl->n_iter = S->n_iter; ctl->n_mig = S->n_mig; ctl->n_drop = S->n_drop; ctl->n_evals = S->n_evals;
    ctl->thr_key = S->thr_key; ctl->status = S->status; ctl->done = S->done;
    ctl->overtime_after = base[(u64)A_OT * nb1 + nch];
    for (u32 i = 0; i < 12; ++i) ctl->phase[i] += S->phase[i];
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
  u32 *keep = nullptr, *scratch32 = nullptr, *hist = nullptr, *tkeys = nullptr;
  u64 *keys = nullptr, *keys_alt = nullptr;
  Cands cd[2] = {};
  u64 *P = nullptr, *fre = nullptr, *H = nullptr, *px = nullptr, *otc = nullptr, *base0 = nullptr, *g_tot = nullptr,
      *g_lazyP = nullptr, *g_minOver = nullptr, *g_lazyH = nullptr, *g_hmax = nullptr, *g_base = nullptr,
      *pressure_after = nullptr,
      *peak_after = nullptr;
  Ctl* ctl = nullptr;
  g10_migration* records = nullptr;
  uint2* rec_ab = nullptr;
  g10_dropped* dropped = nullptr;
  // smart prefetching
  u64 *pf_keys = nullptr, *pf_keys_alt = nullptr, *pf_pressure = nullptr, *pf_stats = nullptr;
  u32 *pf_order = nullptr, *pf_order_alt = nullptr, *pf_gained = nullptr, *pf_last = nullptr;
  u32 *h_pf_order = nullptr, *h_pf_gained = nullptr, *h_pf_last = nullptr;
  u64* h_pf_pressure = nullptr;
  bool planned = false;         // a plan is stored in the handle
  u64 plan_cap = 0, plan_n_mig = 0;
  // host copies handed out through g10_result
  g10_migration* h_records = nullptr;
  g10_dropped* h_dropped = nullptr;
  u64* h_pressure = nullptr;
  hipEvent_t ev[6] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
  void* arena = nullptr;        // the one device allocation all pointers above point into
  u32 max_chunks = 0;           // the chunk limit the timelines were laid out for
};

void plan_work_free(PlanWork* w) {
  if (!w) return;
  if (w->arena) (void)hipFree(w->arena);
  free(w->h_records);
  free(w->h_dropped);
  free(w->h_pressure);
  free(w->h_pf_order); free(w->h_pf_gained); free(w->h_pf_last); free(w->h_pf_pressure);
  for (hipEvent_t e : w->ev) if (e) (void)hipEventDestroy(e);
  delete w;
}

static const u32 PASS_BUDGET = 4096;             // ranking passes per launch of the loop kernel
#ifndef G10_RETILE_PASSES
#define G10_RETILE_PASSES 256
#endif
static const u32 RETILE_PASSES = G10_RETILE_PASSES;   // ... between two re-tilings of a long candidate list
static const u32 RETILE_MIN_CANDS = 8192;        // shorter lists are never re-tiled
static const u64 BATCH_LAUNCH_TICKS = 250000;    // a launch of a batch ends after 2.5 ms (100 MHz clock)

static u32 tile_shift_for(u64 n, u32 max_tiles) { // smallest tile (256 << shift) with at most max_tiles tiles
  u32 sh = 0;
  while ((((n + UNIT - 1) / UNIT) + (1ull << sh) - 1) >> sh > max_tiles) ++sh;
  return sh;
}

static u32 clamp_limit(u32 asked, u32 lib_max) { return asked == 0 || asked > lib_max ? lib_max : asked; }

// One device allocation for all planning workspaces (a handle is often short-lived; every
// hipMalloc / hipFree costs about 0.1 ms): the layout is walked twice, first to measure.
struct Arena {
  char* base = nullptr;
  size_t off = 0;
  template <class T>
  void take(T** out, u64 elems) {
    off = (off + 255) & ~(size_t)255;
    if (base) *out = (T*)(base + off);
    off += (size_t)(elems ? elems : 1) * sizeof(T);
  }
};

static void work_layout(PlanWork* w, Arena& ar) {
  const u32 K = w->K;
  const u64 C = w->C;
  ar.take(&w->win, C);
  ar.take(&w->keep, C + 1);
  const u64 he = radix_hist_elems(C);
  ar.take(&w->hist, he);
  ar.take(&w->scratch32, scan_scratch_elems(he > C ? he : C));
  ar.take(&w->keys, C); ar.take(&w->keys_alt, C);
  ar.take(&w->tkeys, (u64)NT_MAX);
  for (int i = 0; i < 2; ++i) { ar.take(&w->cd[i].A, w->cap_pad); ar.take(&w->cd[i].B, w->cap_pad); ar.take(&w->cd[i].id, w->cap_pad); }
  ar.take(&w->P, K); ar.take(&w->fre, (u64)4 * w->Kp); ar.take(&w->H, K);
  ar.take(&w->px, (u64)PX * K); ar.take(&w->otc, (u64)K + 1);
  ar.take(&w->base0, (u64)w->nch + 1);
  ar.take(&w->g_base, (u64)N_ARR * (w->nch + 1));
  ar.take(&w->g_tot, (u64)N_ARR * w->nch);
  ar.take(&w->g_lazyP, w->nch); ar.take(&w->g_minOver, w->nch);
  ar.take(&w->g_lazyH, w->nch); ar.take(&w->g_hmax, w->nch);
  ar.take(&w->pressure_after, K);
  ar.take(&w->peak_after, 1);
  ar.take(&w->ctl, 1);
  ar.take(&w->records, C);
  ar.take(&w->rec_ab, C);
  ar.take(&w->dropped, C);
  ar.take(&w->pf_keys, C); ar.take(&w->pf_keys_alt, C);
  ar.take(&w->pf_order, C); ar.take(&w->pf_order_alt, C);
  ar.take(&w->pf_gained, C); ar.take(&w->pf_last, C);
  ar.take(&w->pf_pressure, K);
  ar.take(&w->pf_stats, 4);
}

static int work_alloc(g10_plan_s* h, u32 max_chunks, PlanWork** slot) {
  PlanWork* w = new (std::nothrow) PlanWork();
  if (!w) return G10_ENOMEM;
  *slot = w;
  const u32 K = h->K;
  const u64 C = h->n_periods;
  w->K = K; w->C = C;
  w->Kp = (K + 3u) & ~3u;
  w->spt = 1; w->shift_ch = 8;
  w->max_chunks = max_chunks;
  while ((u64)G10_BLOCK * w->spt * max_chunks < K) { w->spt *= 2; w->shift_ch += 1; }
  const u32 ch = G10_BLOCK * w->spt;
  w->nch = (K + ch - 1) / ch;
  // room for the padding of the last tile at any tile size: tiles hold at most max(256, C) candidates
  w->cap_pad = 2 * (C > UNIT ? C : UNIT) + UNIT;
  Arena measure;
  work_layout(w, measure);
  void* q = nullptr;
  if (hipMalloc(&q, measure.off + 256) != hipSuccess) { (void)hipGetLastError(); return G10_ENOMEM; }
  w->arena = q;
  Arena carve;
  carve.base = (char*)q;
  work_layout(w, carve);
  w->h_records = (g10_migration*)malloc((C ? C : 1) * sizeof(g10_migration));
  w->h_dropped = (g10_dropped*)malloc((C ? C : 1) * sizeof(g10_dropped));
  w->h_pressure = (u64*)malloc((u64)K * sizeof(u64));
  if (!w->h_records || !w->h_dropped || !w->h_pressure) return G10_ENOMEM;
  for (hipEvent_t& e : w->ev) G10_HIP(hipEventCreate(&e));
  return G10_OK;
}

static size_t loop_lds_bytes(u32 nch, u32 nt) {
  const size_t ns = (nt + 63) / 64;
  size_t b = 0;
  b += ((size_t)N_ARR * (nch + 1) + (size_t)N_ARR * nch + (size_t)4 * nch + ns + (size_t)4 * LW) * 8;
  b += sizeof(Shared);
  b += ((size_t)nt + ns + (size_t)4 * nch + 8) * 4 + (size_t)nt * 4;
  return (b + 15) & ~(size_t)15;
}

// One plan of a batch, host side.
struct Inst {
  PlanWork* w = nullptr;
  const g10_params* p = nullptr;
  Ctl hc;
  Timelines tl;
  u32 n = 0, n_valid = 0, max_tiles = 0;
  u32 tsh = 0, nt = 0, n_pad = 0;
  int cur = 0;                 // the candidate buffer the loop reads
  u64 retiles = 0, launches = 0, max_launches = 0, overtime_before = 0;
  bool counted = false;        // hc.n_live holds a count of the current list
  bool timed_full = false;
  u64 seen_iter = 0;           // passes done at the last re-tiling
};

static PlanWork** work_slot(g10_plan_s* h, u32 i) { return i == 0 ? &h->work : &h->more[i - 1]; }

// `count` plans on one analysed trace.  The streaming kernels of the plans run one after the
// other (each fills the chip); the greedy loops run side by side, one workgroup per plan, in
// one launch per round; between rounds the long candidate lists are put back into score order.
int plan_batch_run(g10_plan_s* h, const g10_params* params, u32 count, g10_result* outs) {
  hipStream_t s = h->stream;
  const u32 K = h->K;
  const u32 C = (u32)h->n_periods;
  const u32 gC = (C + G10_BLOCK - 1) / G10_BLOCK;
  if (count > 1 + h->n_more) {                             // more workspace slots
    PlanWork** m = (PlanWork**)realloc(h->more, (size_t)(count - 1) * sizeof(PlanWork*));
    if (!m) return G10_ENOMEM;
    for (u32 i = h->n_more; i < count - 1; ++i) m[i] = nullptr;
    h->more = m; h->n_more = count - 1;
  }
  if (count > h->loop_args_cap) {
    if (h->loop_args) { G10_HIP(hipStreamSynchronize(s)); (void)hipFree(h->loop_args); h->loop_args = nullptr; h->loop_args_cap = 0; }
    void* q = nullptr;
    if (hipMalloc(&q, (size_t)count * sizeof(LoopArgs)) != hipSuccess) { (void)hipGetLastError(); return G10_ENOMEM; }
    h->loop_args = q; h->loop_args_cap = count;
  }
  Inst* I = new (std::nothrow) Inst[count];
  LoopArgs* hargs = (LoopArgs*)malloc((size_t)count * sizeof(LoopArgs));
  struct Guard { Inst* i; LoopArgs* a; ~Guard() { delete[] i; free(a); } } guard{I, hargs};
  if (!I || !hargs) return G10_ENOMEM;

  for (u32 i = 0; i < count; ++i) {
    const g10_params* p = params + i;
    const u32 max_chunks = clamp_limit(p->max_chunks, NCH_MAX);
    PlanWork** slot = work_slot(h, i);
    if (*slot && (*slot)->max_chunks != max_chunks) {      // another chunk size: lay the workspaces out again
      G10_HIP(hipStreamSynchronize(s));
      plan_work_free(*slot);
      *slot = nullptr;
    }
    if (!*slot) {
      int rc = work_alloc(h, max_chunks, slot);
      if (rc) { plan_work_free(*slot); *slot = nullptr; return rc; }
    }
    I[i].w = *slot; I[i].p = p; I[i].max_tiles = clamp_limit(p->max_tiles, NT_MAX);
    (*slot)->planned = false;
  }

  // ---- timelines before any eviction, candidate windows --------------------------------
  G10_HIP(hipEventRecord(I[0].w->ev[0], s));
  for (u32 i = 0; i < count; ++i) {
    Inst& x = I[i];
    PlanWork* w = x.w;
    const g10_params* p = x.p;
    Ctl& hc = x.hc;
    memset(&hc, 0, sizeof hc);
    hc.gpu_cap = p->gpu_cap_bytes; hc.host_cap = p->host_cap_bytes;
    for (int d = 0; d < 2; ++d) {
      hc.bw_out[d] = p->bw_out_Bpus[d]; hc.bw_in[d] = p->bw_in_Bpus[d];
      hc.inv_out[d] = hc.bw_out[d] > 1 ? (u64)((((unsigned __int128)1) << 64) / hc.bw_out[d]) : 0;
      hc.inv_in[d] = hc.bw_in[d] > 1 ? (u64)((((unsigned __int128)1) << 64) / hc.bw_in[d]) : 0;
    }
    hc.max_iter = p->max_iterations;
    hc.C = C;
    G10_HIP(hipMemcpyAsync(w->ctl, &hc, sizeof hc, hipMemcpyHostToDevice, s));
    Timelines& tl = x.tl;
    tl.dur = h->dur; tl.P = w->P; tl.fre = w->fre; tl.H = w->H; tl.px = w->px; tl.otc = w->otc;
    tl.K = K; tl.Kp = w->Kp; tl.nch = w->nch; tl.spt = w->spt; tl.shift_ch = w->shift_ch;
    G10_HIP(hipMemsetAsync(w->peak_after, 0, 8, s));
    hipLaunchKernelGGL(k_init_timelines, dim3(w->nch), dim3(G10_BLOCK), 0, s, tl, (const u64*)(h->pressure_buf + 1),
                       (const Ctl*)w->ctl, w->g_tot, w->g_lazyP, w->g_minOver, w->g_lazyH, w->g_hmax);
    hipLaunchKernelGGL(k_level1_init, dim3(1), dim3(LB), 0, s, (const u64*)w->g_tot, w->nch, w->base0, w->ctl);
    hipLaunchKernelGGL(k_ot_full, dim3(K / G10_BLOCK + 1), dim3(G10_BLOCK), 0, s, w->otc, (const u64*)w->base0, K, w->nch, w->shift_ch);
    G10_HIP(hipGetLastError());
    if (C) {      // windows per destination; keep the candidates with at least one valid window
      hipLaunchKernelGGL(k_prep, dim3(gC), dim3(G10_BLOCK), 0, s, (const uint4*)h->per_by_start, (const u64*)h->per_size, h->start, K, h->T, C,
                         (const Ctl*)w->ctl, w->win, w->keep);
      G10_HIP(hipGetLastError());
      G10_TRY(scan_excl_u32(w->keep, w->keep, C, w->scratch32, s));
      G10_HIP(hipMemcpyAsync(&x.n, w->keep + C, sizeof(u32), hipMemcpyDeviceToHost, s));
    }
    G10_HIP(hipMemcpyAsync(&hc, w->ctl, sizeof hc, hipMemcpyDeviceToHost, s));
  }
  G10_HIP(hipStreamSynchronize(s));

  // candidates of plan x into score order, in tiles
  auto retile = [&](Inst& x, bool first) -> int {
    PlanWork* w = x.w;
    x.tsh = tile_shift_for(x.n, x.max_tiles);
    const u32 tile = UNIT << x.tsh;
    x.nt = (u32)(((u64)x.n + tile - 1) / tile);
    x.n_pad = x.nt * tile;
    if (!x.n) return G10_OK;
    const u32 n = x.n, posbits = bits_for(n - 1);
    if (first) {
      const u32 gn = (n + G10_BLOCK - 1) / G10_BLOCK;
      // the two events take the kernel's own begin and end time stamps
      hipExtLaunchKernelGGL(k_score_full, dim3(gn), dim3(G10_BLOCK), 0, s, w->ev[2], w->ev[3], 0, (const uint4*)w->cd[x.cur].A,
                            (const uint4*)w->cd[x.cur].B, n, (const u64*)w->otc, K, posbits, w->keys);
      x.timed_full = true;
    } else {
      u32 gn = (n + G10_BLOCK - 1) / G10_BLOCK;
      if (gn > 2048) gn = 2048;
      G10_HIP(hipMemsetAsync(&w->ctl->n_live, 0, sizeof(u32), s));
      hipLaunchKernelGGL(k_rescore, dim3(gn), dim3(G10_BLOCK), (size_t)N_ARR * (w->nch + 1) * 8, s, w->cd[x.cur], n,
                         (const u64*)w->px, (const u64*)w->g_base, K, w->nch, w->shift_ch, (const Ctl*)w->ctl, posbits,
                         w->keys, &w->ctl->n_live);
    }
    G10_HIP(hipGetLastError());
    u64 *keys = w->keys, *alt = w->keys_alt;
    G10_TRY(radix_sort_u64(&keys, &alt, n, posbits + 23, w->hist, w->scratch32, s));
    G10_HIP(hipMemsetAsync(w->tkeys, 0, (u64)NT_MAX * 4, s));
    hipLaunchKernelGGL(k_tile_gather, dim3(x.n_pad / G10_BLOCK), dim3(G10_BLOCK), 0, s, (const u64*)keys, n, x.n_pad, posbits,
                       w->cd[x.cur], w->cd[x.cur ^ 1], 8 + x.tsh, w->tkeys);
    G10_HIP(hipGetLastError());
    x.cur ^= 1;
    return G10_OK;
  };

  u32 n_active = 0;
  size_t lds_max = 0;
  for (u32 i = 0; i < count; ++i) {
    Inst& x = I[i];
    x.overtime_before = x.hc.overtime_before;
    x.n_valid = x.n;
    // every pass removes a candidate or stops, so the launches are bounded
    x.max_launches = count == 1 ? (u64)x.n / RETILE_PASSES + 3 : (u64)x.n + 3;   // (a launch by the clock makes a pass at least)
    if (x.hc.done) continue;
    ++n_active;
    if (x.n) {
      hipLaunchKernelGGL(k_pack, dim3(gC), dim3(G10_BLOCK), 0, s, (const uint4*)h->per_by_start, (const u64*)h->per_size, (const uint4*)x.w->win,
                         (const u32*)x.w->keep, C, x.w->cd[x.cur]);
      G10_HIP(hipGetLastError());
    }
    G10_TRY(retile(x, true));
    const size_t lds = loop_lds_bytes(x.w->nch, x.nt);
    if (lds > lds_max) lds_max = lds;
  }
  if (!h->lds_opt_in && lds_max > 64 * 1024) {
    G10_HIP(hipFuncSetAttribute((const void*)k_loop, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    h->lds_opt_in = true;
  }

  // ---- the greedy loops: one workgroup per plan, side by side ------------------------------
  // Long lists are put back into score order every RETILE_PASSES passes or more: the tiles the
  // loop looks at are dense with live candidates again, and the list is cut to those that can
  // still score.  A batch ends its launches by the clock instead, so that no plan waits long for
  // the slowest one.
  const bool timed_loop = n_active != 0;
  if (timed_loop) G10_HIP(hipEventRecord(I[0].w->ev[4], s));
  while (n_active) {
    u32 na = 0;
    size_t lds = 0;
    for (u32 i = 0; i < count; ++i) {
      Inst& x = I[i];
      if (x.hc.done) continue;
      if (x.launches++ > x.max_launches) return G10_EDEVICE;
      PlanWork* w = x.w;
      LoopArgs& la = hargs[na++];
      la.tl = x.tl;
      la.g_tot = w->g_tot; la.g_lazyP = w->g_lazyP; la.g_minOver = w->g_minOver; la.g_lazyH = w->g_lazyH; la.g_hmax = w->g_hmax;
      la.g_base = w->g_base;
      la.g_keys = w->tkeys; la.ctl = w->ctl; la.records = w->records; la.rec_ab = w->rec_ab; la.dropped = w->dropped;
      la.cd = w->cd[x.cur]; la.n_pad = x.n_pad; la.nt = x.nt; la.tshift = x.tsh;
      la.pass_budget = x.n > RETILE_MIN_CANDS && count == 1 ? RETILE_PASSES : PASS_BUDGET;
      la.tick_budget = count > 1 ? BATCH_LAUNCH_TICKS : 0;
      const size_t l = loop_lds_bytes(w->nch, x.nt);
      if (l > lds) lds = l;
    }
    G10_HIP(hipMemcpyAsync(h->loop_args, hargs, (size_t)na * sizeof(LoopArgs), hipMemcpyHostToDevice, s));
    hipLaunchKernelGGL(k_loop, dim3(na), dim3(LB), lds, s, (const LoopArgs*)h->loop_args);
    G10_HIP(hipGetLastError());
    for (u32 i = 0; i < count; ++i)
      if (!I[i].hc.done) G10_HIP(hipMemcpyAsync(&I[i].hc, I[i].w->ctl, sizeof(Ctl), hipMemcpyDeviceToHost, s));
    G10_HIP(hipStreamSynchronize(s));
    n_active = 0;
    for (u32 i = 0; i < count; ++i) {
      Inst& x = I[i];
      if (x.hc.done) continue;
      ++n_active;
      if (x.n > RETILE_MIN_CANDS && x.hc.n_iter - x.seen_iter >= RETILE_PASSES) {
        x.seen_iter = x.hc.n_iter;
        if (x.counted && x.hc.n_live < x.n) x.n = x.hc.n_live;   // live candidates come first in the list
        G10_TRY(retile(x, false));
        x.counted = true;
        ++x.retiles;
      }
    }
  }
  if (timed_loop) G10_HIP(hipEventRecord(I[0].w->ev[5], s));

  // ---- results ---------------------------------------------------------------------------
  u64* peaks = (u64*)hargs;                                // reuse as a small host buffer (count <= its size / 8)
  for (u32 i = 0; i < count; ++i) {
    Inst& x = I[i];
    PlanWork* w = x.w;
    const Ctl& hc = x.hc;
    hipLaunchKernelGGL(k_finish, dim3(K / G10_BLOCK / 4 + 1), dim3(G10_BLOCK), 0, s, x.tl, (const u64*)w->g_lazyP, w->pressure_after,
                       w->peak_after);
    G10_HIP(hipGetLastError());
    G10_HIP(hipMemcpyAsync(&peaks[i], w->peak_after, 8, hipMemcpyDeviceToHost, s));
    if (hc.n_mig) G10_HIP(hipMemcpyAsync(w->h_records, w->records, hc.n_mig * sizeof(g10_migration), hipMemcpyDeviceToHost, s));
    if (hc.n_drop) G10_HIP(hipMemcpyAsync(w->h_dropped, w->dropped, hc.n_drop * sizeof(g10_dropped), hipMemcpyDeviceToHost, s));
    G10_HIP(hipMemcpyAsync(w->h_pressure, w->pressure_after, (u64)K * 8, hipMemcpyDeviceToHost, s));
  }
  G10_HIP(hipEventRecord(I[0].w->ev[1], s));
  G10_HIP(hipStreamSynchronize(s));
  float ms = 0.f, loop_ms = 0.f;
  G10_HIP(hipEventElapsedTime(&ms, I[0].w->ev[0], I[0].w->ev[1]));
  if (timed_loop) G10_HIP(hipEventElapsedTime(&loop_ms, I[0].w->ev[4], I[0].w->ev[5]));

  for (u32 i = 0; i < count; ++i) {
    Inst& x = I[i];
    PlanWork* w = x.w;
    const Ctl& hc = x.hc;
    float full_ms = 0.f;
    if (x.timed_full) G10_HIP(hipEventElapsedTime(&full_ms, w->ev[2], w->ev[3]));
#ifdef G10_PHASE_TIMERS
    if (getenv("G10_LOG")) {
      fprintf(stderr, "g10: loop phases (us per pass):");
      for (int q = 0; q < 9; ++q) fprintf(stderr, " %d:%.2f", q, hc.phase[q] / 100.0 / (double)(hc.n_iter ? hc.n_iter : 1));
      fprintf(stderr, "  live/pass %.1f dests/pass %.1f\n", hc.phase[9] / (double)(hc.n_iter ? hc.n_iter : 1), hc.phase[10] / (double)(hc.n_iter ? hc.n_iter : 1));
    }
#endif
    w->planned = true; w->plan_cap = x.p->gpu_cap_bytes; w->plan_n_mig = hc.n_mig;
    g10_result* out = outs + i;
    memset(out, 0, sizeof *out);
    out->status = (int32_t)hc.status;
    out->n_migrations = hc.n_mig; out->n_iterations = hc.n_iter; out->n_dropped = hc.n_drop; out->n_cand_evals = hc.n_evals;
    out->peak_before = h->peak; out->peak_after = peaks[i];
    out->overtime_before_ns = x.overtime_before; out->overtime_after_ns = hc.overtime_after;
    out->migrations = w->h_records; out->dropped = w->h_dropped; out->pressure_after = w->h_pressure;
    out->plan_ms = ms;
    out->score_full_ms = full_ms; out->score_full_cands = x.n_valid;
    out->loop_ms = loop_ms; out->loop_launches = hc.launches; out->loop_retiles = x.retiles;
    out->loop_cands_scored = hc.units_scored * UNIT; out->loop_second_rounds = hc.second_rounds; out->loop_chunk_jobs = hc.jobs_run;
  }
  return G10_OK;
}

int plan_run(g10_plan_s* h, const g10_params* p, g10_result* out) { return plan_batch_run(h, p, 1, out); }

// ===========================================================================
// Smart prefetching (Section 4.4) on a finished plan
// ===========================================================================
// The evicted periods are visited in the order of their latest safe prefetch
// time; each prefetch moves back, in whole kernel slots and not past the first
// absent slot, to the earliest slot from which every slot up to the old
// prefetch can hold the tensor (pressure + size <= capacity); the pressure of
// the slots gained rises by the tensor's size.  Every step depends on the
// pressure the earlier ones left, so this is a serial chain like the eviction
// loop and runs in one workgroup: the pressure in HBM / L2, per chunk a lazy
// add and the chunk maximum in LDS.  The search asks the chunk maxima which
// chunk can hold the last slot that cannot take the tensor and scans only that
// chunk; the update adds lazily to whole chunks and slot by slot at the ends.
namespace {

__global__ __launch_bounds__(G10_BLOCK) void k_pf_keys(const g10_migration* __restrict__ rec, u32 n, const u64* __restrict__ start,
                                                      u32 K, u64 T, u64* __restrict__ keys, u32* __restrict__ order) {
  const u32 i = blockIdx.x * G10_BLOCK + threadIdx.x;
  if (i >= n) return;
  const u64 t_use = start[rec[i].next_use] + (rec[i].wraps ? T : 0ull);
  keys[i] = t_use - rec[i].t_in_ns;              // latest safe prefetch time
  order[i] = i;
}

struct PfShared {
  unsigned long long cand;    // (upper end << 32 | lower end) of the chunk piece that may hold the last refusing slot
  u32 found, q;               // a refusing slot was found; its doubled coordinate
  u32 njobs, pad;
  u64 n_moved, slots;
};

__global__ __launch_bounds__(LB) void k_eager(const g10_migration* __restrict__ rec, const uint2* __restrict__ rec_ab,
                                             const u32* __restrict__ order, u32 n, u64* __restrict__ E, u32 K, u32 nch,
                                             u32 spt, u32 shift_ch, u64 cap, u32* __restrict__ gained,
                                             u32* __restrict__ last, u64* __restrict__ stats) {
  extern __shared__ __align__(16) unsigned char smem[];
  u64* cmax = (u64*)smem;                          // [nch] largest pressure of the chunk (lazy add included)
  u64* ladd = cmax + nch;                          // [nch] added to every slot of the chunk, not yet in E
  PfShared* S = (PfShared*)(ladd + nch);
  u32* jobs = (u32*)(S + 1);                       // [nch] chunks to rewrite slot by slot
  const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6, CH = 1u << shift_ch;

  for (u32 c = wave; c < nch; c += LW) {           // chunk maxima
    u64 m = 0;
    for (u32 st = 0; st < spt; ++st) {
      const u32 j0 = c * CH + st * 256u + lane * 4u;
#pragma unroll
      for (u32 i = 0; i < 4; ++i) if (j0 + i < K) { const u64 x = E[j0 + i]; m = x > m ? x : m; }
    }
    m = wave_max(m);
    if (lane == 0) { cmax[c] = m; ladd[c] = 0; }
  }
  if (tid == 0) { S->n_moved = 0; S->slots = 0; }
  __syncthreads();

  // the next record is fetched while the current one is worked on
  u32 r_next = n ? order[0] : 0u;
  u64 s_next = n ? rec[r_next].size_bytes : 0ull;
  uint2 ab_next = n ? rec_ab[r_next] : make_uint2(0u, 0u);
  for (u32 it = 0; it < n; ++it) {
    const u32 r = r_next;
    const u64 s = s_next;
    const u32 a = ab_next.x, b = ab_next.y;
    if (it + 1 < n) { r_next = order[it + 1]; s_next = rec[r_next].size_bytes; ab_next = rec_ab[r_next]; }
    u32 p = b + 1;                                 // first slot the tensor is back in
    // the slot just before the prefetch decides most cases: if it cannot take the tensor, nothing moves
    const u32 bb = b >= K ? b - K : b;
    if (s <= cap && E[bb] + ladd[bb >> shift_ch] <= cap - s) {
      const u64 lim = cap - s;                     // a slot holds the tensor iff its pressure <= lim
      u32 upper = b;                               // the search is still open over [a, upper]
      p = a;
      while (true) {
        if (tid == 0) { S->cand = 0ull; S->found = 0; }
        __syncthreads();
        if (tid < nch && cmax[tid] > lim) {        // the two places of the chunk on the doubled timeline
          const u64 s0 = (u64)tid * CH, s1 = (s0 + CH - 1 < (u64)K - 1) ? s0 + CH - 1 : (u64)K - 1;
#pragma unroll
          for (u32 rep = 0; rep < 2; ++rep) {
            const u64 o = rep ? K : 0u;
            const u64 plo = s0 + o > a ? s0 + o : a, phi = s1 + o < upper ? s1 + o : upper;
            if (plo <= phi) atomicMax(&S->cand, (unsigned long long)(((phi + 1) << 32) | plo));
          }
        }
        __syncthreads();
        const unsigned long long cd = S->cand;
        if (cd == 0ull) break;                     // no chunk holds a refusing slot inside [a, upper]
        const u32 hi = (u32)(cd >> 32) - 1u, lo = (u32)cd;
        if (wave == 0) {                           // the last refusing slot of the piece, if any
          u32 best = 0;                            // doubled coordinate + 1
          for (u32 j0 = lo; j0 <= hi; j0 += 64) {
            const u32 j = j0 + lane;
            if (j <= hi) {
              const u32 jj = j >= K ? j - K : j;
              if (E[jj] + ladd[jj >> shift_ch] > lim) best = j + 1;      // ascending: the last one stays
            }
          }
          best = wave_max(best);
          if (lane == 0 && best) { S->found = 1; S->q = best - 1; }
        }
        __syncthreads();
        if (S->found) { p = S->q + 1; break; }
        if (lo == a) break;                        // nothing refuses in [a, upper]
        upper = lo - 1;
        __syncthreads();
      }
    }
    __syncthreads();
    const u32 g = b + 1 - p;
    if (tid == 0) {
      gained[r] = g;
      const u32 nl = b - g;                        // last absent slot left (one before a if none)
      last[r] = nl >= K ? nl - K : nl;
      if (g) { S->n_moved += 1; S->slots += g; }
      S->njobs = 0;
    }
    __syncthreads();
    if (g) {                                       // the slots gained take the tensor
      if (tid < nch) {
        u32 len;
        const u32 cv = cover(tid, CH, K, p, b, len);
        if (cv == len) { ladd[tid] += s; cmax[tid] += s; }
        else if (cv) jobs[atomicAdd(&S->njobs, 1u)] = tid;
      }
      __syncthreads();
      const u32 nj = S->njobs;
      for (u32 jb = wave; jb < nj; jb += LW) {
        const u32 c = jobs[jb];
        const u64 lz = ladd[c];
        u64 m = 0;
        for (u32 st = 0; st < spt; ++st) {
          const u32 j0 = c * CH + st * 256u + lane * 4u;
#pragma unroll
          for (u32 i = 0; i < 4; ++i) {
            const u32 j = j0 + i;
            if (j < K) {
              u64 x = E[j];
              if (in_doubled(j, K, p, b) != NONE32) { x += s; E[j] = x; }
              x += lz;
              m = x > m ? x : m;
            }
          }
        }
        m = wave_max(m);
        if (lane == 0) cmax[c] = m;
      }
      __syncthreads();
    }
  }
  // the lazy adds into the slots; the peak
  u64 m = 0;
  for (u32 j = tid; j < K; j += LB) { const u64 x = E[j] + ladd[j >> shift_ch]; E[j] = x; m = x > m ? x : m; }
  m = wave_max(m);
  if (lane == 0) atomicMax((unsigned long long*)&stats[2], (unsigned long long)m);
  if (tid == 0) { stats[0] = S->n_moved; stats[1] = S->slots; }
}

}  // namespace

int prefetch_run(g10_plan_s* h, g10_prefetch_result* out) {
  PlanWork* w = h->work;
  if (!w || !w->planned) return G10_EINVAL;
  hipStream_t s = h->stream;
  const u32 K = h->K, n = (u32)w->plan_n_mig;
  if (!w->h_pf_order) {
    const u64 C = w->C ? w->C : 1;
    w->h_pf_order = (u32*)malloc(C * 4); w->h_pf_gained = (u32*)malloc(C * 4); w->h_pf_last = (u32*)malloc(C * 4);
    w->h_pf_pressure = (u64*)malloc((u64)K * 8);
    if (!w->h_pf_order || !w->h_pf_gained || !w->h_pf_last || !w->h_pf_pressure) return G10_ENOMEM;
  }
  G10_HIP(hipEventRecord(w->ev[0], s));
  G10_HIP(hipMemcpyAsync(w->pf_pressure, w->pressure_after, (u64)K * 8, hipMemcpyDeviceToDevice, s));
  G10_HIP(hipMemsetAsync(w->pf_stats, 0, 4 * 8, s));
  u64* keys = w->pf_keys; u64* alt = w->pf_keys_alt;
  u32* ord = w->pf_order; u32* oalt = w->pf_order_alt;
  if (n) {
    hipLaunchKernelGGL(k_pf_keys, dim3((n + G10_BLOCK - 1) / G10_BLOCK), dim3(G10_BLOCK), 0, s, (const g10_migration*)w->records, n,
                       (const u64*)h->start, K, h->T, keys, ord);
    G10_HIP(hipGetLastError());
    G10_TRY(radix_sort_u64_pairs(&keys, &alt, &ord, &oalt, n, bits_for(2 * h->T), w->hist, w->scratch32, s));
  }
  const size_t lds = ((size_t)2 * w->nch * 8 + sizeof(PfShared) + (size_t)w->nch * 4 + 15) & ~(size_t)15;
  hipLaunchKernelGGL(k_eager, dim3(1), dim3(LB), lds, s, (const g10_migration*)w->records, (const uint2*)w->rec_ab,
                     (const u32*)ord, n, w->pf_pressure, K, w->nch, w->spt, w->shift_ch, w->plan_cap, w->pf_gained, w->pf_last,
                     w->pf_stats);
  G10_HIP(hipGetLastError());
  u64 st[4] = {0, 0, 0, 0};
  G10_HIP(hipMemcpyAsync(st, w->pf_stats, sizeof st, hipMemcpyDeviceToHost, s));
  if (n) {
    G10_HIP(hipMemcpyAsync(w->h_pf_order, ord, (u64)n * 4, hipMemcpyDeviceToHost, s));
    G10_HIP(hipMemcpyAsync(w->h_pf_gained, w->pf_gained, (u64)n * 4, hipMemcpyDeviceToHost, s));
    G10_HIP(hipMemcpyAsync(w->h_pf_last, w->pf_last, (u64)n * 4, hipMemcpyDeviceToHost, s));
  }
  G10_HIP(hipMemcpyAsync(w->h_pf_pressure, w->pf_pressure, (u64)K * 8, hipMemcpyDeviceToHost, s));
  G10_HIP(hipEventRecord(w->ev[1], s));
  G10_HIP(hipStreamSynchronize(s));
  float ms = 0.f;
  G10_HIP(hipEventElapsedTime(&ms, w->ev[0], w->ev[1]));
  memset(out, 0, sizeof *out);
  out->n_migrations = n; out->n_moved = st[0]; out->slots_gained = st[1]; out->peak_bytes = st[2];
  out->order = w->h_pf_order; out->gained = w->h_pf_gained; out->absent_last = w->h_pf_last; out->pressure = w->h_pf_pressure;
  out->ms = ms;
  return G10_OK;
}
