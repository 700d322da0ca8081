// Definitions shared by the planning translation units (gfx950): constants, the control
// block, candidate and timeline views, the 128-bit helpers, the score of one candidate, and
// the per-plan workspaces.  Device functions are inline; kernels live in the .hip files.
#pragma once

#include "g10_internal.h"

#include <hip/hip_runtime.h>


namespace g10 {

enum { A_OT = 0, A_FO = 1, A_FI = 3, N_ARR = 5, PX = 8 };
enum { J_P = 0, J_FO0 = 2, J_FO1 = 3, J_FI0 = 4, J_FI1 = 5, J_HQ = 6, J_CLIP = 7 };   // kinds of chunk jobs

constexpr u32 LB = 512;                // threads of the loop workgroup (at least NCH_MAX)
constexpr u32 LW = LB / G10_WAVE;      // its wavefronts
constexpr u32 UNIT = 256;              // candidates scored by four wavefronts at a time
constexpr u32 NCH_MAX = 512;           // chunks (level-1 arrays live in LDS)
constexpr u32 NT_MAX = 8192;           // tiles  (their bounds live in LDS)
constexpr u32 GUESS_SHIFT = 7;                 // first threshold of a pass: last benefit * (1 - 2^-shift), to begin with
constexpr u32 GUESS_SHIFT_MAX = 24;            // the keys resolve no finer steps
constexpr u64 NONE64 = ~0ull;
constexpr u32 NONE32 = 0xffffffffu;

__device__ __forceinline__ u32 w_fo(u32 d) { return 2 * d; }          // word of FOd in a slot record (OT follows)
__device__ __forceinline__ u32 w_fi(u32 d) { return 4 + 2 * d; }      // word of FId (OT follows)

struct Ctl {
  // parameters
  u64 gpu_cap, host_cap, bw_out[2], bw_in[2], max_iter;
  u32 rank, area;             // G10_RANK_BENEFIT / G10_RANK_RATIO; G10_AREA_BAND / G10_AREA_CLIPPED
  u64 inv_out[2], inv_in[2];  // floor(2^64 / bandwidth), 0 for bandwidth 1
  u64 C;                      // all inactive periods (live before any removal)
  u64 smax;                   // the largest tensor of the trace
  // progress
  u32 done, status;
  u64 n_iter, n_mig, n_drop, n_evals;
  u64 overtime_before, overtime_after;
  u32 thr_key;                // first threshold of the next pass (0: use the largest tile bound)
  u32 n_live;                 // candidates that could still score at the last re-scoring
  u32 gshift, pad1;           // the guess: first threshold = last best * (1 - 2^-gshift); 0 stands for GUESS_SHIFT
  // statistics
  u64 units_scored, second_rounds, jobs_run, launches, passes;
  u64 area_evals, area_refused;   // clipped areas computed in the loop; of those, how many came out below the bound
  u64 wide_rounds;                // scoring rounds left to the scoring kernel
  u64 more_rounds;                // rounds of commits after the first of their ranking pass
  u64 list_rescored;              // list entries scored again for those rounds
};

struct Cands {
  uint4* A;                   // {L1, R, a0, b0}     a > b: no valid window for that destination
  uint4* B;                   // {a1, b1, size lo, size hi}
  uint2* id;                  // {index of the period in the analysis order (the tie-break), tensor}
  // Only for the clipped-area benefit (else null): the last exact value of the candidate, an
  // upper bound of every later one since the pressure only falls.
  uint4* cv;                  // the value, 128 bits, least significant word first
  uint2* ce;                  // {pass in which it was computed, bit 0: there is a value, bit 1: its destination}
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
// ranking by benefit / cost (the alternative key of Section 4.3): exact comparison of the
// fractions by cross multiplication; 31-bit keys from a double approximation with a margin,
// one that is never below the key of the true ratio and one that is never above it
// ---------------------------------------------------------------------------
struct U192 { u64 w2, w1, w0; };
__device__ __forceinline__ U192 mul_128_64(u64 hi, u64 lo, u64 y) {
  U192 r;
  r.w0 = lo * y;
  const u64 c0 = __umul64hi(lo, y), m = hi * y;
  r.w1 = m + c0;
  r.w2 = __umul64hi(hi, y) + (r.w1 < m ? 1ull : 0ull);
  return r;
}
// sign of  B1 / c1 - B2 / c2  (costs > 0)
__device__ __forceinline__ int cmp_ratio(u64 h1, u64 l1, u64 c1, u64 h2, u64 l2, u64 c2) {
  const U192 p = mul_128_64(h1, l1, c2), q = mul_128_64(h2, l2, c1);
  if (p.w2 != q.w2) return p.w2 > q.w2 ? 1 : -1;
  if (p.w1 != q.w1) return p.w1 > q.w1 ? 1 : -1;
  if (p.w0 != q.w0) return p.w0 > q.w0 ? 1 : -1;
  return 0;
}
// B / cost to a relative error far below 2^-40 (five roundings of 2^-53 each)
__device__ __forceinline__ double ratio_approx(u64 hi, u64 lo, u64 cost) {
  return __fma_rn((double)hi, 18446744073709551616.0, (double)lo) / (double)cost;
}
// floor key of a positive double: 7 bits of exponent (values from 2^-20 up; 0 below), 24 bits
// of mantissa; monotone non-decreasing
__device__ __forceinline__ u32 rkey_floor(double r) {
  const long long bits = __double_as_longlong(r);
  const int e = (int)(bits >> 52) - 1023 + 21;
  if (e < 1) return 0u;
  if (e > 126) return (126u << 24) | 0xffffffu;
  return ((u32)e << 24) | (u32)((bits >> 28) & 0xffffffll);
}
// never below the floor key of the true ratio, and at least 1: the bound side
__device__ __forceinline__ u32 rkey_up(double r) { return rkey_floor(r * (1.0 + 0x1p-40)) + 1u; }
// never above the floor key of the true ratio: the side of the best candidate found
__device__ __forceinline__ u32 rkey_dn(double r) { return rkey_floor(r * (1.0 - 0x1p-40)); }

// the ranking key of a benefit (and, for the ratio, the cost that divides it)
template <bool RATIO>
__device__ __forceinline__ u32 key_up_of(u64 hi, u64 lo, u64 cost) {
  if (!RATIO) return upkey(hi, lo);
  return (hi | lo) ? rkey_up(ratio_approx(hi, lo, cost)) : 0u;
}
template <bool RATIO>
__device__ __forceinline__ u32 key_dn_of(u64 hi, u64 lo, u64 cost) {
  if (!RATIO) return upkey(hi, lo);
  return (hi | lo) ? rkey_dn(ratio_approx(hi, lo, cost)) : 0u;
}

// ---------------------------------------------------------------------------
// score of one candidate against the current timelines
// ---------------------------------------------------------------------------
struct Machine {
  u64 bwo0, bwo1, bwi0, bwi1;
  u64 ivo0, ivo1, ivi0, ivi1;  // reciprocals (only the ratio ranking needs every candidate's transfer times)
};

// eviction + prefetch time of a tensor per destination
__device__ __forceinline__ void costs_of(const Machine& mc, u64 s, u64& c0, u64& c1) {
  c0 = ceil_div_x1000(s, mc.bwo0, mc.ivo0) + ceil_div_x1000(s, mc.bwi0, mc.ivi0);
  c1 = ceil_div_x1000(s, mc.bwo1, mc.ivo1) + ceil_div_x1000(s, mc.bwi1, mc.ivi1);
}

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

// ---------------------------------------------------------------------------
// the greedy loop
// ---------------------------------------------------------------------------
struct LoopArgs {
  Cands cd;
  u32 n_pad, nt, tshift;      // tile = UNIT << tshift candidates
  Timelines tl;
  u64 *g_tot, *g_lazyP, *g_minOver, *g_lazyH, *g_hmax, *g_base;
  u32 *g_hmat, *g_hpend;      // host occupancy is brought up to date chunk by chunk, on demand: records applied so far; some may be missing
  u32* g_keys;
  Ctl* ctl;
  g10_migration* records;
  uint2* rec_ab;              // absent window [a, b] of every migration in doubled coordinates
  uint4* rec_h;               // {L + 1, R, size} of every migration to host in doubled coordinates (size 0: to flash)
  g10_dropped* dropped;
  u32 pass_budget;            // the launch ends after this many passes,
  u64 tick_budget;            // or (if not 0) after this many ticks of the 100 MHz wall clock,
  u64 pass_stop;              // or (if not 0) once the plan has made this many passes over all its launches
  // Scoring rounds left to all compute units (ranking by benefit / cost, band reading; else null):
  // the block of loop_wide_bytes() bytes the loop kernel and the scoring kernel talk through, and
  // the length of a round's list, in units of 256 candidates, from which it is left to that kernel
  void* wide;
  u32 wide_min;
  u32 wide_last_seq;          // the launch of the loop kernel (counted from 1 over the plan) behind which no scoring kernel is queued
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
// the same for benefit / cost; "nothing yet" is benefit 0 with cost 1
__device__ __forceinline__ bool better_ratio(u64 hi, u64 lo, u64 cost, u32 cand, u64 bhi, u64 blo, u64 bcost, u32 bcand) {
  const int c = cmp_ratio(hi, lo, cost, bhi, blo, bcost);
  return c ? c > 0 : cand < bcand;
}

// covered slots of chunk c by the doubled range [x, y] (x <= y, y - x < K): the chunk's slots
// appear at [s0, s1] and at [s0 + K, s1 + K] in doubled coordinates
__device__ __forceinline__ u32 cover(u32 c, u32 ch, u32 K, u32 x, u32 y, u32& len) {
  // (all coordinates are below 2 K < 2^32, so 32-bit arithmetic does; an empty range, y = x - 1, covers nothing)
  const u32 s0 = c * ch, s1 = s0 + ch - 1 < K - 1 ? s0 + ch - 1 : K - 1;
  len = s1 - s0 + 1;
  u32 lo = s0 > x ? s0 : x, hi = s1 < y ? s1 : y;
  u32 n = hi >= lo ? hi - lo + 1 : 0u;
  lo = s0 + K > x ? s0 + K : x; hi = s1 + K < y ? s1 + K : y;
  n += hi >= lo ? hi - lo + 1 : 0u;
  return n;
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

inline u32 bits_for(u64 max_value) {            // bits needed to hold values 0..max_value, at least 1
  u32 b = 1;
  while (b < 64 && (max_value >> b)) ++b;
  return b;
}

}  // namespace g10

struct PlanWork {
  u32 K = 0, Kp = 0, nch = 0, spt = 1, shift_ch = 8;
  u64 C = 0, cap_pad = 0;
  uint4* win = nullptr;
  uint4* fw = nullptr;          // the kept candidates' windows {a0, b0, a1, b1} and sizes on their own, for the first scoring pass
  u64* fs = nullptr;
  u32 *keep = nullptr, *scratch32 = nullptr, *hist = nullptr, *tkeys = nullptr;
  u32 *keys = nullptr, *keys_alt = nullptr;   // the keys of the score sort
  u32 *sv = nullptr, *sv_alt = nullptr;   // the values of the score sort: old positions
  g10::Cands cd[2] = {};
  u64 *P = nullptr, *fre = nullptr, *H = nullptr, *px = nullptr, *otc = nullptr, *base0 = nullptr, *g_tot = nullptr,
      *g_lazyP = nullptr, *g_minOver = nullptr, *g_lazyH = nullptr, *g_hmax = nullptr, *g_base = nullptr,
      *pressure_after = nullptr,
      *peak_after = nullptr;
  // kernel durations, slot start times and iteration time this plan runs on: the analysed trace's, or
  // the plan's own (dur_own, start_own) when the parameters bring durations of their own
  const u64 *dur = nullptr, *start = nullptr;
  u64 T = 0;
  u64 *dur_own = nullptr, *start_own = nullptr, *times_scratch = nullptr, *times_stats = nullptr;
  char* wide = nullptr;        // what the loop kernel and the scoring kernel talk through (loop_wide_bytes())
  g10::Ctl* ctl = nullptr;
  g10_migration* records = nullptr;
  uint2* rec_ab = nullptr;
  uint4* rec_h = nullptr;      // {L + 1, R, size} of every migration to host (size 0: to flash)
  u32 *g_hmat = nullptr, *g_hpend = nullptr;   // per chunk: records applied to the host occupancy; some may be missing
  g10_dropped* dropped = nullptr;
  // smart prefetching
  u64 *pf_keys = nullptr, *pf_keys_alt = nullptr, *pf_pressure = nullptr, *pf_stats = nullptr;
  u32 *pf_order = nullptr, *pf_order_alt = nullptr, *pf_gained = nullptr, *pf_last = nullptr;
  u32 *h_pf_order = nullptr, *h_pf_gained = nullptr, *h_pf_last = nullptr;
  u64* h_pf_pressure = nullptr;
  bool planned = false;         // a plan is stored in the handle
  bool prefetched = false;      // smart prefetching has run on that plan (pf_gained is valid)
  u64 plan_cap = 0, plan_n_mig = 0;
  // host copies handed out through g10_result
  int device = 0;              // the GPU the workspaces and events belong to
  void* h_block = nullptr;     // pinned host memory of the three result arrays below
  size_t h_block_bytes = 0;
  g10_migration* h_records = nullptr;
  g10_dropped* h_dropped = nullptr;
  u64* h_pressure = nullptr;
  hipEvent_t ev[6] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
  // plan replay: a device allocation of its own, made at the first replay and sized for the plan's migrations
  void* rp_arena = nullptr;
  u32 rp_cap = 0;
  u64 *rp_keys = nullptr, *rp_alt = nullptr, *rp_res = nullptr, *rp_late = nullptr, *rp_dur = nullptr, *rp_start = nullptr,
      *rp_tscr = nullptr;
  u32 *rp_pos = nullptr, *rp_hist = nullptr, *rp_scr = nullptr;
  void *rp_stats = nullptr, *rp_tstats = nullptr;
  u64* h_rp_late = nullptr;
  void* arena = nullptr;        // the one device allocation all pointers above point into
  u32 max_chunks = 0;           // the chunk limit the timelines were laid out for
  bool has_cache = false;       // the candidate buffers have the cv / ce arrays
};

// plan replay (g10_replay.hip)
void replay_free(PlanWork* w);

// the loop kernel (g10_loop.hip)
size_t loop_lds_bytes(u32 nch, u32 nt);                       // dynamic LDS of one workgroup
int loop_allow_large_lds();                                   // more than 64 KB of LDS for the kernel
size_t loop_wide_bytes();                                     // device memory a plan's loop and the scoring kernel talk through
int loop_wide_launch(const g10::LoopArgs* plans, u32 nch, hipStream_t s);   // the scoring kernel for plans[0]
int loop_launch(const g10::LoopArgs* plans, u32 n_plans, size_t lds, u32 rank, u32 area, hipStream_t s);   // all of one ranking key and benefit reading
