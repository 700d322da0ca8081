// The greedy loop of smart tensor eviction (G10, Section 4.3, Algorithm 1) as one persistent
// workgroup per plan: rank (tile bounds, score, arg-max), decide, commit (lazy chunk adds and
// chunk jobs), level-1 update.  See g10_plan.hip for the data structures and why the plan is
// the one Algorithm 1 makes.

#include "g10_plan_defs.h"

using namespace g10;

namespace {

struct Winner {               // what a commit needs of the winning candidate
  u64 hi, lo;                 // benefit
  u64 cost;                   // eviction + prefetch time (ranking by benefit / cost only)
  u64 s, fo_base, fi_end;     // size; free out-channel time before L1; free in-channel time before R
  u64 tau_o, tau_i;           // eviction and prefetch time to the destination
  u32 cand, tensor, pos, dest, L1, R, a, b;
  u32 exact;                  // clipped-area benefit only: the value was computed in this pass (else it is a bound)
  u32 kU;                     // key of the larger of the two destinations' benefits: bounds every later benefit
  u32 kr;                     // kU if the policy sends the candidate to flash while host could take it too (a flash
                              // reservation in its transfer windows would move it to host, where its benefit may be
                              // larger), else 0
  u32 pad;
};

// Ranking by benefit / cost keeps a bound per candidate that holds whichever destination the
// policy ends up with: most of a long list then reaches the threshold of every pass and has to
// be scored again.  Such a round is left to all compute units: the loop kernel writes the list
// of tiles to score, ends in the middle of its pass, a scoring kernel takes the list (the tile
// bounds go into the array of tile bounds in device memory, every workgroup's best candidate
// into `win`), and the next launch of the loop kernel takes the pass up again with those.
constexpr u32 WIDE_WG = 2 * (LB - 1);   // workgroups of the scoring kernel that take part at most: two winners per thread of the
                                        // loop kernel, whose last thread takes the best of the pass's earlier rounds
struct WideCtx {
  u32 pending;                // the loop kernel has left a list and waits for it to be scored
  u32 nwg, done_wgs;          // workgroups of the scoring kernel that take part; that have finished
  u32 ntl, thr, rest;         // of the round left open: tiles on the list, its threshold, bound of the tiles not on it
  u32 rounds, pass_units;     // of the pass left open: rounds finished, units scored in them
  u32 seq, pad[3];            // launches of the loop kernel on this plan so far
};
struct WideView {
  WideCtx* ctx;
  Winner* win;                // [WIDE_WG], then the best of the earlier rounds
  u64* smark;                 // [NT_MAX / 64]  tiles scored in the pass left open
  unsigned short* alist;      // [NT_MAX]       the list
};
constexpr size_t WIDE_BYTES = sizeof(WideCtx) + (WIDE_WG + 1) * sizeof(Winner) + (NT_MAX / 64) * 8 + (size_t)NT_MAX * 2;
__host__ __device__ __forceinline__ WideView wide_view(void* blob) {
  WideView v;
  char* q = (char*)blob;
  v.ctx = (WideCtx*)q; q += sizeof(WideCtx);
  v.win = (Winner*)q; q += (WIDE_WG + 1) * sizeof(Winner);
  v.smark = (u64*)q; q += (NT_MAX / 64) * 8;
  v.alist = (unsigned short*)q;
  return v;
}
static_assert(sizeof(WideCtx) % 16 == 0 && sizeof(Winner) % 8 == 0, "the arrays of the scoring kernel's block stay aligned");

constexpr u32 MAXM = 16;      // migrations committed in one ranking pass at most (a multiple of 8, at most 16: the job words hold two sets of 16)
static_assert(MAXM % 8 == 0 && MAXM <= 16, "job words and chunk flags are laid out for 8 or 16");

constexpr u32 MC_GUESS_SHIFT_MIN = 4;   // the widest margin of a pass's first threshold under the last benefit: 2^-this
constexpr u32 LIST_MAX = 64;  // candidates of a pass that are looked at for the second and later migrations

struct Shared {               // small per-pass state of the loop workgroup
  Winner mem[MAXM];           // migrations of the pass in commit order; [0] is the winner of the ranking (hi = lo = 0: none)
  Winner wave_win[LW];        // best of every wavefront
  Winner list[LIST_MAX];      // the other candidates whose bound exceeds every bound not looked at one by one
  u32 wave_f2[LW];            // per wavefront: largest bound among the candidates its threads scored but do not hold
  u32 F2, pad0;               // ... over the workgroup
  u32 nlist, m0, cut, need_exact;   // list length; migrations selected; how many of them may be committed; the winner's
                              // host-capacity test needs the exact per-slot maximum
  u32 by_floor, touched;      // the selection ended because the next candidate did not clear the floor; timelines (a bit
                              // per array of level 1) whose chunk totals change in this pass
  u32 Fkeep, more;            // the floor of the pass; another round of commits follows from the same list
  u64 more_rounds, list_rescored;   // such rounds made; list entries scored again for them (statistics)
  u32 sel[MAXM];              // list entries picked, in order
  u64 hq;                     // host-capacity query: maximum over the period
  u64 acc[3];                 // clipped area being summed: bits 0..31, 32..63 and 64.. of the terms, added apart
  u64 evals, refused;         // clipped areas computed; of those, how many came out below the bound
  u32 nl, restL;              // hot list: length; bound of the tiles outside it
  u32 ntl, filt;              // current round: tiles to score; bound of the hot tiles left out
  u32 njobs, ot_changed, stale_hot;
  u32 no_wide;                // this launch may not leave a round to the scoring kernel (none is queued behind it)
  // progress (mirrors Ctl)
  u64 n_iter, n_mig, n_drop, n_evals, units, second, jobs;
  u32 thr_key, status, done, stop;
  u32 gshift, pad2;
  u64 t_start;
};

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

__device__ __forceinline__ u64 read_lane64(u64 v, u32 l) {
  const u32 lo = (u32)__builtin_amdgcn_readlane((int)(u32)v, (int)l), hi = (u32)__builtin_amdgcn_readlane((int)(u32)(v >> 32), (int)l);
  return ((u64)hi << 32) | lo;
}

// The same for benefit / cost.  The approximate keys only narrow the field: a lane stays if
// its upper key reaches the largest lower key.  The lanes that stay are settled exactly: take
// the first, keep the lanes that beat it (fractions compared by cross multiplication, equal
// ones by index), repeat with the first of those.
__device__ __forceinline__ u32 wave_best_lane_ratio(u64 hi, u64 lo, u64 cost, u32 cand) {
  const bool has = (hi | lo) != 0;
  const double r = has ? ratio_approx(hi, lo, cost) : 0.0;
  const u32 kdn_max = wave_max(has ? rkey_dn(r) : 0u);
  u64 m = __ballot(has && rkey_up(r) >= kdn_max);
  if (!m) return NONE32;
  const u32 lane = lane_id();
  u32 p = (u32)__builtin_ctzll(m);
  while (m & (m - 1)) {
    const u64 ph = read_lane64(hi, p), pl = read_lane64(lo, p), pc = read_lane64(cost, p);
    const u32 pcand = (u32)__builtin_amdgcn_readlane((int)cand, (int)p);
    const bool beats = ((m >> lane) & 1ull) && lane != p && better_ratio(hi, lo, cost, cand, ph, pl, pc, pcand);
    m = __ballot(beats);
    if (!m) break;
    p = (u32)__builtin_ctzll(m);
  }
  return p;
}

// Do the doubled slot ranges [x1, y1] and [x2, y2] (each shorter than K) share a kernel slot?  (K < 2^30)
__device__ __forceinline__ bool cyc_overlap32(u32 x1, u32 y1, u32 x2, u32 y2, u32 K) {
  return (x1 <= y2 && x2 <= y1) || (x1 + K <= y2 && x2 <= y1 + K) || (x1 <= y2 + K && x2 + K <= y1);
}

template <bool RATIO>
__device__ __forceinline__ u32 best_lane(u64 hi, u64 lo, u64 cost, u32 cand) {
  if (RATIO) return wave_best_lane_ratio(hi, lo, cost, cand);
  return wave_best_lane(hi, lo, cand);
}

template <bool RATIO, bool CLIP>
__global__ __launch_bounds__(LB) void k_loop(const LoopArgs* __restrict__ plans) {
  // Several migrations per ranking pass (ranking by the benefit itself, band reading): after the
  // winner, the next best candidates of the same pass are committed with it as long as it is
  // certain that each would have won the pass after the one before it - see "more migrations
  // of the same pass" below.
  constexpr bool MC = !RATIO && !CLIP;
  constexpr bool WIDE = RATIO && !CLIP;        // long scoring rounds may be left to the scoring kernel (see WideCtx)
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
  u64* jobs = scr + 4 * LW;                             // [8 * nch + 8]  chunk | kind << 16 | a set of the pass's migrations << 24 | another << 40
  Shared* S = (Shared*)(jobs + 8 * nch + 8);
  u32* keys = (u32*)(S + 1);                            // [nt]  bound of every tile
  u32* skeys = keys + nt;                               // [ns]  largest bound of every group of 64 tiles
  u32* hmat = skeys + ns;                               // [nch] host occupancy: migrations (by index) already added to the chunk's slots
  u32* hpend = hmat + nch;                              // [nch] ... and whether a later one that cuts the chunk is still missing
  unsigned short* tlist = (unsigned short*)(hpend + nch);  // [nt]  the hot list
  unsigned short* alist = tlist + nt;                            // [nt]  tiles scored in the current round

  const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  Ctl* ctl = a.ctl;
  // A pass left open by the last launch: its list has been scored by the scoring kernel (1), or
  // has not (2: it is scored here).  Launches are queued ahead of what is known of the plan's
  // progress; one that finds nothing to do ends at once.
  WideView wv = {};
  u32 resume = 0;
  if (tid == 0) S->no_wide = 0;
  if (WIDE && a.wide) {
    wv = wide_view(a.wide);
    if (wv.ctx->pending) resume = (wv.ctx->nwg && wv.ctx->done_wgs == wv.ctx->nwg) ? 1u : 2u;
    if (tid == 0) {                                  // (read by everyone after the barrier that ends "state in")
      const u32 seq = wv.ctx->seq + 1;
      wv.ctx->seq = seq;
      S->no_wide = seq == a.wide_last_seq ? 1u : 0u;
    }
    if (!resume && (ctl->done || (a.pass_stop && ctl->passes >= a.pass_stop))) return;
  }
  const u64 passes_before = ctl->passes;
  const u64 cap = ctl->gpu_cap, host_cap = ctl->host_cap, max_iter = ctl->max_iter, C = ctl->C;
  const u64 bwo0 = ctl->bw_out[0], bwo1 = ctl->bw_out[1], bwi0 = ctl->bw_in[0], bwi1 = ctl->bw_in[1];
  const u64 ivo0 = ctl->inv_out[0], ivo1 = ctl->inv_out[1], ivi0 = ctl->inv_in[0], ivi1 = ctl->inv_in[1];

  // ---- state in ----------------------------------------------------------------------
  for (u32 i = tid; i < N_ARR * nch; i += LB) tot[i] = a.g_tot[i];
  for (u32 i = tid; i < nch; i += LB) { lazyP[i] = a.g_lazyP[i]; minOver[i] = a.g_minOver[i]; lazyH[i] = a.g_lazyH[i]; hmax[i] = a.g_hmax[i]; hmat[i] = a.g_hmat[i]; hpend[i] = a.g_hpend[i]; }
  for (u32 i = tid; i < nt; i += LB) keys[i] = a.g_keys[i];
  for (u32 i = tid; i < ns; i += LB) smark[i] = 0;
  if (tid == 0) {
    S->n_iter = ctl->n_iter; S->n_mig = ctl->n_mig; S->n_drop = ctl->n_drop; S->n_evals = ctl->n_evals;
    S->units = 0; S->second = 0; S->jobs = 0; S->evals = 0; S->refused = 0; S->more_rounds = 0; S->more = 0; S->list_rescored = 0;
    S->thr_key = ctl->thr_key; S->status = ctl->status; S->done = ctl->done;
    S->gshift = ctl->gshift ? ctl->gshift : GUESS_SHIFT;
    S->nl = 0; S->restL = NONE32; S->stale_hot = 0;
    S->stop = 0; S->t_start = wall_clock64();
    S->mem[0].hi = 0; S->mem[0].lo = 0;
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

  u32 pass_units = 0;           // units of 256 candidates scored in the current pass (the same in every thread)
  // this thread's best candidate of the pass
  Winner mine;
  mine.hi = 0; mine.lo = 0; mine.cost = 1; mine.cand = NONE32; mine.exact = 0; mine.kU = 0; mine.kr = 0; mine.tau_o = 0; mine.tau_i = 0; mine.pad = 0;
  u32 floor2 = 0;               // largest bound among the candidates this thread scored in the pass other than `mine`
  u32 cur_iter = 0;             // number of the current pass (the stamp of the values computed in it)

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
  auto score_list = [&](const u32 thr_pub) {
    const u32 nunits = S->ntl << a.tshift;
    PrefixView pv; pv.px = tl.px; pv.base = base; pv.K = K; pv.nch = nch; pv.shift_ch = tl.shift_ch;
    Machine mc; mc.bwo0 = bwo0; mc.bwo1 = bwo1; mc.bwi0 = bwi0; mc.bwi1 = bwi1;
    mc.ivo0 = ivo0; mc.ivo1 = ivo1; mc.ivi0 = ivi0; mc.ivi1 = ivi1;
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
      u32 exact = 0;
      Score rr = r;
      if (CLIP && (rr.ok0 || rr.ok1)) {          // the band bounds the area; a value computed earlier bounds it closer
        const uint2 e = a.cd.ce[cur.p];
        if (e.y & 1u) {
          const uint4 v = a.cd.cv[cur.p];
          const u64 vlo = ((u64)v.y << 32) | v.x, vhi = ((u64)v.w << 32) | v.z;
          const u32 vd = (e.y >> 1) & 1u, pd = rr.ok0 ? 0u : 1u;
          if (vd == 0u && rr.ok0 && gt128(rr.h0, rr.l0, vhi, vlo)) { rr.h0 = vhi; rr.l0 = vlo; }
          if (vd == 1u && rr.ok1 && gt128(rr.h1, rr.l1, vhi, vlo)) { rr.h1 = vhi; rr.l1 = vlo; }
          exact = (vd == pd && e.x == cur_iter) ? 1u : 0u;
        }
      }
      u64 c0 = 1, c1 = 1;
      u32 kc;                                    // bound of the candidate: the larger of its destinations' keys
      if (RATIO) {
        if (rr.ok0 || rr.ok1) costs_of(mc, ((u64)B.w << 32) | B.z, c0, c1);
        const u32 k0 = key_up_of<true>(rr.h0, rr.l0, c0), k1 = key_up_of<true>(rr.h1, rr.l1, c1);
        kc = k0 > k1 ? k0 : k1;
      } else {
        const bool one = gt128(rr.h1, rr.l1, rr.h0, rr.l0);
        kc = upkey(one ? rr.h1 : rr.h0, one ? rr.l1 : rr.l0);
      }
      const u32 k = wave_max(kc);
      if (lane == 0 && k) atomicMax(&keys[cur.t], k);
      // flash first; host only if flash cannot take it
      const bool ok_any = rr.ok0 || rr.ok1;
      const u32 d = rr.ok0 ? 0u : 1u;
      const u64 hi = ok_any ? (d ? rr.h1 : rr.h0) : 0ull, lo = ok_any ? (d ? rr.l1 : rr.l0) : 0ull, cost = d ? c1 : c0;
      if (MC) {
        // every candidate whose bound reaches the round's threshold goes on the list of the pass
        // with all a commit needs; the others count with their bound only (floor2)
        const bool pub = kc >= thr_pub && kc != 0u;
        const u64 pm = __ballot(pub);
        u32 slot = NONE32;
        if (pm) {
          const u32 leader = (u32)__builtin_ctzll(pm);
          u32 off = 0;
          if (lane == leader) off = atomicAdd(&S->nlist, (u32)__popcll(pm));
          off = (u32)__builtin_amdgcn_readlane((int)off, (int)leader);
          slot = off + (u32)__popcll(pm & ((1ull << lane) - 1ull));
        }
        if (pub && slot < LIST_MAX) {
          Winner& e = S->list[slot];
          e.hi = hi; e.lo = lo; e.cost = cost; e.cand = cur.id.x; e.tensor = cur.id.y; e.pos = cur.p; e.dest = d;
          e.L1 = A.x; e.R = A.y; e.a = d ? B.x : A.z; e.b = d ? B.y : A.w; e.s = ((u64)B.w << 32) | B.z;
          e.fo_base = rr.fo_L; e.fi_end = rr.fi_R; e.exact = 0; e.kU = kc; e.kr = (rr.ok0 && rr.ok1) ? kc : 0u;
        } else if (kc > floor2) floor2 = kc;
      }
      if ((hi | lo) != 0 && (RATIO ? better_ratio(hi, lo, cost, cur.id.x, mine.hi, mine.lo, mine.cost, mine.cand)
                                   : better(hi, lo, cur.id.x, mine.hi, mine.lo, mine.cand))) {
        mine.hi = hi; mine.lo = lo; mine.cost = cost; mine.cand = cur.id.x; mine.tensor = cur.id.y; mine.pos = cur.p; mine.dest = d;
        mine.L1 = A.x; mine.R = A.y; mine.a = d ? B.x : A.z; mine.b = d ? B.y : A.w; mine.s = ((u64)B.w << 32) | B.z;
        mine.fo_base = rr.fo_L; mine.fi_end = rr.fi_R; mine.exact = exact;
      }
      u = un;
      cur = nxt;
    }
    if (tid == 0) S->units += nunits;
    pass_units += nunits;
  };

  // block-wide arg-max of the threads' best (two barriers); refreshes the group bounds in between
  auto reduce_best = [&]() {
    const u32 bl = best_lane<RATIO>(mine.hi, mine.lo, mine.cost, mine.cand);
    if (bl == NONE32) { if (lane == 0) { S->wave_win[wave].hi = 0; S->wave_win[wave].lo = 0; S->wave_win[wave].cost = 1; S->wave_win[wave].cand = NONE32; } }
    else if (lane == bl) S->wave_win[wave] = mine;
    if (MC) {
      const u32 f2 = wave_max(floor2);
      if (lane == 0) S->wave_f2[wave] = f2;
    }
    __syncthreads();                               // all tile bounds and wavefront winners are in LDS
    const u32 ntl = S->ntl;
    for (u32 i = wave - 1; wave && i < ntl; i += LW - 1) {   // bounds of the groups that hold re-scored tiles
      const u32 g = alist[i] >> 6, t = g * 64 + lane;
      const u32 k = wave_max(t < nt ? keys[t] : 0u);
      if (lane == 0) skeys[g] = k;
    }
    if (wave == 0) {
      u64 h = 0, l = 0, cs = 1;
      u32 c = NONE32;
      if (lane < LW) { h = S->wave_win[lane].hi; l = S->wave_win[lane].lo; cs = S->wave_win[lane].cost; c = S->wave_win[lane].cand; }
      const u32 w = best_lane<RATIO>(h, l, cs, c);
      if (MC) {
        const u32 f2 = wave_max(lane < LW ? S->wave_f2[lane] : 0u);
        if (lane == 0) S->F2 = f2;
      }
      if (w == NONE32) { if (lane == 0) { S->mem[0].hi = 0; S->mem[0].lo = 0; } }
      else {
        if (lane == 0) {
          S->mem[0] = S->wave_win[w];
          S->mem[0].tau_o = ceil_div_x1000(S->wave_win[w].s, S->wave_win[w].dest ? bwo1 : bwo0, S->wave_win[w].dest ? ivo1 : ivo0);
        }
        if (lane == 1) S->mem[0].tau_i = ceil_div_x1000(S->wave_win[w].s, S->wave_win[w].dest ? bwi1 : bwi0, S->wave_win[w].dest ? ivi1 : ivi0);
      }
    }
    __syncthreads();
  };

  // ---- chunk jobs: one wavefront rewrites one chunk of one timeline, for all migrations of the
  // pass at once.  A job word: chunk | kind << 16 | set A << 24 | set B << 40, the sets being
  // bits over the pass's migrations: for a transfer-window job, A = the migrations of that
  // destination whose window meets the chunk; for a pressure job, A = those whose absent window
  // cuts the chunk, B = those that cover it whole.  (Host occupancy has no such job: see J_HQ.) --
  auto run_jobs = [&]() {
    const u32 nj = S->njobs;
    for (u32 jb = wave; jb < nj; jb += LW) {
      const u64 jw = jobs[jb];
      const u32 type = (u32)(jw >> 16) & 0xffu, c = (u32)jw & 0xffffu, ma_ = (u32)(jw >> 24) & 0xffffu, mb_ = (u32)(jw >> 40) & 0xffffu;
      const u32 s0 = c * CH, s1 = (s0 + CH - 1 < K - 1) ? s0 + CH - 1 : K - 1;
      if (type >= J_FO0 && type <= J_FI1) {
        // channel time of the transfer windows of this destination that meet the chunk is taken
        // from its slots (the windows of one pass are disjoint); the free-time prefix of the
        // slots after the first window slot is rewritten from a scan of the new values
        const bool out = type < J_FI0;
        const u32 d = (type - J_FO0) & 1u;
        const u32 arr = (out ? A_FO : A_FI) + d, w = out ? w_fo(d) : w_fi(d);
        u64* fr = tl.fre + (u64)((out ? 0u : 2u) + d) * tl.Kp;
        const u64 bc = base[(u64)arr * nb1 + c], ball = base[(u64)arr * nb1 + nch];
        const u32 mask = ma_;                            // the migrations of this destination whose window meets the chunk
        u32 first = NONE32;
        for (u32 pb = mask; pb; pb &= pb - 1) {
          const Winner& W = S->mem[__builtin_ctz(pb)];
          const u32 f = first_covered(s0, s1, K, out ? W.L1 : W.b + 1, out ? W.a - 1 : W.R - 1);
          first = f < first ? f : first;
        }
        u64 carry = 0;
        for (u32 st = 0; st < tl.spt; ++st) {
          const u32 j0 = s0 + st * 256u + lane * 4u;
          u64 f[4], old[4], tau[4], ref[4];
          u32 jj[4];
#pragma unroll
          for (u32 i = 0; i < 4; ++i) {
            const u32 j = j0 + i;
            f[i] = j < K ? fr[j] : 0ull;
            jj[i] = NONE32; tau[i] = 0; ref[i] = 0;
            if (j < K)
              for (u32 pb = mask; pb; pb &= pb - 1) {
                const Winner& W = S->mem[__builtin_ctz(pb)];
                const u32 p = in_doubled(j, K, out ? W.L1 : W.b + 1, out ? W.a - 1 : W.R - 1);
                if (p != NONE32) { jj[i] = p; tau[i] = out ? W.tau_o : W.tau_i; ref[i] = out ? W.fo_base : W.fi_end; }
              }
            old[i] = jj[i] != NONE32 ? tl.px[(u64)j * PX + w] : 0ull;       // free time of the chunk before the slot
          }
          u64 lsum = 0;
#pragma unroll
          for (u32 i = 0; i < 4; ++i) {
            if (jj[i] != NONE32) {
              const u64 before_slot = (jj[i] >= K ? ball : 0ull) + bc + old[i];  // free time before slot jj
              u64 take;
              if (out) {                           // eviction: earliest free time of the window first
                const u64 before = before_slot - ref[i];
                const u64 used = before < tau[i] ? before : tau[i];
                take = f[i] < tau[i] - used ? f[i] : tau[i] - used;
              } else {                             // prefetch: latest free time first
                const u64 after = ref[i] - (before_slot + f[i]);
                const u64 used = after < tau[i] ? after : tau[i];
                take = f[i] < tau[i] - used ? f[i] : tau[i] - used;
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
      } else if (type == J_P) {
        // pressure of the chunk's slots: the migrations whose absent window cuts the chunk are
        // taken off slot by slot, the ones that cover it whole go into the chunk's lazy add
        // (here, not by the chunk's thread); where a slot drops under the capacity the
        // over-capacity prefix after it is rewritten
        const u64 lz0 = lazyP[c];                        // the lazy add before this pass
        u64 lz_full = 0;
        const u32 part = ma_;                            // migrations whose window cuts the chunk; mb_: those that cover it whole
        for (u32 pb = mb_; pb; pb &= pb - 1) lz_full += S->mem[__builtin_ctz(pb)].s;
        const u64 lz = lz0 + lz_full;
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
              const u64 before = p - lz0;                // pressure before this pass
              u64 sub = 0;
              for (u32 pb = part; pb; pb &= pb - 1) {
                const Winner& W = S->mem[__builtin_ctz(pb)];
                if (in_doubled(j, K, W.a, W.b) != NONE32) sub += W.s;
              }
              if (sub) { p -= sub; tl.P[j] = p; }
              const u64 act = p - lz;
              if (act > cap) mn = act < mn ? act : mn;
              else if (before > cap && myfirst == NONE32) myfirst = j;
            }
          }
          const u32 stfirst = wave_min(myfirst);
          if (first == NONE32) first = stfirst;
        }
        mn = wave_min(mn);
        if (lane == 0) { minOver[c] = mn; lazyP[c] = lz; }
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
      } else if (type == J_CLIP) {
        // clipped area of the winner's absent window inside this chunk: per slot over the
        // capacity, duration x min(size, excess)
        const u32 wa = S->mem[0].a, wb = S->mem[0].b;
        const u64 s = S->mem[0].s;
        const u64 lz = lazyP[c];
        u64 alo = 0, ahi = 0;
        for (u32 st = 0; st < tl.spt; ++st) {
          const u32 j0 = s0 + st * 256u + lane * 4u;
#pragma unroll
          for (u32 i = 0; i < 4; ++i) {
            const u32 j = j0 + i;
            if (j < K && in_doubled(j, K, wa, wb) != NONE32) {
              const u64 act = tl.P[j] - lz;
              if (act > cap) {
                const u64 e = act - cap, m = e < s ? e : s, dj = tl.dur[j];
                const u64 plo = dj * m;
                ahi += __umul64hi(dj, m) + (alo + plo < alo ? 1ull : 0ull);
                alo += plo;
              }
            }
          }
        }
        const u64 p0 = wave_sum(alo & 0xffffffffull), p1 = wave_sum(alo >> 32), p2 = wave_sum(ahi);
        if (lane == 0) {
          atomicAdd((unsigned long long*)&S->acc[0], (unsigned long long)p0);
          atomicAdd((unsigned long long*)&S->acc[1], (unsigned long long)p1);
          atomicAdd((unsigned long long*)&S->acc[2], (unsigned long long)p2);
        }
      } else {
        // J_HQ: the largest host occupancy over the winner's period inside the chunk.  The slots'
        // host bytes are kept up to date on demand only: a migration to host that covers a chunk
        // whole goes into the chunk's lazy add when it is committed, one that cuts it is only
        // counted into the chunk's bound then (hmax, hpend); here the migrations committed since
        // the chunk was last brought up to date (hmat) are looked through, 64 at a time, and those
        // that cut the chunk are added to its slots, after which the bound is exact again.
        const u32 L1 = S->mem[0].L1, R = S->mem[0].R;
        const u64 lz = lazyH[c];
        const bool bring = hpend[c] != 0u;
        const u32 from = hmat[c], to = (u32)S->n_mig;
        u64 m_cov = 0, m_all = 0;
        for (u32 st = 0; st < tl.spt; ++st) {
          const u32 j0 = s0 + st * 256u + lane * 4u;
          u64 h[4];
#pragma unroll
          for (u32 i = 0; i < 4; ++i) h[i] = j0 + i < K ? tl.H[j0 + i] : 0ull;
          if (bring) {
            for (u32 r0 = from; r0 < to; r0 += 64u) {
              const u32 r = r0 + lane;
              const uint4 q = r < to ? a.rec_h[r] : make_uint4(0u, 1u, 0u, 0u);
              const u64 qs = ((u64)q.w << 32) | q.z;
              u32 len = 0;
              const u32 cv = qs ? cover(c, CH, K, q.x, q.y - 1, len) : 0u;
              u64 rel = __ballot(qs != 0ull && cv != 0u && cv != len);
              while (rel) {
                const u32 l = (u32)__builtin_ctzll(rel);
                rel &= rel - 1;
                const u32 x = (u32)__builtin_amdgcn_readlane((int)q.x, (int)l), y = (u32)__builtin_amdgcn_readlane((int)q.y, (int)l);
                const u64 sz = read_lane64(qs, l);
#pragma unroll
                for (u32 i = 0; i < 4; ++i)
                  if (j0 + i < K && in_doubled(j0 + i, K, x, y - 1) != NONE32) h[i] += sz;
              }
            }
#pragma unroll
            for (u32 i = 0; i < 4; ++i) if (j0 + i < K) tl.H[j0 + i] = h[i];
          }
#pragma unroll
          for (u32 i = 0; i < 4; ++i) {
            const u32 j = j0 + i;
            if (j < K) {
              const u64 act = h[i] + lz;
              m_all = act > m_all ? act : m_all;
              if (in_doubled(j, K, L1, R - 1) != NONE32) m_cov = act > m_cov ? act : m_cov;
            }
          }
        }
        m_cov = wave_max(m_cov);
        if (bring) {
          m_all = wave_max(m_all);
          if (lane == 0) { hmax[c] = m_all; hmat[c] = to; hpend[c] = 0u; }
        }
        if (lane == 0) atomicMax((unsigned long long*)&S->hq, (unsigned long long)m_cov);
      }
    }
    if (tid == 0) S->jobs += nj;
  };

  // Clipped-area benefit: the ranking went by bounds (the tensor's band, or a value computed
  // in an earlier pass: both can only be too large).  The best by bound stands only with a
  // value computed in this pass.  Otherwise its area is computed here - whole chunks of its
  // window in which every slot over the capacity exceeds it by the tensor's size count
  // size x over-capacity time, the others are summed slot by slot.  Returns true when the
  // winner stands (or nothing is left).  If the area comes out below the bound it is
  // remembered with the candidate and false is returned: the tiles scored in this pass are
  // then listed again (alist) and must be ranked once more.
  auto settle = [&]() -> bool {
    __syncthreads();
    if ((S->mem[0].hi | S->mem[0].lo) == 0 || S->mem[0].exact) return true;
    const u32 wa = S->mem[0].a, wb = S->mem[0].b;
    const u64 s = S->mem[0].s;
    if (tid == 0) { S->acc[0] = 0; S->acc[1] = 0; S->acc[2] = 0; S->njobs = 0; }
    __syncthreads();
    if (tid < nch) {
      u32 len = 0;
      const u32 cv = cover(tid, CH, K, wa, wb, len);
      if (cv) {
        const u64 mo = minOver[tid];
        if (cv == len && mo == NONE64) {
          // no slot of the chunk is over the capacity
        } else if (cv == len && mo - cap >= s) {
          const u64 t = tot[(u64)A_OT * nch + tid], lo = s * t;
          atomicAdd((unsigned long long*)&S->acc[0], (unsigned long long)(lo & 0xffffffffull));
          atomicAdd((unsigned long long*)&S->acc[1], (unsigned long long)(lo >> 32));
          atomicAdd((unsigned long long*)&S->acc[2], (unsigned long long)__umul64hi(s, t));
        } else {
          jobs[atomicAdd(&S->njobs, 1u)] = ((u64)J_CLIP << 16) | tid;
        }
      }
    }
    __syncthreads();
    run_jobs();
    __syncthreads();
    const u64 a0 = S->acc[0], a1 = S->acc[1], a2 = S->acc[2];
    const u64 vlo = a0 + (a1 << 32), vhi = a2 + (a1 >> 32) + (vlo < a0 ? 1ull : 0ull);
    const bool same = vhi == S->mem[0].hi && vlo == S->mem[0].lo;
    __syncthreads();                                   // everyone has read the sums and the bound
    if (tid == 0) {
      S->evals += 1;
      S->njobs = 0;
      if (same) S->mem[0].exact = 1;
      else {
        S->refused += 1;
        a.cd.cv[S->mem[0].pos] = make_uint4((u32)vlo, (u32)(vlo >> 32), (u32)vhi, (u32)(vhi >> 32));
        a.cd.ce[S->mem[0].pos] = make_uint2(cur_iter, 1u | (S->mem[0].dest << 1));
        S->ntl = 0;
      }
    }
    __syncthreads();
    if (same) return true;
    for (u32 g = tid; g < ns; g += LB) {               // every tile scored in this pass, once more
      u64 m = smark[g];
      while (m) {
        const u32 t = g * 64 + (u32)__builtin_ctzll(m);
        m &= m - 1;
        alist[atomicAdd(&S->ntl, 1u)] = (unsigned short)t;
        keys[t] = 0;
      }
    }
    __syncthreads();
    return false;
  };

  __syncthreads();
  // ---- passes ------------------------------------------------------------------------
  u32 passes = 0, used = 0;                          // ranking passes of this launch; with the further rounds of commits: what the budget counts
  bool wide_exit = false;
  while (true) {
    if (!resume) {                                   // (a pass taken up again has passed these tests)
      if (S->done) break;
      if (base[(u64)A_OT * nb1 + nch] == 0) { if (tid == 0) { S->done = 1; S->status = G10_FITS; } break; }
      if (max_iter && S->n_iter >= max_iter) { if (tid == 0) { S->done = 1; S->status = G10_TRUNCATED; } break; }
      if (used >= a.pass_budget || S->stop || (a.pass_stop && passes_before + passes >= a.pass_stop)) break;
      if (WIDE && S->no_wide) break;               // (the last launch of a round only ends the pass left open)
      ++passes; ++used;
    }
    mine.hi = 0; mine.lo = 0; mine.cost = 1; mine.cand = NONE32; mine.exact = 0; mine.kU = 0; mine.kr = 0;
    floor2 = 0;
    pass_units = 0;
    u32 thr = S->thr_key ? S->thr_key : NONE32;
    if (WIDE && resume) thr = wv.ctx->thr;
    __syncthreads();                               // the loop conditions and thr are read
    if (WIDE && resume) {                          // the tiles the open pass has scored, and the list of its open round
      for (u32 i = tid; i < ns; i += LB) smark[i] = wv.smark[i];
      for (u32 i = tid; i < wv.ctx->ntl; i += LB) alist[i] = wv.alist[i];
    } else {
      for (u32 i = tid; i < ns; i += LB) smark[i] = 0;   // no tile scored in this pass yet
    }
    if (tid == 0) {
      if (WIDE && resume) { S->ntl = wv.ctx->ntl; S->filt = 0; S->nl = 0; S->restL = NONE32; S->stale_hot = 0; }
      else { S->n_iter += 1; S->n_evals += C - S->n_mig - S->n_drop; }
      S->hq = 0; S->njobs = 0; S->ot_changed = 0;
      S->mem[0].hi = 0; S->mem[0].lo = 0;
      S->nlist = 0; S->F2 = 0; S->cut = MAXM; S->need_exact = 0; S->m0 = 1; S->by_floor = 0; S->touched = 0;
      if (S->stale_hot) { S->restL = NONE32; S->stale_hot = 0; }
      if (a.tick_budget && wall_clock64() - S->t_start > a.tick_budget) S->stop = 1;
    }
    __syncthreads();
    cur_iter = (u32)S->n_iter;

    // rank: score the hot tiles whose bound reaches a threshold (first a guess a little under
    // the last benefit), lower the threshold to the best benefit found, repeat until no tile
    // left out could hold an equal or better candidate
    u32 rounds = 0, rest_final = 0;
    bool again = false;                          // CLIP: the listed tiles are the ones already scored in this pass
    while (true) {
      u32 rest;
      bool decided = false;                      // the best by bound is known
      if (WIDE && resume) {
        rest = wv.ctx->rest;
        rounds = wv.ctx->rounds;
        pass_units = wv.ctx->pass_units;
        if (tid == LB - 1 && rounds) mine = wv.win[WIDE_WG];    // the best of the rounds before
      } else if (!again) {
        if (S->restL >= thr) {                     // the hot list may miss a tile that reaches thr: build it anew,
          const u32 low = thr == NONE32 ? thr : (thr > (1u << 19) ? thr - (1u << 19) : 1u);   // a few percent lower to last a while
          __syncthreads();
          build_hot(low);
          if (rounds && tid == 0) S->stale_hot = 1;  // built without the tiles already scored: not kept for the next pass
        }
        activate(thr);
        const u32 ntl = S->ntl;
        rest = S->restL > S->filt ? S->restL : S->filt;
        if (ntl == 0) {
          if ((rounds && (S->mem[0].hi | S->mem[0].lo) != 0) || rest == 0) decided = true;   // nothing left that could win
          else {
            thr = rest;                                  // strictly lower than before: start from the largest bound left
            __syncthreads();
            continue;
          }
        }
      } else {
        again = false;
        rest = S->restL > S->filt ? S->restL : S->filt;
        mine.hi = 0; mine.lo = 0; mine.cost = 1; mine.cand = NONE32; mine.exact = 0;
      }
      if (!decided) {
        if (WIDE && a.wide_min && !resume && !S->no_wide && (S->ntl << a.tshift) >= a.wide_min) {
          // a long round: the list, the tiles marked and what the pass needs to go on (with the
          // best of its earlier rounds) are left for the scoring kernel and the next launch
          const u32 ntl = S->ntl, nu = ntl << a.tshift;
          for (u32 i = tid; i < ns; i += LB) wv.smark[i] = smark[i];
          for (u32 i = tid; i < ntl; i += LB) wv.alist[i] = alist[i];
          if (tid == 0) {
            wv.win[WIDE_WG] = S->mem[0];         // (hi = lo = 0: none yet)
            wv.ctx->rounds = rounds; wv.ctx->pass_units = pass_units;
            wv.ctx->ntl = ntl; wv.ctx->thr = thr; wv.ctx->rest = rest;
            wv.ctx->nwg = nu < WIDE_WG ? nu : WIDE_WG; wv.ctx->done_wgs = 0;
            wv.ctx->pending = 1;
            ctl->wide_rounds += 1;
          }
          wide_exit = true;
          break;
        }
        if (WIDE && resume == 1) {                // the scoring kernel's winners, two per thread
          const u32 nw = wv.ctx->nwg;
          if (tid < LB - 1 && tid < nw) mine = wv.win[tid];
          if (tid < LB - 1 && tid + (LB - 1) < nw) {
            const Winner o = wv.win[tid + (LB - 1)];
            if ((o.hi | o.lo) != 0 && better_ratio(o.hi, o.lo, o.cost, o.cand, mine.hi, mine.lo, mine.cost, mine.cand)) mine = o;
          }
          const u32 nu = S->ntl << a.tshift;
          if (tid == 0) S->units += nu;
          pass_units += nu;
        } else score_list(thr);
        if (WIDE && resume) {
          resume = 0;
          if (tid == 0) wv.ctx->pending = 0;
        }
        reduce_best();
        ++rounds;
        const u32 kb = key_dn_of<RATIO>(S->mem[0].hi, S->mem[0].lo, S->mem[0].cost);
        const u32 need = kb ? kb : 1u;
        if (rest < need) decided = true;                 // every tile left out is below the best found
        else {
          // a tile left out may hold an equal or better one; with nothing found yet, step down a few percent
          thr = kb ? kb : (rest > (1u << 19) ? rest - (1u << 19) : 1u);
          if (tid == 0) S->second += 1;
          __syncthreads();
          continue;
        }
      }
      rest_final = rest;
      if (!CLIP || settle()) break;
      again = true;
    }
    if (WIDE && wide_exit) break;

    const bool none = (S->mem[0].hi | S->mem[0].lo) == 0;
    if (none) { __syncthreads(); if (tid == 0) { S->done = 1; S->status = G10_RESIDUAL; } break; }

    // ---- decide and commit -------------------------------------------------------------------
    // More migrations of the same pass (MC): the ranking also tells which candidate comes second,
    // third, ...  Candidate w_j wins the pass after w_1 .. w_(j-1) were committed if (1) nothing
    // those commits change enters its own score - no slot of its absent window can drop under the
    // capacity, and its transfer windows meet none of theirs on the same channel - and (2) no
    // other candidate can have risen above it.  Pressure only falls and reservations only grow,
    // so a benefit rises in one case only: a candidate the policy sends to flash, with a host
    // window as well, loses its flash window to a reservation and moves to host.  Such a
    // candidate is at risk once a committed flash migration's transfer windows meet its own; it
    // then counts with the bound of its host benefit.  Every candidate not on the list of the
    // pass (tiles left out, candidates under the round's threshold, the overflow of the list)
    // counts with its bound: the floor F.
    //
    // Step 1 (the last wavefront, a list entry per lane): the candidates in the order of their
    // benefit, as far as (2) and the transfer windows allow.  Where a round of commits ends with
    // entries still on the list that might clear the floor, the steps are taken again from here
    // (cround > 0) instead of from a new ranking.
    for (u32 cround = 0;; ++cround) {
    if (MC && wave == LW - 1 && S->nlist > 1u && K < (1u << 30)) {
      const u32 nl_ = S->nlist, n = nl_ < LIST_MAX ? nl_ : LIST_MAX;
      const bool have = lane < n;
      Winner e;
      if (have) e = S->list[lane];
      else { e.hi = 0; e.lo = 0; e.cand = NONE32; e.dest = 1; e.kr = 0; e.L1 = 0; e.R = 0; e.a = 1; e.b = 0; e.s = 0; e.pos = 0; }
      u32 F = rest_final > S->F2 ? rest_final : S->F2;
      u32 allowed = MAXM;                              // passes of Algorithm 1 this round may stand for
      bool picked;
      if (cround == 0u) {
        picked = have && e.cand == S->mem[0].cand;     // a migration of this pass already
        if (max_iter && max_iter - S->n_iter + 1 < allowed) allowed = (u32)(max_iter - S->n_iter + 1);   // (n_iter counts this pass already)
        if (lane == 0) S->Fkeep = F;
      } else {
        // Another round from the same list: its entries are scored again against the timelines as
        // the earlier rounds left them (a committed candidate has no window any more and scores
        // nothing), and the best of them wins the next pass of Algorithm 1 if its key clears the
        // floor - every candidate not on the list is still bounded by it, since bounds only fall.
        F = S->Fkeep;
        if (max_iter && max_iter - S->n_iter < allowed) allowed = (u32)(max_iter - S->n_iter);
        if (lane == 0) { S->njobs = 0; S->cut = MAXM; S->need_exact = 0; S->touched = 0; S->ot_changed = 0; S->hq = 0; S->list_rescored += n; }
        PrefixView pv; pv.px = tl.px; pv.base = base; pv.K = K; pv.nch = nch; pv.shift_ch = tl.shift_ch;
        Machine mc; mc.bwo0 = bwo0; mc.bwo1 = bwo1; mc.bwi0 = bwi0; mc.bwi1 = bwi1;
        mc.ivo0 = ivo0; mc.ivo1 = ivo1; mc.ivi0 = ivi0; mc.ivi1 = ivi1;
        if (have) {
          const uint4 A = a.cd.A[e.pos], B = a.cd.B[e.pos];
          const Score r = score_candidate(pv, mc, A, B);
          const bool ok_any = r.ok0 || r.ok1;
          const u32 d = r.ok0 ? 0u : 1u;
          const bool one = gt128(r.h1, r.l1, r.h0, r.l0);
          const u32 kc = upkey(one ? r.h1 : r.h0, one ? r.l1 : r.l0);
          e.hi = ok_any ? (d ? r.h1 : r.h0) : 0ull; e.lo = ok_any ? (d ? r.l1 : r.l0) : 0ull;
          e.dest = d; e.a = d ? B.x : A.z; e.b = d ? B.y : A.w;
          e.fo_base = r.fo_L; e.fi_end = r.fi_R; e.kU = kc; e.kr = (r.ok0 && r.ok1) ? kc : 0u;
          S->list[lane] = e;
        }
        const u32 b1 = wave_best_lane(e.hi, e.lo, e.cand);
        const u32 k1 = b1 == NONE32 ? 0u : upkey(read_lane64(e.hi, b1), read_lane64(e.lo, b1));
        if (allowed == 0u || k1 <= F) allowed = 0u;    // nothing on the list clears the floor: the pass is over
        else if (lane == b1) {
          e.tau_o = ceil_div_x1000(e.s, e.dest ? bwo1 : bwo0, e.dest ? ivo1 : ivo0);
          e.tau_i = ceil_div_x1000(e.s, e.dest ? bwi1 : bwi0, e.dest ? ivi1 : ivi0);
          S->mem[0] = e;
        }
        picked = allowed != 0u && lane == b1;
      }
      u32 m = 0, by_floor = 0;
      if (allowed) {
        const Winner& W1 = S->mem[0];
        u32 kB = (have && !picked) ? upkey(e.hi, e.lo) : 0u;       // (0: cannot be picked)
        const u32 eE0 = e.L1, eE1 = e.a - 1, eW0 = e.b + 1, eW1 = e.R - 1, ed = e.dest;
        const u32 kr = ed == 0u ? e.kr : 0u;
        bool ov = false;                               // a transfer window meets one of a committed migration on the same channel
        auto meet = [&](u32 wd, u32 wL1, u32 wa, u32 wb, u32 wR) {
          const bool hit = cyc_overlap32(eE0, eE1, wL1, wa - 1, K) || cyc_overlap32(eW0, eW1, wb + 1, wR - 1, K);
          ov = ov || (hit && ed == wd && !picked);
        };
        meet(W1.dest, W1.L1, W1.a, W1.b, W1.R);
        const u32 mmax = allowed;
        m = 1;
        while (m < mmax) {
          const u32 kmax = wave_max(kB);
          if (kmax <= F) { by_floor = 1; break; }      // (also when nothing is left)
          u64 mk = __ballot(kB == kmax);
          if (mk & (mk - 1)) {                         // equal keys: high word, low word, lowest index
            const bool in1 = kB == kmax;
            const u64 hmx = wave_max(in1 ? e.hi : 0ull);
            const bool in2 = in1 && e.hi == hmx;
            const u64 lmx = wave_max(in2 ? e.lo : 0ull);
            const bool in3 = in2 && e.lo == lmx;
            const u32 cmin = wave_min(in3 ? e.cand : NONE32);
            mk = __ballot(in3 && e.cand == cmin);
          }
          const u32 bl = (u32)__builtin_ctzll(mk);
          const u64 ovm = __ballot(ov);
          if ((ovm >> bl) & 1ull) break;               // its own windows are not what they were
          if (ovm && wave_max(ov ? kr : 0u) >= kmax) break;   // a candidate at risk might rise above it
          if (lane == 0) S->sel[m] = bl;
          if (lane == bl) { kB = 0u; picked = true; ov = false; }
          meet((u32)__builtin_amdgcn_readlane((int)ed, (int)bl), (u32)__builtin_amdgcn_readlane((int)e.L1, (int)bl),
               (u32)__builtin_amdgcn_readlane((int)e.a, (int)bl), (u32)__builtin_amdgcn_readlane((int)e.b, (int)bl),
               (u32)__builtin_amdgcn_readlane((int)e.R, (int)bl));
          ++m;
        }
        if (lane >= 1 && lane < m) {                   // the picked entries become migrations 1 .. m - 1
          Winner x = S->list[S->sel[lane]];
          x.tau_o = ceil_div_x1000(x.s, x.dest ? bwo1 : bwo0, x.dest ? ivo1 : ivo0);
          x.tau_i = ceil_div_x1000(x.s, x.dest ? bwi1 : bwi0, x.dest ? ivi1 : ivi0);
          S->mem[lane] = x;
        }
      }
      if (lane == 0) { S->m0 = m; S->by_floor = by_floor; }
    } else if (MC && wave == LW - 1 && lane == 0) S->by_floor = 1;     // (nothing else on the list)
    __syncthreads();

    // Step 2, chunk by chunk: what every picked migration does to the chunk (kept in `fl`, six bits
    // each), and how many of them can go together: the first that might let a slot drop under the
    // capacity, or that host memory might not hold on top of the earlier ones, ends the set (it
    // is ranked again in the next pass).  For the winner itself the two tests only decide how it
    // is committed: alone, and with the exact host-capacity test.
    enum { F_E = 1, F_W = 2, F_ACUT = 4, F_AALL = 8, F_PCUT = 16, F_PALL = 32 };
    const u32 m0 = S->m0;
    if (MC && m0 == 0u) break;                           // (a later round found nothing above the floor)
    u64 fl[MAXM / 8] = {};
    if (tid < ((nch + 63u) & ~63u)) {
      u32 cut = MAXM;
      bool ex0 = false;
      if (tid < nch) {
        const u64 mo = minOver[tid], hm = hmax[tid];
        u64 runP = 0, runH = 0;
        for (u32 i = 0; i < m0; ++i) {
          const Winner& M = S->mem[i];
          const u32 mL1 = M.L1, mR = M.R, ma = M.a, mb = M.b, md = M.dest;
          const u64 ms = M.s;
          u32 len = 0;
          const u32 cP = cover(tid, CH, K, mL1, mR - 1, len);       // the period: eviction window, absent window, prefetch window
          if (!cP) continue;                                        // (most migrations do not touch most chunks)
          const u32 cE = cover(tid, CH, K, mL1, ma - 1, len), cA = cover(tid, CH, K, ma, mb, len), cW = cP - cE - cA;
          u32 f = (cE ? F_E : 0u) | (cW ? F_W : 0u) | (cA == len ? F_AALL : cA ? F_ACUT : 0u);
          if (cA) {
            runP += ms;
            if (mo != NONE64 && mo - cap <= runP) { const u32 lim = i ? i : 1u; cut = lim < cut ? lim : cut; }
          }
          if (md == G10_HOST && cP) {
            f |= cP == len ? F_PALL : F_PCUT;
            if (ms > host_cap || hm + runH > host_cap - ms) { if (i == 0) ex0 = true; else cut = i < cut ? i : cut; }
            runH += ms;
          }
          fl[i >> 3] |= (u64)f << (8 * (i & 7u));
        }
      }
      cut = wave_min(cut);
      if (lane == 0 && cut < MAXM) atomicMin(&S->cut, cut);
      if (ex0) S->need_exact = 1;
    }
    __syncthreads();
    u32 m = m0 < S->cut ? m0 : S->cut;
    bool room = true;
    if (MC && cround && S->need_exact) break;            // (the exact host-memory test is left to the next ranking pass)
    if (S->need_exact) {                                 // the winner alone; host memory slot by slot where its period cuts a chunk
      m = 1;
      const u64 s = S->mem[0].s;
      const u32 f0 = (u32)fl[0] & 0xffu;
      if (tid == 0) S->hq = 0;
      __syncthreads();
      if ((f0 & F_PCUT) || ((f0 & F_PALL) && hpend[tid])) jobs[atomicAdd(&S->njobs, 1u)] = ((u64)J_HQ << 16) | tid;
      else if (f0 & F_PALL) atomicMax((unsigned long long*)&S->hq, (unsigned long long)hmax[tid]);   // (exact: nothing is missing there)
      __syncthreads();
      run_jobs();
      __syncthreads();
      room = s <= host_cap && S->hq <= host_cap - s;
      __syncthreads();
      if (tid == 0) S->njobs = 0;
      __syncthreads();
    }

    // Step 3: the plan records, the counters and the next pass's first threshold (the last
    // wavefront, lane i takes migration i) beside the commit chunk by chunk: a chunk a migration
    // covers whole takes a lazy add; a chunk that is cut, that holds a transfer window, or in
    // which a slot drops under the capacity gets a job (with the migrations it is about)
    if (wave == LW - 1) {
      const u64 nm = S->n_mig, nd = S->n_drop;
      if (lane < m) {
        const Winner& M = S->mem[lane];
        const u32 mL1 = M.L1, mR = M.R, ma = M.a, mb = M.b;
        const u64 ms = M.s;
        a.cd.A[M.pos] = make_uint4(mL1, mR, 1u, 0u);       // the candidate leaves the live set
        a.cd.B[M.pos] = make_uint4(1u, 0u, (u32)ms, (u32)(ms >> 32));
        if (!room) {
          g10_dropped dr; dr.iteration = S->n_iter - 1; dr.cand = M.cand; dr.reserved = 0;
          a.dropped[nd] = dr;
        } else {
          g10_migration mg;
          mg.cand = M.cand; mg.tensor = M.tensor;
          mg.evict_after = mL1 - 1; mg.absent_first = ma >= K ? ma - K : ma; mg.absent_last = mb >= K ? mb - K : mb;
          mg.next_use = mR >= K ? mR - K : mR;
          mg.dest = M.dest; mg.wraps = mR >= K ? 1u : 0u;
          mg.size_bytes = ms; mg.t_out_ns = M.tau_o; mg.t_in_ns = M.tau_i; mg.benefit_lo = M.lo; mg.benefit_hi = M.hi;
          a.records[nm + lane] = mg;
          a.rec_ab[nm + lane] = make_uint2(ma, mb);
          a.rec_h[nm + lane] = M.dest == G10_HOST ? make_uint4(mL1, mR, (u32)ms, (u32)(ms >> 32)) : make_uint4(mL1, mR, 0u, 0u);
          atomicOr(&S->touched, (1u << (A_FO + M.dest)) | (1u << (A_FI + M.dest)));
        }
      }
      if (lane == 0) {
        // first threshold of the next pass: a little under the last benefit.  How little adapts:
        // where many candidates are nearly equal (a pass scored thousands) the margin halves; it
        // doubles when a pass ran out of candidates above the floor with little scored
        u32 gs = S->gshift;
        if (cround) {
          // (the margin adapts once per ranking pass)
        } else if (WIDE && a.wide_min) {
          // with the scoring kernel a longer list costs little and a second round a pair of launches:
          // the margin doubles whenever a pass needed one, and narrows only now and then
          if (rounds > 1u) { if (gs > 2u) --gs; }
          else if ((S->n_iter & 31u) == 0u && gs < GUESS_SHIFT) ++gs;
        } else if (pass_units > 8u && gs < GUESS_SHIFT_MAX) ++gs;
        else if (MC) { if ((S->by_floor || rounds > 1u) && pass_units <= 4u && gs > MC_GUESS_SHIFT_MIN) --gs; }
        else if (rounds > 1u && pass_units <= 2u && gs > GUESS_SHIFT) --gs;
        S->gshift = gs;
        const Winner& Z = S->mem[m - 1];
        u64 ghi = Z.hi, glo = Z.lo;
        const u64 dlo = (glo >> gs) | (ghi << (64 - gs)), dhi = ghi >> gs;
        const u64 nlo = glo - dlo;
        ghi = ghi - dhi - (glo < dlo ? 1ull : 0ull);
        S->thr_key = RATIO ? rkey_dn(ratio_approx(Z.hi, Z.lo, Z.cost) * (1.0 - 1.0 / (double)(1u << gs))) : upkey(ghi, nlo);
        if (!room) { S->n_drop = nd + 1; S->more = 0; }
        else {
          // the passes of Algorithm 1 this round stands for beyond the one the ranking pass counted
          // at its top (a later round: all of its own), each with one live candidate fewer to rank
          const u64 x = cround ? m : m - 1, live = C - nm - nd;
          S->n_mig = nm + m; S->n_iter += x;
          S->n_evals += cround ? x * live - x * (x - 1) / 2 : x * live - x * (x + 1) / 2;
          // another round of commits from the same list: unless the picking ran out of entries above
          // the floor and every one it picked was committed
          const bool more = MC && S->nlist > 1u && K < (1u << 30) && (!S->by_floor || m < m0) && !(max_iter && S->n_iter >= max_iter);
          S->more = more ? 1u : 0u;
          if (cround) S->more_rounds += 1;
        }
      }
    }
    if (!room) { __syncthreads(); break; }
    if (tid < nch) {
      const u32 c = tid;
      u64 lzP = 0, lzH = 0, cutHs = 0;
      u32 cutP = 0, allP = 0, cutH = 0, fo[2] = {0, 0}, fi[2] = {0, 0};
      for (u32 i = 0; i < m; ++i) {
        const u32 f = (u32)(fl[i >> 3] >> (8 * (i & 7u))) & 0xffu;
        if (!f) continue;
        const u64 ms = S->mem[i].s;
        const u32 md = S->mem[i].dest;
        if (f & F_AALL) { lzP += ms; allP |= 1u << i; }
        if (f & F_ACUT) cutP |= 1u << i;
        if (f & F_PALL) lzH += ms;
        if (f & F_PCUT) { cutH |= 1u << i; cutHs += ms; }
        if (f & F_E) fo[md] |= 1u << i;
        if (f & F_W) fi[md] |= 1u << i;
      }
      bool jobP = cutP != 0;
      if (lzP) {
        const u64 mo = minOver[c];
        if (mo != NONE64 && mo - cap <= lzP) jobP = true;       // a slot drops under the capacity
        if (!jobP) { lazyP[c] += lzP; if (mo != NONE64) minOver[c] = mo - lzP; }
      }
      // host occupancy: whole covers into the lazy add; cuts only into the chunk's bound, the slots follow on demand (J_HQ)
      if (lzH | cutHs) { lazyH[c] += lzH; hmax[c] += lzH + cutHs; }
      if (cutH) hpend[c] = 1u;
      // (a job adds the sizes of the migrations that cover its chunk whole itself)
      if (jobP) jobs[atomicAdd(&S->njobs, 1u)] = ((u64)allP << 40) | ((u64)cutP << 24) | ((u64)J_P << 16) | c;
      if (fo[0]) jobs[atomicAdd(&S->njobs, 1u)] = ((u64)fo[0] << 24) | ((u64)J_FO0 << 16) | c;
      if (fo[1]) jobs[atomicAdd(&S->njobs, 1u)] = ((u64)fo[1] << 24) | ((u64)J_FO1 << 16) | c;
      if (fi[0]) jobs[atomicAdd(&S->njobs, 1u)] = ((u64)fi[0] << 24) | ((u64)J_FI0 << 16) | c;
      if (fi[1]) jobs[atomicAdd(&S->njobs, 1u)] = ((u64)fi[1] << 24) | ((u64)J_FI1 << 16) | c;
    }
    __syncthreads();
    run_jobs();
    __syncthreads();
    // level 1: the bases of the timelines whose chunk totals changed, one wavefront per timeline
    {
      const u32 touched = S->touched | (S->ot_changed ? 1u : 0u);
      if (wave < N_ARR && ((touched >> wave) & 1u)) {
        const u32 arr = wave;
        constexpr u32 PER = (NCH_MAX + G10_WAVE - 1) / G10_WAVE;
        u64 v[PER], sum = 0;
#pragma unroll
        for (u32 k = 0; k < PER; ++k) {
          const u32 c = lane * PER + k;
          v[k] = c < nch ? tot[(u64)arr * nch + c] : 0ull;
          sum += v[k];
        }
        const u64 inc = wave_scan_incl(sum);
        u64 run = inc - sum;
#pragma unroll
        for (u32 k = 0; k < PER; ++k) {
          const u32 c = lane * PER + k;
          if (c < nch) base[(u64)arr * nb1 + c] = run;
          run += v[k];
        }
        if (lane == G10_WAVE - 1) base[(u64)arr * nb1 + nch] = inc;
      }
      __syncthreads();
    }
    if (!MC || !S->more) break;
    ++used;
    }                                                    // (rounds of commits of one ranking pass)
  }
  __syncthreads();

  // ---- state out ---------------------------------------------------------------------
  for (u32 i = tid; i < N_ARR * nch; i += LB) a.g_tot[i] = tot[i];
  for (u32 i = tid; i < nch; i += LB) { a.g_lazyP[i] = lazyP[i]; a.g_minOver[i] = minOver[i]; a.g_lazyH[i] = lazyH[i]; a.g_hmax[i] = hmax[i]; a.g_hmat[i] = hmat[i]; a.g_hpend[i] = hpend[i]; }
  for (u32 i = tid; i < nt; i += LB) a.g_keys[i] = keys[i];
  for (u32 i = tid; i < N_ARR * nb1; i += LB) a.g_base[i] = base[i];
  if (tid == 0) {
    ctl->n_iter = S->n_iter; ctl->n_mig = S->n_mig; ctl->n_drop = S->n_drop; ctl->n_evals = S->n_evals;
    ctl->thr_key = S->thr_key; ctl->status = S->status; ctl->done = S->done;
    ctl->gshift = S->gshift;
    ctl->overtime_after = base[(u64)A_OT * nb1 + nch];
    ctl->units_scored += S->units; ctl->second_rounds += S->second; ctl->jobs_run += S->jobs; ctl->launches += 1;
    ctl->passes += passes;
    ctl->area_evals += S->evals; ctl->area_refused += S->refused;
    ctl->more_rounds += S->more_rounds; ctl->list_rescored += S->list_rescored;
  }
}

// The scoring kernel of WideCtx: workgroup b scores the units b, b + nwg, ... of the list the
// loop kernel left (256 candidates each, scored as the loop kernel's own rounds score them),
// raises the bounds of their tiles in device memory and leaves its best candidate in win[b].
__global__ __launch_bounds__(UNIT) void k_wide_score(const LoopArgs* __restrict__ plans) {
  extern __shared__ __align__(16) unsigned char smem[];
  const LoopArgs a = plans[0];
  if (!a.wide) return;
  const WideView wv = wide_view(a.wide);
  const u32 nwg = wv.ctx->nwg;
  if (!wv.ctx->pending || blockIdx.x >= nwg) return;
  const Timelines tl = a.tl;
  const u32 nch = tl.nch, K = tl.K;
  const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  Winner* wwin = (Winner*)smem;                         // [UNIT / 64]
  const Ctl* ctl = a.ctl;
  PrefixView pv; pv.px = tl.px; pv.K = K; pv.nch = nch; pv.shift_ch = tl.shift_ch;
  pv.base = a.g_base;                                   // (a few entries per candidate, read where they lie)
  Machine mc; mc.bwo0 = ctl->bw_out[0]; mc.bwo1 = ctl->bw_out[1]; mc.bwi0 = ctl->bw_in[0]; mc.bwi1 = ctl->bw_in[1];
  mc.ivo0 = ctl->inv_out[0]; mc.ivo1 = ctl->inv_out[1]; mc.ivi0 = ctl->inv_in[0]; mc.ivi1 = ctl->inv_in[1];
  Winner mine;
  mine.hi = 0; mine.lo = 0; mine.cost = 1; mine.cand = NONE32; mine.exact = 0; mine.kU = 0; mine.kr = 0; mine.tau_o = 0; mine.tau_i = 0; mine.pad = 0;
  mine.s = 0; mine.fo_base = 0; mine.fi_end = 0; mine.tensor = 0; mine.pos = 0; mine.dest = 0; mine.L1 = 0; mine.R = 0; mine.a = 1; mine.b = 0;
  const u32 nunits = wv.ctx->ntl << a.tshift;
  for (u32 u = blockIdx.x; u < nunits; u += nwg) {
    const u32 t = wv.alist[u >> a.tshift];
    const u32 p = (((t << a.tshift) + (u & ((1u << a.tshift) - 1u))) << 8) + tid;
    const uint4 A = a.cd.A[p], B = a.cd.B[p];
    const uint2 id = a.cd.id[p];
    const Score r = score_candidate(pv, mc, A, B);
    if (r.strike0) a.cd.A[p] = make_uint4(A.x, A.y, 1u, 0u);
    if (r.strike1) a.cd.B[p] = make_uint4(1u, 0u, B.z, B.w);
    u64 c0 = 1, c1 = 1;
    if (r.ok0 || r.ok1) costs_of(mc, ((u64)B.w << 32) | B.z, c0, c1);
    const u32 k0 = key_up_of<true>(r.h0, r.l0, c0), k1 = key_up_of<true>(r.h1, r.l1, c1);
    const u32 k = wave_max(k0 > k1 ? k0 : k1);         // the tile's bound holds for either destination
    if (lane == 0 && k) atomicMax(&a.g_keys[t], k);
    const bool ok_any = r.ok0 || r.ok1;                // flash first; host only if flash cannot take it
    const u32 d = r.ok0 ? 0u : 1u;
    const u64 hi = ok_any ? (d ? r.h1 : r.h0) : 0ull, lo = ok_any ? (d ? r.l1 : r.l0) : 0ull, cost = d ? c1 : c0;
    if ((hi | lo) != 0 && better_ratio(hi, lo, cost, id.x, mine.hi, mine.lo, mine.cost, mine.cand)) {
      mine.hi = hi; mine.lo = lo; mine.cost = cost; mine.cand = id.x; mine.tensor = id.y; mine.pos = p; mine.dest = d;
      mine.L1 = A.x; mine.R = A.y; mine.a = d ? B.x : A.z; mine.b = d ? B.y : A.w; mine.s = ((u64)B.w << 32) | B.z;
      mine.fo_base = r.fo_L; mine.fi_end = r.fi_R;
    }
  }
  const u32 bl = wave_best_lane_ratio(mine.hi, mine.lo, mine.cost, mine.cand);
  if (bl == NONE32) { if (lane == 0) { mine.hi = 0; mine.lo = 0; mine.cost = 1; mine.cand = NONE32; wwin[wave] = mine; } }
  else if (lane == bl) wwin[wave] = mine;
  __syncthreads();
  if (wave == 0) {
    u64 h = 0, l = 0, cs = 1;
    u32 c = NONE32;
    if (lane < UNIT / 64) { h = wwin[lane].hi; l = wwin[lane].lo; cs = wwin[lane].cost; c = wwin[lane].cand; }
    const u32 w = wave_best_lane_ratio(h, l, cs, c);
    if (lane == 0) {
      wv.win[blockIdx.x] = wwin[w == NONE32 ? 0u : w];  // (none: any of the four, all empty)
      __threadfence();
      atomicAdd(&wv.ctx->done_wgs, 1u);
    }
  }
}

}  // namespace

size_t loop_wide_bytes() { return WIDE_BYTES; }

int loop_wide_launch(const LoopArgs* plans, u32 nch, hipStream_t s) {
  (void)nch;
  const size_t lds = (UNIT / 64) * sizeof(Winner);
  hipLaunchKernelGGL(k_wide_score, dim3(WIDE_WG), dim3(UNIT), lds, s, plans);
  G10_HIP(hipGetLastError());
  return G10_OK;
}

size_t loop_lds_bytes(u32 nch, u32 nt) {
  const size_t ns = (nt + 63) / 64;
  size_t b = 0;
  b += ((size_t)N_ARR * (nch + 1) + (size_t)N_ARR * nch + (size_t)4 * nch + ns + (size_t)4 * LW + (size_t)8 * nch + 8) * 8;
  b += sizeof(Shared);
  b += ((size_t)nt + ns + 2 * (size_t)nch) * 4 + (size_t)nt * 4;
  return (b + 15) & ~(size_t)15;
}

typedef void (*LoopKernel)(const LoopArgs*);
static LoopKernel loop_kernel(u32 rank, u32 area) {
  if (area == G10_AREA_CLIPPED) return rank == G10_RANK_RATIO ? k_loop<true, true> : k_loop<false, true>;
  return rank == G10_RANK_RATIO ? k_loop<true, false> : k_loop<false, false>;
}

int loop_allow_large_lds() {                     // (once per device: the attribute belongs to the kernel, not to a handle)
  static bool done[64] = {};
  int dev = 0;
  G10_HIP(hipGetDevice(&dev));
  if (dev >= 0 && dev < 64 && done[dev]) return G10_OK;
  for (u32 rank = 0; rank < 2; ++rank)
    for (u32 area = 0; area < 2; ++area)
      G10_HIP(hipFuncSetAttribute((const void*)loop_kernel(rank, area), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
  if (dev >= 0 && dev < 64) done[dev] = true;
  return G10_OK;
}

int loop_launch(const LoopArgs* plans, u32 n_plans, size_t lds, u32 rank, u32 area, hipStream_t s) {
  hipLaunchKernelGGL(loop_kernel(rank, area), dim3(n_plans), dim3(LB), lds, s, plans);
  G10_HIP(hipGetLastError());
  return G10_OK;
}
