// CPU oracle for G10's tensor vitality analysis and smart tensor eviction.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, single-threaded reference
// that the GPU library is checked against.  Nothing in the product path may
// include, link or call it; it shares no code with the GPU library.
//
// What it follows (G10, MICRO'23):
//   * Section 3: a tensor is active while the executing kernel uses it;
//     an inactive period is an interval in which it is unused but will be
//     used again.
//   * Section 4.2 (tensor vitality analysis): global tensors live for the
//     whole iteration and their last inactive period runs into the next
//     iteration; intermediate tensors are born at their first use and dead
//     after their last; period lengths come from profiled kernel times;
//     eviction / prefetch overheads are size / bandwidth.
//   * Section 4.3 and Algorithm 1 (smart tensor eviction): repeat { stop if
//     the pressure never exceeds the capacity; rank all remaining inactive
//     periods by the over-capacity pressure they would remove; take the best
//     if its benefit is positive; send it to flash unless the flash channel
//     is full during the transfer, in which case send it to host memory if
//     host memory has room; update pressure and traffic }.
//   * Section 4.4: Algorithm 1 assumes each prefetch starts at the latest
//     time that still completes before the next use (the latest safe prefetch
//     time).  Smart prefetching then takes the evicted periods in the order of
//     that time and moves each prefetch back to the earliest time from which
//     the GPU can hold the whole tensor without exceeding its capacity,
//     raising the pressure curve in between.
//
// The paper leaves the discretisation open.  The readings taken here:
//   * the timeline is divided into kernel slots (instructions can only be
//     inserted between kernels, Figure 6); two iterations are laid end to end
//     ("doubled coordinates") so that a weight's period can run into the next;
//   * an eviction is issued at the start of the period, a prefetch ends at the
//     next use; memory counts as freed only from the first slot boundary after
//     the eviction ends to the last slot boundary before the prefetch starts;
//   * "traffic is full during the transfer" = the channel time not yet
//     reserved inside the slot-rounded transfer window cannot carry the
//     transfer; tested for the eviction and for the prefetch;
//   * benefit = size x time spent over capacity inside the absent window;
//     ranking by benefit alone, ties to the lowest period index;
//   * flash full and host memory without room: the candidate is dropped;
//   * smart prefetching: the prefetch moves back in whole kernel slots, at most
//     to the slot boundary at which the eviction has ended; a slot can take
//     the tensor if its pressure plus the tensor's size stays within the
//     capacity; equal prefetch times keep the plan's order; only the pressure
//     curve is updated (the paper says nothing of the channels here).
//
// Two readings have an alternative that the text of Section 4.3 supports as
// well; both alternatives can be switched on per plan:
//   * area = 1 ("clipped"): the benefit is the area between the pressure curve
//     and the capacity line that the eviction removes, i.e. per slot of the
//     absent window  duration x min(size, pressure - capacity)  where the
//     pressure is over the capacity; the default counts the tensor's whole
//     band, size x duration, in such a slot.  The two agree whenever every
//     over-capacity slot of the window exceeds the capacity by at least the
//     tensor's size.
//   * rank = 1 ("ratio"): periods are ranked by benefit / cost with
//     cost = eviction time + prefetch time of the chosen destination (the
//     benefit-cost ratio of the section's example), compared exactly as
//     fractions; the default ranks by the benefit alone, as Algorithm 1 does.
//     Ties go to the lowest period index either way.
//
// Beyond the paper's planner, replay() plays a finished plan back slot by slot under given
// kernel durations (stall time, traffic per destination): a stand-in for the breakdown the
// paper's simulator reports; its model is stated at the function.  parity unpinned against the
// paper (which prints no such numbers for a trace we have); pinned as defined by tests/.
//
// Two evaluation modes compute the same values:
//   mode 0 ("direct"):  every sum / max / search is the literal loop of its
//                       definition over kernel slots.  O(window) per query.
//   mode 1 ("prefix"):  range sums come from prefix arrays rebuilt from
//                       scratch at the top of every iteration, window ends
//                       from binary search, the pressure timeline from a
//                       difference array.  Same integers, usable on large
//                       traces.  Tests tie mode 1 to mode 0.
//
// All times are integer nanoseconds, sizes integer bytes, bandwidths bytes
// per microsecond; benefits are 128-bit byte-nanoseconds.
//
// Parity status of the readings that the paper does not fix numerically
// (benefit clipping, benefit-only ranking key, prefetch-side channel test,
// slot rounding, dropping on flash-full + host-full, and in smart prefetching
// the slot granularity, the lower limit and leaving the channels alone):
// parity unpinned — the
// paper prints no value that separates the alternatives.  Everything else is
// pinned by the tests under tests/ (worked examples, closed forms,
// invariants, brute force).

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <new>
#include <vector>

typedef unsigned __int128 u128;
typedef uint64_t u64;
typedef uint32_t u32;

extern "C" {

struct g10o_trace {
  u32 K, N;
  u64 P;
  const u64* dur_ns;      // [K]
  const u64* size_bytes;  // [N]
  const uint8_t* is_global;  // [N]
  const u32* use_kernel;  // [P]
  const u32* use_tensor;  // [P]
  u32 no_wrap;            // 1: ignore cross-iteration periods of global tensors
};

struct g10o_params {
  u64 gpu_cap, host_cap;
  u64 bw_out[2], bw_in[2];  // [0] flash, [1] host; bytes per microsecond
  u32 rank;                 // 0: by benefit; 1: by benefit / (eviction + prefetch time)
  u32 area;                 // 0: the tensor's band over capacity; 1: clipped at the capacity line
};

struct g10o_record {  // one committed migration, in commit order
  u32 cand, tensor, evict_after, absent_first, absent_last, next_use;
  u32 dest, wraps;
  u64 size, t_out, t_in, benefit_lo, benefit_hi;
};

struct g10o_summary {
  int32_t status;  // 0 fits, 1 residual, 2 stopped by max_iters
  u64 n_migrations, n_iterations, n_null, n_cand_evals;
  u64 peak_before, peak_after, overtime_before, overtime_after;
};

}  // extern "C"

namespace {

enum { FLASH = 0, HOST = 1, OUT = 0, IN = 1 };

struct Dest {
  bool valid;
  u32 a, b;        // absent slots [a, b], doubled coordinates
  u64 tau_o, tau_i;
};

struct Cand {
  u32 t, L, R;     // tensor, last use before, next use (R may be >= K)
  u64 s;
  Dest d[2];
};

struct Oracle {
  // trace
  u32 K = 0, N = 0;
  std::vector<u64> dur, size;
  std::vector<uint8_t> glob;
  // vitality
  std::vector<u64> use_off;          // [N+1]
  std::vector<u32> use_k;            // distinct uses, tensor-major
  std::vector<u32> birth, death;     // [N], meaningful where the tensor is used
  std::vector<u32> per_t, per_L, per_R;
  std::vector<u64> start;            // [K+1]
  std::vector<u64> pressure0;        // [K]
  u64 peak = 0, T = 0;
  // plan output
  std::vector<g10o_record> records;
  std::vector<u32> null_cands;
  std::vector<u64> null_iters;       // rank pass (0-based) in which each was dropped
  std::vector<u64> pressure_after;
  std::vector<u64> busy_after[2][2];
  std::vector<u64> host_after;
  std::vector<u32> rec_a, rec_b, rec_R;  // per record: absent slots [a, b] and next use, doubled coordinates
  u64 plan_cap = 0;                  // GPU capacity the plan was made for
  // smart prefetching output
  std::vector<u32> pf_order;         // records in the order they were visited
  std::vector<u32> pf_gained;        // per record: kernel slots by which its prefetch moved back
  std::vector<u64> pressure_eager;   // pressure with the earlier prefetches
};

inline u64 ceil_div(u128 x, u64 y) { return (u64)((x + y - 1) / y); }

// x * y as a 192-bit number, most significant word first
struct U192 { u64 w[3]; };
inline U192 mul_128_64(u128 x, u64 y) {
  const u128 lo = (u128)(u64)x * y, hi = (u128)(u64)(x >> 64) * y + (u64)(lo >> 64);
  return U192{{(u64)(hi >> 64), (u64)hi, (u64)lo}};
}
inline bool greater(const U192& p, const U192& q) {
  for (int i = 0; i < 3; ++i) if (p.w[i] != q.w[i]) return p.w[i] > q.w[i];
  return false;
}

// start time of slot j on the doubled timeline, j in [0, 2K]   (two
// back-to-back iterations that follow the same plan)
inline u64 start2(const Oracle& o, u64 j) {
  return j < o.K ? o.start[j] : o.start[j - o.K] + o.T;
}

// ---------------------------------------------------------------- vitality
int vitality(Oracle& o, const g10o_trace& tr, int mode) {
  if (!tr.K || !tr.N || tr.K >= (1u << 31)) return -1;
  if (!tr.dur_ns || !tr.size_bytes || !tr.is_global) return -1;
  if (tr.P && (!tr.use_kernel || !tr.use_tensor)) return -1;
  o.K = tr.K;
  o.N = tr.N;
  o.dur.assign(tr.dur_ns, tr.dur_ns + tr.K);
  o.size.assign(tr.size_bytes, tr.size_bytes + tr.N);
  o.glob.assign(tr.is_global, tr.is_global + tr.N);
  for (u64 d : o.dur) if (!d) return -1;
  for (u64 s : o.size) if (!s) return -1;
  for (u64 s : o.size) if (((u128)s * 1000) >> 64) return -2;
  for (u64 p = 0; p < tr.P; ++p)
    if (tr.use_kernel[p] >= tr.K || tr.use_tensor[p] >= tr.N) return -1;

  // slot start times (Section 4.2: kernel times give the period lengths)
  o.start.assign(o.K + 1, 0);
  u128 tt = 0;
  for (u32 k = 0; k < o.K; ++k) {
    tt += o.dur[k];
    if (tt >> 62) return -2;
    o.start[k + 1] = (u64)tt;
  }
  o.T = o.start[o.K];

  // use lists: the distinct kernels touching each tensor, ascending
  std::vector<std::vector<u32>> uses(o.N);
  for (u64 p = 0; p < tr.P; ++p) uses[tr.use_tensor[p]].push_back(tr.use_kernel[p]);
  o.use_off.assign(o.N + 1, 0);
  o.use_k.clear();
  o.birth.assign(o.N, 0);
  o.death.assign(o.N, 0);
  for (u32 t = 0; t < o.N; ++t) {
    std::vector<u32>& u = uses[t];
    std::sort(u.begin(), u.end());
    u.erase(std::unique(u.begin(), u.end()), u.end());
    o.use_off[t] = o.use_k.size();
    o.use_k.insert(o.use_k.end(), u.begin(), u.end());
    if (!u.empty()) { o.birth[t] = u.front(); o.death[t] = u.back(); }
  }
  o.use_off[o.N] = o.use_k.size();

  // inactive periods: gaps of at least one whole kernel between two uses;
  // for a global tensor also the gap from its last use to its first use in
  // the next iteration.  Order: tensor, then period start; wrap period last.
  o.per_t.clear(); o.per_L.clear(); o.per_R.clear();
  for (u32 t = 0; t < o.N; ++t) {
    const std::vector<u32>& u = uses[t];
    for (size_t i = 0; i + 1 < u.size(); ++i)
      if (u[i + 1] - u[i] >= 2) { o.per_t.push_back(t); o.per_L.push_back(u[i]); o.per_R.push_back(u[i + 1]); }
    if (o.glob[t] && !tr.no_wrap && !u.empty()) {
      u64 R = (u64)u.front() + o.K;
      if (R - u.back() >= 2) { o.per_t.push_back(t); o.per_L.push_back(u.back()); o.per_R.push_back((u32)R); }
    }
  }

  // memory pressure: bytes resident in each kernel slot with nothing evicted
  o.pressure0.assign(o.K, 0);
  u128 total = 0;
  for (u32 t = 0; t < o.N; ++t) if (!uses[t].empty()) total += o.size[t];
  if (total >> 64) return -2;
  if (mode == 0) {
    for (u32 t = 0; t < o.N; ++t) {
      if (uses[t].empty()) continue;
      u32 lo = o.glob[t] ? 0 : o.birth[t], hi = o.glob[t] ? o.K - 1 : o.death[t];
      for (u32 k = lo; k <= hi; ++k) o.pressure0[k] += o.size[t];
    }
  } else {
    std::vector<u64> diff(o.K + 1, 0);
    for (u32 t = 0; t < o.N; ++t) {
      if (uses[t].empty()) continue;
      u32 lo = o.glob[t] ? 0 : o.birth[t], hi = o.glob[t] ? o.K - 1 : o.death[t];
      diff[lo] += o.size[t];
      diff[hi + 1] -= o.size[t];
    }
    u64 run = 0;
    for (u32 k = 0; k < o.K; ++k) { run += diff[k]; o.pressure0[k] = run; }
  }
  o.peak = 0;
  for (u64 p : o.pressure0) o.peak = std::max(o.peak, p);
  return 0;
}

// ---------------------------------------------------------------- planning
struct Planner {
  const Oracle& o;
  const g10o_params& pr;
  int mode;
  u32 K;
  std::vector<Cand> cand;
  std::vector<uint8_t> live;
  u64 n_live = 0;
  std::vector<u64> pressure, host_used;
  std::vector<u64> busy[2][2];
  // mode 1 only: prefix arrays, rebuilt at the top of every iteration
  std::vector<u64> OT;           // over-capacity time before slot k
  std::vector<u64> FP[2][2];     // free channel time before slot k

  Planner(const Oracle& o_, const g10o_params& p_, int m) : o(o_), pr(p_), mode(m), K(o_.K) {}

  // -- per candidate and destination: transfer times and the absent window
  void prepare() {
    size_t C = o.per_t.size();
    cand.resize(C);
    for (size_t c = 0; c < C; ++c) {
      Cand& x = cand[c];
      x.t = o.per_t[c]; x.L = o.per_L[c]; x.R = o.per_R[c]; x.s = o.size[x.t];
      for (int d = 0; d < 2; ++d) {
        Dest& D = x.d[d];
        D.tau_o = ceil_div((u128)x.s * 1000, pr.bw_out[d]);
        D.tau_i = ceil_div((u128)x.s * 1000, pr.bw_in[d]);
        u64 t_r = start2(o, (u64)x.L + 1);           // eviction issued at the period start
        u64 t_use = start2(o, x.R);                  // tensor needed again here
        bool has_a = false, has_b = false;
        u64 a = 0, b = 0;
        if (mode == 0) {
          for (u64 j = (u64)x.L + 1; j <= x.R; ++j)
            if ((u128)start2(o, j) >= (u128)t_r + D.tau_o) { a = j; has_a = true; break; }
          if (D.tau_i <= t_use)
            for (u64 j = x.R; j-- > x.L;)              // j = R-1 ... L
              if (start2(o, j + 1) <= t_use - D.tau_i) { b = j; has_b = true; break; }
        } else {
          if ((u128)t_use >= (u128)t_r + D.tau_o) {   // first slot boundary at/after eviction end
            u64 lo = (u64)x.L + 1, hi = x.R;
            while (lo < hi) { u64 mid = (lo + hi) / 2; if (start2(o, mid) >= t_r + D.tau_o) hi = mid; else lo = mid + 1; }
            a = lo; has_a = true;
          }
          if (D.tau_i <= t_use && start2(o, (u64)x.L + 1) <= t_use - D.tau_i) {
            u64 lo = x.L, hi = (u64)x.R - 1;          // last slot whose end is at/before prefetch start
            while (lo < hi) { u64 mid = (lo + hi + 1) / 2; if (start2(o, mid + 1) <= t_use - D.tau_i) lo = mid; else hi = mid - 1; }
            b = lo; has_b = true;
          }
        }
        D.valid = has_a && has_b && a <= b;
        D.a = (u32)a; D.b = (u32)b;
      }
    }
    live.assign(C, 1);
    n_live = C;
    pressure = o.pressure0;
    host_used.assign(K, 0);
    for (int d = 0; d < 2; ++d) for (int r = 0; r < 2; ++r) busy[d][r].assign(K, 0);
  }

  bool over(u32 k) const { return pressure[k] > pr.gpu_cap; }

  void rebuild_prefix() {
    OT.assign(K + 1, 0);
    for (u32 k = 0; k < K; ++k) OT[k + 1] = OT[k] + (over(k) ? o.dur[k] : 0);
    for (int d = 0; d < 2; ++d) for (int r = 0; r < 2; ++r) {
      FP[d][r].assign(K + 1, 0);
      for (u32 k = 0; k < K; ++k) FP[d][r][k + 1] = FP[d][r][k] + (o.dur[k] - busy[d][r][k]);
    }
  }
  static u64 pref2(const std::vector<u64>& P, u32 K, u64 j) { return j <= K ? P[j] : P[j - K] + P[K]; }

  // sums over doubled-coordinate slot ranges [x, y] (empty if x > y)
  u64 free_time(int d, int r, u64 x, u64 y) const {
    if (x > y) return 0;
    if (mode == 1) return pref2(FP[d][r], K, y + 1) - pref2(FP[d][r], K, x);
    u64 s = 0;
    for (u64 j = x; j <= y; ++j) s += o.dur[j % K] - busy[d][r][j % K];
    return s;
  }
  u64 over_time(u64 x, u64 y) const {
    if (x > y) return 0;
    if (mode == 1) return pref2(OT, K, y + 1) - pref2(OT, K, x);
    u64 s = 0;
    for (u64 j = x; j <= y; ++j) if (over((u32)(j % K))) s += o.dur[j % K];
    return s;
  }

  // "is the channel full during the transfer": can the unreserved channel
  // time inside the slot-rounded transfer windows still carry this tensor
  bool feasible(const Cand& x, int d) const {
    const Dest& D = x.d[d];
    return free_time(d, OUT, (u64)x.L + 1, (u64)D.a - 1) >= D.tau_o &&
           free_time(d, IN, (u64)D.b + 1, (u64)x.R - 1) >= D.tau_i;
  }

  // what evicting s bytes during slots [x, y] takes away from the pressure above the capacity
  u128 benefit(u64 s, u64 x, u64 y) const {
    if (pr.area == 0) return (u128)s * over_time(x, y);              // the tensor's band, where over capacity
    u128 B = 0;
    if (mode == 0) {                                                   // slot by slot: min(size, excess)
      for (u64 j = x; j <= y; ++j) {
        const u32 k = (u32)(j % K);
        if (over(k)) B += (u128)o.dur[k] * std::min(s, pressure[k] - pr.gpu_cap);
      }
    } else {                                                           // the band minus what sticks out below the line
      B = (u128)s * over_time(x, y);
      for (u64 j = x; j <= y; ++j) {
        const u32 k = (u32)(j % K);
        if (over(k) && pressure[k] - pr.gpu_cap < s) B -= (u128)o.dur[k] * (s - (pressure[k] - pr.gpu_cap));
      }
    }
    return B;
  }

  // flash first; host only if flash cannot take it; benefit of that choice
  void score(const Cand& x, int& dest, u128& B) const {
    dest = -1; B = 0;
    for (int d = 0; d < 2; ++d) {
      if (!x.d[d].valid || !feasible(x, d)) continue;
      dest = d;
      B = benefit(x.s, x.d[d].a, x.d[d].b);
      return;
    }
  }

  bool host_has_room(const Cand& x) const {
    u64 mx = 0;
    for (u64 j = (u64)x.L + 1; j + 1 <= x.R; ++j) mx = std::max(mx, host_used[j % K]);
    return x.s <= pr.host_cap && mx <= pr.host_cap - x.s;
  }

  void commit(const Cand& x, int d) {
    const Dest& D = x.d[d];
    for (u64 j = D.a; j <= D.b; ++j) pressure[j % K] -= x.s;
    u64 rem = D.tau_o;                                  // eviction: earliest free channel time first
    for (u64 j = (u64)x.L + 1; j < D.a && rem; ++j) {
      u64 k = j % K, f = o.dur[k] - busy[d][OUT][k], take = std::min(f, rem);
      busy[d][OUT][k] += take; rem -= take;
    }
    rem = D.tau_i;                                      // prefetch: latest free channel time first
    for (u64 j = x.R; j-- > (u64)D.b + 1 && rem;) {
      u64 k = j % K, f = o.dur[k] - busy[d][IN][k], take = std::min(f, rem);
      busy[d][IN][k] += take; rem -= take;
    }
    if (d == HOST)
      for (u64 j = (u64)x.L + 1; j + 1 <= x.R; ++j) host_used[j % K] += x.s;
  }

  u64 max_pressure() const { u64 m = 0; for (u64 p : pressure) m = std::max(m, p); return m; }
  u64 total_over_time() const { u64 s = 0; for (u32 k = 0; k < K; ++k) if (over(k)) s += o.dur[k]; return s; }
};

int plan(Oracle& o, const g10o_params& pr, int mode, u64 max_iters, g10o_summary& S) {
  std::memset(&S, 0, sizeof S);
  for (int d = 0; d < 2; ++d) if (!pr.bw_out[d] || !pr.bw_in[d]) return -1;
  if (pr.rank > 1 || pr.area > 1) return -1;
  Planner P(o, pr, mode);
  P.prepare();
  o.records.clear();
  o.null_cands.clear();
  o.null_iters.clear();
  o.rec_a.clear(); o.rec_b.clear(); o.rec_R.clear();
  o.plan_cap = pr.gpu_cap;
  S.peak_before = P.max_pressure();
  S.overtime_before = P.total_over_time();
  const size_t C = P.cand.size();
  for (;;) {
    if (P.max_pressure() <= pr.gpu_cap) { S.status = 0; break; }       // fits
    if (S.n_iterations >= max_iters) { S.status = 2; break; }
    ++S.n_iterations;
    S.n_cand_evals += P.n_live;
    if (mode == 1) P.rebuild_prefix();
    size_t w = C; int wd = -1; u128 wB = 0;
    u64 wcost = 1;
    for (size_t c = 0; c < C; ++c) {                                    // rank: best key, lowest index
      if (!P.live[c]) continue;
      int d; u128 B;
      P.score(P.cand[c], d, B);
      if (B == 0) continue;
      bool better;
      u64 cost = 1;
      if (pr.rank == 0) {
        better = B > wB;
      } else {                                                          // B / cost > wB / wcost, as fractions
        cost = P.cand[c].d[d].tau_o + P.cand[c].d[d].tau_i;
        better = greater(mul_128_64(B, wcost), mul_128_64(wB, cost));
      }
      if (better) { wB = B; w = c; wd = d; wcost = cost; }
    }
    if (wB == 0) { S.status = 1; break; }                               // nothing beneficial is left
    const Cand& x = P.cand[w];
    P.live[w] = 0; --P.n_live;
    if (wd == HOST && !P.host_has_room(x)) {
      ++S.n_null; o.null_cands.push_back((u32)w); o.null_iters.push_back(S.n_iterations - 1);
      continue;
    }
    g10o_record r;
    std::memset(&r, 0, sizeof r);
    const Dest& D = x.d[wd];
    r.cand = (u32)w; r.tensor = x.t; r.evict_after = x.L;
    r.absent_first = D.a % P.K; r.absent_last = D.b % P.K; r.next_use = x.R % P.K;
    r.dest = (u32)wd; r.wraps = x.R >= P.K;
    r.size = x.s; r.t_out = D.tau_o; r.t_in = D.tau_i;
    r.benefit_lo = (u64)wB; r.benefit_hi = (u64)(wB >> 64);
    o.records.push_back(r);
    o.rec_a.push_back(D.a); o.rec_b.push_back(D.b); o.rec_R.push_back(x.R);
    P.commit(x, wd);
  }
  S.n_migrations = o.records.size();
  S.peak_after = P.max_pressure();
  S.overtime_after = P.total_over_time();
  o.pressure_after = P.pressure;
  o.host_after = P.host_used;
  for (int d = 0; d < 2; ++d) for (int r = 0; r < 2; ++r) o.busy_after[d][r] = P.busy[d][r];
  return 0;
}

// ------------------------------------------------------- smart prefetching
// Section 4.4.  The evicted periods are visited in the order of their latest
// safe prefetch time t_i = (start of the next use) - (prefetch time); equal
// times in plan order.  From the slot before the prefetch the search goes back
// while the slot can hold the tensor (pressure + size <= capacity), not past
// the first absent slot; the prefetch is issued before the earliest such slot
// and the pressure of the slots gained rises by the tensor's size.
//   mode 0: the backward search as stated.
//   mode 1: one forward sweep over the absent window that remembers the last
//           slot that cannot hold the tensor.
int prefetch(Oracle& o, int mode) {
  const size_t n = o.records.size();
  const u32 K = o.K;
  const u64 cap = o.plan_cap;
  o.pf_order.resize(n);
  for (size_t i = 0; i < n; ++i) o.pf_order[i] = (u32)i;
  std::vector<u64> t_safe(n);
  for (size_t i = 0; i < n; ++i) t_safe[i] = start2(o, o.rec_R[i]) - o.records[i].t_in;
  std::stable_sort(o.pf_order.begin(), o.pf_order.end(), [&](u32 x, u32 y) { return t_safe[x] < t_safe[y]; });
  o.pressure_eager = o.pressure_after;
  o.pf_gained.assign(n, 0);
  std::vector<u64>& pr = o.pressure_eager;
  for (u32 i : o.pf_order) {
    const u64 s = o.records[i].size;
    const u64 a = o.rec_a[i], b = o.rec_b[i];
    auto holds = [&](u64 j) { const u64 x = pr[j % K]; return x <= cap && s <= cap - x; };
    u64 p = b + 1;                                   // first slot the tensor is back in
    if (mode == 0) {
      while (p > a && holds(p - 1)) --p;
    } else {
      p = a;
      for (u64 j = a; j <= b; ++j) if (!holds(j)) p = j + 1;
    }
    for (u64 j = p; j <= b; ++j) pr[j % K] += s;
    o.pf_gained[i] = (u32)(b + 1 - p);
  }
  return 0;
}

// ------------------------------------------------------------ plan replay
// Not a step of the paper's planner: a slot-level replay of a finished plan, a small stand-in
// for the breakdown the paper's simulator reports (stall time next to compute time, traffic per
// destination; Sections 7.2-7.3), under kernel durations that may differ from the profiled ones
// the plan was made for (Section 7.6).  The model:
//   * kernels run in order; instructions sit between kernels (Figure 6): the eviction of a
//     migration is issued when kernel `evict_after` has finished, its prefetch when the last
//     absent kernel has finished (with smart prefetching: the earlier slot it was moved to);
//   * every (destination, direction) pair is one channel that serves its transfers one after
//     the other in the order they were issued (same instant: plan order); a transfer takes the
//     eviction / prefetch time of the plan; a prefetch cannot start before its eviction is done;
//   * a kernel starts when the previous one has finished and every prefetch whose tensor it
//     uses is done; the time it waits beyond the previous kernel's end is stall time.
// Two iterations are replayed end to end, every migration in both (a weight evicted in the
// first comes back in the second); what is reported is the second one, the steady state.
struct ReplayOut {
  u64 iter_ns, planned_ns, stall_ns, n_stalled;
  u64 bytes[2], busy_out_ns[2], busy_in_ns[2];
};

int replay(Oracle& o, const u64* dur_in, int eager, ReplayOut& R, std::vector<u64>& late) {
  const u32 K = o.K;
  const size_t n = o.records.size();
  if (eager && o.pf_gained.size() != n) return -1;
  std::vector<u64> dur(o.dur);
  if (dur_in) {
    u128 tot = 0;
    for (u32 k = 0; k < K; ++k) { if (!dur_in[k]) return -1; dur[k] = dur_in[k]; tot += dur_in[k]; }
    if (tot >> 62) return -2;
  }
  std::memset(&R, 0, sizeof R);
  late.assign(n, 0);
  // what happens at the point before kernel j (doubled coordinates, two iterations): (copy, record)
  struct Ev { u32 copy, rec; };
  std::vector<std::vector<Ev>> evict_at(2 * (size_t)K), fetch_at(2 * (size_t)K), use_at(2 * (size_t)K);
  for (u32 c = 0; c < 2; ++c)
    for (size_t i = 0; i < n; ++i) {
      const u64 L = o.records[i].evict_after, b = o.rec_b[i], Ruse = o.rec_R[i];
      const u64 issue = b + 1 - (eager ? o.pf_gained[i] : 0);
      const u64 je = L + 1 + (u64)c * K, jf = issue + (u64)c * K, ju = Ruse + (u64)c * K;
      if (je < 2 * (u64)K) evict_at[je].push_back(Ev{c, (u32)i});
      if (jf < 2 * (u64)K) fetch_at[jf].push_back(Ev{c, (u32)i});
      if (ju < 2 * (u64)K) use_at[ju].push_back(Ev{c, (u32)i});
    }
  auto plan_order = [](const Ev& x, const Ev& y) { return x.rec < y.rec; };   // same instant: plan order
  for (size_t j = 0; j < 2 * (size_t)K; ++j) {
    std::stable_sort(evict_at[j].begin(), evict_at[j].end(), plan_order);
    std::stable_sort(fetch_at[j].begin(), fetch_at[j].end(), plan_order);
  }
  std::vector<u64> E[2] = {std::vector<u64>(n, 0), std::vector<u64>(n, 0)}, F[2] = {std::vector<u64>(n, 0), std::vector<u64>(n, 0)};
  u64 chan_out[2] = {0, 0}, chan_in[2] = {0, 0};
  u64 done_prev = 0, end_first = 0;                  // end of the previous kernel; end of the first iteration
  for (u64 j = 0; j < 2 * (u64)K; ++j) {
    for (const Ev& e : evict_at[j]) {
      const g10o_record& r = o.records[e.rec];
      const u64 t = std::max(done_prev, chan_out[r.dest]) + r.t_out;
      E[e.copy][e.rec] = t; chan_out[r.dest] = t;
    }
    for (const Ev& e : fetch_at[j]) {
      const g10o_record& r = o.records[e.rec];
      const u64 t = std::max(std::max(done_prev, E[e.copy][e.rec]), chan_in[r.dest]) + r.t_in;
      F[e.copy][e.rec] = t; chan_in[r.dest] = t;
    }
    u64 start = done_prev;
    for (const Ev& e : use_at[j]) {
      start = std::max(start, F[e.copy][e.rec]);
      if (j >= K && F[e.copy][e.rec] > done_prev) late[e.rec] = F[e.copy][e.rec] - done_prev;
    }
    if (j >= K && start > done_prev) { R.stall_ns += start - done_prev; ++R.n_stalled; }
    done_prev = start + dur[j % K];
    if (j == (u64)K - 1) end_first = done_prev;
  }
  R.iter_ns = done_prev - end_first;
  for (u32 k = 0; k < K; ++k) R.planned_ns += dur[k];
  for (size_t i = 0; i < n; ++i) {
    const g10o_record& r = o.records[i];
    R.bytes[r.dest] += r.size; R.busy_out_ns[r.dest] += r.t_out; R.busy_in_ns[r.dest] += r.t_in;
  }
  return 0;
}

template <class T>
void copy_out(const std::vector<T>& v, void* dst) { if (!v.empty()) std::memcpy(dst, v.data(), v.size() * sizeof(T)); }

}  // namespace

extern "C" {

int g10o_vitality(const g10o_trace* tr, int mode, void** handle) {
  if (!tr || !handle) return -1;
  Oracle* o = new (std::nothrow) Oracle();
  if (!o) return -3;
  int rc = vitality(*o, *tr, mode);
  if (rc) { delete o; return rc; }
  *handle = o;
  return 0;
}

// out[0..4] = distinct uses, periods, peak bytes, iteration time, plan records
void g10o_counts(void* h, u64* out) {
  Oracle* o = (Oracle*)h;
  out[0] = o->use_k.size(); out[1] = o->per_t.size(); out[2] = o->peak; out[3] = o->T;
  out[4] = o->records.size(); out[5] = o->null_cands.size();
}

// which: 0 use_off 1 use_k 2 birth 3 death 4 per_t 5 per_L 6 per_R 7 start
//        8 pressure0 9 records 10 pressure_after 11 null_cands 12 host_after
//        13 null_iters
//        20 prefetch order 21 slots gained 22 pressure with the earlier prefetches
//        23 / 24 absent window of every record in doubled coordinates
//        16 + 2*d + r : busy_after[d][r]
int g10o_copy(void* h, int which, void* dst) {
  Oracle* o = (Oracle*)h;
  switch (which) {
    case 0: copy_out(o->use_off, dst); break;
    case 1: copy_out(o->use_k, dst); break;
    case 2: copy_out(o->birth, dst); break;
    case 3: copy_out(o->death, dst); break;
    case 4: copy_out(o->per_t, dst); break;
    case 5: copy_out(o->per_L, dst); break;
    case 6: copy_out(o->per_R, dst); break;
    case 7: copy_out(o->start, dst); break;
    case 8: copy_out(o->pressure0, dst); break;
    case 9: copy_out(o->records, dst); break;
    case 10: copy_out(o->pressure_after, dst); break;
    case 11: copy_out(o->null_cands, dst); break;
    case 12: copy_out(o->host_after, dst); break;
    case 13: copy_out(o->null_iters, dst); break;
    case 20: copy_out(o->pf_order, dst); break;
    case 21: copy_out(o->pf_gained, dst); break;
    case 22: copy_out(o->pressure_eager, dst); break;
    case 23: copy_out(o->rec_a, dst); break;
    case 24: copy_out(o->rec_b, dst); break;
    case 16: case 17: case 18: case 19:
      copy_out(o->busy_after[(which - 16) / 2][(which - 16) % 2], dst); break;
    default: return -1;
  }
  return 0;
}

int g10o_plan(void* h, const g10o_params* pr, int mode, u64 max_iters, g10o_summary* out) {
  if (!h || !pr || !out) return -1;
  return plan(*(Oracle*)h, *pr, mode, max_iters, *out);
}

// per candidate and destination: validity and absent window, for window tests
// out arrays have length C: valid (u8), a, b (u32, doubled coords), tau_o, tau_i
int g10o_windows(void* h, const g10o_params* pr, int mode, int dest,
                 uint8_t* valid, u32* a, u32* b, u64* tau_o, u64* tau_i) {
  if (!h || !pr || dest < 0 || dest > 1) return -1;
  Oracle& o = *(Oracle*)h;
  Planner P(o, *pr, mode);
  P.prepare();
  for (size_t c = 0; c < P.cand.size(); ++c) {
    const Dest& D = P.cand[c].d[dest];
    valid[c] = D.valid; a[c] = D.a; b[c] = D.b; tau_o[c] = D.tau_o; tau_i[c] = D.tau_i;
  }
  return 0;
}

// smart prefetching on the plan made last (g10o_plan must have run)
int g10o_prefetch(void* h, int mode) {
  if (!h) return -1;
  return prefetch(*(Oracle*)h, mode);
}

// replay of the plan made last; dur: K durations or NULL (the trace's); eager: use the prefetch
// slots of g10o_prefetch (which must have run).  out[0..9]: iteration, planned, stall, stalled
// kernels, bytes[2], busy out[2], busy in[2]; late: per record, how long its next use in the
// second iteration waited for it beyond the end of the previous kernel
int g10o_replay(void* h, const u64* dur, int eager, u64* out, u64* late) {
  if (!h || !out) return -1;
  Oracle& o = *(Oracle*)h;
  ReplayOut R;
  std::vector<u64> l;
  const int rc = replay(o, dur, eager, R, l);
  if (rc) return rc;
  out[0] = R.iter_ns; out[1] = R.planned_ns; out[2] = R.stall_ns; out[3] = R.n_stalled;
  for (int d = 0; d < 2; ++d) { out[4 + d] = R.bytes[d]; out[6 + d] = R.busy_out_ns[d]; out[8 + d] = R.busy_in_ns[d]; }
  if (late) copy_out(l, late);
  return 0;
}

void g10o_free(void* h) { delete (Oracle*)h; }

}  // extern "C"
