// Slot-level replay of a finished plan under given kernel durations.
//
// Not a step of G10's planner: a small stand-in for the breakdown its simulator reports (stall
// time next to compute time, traffic per destination; evaluation Sections 7.2, 7.3, 7.6).  The
// model: kernels run in order; the eviction of a migration is issued when kernel
// `evict_after` has finished, its prefetch when the last absent kernel has finished (or at the
// earlier slot smart prefetching moved it to); every (destination, direction) pair is one
// channel that serves its transfers one after the other in the order they were issued (same
// instant: plan order), a transfer taking the plan's eviction / prefetch time; a prefetch does
// not start before its eviction is done; a kernel starts when the previous one has finished and
// every prefetch whose tensor it uses is done, and what it waits beyond the previous kernel's
// end is stall time.  Two iterations are replayed end to end with every migration in both (a
// weight evicted in the first comes back in the second); the second one is reported.
//
// On the device: every migration gives up to three events per iteration (eviction issued,
// prefetch issued, tensor used), keyed by (point before kernel j, kind, plan order) and put in
// order by the radix sort.  The replay itself is a serial chain - each completion time depends
// on the channel and on the stalls before it - and runs in one wavefront: 64 events at a time
// are decoded and their operands gathered by the 64 lanes in parallel, then walked in order with
// the state (stall so far, the four channels) in scalar registers and the events' operands read
// lane by lane; a result needed by a later event of the same 64 is passed on through a lane of a
// register, older ones come from the result array.

#include "g10_plan_defs.h"

#include <stdlib.h>
#include <string.h>

using namespace g10;

namespace {

enum { EV_EVICT = 0, EV_FETCH = 1, EV_USE = 2 };

struct ReplayStats {
  u64 iter_ns, stall_ns, n_stalled, pad;
  u64 bytes[2], busy_out[2], busy_in[2];
};

// keys of the events of migration i in both iterations; ~0 for events beyond the second iteration
__global__ __launch_bounds__(G10_BLOCK) void k_rp_events(const g10_migration* __restrict__ rec, const uint2* __restrict__ rec_ab,
                                                        const u32* __restrict__ gained, u32 n, u32 K, u32 rbits,
                                                        u64* __restrict__ keys, ReplayStats* __restrict__ st) {
  __shared__ u64 tmp[G10_WAVES + 1];
  const u32 i = blockIdx.x * G10_BLOCK + threadIdx.x;
  u64 by[2] = {0, 0}, bo[2] = {0, 0}, bi[2] = {0, 0};
  if (i < n) {
    const g10_migration m = rec[i];
    const u32 b2 = rec_ab[i].y, R2 = m.next_use + (m.wraps ? K : 0u);
    const u32 issue = b2 + 1 - (gained ? gained[i] : 0u);
    for (u32 c = 0; c < 2; ++c) {
      const u32 pt[3] = {m.evict_after + 1 + c * K, issue + c * K, R2 + c * K};
      for (u32 t = 0; t < 3; ++t)
        keys[(u64)6 * i + 3 * c + t] = pt[t] < 2 * K ? ((((u64)pt[t] * 4 + t) << (rbits + 1)) | ((u64)i << 1) | c) : NONE64;
    }
    by[m.dest] = m.size_bytes; bo[m.dest] = m.t_out_ns; bi[m.dest] = m.t_in_ns;
  }
  for (u32 d = 0; d < 2; ++d) {                       // traffic and channel time per destination
    const u64 a = block_sum(by[d], tmp), b = block_sum(bo[d], tmp), c = block_sum(bi[d], tmp);
    if (threadIdx.x == 0) {
      if (a) atomicAdd((unsigned long long*)&st->bytes[d], (unsigned long long)a);
      if (b) atomicAdd((unsigned long long*)&st->busy_out[d], (unsigned long long)b);
      if (c) atomicAdd((unsigned long long*)&st->busy_in[d], (unsigned long long)c);
    }
  }
}

// where the eviction and the prefetch of every (iteration, migration) stand in the sorted order
__global__ __launch_bounds__(G10_BLOCK) void k_rp_index(const u64* __restrict__ sorted, u32 ne, u32 n, u32 rbits,
                                                       u32* __restrict__ pos_of) {
  const u32 p = blockIdx.x * G10_BLOCK + threadIdx.x;
  if (p >= ne) return;
  const u64 k = sorted[p];
  if (k == NONE64) return;
  const u32 c = (u32)(k & 1ull), i = (u32)((k >> 1) & ((1ull << rbits) - 1ull)), t = (u32)((k >> (rbits + 1)) & 3ull);
  if (t != EV_USE) pos_of[(u64)(t * 2 + c) * n + i] = p;
}

__device__ __forceinline__ u64 lane_get(u64 v, u32 l) {
  const u32 lo = (u32)__builtin_amdgcn_readlane((int)(u32)v, (int)l), hi = (u32)__builtin_amdgcn_readlane((int)(u32)(v >> 32), (int)l);
  return ((u64)hi << 32) | lo;
}
// the value of lane l replaced by x (x is the same in every lane)
__device__ __forceinline__ u64 lane_put(u64 v, u32 l, u64 x) { return threadIdx.x == l ? x : v; }

__global__ __launch_bounds__(G10_WAVE) void k_replay(const u64* __restrict__ sorted, u32 ne, const g10_migration* __restrict__ rec,
                                                    u32 n, u32 rbits, const u32* __restrict__ pos_of,
                                                    const u64* __restrict__ start, u32 K, u64 T, u64* __restrict__ res,
                                                    u64* __restrict__ late, ReplayStats* __restrict__ st) {
  const u32 lane = threadIdx.x;
  // the state of the walk; the same in every lane
  u64 delta = 0;                        // end of the previous kernel minus its end without any stall
  u64 delta_first = 0;                  // the same when the second iteration begins
  bool second = false;
  u64 ch_out0 = 0, ch_out1 = 0, ch_in0 = 0, ch_in1 = 0;    // when each channel is free again
  u64 stall = 0, n_stalled = 0;
  u32 use_pt = NONE32, stalled_pt = NONE32;
  u64 delta_pt = 0;                     // delta when the uses of the current point began
  // One event per lane, gathered one step ahead of the walk: key, record fields, the point's time
  // without stalls, and the result the event waits for.  While batch b is walked the results of
  // the batches before b are in memory, so an older one is loaded here; one of batch b or of the
  // batch gathered itself is noted by its lane and read from a register during the walk.
  struct Ev { u64 tau, sp, pval; u32 type, i, pt, dest, pin, psrc; bool valid; };   // psrc 0: pval; 1: this batch; 2: the batch before
  auto gather = [&](u32 base, u32 done) -> Ev {           // results of positions < done are in memory
    Ev v;
    v.tau = 0; v.sp = 0; v.pval = 0; v.type = 3; v.i = 0; v.pt = 0; v.dest = 0; v.pin = 0; v.psrc = 0;
    const u32 p = base + lane;
    const u64 k = p < ne ? sorted[p] : NONE64;
    v.valid = k != NONE64;
    if (v.valid) {
      const u32 c = (u32)(k & 1ull);
      v.i = (u32)((k >> 1) & ((1ull << rbits) - 1ull));
      const u64 q = k >> (rbits + 1);
      v.type = (u32)(q & 3ull); v.pt = (u32)(q >> 2);
      const g10_migration m = rec[v.i];
      v.dest = m.dest;
      v.tau = v.type == EV_EVICT ? m.t_out_ns : m.t_in_ns;
      v.sp = v.pt < K ? start[v.pt] : start[v.pt - K] + T;     // end of kernel pt - 1 without any stall
      if (v.type != EV_EVICT) {                                 // its eviction / its prefetch
        const u32 pp = pos_of[(u64)((v.type - 1) * 2 + c) * n + v.i];
        if (pp >= base) { v.psrc = 1; v.pin = pp - base; }
        else if (pp >= done) { v.psrc = 2; v.pin = pp - done; }
        else v.pval = res[pp];
      }
    }
    return v;
  };
  Ev nxt = gather(0, 0);
  u64 resv_prev = 0;                    // results of the batch before, one per lane
  for (u32 base = 0; base < ne; base += G10_WAVE) {
    const Ev cur = nxt;
    const u32 p = base + lane;
    const bool valid = cur.valid;
    const u32 type = cur.type, i = cur.i, pt = cur.pt, dest = cur.dest;
    const u64 tau = cur.tau, sp = cur.sp;
    if (base + G10_WAVE < ne) nxt = gather(base + G10_WAVE, base);   // in flight during the walk
    const u32 cnt = (u32)__popcll(__ballot(valid));             // the valid events come first
    u64 resv = 0, latev = 0;
    // ---- the walk ----------------------------------------------------------------------
    for (u32 e = 0; e < cnt; ++e) {
      const u32 ty = (u32)__builtin_amdgcn_readlane((int)type, (int)e), d = (u32)__builtin_amdgcn_readlane((int)dest, (int)e);
      const u32 ept = (u32)__builtin_amdgcn_readlane((int)pt, (int)e);
      const u64 esp = lane_get(sp, e), etau = lane_get(tau, e);
      if (!second && ept >= K) { second = true; delta_first = delta; }
      u64 pv = 0;
      if (ty != EV_EVICT) {
        const u32 src = (u32)__builtin_amdgcn_readlane((int)cur.psrc, (int)e), pin = (u32)__builtin_amdgcn_readlane((int)cur.pin, (int)e);
        pv = src == 1 ? lane_get(resv, pin) : (src == 2 ? lane_get(resv_prev, pin) : lane_get(cur.pval, e));
      }
      const u64 free_at = esp + delta;                          // end of the previous kernel
      if (ty == EV_EVICT) {
        const u64 chn = d ? ch_out1 : ch_out0;
        const u64 t = (free_at > chn ? free_at : chn) + etau;
        if (d) ch_out1 = t; else ch_out0 = t;
        resv = lane_put(resv, e, t);
      } else if (ty == EV_FETCH) {
        const u64 chn = d ? ch_in1 : ch_in0;
        u64 t = free_at > pv ? free_at : pv;
        t = (t > chn ? t : chn) + etau;
        if (d) ch_in1 = t; else ch_in0 = t;
        resv = lane_put(resv, e, t);
      } else {
        if (ept != use_pt) { use_pt = ept; delta_pt = delta; }
        const u64 prev_end = esp + delta_pt;                    // the previous kernel's end, before any wait of this one
        if (pv > prev_end && ept >= K) latev = lane_put(latev, e, pv - prev_end);
        if (pv > free_at) {                                     // the kernel waits for this prefetch
          if (ept >= K) {
            stall += pv - free_at;
            if (stalled_pt != ept) { stalled_pt = ept; n_stalled += 1; }
          }
          delta = pv - esp;
        }
      }
    }
    // ---- results out ---------------------------------------------------------------------
    if (valid && type != EV_USE) res[p] = resv;
    if (valid && type == EV_USE && pt >= K) late[i] = latev;
    resv_prev = resv;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);                              // the next gather may read what was just written
    if (cnt < G10_WAVE) break;
  }
  if (!second) delta_first = delta;
  if (lane == 0) {
    st->iter_ns = T + delta - delta_first;
    st->stall_ns = stall;
    st->n_stalled = n_stalled;
  }
}

}  // namespace

void replay_free(PlanWork* w) {
  mem_dev_free(w->rp_arena);
  w->rp_arena = nullptr; w->rp_cap = 0;
  free(w->h_rp_late); w->h_rp_late = nullptr;
}

int replay_run(g10_plan_s* h, const u64* dur_ns, u32 eager, g10_replay_result* out) {
  PlanWork* w = h->work;
  if (!w || !w->planned) return G10_EINVAL;
  if (eager && !w->prefetched) return G10_EINVAL;
  hipStream_t s = h->stream;
  const u32 K = h->K, n = (u32)w->plan_n_mig;
  const u64 ne = (u64)6 * n;
  if (ne >= (1ull << 32)) return G10_EINVAL;
  // workspace of its own, sized for this plan's migrations
  if (!w->rp_arena || w->rp_cap < n) {
    G10_HIP(hipStreamSynchronize(s));
    replay_free(w);
    const u64 cap = n ? n : 1, ce = 6 * cap;
    const u64 he = radix_hist_elems(ce), se = scan_scratch_elems(he > ce ? he : ce);
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += (bytes + 255) & ~(size_t)255; return o; };
    const size_t o_keys = take(ce * 8), o_alt = take(ce * 8), o_res = take(ce * 8), o_late = take(cap * 8), o_pos = take(4 * cap * 4),
                 o_hist = take(he * 4), o_scr = take(se * 4), o_st = take(sizeof(ReplayStats)), o_dur = take((u64)K * 8),
                 o_start = take(((u64)K + 1) * 8), o_ts = take(scan_scratch_elems(K) * 8), o_tst = take(128);
    void* q = nullptr;
    G10_TRY(mem_dev_alloc(&q, off));
    char* b = (char*)q;
    w->rp_arena = q; w->rp_cap = (u32)cap;
    w->rp_keys = (u64*)(b + o_keys); w->rp_alt = (u64*)(b + o_alt); w->rp_res = (u64*)(b + o_res); w->rp_late = (u64*)(b + o_late);
    w->rp_pos = (u32*)(b + o_pos); w->rp_hist = (u32*)(b + o_hist); w->rp_scr = (u32*)(b + o_scr); w->rp_stats = (void*)(b + o_st);
    w->rp_dur = (u64*)(b + o_dur); w->rp_start = (u64*)(b + o_start); w->rp_tscr = (u64*)(b + o_ts); w->rp_tstats = (void*)(b + o_tst);
    w->h_rp_late = (u64*)malloc(cap * 8);
    if (!w->h_rp_late) return G10_ENOMEM;
  }
  // the durations to replay with: the given ones, else the ones the plan was made for
  const u64* start = w->start;
  u64 T = w->T;
  if (dur_ns) {
    u64 check[16];
    G10_TRY(slot_times_begin(dur_ns, K, w->rp_dur, w->rp_start, w->rp_tscr, w->rp_tstats, check, s));
    G10_HIP(hipStreamSynchronize(s));
    G10_TRY(slot_times_end(check, &T));
    start = w->rp_start;
  }
  G10_HIP(hipEventRecord(w->ev[0], s));
  ReplayStats* st = (ReplayStats*)w->rp_stats;
  G10_HIP(hipMemsetAsync(st, 0, sizeof(ReplayStats), s));
  if (n) G10_HIP(hipMemsetAsync(w->rp_late, 0, (u64)n * 8, s));
  u32 rbits = bits_for(n ? n - 1 : 0);
  u64 *keys = w->rp_keys, *alt = w->rp_alt;
  if (n) {
    hipLaunchKernelGGL(k_rp_events, dim3((n + G10_BLOCK - 1) / G10_BLOCK), dim3(G10_BLOCK), 0, s, (const g10_migration*)w->records,
                       (const uint2*)w->rec_ab, eager ? (const u32*)w->pf_gained : (const u32*)nullptr, n, K, rbits, keys, st);
    G10_HIP(hipGetLastError());
    G10_TRY(radix_sort_u64(&keys, &alt, ne, bits_for(2ull * K) + 2 + rbits + 1, w->rp_hist, w->rp_scr, s));
    hipLaunchKernelGGL(k_rp_index, dim3((u32)((ne + G10_BLOCK - 1) / G10_BLOCK)), dim3(G10_BLOCK), 0, s, (const u64*)keys, (u32)ne, n, rbits,
                       w->rp_pos);
    G10_HIP(hipGetLastError());
  }
  hipLaunchKernelGGL(k_replay, dim3(1), dim3(G10_WAVE), 0, s, (const u64*)keys, (u32)ne, (const g10_migration*)w->records, n, rbits,
                     (const u32*)w->rp_pos, start, K, T, w->rp_res, w->rp_late, st);
  G10_HIP(hipGetLastError());
  ReplayStats hs;
  G10_HIP(hipMemcpyAsync(&hs, st, sizeof hs, hipMemcpyDeviceToHost, s));
  if (n) G10_HIP(hipMemcpyAsync(w->h_rp_late, w->rp_late, (u64)n * 8, hipMemcpyDeviceToHost, s));
  G10_HIP(hipEventRecord(w->ev[1], s));
  G10_HIP(hipStreamSynchronize(s));
  float ms = 0.f;
  G10_HIP(hipEventElapsedTime(&ms, w->ev[0], w->ev[1]));
  memset(out, 0, sizeof *out);
  out->iter_ns = hs.iter_ns; out->planned_ns = T; out->stall_ns = hs.stall_ns; out->n_stalled = hs.n_stalled;
  for (int d = 0; d < 2; ++d) { out->bytes[d] = hs.bytes[d]; out->busy_out_ns[d] = hs.busy_out[d]; out->busy_in_ns[d] = hs.busy_in[d]; }
  out->n_migrations = n; out->late_ns = w->h_rp_late; out->ms = ms;
  return G10_OK;
}
