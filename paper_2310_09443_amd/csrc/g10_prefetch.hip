// Smart tensor prefetching (G10, Section 4.4) on a finished plan.
//
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

#include "g10_plan_defs.h"

#include <stdlib.h>
#include <string.h>

using namespace g10;

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
                       w->start, K, w->T, keys, ord);
    G10_HIP(hipGetLastError());
    G10_TRY(radix_sort_u64_pairs(&keys, &alt, &ord, &oalt, n, bits_for(2 * w->T), w->hist, w->scratch32, s));
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
  w->prefetched = true;
  return G10_OK;
}
