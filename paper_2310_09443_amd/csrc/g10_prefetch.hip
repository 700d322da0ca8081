// Smart tensor prefetching (G10, Section 4.4) on a finished plan.
//
// The evicted periods are visited in the order of their latest safe prefetch
// time; each prefetch moves back, in whole kernel slots and not past the first
// absent slot, to the earliest slot from which every slot up to the old
// prefetch can hold the tensor (pressure + size <= capacity); the pressure of
// the slots gained rises by the tensor's size.  Every step depends on the
// pressure the earlier ones left, so this is a serial chain like the eviction
// loop: one wavefront walks it (a workgroup sets the timeline up and finishes
// it), the pressure in HBM / L2, per chunk a lazy add and the chunk maximum in
// LDS.  The search asks the chunk maxima which chunk can hold the last slot
// that cannot take the tensor and scans only that chunk; the update adds
// lazily to whole chunks and slot by slot at the ends.

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

__device__ __forceinline__ u64 lane_value64(u64 v, u32 l) {      // lane l's v (l the same in the whole wavefront)
  const u32 lo = (u32)__builtin_amdgcn_readlane((int)(u32)v, (int)l), hi = (u32)__builtin_amdgcn_readlane((int)(u32)(v >> 32), (int)l);
  return ((u64)hi << 32) | lo;
}

struct PfShared {
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

  // The chain itself runs in the first wavefront alone: every step waits for the one before, and one wavefront
  // needs no barrier between them (the others wait at the barrier below; they set up and finish the timeline).
  // Most prefetches cannot move at all: the slot just before them cannot take the tensor.  That test reads one
  // slot, and the pressure changes only when a prefetch does move; so 64 records are tested at once, one per
  // lane; those before the first that passes are done - nothing gained - and only that one takes the search.
  // (the records of the next 64 are loaded before that search: they do not depend on it)
  if (wave == 0) {
    const u32 ncl = (nch + 63u) / 64u;             // chunks per lane: lane, lane + 64, ...
    u64 n_moved = 0, slots = 0;
    u32 it = 0;
    u32 nr = 0, na = 0, nb = 0;
    u64 nsz = 0;
    if (lane < n) { nr = order[lane]; nsz = rec[nr].size_bytes; const uint2 ab = rec_ab[nr]; na = ab.x; nb = ab.y; }
    while (it < n) {
      const u32 idx = it + lane;
      bool pass = false;
      if (idx < n) {
        const u32 bb = nb >= K ? nb - K : nb;
        pass = nsz <= cap && E[bb] + ladd[bb >> shift_ch] <= cap - nsz;
      }
      const u64 pm = __ballot(pass);
      const u32 left = n - it < 64u ? n - it : 64u;
      const u32 f = pm ? (u32)__builtin_ctzll(pm) : left;      // records it .. it + f - 1 stay where they are
      if (lane < f) { gained[nr] = 0u; last[nr] = nb >= K ? nb - K : nb; }
      u32 r = 0, a = 0, b = 0;
      u64 s = 0;
      if (pm) {
        r = (u32)__builtin_amdgcn_readlane((int)nr, (int)f);
        a = (u32)__builtin_amdgcn_readlane((int)na, (int)f);
        b = (u32)__builtin_amdgcn_readlane((int)nb, (int)f);
        s = lane_value64(nsz, f);
      }
      it += f + (pm ? 1u : 0u);
      if (it + lane < n) { nr = order[it + lane]; nsz = rec[nr].size_bytes; const uint2 ab = rec_ab[nr]; na = ab.x; nb = ab.y; }
      if (!pm) continue;

      // the earliest slot from which every slot up to b can hold the tensor: one past the last slot of [a, b]
      // that cannot.  The chunk maxima say which piece of a chunk may hold it, highest first; that piece is scanned.
      const u64 lim = cap - s;                     // a slot holds the tensor iff its pressure <= lim
      u32 upper = b;                               // the search is still open over [a, upper]
      u32 p = a;
      while (true) {
        unsigned long long cd = 0ull;              // (upper end + 1) << 32 | lower end of the highest such piece
        for (u32 q = 0; q < ncl; ++q) {
          const u32 c = q * 64u + lane;
          if (c < nch && cmax[c] > lim) {          // the two places of the chunk on the doubled timeline
            const u64 s0 = (u64)c * CH, s1 = (s0 + CH - 1 < (u64)K - 1) ? s0 + CH - 1 : (u64)K - 1;
#pragma unroll
            for (u32 rep = 0; rep < 2; ++rep) {
              const u64 o = rep ? K : 0u;
              const u64 plo = s0 + o > a ? s0 + o : a, phi = s1 + o < upper ? s1 + o : upper;
              if (plo <= phi) { const unsigned long long v = ((phi + 1) << 32) | plo; cd = v > cd ? v : cd; }
            }
          }
        }
        cd = wave_max((u64)cd);
        if (cd == 0ull) break;                     // no chunk holds a refusing slot inside [a, upper]
        const u32 hi = (u32)(cd >> 32) - 1u, lo = (u32)cd;
        u32 best = 0;                              // doubled coordinate + 1 of the last refusing slot of the piece
        for (u64 j0 = lo; j0 <= hi; j0 += 256) {   // four loads in flight per lane (64-bit counter: hi may be near 2^32)
          u64 x[4];
#pragma unroll
          for (u32 i = 0; i < 4; ++i) {
            const u64 j = j0 + i * 64u + lane;
            const u32 jj = j >= K ? (u32)(j - K) : (u32)j;
            x[i] = j <= hi ? E[jj] + ladd[jj >> shift_ch] : 0ull;
          }
#pragma unroll
          for (u32 i = 0; i < 4; ++i)
            if (x[i] > lim) best = (u32)j0 + i * 64u + lane + 1;         // ascending: the last one stays
        }
        best = wave_max(best);
        if (best) { p = best; break; }
        if (lo == a) break;                        // nothing refuses in [a, upper]
        upper = lo - 1;
      }
      const u32 g = b + 1 - p;
      if (lane == 0) {
        gained[r] = g;
        const u32 nl = b - g;                      // last absent slot left (one before a if none)
        last[r] = nl >= K ? nl - K : nl;
      }
      if (g) {                                     // the slots gained take the tensor
        n_moved += 1; slots += g;
        for (u32 q = 0; q < ncl; ++q) {
          const u32 c = q * 64u + lane;
          u32 len = 0, cv = 0;
          if (c < nch) cv = cover(c, CH, K, p, b, len);
          if (cv && cv == len) { ladd[c] += s; cmax[c] += s; }
          u64 part = __ballot(cv && cv != len);    // chunks the range cuts: slot by slot, the whole wavefront on each
          while (part) {
            const u32 cc = q * 64u + (u32)__builtin_ctzll(part);
            part &= part - 1;
            const u64 lz = ladd[cc];
            u64 m = 0;
            for (u32 st = 0; st < spt; ++st) {
              const u32 j0 = cc * CH + st * 256u + lane * 4u;
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
            if (lane == 0) cmax[cc] = m;
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");   // the next tests read the slots just written
      }
    }
    if (lane == 0) { S->n_moved = n_moved; S->slots = slots; }
  }
  __syncthreads();
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
    if (!w->h_pf_order || !w->h_pf_gained || !w->h_pf_last || !w->h_pf_pressure) {
      // all four or none: the next call must find the same state as the first
      free(w->h_pf_order); free(w->h_pf_gained); free(w->h_pf_last); free(w->h_pf_pressure);
      w->h_pf_order = nullptr; w->h_pf_gained = nullptr; w->h_pf_last = nullptr; w->h_pf_pressure = nullptr;
      return G10_ENOMEM;
    }
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
  const size_t lds = ((size_t)2 * w->nch * 8 + sizeof(PfShared) + 15) & ~(size_t)15;
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
