// Tensor vitality analysis on the device (G10, Section 4.2).
//
//   pairs (kernel, tensor)  --pack-->  64-bit keys (tensor << kbits | kernel)
//     --LSD radix sort, 8-bit digits, only the significant digits-->
//     --adjacent compare + scan-->  distinct keys = per-tensor use lists
//     --adjacent difference-->      inactive periods (gap of >= 1 whole kernel),
//                                   plus the cross-iteration period of globals
//   lifetimes --interval add into a difference array + scan--> pressure[K]
//     --wavefront-shuffle max--> peak
//
// Everything is integer work bound by memory traffic; no matrix cores.

#include "g10_internal.h"

#include <stdio.h>
#include <stdlib.h>
#include <string.h>

namespace {

constexpr int ITEMS = 8;                        // elements per thread in tiled kernels
constexpr int TILE = G10_BLOCK * ITEMS;         // 2048

// ===========================================================================
// device-wide exclusive scan
// ===========================================================================
template <class T>
__global__ __launch_bounds__(G10_BLOCK) void k_scan_tiles(const T* __restrict__ in, T* out, u64 n, T* sums) {
  __shared__ T tmp[G10_WAVES + 1];
  const u64 base = (u64)blockIdx.x * TILE + (u64)threadIdx.x * ITEMS;
  T v[ITEMS];
  T acc = 0;
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) {
    v[i] = base + i < n ? in[base + i] : (T)0;
    acc += v[i];
  }
  T total;
  T run = block_scan_excl(acc, tmp, total);
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) {
    if (base + i < n) out[base + i] = run;
    run += v[i];
  }
  if (threadIdx.x == 0) {
    if (sums) sums[blockIdx.x] = total;
    else out[n] = total;                        // single tile: finished
  }
}

template <class T>
__global__ __launch_bounds__(G10_BLOCK) void k_scan_add(T* out, u64 n, const T* __restrict__ sums, u32 nb) {
  const T add = sums[blockIdx.x];
  const u64 base = (u64)blockIdx.x * TILE + (u64)threadIdx.x * ITEMS;
#pragma unroll
  for (int i = 0; i < ITEMS; ++i)
    if (base + i < n) out[base + i] += add;
  if (blockIdx.x == 0 && threadIdx.x == 0) out[n] = sums[nb];
}

template <class T>
int scan_excl(const T* in, T* out, u64 n, T* scratch, hipStream_t s) {
  if (n == 0) {                                  // out[0] = 0
    G10_HIP(hipMemsetAsync(out, 0, sizeof(T), s));
    return G10_OK;
  }
  const u64 nb = (n + TILE - 1) / TILE;
  if (nb == 1) {
    hipLaunchKernelGGL(k_scan_tiles<T>, dim3(1), dim3(G10_BLOCK), 0, s, in, out, n, (T*)nullptr);
    G10_HIP(hipGetLastError());
    return G10_OK;
  }
  hipLaunchKernelGGL(k_scan_tiles<T>, dim3((u32)nb), dim3(G10_BLOCK), 0, s, in, out, n, scratch);
  G10_HIP(hipGetLastError());
  int rc = scan_excl<T>(scratch, scratch, nb, scratch + nb + 1, s);
  if (rc) return rc;
  hipLaunchKernelGGL(k_scan_add<T>, dim3((u32)nb), dim3(G10_BLOCK), 0, s, out, n, scratch, (u32)nb);
  G10_HIP(hipGetLastError());
  return G10_OK;
}

// ===========================================================================
// validation of array contents (one pass each, flags + wide sums)
// ===========================================================================
struct VitStats {
  u32 bad_index, zero_dur, zero_size, size_overflow;
  u32 big_size, pad;         // a tensor of 2^43 bytes or more
  u64 max_size;              // the largest tensor
  u64 dur_lo, dur_hi;        // sum of low / high 32-bit halves of the durations
  u64 used_lo, used_hi;      // same for the sizes of used tensors
  u64 n_uses, n_periods, peak;
};

__global__ __launch_bounds__(G10_BLOCK) void k_check_dur(const u64* __restrict__ dur, u32 K, VitStats* st) {
  __shared__ u64 tmp[G10_WAVES + 1];
  u64 lo = 0, hi = 0;
  u32 zero = 0;
  for (u64 i = (u64)blockIdx.x * G10_BLOCK + threadIdx.x; i < K; i += (u64)gridDim.x * G10_BLOCK) {
    u64 d = dur[i];
    zero |= d == 0;
    lo += d & 0xffffffffull;
    hi += d >> 32;
  }
  lo = block_sum(lo, tmp);
  hi = block_sum(hi, tmp);
  if (__any(zero) && lane_id() == 0) atomicOr(&st->zero_dur, 1u);
  if (threadIdx.x == 0) {
    atomicAdd((unsigned long long*)&st->dur_lo, (unsigned long long)lo);
    atomicAdd((unsigned long long*)&st->dur_hi, (unsigned long long)hi);
  }
}

__global__ __launch_bounds__(G10_BLOCK) void k_check_size(const u64* __restrict__ size, u32 N, VitStats* st) {
  u32 zero = 0, ovf = 0, big = 0;
  u64 mx = 0;
  for (u64 i = (u64)blockIdx.x * G10_BLOCK + threadIdx.x; i < N; i += (u64)gridDim.x * G10_BLOCK) {
    u64 s = size[i];
    mx = s > mx ? s : mx;
    zero |= s == 0;
    ovf |= s > 0xffffffffffffffffull / 1000ull;
    big |= (s >> 43) != 0;
  }
  if (__any(zero) && lane_id() == 0) atomicOr(&st->zero_size, 1u);
  if (__any(ovf) && lane_id() == 0) atomicOr(&st->size_overflow, 1u);
  if (__any(big) && lane_id() == 0) atomicOr(&st->big_size, 1u);
  // (atomics on one address queue up behind each other: one per workgroup, and only where it can still raise the maximum)
  __shared__ u64 tmp[G10_WAVES + 1];
  mx = block_max(mx, tmp);
  if (threadIdx.x == 0 && mx > *(volatile u64*)&st->max_size) atomicMax((unsigned long long*)&st->max_size, (unsigned long long)mx);
}

// ===========================================================================
// use lists: key pack, radix sort, distinct
// ===========================================================================
// Sort keys (tensor, kernel) of the pairs.  A pair that names no kernel or no tensor of the trace is
// reported and stands in as (0, 0): every later kernel then indexes inside its arrays, and the host
// rejects the trace when it reads the report at the end of the analysis.
__global__ __launch_bounds__(G10_BLOCK) void k_pack(const u32* __restrict__ uk, const u32* __restrict__ ut, u64 P,
                                                   u32 K, u32 N, u32 kbits, u64* __restrict__ keys, VitStats* st) {
  u32 bad = 0;
  for (u64 i = (u64)blockIdx.x * G10_BLOCK + threadIdx.x; i < P; i += (u64)gridDim.x * G10_BLOCK) {
    u32 k = uk[i], t = ut[i];
    if (k >= K || t >= N) { bad = 1; k = 0; t = 0; }
    keys[i] = ((u64)t << kbits) | k;
  }
  if (__any(bad) && lane_id() == 0) atomicOr(&st->bad_index, 1u);
}

// Tile layout of the sort kernels: wavefront w of a workgroup owns the
// contiguous keys [tile + w*512, tile + (w+1)*512); in round r lane l holds key
// tile + w*512 + r*64 + l.  Key order = (wavefront, round, lane): that is what
// makes the per-digit ranks stable.
__device__ __forceinline__ u64 tile_index(u32 r) {
  return (u64)blockIdx.x * TILE + (u64)wave_id() * (G10_WAVE * ITEMS) + (u64)r * G10_WAVE + lane_id();
}

// The two kernels of a sort pass; blockIdx.x is the tile (the batched forms below put the job in blockIdx.y).
template <class KT>
__device__ __forceinline__ void radix_hist_tile(const KT* __restrict__ keys, u64 P, u32 shift, u32* __restrict__ hist, u32 nblocks,
                                                u32* cnt) {
  cnt[threadIdx.x] = 0;
  __syncthreads();
#pragma unroll
  for (u32 r = 0; r < ITEMS; ++r) {
    u64 i = tile_index(r);
    if (i < P) atomicAdd(&cnt[(keys[i] >> shift) & 255u], 1u);
  }
  __syncthreads();
  hist[(u64)threadIdx.x * nblocks + blockIdx.x] = cnt[threadIdx.x];     // digit-major
}

template <class KT>
__global__ __launch_bounds__(G10_BLOCK) void k_radix_hist(const KT* __restrict__ keys, u64 P, u32 shift,
                                                         u32* __restrict__ hist, u32 nblocks) {
  __shared__ u32 cnt[256];
  radix_hist_tile<KT>(keys, P, shift, hist, nblocks, cnt);
}

template <class KT, bool PAIRS>
__device__ __forceinline__ void radix_scatter_tile(const KT* __restrict__ keys, KT* __restrict__ out,
                                                   const u32* __restrict__ vals, u32* __restrict__ vout,
                                                   u64 P, u32 shift, const u32* __restrict__ offs,
                                                   u32 nblocks, u32 (*cnt)[256], u32* gbase) {
  for (u32 i = threadIdx.x; i < G10_WAVES * 256; i += G10_BLOCK) (&cnt[0][0])[i] = 0;
  __syncthreads();
  const u32 w = wave_id(), l = lane_id();
  const u64 lt = (1ull << l) - 1ull;
  KT key[ITEMS];
  u32 rank[ITEMS], val[ITEMS];
#pragma unroll
  for (u32 r = 0; r < ITEMS; ++r) {
    const u64 i = tile_index(r);
    const bool ok = i < P;
    key[r] = ok ? keys[i] : (KT)0;
    val[r] = PAIRS && ok ? (vals ? vals[i] : (u32)i) : 0u;     // no values given: the positions themselves
    const u32 dig = (u32)(key[r] >> shift) & 255u;
    u64 peers = __ballot(ok);
#pragma unroll
    for (u32 b = 0; b < 8; ++b) {
      const u64 m = __ballot((dig >> b) & 1u);
      peers &= ((dig >> b) & 1u) ? m : ~m;
    }
    const u32 before = cnt[w][dig];          // all peers read, then the first one adds
    rank[r] = before + __popcll(peers & lt);
    __builtin_amdgcn_wave_barrier();
    if (ok && (peers & lt) == 0) cnt[w][dig] = before + __popcll(peers);
    __builtin_amdgcn_wave_barrier();
  }
  __syncthreads();
  {                                           // one thread per digit: offsets of the wavefronts
    const u32 d = threadIdx.x;
    u32 run = 0;
#pragma unroll
    for (u32 ww = 0; ww < G10_WAVES; ++ww) {
      u32 c = cnt[ww][d];
      cnt[ww][d] = run;
      run += c;
    }
    gbase[d] = offs[(u64)d * nblocks + blockIdx.x];
  }
  __syncthreads();
#pragma unroll
  for (u32 r = 0; r < ITEMS; ++r) {
    const u64 i = tile_index(r);
    if (i < P) {
      const u32 dig = (u32)(key[r] >> shift) & 255u;
      const u64 pos = (u64)gbase[dig] + cnt[w][dig] + rank[r];
      out[pos] = key[r];
      if (PAIRS) vout[pos] = val[r];
    }
  }
}

template <class KT, bool PAIRS>
__global__ __launch_bounds__(G10_BLOCK) void k_radix_scatter(const KT* __restrict__ keys, KT* __restrict__ out,
                                                            const u32* __restrict__ vals, u32* __restrict__ vout,
                                                            u64 P, u32 shift, const u32* __restrict__ offs,
                                                            u32 nblocks) {
  __shared__ u32 cnt[G10_WAVES][256];        // per wavefront: running count per digit
  __shared__ u32 gbase[256];
  radix_scatter_tile<KT, PAIRS>(keys, out, vals, vout, P, shift, offs, nblocks, cnt, gbase);
}

// ---- many sorts of (32-bit key, 32-bit value) pairs at once: job = blockIdx.y -------------------------
__global__ __launch_bounds__(G10_BLOCK) void k_radix_hist_jobs(const SortJob* __restrict__ jobs, u32 shift, u32 flip) {
  __shared__ u32 cnt[256];
  const SortJob j = jobs[blockIdx.y];
  if (blockIdx.x >= j.nb) return;
  radix_hist_tile<u32>(flip ? j.alt : j.keys, j.n, shift, j.hist, j.nb, cnt);
}

// exclusive scan of a job's 256 * nb counts in place, one workgroup of 1024 threads per job
__global__ __launch_bounds__(1024) void k_radix_scan_jobs(const SortJob* __restrict__ jobs) {
  __shared__ u32 wsum[16];
  __shared__ u32 carry_s;
  const SortJob j = jobs[blockIdx.y];
  const u32 total = 256u * j.nb, w = threadIdx.x >> 6, l = threadIdx.x & 63u;
  u32* h = j.hist;
  u32 carry = 0;
  for (u32 base = 0; base < total; base += 4096u) {
    const u32 i = base + threadIdx.x * 4u;
    u32 v[4];
#pragma unroll
    for (u32 q = 0; q < 4; ++q) v[q] = i + q < total ? h[i + q] : 0u;
    const u32 mine = v[0] + v[1] + v[2] + v[3];
    const u32 inc = wave_scan_incl(mine);
    if (l == 63u) wsum[w] = inc;
    __syncthreads();
    if (w == 0) {
      const u32 x = l < 16u ? wsum[l] : 0u;
      const u32 xi = wave_scan_incl(x);
      if (l < 16u) wsum[l] = xi - x;
      if (l == 15u) carry_s = xi;
    }
    __syncthreads();
    u32 run = carry + wsum[w] + inc - mine;
#pragma unroll
    for (u32 q = 0; q < 4; ++q) {
      if (i + q < total) h[i + q] = run;
      run += v[q];
    }
    carry += carry_s;
    __syncthreads();                          // wsum and carry_s are read before the next round writes them
  }
}

__global__ __launch_bounds__(G10_BLOCK) void k_radix_scatter_jobs(const SortJob* __restrict__ jobs, u32 shift, u32 flip, u32 iota) {
  __shared__ u32 cnt[G10_WAVES][256];
  __shared__ u32 gbase[256];
  const SortJob j = jobs[blockIdx.y];
  if (blockIdx.x >= j.nb) return;
  radix_scatter_tile<u32, true>(flip ? j.alt : j.keys, flip ? j.keys : j.alt, iota ? (const u32*)nullptr : (const u32*)(flip ? j.valt : j.vals),
                                flip ? j.vals : j.valt, j.n, shift, j.hist, j.nb, cnt, gbase);
}

__global__ __launch_bounds__(G10_BLOCK) void k_flag_distinct(const u64* __restrict__ keys, u64 P, u32* __restrict__ flag) {
  for (u64 i = (u64)blockIdx.x * G10_BLOCK + threadIdx.x; i < P; i += (u64)gridDim.x * G10_BLOCK)
    flag[i] = (i == 0 || keys[i] != keys[i - 1]) ? 1u : 0u;
}

__global__ __launch_bounds__(G10_BLOCK) void k_compact_distinct(const u64* __restrict__ keys, u64 P,
                                                               const u32* __restrict__ pos, u64* __restrict__ ukeys,
                                                               u32* __restrict__ use_k, u32 kbits) {
  for (u64 i = (u64)blockIdx.x * G10_BLOCK + threadIdx.x; i < P; i += (u64)gridDim.x * G10_BLOCK)
    if (pos[i + 1] != pos[i]) {
      ukeys[pos[i]] = keys[i];
      use_k[pos[i]] = (u32)(keys[i] & ((1ull << kbits) - 1ull));
    }
}

// use_off[t] = first position whose key has tensor >= t  (t in [0, N])
__global__ __launch_bounds__(G10_BLOCK) void k_use_off(const u64* __restrict__ ukeys, const u32* __restrict__ n_uses_p,
                                                      u32 N, u32 kbits, u64* __restrict__ use_off) {
  const u64 n = *n_uses_p;
  for (u64 t = (u64)blockIdx.x * G10_BLOCK + threadIdx.x; t <= N; t += (u64)gridDim.x * G10_BLOCK) {
    const u64 want = t << kbits;
    u64 lo = 0, hi = n;
    while (lo < hi) {
      u64 mid = (lo + hi) >> 1;
      if (ukeys[mid] >= want) hi = mid; else lo = mid + 1;
    }
    use_off[t] = lo;
  }
}

// ===========================================================================
// inactive periods: adjacent difference inside each tensor's use list
// ===========================================================================
// Position i of the distinct keys ends an in-iteration period when its
// predecessor is the same tensor at least two kernels earlier; the last use of
// a global tensor additionally starts the cross-iteration period.
__device__ __forceinline__ void period_at(const u64* ukeys, const u64* use_off, const uint8_t* glob, u64 i, u32 K,
                                          u32 kbits, u32 no_wrap, bool& inner, bool& wrap, u32& t, u32& k, u32& kprev,
                                          u32& kfirst) {
  const u64 key = ukeys[i];
  const u64 kmask = (1ull << kbits) - 1ull;
  t = (u32)(key >> kbits);
  k = (u32)(key & kmask);
  const u64 b = use_off[t], e = use_off[t + 1];
  inner = false;
  wrap = false;
  kprev = 0;
  kfirst = 0;
  if (i > b) {
    kprev = (u32)(ukeys[i - 1] & kmask);
    inner = k - kprev >= 2;
  }
  if (i + 1 == e && glob[t] && !no_wrap) {
    kfirst = (u32)(ukeys[b] & kmask);
    wrap = (u64)kfirst + K - k >= 2;
  }
}

__global__ __launch_bounds__(G10_BLOCK) void k_period_count(const u64* __restrict__ ukeys, const u64* __restrict__ use_off,
                                                           const uint8_t* __restrict__ glob, const u32* __restrict__ n_uses_p,
                                                           u32 K, u32 kbits, u32 no_wrap, u32* __restrict__ cnt) {
  const u64 n = *n_uses_p;
  for (u64 i = (u64)blockIdx.x * G10_BLOCK + threadIdx.x; i < n; i += (u64)gridDim.x * G10_BLOCK) {
    bool inner, wrap;
    u32 t, k, kp, kf;
    period_at(ukeys, use_off, glob, i, K, kbits, no_wrap, inner, wrap, t, k, kp, kf);
    cnt[i] = (u32)inner + (u32)wrap;
  }
}

__global__ __launch_bounds__(G10_BLOCK) void k_period_write(const u64* __restrict__ ukeys, const u64* __restrict__ use_off,
                                                           const uint8_t* __restrict__ glob, const u32* __restrict__ n_uses_p,
                                                           u32 K, u32 kbits, u32 no_wrap, const u32* __restrict__ pos,
                                                           u32* __restrict__ per_t, u32* __restrict__ per_L,
                                                           u32* __restrict__ per_R) {
  const u64 n = *n_uses_p;
  for (u64 i = (u64)blockIdx.x * G10_BLOCK + threadIdx.x; i < n; i += (u64)gridDim.x * G10_BLOCK) {
    bool inner, wrap;
    u32 t, k, kp, kf;
    period_at(ukeys, use_off, glob, i, K, kbits, no_wrap, inner, wrap, t, k, kp, kf);
    u32 o = pos[i];
    if (inner) { per_t[o] = t; per_L[o] = kp; per_R[o] = k; ++o; }
    if (wrap) { per_t[o] = t; per_L[o] = k; per_R[o] = kf + K; }
  }
}

// the periods gathered in the order of their start (order[i]: index of the i-th) as {L, R, tensor, index}
__global__ __launch_bounds__(G10_BLOCK) void k_gather_periods(const u32* __restrict__ order, u64 C,
                                                             const u32* __restrict__ per_t, const u32* __restrict__ per_L,
                                                             const u32* __restrict__ per_R, const u64* __restrict__ size,
                                                             uint4* __restrict__ out, u64* __restrict__ out_size) {
  for (u64 i = (u64)blockIdx.x * G10_BLOCK + threadIdx.x; i < C; i += (u64)gridDim.x * G10_BLOCK) {
    const u32 c = order[i];
    const u32 t = per_t[c];
    out[i] = make_uint4(per_L[c], per_R[c], t, c);
    out_size[i] = size[t];
  }
}

// ===========================================================================
// memory pressure: interval adds into a difference array, scan, max
// ===========================================================================
__global__ __launch_bounds__(G10_BLOCK) void k_fill_u64(u64* p, u64 n, u64 v) {
  for (u64 i = (u64)blockIdx.x * G10_BLOCK + threadIdx.x; i < n; i += (u64)gridDim.x * G10_BLOCK) p[i] = v;
}
__global__ __launch_bounds__(G10_BLOCK) void k_fill_u32(u32* p, u64 n, u32 v) {
  for (u64 i = (u64)blockIdx.x * G10_BLOCK + threadIdx.x; i < n; i += (u64)gridDim.x * G10_BLOCK) p[i] = v;
}

__global__ __launch_bounds__(G10_BLOCK) void k_lifetime_adds(const u64* __restrict__ ukeys, const u64* __restrict__ use_off,
                                                            const u64* __restrict__ size, const uint8_t* __restrict__ glob,
                                                            u32 N, u32 K, u32 kbits, u64* diff, VitStats* st) {
  __shared__ u64 tmp[G10_WAVES + 1];
  const u64 kmask = (1ull << kbits) - 1ull;
  u64 gsum = 0, lo32 = 0, hi32 = 0;
  for (u64 t = (u64)blockIdx.x * G10_BLOCK + threadIdx.x; t < N; t += (u64)gridDim.x * G10_BLOCK) {
    const u64 b = use_off[t], e = use_off[t + 1];
    if (b == e) continue;                       // never used: ignored everywhere
    const u64 s = size[t];
    lo32 += s & 0xffffffffull;
    hi32 += s >> 32;
    if (glob[t]) {
      gsum += s;                                // resident in every slot
    } else {
      const u32 birth = (u32)(ukeys[b] & kmask), death = (u32)(ukeys[e - 1] & kmask);
      atomicAdd((unsigned long long*)&diff[birth], (unsigned long long)s);
      atomicAdd((unsigned long long*)&diff[death + 1], (unsigned long long)(0ull - s));
    }
  }
  gsum = block_sum(gsum, tmp);
  lo32 = block_sum(lo32, tmp);
  hi32 = block_sum(hi32, tmp);
  if (threadIdx.x == 0) {
    if (gsum) {
      atomicAdd((unsigned long long*)&diff[0], (unsigned long long)gsum);
      atomicAdd((unsigned long long*)&diff[K], (unsigned long long)(0ull - gsum));
    }
    atomicAdd((unsigned long long*)&st->used_lo, (unsigned long long)lo32);
    atomicAdd((unsigned long long*)&st->used_hi, (unsigned long long)hi32);
  }
}

__global__ __launch_bounds__(G10_BLOCK) void k_max_u64(const u64* __restrict__ v, u64 n, u64* out) {
  __shared__ u64 tmp[G10_WAVES + 1];
  u64 m = 0;
  for (u64 i = (u64)blockIdx.x * G10_BLOCK + threadIdx.x; i < n; i += (u64)gridDim.x * G10_BLOCK) m = v[i] > m ? v[i] : m;
  m = block_max(m, tmp);                        // wavefront shuffles, then 4 partials
  if (threadIdx.x == 0) atomicMax((unsigned long long*)out, (unsigned long long)m);
}

__global__ void k_store_counts(const u32* n_uses_p, const u32* n_per_p, VitStats* st) {
  st->n_uses = *n_uses_p;
  st->n_periods = *n_per_p;
}

inline u32 grid_for(u64 n, u32 cap = 4096) {
  u64 g = (n + G10_BLOCK - 1) / G10_BLOCK;
  return (u32)(g < 1 ? 1 : (g > cap ? cap : g));
}

inline u32 bits_for(u64 max_value) {            // bits needed to hold values 0..max_value, at least 1
  u32 b = 1;
  while (b < 64 && (max_value >> b)) ++b;
  return b;
}

// One device allocation carved into arrays (every hipMalloc / hipFree costs about 0.1 ms of host
// time, and the analysis needs twenty arrays).
struct Pool {
  char* base = nullptr;
  size_t off = 0, cap = 0;
  static size_t need(u64 elems, size_t size) { return (((elems ? elems : 1) * size) + 255) & ~(size_t)255; }
  int reserve(size_t bytes) {
    void* q = nullptr;
    G10_TRY(mem_dev_alloc(&q, bytes));
    base = (char*)q; cap = bytes; off = 0;
    return G10_OK;
  }
  template <class T>
  int take(T** out, u64 elems) {
    const size_t b = need(elems, sizeof(T));
    if (off + b > cap) return G10_ENOMEM;
    *out = (T*)(base + off);
    off += b;
    return G10_OK;
  }
};

}  // namespace

size_t scan_scratch_elems(u64 n) {
  size_t tot = 0;
  while (n > (u64)TILE) {
    n = (n + TILE - 1) / TILE;
    tot += n + 1;
  }
  return tot + 2;
}
int scan_excl_u32(const u32* in, u32* out, u64 n, u32* scratch, hipStream_t s) { return scan_excl<u32>(in, out, n, scratch, s); }
int scan_excl_u64(const u64* in, u64* out, u64 n, u64* scratch, hipStream_t s) { return scan_excl<u64>(in, out, n, scratch, s); }

int g10_hip_fail(hipError_t e, const char* file, int line) {
  if (getenv("G10_LOG")) fprintf(stderr, "g10: HIP error %d (%s) at %s:%d\n", (int)e, hipGetErrorString(e), file, line);
  (void)hipGetLastError();
  return e == hipErrorOutOfMemory ? G10_ENOMEM : G10_EDEVICE;
}


size_t radix_hist_elems(u64 n) { return (size_t)256 * ((n + TILE - 1) / TILE ? (n + TILE - 1) / TILE : 1) + 1; }

// LSD radix sort of the low `bits` bits of 64-bit keys, 8 bits per pass, stable.
// On return *keys points at the sorted data and *alt at the other buffer.
// hist: radix_hist_elems(n) words; scratch: scan_scratch_elems(radix_hist_elems(n)) words.
int radix_sort_u64(u64** keys, u64** alt, u64 n, u32 bits, u32* hist, u32* scratch, hipStream_t s) {
  if (n == 0) return G10_OK;
  const u32 nb = (u32)((n + TILE - 1) / TILE);
  for (u32 shift = 0; shift < bits; shift += 8) {
    hipLaunchKernelGGL(k_radix_hist<u64>, dim3(nb), dim3(G10_BLOCK), 0, s, *keys, n, shift, hist, nb);
    G10_TRY(scan_excl_u32(hist, hist, (u64)256 * nb, scratch, s));
    hipLaunchKernelGGL((k_radix_scatter<u64, false>), dim3(nb), dim3(G10_BLOCK), 0, s, *keys, *alt, (const u32*)nullptr, (u32*)nullptr, n,
                       shift, hist, nb);
    u64* t = *keys; *keys = *alt; *alt = t;
  }
  G10_HIP(hipGetLastError());
  return G10_OK;
}

// The same with a 32-bit value carried along with every key; *vals / *valt swap like the keys.
// iota: the values are the positions 0..n-1 (the first pass makes them; *vals need not be filled).
int radix_sort_u64_pairs(u64** keys, u64** alt, u32** vals, u32** valt, u64 n, u32 bits, u32* hist, u32* scratch,
                         hipStream_t s, bool iota) {
  if (n == 0) return G10_OK;
  const u32 nb = (u32)((n + TILE - 1) / TILE);
  for (u32 shift = 0; shift < bits; shift += 8) {
    hipLaunchKernelGGL(k_radix_hist<u64>, dim3(nb), dim3(G10_BLOCK), 0, s, *keys, n, shift, hist, nb);
    G10_TRY(scan_excl_u32(hist, hist, (u64)256 * nb, scratch, s));
    hipLaunchKernelGGL((k_radix_scatter<u64, true>), dim3(nb), dim3(G10_BLOCK), 0, s, *keys, *alt,
                       iota && shift == 0 ? (const u32*)nullptr : (const u32*)*vals, *valt, n, shift, hist, nb);
    u64* t = *keys; *keys = *alt; *alt = t;
    u32* v = *vals; *vals = *valt; *valt = v;
  }
  G10_HIP(hipGetLastError());
  return G10_OK;
}

// 32-bit keys with a 32-bit value each (the score order of the planner's candidates).
int radix_sort_u32_pairs(u32** keys, u32** alt, u32** vals, u32** valt, u64 n, u32 bits, u32* hist, u32* scratch,
                         hipStream_t s, bool iota) {
  if (n == 0) return G10_OK;
  const u32 nb = (u32)((n + TILE - 1) / TILE);
  for (u32 shift = 0; shift < bits; shift += 8) {
    hipLaunchKernelGGL(k_radix_hist<u32>, dim3(nb), dim3(G10_BLOCK), 0, s, (const u32*)*keys, n, shift, hist, nb);
    G10_TRY(scan_excl_u32(hist, hist, (u64)256 * nb, scratch, s));
    hipLaunchKernelGGL((k_radix_scatter<u32, true>), dim3(nb), dim3(G10_BLOCK), 0, s, (const u32*)*keys, *alt,
                       iota && shift == 0 ? (const u32*)nullptr : (const u32*)*vals, *valt, n, shift, hist, nb);
    u32* t = *keys; *keys = *alt; *alt = t;
    u32* v = *vals; *vals = *valt; *valt = v;
  }
  G10_HIP(hipGetLastError());
  return G10_OK;
}

// `njobs` sorts of pairs in the same launches (jobs: device array; max_nb: the largest nb among them).  The
// sorted pairs of a job end in (keys, vals) after an even number of passes, in (alt, valt) after an odd one;
// iota: the values are the positions 0..n-1 (vals need not be filled).  Every job has n > 0.
u32 radix_blocks(u64 n) { return (u32)((n + TILE - 1) / TILE); }
int radix_sort_u32_pairs_jobs(const SortJob* jobs, u32 njobs, u32 max_nb, u32 bits, bool iota, hipStream_t s) {
  if (njobs == 0 || max_nb == 0) return G10_OK;
  u32 flip = 0;
  for (u32 shift = 0; shift < bits; shift += 8, flip ^= 1u) {
    hipLaunchKernelGGL(k_radix_hist_jobs, dim3(max_nb, njobs), dim3(G10_BLOCK), 0, s, jobs, shift, flip);
    hipLaunchKernelGGL(k_radix_scan_jobs, dim3(1, njobs), dim3(1024), 0, s, jobs);
    hipLaunchKernelGGL(k_radix_scatter_jobs, dim3(max_nb, njobs), dim3(G10_BLOCK), 0, s, jobs, shift, flip, iota && shift == 0 ? 1u : 0u);
  }
  G10_HIP(hipGetLastError());
  return G10_OK;
}

// Durations given for one plan instead of the analysed trace's: own copy, the same checks as
// the analysis makes, slot start times.  `stats_dev` is 128 bytes of device memory, `check` 128
// bytes of host memory that slot_times_end reads once the stream has been synchronised.
static_assert(sizeof(VitStats) <= 128, "the callers keep 128 bytes for the checks");
int slot_times_begin(const u64* src, u32 K, u64* dur, u64* start, u64* scratch64, void* stats_dev, void* check,
                     hipStream_t s) {
  VitStats* st = (VitStats*)stats_dev;
  G10_HIP(hipMemsetAsync(st, 0, sizeof(VitStats), s));
  G10_HIP(hipMemcpyAsync(dur, src, (u64)K * 8, hipMemcpyDeviceToDevice, s));
  hipLaunchKernelGGL(k_check_dur, dim3(grid_for(K)), dim3(G10_BLOCK), 0, s, (const u64*)dur, K, st);
  G10_HIP(hipGetLastError());
  G10_HIP(hipMemcpyAsync(check, st, sizeof(VitStats), hipMemcpyDeviceToHost, s));
  return scan_excl_u64(dur, start, K, scratch64, s);
}

int slot_times_end(const void* check, u64* T_out) {
  VitStats hs;
  memcpy(&hs, check, sizeof hs);
  if (hs.zero_dur) return G10_EINVAL;
  const unsigned __int128 T = ((unsigned __int128)hs.dur_hi << 32) + hs.dur_lo;
  if (T >> 62) return G10_EOVERFLOW;
  *T_out = (u64)T;
  return G10_OK;
}

// Device memory an analysis of K kernels, N tensors and P pairs takes: the temporaries of the call,
// and what outlives it (`planning`: with own copies of the trace's arrays and the periods in the
// order of their start, which only planning needs).
static size_t vit_tmp_bytes(u32 K, u32 N, u64 P) {
  const u64 ss_kn = scan_scratch_elems(K > N ? K : N), rh = radix_hist_elems(P), ss_p = scan_scratch_elems(rh > P ? rh : P);
  return Pool::need(1, sizeof(VitStats)) + Pool::need(ss_kn, 8) + 2 * Pool::need(P, 8) + 2 * Pool::need(P + 1, 4) +
         Pool::need(rh, 4) + Pool::need(ss_p, 4);
}
static size_t vit_keep_bytes(u32 K, u32 N, u64 P, bool planning) {
  // (the arrays per period are sized for P entries: there are fewer periods than uses, fewer uses than pairs)
  size_t b = Pool::need((u64)K + 1, 8) + Pool::need(P, 8) + Pool::need(P, 4) + Pool::need((u64)N + 1, 8) + 3 * Pool::need(P, 4) +
             Pool::need((u64)K + 2, 8);
  if (planning) b += Pool::need(K, 8) + Pool::need(N, 8) + Pool::need(N, 1) + Pool::need(P, 16) + Pool::need(P, 8);
  return b;
}

// The analysis proper, in memory the caller of this function provides (two pools of at least
// vit_tmp_bytes / vit_keep_bytes).
static int vitality_core(g10_plan_s* h, const g10_trace* tr, Pool& tmp, Pool& keep, const bool planning) {
  hipStream_t s = h->stream;
  const u32 K = h->K, N = h->N;
  const u64 P = h->P;

  VitStats* st = nullptr;
  G10_TRY(tmp.take(&st, 1));
  static_assert(sizeof(VitStats) % 8 == 0, "cleared as 64-bit words");
  hipLaunchKernelGGL(k_fill_u64, dim3(1), dim3(G10_BLOCK), 0, s, (u64*)st, (u64)(sizeof(VitStats) / 8), 0ull);
  G10_HIP(hipGetLastError());

  if (planning) {                                 // own copies of what planning needs later
    G10_TRY(keep.take(&h->dur, K));
    G10_TRY(keep.take(&h->size, N));
    G10_TRY(keep.take(&h->glob, N));
    G10_HIP(hipMemcpyAsync(h->dur, tr->dur_ns, (u64)K * 8, hipMemcpyDeviceToDevice, s));
    G10_HIP(hipMemcpyAsync(h->size, tr->size_bytes, (u64)N * 8, hipMemcpyDeviceToDevice, s));
    G10_HIP(hipMemcpyAsync(h->glob, tr->is_global, (u64)N, hipMemcpyDeviceToDevice, s));
  } else {                                        // the caller's arrays are read in place, during the call only
    h->dur = const_cast<u64*>(tr->dur_ns);
    h->size = const_cast<u64*>(tr->size_bytes);
    h->glob = const_cast<uint8_t*>(tr->is_global);
  }

  // ---- validation (read by the host with the counts, at the one synchronisation below: nothing
  // a kernel does with a zero duration, a zero or huge size or a wrapped sum leaves its arrays) ---
  hipLaunchKernelGGL(k_check_dur, dim3(grid_for(K)), dim3(G10_BLOCK), 0, s, h->dur, K, st);
  hipLaunchKernelGGL(k_check_size, dim3(grid_for(N, 512)), dim3(G10_BLOCK), 0, s, h->size, N, st);
  G10_HIP(hipGetLastError());

  // ---- slot start times ----------------------------------------------------
  u64* scratch64 = nullptr;
  G10_TRY(tmp.take(&scratch64, scan_scratch_elems(K > N ? K : N)));
  G10_TRY(keep.take(&h->start, (u64)K + 1));
  G10_TRY(scan_excl_u64(h->dur, h->start, K, scratch64, s));

  // ---- use lists -------------------------------------------------------------
  h->kbits = bits_for(K - 1);
  const u32 tbits = bits_for(N - 1);
  u64 *keys = nullptr, *alt = nullptr;
  u32 *flag = nullptr, *scratch32 = nullptr, *hist = nullptr;
  G10_TRY(tmp.take(&keys, P));
  G10_TRY(tmp.take(&alt, P));
  G10_TRY(tmp.take(&flag, P + 1));
  G10_TRY(tmp.take(&hist, radix_hist_elems(P)));
  G10_TRY(tmp.take(&scratch32, scan_scratch_elems(radix_hist_elems(P) > P ? radix_hist_elems(P) : P)));
  if (P) {
    hipLaunchKernelGGL(k_pack, dim3(grid_for(P)), dim3(G10_BLOCK), 0, s, tr->use_kernel, tr->use_tensor, P, K, N, h->kbits, keys, st);
    G10_TRY(radix_sort_u64(&keys, &alt, P, h->kbits + tbits, hist, scratch32, s));
    hipLaunchKernelGGL(k_flag_distinct, dim3(grid_for(P)), dim3(G10_BLOCK), 0, s, keys, P, flag);
    G10_HIP(hipGetLastError());
  }
  G10_TRY(scan_excl_u32(flag, flag, P, scratch32, s));           // flag[i] = position, flag[P] = n_uses
  const u32* n_uses_p = flag + P;
  G10_TRY(keep.take(&h->ukeys, P));                               // upper bounds: no host round trip here
  G10_TRY(keep.take(&h->use_k, P));
  G10_TRY(keep.take(&h->use_off, (u64)N + 1));
  if (P) hipLaunchKernelGGL(k_compact_distinct, dim3(grid_for(P)), dim3(G10_BLOCK), 0, s, keys, P, flag, h->ukeys, h->use_k, h->kbits);
  hipLaunchKernelGGL(k_use_off, dim3(grid_for((u64)N + 1)), dim3(G10_BLOCK), 0, s, h->ukeys, n_uses_p, N, h->kbits, h->use_off);
  G10_HIP(hipGetLastError());

  // ---- inactive periods --------------------------------------------------------
  u32* pcnt = nullptr;
  G10_TRY(tmp.take(&pcnt, P + 1));
  const u32 no_wrap = (h->flags & G10_NO_WRAP) ? 1u : 0u;
  hipLaunchKernelGGL(k_fill_u32, dim3(grid_for(P + 1)), dim3(G10_BLOCK), 0, s, pcnt, P + 1, 0u);
  if (P) hipLaunchKernelGGL(k_period_count, dim3(grid_for(P)), dim3(G10_BLOCK), 0, s, h->ukeys, h->use_off, h->glob, n_uses_p, K, h->kbits, no_wrap, pcnt);
  G10_TRY(scan_excl_u32(pcnt, pcnt, P, scratch32, s));           // pcnt[P] = n_periods (entries past n_uses are 0)
  G10_TRY(keep.take(&h->per_t, P));
  G10_TRY(keep.take(&h->per_L, P));
  G10_TRY(keep.take(&h->per_R, P));
  if (P) hipLaunchKernelGGL(k_period_write, dim3(grid_for(P)), dim3(G10_BLOCK), 0, s, h->ukeys, h->use_off, h->glob, n_uses_p, K, h->kbits, no_wrap, pcnt, h->per_t, h->per_L, h->per_R);
  G10_HIP(hipGetLastError());

  // ---- memory pressure -----------------------------------------------------------
  G10_TRY(keep.take(&h->pressure_buf, (u64)K + 2));
  hipLaunchKernelGGL(k_fill_u64, dim3(grid_for((u64)K + 2)), dim3(G10_BLOCK), 0, s, h->pressure_buf, (u64)K + 2, 0ull);
  hipLaunchKernelGGL(k_lifetime_adds, dim3(grid_for(N)), dim3(G10_BLOCK), 0, s, h->ukeys, h->use_off, h->size, h->glob, N, K, h->kbits, h->pressure_buf, st);
  G10_HIP(hipGetLastError());
  // exclusive scan of diff[0..K] in place: buf[k + 1] = sum diff[0..k] = pressure[k]
  G10_TRY(scan_excl_u64(h->pressure_buf, h->pressure_buf, (u64)K, scratch64, s));
  hipLaunchKernelGGL(k_max_u64, dim3(grid_for(K, 1024)), dim3(G10_BLOCK), 0, s, h->pressure_buf + 1, (u64)K, &st->peak);
  hipLaunchKernelGGL(k_store_counts, dim3(1), dim3(1), 0, s, n_uses_p, pcnt + P, st);
  G10_HIP(hipGetLastError());
  VitStats hs;
  G10_HIP(hipMemcpyAsync(&hs, st, sizeof hs, hipMemcpyDeviceToHost, s));
  G10_HIP(hipStreamSynchronize(s));
  if (hs.bad_index || hs.zero_dur || hs.zero_size) return G10_EINVAL;
  if (hs.size_overflow) return G10_EOVERFLOW;
  {
    unsigned __int128 T = ((unsigned __int128)hs.dur_hi << 32) + hs.dur_lo;
    if (T >> 62) return G10_EOVERFLOW;
    h->T = (u64)T;
    unsigned __int128 used = ((unsigned __int128)hs.used_hi << 32) + hs.used_lo;
    if (used >> 64) return G10_EOVERFLOW;
  }
  h->big_size = hs.big_size != 0;
  h->max_size = hs.max_size;
  h->n_uses = hs.n_uses;
  h->n_periods = hs.n_periods;
  h->peak = hs.peak;

  if (!planning) return G10_OK;

  // ---- the periods once more, ordered by their start --------------------------------------
  // Planning walks the periods with one thread each and looks up the timeline around their
  // start and end; in this order neighbouring threads look at neighbouring slots.
  const u64 C = h->n_periods;
  G10_TRY(keep.take(&h->per_by_start, C));      // (C <= P)
  G10_TRY(keep.take(&h->per_size, C));
  if (C) {
    // (a stable sort of the starts alone, the position carried along: equal starts keep the order of the periods)
    u32 *k32 = (u32*)keys, *k32_alt = k32 + C, *ord = (u32*)alt, *ord_alt = ord + C;      // (C <= P: two arrays of C words in one of P keys)
    G10_HIP(hipMemcpyAsync(k32, h->per_L, C * 4, hipMemcpyDeviceToDevice, s));
    G10_TRY(radix_sort_u32_pairs(&k32, &k32_alt, &ord, &ord_alt, C, h->kbits, hist, scratch32, s, true));
    hipLaunchKernelGGL(k_gather_periods, dim3(grid_for(C)), dim3(G10_BLOCK), 0, s, (const u32*)ord, C, h->per_t, h->per_L, h->per_R,
                       h->size, h->per_by_start, h->per_size);
    G10_HIP(hipGetLastError());                     // (still running when this function returns: see vitality_run)
  }
  return G10_OK;
}

int vitality_run(g10_plan_s* h, const g10_trace* tr) {
  if (h->P >= (1ull << 32)) return G10_EINVAL;    // positions and counts are 32-bit on the device
  // The temporaries of the call and what the handle keeps.  The last kernels of the analysis
  // still read the temporaries when the call returns (planning follows on the same stream and
  // need not wait for them): they are released at the next point where the stream has been
  // waited for, at the latest with the handle.
  Pool tmp, keep;
  G10_TRY(tmp.reserve(vit_tmp_bytes(h->K, h->N, h->P)));
  h->tmp_arena = tmp.base;
  G10_TRY(keep.reserve(vit_keep_bytes(h->K, h->N, h->P, true)));
  h->arena = keep.base;
  return vitality_core(h, tr, tmp, keep, true);
}

// ===========================================================================
// The analysis for callers that cannot allocate: all device memory beyond the caller's inputs
// and outputs is this array, one copy per GPU, held until the process ends.  Its address on the
// current device is asked for once per device (the array's name itself is only a host-side
// stand-in and is never passed to a kernel or a copy).
// ===========================================================================
static __device__ __align__(256) unsigned char scratch[G10_STATIC_SCRATCH_BYTES];

enum { G10_MAX_DEVICES = 64 };
static unsigned char* scratch_on_device[G10_MAX_DEVICES] = {};

extern "C" int g10_vitality_static(const g10_trace* tr, void* hip_stream, const g10_vitality_buffers* out,
                                   g10_vitality_stats* stats) {
  if (stats) memset(stats, 0, sizeof *stats);
  if (!tr || !out || !stats) return G10_EINVAL;
  if (!tr->K || !tr->N) return G10_EINVAL;
  if (!tr->dur_ns || !tr->size_bytes || !tr->is_global) return G10_EINVAL;
  if (tr->P && (!tr->use_kernel || !tr->use_tensor)) return G10_EINVAL;
  if (!out->use_off || !out->start || !out->pressure) return G10_EINVAL;
  if (tr->P && (!out->use_k || !out->per_tensor || !out->per_L || !out->per_R)) return G10_EINVAL;
  if (tr->K > G10_STATIC_MAX_K || tr->N > G10_STATIC_MAX_N || tr->P > G10_STATIC_MAX_P) return G10_ELIMIT;
  const size_t need_tmp = vit_tmp_bytes(tr->K, tr->N, tr->P), need_keep = vit_keep_bytes(tr->K, tr->N, tr->P, false);
  if (need_tmp + need_keep > (size_t)G10_STATIC_SCRATCH_BYTES) return G10_ELIMIT;
  int dev = 0;
  G10_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= G10_MAX_DEVICES) return G10_EDEVICE;
  if (!scratch_on_device[dev]) {
    void* q = nullptr;
    G10_HIP(hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)));
    if (!q) return G10_EDEVICE;
    scratch_on_device[dev] = (unsigned char*)q;
  }
  unsigned char* const mem = scratch_on_device[dev];

  g10_plan_s h;                                   // (lives on the stack for the call; nothing of it is handed out)
  h.device = dev;
  h.stream = (hipStream_t)hip_stream;
  h.K = tr->K; h.N = tr->N; h.P = tr->P; h.flags = tr->flags;
  Pool tmp, keep;                                 // both inside the array
  tmp.base = (char*)mem; tmp.cap = need_tmp;
  keep.base = (char*)mem + need_tmp; keep.cap = need_keep;
  hipStream_t s = h.stream;
  int rc = vitality_core(&h, tr, tmp, keep, false);
  if (rc) { (void)hipStreamSynchronize(s); return rc; }
  // the results go into the caller's buffers
  G10_HIP(hipMemcpyAsync(out->use_off, h.use_off, ((u64)h.N + 1) * 8, hipMemcpyDeviceToDevice, s));
  G10_HIP(hipMemcpyAsync(out->start, h.start, ((u64)h.K + 1) * 8, hipMemcpyDeviceToDevice, s));
  G10_HIP(hipMemcpyAsync(out->pressure, h.pressure_buf + 1, (u64)h.K * 8, hipMemcpyDeviceToDevice, s));
  if (h.n_uses) G10_HIP(hipMemcpyAsync(out->use_k, h.use_k, h.n_uses * 4, hipMemcpyDeviceToDevice, s));
  if (h.n_periods) {
    G10_HIP(hipMemcpyAsync(out->per_tensor, h.per_t, h.n_periods * 4, hipMemcpyDeviceToDevice, s));
    G10_HIP(hipMemcpyAsync(out->per_L, h.per_L, h.n_periods * 4, hipMemcpyDeviceToDevice, s));
    G10_HIP(hipMemcpyAsync(out->per_R, h.per_R, h.n_periods * 4, hipMemcpyDeviceToDevice, s));
  }
  G10_HIP(hipStreamSynchronize(s));
  stats->n_uses = h.n_uses; stats->n_periods = h.n_periods; stats->peak_bytes = h.peak; stats->iter_ns = h.T;
  return G10_OK;
}
