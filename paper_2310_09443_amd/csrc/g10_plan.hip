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
// runs in ONE persistent workgroup of 512 threads per plan (k_loop, in
// g10_loop.hip): no grid barrier and no kernel boundary per pass, the level-1
// state in LDS, the slot arrays in L2.  Range updates over a period are chunked: whole chunks take a lazy
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
//
// This file: the host side of a planning call (workspaces, launches, re-tiling
// between launches of the loop, batches of plans) and the streaming kernels
// (candidate preparation, timelines, the full scoring pass, re-scoring, tile
// gather).  The two alternative readings of Section 4.3 (rank by benefit /
// cost; benefit as the area removed above the capacity line) instantiate the
// same kernels; what they change is stated in g10_plan_defs.h and g10_loop.hip.

#include "g10_plan_defs.h"

#include <hip/hip_ext.h>
#include <chrono>
#include <new>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

using namespace g10;

namespace {

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

// The copy of a candidate for the first scoring pass in 16 bytes instead of 24, where the trace allows it:
// four window ends of 21 bits (2 K <= 2^21) and a size of 43 bits (no tensor of 8 TiB or more).
constexpr u32 PACK_END_BITS = 21, PACK_SIZE_BITS = 43;
static_assert(3 * PACK_END_BITS <= 64 && PACK_END_BITS + PACK_SIZE_BITS == 64, "three ends in one word, the fourth and the size in the other");
__device__ __forceinline__ uint4 pack_windows(const uint4 w, const u64 s) {
  const u64 lo = (u64)w.x | ((u64)w.y << PACK_END_BITS) | ((u64)w.z << (2 * PACK_END_BITS));
  const u64 hi = (u64)w.w | (s << PACK_END_BITS);
  return make_uint4((u32)lo, (u32)(lo >> 32), (u32)hi, (u32)(hi >> 32));
}
__device__ __forceinline__ void unpack_windows(const uint4 q, uint4& w, u64& s) {
  const u64 lo = ((u64)q.y << 32) | q.x, hi = ((u64)q.w << 32) | q.z;
  const u32 m = (1u << PACK_END_BITS) - 1u;
  w = make_uint4((u32)lo & m, (u32)(lo >> PACK_END_BITS) & m, (u32)(lo >> (2 * PACK_END_BITS)) & m, (u32)hi & m);
  s = hi >> PACK_END_BITS;
}

// candidates with at least one valid window, packed in the order of their start
__global__ __launch_bounds__(G10_BLOCK) void k_pack(const uint4* __restrict__ per, const u64* __restrict__ size,
                                                   const uint4* __restrict__ win, const u32* __restrict__ pos, u32 C,
                                                   Cands out, uint4* __restrict__ fw, u64* __restrict__ fs, u32 packed) {
  const u32 c = blockIdx.x * G10_BLOCK + threadIdx.x;
  if (c >= C || pos[c + 1] == pos[c]) return;
  const uint4 pd = per[c];                  // {L, R, tensor, period index}
  const u32 o = pos[c];
  const uint4 w = win[c];
  const u64 s = size[c];                    // sizes in the same order
  out.A[o] = make_uint4(pd.x + 1, pd.y, w.x, w.y);
  out.B[o] = make_uint4(w.z, w.w, (u32)s, (u32)(s >> 32));
  out.id[o] = make_uint2(pd.w, pd.z);
  if (fw) {                                 // what the first scoring pass needs, on its own: the two windows and the size
    if (packed) fw[o] = pack_windows(w, s);
    else {
      fw[o] = w;
      fs[o] = s;
    }
  }
  if (out.ce) out.ce[o] = make_uint2(0u, 0u);        // no value of the clipped area yet
}

// ---------------------------------------------------------------------------
// timelines before any eviction: slot arrays, chunk-local prefixes, chunk totals
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(G10_BLOCK) void k_init_timelines(Timelines tl, const u64* __restrict__ pressure0, const Ctl* ctl,
                                                             u64* __restrict__ g_tot, u64* __restrict__ g_lazyP,
                                                             u64* __restrict__ g_minOver, u64* __restrict__ g_lazyH,
                                                             u64* __restrict__ g_hmax, u32* __restrict__ g_hmat,
                                                             u32* __restrict__ g_hpend) {
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
    g_lazyP[chunk] = 0; g_minOver[chunk] = m; g_lazyH[chunk] = 0; g_hmax[chunk] = 0; g_hmat[chunk] = 0; g_hpend[chunk] = 0;
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
// U = size * (largest over-capacity time of the valid windows).  The period's
// ends are not needed for that, so the pass reads a copy of the candidates
// made for it - the two windows and the size, 24 bytes - gathers two words per
// window of a prefix table that fits L2 (8 bytes per slot; a window inside the
// other one is skipped), and writes the 8-byte sort key: the 31-bit score key
// rounded up to its top 23 bits (descending), then the position.
// ---------------------------------------------------------------------------
// (ascending sort = descending score; the sort is stable, so equal keys stay in the order of their positions)
__device__ __forceinline__ u32 sort_key(u32 key31) { return 0x7fffffu - ((key31 + 255u) >> 8); }
// the bound a sort key stands for: at least the score key it was made from, 0 only for 0
__device__ __forceinline__ u32 bound_of_sort_key(u32 sk) { return (0x7fffffu - sk) << 8; }

// RATIO: ranking by benefit / cost; a window inside the other may then still have the larger
// key (its transfers can be the shorter ones), so both are looked up.
// PACKED: the copy is the 16-byte form (fs is not read).
template <bool RATIO, bool PACKED>
__global__ __launch_bounds__(G10_BLOCK) void k_score_full(const uint4* __restrict__ fw, const u64* __restrict__ fs, u32 n,
                                                         const u64* __restrict__ ot, u32 K,
                                                         u32* __restrict__ sortkeys, const Ctl* __restrict__ ctl) {
  const u32 p = blockIdx.x * G10_BLOCK + threadIdx.x;
  if (p >= n) return;
  uint4 W = fw[p];                            // {a0, b0, a1, b1}
  u64 s;
  if (PACKED) unpack_windows(W, W, s);
  else s = fs[p];
  const u64 total = ot[K];
  bool v0 = W.x <= W.y, v1 = W.z <= W.w;
  // the prefix is monotone: a window inside the other one cannot hold more over-capacity time
  if (!RATIO && v0 && v1) {
    if (W.z <= W.x && W.w >= W.y) v0 = false;
    else if (W.x <= W.z && W.y >= W.w) v1 = false;
  }
  u64 t0 = 0, t1 = 0;
  if (v0) {
    const u32 a = W.x, b = W.y + 1;
    const u64 oa = ot[a >= K ? a - K : a], ob = ot[b >= K ? b - K : b];
    t0 = (ob + (b >= K ? total : 0ull)) - (oa + (a >= K ? total : 0ull));
  }
  if (v1) {
    const u32 a = W.z, b = W.w + 1;
    const u64 oa = ot[a >= K ? a - K : a], ob = ot[b >= K ? b - K : b];
    t1 = (ob + (b >= K ? total : 0ull)) - (oa + (a >= K ? total : 0ull));
  }
  if (RATIO) {
    Machine mc;
    mc.bwo0 = ctl->bw_out[0]; mc.bwo1 = ctl->bw_out[1]; mc.bwi0 = ctl->bw_in[0]; mc.bwi1 = ctl->bw_in[1];
    mc.ivo0 = ctl->inv_out[0]; mc.ivo1 = ctl->inv_out[1]; mc.ivi0 = ctl->inv_in[0]; mc.ivi1 = ctl->inv_in[1];
    u64 c0, c1;
    costs_of(mc, s, c0, c1);
    const u32 k0 = key_up_of<true>(__umul64hi(s, t0), s * t0, c0), k1 = key_up_of<true>(__umul64hi(s, t1), s * t1, c1);
    sortkeys[p] = sort_key(k0 > k1 ? k0 : k1);
    return;
  }
  const u64 t = t1 > t0 ? t1 : t0;
  sortkeys[p] = sort_key(upkey(__umul64hi(s, t), s * t));
}

// candidates into score order; the tile bound is the largest bound of its members
__device__ __forceinline__ void tile_gather_at(const u32 r, const u32* __restrict__ sorted, const u32* __restrict__ from, u32 n, u32 n_pad,
                                               const Cands& src, const Cands& dst, u32 tile_shift, u32* __restrict__ tkeys) {
  if (r >= n_pad) return;
  u32 k = 0;
  if (r < n) {
    const u32 sk = sorted[r];
    const u32 p = from[r];
    dst.A[r] = src.A[p];
    dst.B[r] = src.B[p];
    dst.id[r] = src.id[p];
    if (src.ce) {
      const uint2 e = src.ce[p];
      dst.ce[r] = e;
      if (e.y & 1u) dst.cv[r] = src.cv[p];
    } else if (dst.ce) dst.ce[r] = make_uint2(0u, 0u);     // (gathered from another plan's fresh list: no value yet)
    k = bound_of_sort_key(sk);
  } else {                                       // padding of the last tile: no valid window
    dst.A[r] = make_uint4(0u, 0u, 1u, 0u);
    dst.B[r] = make_uint4(1u, 0u, 0u, 0u);
    dst.id[r] = make_uint2(NONE32, 0u);
    if (dst.ce) dst.ce[r] = make_uint2(0u, 0u);
  }
  k = wave_max(k);
  if (lane_id() == 0 && k) atomicMax(&tkeys[r >> tile_shift], k);
}
__global__ __launch_bounds__(G10_BLOCK) void k_tile_gather(const u32* __restrict__ sorted, const u32* __restrict__ from, u32 n, u32 n_pad,
                                                          Cands src, Cands dst, u32 tile_shift, u32* __restrict__ tkeys) {
  tile_gather_at(blockIdx.x * G10_BLOCK + threadIdx.x, sorted, from, n, n_pad, src, dst, tile_shift, tkeys);
}

// Re-scores every candidate of the list against the current timelines (all
// workgroups of the chip; used between launches of the loop kernel to put the
// candidates back into score order).  Writes the sort key;
// strikes dead destinations; counts the candidates that can still score.
template <bool RATIO>
__device__ __forceinline__ void rescore_block(const Cands& cd, u32 n, const u64* __restrict__ px, const u64* __restrict__ g_base,
                                              u32 K, u32 nch, u32 shift_ch, const Ctl* ctl,
                                              u32* __restrict__ sortkeys, u32* __restrict__ n_live, u64* lb, u32* tmp) {
  for (u32 i = threadIdx.x; i < N_ARR * (nch + 1); i += G10_BLOCK) lb[i] = g_base[i];
  __syncthreads();
  PrefixView pv; pv.px = px; pv.base = lb; pv.K = K; pv.nch = nch; pv.shift_ch = shift_ch;
  Machine mc; mc.bwo0 = ctl->bw_out[0]; mc.bwo1 = ctl->bw_out[1]; mc.bwi0 = ctl->bw_in[0]; mc.bwi1 = ctl->bw_in[1];
  mc.ivo0 = ctl->inv_out[0]; mc.ivo1 = ctl->inv_out[1]; mc.ivi0 = ctl->inv_in[0]; mc.ivi1 = ctl->inv_in[1];
  u32 live = 0;
  for (u32 p = blockIdx.x * G10_BLOCK + threadIdx.x; p < n; p += gridDim.x * G10_BLOCK) {
    const uint4 A = cd.A[p], B = cd.B[p];
    const Score r = score_candidate(pv, mc, A, B);
    if (r.strike0) cd.A[p] = make_uint4(A.x, A.y, 1u, 0u);
    if (r.strike1) cd.B[p] = make_uint4(1u, 0u, B.z, B.w);
    u32 k;
    if (RATIO) {
      u64 c0 = 1, c1 = 1;
      if (r.ok0 || r.ok1) costs_of(mc, ((u64)B.w << 32) | B.z, c0, c1);
      const u32 k0 = key_up_of<true>(r.h0, r.l0, c0), k1 = key_up_of<true>(r.h1, r.l1, c1);
      k = k0 > k1 ? k0 : k1;
    } else {
      const bool one = gt128(r.h1, r.l1, r.h0, r.l0);
      k = upkey(one ? r.h1 : r.h0, one ? r.l1 : r.l0);
    }
    sortkeys[p] = sort_key(k);
    live += k != 0;
  }
  live = block_sum(live, tmp);
  if (threadIdx.x == 0 && live) atomicAdd(n_live, live);
}
template <bool RATIO>
__global__ __launch_bounds__(G10_BLOCK) void k_rescore(Cands cd, u32 n, const u64* __restrict__ px, const u64* __restrict__ g_base,
                                                      u32 K, u32 nch, u32 shift_ch, const Ctl* ctl,
                                                      u32* __restrict__ sortkeys, u32* __restrict__ n_live) {
  extern __shared__ u64 lb[];                  // [5][nch + 1]
  __shared__ u32 tmp[G10_WAVES + 1];
  rescore_block<RATIO>(cd, n, px, g_base, K, nch, shift_ch, ctl, sortkeys, n_live, lb, tmp);
}

// ---- the re-tilings of a round of a batch, all plans in the same launches: job = blockIdx.y ----
struct TileJob {
  Cands src, dst;              // the list as the loop left it; the buffer that takes the new order
  u32 n, n_pad, tile_shift, rank;
  u32 *sortkeys, *sorted, *from, *tkeys;     // keys out of the re-scoring; keys and old positions in the new order; tile bounds
  const u64 *px, *g_base;
  Ctl* ctl;
  u32 K, nch, shift_ch, pad;
};

__global__ __launch_bounds__(G10_BLOCK) void k_retile_begin_jobs(const TileJob* __restrict__ jobs) {
  const TileJob& j = jobs[blockIdx.y];
  for (u32 i = threadIdx.x; i < NT_MAX; i += G10_BLOCK) j.tkeys[i] = 0u;
  if (threadIdx.x == 0) j.ctl->n_live = 0u;
}

__global__ __launch_bounds__(G10_BLOCK) void k_rescore_jobs(const TileJob* __restrict__ jobs) {
  extern __shared__ u64 lb[];                  // [5][nch + 1], the largest nch of the jobs
  __shared__ u32 tmp[G10_WAVES + 1];
  const TileJob j = jobs[blockIdx.y];
  if (blockIdx.x * G10_BLOCK >= j.n) return;
  if (j.rank == G10_RANK_RATIO) rescore_block<true>(j.src, j.n, j.px, j.g_base, j.K, j.nch, j.shift_ch, j.ctl, j.sortkeys, &j.ctl->n_live, lb, tmp);
  else rescore_block<false>(j.src, j.n, j.px, j.g_base, j.K, j.nch, j.shift_ch, j.ctl, j.sortkeys, &j.ctl->n_live, lb, tmp);
}

__global__ __launch_bounds__(G10_BLOCK) void k_tile_gather_jobs(const TileJob* __restrict__ jobs) {
  const TileJob j = jobs[blockIdx.y];
  tile_gather_at(blockIdx.x * G10_BLOCK + threadIdx.x, j.sorted, j.from, j.n, j.n_pad, j.src, j.dst, j.tile_shift, j.tkeys);
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

// The progress blocks of the plans of a launch, side by side, so that one copy brings them to the host.
__global__ __launch_bounds__(G10_WAVE) void k_ctl_collect(const LoopArgs* __restrict__ args, Ctl* __restrict__ out) {
  static_assert(sizeof(Ctl) % 8 == 0, "copied as 64-bit words");
  const u64* src = (const u64*)args[blockIdx.x].ctl;
  u64* dst = (u64*)(out + blockIdx.x);
  for (u32 i = threadIdx.x; i < sizeof(Ctl) / 8; i += G10_WAVE) dst[i] = src[i];
}

}  // namespace

void plan_work_free(PlanWork* w) {
  if (!w) return;
  mem_dev_free(w->arena);
  replay_free(w);
  mem_host_free(w->h_block);
  free(w->h_pf_order); free(w->h_pf_gained); free(w->h_pf_last); free(w->h_pf_pressure);
  for (hipEvent_t e : w->ev) mem_event_put(e, w->device);
  delete w;
}

static const u32 SCORE_SORT_BITS = 23;           // significant bits of a score sort key
static const u32 SCORE_SORT_PASSES = (SCORE_SORT_BITS + 7) / 8;
static const u32 PASS_BUDGET = 4096;             // ranking passes per launch of the loop kernel
static const u32 RETILE_PASSES = 128;   // ... between two re-tilings of a long candidate list
static const u32 RETILE_MIN_CANDS = 8192;        // shorter lists are never re-tiled
static const u64 BATCH_LAUNCH_TICKS = 250000;    // a launch of a batch ends after 2.5 ms (100 MHz clock)
// Ranking by benefit / cost on a long list (one plan, band reading): a scoring round of WIDE_MIN_UNITS
// x 256 candidates or more is left to a kernel on all compute units.  The loop kernel then ends in
// the middle of its pass and takes it up in its next launch, so such launches are queued in pairs,
// a round of them ahead of what the host knows.
static const u32 WIDE_MIN_UNITS = 32;
static const u64 WIDE_MIN_CANDS = 65536;

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
  ar.take(&w->sv, C); ar.take(&w->sv_alt, C);
  ar.take(&w->tkeys, (u64)NT_MAX);
  ar.take(&w->fw, C); ar.take(&w->fs, C);
  for (int i = 0; i < 2; ++i) {
    ar.take(&w->cd[i].A, w->cap_pad); ar.take(&w->cd[i].B, w->cap_pad); ar.take(&w->cd[i].id, w->cap_pad);
    if (w->has_cache) { ar.take(&w->cd[i].cv, w->cap_pad); ar.take(&w->cd[i].ce, w->cap_pad); }
  }
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
  ar.take(&w->rec_h, C);
  ar.take(&w->g_hmat, w->nch); ar.take(&w->g_hpend, w->nch);
  ar.take(&w->dropped, C);
  ar.take(&w->pf_keys, C); ar.take(&w->pf_keys_alt, C);
  ar.take(&w->pf_order, C); ar.take(&w->pf_order_alt, C);
  ar.take(&w->pf_gained, C); ar.take(&w->pf_last, C);
  ar.take(&w->pf_pressure, K);
  ar.take(&w->pf_stats, 4);
  ar.take(&w->dur_own, K); ar.take(&w->start_own, (u64)K + 1);
  ar.take(&w->times_scratch, scan_scratch_elems(K)); ar.take(&w->times_stats, 16);
  ar.take(&w->wide, loop_wide_bytes());
}

static int work_alloc(g10_plan_s* h, u32 max_chunks, bool cache, PlanWork** slot) {
  PlanWork* w = new (std::nothrow) PlanWork();
  if (!w) return G10_ENOMEM;
  *slot = w;
  const u32 K = h->K;
  const u64 C = h->n_periods;
  w->K = K; w->C = C;
  w->device = h->device;
  w->Kp = (K + 3u) & ~3u;
  w->spt = 1; w->shift_ch = 8;
  w->max_chunks = max_chunks;
  w->has_cache = cache;
  while ((u64)G10_BLOCK * w->spt * max_chunks < K) { w->spt *= 2; w->shift_ch += 1; }
  const u32 ch = G10_BLOCK * w->spt;
  w->nch = (K + ch - 1) / ch;
  // room for the padding of the last tile at any tile size: tiles hold at most max(256, C) candidates
  w->cap_pad = 2 * (C > UNIT ? C : UNIT) + UNIT;
  Arena measure;
  work_layout(w, measure);
  void* q = nullptr;
  G10_TRY(mem_dev_alloc(&q, measure.off + 256));
  w->arena = q;
  Arena carve;
  carve.base = (char*)q;
  work_layout(w, carve);
  for (hipEvent_t& e : w->ev) G10_TRY(mem_event_get(&e));
  return G10_OK;
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
  u64 retiles = 0, retile_cands = 0, launches = 0, max_launches = 0, overtime_before = 0;
  bool counted = false;        // hc.n_live holds a count of the current list
  bool timed_full = false;
  u64 times_check[16] = {};     // the checks of the plan's own durations come back here
  u64 seen_passes = 0;         // passes of the loop kernel done at the last re-tiling
  u64 seen_units = 0, seen_passes_w = 0;   // units scored and passes done when the last round of launches began
  bool wide = false;           // long scoring rounds are left to the scoring kernel in the current round of launches
  u32 loop_seq = 0;            // launches of the loop kernel queued so far (with a block for the scoring kernel)
  u32 lead = 0;                // the plan of the batch whose candidate windows this one reads (itself, or an
                               // earlier plan with the same bandwidths and durations: the windows depend on nothing else)
  bool fw_done = false;        // (of such a plan) the copy of the windows for the first scoring pass is written or on its way
  Cands pack_src = {};         // (of such a plan) the candidates in the order of their start, as the first plan of the group packed
                               // them: the other plans of the group gather their first order from there
  bool own_pack = true;        // this plan's first order is gathered from its own packed list
  bool results_sent = false;   // the plan is finished and its results are on their way to the host
};

static PlanWork** work_slot(g10_plan_s* h, u32 i) { return i == 0 ? &h->work : &h->more[i - 1]; }

// `count` plans on one analysed trace.  The streaming kernels of the plans run one after the
// other (each fills the chip); the greedy loops run side by side, one workgroup per plan, in
// one launch per round; between rounds the long candidate lists are put back into score order.
typedef void (*ScoreFullKernel)(const uint4*, const u64*, u32, const u64*, u32, u32*, const Ctl*);
static ScoreFullKernel score_full_kernel(u32 rank, bool packed) {
  if (packed) return rank == G10_RANK_RATIO ? k_score_full<true, true> : k_score_full<false, true>;
  return rank == G10_RANK_RATIO ? k_score_full<true, false> : k_score_full<false, false>;
}

int plan_batch_run(g10_plan_s* h, const g10_params* params, u32 count, g10_result* outs) {
  hipStream_t s = h->stream;
  const u32 K = h->K;
  const bool packed = !h->big_size && 2ull * K <= (1ull << PACK_END_BITS);   // the first scoring pass reads 16-byte copies
  const u32 C = (u32)h->n_periods;
  const u32 gC = (C + G10_BLOCK - 1) / G10_BLOCK;
  if (count > 1 + h->n_more) {                             // more workspace slots
    PlanWork** m = (PlanWork**)realloc(h->more, (size_t)(count - 1) * sizeof(PlanWork*));
    if (!m) return G10_ENOMEM;
    for (u32 i = h->n_more; i < count - 1; ++i) m[i] = nullptr;
    h->more = m; h->n_more = count - 1;
  }
  if (count > h->loop_args_cap) {
    if (h->loop_args) { G10_HIP(hipStreamSynchronize(s)); mem_dev_free(h->loop_args); h->loop_args = nullptr; h->loop_args_cap = 0; }
    void* q = nullptr;
    G10_TRY(mem_dev_alloc(&q, (size_t)count * (sizeof(LoopArgs) + sizeof(Ctl) + sizeof(SortJob) + sizeof(TileJob))));
    h->loop_args = q; h->loop_args_cap = count;
  }
  Ctl* const ctl_side = (Ctl*)((LoopArgs*)h->loop_args + h->loop_args_cap);    // the progress blocks of a launch, collected
  SortJob* const sort_jobs = (SortJob*)(ctl_side + h->loop_args_cap);          // the re-tilings of a round of a batch
  TileJob* const tile_jobs = (TileJob*)(sort_jobs + h->loop_args_cap);
  // host wall clock of the call's phases (a batch of several plans only: it costs a synchronisation per round)
  const bool clocked = count > 1;
  double phase_ms[4] = {0, 0, 0, 0};                     // preparation and first ordering; loops; re-tilings; results
  auto now_ms = [] { return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now().time_since_epoch()).count(); };
  double t_mark = now_ms();
  auto phase_end = [&](int k) { const double t = now_ms(); phase_ms[k] += t - t_mark; t_mark = t; };
  h->n_counters = 0;
  {
    g10_counters* q = (g10_counters*)realloc(h->counters, (size_t)count * sizeof(g10_counters));
    if (!q) return G10_ENOMEM;
    h->counters = q;
    memset(q, 0, (size_t)count * sizeof(g10_counters));
  }
  Inst* I = new (std::nothrow) Inst[count];
  LoopArgs* hargs = (LoopArgs*)malloc((size_t)count * sizeof(LoopArgs));
  Ctl* hctl = (Ctl*)malloc((size_t)count * sizeof(Ctl));
  u32* who = (u32*)malloc((size_t)count * sizeof(u32));                       // the plan of every entry of a launch
  u64* peaks = (u64*)malloc((size_t)count * sizeof(u64));                     // the plans' final peaks come back here
  SortJob* hsj = (SortJob*)malloc((size_t)count * sizeof(SortJob));
  TileJob* htj = (TileJob*)malloc((size_t)count * sizeof(TileJob));
  // whatever way this function is left, nothing is in flight that reads or writes these host arrays
  struct Guard {
    g10_plan_s* h; Inst* i; LoopArgs* a; Ctl* c; u32* w; SortJob* sj; TileJob* tj; u64* pk;
    ~Guard() {
      for (u32 k = 0; k < h->n_aux; ++k) (void)hipStreamSynchronize(h->aux[k]);
      (void)hipStreamSynchronize(h->stream);
      delete[] i; free(a); free(c); free(w); free(sj); free(tj); free(pk);
    }
  } guard{h, I, hargs, hctl, who, hsj, htj, peaks};
  if (!I || !hargs || !hctl || !who || !hsj || !htj || !peaks) return G10_ENOMEM;

  for (u32 i = 0; i < count; ++i) {
    const g10_params* p = params + i;
    const u32 max_chunks = clamp_limit(h->max_chunks, NCH_MAX);
    PlanWork** slot = work_slot(h, i);
    bool cache = p->area == G10_AREA_CLIPPED;
    if (*slot && ((*slot)->max_chunks != max_chunks || (cache && !(*slot)->has_cache))) {
      // another chunk size, or the first plan with clipped areas: lay the workspaces out again
      cache = cache || (*slot)->has_cache;
      G10_HIP(hipStreamSynchronize(s));
      plan_work_free(*slot);
      *slot = nullptr;
    }
    if (!*slot) {
      int rc = work_alloc(h, max_chunks, cache, slot);
      if (rc) {
        // (out of memory, most likely: the workspaces of the other plans of the batch go too, so that a failed
        // call does not keep the device full; the first plan's stay)
        plan_work_free(*slot); *slot = nullptr;
        for (u32 j = 0; j < h->n_more; ++j) { plan_work_free(h->more[j]); h->more[j] = nullptr; }
        return rc;
      }
    }
    I[i].w = *slot; I[i].p = p; I[i].max_tiles = clamp_limit(h->max_tiles, NT_MAX);
    (*slot)->planned = false; (*slot)->prefetched = false;
  }

  // ---- the durations every plan runs on ---------------------------------------------------
  {
    bool own = false;
    for (u32 i = 0; i < count; ++i) {
      Inst& x = I[i];
      PlanWork* w = x.w;
      if (x.p->dur_ns) {
        own = true;
        G10_TRY(slot_times_begin(x.p->dur_ns, K, w->dur_own, w->start_own, w->times_scratch, w->times_stats, x.times_check, s));
        w->dur = w->dur_own; w->start = w->start_own;
      } else {
        w->dur = h->dur; w->start = h->start; w->T = h->T;
      }
    }
    if (own) {
      G10_HIP(hipStreamSynchronize(s));
      for (u32 i = 0; i < count; ++i)
        if (I[i].p->dur_ns) G10_TRY(slot_times_end(I[i].times_check, &I[i].w->T));
    }
  }

  // The streaming kernels of the plans of a batch are short and many (a sort alone is a dozen launches):
  // they go to a few streams of the handle, plan by plan in turn, so that the plans' sequences overlap;
  // the loop launches and everything of a single plan stay on the caller's stream.
  if (count > 1 && !h->n_aux) {
    for (u32 k = 0; k < G10_AUX_STREAMS; ++k) {
      G10_HIP(hipStreamCreateWithFlags(&h->aux[k], hipStreamNonBlocking));
      h->n_aux = k + 1;
    }
  }
  auto stream_of = [&](u32 i) -> hipStream_t { return count == 1 ? s : h->aux[i % h->n_aux]; };
  auto sync_all = [&]() -> int {
    if (count > 1) for (u32 k = 0; k < h->n_aux; ++k) G10_HIP(hipStreamSynchronize(h->aux[k]));
    G10_HIP(hipStreamSynchronize(s));
    return G10_OK;
  };

  // ---- timelines before any eviction, candidate windows --------------------------------
  G10_HIP(hipEventRecord(I[0].w->ev[0], s));
  for (u32 i = 0; i < count; ++i) {
    Inst& x = I[i];
    hipStream_t q = stream_of(i);
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
    hc.rank = p->rank; hc.area = p->area;
    hc.C = C;
    hc.smax = h->max_size;
    G10_HIP(hipMemcpyAsync(w->ctl, &hc, sizeof hc, hipMemcpyHostToDevice, q));
    Timelines& tl = x.tl;
    tl.dur = w->dur; tl.P = w->P; tl.fre = w->fre; tl.H = w->H; tl.px = w->px; tl.otc = w->otc;
    tl.K = K; tl.Kp = w->Kp; tl.nch = w->nch; tl.spt = w->spt; tl.shift_ch = w->shift_ch;
    G10_HIP(hipMemsetAsync(w->peak_after, 0, 8, q));
    G10_HIP(hipMemsetAsync(w->wide, 0, 64, q));           // (no pass left open)
    hipLaunchKernelGGL(k_init_timelines, dim3(w->nch), dim3(G10_BLOCK), 0, q, tl, (const u64*)(h->pressure_buf + 1),
                       (const Ctl*)w->ctl, w->g_tot, w->g_lazyP, w->g_minOver, w->g_lazyH, w->g_hmax, w->g_hmat, w->g_hpend);
    hipLaunchKernelGGL(k_level1_init, dim3(1), dim3(LB), 0, q, (const u64*)w->g_tot, w->nch, w->base0, w->ctl);
    hipLaunchKernelGGL(k_ot_full, dim3(K / G10_BLOCK + 1), dim3(G10_BLOCK), 0, q, w->otc, (const u64*)w->base0, K, w->nch, w->shift_ch);
    G10_HIP(hipGetLastError());
    x.lead = i;
    for (u32 j = 0; j < i; ++j) {
      const g10_params* o = params + j;
      if (I[j].lead == j && o->dur_ns == p->dur_ns && o->bw_out_Bpus[0] == p->bw_out_Bpus[0] && o->bw_out_Bpus[1] == p->bw_out_Bpus[1] &&
          o->bw_in_Bpus[0] == p->bw_in_Bpus[0] && o->bw_in_Bpus[1] == p->bw_in_Bpus[1]) { x.lead = j; break; }
    }
    if (C && x.lead == i) {      // windows per destination; keep the candidates with at least one valid window
      hipLaunchKernelGGL(k_prep, dim3(gC), dim3(G10_BLOCK), 0, q, (const uint4*)h->per_by_start, (const u64*)h->per_size, w->start, K, w->T, C,
                         (const Ctl*)w->ctl, w->win, w->keep);
      G10_HIP(hipGetLastError());
      G10_TRY(scan_excl_u32(w->keep, w->keep, C, w->scratch32, q));
      G10_HIP(hipMemcpyAsync(&x.n, w->keep + C, sizeof(u32), hipMemcpyDeviceToHost, q));
    }
    G10_HIP(hipMemcpyAsync(&hc, w->ctl, sizeof hc, hipMemcpyDeviceToHost, q));
  }
  G10_TRY(sync_all());
  for (u32 i = 0; i < count; ++i) I[i].n = I[I[i].lead].n;

  // the candidate buffers of a plan; the value cache only where the plan reads the benefit as the clipped area
  auto cands_of = [](const Inst& x, int which) {
    Cands c = x.w->cd[which];
    if (x.p->area != G10_AREA_CLIPPED) { c.cv = nullptr; c.ce = nullptr; }
    return c;
  };

  // candidates of plan x into score order, in tiles
  auto retile = [&](Inst& x, bool first, hipStream_t q) -> int {
    PlanWork* w = x.w;
    x.tsh = tile_shift_for(x.n, x.max_tiles);
    const u32 tile = UNIT << x.tsh;
    x.nt = (u32)(((u64)x.n + tile - 1) / tile);
    x.n_pad = x.nt * tile;
    if (!x.n) return G10_OK;
    const u32 n = x.n;
    if (first) {
      const u32 gn = (n + G10_BLOCK - 1) / G10_BLOCK;
      // the two events take the kernel's own begin and end time stamps
      hipExtLaunchKernelGGL(score_full_kernel(x.p->rank, packed), dim3(gn), dim3(G10_BLOCK), 0, q, w->ev[2], w->ev[3], 0, (const uint4*)w->fw,
                            (const u64*)w->fs, n, (const u64*)w->otc, K, w->keys, (const Ctl*)w->ctl);
      x.timed_full = true;
    } else {
      u32 gn = (n + G10_BLOCK - 1) / G10_BLOCK;
      if (gn > 2048) gn = 2048;
      G10_HIP(hipMemsetAsync(&w->ctl->n_live, 0, sizeof(u32), q));
      if (x.p->rank == G10_RANK_RATIO)
        hipLaunchKernelGGL(k_rescore<true>, dim3(gn), dim3(G10_BLOCK), (size_t)N_ARR * (w->nch + 1) * 8, q, w->cd[x.cur], n,
                           (const u64*)w->px, (const u64*)w->g_base, K, w->nch, w->shift_ch, (const Ctl*)w->ctl,
                           w->keys, &w->ctl->n_live);
      else
        hipLaunchKernelGGL(k_rescore<false>, dim3(gn), dim3(G10_BLOCK), (size_t)N_ARR * (w->nch + 1) * 8, q, w->cd[x.cur], n,
                           (const u64*)w->px, (const u64*)w->g_base, K, w->nch, w->shift_ch, (const Ctl*)w->ctl,
                           w->keys, &w->ctl->n_live);
    }
    G10_HIP(hipGetLastError());
    u32 *keys = w->keys, *alt = w->keys_alt;
    u32 *from = w->sv, *from_alt = w->sv_alt;          // where every candidate of the new order stood in the old one
    G10_TRY(radix_sort_u32_pairs(&keys, &alt, &from, &from_alt, n, SCORE_SORT_BITS, w->hist, w->scratch32, q, true));
    G10_HIP(hipMemsetAsync(w->tkeys, 0, (u64)NT_MAX * 4, q));
    hipLaunchKernelGGL(k_tile_gather, dim3(x.n_pad / G10_BLOCK), dim3(G10_BLOCK), 0, q, (const u32*)keys, (const u32*)from, n, x.n_pad,
                       cands_of(x, x.cur), cands_of(x, x.cur ^ 1), 8 + x.tsh, w->tkeys);
    G10_HIP(hipGetLastError());
    x.cur ^= 1;
    return G10_OK;
  };

  // the same for many plans of a batch in the same launches: the jobs are filled plan by plan, then run on the caller's stream
  struct JobMax { u32 nb = 0, gn = 0, pad = 0, nch = 0; };
  auto fill_jobs = [&](Inst& x, u32 at, JobMax& m) {      // geometry (tsh, nt, n_pad) set, n > 0; the caller flips x.cur afterwards
    PlanWork* w = x.w;
    SortJob& sj = hsj[at];
    sj.keys = w->keys; sj.alt = w->keys_alt; sj.vals = w->sv; sj.valt = w->sv_alt; sj.hist = w->hist;
    sj.n = x.n; sj.nb = radix_blocks(x.n);
    TileJob& tj = htj[at];
    tj.src = x.own_pack ? cands_of(x, x.cur) : I[x.lead].pack_src; tj.dst = cands_of(x, x.cur ^ 1);
    x.own_pack = true;                                    // (every later order comes from the plan's own list)
    tj.n = x.n; tj.n_pad = x.n_pad; tj.tile_shift = 8 + x.tsh; tj.rank = x.p->rank;
    tj.sortkeys = w->keys; tj.tkeys = w->tkeys;
    tj.sorted = SCORE_SORT_PASSES & 1u ? w->keys_alt : w->keys; tj.from = SCORE_SORT_PASSES & 1u ? w->sv_alt : w->sv;
    tj.px = w->px; tj.g_base = w->g_base; tj.ctl = w->ctl; tj.K = K; tj.nch = w->nch; tj.shift_ch = w->shift_ch; tj.pad = 0;
    const u32 gn = (x.n + G10_BLOCK - 1) / G10_BLOCK;
    if (sj.nb > m.nb) m.nb = sj.nb;
    if (gn > m.gn) m.gn = gn;
    if (x.n_pad > m.pad) m.pad = x.n_pad;
    if (w->nch > m.nch) m.nch = w->nch;
  };
  auto run_jobs = [&](u32 nj, const JobMax& m, bool rescore) -> int {   // rescore: the keys come from a re-scoring of the lists (else they are there)
    if (!nj) return G10_OK;
    G10_HIP(hipMemcpyAsync(sort_jobs, hsj, (size_t)nj * sizeof(SortJob), hipMemcpyHostToDevice, s));
    G10_HIP(hipMemcpyAsync(tile_jobs, htj, (size_t)nj * sizeof(TileJob), hipMemcpyHostToDevice, s));
    hipLaunchKernelGGL(k_retile_begin_jobs, dim3(1, nj), dim3(G10_BLOCK), 0, s, (const TileJob*)tile_jobs);
    if (rescore)
      hipLaunchKernelGGL(k_rescore_jobs, dim3(m.gn > 2048 ? 2048 : m.gn, nj), dim3(G10_BLOCK), (size_t)N_ARR * (m.nch + 1) * 8, s,
                         (const TileJob*)tile_jobs);
    G10_HIP(hipGetLastError());
    G10_TRY(radix_sort_u32_pairs_jobs(sort_jobs, nj, m.nb, SCORE_SORT_BITS, true, s));
    hipLaunchKernelGGL(k_tile_gather_jobs, dim3(m.pad / G10_BLOCK, nj), dim3(G10_BLOCK), 0, s, (const TileJob*)tile_jobs);
    G10_HIP(hipGetLastError());
    return G10_OK;
  };

  u32 n_active = 0, nj0 = 0;
  JobMax max0;
  size_t lds_max = 0;
  for (u32 i = 0; i < count; ++i) {
    Inst& x = I[i];
    x.overtime_before = x.hc.overtime_before;
    x.n_valid = x.n;
    // every pass removes a candidate or stops, so the launches are bounded
    x.max_launches = count == 1 ? (u64)x.n / RETILE_PASSES + 3 : (u64)x.n + 3;   // (a launch by the clock makes a pass at least)
    if (x.hc.done) continue;
    ++n_active;
    // the windows, and the copy of them the first scoring pass reads, may be another plan's; the first plan
    // of such a group that gets here writes the copy
    PlanWork* const lw = I[x.lead].w;
    const bool writes_fw = !I[x.lead].fw_done;
    if (x.n && (writes_fw || count == 1)) {
      // (the packed list depends on the windows only: in a batch the first plan of a group packs it, the
      // others gather their first order straight from that list, which nobody writes before they have)
      hipLaunchKernelGGL(k_pack, dim3(gC), dim3(G10_BLOCK), 0, stream_of(i), (const uint4*)h->per_by_start, (const u64*)h->per_size, (const uint4*)lw->win,
                         (const u32*)lw->keep, C, cands_of(x, x.cur), writes_fw ? lw->fw : (uint4*)nullptr, writes_fw ? lw->fs : (u64*)nullptr, packed ? 1u : 0u);
      G10_HIP(hipGetLastError());
      if (writes_fw) {
        I[x.lead].fw_done = true;
        I[x.lead].pack_src = x.w->cd[x.cur];
        I[x.lead].pack_src.cv = nullptr; I[x.lead].pack_src.ce = nullptr;
        if (count > 1) G10_HIP(hipEventRecord(lw->ev[2], stream_of(i)));
      }
    } else if (x.n) x.own_pack = false;
    if (count == 1) G10_TRY(retile(x, true, s));
    else {
      // a batch: every plan's scoring pass on its stream, then the sorts and the tiles of all plans in the same launches
      PlanWork* w = x.w;
      x.tsh = tile_shift_for(x.n, x.max_tiles);
      const u32 tile = UNIT << x.tsh;
      x.nt = (u32)(((u64)x.n + tile - 1) / tile);
      x.n_pad = x.nt * tile;
      if (x.n) {
        const u32 gn = (x.n + G10_BLOCK - 1) / G10_BLOCK;
        if (!writes_fw) G10_HIP(hipStreamWaitEvent(stream_of(i), lw->ev[2], 0));         // (recorded when an earlier plan wrote the copy)
        hipLaunchKernelGGL(score_full_kernel(x.p->rank, packed), dim3(gn), dim3(G10_BLOCK), 0, stream_of(i), (const uint4*)lw->fw, (const u64*)lw->fs, x.n,
                           (const u64*)w->otc, K, w->keys, (const Ctl*)w->ctl);
        G10_HIP(hipGetLastError());
        fill_jobs(x, nj0, max0);
        ++nj0;
        x.cur ^= 1;
      }
    }
    const size_t lds = loop_lds_bytes(x.w->nch, x.nt);
    if (lds > lds_max) lds_max = lds;
  }
  if (count > 1) {
    G10_TRY(sync_all());
    G10_TRY(run_jobs(nj0, max0, false));
  }
  if (!h->lds_opt_in && lds_max > 64 * 1024) {
    G10_TRY(loop_allow_large_lds());
    h->lds_opt_in = true;
  }

  // ---- the greedy loops: one workgroup per plan, side by side ------------------------------
  // Long lists are put back into score order every RETILE_PASSES passes or more: the tiles the
  // loop looks at are dense with live candidates again, and the list is cut to those that can
  // still score.  A batch ends its launches by the clock instead, so that no plan waits long for
  // the slowest one.
  // (a batch re-tiles half as often: its loops run side by side, its re-tilings one after the other)
  const u32 retile_every = count == 1 ? RETILE_PASSES : 2 * RETILE_PASSES;
  const bool timed_loop = n_active != 0;
  // The results of a finished plan: the pressure with the lazy adds applied and its peak, then the
  // copies to one block of pinned host memory (so that they run as plain DMA), grown when a plan
  // needs more.  In a batch they go out on the plan's own stream as soon as the plan is done, beside
  // the loops of the others.
  auto send_results = [&](u32 i) -> int {
    Inst& x = I[i];
    PlanWork* w = x.w;
    const Ctl& hc = x.hc;
    hipStream_t q = stream_of(i);
    x.results_sent = true;
    hipLaunchKernelGGL(k_finish, dim3(K / G10_BLOCK / 4 + 1), dim3(G10_BLOCK), 0, q, x.tl, (const u64*)w->g_lazyP, w->pressure_after,
                       w->peak_after);
    G10_HIP(hipGetLastError());
    G10_HIP(hipMemcpyAsync(&peaks[i], w->peak_after, 8, hipMemcpyDeviceToHost, q));
    const size_t need = (size_t)K * 8 + hc.n_mig * sizeof(g10_migration) + hc.n_drop * sizeof(g10_dropped);
    if (need > w->h_block_bytes) {
      if (w->h_block) { mem_host_free(w->h_block); w->h_block = nullptr; w->h_block_bytes = 0; }
      const size_t want = need + need / 4 + 4096;
      if (mem_host_alloc(&w->h_block, want) != G10_OK) { w->h_block = nullptr; return G10_ENOMEM; }
      w->h_block_bytes = want;
    }
    w->h_pressure = (u64*)w->h_block;
    w->h_records = (g10_migration*)(w->h_pressure + K);
    w->h_dropped = (g10_dropped*)(w->h_records + hc.n_mig);
    if (hc.n_mig) G10_HIP(hipMemcpyAsync(w->h_records, w->records, hc.n_mig * sizeof(g10_migration), hipMemcpyDeviceToHost, q));
    if (hc.n_drop) G10_HIP(hipMemcpyAsync(w->h_dropped, w->dropped, hc.n_drop * sizeof(g10_dropped), hipMemcpyDeviceToHost, q));
    G10_HIP(hipMemcpyAsync(w->h_pressure, w->pressure_after, (u64)K * 8, hipMemcpyDeviceToHost, q));
    return G10_OK;
  };

  if (timed_loop) G10_HIP(hipEventRecord(I[0].w->ev[4], s));
  if (clocked) { G10_HIP(hipStreamSynchronize(s)); phase_end(0); }
  while (n_active) {
    u32 na = 0, n_by_kind[4] = {0, 0, 0, 0};
    size_t lds = 0;
    for (u32 pass = 0; pass < 4 * count; ++pass) {         // the plans of one ranking key and benefit reading side by side: one kernel each
      const u32 i = pass % count, kind = pass / count;
      Inst& x = I[i];
      if (x.hc.done || 2 * x.p->area + x.p->rank != kind) continue;
      ++n_by_kind[kind];
      if (x.launches++ > x.max_launches) return G10_EDEVICE;
      PlanWork* w = x.w;
      who[na] = i;
      LoopArgs& la = hargs[na++];
      la.tl = x.tl;
      la.g_tot = w->g_tot; la.g_lazyP = w->g_lazyP; la.g_minOver = w->g_minOver; la.g_lazyH = w->g_lazyH; la.g_hmax = w->g_hmax;
      la.g_base = w->g_base;
      la.g_keys = w->tkeys; la.ctl = w->ctl; la.records = w->records; la.rec_ab = w->rec_ab; la.dropped = w->dropped;
      la.rec_h = w->rec_h; la.g_hmat = w->g_hmat; la.g_hpend = w->g_hpend;
      la.cd = cands_of(x, x.cur); la.n_pad = x.n_pad; la.nt = x.nt; la.tshift = x.tsh;
      la.pass_budget = x.n > RETILE_MIN_CANDS && count == 1 ? RETILE_PASSES : PASS_BUDGET;
      la.tick_budget = count > 1 ? BATCH_LAUNCH_TICKS : 0;
      // one plan ranked by benefit / cost: with the scoring kernel where the list is long and the
      // last round of launches scored much of it per pass (or none has run yet)
      la.wide = nullptr; la.wide_min = 0; la.pass_stop = 0; la.wide_last_seq = 0;
      x.wide = false;
      if (count == 1 && x.p->rank == G10_RANK_RATIO && x.p->area == G10_AREA_BAND && x.n >= WIDE_MIN_CANDS) {
        const u64 dp = x.hc.passes - x.seen_passes_w, du = x.hc.units_scored - x.seen_units;
        la.wide = w->wide;                       // (always there for this kind of plan: a pass may have been left open)
        if (x.launches == 1 || du >= (u64)WIDE_MIN_UNITS * dp) {
          x.wide = true;
          la.wide_min = WIDE_MIN_UNITS;
          la.pass_stop = x.hc.passes + la.pass_budget;
          la.wide_last_seq = x.loop_seq + la.pass_budget + 1;
        }
        x.loop_seq += x.wide ? la.pass_budget + 1 : 1;
        x.seen_passes_w = x.hc.passes; x.seen_units = x.hc.units_scored;
      }
      const size_t l = loop_lds_bytes(w->nch, x.nt);
      if (l > lds) lds = l;
    }
    G10_HIP(hipMemcpyAsync(h->loop_args, hargs, (size_t)na * sizeof(LoopArgs), hipMemcpyHostToDevice, s));
    if (count == 1 && I[0].wide) {
      // pairs of loop and scoring kernel: every launch of the loop kernel starts a pass at least (or
      // finds nothing left to do), so this many reach the round's last pass; one more launch ends
      // the pass the last pair may have left open
      for (u32 g = 0; g < hargs[0].pass_budget; ++g) {
        G10_TRY(loop_launch((const LoopArgs*)h->loop_args, 1, lds, 1u, 0u, s));
        G10_TRY(loop_wide_launch((const LoopArgs*)h->loop_args, I[0].w->nch, s));
      }
      G10_TRY(loop_launch((const LoopArgs*)h->loop_args, 1, lds, 1u, 0u, s));
    } else
    for (u32 kind = 0, first = 0; kind < 4; first += n_by_kind[kind], ++kind)
      if (n_by_kind[kind]) G10_TRY(loop_launch((const LoopArgs*)h->loop_args + first, n_by_kind[kind], lds, kind & 1u, kind >> 1, s));
    hipLaunchKernelGGL(k_ctl_collect, dim3(na), dim3(G10_WAVE), 0, s, (const LoopArgs*)h->loop_args, ctl_side);
    G10_HIP(hipGetLastError());
    G10_HIP(hipMemcpyAsync(hctl, ctl_side, (size_t)na * sizeof(Ctl), hipMemcpyDeviceToHost, s));
    G10_HIP(hipStreamSynchronize(s));
    if (clocked) phase_end(1);
    for (u32 k = 0; k < na; ++k) I[who[k]].hc = hctl[k];
    n_active = 0;
    u32 nj = 0;                                               // the re-tilings of a batch: every plan's in the same launches
    JobMax mx;
    for (u32 i = 0; i < count; ++i) {
      Inst& x = I[i];
      if (x.hc.done) {
        if (count > 1 && !x.results_sent) G10_TRY(send_results(i));     // (the stream was synchronised: the plan's state is final)
        continue;
      }
      ++n_active;
      // (the cadence counts the rounds of commits: ranking passes and the further rounds made from their lists)
      if (x.n > RETILE_MIN_CANDS && x.hc.passes + x.hc.more_rounds - x.seen_passes >= retile_every) {
        x.seen_passes = x.hc.passes + x.hc.more_rounds;
        if (x.counted && x.hc.n_live < x.n) x.n = x.hc.n_live;   // live candidates come first in the list
        x.retile_cands += x.n;
        if (count == 1) G10_TRY(retile(x, false, s));
        else {
          x.tsh = tile_shift_for(x.n, x.max_tiles);
          const u32 tile = UNIT << x.tsh;
          x.nt = (u32)(((u64)x.n + tile - 1) / tile);
          x.n_pad = x.nt * tile;
          if (x.n) {
            fill_jobs(x, nj, mx);
            ++nj;
            x.cur ^= 1;
          }
        }
        x.counted = true;
        ++x.retiles;
      }
    }
    G10_TRY(run_jobs(nj, mx, true));
    if (clocked && nj) { G10_HIP(hipStreamSynchronize(s)); phase_end(2); }
  }
  if (timed_loop) G10_HIP(hipEventRecord(I[0].w->ev[5], s));

  // ---- results ---------------------------------------------------------------------------
  for (u32 i = 0; i < count; ++i)
    if (!I[i].results_sent) G10_TRY(send_results(i));
  if (count > 1) for (u32 k = 0; k < h->n_aux; ++k) G10_HIP(hipStreamSynchronize(h->aux[k]));
  G10_HIP(hipEventRecord(I[0].w->ev[1], s));
  G10_HIP(hipStreamSynchronize(s));
  if (clocked) phase_end(3);
  float ms = 0.f, loop_ms = 0.f;
  G10_HIP(hipEventElapsedTime(&ms, I[0].w->ev[0], I[0].w->ev[1]));
  if (timed_loop) G10_HIP(hipEventElapsedTime(&loop_ms, I[0].w->ev[4], I[0].w->ev[5]));

  for (u32 i = 0; i < count; ++i) {
    Inst& x = I[i];
    PlanWork* w = x.w;
    const Ctl& hc = x.hc;
    float full_ms = 0.f;
    if (x.timed_full) G10_HIP(hipEventElapsedTime(&full_ms, w->ev[2], w->ev[3]));
    w->planned = true; w->plan_cap = x.p->gpu_cap_bytes; w->plan_n_mig = hc.n_mig;
    g10_result* out = outs + i;
    memset(out, 0, sizeof *out);
    out->status = (int32_t)hc.status;
    out->n_migrations = hc.n_mig; out->n_iterations = hc.n_iter; out->n_dropped = hc.n_drop; out->n_cand_evals = hc.n_evals;
    out->peak_before = h->peak; out->peak_after = peaks[i];
    out->overtime_before_ns = x.overtime_before; out->overtime_after_ns = hc.overtime_after;
    out->migrations = w->h_records; out->dropped = w->h_dropped; out->pressure_after = w->h_pressure;
    out->plan_ms = ms;
    g10_counters& ct = h->counters[i];
    ct.score_full_ms = full_ms; ct.score_full_cands = x.n_valid;
    ct.loop_ms = loop_ms; ct.loop_launches = hc.launches; ct.loop_passes = hc.passes; ct.loop_retiles = x.retiles;
    ct.retile_cands = x.retile_cands;
    ct.loop_cands_scored = hc.units_scored * UNIT + hc.list_rescored; ct.loop_second_rounds = hc.second_rounds; ct.loop_chunk_jobs = hc.jobs_run;
    ct.loop_area_evals = hc.area_evals; ct.loop_area_refused = hc.area_refused;
    ct.loop_wide_rounds = hc.wide_rounds;
    ct.loop_more_rounds = hc.more_rounds;
    ct.batch_prepare_ms = phase_ms[0]; ct.batch_loops_ms = phase_ms[1]; ct.batch_retile_ms = phase_ms[2]; ct.batch_results_ms = phase_ms[3];
  }
  h->n_counters = count;
  return G10_OK;
}

int plan_run(g10_plan_s* h, const g10_params* p, g10_result* out) { return plan_batch_run(h, p, 1, out); }

