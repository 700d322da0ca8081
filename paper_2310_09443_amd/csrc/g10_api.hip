// C-ABI entry points: argument checks, handle lifetime, read-backs.
#include "g10_internal.h"

#include <new>
#include <stdlib.h>
#include <string.h>

// The analysis' temporaries, once the handle's stream has been waited for after the analysis.
static void release_tmp(g10_plan_s* h) {
  mem_dev_free(h->tmp_arena);
  h->tmp_arena = nullptr;
}

static void handle_free(g10_plan_s* h) {
  if (!h) return;
  // what is released below is kept for the next call, not handed to the driver (which would wait
  // for the device by itself): nothing of this handle may still be running
  (void)hipStreamSynchronize(h->stream);
  for (u32 k = 0; k < h->n_aux; ++k) (void)hipStreamSynchronize(h->aux[k]);
  plan_work_free(h->work);
  for (u32 i = 0; i < h->n_more; ++i) plan_work_free(h->more[i]);
  free(h->more);
  free(h->counters);
  mem_dev_free(h->loop_args);
  for (u32 k = 0; k < h->n_aux; ++k) (void)hipStreamDestroy(h->aux[k]);
  mem_dev_free(h->arena);                      // every array of the analysis
  release_tmp(h);
  delete h;
}

extern "C" int g10_vitality(const g10_trace* tr, void* hip_stream, g10_plan_t** out_handle) {
  if (!tr || !out_handle) return G10_EINVAL;
  if (!tr->K || !tr->N || tr->K >= (1u << 31)) return G10_EINVAL;
  if (!tr->dur_ns || !tr->size_bytes || !tr->is_global) return G10_EINVAL;
  if (tr->P && (!tr->use_kernel || !tr->use_tensor)) return G10_EINVAL;
  g10_plan_s* h = new (std::nothrow) g10_plan_s();
  if (!h) return G10_ENOMEM;
  if (hipGetDevice(&h->device) != hipSuccess) { delete h; return G10_EDEVICE; }
  h->stream = (hipStream_t)hip_stream;
  h->K = tr->K; h->N = tr->N; h->P = tr->P; h->flags = tr->flags;
  const int rc = vitality_run(h, tr);
  if (rc) {
    (void)hipStreamSynchronize(h->stream);
    handle_free(h);
    return rc;
  }
  *out_handle = h;
  return G10_OK;
}

extern "C" int g10_vitality_info(const g10_plan_t* h, g10_vitality_stats* out) {
  if (!h || !out) return G10_EINVAL;
  out->n_uses = h->n_uses; out->n_periods = h->n_periods; out->peak_bytes = h->peak; out->iter_ns = h->T;
  return G10_OK;
}

extern "C" int g10_vitality_read(const g10_plan_t* h, int which, void* dst, uint64_t bytes) {
  if (!h || !dst) return G10_EINVAL;
  const void* src = nullptr;
  u64 want = 0;
  switch (which) {
    case 0: src = h->use_off; want = ((u64)h->N + 1) * 8; break;
    case 1: src = h->use_k; want = h->n_uses * 4; break;
    case 2: src = h->per_t; want = h->n_periods * 4; break;
    case 3: src = h->per_L; want = h->n_periods * 4; break;
    case 4: src = h->per_R; want = h->n_periods * 4; break;
    case 5: src = h->start; want = ((u64)h->K + 1) * 8; break;
    case 6: src = h->pressure_buf + 1; want = (u64)h->K * 8; break;
    default: return G10_EINVAL;
  }
  if (bytes != want) return G10_EINVAL;
  if (!want) return G10_OK;
  G10_HIP(hipMemcpyAsync(dst, src, want, hipMemcpyDeviceToHost, h->stream));
  G10_HIP(hipStreamSynchronize(h->stream));
  return G10_OK;
}

extern "C" int g10_plan(g10_plan_t* h, const g10_params* p, g10_result* out) {
  if (out) memset(out, 0, sizeof *out);
  if (!h || !p || !out) return G10_EINVAL;
  for (int d = 0; d < 2; ++d)
    if (!p->bw_out_Bpus[d] || !p->bw_in_Bpus[d]) return G10_EINVAL;
  if (p->rank > G10_RANK_RATIO || p->area > G10_AREA_CLIPPED) return G10_EINVAL;
  const int rc = plan_run(h, p, out);
  if (rc) {
    (void)hipStreamSynchronize(h->stream);
    memset(out, 0, sizeof *out);
  }
  release_tmp(h);                                 // (the results have been waited for, or the line above has)
  return rc;
}

extern "C" int g10_plan_counters(const g10_plan_t* h, uint32_t plan_index, g10_counters* out) {
  if (!h || !out || plan_index >= h->n_counters) return G10_EINVAL;
  *out = h->counters[plan_index];
  return G10_OK;
}

extern "C" int g10_plan_limits(g10_plan_t* h, uint32_t max_tiles, uint32_t max_chunks) {
  if (!h) return G10_EINVAL;
  h->max_tiles = max_tiles; h->max_chunks = max_chunks;
  return G10_OK;
}

extern "C" int g10_plan_batch(g10_plan_t* h, const g10_params* params, uint32_t count, g10_result* outs) {
  if (outs && count) memset(outs, 0, sizeof(g10_result) * (size_t)count);
  if (!h || !params || !outs || !count || count > 4096) return G10_EINVAL;
  for (uint32_t i = 0; i < count; ++i) {
    for (int d = 0; d < 2; ++d)
      if (!params[i].bw_out_Bpus[d] || !params[i].bw_in_Bpus[d]) return G10_EINVAL;
    if (params[i].rank > G10_RANK_RATIO || params[i].area > G10_AREA_CLIPPED) return G10_EINVAL;
  }
  const int rc = plan_batch_run(h, params, count, outs);
  if (rc) {
    (void)hipStreamSynchronize(h->stream);
    memset(outs, 0, sizeof(g10_result) * (size_t)count);
  }
  release_tmp(h);
  return rc;
}

extern "C" int g10_prefetch(g10_plan_t* h, g10_prefetch_result* out) {
  if (out) memset(out, 0, sizeof *out);
  if (!h || !out) return G10_EINVAL;
  const int rc = prefetch_run(h, out);
  if (rc) {
    (void)hipStreamSynchronize(h->stream);
    memset(out, 0, sizeof *out);
  }
  return rc;
}

extern "C" int g10_replay(g10_plan_t* h, const uint64_t* dur_ns, uint32_t eager, g10_replay_result* out) {
  if (out) memset(out, 0, sizeof *out);
  if (!h || !out) return G10_EINVAL;
  const int rc = replay_run(h, dur_ns, eager, out);
  if (rc) {
    (void)hipStreamSynchronize(h->stream);
    memset(out, 0, sizeof *out);
  }
  return rc;
}

extern "C" void g10_plan_free(g10_plan_t* h) { handle_free(h); }
