// Host side of the C ABI declared in include/ams.h: argument checks, workspace carving and the
// order of the launches.  Nothing here touches device memory or waits for the stream.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include "ams_internal.h"

namespace ams {

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Number of 32-query column blocks the scoring kernels are instantiated for.
static int padded_queries(int n, bool bf16) {
  const int nb = (n + 31) / 32;
  const int avail_bf16[] = {1, 2, 4, 7, 8}, avail_f32[] = {1, 2, 4};
  if (bf16) {
    for (int v : avail_bf16)
      if (nb <= v) return v * 32;
  } else {
    for (int v : avail_f32)
      if (nb <= v) return v * 32;
  }
  return 0;
}

// Tokens per workgroup of the scoring sweeps: as many as possible (the query window is loaded once per
// workgroup), but few enough that the launch has a couple of thousand workgroups to fill 256 CUs.
static int pick_score_chunk(size_t units, int t_max, bool paged) {
  // measured on 256 units: 4096 tokens at 32k positions (1.060 ms per step against 1.077 with 2048 and
  // 1.13 with 1024), 1024 at 2176 positions (0.208 against 0.229 with 2048); 512 and 256 lose to the
  // per-workgroup load of the query window
  // paged pools (16384 ragged units of up to 16384 positions): 26.4 ms per step with 1024 against 27.3 with
  // 2048, 30.8 with 4096 and 28.0 with 512 -- the eight heads of a (layer, sequence, chunk) share each 2 KB
  // stripe of the pool, and short chunks keep their workgroups close together in time
  int chunk = paged ? 1024 : kScoreChunk;
  while (chunk > 1024 && units * (size_t)div_up(t_max, chunk) < 2048) chunk /= 2;
  return chunk;
}

WsLayout ws_layout(const ams_params* p) {
  WsLayout w;
  const size_t units = (size_t)p->n_layers * p->batch * p->n_kv_heads;
  w.score_chunk = pick_score_chunk(units, p->t_max, false);
  w.score_chunk_paged = pick_score_chunk(units, p->t_max, true);
  w.n_chunks = div_up(p->t_max, w.score_chunk);
  w.n_chunks_paged = div_up(p->t_max, w.score_chunk_paged);
  const size_t nc_cap = (size_t)max(w.n_chunks, w.n_chunks_paged);  // the parameters do not say which layout comes
  w.n_pad = padded_queries(p->group * p->window, p->kv_dtype == AMS_BF16);
  const size_t vec = align256(units * (size_t)p->t_stride * sizeof(float));
  size_t o = 0;
  w.part_stats = o; o += align256(units * (nc_cap + 1) * (size_t)w.n_pad * sizeof(float2));
  w.fin_stats = o;  o += align256(units * (size_t)w.n_pad * sizeof(float4));
  w.u = o;          o += vec;
  w.g = o;          o += vec;
  w.m_used = o;     o += vec;
  w.bounds = o;     o += align256(units * (size_t)(p->n_segments + 1) * sizeof(int32_t));
  w.seg_mass = o;   o += align256(units * (size_t)p->n_segments * sizeof(float));
  w.quota = o;      o += align256(units * (size_t)p->n_segments * sizeof(int32_t));
  w.kbar = o;       o += align256(units * nc_cap * (size_t)p->head_dim * sizeof(double));
  w.park = o;       o += align256(park_score_ws_bytes(w.n_pad));
  w.n_chunks4k = div_up(p->t_max, kChunk);
  w.vc_part = o;    o += align256(units * (size_t)div_up(p->t_max, 128) * 2 * sizeof(double));  // finest producer: 256 positions per entry
  w.mpart = o;      o += align256(units * w.n_chunks4k * sizeof(double));
  w.cpre = o;       o += align256(units * (size_t)(p->n_segments + 1) * sizeof(double));
  w.n_words = div_up(p->t_max, 32);
  w.flags = o;      o += align256(units * (size_t)w.n_words * sizeof(uint32_t));
  w.csum = o;       o += align256(units * sizeof(double));
  w.total = o;
  return w;
}

static int check_params(const ams_params* p) {
  if (!p) return AMS_ERR_INVALID_ARG;
  if (p->n_layers < 1 || p->batch < 1 || p->n_kv_heads < 1 || p->group < 1 || p->window < 1 ||
      p->head_dim < 1 || p->t_max < 1 || p->t_stride < p->t_max || p->budget < 1 || p->n_segments < 1 ||
      p->q_min < 0 || p->n_sink < 0 || p->n_last < 0 || (p->causal != 0 && p->causal != 1))
    return AMS_ERR_INVALID_ARG;
  if (p->kv_dtype != AMS_F32 && p->kv_dtype != AMS_BF16) return AMS_ERR_INVALID_ARG;
  if (!(p->seg_delta >= 0.f) || p->l_min < 0 || p->l_max < 0 || p->pool_kernel < 0) return AMS_ERR_INVALID_ARG;
  if (p->pool_kernel > 1 && (p->pool_kernel % 2 == 0 || p->pool_kernel > 63)) return AMS_ERR_INVALID_ARG;
  if (p->seg_delta == 0.f && (p->l_min != 0 || p->l_max != 0)) return AMS_ERR_INVALID_ARG;
  if (p->seg_delta > 0.f) {
    if (p->seg_delta < 1.f / 1024.f || (p->l_max > 0 && p->l_min > p->l_max)) return AMS_ERR_INVALID_ARG;
    // room for every segment the split / merge pass can produce
    const int64_t most = (int64_t)initial_segments(p->seg_delta) + (p->l_max > 0 ? p->t_max / p->l_max : 0);
    if (p->n_segments < most) return AMS_ERR_INVALID_ARG;
  }
  if (!(p->ema_lambda >= 0.f && p->ema_lambda < 1.f) || !(p->ema_beta >= 0.f && p->ema_beta <= 1.f) ||
      !(p->mass_eps > 0.f) || isinf(p->mass_eps))
    return AMS_ERR_INVALID_ARG;
  if (p->scorer < AMS_SCORER_LAST_QUERY || p->scorer > AMS_SCORER_REDUNDANCY) return AMS_ERR_INVALID_ARG;
  if (p->scorer == AMS_SCORER_REDUNDANCY &&
      (!(p->mix_lambda >= 0.f && p->mix_lambda <= 1.f) || p->score_kernel < 0 || p->score_kernel > 63 ||
       (p->score_kernel > 1 && p->score_kernel % 2 == 0)))
    return AMS_ERR_INVALID_ARG;
  if (p->scorer == AMS_SCORER_EXPECTED_VNORM && !(p->vnorm_eps >= 0.f)) return AMS_ERR_INVALID_ARG;
  if (p->score_path < AMS_SCORE_PATH_AUTO || p->score_path > AMS_SCORE_PATH_ONE_LAUNCH) return AMS_ERR_INVALID_ARG;
  if (p->head_dim != 64 && p->head_dim != 128) return AMS_ERR_UNSUPPORTED;
  if (p->n_segments > 1024) return AMS_ERR_UNSUPPORTED;
  const int64_t units = (int64_t)p->n_layers * p->batch * p->n_kv_heads;
  if (units > 65535) return AMS_ERR_UNSUPPORTED;
  if ((int64_t)p->group * p->window > 256) return AMS_ERR_UNSUPPORTED;
  if (padded_queries(p->group * p->window, p->kv_dtype == AMS_BF16) == 0) return AMS_ERR_UNSUPPORTED;
  return AMS_OK;
}

static int check_view(const ams_params* p, const ams_kv_view* v, int64_t rows_needed, bool need_v) {
  if (!v || !v->k || (need_v && !v->v)) return AMS_ERR_INVALID_ARG;
  if (v->layout == AMS_LAYOUT_DENSE) {
    if (v->t_capacity < rows_needed) return AMS_ERR_INVALID_ARG;
  } else if (v->layout == AMS_LAYOUT_PAGED) {
    if (!v->block_table || v->max_blocks_per_seq < 1 || v->n_slots < 16) return AMS_ERR_INVALID_ARG;
    if (v->block_size != 16) return AMS_ERR_UNSUPPORTED;
    if ((int64_t)v->max_blocks_per_seq * 16 < rows_needed) return AMS_ERR_INVALID_ARG;
  } else {
    return AMS_ERR_INVALID_ARG;
  }
  (void)p;
  return AMS_OK;
}

static Dims make_dims(const ams_params* p) {
  Dims d;
  d.L = p->n_layers;
  d.B = p->batch;
  d.H = p->n_kv_heads;
  d.G = p->group;
  d.W = p->window;
  d.D = p->head_dim;
  d.N = p->group * p->window;
  d.units = p->n_layers * p->batch * p->n_kv_heads;
  d.t_max = p->t_max;
  d.t_stride = p->t_stride;
  return d;
}

static KvDev make_kv(const ams_params* p, const ams_kv_view* v, void* base) {
  KvDev k;
  k.base = (char*)base;
  k.block_table = v->block_table;
  k.t_capacity = v->t_capacity;
  k.n_slots = v->n_slots;
  k.layout = v->layout;
  k.max_blocks = v->max_blocks_per_seq;
  k.B = p->batch;
  k.H = p->n_kv_heads;
  k.row_bytes = p->head_dim * (p->kv_dtype == AMS_BF16 ? 2 : 4);
  return k;
}


// ---- per-kernel timing (host-side bookkeeping of HIP events; no device memory) ----
namespace {
constexpr int kMaxMarks = 4096;
struct Profiler {
  bool on = false;
  int n = 0;
  hipEvent_t ev[kMaxMarks];
  const char* label[kMaxMarks];
  int created = 0;
} g_prof;
}  // namespace

void prof_mark(const char* label, hipStream_t s);
static int status_of(hipError_t e) {
  if (e == hipSuccess) return AMS_OK;
  return e == hipErrorNotSupported ? AMS_ERR_UNSUPPORTED : AMS_ERR_HIP;  // a pinned path that does not apply
}
static int hip_status(hipError_t e, hipStream_t s) {
  prof_mark("end", s);  // closes the interval of the call's last kernel
  return status_of(e);
}

void prof_mark(const char* label, hipStream_t s) {
  if (!g_prof.on || g_prof.n >= kMaxMarks) return;
  if (g_prof.n >= g_prof.created) {
    if (hipEventCreate(&g_prof.ev[g_prof.created]) != hipSuccess) return;
    ++g_prof.created;
  }
  if (hipEventRecord(g_prof.ev[g_prof.n], s) != hipSuccess) return;
  g_prof.label[g_prof.n++] = label;
}

}  // namespace ams

using namespace ams;

extern "C" {

const char* ams_status_string(int status) {
  switch (status) {
    case AMS_OK: return "ok";
    case AMS_ERR_INVALID_ARG: return "invalid argument";
    case AMS_ERR_UNSUPPORTED: return "unsupported configuration";
    case AMS_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case AMS_ERR_HIP: return "HIP launch failed";
    default: return "unknown status";
  }
}

size_t ams_workspace_bytes(const ams_params* p) {
  if (check_params(p) != AMS_OK) return 0;
  return ws_layout(p).total;
}

int ams_debug_set_wait_limit(int polls) {
  if (polls < 0) return AMS_ERR_INVALID_ARG;
  set_park_wait_limit(polls);
  return AMS_OK;
}

int ams_profile_begin(void) {
  g_prof.n = 0;
  g_prof.on = true;
  return AMS_OK;
}

int ams_profile_end(void* stream, int max_entries, const char** labels, float* ms) {
  if (!g_prof.on) return 0;
  prof_mark("end", (hipStream_t)stream);
  g_prof.on = false;
  if (g_prof.n < 2) return 0;
  if (hipEventSynchronize(g_prof.ev[g_prof.n - 1]) != hipSuccess) return -AMS_ERR_HIP;
  int out = 0;
  for (int i = 0; i + 1 < g_prof.n && out < max_entries; ++i) {
    if (!strcmp(g_prof.label[i], "end")) continue;
    float t = 0.f;
    if (hipEventElapsedTime(&t, g_prof.ev[i], g_prof.ev[i + 1]) != hipSuccess) return -AMS_ERR_HIP;
    if (labels) labels[out] = g_prof.label[i];
    if (ms) ms[out] = t;
    ++out;
  }
  return out;
}

int ams_workspace_layout(const ams_params* p, ams_workspace_view* out) {
  const int rc = check_params(p);
  if (rc) return rc;
  if (!out) return AMS_ERR_INVALID_ARG;
  const WsLayout wl = ws_layout(p);
  out->u = wl.u;
  out->g = p->scorer == AMS_SCORER_MEAN_WINDOW ? wl.u : wl.g;
  out->m_used = wl.m_used;
  out->bounds = wl.bounds;
  out->seg_mass = wl.seg_mass;
  out->quota = wl.quota;
  return AMS_OK;
}

int ams_score(const ams_params* p, const ams_kv_view* src, const int32_t* seq_lens, const void* q,
              float* u, float* g, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_params(p);
  if (rc) return rc;
  const bool need_v = p->scorer == AMS_SCORER_EXPECTED_VNORM;
  if ((rc = check_view(p, src, p->t_max, need_v))) return rc;
  if (!seq_lens || !q || !u || !ws) return AMS_ERR_INVALID_ARG;
  if (p->scorer != AMS_SCORER_EXTERNAL && !g) return AMS_ERR_INVALID_ARG;
  if (p->scorer != AMS_SCORER_MEAN_WINDOW && p->scorer != AMS_SCORER_EXTERNAL && g == u)
    return AMS_ERR_INVALID_ARG;
  const WsLayout wl = ws_layout(p);
  if (ws_bytes < wl.total) return AMS_ERR_WORKSPACE_TOO_SMALL;
  const KvDev vdev = make_kv(p, src, src->v);
  return hip_status(launch_score(p, make_dims(p), make_kv(p, src, src->k), need_v ? &vdev : nullptr, seq_lens, q, u, g,
                                 nullptr, nullptr, (char*)ws, wl, (hipStream_t)stream), (hipStream_t)stream);
}

int ams_ema_update(const ams_params* p, const int32_t* seq_lens, const float* u, float* credit,
                   float* m_used, void* ws, size_t ws_bytes, void* stream) {
  const int rc = check_params(p);
  if (rc) return rc;
  if (!seq_lens || !u || !credit || !m_used || !ws) return AMS_ERR_INVALID_ARG;
  const WsLayout wl = ws_layout(p);
  if (ws_bytes < wl.total) return AMS_ERR_WORKSPACE_TOO_SMALL;
  return hip_status(launch_ema(p, make_dims(p), seq_lens, u, credit, m_used, VcInfo{false, 0, 0}, (char*)ws, wl,
                               (hipStream_t)stream), (hipStream_t)stream);
}

int ams_mass_segment(const ams_params* p, const int32_t* seq_lens, const float* m_used,
                     int32_t* bounds, float* seg_mass, void* ws, size_t ws_bytes, void* stream) {
  const int rc = check_params(p);
  if (rc) return rc;
  if (!seq_lens || !m_used || !bounds || !seg_mass || !ws) return AMS_ERR_INVALID_ARG;
  const WsLayout wl = ws_layout(p);
  if (ws_bytes < wl.total) return AMS_ERR_WORKSPACE_TOO_SMALL;
  return hip_status(launch_segment(p, make_dims(p), seq_lens, m_used, bounds, seg_mass, (char*)ws, wl,
                                   (hipStream_t)stream), (hipStream_t)stream);
}

int ams_mass_segment_static(const ams_params* p, const int32_t* seq_lens, const float* m_used,
                            int32_t* bounds, float* seg_mass, void* stream) {
  const int rc = check_params(p);
  if (rc) return rc;
  if (!seq_lens || !m_used || !bounds || !seg_mass) return AMS_ERR_INVALID_ARG;
  // the chunk totals and the prefix values at the cuts live in the library's own array
  WsLayout wl = ws_layout(p);
  const size_t units = (size_t)p->n_layers * p->batch * p->n_kv_heads;
  wl.vc_part = 0;  // not touched by the segmentation kernels
  wl.mpart = 0;
  wl.cpre = align256(units * (size_t)wl.n_chunks4k * sizeof(double));
  const size_t need = wl.cpre + align256(units * (size_t)(p->n_segments + 1) * sizeof(double));
  if (need > kStaticScratchBytes) return AMS_ERR_UNSUPPORTED;
  char* scratch_ptr = nullptr;
  if (static_scratch(&scratch_ptr) != hipSuccess) return AMS_ERR_HIP;
  return hip_status(launch_segment(p, make_dims(p), seq_lens, m_used, bounds, seg_mass, scratch_ptr, wl,
                                   (hipStream_t)stream), (hipStream_t)stream);
}

int ams_select(const ams_params* p, const int32_t* seq_lens, const float* g, const int32_t* bounds,
               const float* seg_mass, int32_t* quota, int32_t* idx, int32_t* n_kept,
               void* ws, size_t ws_bytes, void* stream) {
  const int rc = check_params(p);
  if (rc) return rc;
  if (!seq_lens || !g || !bounds || !seg_mass || !quota || !idx || !n_kept) return AMS_ERR_INVALID_ARG;
  uint32_t* flags = nullptr;
  const WsLayout wl = ws_layout(p);
  if (p->n_sink > 0 || p->n_last > 0) {  // the kept set is assembled in a bitmap
    if (!ws) return AMS_ERR_INVALID_ARG;
    if (ws_bytes < wl.total) return AMS_ERR_WORKSPACE_TOO_SMALL;
    flags = (uint32_t*)((char*)ws + wl.flags);
  }
  return hip_status(launch_select(p, make_dims(p), seq_lens, g, bounds, const_cast<float*>(seg_mass), quota, idx,
                                  n_kept, flags, wl.n_words, (hipStream_t)stream),
                    (hipStream_t)stream);
}

int ams_compact(const ams_params* p, const ams_kv_view* src, const int32_t* idx, const int32_t* n_kept,
                const ams_kv_view* dst, const float* credit_src, float* credit_dst, void* stream) {
  int rc = check_params(p);
  if (rc) return rc;
  const int64_t keep = p->budget < p->t_max ? p->budget : p->t_max;
  if ((rc = check_view(p, src, p->t_max, true))) return rc;
  if ((rc = check_view(p, dst, keep, true))) return rc;
  if (!idx || !n_kept) return AMS_ERR_INVALID_ARG;
  if (src->layout == AMS_LAYOUT_DENSE && dst->layout == AMS_LAYOUT_DENSE &&
      (src->k == dst->k || src->v == dst->v))
    return AMS_ERR_INVALID_ARG;  // out of place only; paged views may share a pool (other blocks)
  return hip_status(launch_compact(p, make_dims(p), make_kv(p, src, src->k), make_kv(p, src, src->v),
                                   make_kv(p, dst, dst->k), make_kv(p, dst, dst->v), idx, n_kept,
                                   credit_src, credit_dst, (hipStream_t)stream), (hipStream_t)stream);
}

int ams_compress_step(const ams_params* p, const ams_kv_view* src, const int32_t* seq_lens,
                      const void* q, float* credit, const ams_kv_view* dst, float* credit_dst,
                      int32_t* idx, int32_t* n_kept, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_params(p);
  if (rc) return rc;
  if (p->scorer == AMS_SCORER_EXTERNAL) return AMS_ERR_INVALID_ARG;
  const int64_t keep = p->budget < p->t_max ? p->budget : p->t_max;
  if ((rc = check_view(p, src, p->t_max, true))) return rc;
  if ((rc = check_view(p, dst, keep, true))) return rc;
  if (!seq_lens || !q || !credit || !idx || !n_kept || !ws) return AMS_ERR_INVALID_ARG;
  if (src->layout == AMS_LAYOUT_DENSE && dst->layout == AMS_LAYOUT_DENSE &&
      (src->k == dst->k || src->v == dst->v))
    return AMS_ERR_INVALID_ARG;  // out of place only; paged views may share a pool (other blocks)
  const WsLayout wl = ws_layout(p);
  if (ws_bytes < wl.total) return AMS_ERR_WORKSPACE_TOO_SMALL;
  char* w = (char*)ws;
  const Dims d = make_dims(p);
  hipStream_t s = (hipStream_t)stream;
  float* u = (float*)(w + wl.u);
  float* g = p->scorer == AMS_SCORER_MEAN_WINDOW ? u : (float*)(w + wl.g);
  float* m_used = (float*)(w + wl.m_used);
  int32_t* bounds = (int32_t*)(w + wl.bounds);
  float* seg_mass = (float*)(w + wl.seg_mass);
  int32_t* quota = (int32_t*)(w + wl.quota);
  hipError_t e;
  VcInfo vc{false, 0, 0};
  const KvDev vdev = make_kv(p, src, src->v);
  if ((e = launch_score(p, d, make_kv(p, src, src->k), &vdev, seq_lens, q, u, g, credit, &vc, w, wl, s)) != hipSuccess)
    return status_of(e);
  if ((e = launch_unit_mass(p, d, seq_lens, u, credit, m_used, bounds, seg_mass, quota, idx, n_kept,
                            (uint32_t*)(w + wl.flags), wl.n_words, vc, w, wl, s)) != hipSuccess)
    return AMS_ERR_HIP;
  if ((e = launch_select(p, d, seq_lens, g, bounds, seg_mass, quota, idx, n_kept, (uint32_t*)(w + wl.flags),
                         wl.n_words, s, true)) != hipSuccess)
    return AMS_ERR_HIP;
  if ((e = launch_compact(p, d, make_kv(p, src, src->k), make_kv(p, src, src->v), make_kv(p, dst, dst->k),
                          make_kv(p, dst, dst->v), idx, n_kept, credit, credit_dst, s)) != hipSuccess)
    return AMS_ERR_HIP;
  prof_mark("end", s);
  return AMS_OK;
}

}  // extern "C"
