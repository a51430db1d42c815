// Shared declarations of the HIP implementation behind include/ams.h.
#ifndef AMS_INTERNAL_H
#define AMS_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ams.h"

namespace ams {

// Device-side description of one of K / V of a cache.
struct KvDev {
  char* base;
  const int32_t* block_table;
  int64_t t_capacity;  // dense: rows per unit slab
  int64_t n_slots;     // paged: slots per layer
  int32_t layout;
  int32_t max_blocks;
  int32_t B, H;
  int32_t row_bytes;
};

// Address of the row of token t of unit (l, b, h).
__device__ __forceinline__ char* kv_row(const KvDev& kv, int l, int b, int h, int t) {
  if (kv.layout == AMS_LAYOUT_DENSE) {
    const int64_t unit = ((int64_t)l * kv.B + b) * kv.H + h;
    return kv.base + (unit * kv.t_capacity + t) * (int64_t)kv.row_bytes;
  }
  int64_t slot = (int64_t)kv.block_table[(int64_t)b * kv.max_blocks + (t >> 4)] * 16 + (t & 15);
  slot = slot < 0 ? 0 : (slot >= kv.n_slots ? kv.n_slots - 1 : slot);  // a bad table entry stays inside the pool
  return kv.base + (((int64_t)l * kv.n_slots + slot) * kv.H + h) * (int64_t)kv.row_bytes;
}

struct Dims {
  int32_t L, B, H, G, W, D, N;  // N = G*W
  int32_t units;
  int32_t t_max;
  int64_t t_stride;
};

__device__ __forceinline__ void unit_coords(const Dims& d, int unit, int& l, int& b, int& h) {
  h = unit % d.H;
  const int lb = unit / d.H;
  b = lb % d.B;
  l = lb / d.B;
}

// Length of sequence b as the kernels use it: a value outside [0, t_max] (a caller's mistake) is
// clamped, so that no kernel leaves the arrays sized for t_max.
__device__ __forceinline__ int seq_len(const Dims& d, const int32_t* seq_lens, int b) {
  return max(0, min(seq_lens[b], d.t_max));
}

#ifndef AMS_SCORE_CHUNK
#define AMS_SCORE_CHUNK 4096
#endif
constexpr int kScoreChunk = AMS_SCORE_CHUNK;  // most tokens per workgroup of the scoring kernels
constexpr int kChunk = 4096;       // positions per workgroup of the mass / prefix kernels

// Segments the thresholds k*delta (every k >= 1 with k*delta < 1) cut the unit interval into.
inline int initial_segments(float delta) {
  int k = 1;
  while (k <= 4096 && (double)k * (double)delta < 1.0) ++k;
  return k;
}

inline int div_up(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

// Workspace carving (offsets in bytes, 256-byte aligned).
struct WsLayout {
  size_t part_stats, fin_stats, u, g, m_used, bounds, seg_mass, quota, kbar, park, vc_part, mpart, cpre, flags, csum, total;
  int n_chunks, n_pad;
  int score_chunk;  // tokens per workgroup of the scoring kernels for these parameters, dense cache
  int score_chunk_paged, n_chunks_paged;  // the same for a paged cache
  int n_chunks4k;  // chunks of kChunk positions per unit
  int n_words;     // 32-position words of the kept-set bitmap per unit
};
WsLayout ws_layout(const ams_params* p);

// Where the scorer left the per-chunk sums that Eq. (1) and the EMA need (have = false: nowhere).
struct VcInfo {
  bool have;
  int stride;  // entries per unit row of ws + wl.vc_part
  int tokens;  // positions covered by one entry
};

// Optional per-kernel timing: when collection is on, every launcher calls prof_mark(label, stream)
// right before a kernel launch, which records a HIP event on that stream.  Off: a single branch.
void prof_mark(const char* label, hipStream_t s);

// Scratch that belongs to the library (a __device__ array, one copy per GPU) for the entry point that may
// not take a workspace: its size, and its address on the current device (looked up once per device).
constexpr size_t kStaticScratchBytes = 1u << 20;
hipError_t static_scratch(char** out);

// ---- launchers (each returns hipGetLastError() of its launches) ----
// credit and vc are optional: when vc is given, the scorer also leaves the per-chunk sums that
// launch_ema needs in the workspace and describes them in *vc.
// v: the values of the cache, read by AMS_SCORER_EXPECTED_VNORM only (else may be null)
hipError_t launch_score(const ams_params* p, const Dims& d, const KvDev& k, const KvDev* v,
                        const int32_t* seq_lens,
                        const void* q, float* u, float* g, const float* credit, VcInfo* vc, char* ws,
                        const WsLayout& wl, hipStream_t s);
// The one-read scorer (score_park.hip): limits of its cluster bookkeeping, bytes of its exchange area, and the
// word in that area that a bounded wait raises when it expires (the kernels after the scorer read it).
constexpr int kParkMaxWorkgroups = 1024, kParkMaxClusters = 1024, kParkMaxMembers = 1024;
size_t park_score_ws_bytes(int n_pad);
int32_t* park_status_word(char* ws, const WsLayout& wl);
void set_park_wait_limit(int polls);  // polls a bounded wait of that scorer may take (0: its default)
hipError_t launch_score_oneread(const ams_params* p, const Dims& d, const KvDev& k, const int32_t* seq_lens,
                                const void* q, float* u, float* g, const float* credit, bool want_vc,
                                int* vc_stride, int* vc_tokens, char* ws, const WsLayout& wl,
                                hipStream_t s, bool* ran);
// The one-launch scorer for short caches (score_unit.hip); *ran = false when it does not apply.  It leaves
// one (sum of max(u,0)+eps, sum of old credit) entry per unit at a.vc_part[unit] when a.vc_part is set.
struct ScoreArgs;
hipError_t launch_score_unit(const ScoreArgs& a, bool bf16, int head_dim, int mode, hipStream_t s, bool* ran);
constexpr int kUnitScorerMinUnits = 128;  // fewer units leave most of the 256 CUs idle: the sweeps win there

// The chunked kernels behind ams_ema_update and ams_mass_segment (the fused step uses launch_unit_mass).
hipError_t launch_ema(const ams_params* p, const Dims& d, const int32_t* seq_lens, const float* u,
                      float* credit, float* m_used, const VcInfo& vc, char* ws, const WsLayout& wl,
                      hipStream_t s);
hipError_t launch_segment(const ams_params* p, const Dims& d, const int32_t* seq_lens,
                          const float* m_used, int32_t* bounds, float* seg_mass, char* ws, const WsLayout& wl,
                          hipStream_t s);
// The fused step's mass / EMA / segmentation / quota stages in one launch (one workgroup per unit); it also
// leaves the -1 tail of idx, the kept counts and the cleared bitmap, so launch_select follows with
// quota_done = true.  vc: the chunk sums the scorer left, if any.
hipError_t launch_unit_mass(const ams_params* p, const Dims& d, const int32_t* seq_lens, const float* u,
                            float* credit, float* m_used, int32_t* bounds, float* seg_mass, int32_t* quota,
                            int32_t* idx, int32_t* n_kept, uint32_t* flags, int n_words, const VcInfo& vc,
                            char* ws, const WsLayout& wl, hipStream_t s);
// flags (n_words words per unit): bitmap of the kept set, needed when a must-keep set is configured, else
// may be null.  quota_done: the quotas (and what the quota kernels do besides) are already in place.
hipError_t launch_select(const ams_params* p, const Dims& d, const int32_t* seq_lens, const float* g,
                         const int32_t* bounds, float* seg_mass, int32_t* quota, int32_t* idx,
                         int32_t* n_kept, uint32_t* flags, int n_words, hipStream_t s, bool quota_done = false);
hipError_t launch_compact(const ams_params* p, const Dims& d, const KvDev& ks, const KvDev& vs,
                          const KvDev& kd, const KvDev& vd, const int32_t* idx, const int32_t* n_kept,
                          const float* credit_src, float* credit_dst, hipStream_t s);

}  // namespace ams
#endif
