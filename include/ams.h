/*
 * ams.h - C ABI of the MI355X (gfx950) hot path of Adaptive Mass-Segmented
 * (AMS) KV-cache compression.
 *
 * One "compression event" (Alg. 1 of the paper) bounds a KV cache of length T
 * to a budget T_keep.  It runs independently for every unit = (layer,
 * sequence, KV head) ("retention policies [are computed] independently for
 * each attention head", Sec. 3.1).  The entry points below are the stages of
 * that event plus a fused call that chains them.
 *
 * General conventions
 *  - Pointers marked [dev] are DEVICE pointers owned by the caller; pointers
 *    marked [host] are host pointers read before the call returns.  The
 *    library allocates no device memory, never frees anything and never
 *    synchronises: all work is enqueued on `stream` (a hipStream_t passed as
 *    void*, NULL = the default stream) and the call returns at once.
 *  - Every call returns an ams_status.  Argument errors are found on the host
 *    before anything is launched; nothing aborts or throws.
 *  - Units are ordered unit = (layer * batch + b) * n_kv_heads + h.
 *  - Per-unit fp32 vectors (u, g, credit, m_used) are rows of a
 *    [units, t_stride] array; only the first seq_lens[b] entries of a row are
 *    read or written.
 *  - A seq_lens[b] outside [0, t_max] is read as the nearest bound, and the
 *    compaction skips an index outside [0, t_max): wrong lengths or indices give
 *    wrong results for that unit, never an access outside the caller's buffers
 *    (as long as those have the documented sizes).
 *  - Positions are 0-based positions in the CURRENT cache (the mass curve is
 *    defined "over current KV-cache positions", Fig. 3 caption).
 *  - KV head h owns query heads h*group .. h*group + group - 1.
 */
#ifndef AMS_H
#define AMS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  AMS_OK = 0,
  AMS_ERR_INVALID_ARG = 1,         /* null pointer, size < 1, value out of range          */
  AMS_ERR_UNSUPPORTED = 2,         /* valid request this build has no kernel for          */
  AMS_ERR_WORKSPACE_TOO_SMALL = 3, /* ws_bytes < ams_workspace_bytes(...)                 */
  AMS_ERR_HIP = 4                  /* a HIP launch reported an error                      */
} ams_status;

typedef enum { AMS_F32 = 0, AMS_BF16 = 1 } ams_dtype;

/* Plug-in base scorer g (Sec. 3.3 "In-Segment Selection with a Plug-and-Play
 * Scorer").  The mass that places segments always comes from the mean
 * recent-window attention (Sec. 3.2); only the in-segment ranking changes. */
typedef enum {
  AMS_SCORER_LAST_QUERY = 0,  /* attention of the newest query of each head (TOVA-style)   */
  AMS_SCORER_MEAN_WINDOW = 1, /* g = u, the mean attention over the query window           */
  AMS_SCORER_KEYDIFF = 2,     /* negative cosine between a key and the mean key            */
  AMS_SCORER_EXPECTED = 3,    /* log Gaussian moment of the window's query distribution    */
  AMS_SCORER_EXTERNAL = 4,    /* caller supplies g (stage calls only)                      */
  AMS_SCORER_EXPECTED_VNORM = 5, /* value-weighted expected attention: p = softmax over the
                                   cache of the AMS_SCORER_EXPECTED scores,
                                   g = (p + vnorm_eps) * ||v||_2; reads V                  */
  AMS_SCORER_REDUNDANCY = 6   /* redundancy-aware score (Sec. 4 "Universality across diverse base
                                 scorers"): g = mix_lambda * a - (1 - mix_lambda) * p, a = u (averaged
                                 over score_kernel positions when that is > 1), p = softmax over the
                                 cache of r_t = mean cosine similarity of key t to the unit's other keys */
} ams_scorer;

/* How ams_score / ams_compress_step form the softmax statistics (the results agree to rounding;
 * ams_params.score_path).  AUTO lets the library choose; the other two pin the choice, for
 * measurements and tests. */
typedef enum {
  AMS_SCORE_PATH_AUTO = 0,
  AMS_SCORE_PATH_TWO_SWEEPS = 1, /* K is streamed twice: statistics, then usage; every configuration  */
  AMS_SCORE_PATH_ONE_READ = 2,   /* K is read once and held on chip between the two products: bf16,
                                    head_dim 128, at most 128 queries per KV head, dense layout, no
                                    causal window, mean-window / last-query / key-diversity scorers;
                                    AMS_ERR_UNSUPPORTED otherwise.  Its workgroups wait for one
                                    another (every wait bounded), so it wants the GPU to itself: if
                                    a wait expires, ams_compress_step writes n_kept = -1 for every
                                    unit and the outputs of the call are not to be used.  Slower
                                    than TWO_SWEEPS on the measured workloads; AUTO never takes it   */
  AMS_SCORE_PATH_ONE_LAUNCH = 3  /* short caches (t_max <= 4096): one workgroup walks a unit's keys
                                    twice in one launch; at most 128 queries per KV head, no causal
                                    window, no moment-based scorer; AMS_ERR_UNSUPPORTED otherwise.
                                    AUTO takes it when it applies and there are >= 128 units        */
} ams_score_path;

typedef enum {
  AMS_LAYOUT_DENSE = 0, /* K, V = [layers, batch, kv_heads, t_capacity, head_dim]          */
  AMS_LAYOUT_PAGED = 1  /* per layer a pool [n_slots, kv_heads, head_dim]; token p of
                           sequence b lives in slot block_table[b][p / 16] * 16 + p % 16  */
} ams_layout;

/* Problem statement of one event (Alg. 1 "Require").  Plain data, [host]. */
typedef struct {
  int32_t n_layers, batch, n_kv_heads;
  int32_t group;      /* G: query heads per KV head                                        */
  int32_t head_dim;   /* D: 64 or 128                                                      */
  int32_t window;     /* W: recent decoding queries per query head (Sec. 3.2)             */
  int32_t kv_dtype;   /* ams_dtype of K, V and Q                                           */
  int32_t t_max;      /* upper bound of every seq_lens[b]; sizes the launches              */
  int64_t t_stride;   /* row stride (elements) of the per-unit fp32 vectors, >= t_max      */
  int32_t budget;     /* T_keep                                                            */
  int32_t n_segments; /* S: segments of target mass Delta = 1/S (Sec. 3.3)                 */
  int32_t q_min;      /* minimum quota per non-empty segment (paper default 1)            */
  float ema_lambda;   /* credit decay, 0 <= lambda < 1; 0 = credit not used                */
  float ema_beta;     /* mass mixing, 0 <= beta <= 1 (paper default 0.9)                   */
  float mass_eps;     /* epsilon of Eq. (1), > 0                                           */
  int32_t scorer;     /* ams_scorer                                                        */
  int32_t n_sink;     /* must-keep: first n_sink positions always kept (Sec. 3.3); 0 = none */
  int32_t n_last;     /* must-keep: last n_last positions always kept; 0 = none            */
  int32_t causal;     /* 1: causal window with padded observations (App. A), see ams_score */
  float seg_delta;    /* 0: exactly n_segments segments of target mass 1/n_segments.
                         > 0: target mass Delta as printed (Sec. 3.3), variable number of
                         segments; n_segments is then the CAPACITY of the per-unit segment
                         arrays, see ams_mass_segment                                      */
  int32_t l_min;      /* seg_delta > 0: segments shorter than this are merged (0 = off)    */
  int32_t l_max;      /* seg_delta > 0: segments longer than this are split (0 = off)      */
  int32_t pool_kernel;/* odd k > 1: Eq. (1) sees the k-point centred mean of u (App. A); 0/1 = off */
  float vnorm_eps;    /* epsilon of AMS_SCORER_EXPECTED_VNORM, >= 0 (1e-2 in the paper's runs) */
  int32_t score_path; /* ams_score_path; 0 = the library chooses                                   */
  float mix_lambda;   /* AMS_SCORER_REDUNDANCY: weight of the importance term, in [0, 1] (0.07 in the
                         paper's runs)                                                              */
  int32_t score_kernel; /* AMS_SCORER_REDUNDANCY: odd k > 1 averages u over k positions first (7 in
                         the paper's runs); 0 / 1 = off                                            */
} ams_params;

/* A KV cache as the library sees it.  Plain data, [host]; k, v, block_table [dev]. */
typedef struct {
  int32_t layout;             /* ams_layout                                                */
  void* k;                    /* [dev]                                                     */
  void* v;                    /* [dev] may be NULL for ams_score                           */
  int64_t t_capacity;         /* dense: rows per unit slab                                 */
  const int32_t* block_table; /* paged: [dev] [batch, max_blocks_per_seq]                  */
  int32_t max_blocks_per_seq; /* paged                                                     */
  int32_t block_size;         /* paged: must be 16                                         */
  int64_t n_slots;            /* paged: slots per layer pool                               */
} ams_kv_view;

const char* ams_status_string(int status);

/* Bytes of scratch the calls below need for these parameters ([host], pure). */
size_t ams_workspace_bytes(const ams_params* p);

/* Where ams_compress_step leaves its intermediates inside the workspace (byte
 * offsets, [host], pure): u, g, m_used are fp32 [units, t_stride] (g == u for
 * AMS_SCORER_MEAN_WINDOW), bounds int32 [units, S+1], seg_mass fp32 [units, S],
 * quota int32 [units, S].  For inspection and tests; the layout is otherwise
 * private. */
typedef struct {
  size_t u, g, m_used, bounds, seg_mass, quota;
} ams_workspace_view;
int ams_workspace_layout(const ams_params* p, ams_workspace_view* out);

/*
 * Per-kernel timing for benchmarks (no citation: measurement aid, not part of
 * the method).  Between ams_profile_begin() and ams_profile_end() every kernel
 * the library launches is preceded by a HIP event on its stream.
 * ams_profile_end() records a final event on `stream`, WAITS for it (the only
 * call of this library that blocks the host), and writes up to max_entries
 * (label, milliseconds) pairs in launch order: the time from one kernel's
 * start marker to the next marker.  labels[i] points to a static string.
 * Returns the number of pairs written, or a negative ams_status.  Collection
 * is process-wide and not thread-safe; at most 4096 markers are kept.
 */
int ams_profile_begin(void);
int ams_profile_end(void* stream, int max_entries, const char** labels, float* ms);

/*
 * Testing aid for the one path of the library whose workgroups wait for one
 * another, AMS_SCORE_PATH_ONE_READ (no citation: not part of the method).  Its
 * waits are bounded polls; `polls` > 0 sets that bound for the launches that
 * follow (process-wide, not thread-safe), 0 restores the built-in one (about
 * 0.1 s).  With a bound of 1 every wait that is not satisfied at once expires,
 * every kernel still runs to its end, and ams_compress_step reports the expiry
 * as documented at ams_score_path (n_kept = -1 for every unit): the error path
 * can be exercised without hanging anything.  [host]; AMS_ERR_INVALID_ARG for a
 * negative bound.
 */
int ams_debug_set_wait_limit(int polls);

/*
 * ams_score - usage u and base score g (Alg. 1 step 1; Sec. 3.2; Sec. 3.3).
 *   s[n][t] = q_n . k_t / sqrt(D) over the N = G*W recent queries of the unit,
 *   p = softmax over t, u[t] = mean_n p[n][t]; g per p->scorer (g may equal u
 *   as a pointer only for AMS_SCORER_MEAN_WINDOW; for AMS_SCORER_EXTERNAL g is
 *   left untouched).
 *   p->causal == 1 (App. A "Mass construction"): query w of the window sits at
 *   position T-W+w and sees keys 0..T-W+w only (a query before position 0 does
 *   not exist); for a key seen by fewer than N (head, query) pairs every missing
 *   observation counts as the largest probability the key received from the
 *   pairs that see it.  The last-query, key-diversity and moment-based g are not
 *   affected (the newest query sees every key; the other two use no softmax).
 *   q  [dev] [layers, batch, kv_heads*group, window, head_dim], kv_dtype
 *   seq_lens [dev] [batch] int32, each in [1, t_max]
 *   u, g [dev] fp32 [units, t_stride], written
 *   Accuracy: the products run on the matrix cores with fp32 accumulation, so a
 *   logit carries an absolute error of about 1e-7 times the sum of the magnitudes
 *   of its D products, and a probability inherits it as a RELATIVE error.  u and
 *   g agree with an fp64 evaluation to 1e-5 relative while
 *   sum_d |q_d k_d| / sqrt(D) stays below about 100 (|logits| of a few tens:
 *   unit-variance queries and keys at D = 128 give about 7); beyond that the
 *   bound widens in proportion (3e-4 observed at magnitudes of a few thousand,
 *   fp32 cache).  No input overflows: the softmax is taken relative to the row
 *   maximum at any scale.
 */
int ams_score(const ams_params* p, const ams_kv_view* src, const int32_t* seq_lens, const void* q,
              float* u, float* g, void* ws, size_t ws_bytes, void* stream);

/*
 * ams_ema_update - Eq. (1) followed by the EMA credit (Sec. 3.3 "EMA Credit for
 * Temporal Stability"; Alg. 1 step 2):
 *   m = normalize(max(u',0)+eps), u' = u or, with pool_kernel = k > 1, the mean of u
 *   over the k positions centred on t that exist (App. A; Alg. 1 step 1);
 *   credit <- lambda*credit + (1-lambda)*m;
 *   m_used = normalize(beta*m + (1-beta)*normalize(credit)).
 * lambda == 0: m_used = m and credit <- m.
 *   u [dev] in; credit [dev] in/out; m_used [dev] out; all fp32 [units, t_stride]
 *   ws [dev] scratch of at least ams_workspace_bytes(p)
 */
int ams_ema_update(const ams_params* p, const int32_t* seq_lens, const float* u, float* credit,
                   float* m_used, void* ws, size_t ws_bytes, void* stream);

/*
 * ams_mass_segment - prefix sum of the mass and cut points (Sec. 3.3
 * "Mass-based adaptive segmentation"; Alg. 1 step 3).
 * seg_delta == 0 (Delta = 1/S, no length rules, exactly S = n_segments segments):
 *   bounds[0] = 0, bounds[S] = T, bounds[k] = 1 + min{ j : c(j) >= k/S } (T if the
 *   threshold is never reached); seg_mass[i] = sum of m_used over segment i.
 * seg_delta > 0 (as printed): cut points at the thresholds k*Delta (every k >= 1 with
 *   k*Delta < 1), then one pass over the initial segments from the left: a segment
 *   longer than l_max is split into ceil(L/l_max) parts whose lengths differ by at most
 *   one (longer parts first); a segment shorter than l_min joins its left neighbour,
 *   the very first one its right neighbour; empty segments vanish.  All resulting
 *   segments are non-empty; entries of bounds / seg_mass past them are T / 0.
 *   n_segments must be at least ceil(1/Delta) + t_max / l_max (AMS_ERR_INVALID_ARG
 *   otherwise), Delta at least 1/1024.
 *   bounds [dev] int32 [units, S+1]; seg_mass [dev] fp32 [units, S]
 *   ws [dev] scratch of at least ams_workspace_bytes(p)
 */
int ams_mass_segment(const ams_params* p, const int32_t* seq_lens, const float* m_used,
                     int32_t* bounds, float* seg_mass, void* ws, size_t ws_bytes, void* stream);

/*
 * ams_mass_segment_static - ams_mass_segment for callers that cannot allocate or carry a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same inputs, same
 * outputs, same kernels, but the scratch (chunk totals and prefix values at the cuts) is an array that
 * belongs to the library, 1 MiB per GPU, held until the process ends.  The call allocates nothing.
 *   Limit: 256-byte-rounded units * ceil(t_max / 4096) * 8 + units * (n_segments + 1) * 8 bytes must fit
 *   in 1 MiB (config 1: 51 KB); AMS_ERR_UNSUPPORTED otherwise, nothing launched.
 *   All calls on one GPU share the array: calls that overlap in time on one GPU (different streams) race;
 *   calls in stream order do not (every call rewrites what it reads).
 */
int ams_mass_segment_static(const ams_params* p, const int32_t* seq_lens, const float* m_used,
                            int32_t* bounds, float* seg_mass, void* stream);

/*
 * ams_select - segment quotas, in-segment top-k and the final kept set (Sec. 3.3
 * "Segment-wise Quota Allocation", "In-Segment Selection", must-keep rules; Alg. 1
 * steps 4-5).
 *   kept = min(budget, T).  Must-keep set: the first min(n_sink, kept) positions and
 *   the last min(n_last, kept - sinks) positions (the recent suffix gives way, sinks
 *   never do).  The segments share seg_budget = kept - |must-keep|.
 *   quota: floor min(q_min, L_i), remainder shared in proportion to seg_mass,
 *   no quota above the segment length, sum = seg_budget.
 *   idx: per segment the quota[i] positions of largest g (equal scores: lower
 *   position first; NaN ranks below everything), united with the must-keep set,
 *   duplicates removed, ascending; when the union is short of kept (a segment
 *   picked a must-keep position) the highest-scoring positions not yet in it are
 *   added, equal scores by lower position.  Entries from n_kept to budget are -1.
 *   quota [dev] int32 [units, S]; idx [dev] int32 [units, budget]; n_kept [dev] int32 [units]
 *   ws: may be NULL when n_sink == n_last == 0 (no scratch needed); otherwise [dev]
 *   scratch of at least ams_workspace_bytes(p), else AMS_ERR_INVALID_ARG /
 *   AMS_ERR_WORKSPACE_TOO_SMALL.
 */
int ams_select(const ams_params* p, const int32_t* seq_lens, const float* g, const int32_t* bounds,
               const float* seg_mass, int32_t* quota, int32_t* idx, int32_t* n_kept,
               void* ws, size_t ws_bytes, void* stream);

/*
 * ams_compact - gather of the kept rows (Alg. 1 step 6: K' = K[idx], V' = V[idx]);
 * with a paged destination it is the head-wise compaction of App. E:
 *   K_new[pi_new(b, j), h, :] <- K_old[pi_old(b, idx[b,h,j]), h, :].
 * Row j of unit (l,b,h) goes to row j of the destination unit slab (dense) or to
 * slot dst.block_table[b][j/16]*16 + j%16 (paged).  src and dst must not overlap.
 *   credit_src [dev] fp32 [units, t_stride] or NULL; credit_dst [dev] fp32
 *   [units, budget] (row j = credit_src[idx[j]]) or NULL.
 */
int ams_compact(const ams_params* p, const ams_kv_view* src, const int32_t* idx,
                const int32_t* n_kept, const ams_kv_view* dst, const float* credit_src,
                float* credit_dst, void* stream);

/*
 * ams_compress_step - one whole event (Alg. 1): score -> Eq. (1) -> EMA -> prefix
 * sum and boundaries -> quotas -> segmented top-k (+ must-keep set) ->
 * gather-compact, in that order, all enqueued on `stream`; every optional rule of
 * ams_params (causal window, pooling, target mass with split / merge, must-keep
 * set, scorer) applies as documented at the stage calls.  credit [units,
 * t_stride] is updated in place at full length; credit_dst [units, budget]
 * receives the kept tokens' credit.  src->v is read by the compaction and by
 * AMS_SCORER_EXPECTED_VNORM.  The call allocates nothing and waits for nothing,
 * so it may be recorded into a HIP graph.
 * Errors: AMS_ERR_INVALID_ARG for a null pointer, for p->scorer ==
 * AMS_SCORER_EXTERNAL and for dense src and dst that share a buffer;
 * AMS_ERR_WORKSPACE_TOO_SMALL; AMS_ERR_HIP if a launch fails.
 */
int ams_compress_step(const ams_params* p, const ams_kv_view* src, const int32_t* seq_lens,
                      const void* q, float* credit, const ams_kv_view* dst, float* credit_dst,
                      int32_t* idx, int32_t* n_kept, void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif
