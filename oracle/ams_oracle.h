/*
 * CPU oracle for one Adaptive Mass-Segmented (AMS) KV compression event.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the plain, slow definition of what the
 * GPU library must compute; it is imported by tests, by the smoke check and by
 * the benchmark's CPU-baseline leg, never by the product path.  It shares no
 * code with the HIP kernels.
 *
 * Every function works on ONE unit = one (layer, sequence, KV head) triple
 * ("retention policies [are computed] independently for each attention head",
 * Sec. 3.1) with host pointers.  All accumulation is in double; every stored
 * result is rounded once to float.  Stages take the float outputs of the
 * previous stage, so a stage can be checked on its own.
 *
 * Pinned by tests (see tests/test_oracle_*.py): every function below.
 * Parity unpinned (documented choices nothing in the paper can confirm): the
 * value of eps in Eq. (1); plain-mean aggregation of the window softmax over
 * the G*W (head, query) pairs with scale 1/sqrt(D); the largest-remainder
 * reading of "round ... followed by a lightweight adjustment step"; credit of
 * gathered / appended tokens; population covariance and no value-norm term in
 * the expected-attention score; raw-key mean in the key-diversity score; which
 * probability stands in for a missing causal observation (the per-key maximum
 * over the pairs that see the key); the order in which equal scores are
 * trimmed or backfilled; the split / merge rules of amso_segment_adaptive
 * (the paper says "roughly equal" and "a neighboring segment") and the edge
 * handling of amso_pool; the form of the value weighting in amso_value_weight
 * (the paper names the scorer and its epsilon only); the whole form of
 * amso_redundancy_score (the paper gives one sentence and four parameter names).
 */
#ifndef AMS_ORACLE_H
#define AMS_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  AMSO_SCORER_LAST_QUERY = 0,  /* attention of the newest query of each head   */
  AMSO_SCORER_MEAN_WINDOW = 1, /* the usage u itself                            */
  AMSO_SCORER_KEYDIFF = 2,     /* negative cosine to the mean key               */
  AMSO_SCORER_EXPECTED = 3,    /* log Gaussian moment of the query window       */
  AMSO_SCORER_EXPECTED_VNORM = 5, /* amso_value_weight of the above (whole event only) */
  AMSO_SCORER_REDUNDANCY = 6   /* amso_redundancy_score of the usage (whole event only)  */
};

/* Step 1 of Alg. 1 (usage) + the plug-in base score g (Sec. 3.3 "In-Segment
 * Selection").  Q is [G][W][D] (query heads of this KV head, then window
 * position), K is [T][D], both already widened to float.  u, g are [T].
 * causal != 0 (App. A, "Mass construction"): query w of the window sits at
 * position T-W+w and sees keys 0..T-W+w; for a key seen by fewer than N
 * (head, query) pairs every missing observation counts as the largest
 * probability the key received from the pairs that see it. */
int amso_score(const float* Q, const float* K, int G, int W, int T, int D,
               int scorer, int causal, float* u, float* g);

/* Value-weighted expected attention: p = softmax over the cache of the log-moment
 * scores e [T]; g_t = (p_t + eps) * ||v_t||_2 with V [T][D] widened to float. */
int amso_value_weight(const float* e, const float* V, int T, int D, float eps, float* g);

/* Redundancy-aware score (Sec. 4 "Universality across diverse base scorers"; App. "Baseline
 * Configurations": recent attention importance combined with a cosine-similarity-based
 * redundancy penalty over the cached keys, parameters window 8, kernel 7, lambda 0.07).
 * Reading taken here:
 *   a   = u, or with kernel > 1 (odd) the amso_pool of u          (recent attention importance)
 *   r_t = mean over s != t of cos(k_t, k_s)  (0 for T == 1; a zero key has cosine 0 to everything)
 *   p   = softmax over t of r                                      (redundancy, on the scale of a: sums to 1)
 *   g_t = mix_lambda * a_t - (1 - mix_lambda) * p_t.
 * K [T][D] widened to float.  O(T^2 D): the definition written out. */
int amso_redundancy_score(const float* u, const float* K, int T, int D, float mix_lambda, int kernel,
                          float* g);

/* Eq. (1): m_t = (max(u_t,0)+eps) / sum_v (max(u_v,0)+eps). */
int amso_mass(const float* u, int T, float eps, float* m_cur);

/* Sec. 3.3 "EMA Credit" / Alg. 1 step 2.  credit is updated in place.
 * lambda == 0 takes the "credit not used" branch: m_used = m_cur bit for bit
 * (credit still becomes m_cur). */
int amso_ema(const float* m_cur, float* credit, int T, float lambda, float beta,
             float* m_used);

/* Alg. 1 step 3 with Delta = 1/S and no split/merge: bounds[0]=0,
 * bounds[S]=T, bounds[k] = 1 + first 0-based j whose inclusive prefix sum
 * reaches k/S (T if none).  seg_mass[i] = sum of m over [bounds[i],bounds[i+1]). */
int amso_segment(const float* m_used, int T, int S, int32_t* bounds, float* seg_mass);

/* Alg. 1 step 1 "optionally smooth" / App. A: mean of u over the `kernel` (odd)
 * positions centred on t that exist. */
int amso_pool(const float* u, int T, int kernel, float* out);

/* Alg. 1 step 3 as printed: thresholds k*delta (k*delta < 1), then split
 * (> l_max: ceil(L/l_max) near-equal parts, longer parts first) and merge
 * (< l_min: into the left neighbour; the first one into the right) in one pass
 * from the left; 0 switches a rule off.  bounds [cap+1], seg_mass [cap]; unused
 * entries are T and 0; *n_seg = number of segments (all non-empty).  -5 if cap
 * is too small. */
int amso_segment_adaptive(const float* m_used, int T, float delta, int l_min, int l_max, int cap,
                          int32_t* bounds, float* seg_mass, int32_t* n_seg);

/* Alg. 1 step 4: minimum quota, proportional share of the remainder, clip to
 * the segment length, adjust so the quotas sum to min(budget, T).  budget may be
 * 0 (a must-keep set that uses up everything): all quotas are 0 then. */
int amso_quota(const int32_t* bounds, const float* seg_mass, int S, int budget,
               int q_min, int32_t* quota);

/* Sec. 3.3 "must-keep rules": kept = min(budget, T); sink_eff = min(n_sink,
 * kept); last_eff = min(n_last, kept - sink_eff) (the recent suffix gives way,
 * sinks never do); seg_budget = kept - sink_eff - last_eff goes to amso_quota. */
int amso_must_keep(int T, int budget, int n_sink, int n_last, int* sink_eff, int* last_eff,
                   int* seg_budget);

/* Alg. 1 step 5, in-segment part: per segment the quota[i] largest g,
 * equal scores resolved towards the lower index, result ascending.
 * idx has room for sum(quota); returns the number written in *n_kept. */
int amso_select(const float* g, const int32_t* bounds, const int32_t* quota, int S,
                int32_t* idx, int32_t* n_kept);

/* Alg. 1 step 5, set part: union of seg_idx [n_seg] with the first sink_eff and
 * the last last_eff positions, duplicates removed, ascending; trimmed (lowest g
 * outside the must-keep set first, higher index first among equals) or
 * backfilled (highest g not yet kept, lower index first among equals) to
 * exactly target positions.  idx has room for target. */
int amso_finalize(const float* g, int T, const int32_t* seg_idx, int n_seg, int sink_eff,
                  int last_eff, int target, int32_t* idx, int32_t* n_kept);

/* Alg. 1 step 6: row gather of K, V (row_bytes bytes per token) and credit. */
int amso_compact(const void* K, const void* V, const float* credit, int64_t row_bytes,
                 const int32_t* idx, int n_kept, void* K_out, void* V_out, float* credit_out);

/* Paged form of the same gather (App. E): token p of the sequence lives in
 * physical slot table[p/block]*block + p%block; a slot holds H rows, row of
 * head h at ((slot*H)+h)*row_bytes.  Destination slot of compact position j is
 * taken from dst_table the same way. */
int amso_compact_paged(const void* K_pool, const void* V_pool, const int32_t* src_table,
                       void* K_pool_out, void* V_pool_out, const int32_t* dst_table,
                       int block, int H, int h, int64_t row_bytes,
                       const int32_t* idx, int n_kept);

/* One whole event for one unit, stages chained through their float outputs.
 * Any of the optional outputs may be NULL.  credit [T] in/out (full length,
 * updated), credit_out [n_kept] gathered. */
typedef struct {
  int G, W, T, D;
  int scorer;
  int budget, S, q_min;
  float lambda, beta, eps;
  int n_sink, n_last; /* must-keep sizes; 0, 0 = none */
  int causal;         /* see amso_score */
  float delta;        /* > 0: amso_segment_adaptive with S as the capacity; 0: amso_segment(S) */
  int l_min, l_max;   /* with delta > 0 */
  int pool_kernel;    /* > 1: amso_pool before Eq. (1) */
  float vnorm_eps;    /* eps of amso_value_weight (scorer AMSO_SCORER_EXPECTED_VNORM) */
  float mix_lambda;   /* amso_redundancy_score (scorer AMSO_SCORER_REDUNDANCY) */
  int score_kernel;   /* its pooling kernel (odd; 0 or 1 = none) */
} amso_unit_params;

int amso_compress_unit(const amso_unit_params* p, const float* Q, const float* K,
                       const float* V /* [T][D] widened; only read by AMSO_SCORER_EXPECTED_VNORM, else may be NULL */,
                       const void* K_rows, const void* V_rows, int64_t row_bytes,
                       float* credit,
                       float* u, float* g, float* m_used, int32_t* bounds, float* seg_mass,
                       int32_t* quota, int32_t* idx, int32_t* n_kept,
                       void* K_out, void* V_out, float* credit_out);

/* Runs amso_compress_unit over n_units independent units laid out back to back
 * (strides given in elements / bytes), with a plain thread parallel-for over
 * units.  Used for timing the oracle and for checking many units at once.
 * Outputs idx [n_units][budget] (tail -1), n_kept [n_units], u/g [n_units][T]
 * (either may be NULL).  When K_rows, V_rows ([n_units][T] rows of row_bytes in the
 * storage dtype) and K_out, V_out ([n_units][budget] rows) are given the rows are
 * gathered too, credit_out [n_units][budget] likewise.
 * Returns the number of threads used (>0) or <0 on error. */
int amso_compress_many(const amso_unit_params* p, int n_units, int n_threads,
                       const float* Q, int64_t q_stride,
                       const float* K, int64_t k_stride,
                       const float* V /* [n_units][T][D] or NULL, see amso_compress_unit */,
                       float* credit, int64_t c_stride,
                       float* u, float* g, int32_t* idx, int32_t* n_kept,
                       const void* K_rows, const void* V_rows, int64_t row_bytes,
                       void* K_out, void* V_out, float* credit_out);

#ifdef __cplusplus
}
#endif
#endif
