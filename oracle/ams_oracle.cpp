// CPU oracle for one AMS KV-compression event.  TEST INFRASTRUCTURE ONLY: see
// ams_oracle.h.  Plain loops, double accumulation, one rounding to float per
// stored value, no blocking or fusion beyond what the paper's steps state.
#include "ams_oracle.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <thread>
#include <vector>

namespace {

inline bool is_nan(float x) { return x != x; }

// Ordering used by the in-segment top-k: larger score first, NaN counts as
// -infinity, equal scores (including -0 == +0) keep the lower index first.
inline float sel_value(float x) { return is_nan(x) ? -INFINITY : x; }

}  // namespace

extern "C" {

// ---------------------------------------------------------------------------
// Usage u (Sec. 3.2; Alg. 1 step 1) and base score g (Sec. 3.3).
//   s[n][t] = q_n . k_t / sqrt(D)
//   p[n][t] = softmax over t of s[n][:]
//   u[t]    = mean over the N = G*W (head, query) pairs of p[n][t]
//
// causal != 0 (App. A "Mass construction"): the window's queries sit at the last W
// positions, query w at position T-W+w, and see the keys up to their own position
// only; a query whose position would be negative does not exist.  A key among the
// newest W-1 is therefore observed by fewer than N pairs; each missing observation
// is replaced by the largest probability that key received from the pairs that do
// see it.
// ---------------------------------------------------------------------------
int amso_score(const float* Q, const float* K, int G, int W, int T, int D,
               int scorer, int causal, float* u, float* g) {
  if (!Q || !K || !u || !g || G < 1 || W < 1 || T < 1 || D < 1) return -1;
  const int N = G * W;
  const double inv_sqrt_d = 1.0 / std::sqrt((double)D);
  std::vector<double> s((size_t)T), usage((size_t)T, 0.0), last((size_t)T, 0.0);
  std::vector<double> seen_max((size_t)T, 0.0);
  std::vector<int> seen((size_t)T, 0);

  for (int n = 0; n < N; ++n) {
    const float* q = Q + (size_t)n * D;
    const int w = n % W;
    const int visible = causal ? T - W + w + 1 : T;  // keys 0 .. visible-1
    if (visible < 1) continue;
    double smax = -INFINITY;
    for (int t = 0; t < visible; ++t) {
      const float* k = K + (size_t)t * D;
      double dot = 0.0;
      for (int d = 0; d < D; ++d) dot += (double)q[d] * (double)k[d];
      s[t] = dot * inv_sqrt_d;
      smax = std::max(smax, s[t]);
    }
    double z = 0.0;
    for (int t = 0; t < visible; ++t) {
      s[t] = std::exp(s[t] - smax);
      z += s[t];
    }
    const bool newest = w == W - 1;  // last query of this head's window
    for (int t = 0; t < visible; ++t) {
      const double p = s[t] / z;
      usage[t] += p;
      seen[t] += 1;
      seen_max[t] = std::max(seen_max[t], p);
      if (newest) last[t] += p;
    }
  }
  for (int t = 0; t < T; ++t)
    u[t] = (float)((usage[t] + (double)(N - seen[t]) * seen_max[t]) / (double)N);

  switch (scorer) {
    case AMSO_SCORER_MEAN_WINDOW:
      for (int t = 0; t < T; ++t) g[t] = u[t];
      break;
    case AMSO_SCORER_LAST_QUERY:
      for (int t = 0; t < T; ++t) g[t] = (float)(last[t] / (double)G);
      break;
    case AMSO_SCORER_KEYDIFF: {
      // g_t = -cos(k_t, kbar), kbar = mean key of the unit.
      std::vector<double> kbar((size_t)D, 0.0);
      for (int t = 0; t < T; ++t)
        for (int d = 0; d < D; ++d) kbar[d] += (double)K[(size_t)t * D + d];
      double nb = 0.0;
      for (int d = 0; d < D; ++d) {
        kbar[d] /= (double)T;
        nb += kbar[d] * kbar[d];
      }
      nb = std::sqrt(nb);
      for (int t = 0; t < T; ++t) {
        const float* k = K + (size_t)t * D;
        double dot = 0.0, nk = 0.0;
        for (int d = 0; d < D; ++d) {
          dot += (double)k[d] * kbar[d];
          nk += (double)k[d] * (double)k[d];
        }
        const double den = std::sqrt(nk) * nb;
        g[t] = den > 0.0 ? (float)(-dot / den) : 0.0f;
      }
      break;
    }
    case AMSO_SCORER_EXPECTED: {
      // Queries of the window modelled as Gaussian(mu, Sigma); the score is the
      // log of E[exp(q.k/sqrt(D))] = mu.k/sqrt(D) + k' Sigma k / (2 D).
      std::vector<double> mu((size_t)D, 0.0), sigma((size_t)D * D, 0.0);
      for (int n = 0; n < N; ++n)
        for (int d = 0; d < D; ++d) mu[d] += (double)Q[(size_t)n * D + d];
      for (int d = 0; d < D; ++d) mu[d] /= (double)N;
      for (int n = 0; n < N; ++n)
        for (int a = 0; a < D; ++a) {
          const double da = (double)Q[(size_t)n * D + a] - mu[a];
          for (int b = 0; b < D; ++b)
            sigma[(size_t)a * D + b] += da * ((double)Q[(size_t)n * D + b] - mu[b]);
        }
      for (size_t i = 0; i < sigma.size(); ++i) sigma[i] /= (double)N;
      for (int t = 0; t < T; ++t) {
        const float* k = K + (size_t)t * D;
        double lin = 0.0, quad = 0.0;
        for (int a = 0; a < D; ++a) {
          lin += mu[a] * (double)k[a];
          double row = 0.0;
          for (int b = 0; b < D; ++b) row += sigma[(size_t)a * D + b] * (double)k[b];
          quad += (double)k[a] * row;
        }
        g[t] = (float)(lin * inv_sqrt_d + quad / (2.0 * (double)D));
      }
      break;
    }
    default:
      return -2;
  }
  return 0;
}

// Value-weighted expected attention (Sec. 3.3 plug-in scorer, "expected-attention-based scorer"
// with its epsilon): the log-moment scores e are turned into a distribution over the cache,
// p = softmax_t(e), and every token is weighted by the length of its value vector:
// g_t = (p_t + eps) * ||v_t||_2.
int amso_value_weight(const float* e, const float* V, int T, int D, float eps, float* g) {
  if (!e || !V || !g || T < 1 || D < 1 || !(eps >= 0.0f)) return -1;
  double emax = -INFINITY;
  for (int t = 0; t < T; ++t) emax = std::max(emax, (double)e[t]);
  double z = 0.0;
  for (int t = 0; t < T; ++t) z += std::exp((double)e[t] - emax);
  for (int t = 0; t < T; ++t) {
    double n2 = 0.0;
    for (int d = 0; d < D; ++d) n2 += (double)V[(size_t)t * D + d] * (double)V[(size_t)t * D + d];
    g[t] = (float)((std::exp((double)e[t] - emax) / z + (double)eps) * std::sqrt(n2));
  }
  return 0;
}

// Redundancy-aware score: importance minus a softmax-normalised mean cosine similarity to the other keys.
int amso_redundancy_score(const float* u, const float* K, int T, int D, float mix_lambda, int kernel, float* g) {
  if (!u || !K || !g || T < 1 || D < 1 || !(mix_lambda >= 0.0f && mix_lambda <= 1.0f)) return -1;
  if (kernel < 0 || (kernel > 1 && kernel % 2 == 0)) return -1;
  std::vector<float> a(u, u + T);
  if (kernel > 1) {
    const int rc = amso_pool(u, T, kernel, a.data());
    if (rc) return rc;
  }
  std::vector<double> norm((size_t)T);
  for (int t = 0; t < T; ++t) {
    double n2 = 0.0;
    for (int d = 0; d < D; ++d) n2 += (double)K[(size_t)t * D + d] * (double)K[(size_t)t * D + d];
    norm[t] = std::sqrt(n2);
  }
  std::vector<double> r((size_t)T, 0.0);
  for (int t = 0; t < T && T > 1; ++t) {
    double acc = 0.0;
    for (int s = 0; s < T; ++s) {
      if (s == t) continue;
      double dot = 0.0;
      for (int d = 0; d < D; ++d) dot += (double)K[(size_t)t * D + d] * (double)K[(size_t)s * D + d];
      const double den = norm[t] * norm[s];
      acc += den > 0.0 ? dot / den : 0.0;
    }
    r[t] = acc / (double)(T - 1);
  }
  double rmax = -INFINITY;
  for (int t = 0; t < T; ++t) rmax = std::max(rmax, r[t]);
  double z = 0.0;
  for (int t = 0; t < T; ++t) z += std::exp(r[t] - rmax);
  const double lam = (double)mix_lambda;
  for (int t = 0; t < T; ++t) g[t] = (float)(lam * (double)a[t] - (1.0 - lam) * (std::exp(r[t] - rmax) / z));
  return 0;
}

// Eq. (1).
int amso_mass(const float* u, int T, float eps, float* m_cur) {
  if (!u || !m_cur || T < 1 || !(eps > 0.0f)) return -1;
  double z = 0.0;
  for (int t = 0; t < T; ++t) z += std::max((double)u[t], 0.0) + (double)eps;
  for (int t = 0; t < T; ++t)
    m_cur[t] = (float)((std::max((double)u[t], 0.0) + (double)eps) / z);
  return 0;
}

// c <- lambda c + (1-lambda) m_cur ; m_used = normalize(beta m_cur + (1-beta) normalize(c)).
int amso_ema(const float* m_cur, float* credit, int T, float lambda, float beta,
             float* m_used) {
  if (!m_cur || !credit || !m_used || T < 1) return -1;
  if (!(lambda >= 0.0f && lambda < 1.0f) || !(beta >= 0.0f && beta <= 1.0f)) return -1;
  const double lam = (double)lambda, bet = (double)beta;
  if (lambda == 0.0f) {  // credit not used
    for (int t = 0; t < T; ++t) {
      credit[t] = m_cur[t];
      m_used[t] = m_cur[t];
    }
    return 0;
  }
  double csum = 0.0;
  for (int t = 0; t < T; ++t) {
    credit[t] = (float)(lam * (double)credit[t] + (1.0 - lam) * (double)m_cur[t]);
    csum += (double)credit[t];
  }
  std::vector<double> mix((size_t)T);
  double msum = 0.0;
  for (int t = 0; t < T; ++t) {
    const double ctil = csum > 0.0 ? (double)credit[t] / csum : (double)m_cur[t];
    mix[t] = bet * (double)m_cur[t] + (1.0 - bet) * ctil;
    msum += mix[t];
  }
  for (int t = 0; t < T; ++t) m_used[t] = (float)(mix[t] / msum);
  return 0;
}

// Prefix sums, cut points at k/S, segment masses.
int amso_segment(const float* m_used, int T, int S, int32_t* bounds, float* seg_mass) {
  if (!m_used || !bounds || !seg_mass || T < 1 || S < 1) return -1;
  bounds[0] = 0;
  bounds[S] = T;
  int k = 1;
  double c = 0.0;
  for (int t = 0; t < T; ++t) {
    c += (double)m_used[t];
    // one token may carry the curve across several thresholds at once
    while (k < S && c >= (double)k / (double)S) {
      bounds[k] = t + 1;  // the crossing token closes the earlier segment
      ++k;
    }
  }
  for (; k < S; ++k) bounds[k] = T;  // threshold never reached
  for (int i = 0; i < S; ++i) {
    double m = 0.0;
    for (int t = bounds[i]; t < bounds[i + 1]; ++t) m += (double)m_used[t];
    seg_mass[i] = (float)m;
  }
  return 0;
}

// 1-D average pooling of the usage scores (App. A "Mass construction"; Alg. 1 step 1
// "optionally smooth"): window of `kernel` positions centred on t, cut at the ends of
// the sequence (the mean is over the positions that exist).
int amso_pool(const float* u, int T, int kernel, float* out) {
  if (!u || !out || T < 1 || kernel < 1 || kernel % 2 == 0) return -1;
  const int r = kernel / 2;
  for (int t = 0; t < T; ++t) {
    const int lo = std::max(0, t - r), hi = std::min(T - 1, t + r);
    double sum = 0.0;
    for (int j = lo; j <= hi; ++j) sum += (double)u[j];
    out[t] = (float)(sum / (double)(hi - lo + 1));
  }
  return 0;
}

// Alg. 1 step 3 as printed (Sec. 3.3 "Mass-based adaptive segmentation"): cut points at the
// thresholds k*delta (every k >= 1 with k*delta < 1), then one pass over the initial segments,
// left to right: a segment longer than l_max is split into ceil(L / l_max) parts whose lengths
// differ by at most one (the longer parts first); a segment shorter than l_min is merged into
// its left neighbour (the segment produced last), the very first one into its right neighbour
// (it is prepended to the next initial segment before that one is looked at); empty initial
// segments vanish.  l_max == 0 / l_min == 0 switch the respective rule off.
// bounds has cap+1 entries, seg_mass cap; entries past the *n_seg segments are T and 0.
int amso_segment_adaptive(const float* m_used, int T, float delta, int l_min, int l_max, int cap,
                          int32_t* bounds, float* seg_mass, int32_t* n_seg) {
  if (!m_used || !bounds || !seg_mass || !n_seg || T < 1 || cap < 1) return -1;
  if (!(delta > 0.0f) || l_min < 0 || l_max < 0 || (l_max > 0 && l_min > l_max)) return -1;
  // initial cut points
  std::vector<int> cuts;
  cuts.push_back(0);
  {
    int k = 1;
    double c = 0.0;
    for (int t = 0; t < T; ++t) {
      c += (double)m_used[t];
      while ((double)k * (double)delta < 1.0 && c >= (double)k * (double)delta) {
        cuts.push_back(t + 1);  // the crossing token closes the earlier segment
        ++k;
      }
    }
    // thresholds below 1 that the curve never reached close empty segments at the end
    cuts.push_back(T);
  }
  std::vector<int> out;  // ends of the final segments
  int start = 0;         // start of the segment being formed (moves left of an initial start only
                         // for a too-short first segment)
  bool have_left = false;
  for (size_t i = 0; i + 1 < cuts.size(); ++i) {
    const int b = cuts[i + 1];
    const int L = b - start;
    if (L == 0) continue;
    if (l_max > 0 && L > l_max) {
      const int n = (L + l_max - 1) / l_max, base = L / n, extra = L % n;
      int e = start;
      for (int j = 0; j < n; ++j) {
        e += base + (j < extra ? 1 : 0);
        out.push_back(e);
      }
      have_left = true;
      start = b;
    } else if (l_min > 0 && L < l_min) {
      if (have_left) {
        out.back() = b;  // into the left neighbour
        start = b;
      }
      // else: first segment, kept open; the next initial segment starts at `start`
    } else {
      out.push_back(b);
      have_left = true;
      start = b;
    }
  }
  if (start < T) out.push_back(T);  // the whole sequence was one too-short segment
  if ((int)out.size() > cap) return -5;
  *n_seg = (int32_t)out.size();
  bounds[0] = 0;
  for (int i = 0; i < cap; ++i) bounds[i + 1] = i < (int)out.size() ? out[(size_t)i] : T;
  for (int i = 0; i < cap; ++i) {
    double m = 0.0;
    for (int t = bounds[i]; t < bounds[i + 1]; ++t) m += (double)m_used[t];
    seg_mass[i] = (float)m;
  }
  return 0;
}

// Quotas: floor q_min, remainder shared in proportion to segment mass, no
// segment above its length, total exactly min(budget, T).
int amso_quota(const int32_t* bounds, const float* seg_mass, int S, int budget,
               int q_min, int32_t* quota) {
  if (!bounds || !seg_mass || !quota || S < 1 || budget < 0 || q_min < 0) return -1;
  const int T = bounds[S];
  const int64_t bud = std::min<int64_t>(budget, T);
  std::vector<int64_t> len((size_t)S), qlo((size_t)S), room((size_t)S);
  int nonempty = 0;
  for (int i = 0; i < S; ++i) {
    len[i] = bounds[i + 1] - bounds[i];
    if (len[i] < 0) return -1;
    if (len[i] > 0) ++nonempty;
  }
  int64_t floor_q = q_min, need = 0;
  for (int i = 0; i < S; ++i) need += std::min<int64_t>(floor_q, len[i]);
  if (need > bud) floor_q = nonempty > 0 ? bud / nonempty : 0;  // budget too small for q_min each
  int64_t rem = bud;
  std::vector<char> active((size_t)S);
  for (int i = 0; i < S; ++i) {
    qlo[i] = std::min<int64_t>(floor_q, len[i]);
    room[i] = len[i] - qlo[i];
    active[i] = room[i] > 0;
    quota[i] = (int32_t)qlo[i];
    rem -= qlo[i];
  }
  std::vector<double> raw((size_t)S, 0.0);
  // Proportional shares; a segment whose share reaches its room is filled and
  // leaves the pool, and the shares of the others are recomputed.
  for (;;) {
    int n_active = 0;
    double msum = 0.0;
    for (int i = 0; i < S; ++i)
      if (active[i]) {
        ++n_active;
        msum += (double)seg_mass[i];
      }
    if (n_active == 0 || rem <= 0) break;
    bool filled = false;
    for (int i = 0; i < S; ++i)
      if (active[i])
        raw[i] = msum > 0.0 ? (double)rem * (double)seg_mass[i] / msum
                            : (double)rem / (double)n_active;
    int64_t taken = 0;
    for (int i = 0; i < S; ++i)
      if (active[i] && raw[i] >= (double)room[i]) {
        quota[i] = (int32_t)len[i];
        taken += room[i];
        active[i] = 0;
        filled = true;
      }
    rem -= taken;
    if (!filled) break;
  }
  if (rem > 0) {
    // integer parts, then one extra unit each to the largest fractional parts
    std::vector<int> order;
    std::vector<double> frac((size_t)S, 0.0);
    int64_t given = 0;
    for (int i = 0; i < S; ++i)
      if (active[i]) {
        const double fl = std::floor(raw[i]);
        frac[i] = raw[i] - fl;
        quota[i] += (int32_t)fl;
        given += (int64_t)fl;
        order.push_back(i);
      }
    std::stable_sort(order.begin(), order.end(),
                     [&](int a, int b) { return frac[a] > frac[b]; });
    int64_t left = rem - given;
    while (left > 0) {
      bool any = false;
      for (size_t j = 0; j < order.size() && left > 0; ++j) {
        const int i = order[j];
        if (quota[i] < len[i]) {
          ++quota[i];
          --left;
          any = true;
        }
      }
      if (!any) return -3;
    }
  }
  return 0;
}

int amso_select(const float* g, const int32_t* bounds, const int32_t* quota, int S,
                int32_t* idx, int32_t* n_kept) {
  if (!g || !bounds || !quota || !idx || !n_kept || S < 1) return -1;
  int out = 0;
  std::vector<int32_t> pos;
  for (int i = 0; i < S; ++i) {
    const int a = bounds[i], b = bounds[i + 1], q = quota[i];
    if (q < 0 || q > b - a) return -1;
    pos.resize((size_t)(b - a));
    for (int t = a; t < b; ++t) pos[(size_t)(t - a)] = t;
    std::stable_sort(pos.begin(), pos.end(), [&](int32_t x, int32_t y) {
      return sel_value(g[x]) > sel_value(g[y]);
    });
    std::sort(pos.begin(), pos.begin() + q);
    for (int j = 0; j < q; ++j) idx[out++] = pos[(size_t)j];
  }
  *n_kept = out;
  return 0;
}

// Sizes of the must-keep set (Sec. 3.3 "must-keep rules"): sinks come first and are never
// given up, the recent suffix shrinks until both fit into the number of kept tokens, the
// segments share what is left.
int amso_must_keep(int T, int budget, int n_sink, int n_last, int* sink_eff, int* last_eff,
                   int* seg_budget) {
  if (T < 1 || budget < 1 || n_sink < 0 || n_last < 0 || !sink_eff || !last_eff || !seg_budget) return -1;
  const int kept = std::min(budget, T);
  *sink_eff = std::min(n_sink, kept);
  *last_eff = std::min(n_last, kept - *sink_eff);
  *seg_budget = kept - *sink_eff - *last_eff;
  return 0;
}

// Alg. 1 step 5, second half: union of the in-segment picks with the must-keep positions
// (the first sink_eff and the last last_eff of T), duplicates removed, ascending; while the
// set is larger than target the lowest-scoring position outside the must-keep set leaves
// (of equal scores the higher index first); while it is smaller the highest-scoring
// position not yet in it joins (of equal scores the lower index first).
int amso_finalize(const float* g, int T, const int32_t* seg_idx, int n_seg, int sink_eff,
                  int last_eff, int target, int32_t* idx, int32_t* n_kept) {
  if (!g || !idx || !n_kept || T < 1 || n_seg < 0 || (n_seg > 0 && !seg_idx)) return -1;
  if (sink_eff < 0 || last_eff < 0 || sink_eff + last_eff > T || target < sink_eff + last_eff || target > T)
    return -1;
  std::vector<char> in((size_t)T, 0), must((size_t)T, 0);
  for (int t = 0; t < sink_eff; ++t) must[(size_t)t] = 1;
  for (int t = T - last_eff; t < T; ++t) must[(size_t)t] = 1;
  for (int j = 0; j < n_seg; ++j) {
    if (seg_idx[j] < 0 || seg_idx[j] >= T) return -1;
    in[(size_t)seg_idx[j]] = 1;
  }
  int count = 0;
  for (int t = 0; t < T; ++t) {
    if (must[(size_t)t]) in[(size_t)t] = 1;
    count += in[(size_t)t];
  }
  while (count > target) {
    int worst = -1;
    for (int t = 0; t < T; ++t)
      if (in[(size_t)t] && !must[(size_t)t] && (worst < 0 || sel_value(g[t]) <= sel_value(g[worst]))) worst = t;
    if (worst < 0) return -3;
    in[(size_t)worst] = 0;
    --count;
  }
  while (count < target) {
    int best = -1;
    for (int t = 0; t < T; ++t)
      if (!in[(size_t)t] && (best < 0 || sel_value(g[t]) > sel_value(g[best]))) best = t;
    if (best < 0) return -3;
    in[(size_t)best] = 1;
    ++count;
  }
  int out = 0;
  for (int t = 0; t < T; ++t)
    if (in[(size_t)t]) idx[out++] = t;
  *n_kept = out;
  return 0;
}

int amso_compact(const void* K, const void* V, const float* credit, int64_t row_bytes,
                 const int32_t* idx, int n_kept, void* K_out, void* V_out, float* credit_out) {
  if (!idx || n_kept < 0 || row_bytes < 1) return -1;
  for (int j = 0; j < n_kept; ++j) {
    const int64_t src = (int64_t)idx[j] * row_bytes, dst = (int64_t)j * row_bytes;
    if (K && K_out) std::memcpy((char*)K_out + dst, (const char*)K + src, (size_t)row_bytes);
    if (V && V_out) std::memcpy((char*)V_out + dst, (const char*)V + src, (size_t)row_bytes);
    if (credit && credit_out) credit_out[j] = credit[idx[j]];
  }
  return 0;
}

int amso_compact_paged(const void* K_pool, const void* V_pool, const int32_t* src_table,
                       void* K_pool_out, void* V_pool_out, const int32_t* dst_table,
                       int block, int H, int h, int64_t row_bytes,
                       const int32_t* idx, int n_kept) {
  if (!src_table || !dst_table || !idx || block < 1 || H < 1 || h < 0 || h >= H) return -1;
  for (int j = 0; j < n_kept; ++j) {
    const int p = idx[j];
    const int64_t s_src = (int64_t)src_table[p / block] * block + p % block;
    const int64_t s_dst = (int64_t)dst_table[j / block] * block + j % block;
    const int64_t o_src = (s_src * H + h) * row_bytes, o_dst = (s_dst * H + h) * row_bytes;
    if (K_pool && K_pool_out)
      std::memcpy((char*)K_pool_out + o_dst, (const char*)K_pool + o_src, (size_t)row_bytes);
    if (V_pool && V_pool_out)
      std::memcpy((char*)V_pool_out + o_dst, (const char*)V_pool + o_src, (size_t)row_bytes);
  }
  return 0;
}

int amso_compress_unit(const amso_unit_params* p, const float* Q, const float* K, const float* V,
                       const void* K_rows, const void* V_rows, int64_t row_bytes,
                       float* credit,
                       float* u, float* g, float* m_used, int32_t* bounds, float* seg_mass,
                       int32_t* quota, int32_t* idx, int32_t* n_kept,
                       void* K_out, void* V_out, float* credit_out) {
  if (!p || !credit || !idx || !n_kept) return -1;
  const int T = p->T, S = p->S;
  std::vector<float> u_((size_t)T), g_((size_t)T), mc((size_t)T), mu((size_t)T), sm((size_t)S);
  std::vector<int32_t> bd((size_t)S + 1), qt((size_t)S);
  int rc;
  const bool vnorm = p->scorer == AMSO_SCORER_EXPECTED_VNORM, redun = p->scorer == AMSO_SCORER_REDUNDANCY;
  if (vnorm && !V) return -1;
  if ((rc = amso_score(Q, K, p->G, p->W, T, p->D,
                       vnorm ? AMSO_SCORER_EXPECTED : (redun ? AMSO_SCORER_MEAN_WINDOW : p->scorer), p->causal,
                       u_.data(), g_.data())))
    return rc;
  if (redun && (rc = amso_redundancy_score(u_.data(), K, T, p->D, p->mix_lambda, p->score_kernel, g_.data())))
    return rc;
  if (vnorm) {
    std::vector<float> e(g_);
    if ((rc = amso_value_weight(e.data(), V, T, p->D, p->vnorm_eps, g_.data()))) return rc;
  }
  std::vector<float> up;  // smoothed usage feeds the mass only; the base score keeps the raw one
  if (p->pool_kernel > 1) {
    up.resize((size_t)T);
    if ((rc = amso_pool(u_.data(), T, p->pool_kernel, up.data()))) return rc;
  }
  if ((rc = amso_mass(up.empty() ? u_.data() : up.data(), T, p->eps, mc.data()))) return rc;
  if ((rc = amso_ema(mc.data(), credit, T, p->lambda, p->beta, mu.data()))) return rc;
  if (p->delta > 0.0f) {  // S is the capacity of the segment arrays
    int32_t n_seg = 0;
    if ((rc = amso_segment_adaptive(mu.data(), T, p->delta, p->l_min, p->l_max, S, bd.data(), sm.data(), &n_seg)))
      return rc;
  } else if ((rc = amso_segment(mu.data(), T, S, bd.data(), sm.data()))) {
    return rc;
  }
  int sink_eff, last_eff, seg_budget;
  if ((rc = amso_must_keep(T, p->budget, p->n_sink, p->n_last, &sink_eff, &last_eff, &seg_budget))) return rc;
  if ((rc = amso_quota(bd.data(), sm.data(), S, seg_budget, p->q_min, qt.data()))) return rc;
  std::vector<int32_t> seg_idx((size_t)std::max(seg_budget, 1));
  int32_t n_seg = 0;
  if ((rc = amso_select(g_.data(), bd.data(), qt.data(), S, seg_idx.data(), &n_seg))) return rc;
  if ((rc = amso_finalize(g_.data(), T, seg_idx.data(), n_seg, sink_eff, last_eff, std::min(p->budget, T),
                          idx, n_kept)))
    return rc;
  if ((rc = amso_compact(K_rows, V_rows, credit, row_bytes, idx, *n_kept, K_out, V_out, credit_out)))
    return rc;
  if (u) std::memcpy(u, u_.data(), sizeof(float) * (size_t)T);
  if (g) std::memcpy(g, g_.data(), sizeof(float) * (size_t)T);
  if (m_used) std::memcpy(m_used, mu.data(), sizeof(float) * (size_t)T);
  if (bounds) std::memcpy(bounds, bd.data(), sizeof(int32_t) * ((size_t)S + 1));
  if (seg_mass) std::memcpy(seg_mass, sm.data(), sizeof(float) * (size_t)S);
  if (quota) std::memcpy(quota, qt.data(), sizeof(int32_t) * (size_t)S);
  return 0;
}

int amso_compress_many(const amso_unit_params* p, int n_units, int n_threads,
                       const float* Q, int64_t q_stride,
                       const float* K, int64_t k_stride, const float* V,
                       float* credit, int64_t c_stride,
                       float* u, float* g, int32_t* idx, int32_t* n_kept,
                       const void* K_rows, const void* V_rows, int64_t row_bytes,
                       void* K_out, void* V_out, float* credit_out) {
  if (!p || n_units < 1 || !Q || !K || !credit || !idx || !n_kept) return -1;
  const bool gather = K_rows && V_rows && K_out && V_out && row_bytes > 0;
  if (n_threads < 1) n_threads = (int)std::thread::hardware_concurrency();
  if (n_threads < 1) n_threads = 1;
  n_threads = std::min(n_threads, n_units);
  std::atomic<int> next(0), failed(0);
  auto work = [&]() {
    for (;;) {
      const int i = next.fetch_add(1);
      if (i >= n_units) return;
      int32_t* my_idx = idx + (size_t)i * p->budget;
      for (int j = 0; j < p->budget; ++j) my_idx[j] = -1;
      const size_t src_off = (size_t)i * p->T * (size_t)row_bytes;
      const size_t dst_off = (size_t)i * p->budget * (size_t)row_bytes;
      const int rc = amso_compress_unit(
          p, Q + (size_t)i * q_stride, K + (size_t)i * k_stride, V ? V + (size_t)i * k_stride : nullptr,
          gather ? (const char*)K_rows + src_off : nullptr, gather ? (const char*)V_rows + src_off : nullptr,
          gather ? row_bytes : 1, credit + (size_t)i * c_stride,
          u ? u + (size_t)i * p->T : nullptr, g ? g + (size_t)i * p->T : nullptr,
          nullptr, nullptr, nullptr, nullptr, my_idx, n_kept + i,
          gather ? (char*)K_out + dst_off : nullptr, gather ? (char*)V_out + dst_off : nullptr,
          credit_out ? credit_out + (size_t)i * p->budget : nullptr);
      if (rc) failed.store(rc);
    }
  };
  std::vector<std::thread> pool;
  for (int t = 1; t < n_threads; ++t) pool.emplace_back(work);
  work();
  for (auto& th : pool) th.join();
  return failed.load() ? -4 : n_threads;
}

}  // extern "C"
