// Eq. (1) + EMA credit (Sec. 3.2, 3.3; Alg. 1 steps 1-2) and the mass prefix sum with its cut
// points (Sec. 3.3 "Mass-based adaptive segmentation"; Alg. 1 step 3): thresholds k/S for exactly S
// segments, or k*Delta followed by the split / merge pass over the segment lengths.
//
// Two forms.  The stage calls (ams_ema_update, ams_mass_segment) cut every unit into chunks of 4096
// positions and make each (chunk, unit) one workgroup:
//
//   vc_sums_kernel       partial sums of max(u,0)+eps and of the old credit per chunk
//   mass_ema_kernel      m = v/Z, c <- lambda c + (1-lambda) m, m_used
//   chunk_total_kernel   chunk totals of a given m_used
//   segment_scan_kernel  inclusive prefix P(j) and the first j with P(j) >= k/S for every k
//   segment_finalize_kernel  segment masses from the prefix at the cuts
//   resegment_kernel     (Delta mode) split above L_max / merge below L_min, one pass from the left
//   segment_mass_kernel  (Delta mode) segment masses by summing m_used over the final segments
//
// The fused step runs all of it, and the quotas, in one workgroup per unit (unit_mass_kernel below).
//
// Normalisers: Z is the actual sum of max(u,0)+eps.  The credit normaliser sum(c_new) is taken as
// lambda * sum(c_old) + (1 - lambda) and the outer normaliser as 1: both identities hold exactly in
// real arithmetic (sum(m) = 1) and to ~1e-8 in floating point, far inside the fp32 tolerance, and
// they remove two dependent sweeps over T.
//
// Prefix: P(j) = C[chunk] + p_local(j) with C[c] the sequential sum of the chunk totals before c and
// p_local the in-chunk scan; a chunk total IS p_local of the chunk's last position, so
// P(last of chunk c-1) == C[c] bit for bit and the chain of "first position that reaches k/S"
// tests is consistent across chunks.  Everything that feeds a comparison is double.
#include <type_traits>

#include "ams_internal.h"
#include "quota.h"

namespace ams {
namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / 64;
constexpr int kPer = 16;  // consecutive positions per thread
constexpr int kMaxSegments = 1024;
static_assert(kBlock * kPer == kChunk, "one workgroup covers one chunk");

// Sum over the workgroup, same value in every thread, fixed order.
__device__ __forceinline__ double block_sum(double v, double* sm) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  __syncthreads();  // sm may still be read from a previous call
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
  __syncthreads();
  double t = 0.0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) t += sm[w];
  return t;
}

// In-chunk inclusive prefix of the kPer consecutive positions each thread owns, and the chunk
// total (= prefix of the very last position).  The association is fixed by the thread layout.
__device__ __forceinline__ void chunk_scan(const float (&x)[kPer], double (&p)[kPer], double& total,
                                           double* wave_tot, double* bcast) {
  double ts = 0.0;
#pragma unroll
  for (int i = 0; i < kPer; ++i) ts += (double)x[i];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  double incl = ts;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const double v = __shfl_up(incl, o);
    if (lane >= o) incl += v;
  }
  __syncthreads();
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  double off = 0.0;
  for (int w = 0; w < wave; ++w) off += wave_tot[w];
  double run = off + (incl - ts);
#pragma unroll
  for (int i = 0; i < kPer; ++i) {
    run += (double)x[i];
    p[i] = run;
  }
  if (threadIdx.x == kBlock - 1) *bcast = run;
  __syncthreads();
  total = *bcast;
}

// Sum of p[0..n) in index order (bit-reproducible), same value in every thread of the workgroup.
// One wave fetches 64 entries at a time in parallel and adds them up through lane broadcasts, so
// the cost is one memory latency per 64 entries instead of one per entry.
__device__ __forceinline__ double2 ordered_sum2(const double2* p, int n, double2* sm) {
  if (threadIdx.x < 64) {
    double2 acc = make_double2(0.0, 0.0);
    for (int base = 0; base < n; base += 64) {
      const int k = min(64, n - base);
      double2 v = make_double2(0.0, 0.0);
      if ((int)threadIdx.x < k) v = p[base + threadIdx.x];
      for (int j = 0; j < k; ++j) {
        acc.x += __shfl(v.x, j);
        acc.y += __shfl(v.y, j);
      }
    }
    if (threadIdx.x == 0) *sm = acc;
  }
  __syncthreads();
  return *sm;
}
__device__ __forceinline__ double ordered_sum(const double* p, int n, double2* sm) {
  if (threadIdx.x < 64) {
    double acc = 0.0;
    for (int base = 0; base < n; base += 64) {
      const int k = min(64, n - base);
      double v = 0.0;
      if ((int)threadIdx.x < k) v = p[base + threadIdx.x];
      for (int j = 0; j < k; ++j) acc += __shfl(v, j);
    }
    if (threadIdx.x == 0) sm->x = acc;
  }
  __syncthreads();
  return sm->x;
}

// kPer consecutive fp32 of a row: 16-byte accesses when the row allows it.
template <int N>
__device__ __forceinline__ void load_run(const float* row, int j0, int T, bool vec, float (&x)[N], float fill) {
  if (vec && j0 + N <= T) {
#pragma unroll
    for (int q = 0; q < N / 4; ++q) {
      const float4 v = *reinterpret_cast<const float4*>(row + j0 + 4 * q);
      x[4 * q] = v.x; x[4 * q + 1] = v.y; x[4 * q + 2] = v.z; x[4 * q + 3] = v.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < N; ++i) x[i] = (j0 + i < T) ? row[j0 + i] : fill;
  }
}
template <int N>
__device__ __forceinline__ void store_run(float* row, int j0, int T, bool vec, const float (&x)[N]) {
  if (vec && j0 + N <= T) {
#pragma unroll
    for (int q = 0; q < N / 4; ++q)
      *reinterpret_cast<float4*>(row + j0 + 4 * q) = make_float4(x[4 * q], x[4 * q + 1], x[4 * q + 2], x[4 * q + 3]);
  } else {
#pragma unroll
    for (int i = 0; i < N; ++i)
      if (j0 + i < T) row[j0 + i] = x[i];
  }
}

struct MsArgs {
  Dims d;
  const int32_t* seq_lens;
  int n_chunks;      // chunks per unit (stride of the per-chunk arrays)
  int S;             // entries of the per-unit segment arrays
  int K;             // initial segments: thresholds k = 1..K-1 (K == S unless delta > 0)
  double delta;      // > 0: thresholds k*delta; 0: thresholds k/S
  int l_min, l_max;  // delta > 0 only: length rules of the split / merge pass (0 = off)
  int pool_r;        // radius of the average pooling of u before Eq. (1) (0 = off)
  double2* vc_part;  // [units][vc_stride] (sum of max(u,0)+eps, sum of old credit) per vc_tokens positions
  int vc_stride, vc_tokens;
  double* mpart;     // [units][n_chunks]  chunk totals of m_used
  double* cpre;      // [units][S+1]       prefix at the cuts (negative = threshold never reached)
  int32_t* bounds;   // [units][S+1]
  bool vec;          // rows of the fp32 vectors are 16-byte aligned
};

__device__ __forceinline__ void init_cuts(const MsArgs& a, int unit, int T) {
  int32_t* bounds = a.bounds + (int64_t)unit * (a.S + 1);
  double* cpre = a.cpre + (int64_t)unit * (a.S + 1);
  for (int k = threadIdx.x; k <= a.S; k += kBlock) {
    bounds[k] = (k == 0) ? 0 : T;
    cpre[k] = (k == 0) ? 0.0 : -1.0;
  }
}

// Usage as Eq. (1) sees it: with pooling (App. A; Alg. 1 step 1 "optionally smooth") the mean of u
// over the positions t-r .. t+r that exist, rounded to fp32 like a stored intermediate.  The chunk's
// scores and r more on either side are staged in LDS once; every thread then reads its windows there.
constexpr int kMaxPoolR = 31;
__device__ __forceinline__ void pool_run(const float* u, int chunk0, int j0, int T, int r, float* tile,
                                         float* pooled, float (&x)[kPer]) {
  const int first = chunk0 - r;  // position of tile[0]
  for (int e = threadIdx.x; e < kChunk + 2 * r; e += kBlock) {
    const int t = first + e;
    tile[e] = (t >= 0 && t < T) ? u[t] : 0.f;
  }
  __syncthreads();
  // consecutive threads take consecutive positions here (no bank conflicts); the runs of kPer
  // positions each thread owns afterwards are read back from the pooled copy
  const double inv_full = 1.0 / (double)(2 * r + 1);
  for (int e = threadIdx.x; e < kChunk; e += kBlock) {
    const int t = chunk0 + e;
    if (t < T) {
      const int lo = max(0, t - r), hi = min(T - 1, t + r);
      double sum = 0.0;
      for (int j = lo; j <= hi; ++j) sum += (double)tile[j - first];
      const int n = hi - lo + 1;
      pooled[e] = (float)(n == 2 * r + 1 ? sum * inv_full : sum / (double)n);
    }
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kPer; ++i)
    if (j0 + i < T) x[i] = pooled[j0 - chunk0 + i];
}

__global__ __launch_bounds__(kBlock) void vc_sums_kernel(MsArgs a, const float* u_all, const float* credit_all,
                                                          float eps_f) {
  __shared__ double sm[kWaves];
  __shared__ float tile[kChunk + 2 * kMaxPoolR], pooled[kChunk];
  const int unit = blockIdx.y, chunk = blockIdx.x;
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T = seq_len(a.d, a.seq_lens, b);
  const int j0 = chunk * kChunk + threadIdx.x * kPer;
  if (chunk * kChunk >= T) return;
  const float* u = u_all + (int64_t)unit * a.d.t_stride;
  const float* credit = credit_all + (int64_t)unit * a.d.t_stride;
  double v = 0.0, c = 0.0;
  float ux[kPer], cx[kPer];
  load_run(u, j0, T, a.vec, ux, 0.f);
  load_run(credit, j0, T, a.vec, cx, 0.f);
  if (a.pool_r > 0) pool_run(u, chunk * kChunk, j0, T, a.pool_r, tile, pooled, ux);
#pragma unroll
  for (int i = 0; i < kPer; ++i)
    if (j0 + i < T) {
      v += fmax((double)ux[i], 0.0) + (double)eps_f;
      c += (double)cx[i];
    }
  v = block_sum(v, sm);
  c = block_sum(c, sm);
  if (threadIdx.x == 0) a.vc_part[(int64_t)unit * a.vc_stride + chunk] = make_double2(v, c);
}

__global__ __launch_bounds__(kBlock) void mass_ema_kernel(MsArgs a, const float* u_all, float* credit_all,
                                                           float* m_used_all, float lambda, float beta,
                                                           float eps_f) {
  __shared__ float tile[kChunk + 2 * kMaxPoolR], pooled[kChunk];
  const int unit = blockIdx.y, chunk = blockIdx.x;
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T = seq_len(a.d, a.seq_lens, b);
  if (chunk * kChunk >= T) return;
  __shared__ double2 sums;
  const float* u = u_all + (int64_t)unit * a.d.t_stride;
  float* credit = credit_all + (int64_t)unit * a.d.t_stride;
  float* m_used = m_used_all + (int64_t)unit * a.d.t_stride;
  const int j0 = chunk * kChunk + threadIdx.x * kPer;
  float mu[kPer], ux[kPer], cx[kPer];
  load_run(u, j0, T, a.vec, ux, 0.f);  // in flight while the normalisers are summed
  load_run(credit, j0, T, a.vec, cx, 0.f);
  if (a.pool_r > 0) pool_run(u, chunk * kChunk, j0, T, a.pool_r, tile, pooled, ux);
  const int nvc = (T + a.vc_tokens - 1) / a.vc_tokens;
  const double2 zc = ordered_sum2(a.vc_part + (int64_t)unit * a.vc_stride, nvc, &sums);
  const double Z = zc.x, c_old = zc.y;
  const double lam = (double)lambda, bet = (double)beta, eps = (double)eps_f;
  const double inv_z = 1.0 / Z, inv_csum = 1.0 / (lam * c_old + (1.0 - lam));
#pragma unroll
  for (int i = 0; i < kPer; ++i) {
    mu[i] = 0.f;
    if (j0 + i < T) {
      const float mc = (float)((fmax((double)ux[i], 0.0) + eps) * inv_z);
      float cn = mc;
      mu[i] = mc;  // lambda == 0: credit not used, the mass passes through unchanged
      if (lambda != 0.f) {
        cn = (float)(lam * (double)cx[i] + (1.0 - lam) * (double)mc);
        mu[i] = (float)(bet * (double)mc + (1.0 - bet) * ((double)cn * inv_csum));
      }
      cx[i] = cn;
    }
  }
  store_run(credit, j0, T, a.vec, cx);
  store_run(m_used, j0, T, a.vec, mu);
}

__global__ __launch_bounds__(kBlock) void chunk_total_kernel(MsArgs a, const float* m_all) {
  __shared__ double wave_tot[kWaves];
  __shared__ double bcast;
  const int unit = blockIdx.y, chunk = blockIdx.x;
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T = seq_len(a.d, a.seq_lens, b);
  if (chunk * kChunk >= T) return;
  if (chunk == 0) init_cuts(a, unit, T);
  const float* m = m_all + (int64_t)unit * a.d.t_stride;
  const int j0 = chunk * kChunk + threadIdx.x * kPer;
  float x[kPer];
  load_run(m, j0, T, a.vec, x, 0.f);
  double p[kPer], total;
  chunk_scan(x, p, total, wave_tot, &bcast);
  if (threadIdx.x == 0) a.mpart[(int64_t)unit * a.n_chunks + chunk] = total;
}

// Number of thresholds thr[k], k = 1..S-1, that are <= c.  thr[k] holds (double)k / (double)S (or
// (double)k * delta), the exact value the comparison is defined with; the table keeps divisions out
// of the per-thread path.  scale (S or 1/delta) only gives the first guess.
__device__ __forceinline__ int thresholds_reached(double c, int S, const double* thr, double scale) {
  int f = (int)floor(c * scale);
  f = max(0, min(S - 1, f));
  while (f < S - 1 && c >= thr[f + 1]) ++f;
  while (f > 0 && c < thr[f]) --f;
  return f;
}

__global__ __launch_bounds__(kBlock) void segment_scan_kernel(MsArgs a, const float* m_all) {
  __shared__ double wave_tot[kWaves];
  __shared__ double bcast;
  __shared__ double ends[kBlock];
  __shared__ double thr[kMaxSegments + 1];
  const int unit = blockIdx.y, chunk = blockIdx.x;
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T = seq_len(a.d, a.seq_lens, b);
  if (chunk * kChunk >= T) return;
  const float* m = m_all + (int64_t)unit * a.d.t_stride;
  __shared__ double2 sums;
  const int K = a.K;
  const double scale = a.delta > 0.0 ? 1.0 / a.delta : (double)a.S;
  for (int k = threadIdx.x; k <= K; k += kBlock) thr[k] = a.delta > 0.0 ? (double)k * a.delta : (double)k / (double)a.S;
  const int j0 = chunk * kChunk + threadIdx.x * kPer;
  float x[kPer];
  load_run(m, j0, T, a.vec, x, 0.f);
  const double C = ordered_sum(a.mpart + (int64_t)unit * a.n_chunks, chunk, &sums);  // prefix before this chunk
  double p[kPer], total;
  chunk_scan(x, p, total, wave_tot, &bcast);
  ends[threadIdx.x] = C + p[kPer - 1];
  __syncthreads();
  const double prev_end = threadIdx.x > 0 ? ends[threadIdx.x - 1] : C;
  int f_prev = thresholds_reached(prev_end, K, thr, scale);
  int32_t* bounds = a.bounds + (int64_t)unit * (a.S + 1);
  double* cpre = a.cpre + (int64_t)unit * (a.S + 1);
  // most threads see no threshold between their neighbour's prefix and their own largest one
  double p_max = p[0];
#pragma unroll
  for (int i = 1; i < kPer; ++i) p_max = fmax(p_max, p[i]);
  if (thresholds_reached(C + p_max, K, thr, scale) <= f_prev) return;
#pragma unroll
  for (int i = 0; i < kPer; ++i) {
    if (j0 + i < T) {
      const double P = C + p[i];
      const int f_cur = thresholds_reached(P, K, thr, scale);
      for (int k = f_prev + 1; k <= f_cur; ++k) {  // position j0+i is the first to reach k/S
        atomicMin(&bounds[k], j0 + i + 1);
        cpre[k] = P;
      }
      f_prev = max(f_prev, f_cur);
    }
  }
}

__global__ void segment_finalize_kernel(MsArgs a, float* seg_mass_all) {
  const int unit = blockIdx.x;
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T = seq_len(a.d, a.seq_lens, b);
  const int nch = (T + kChunk - 1) / kChunk;
  double total = 0.0;
  for (int c = 0; c < nch; ++c) total += a.mpart[(int64_t)unit * a.n_chunks + c];
  const double* cpre = a.cpre + (int64_t)unit * (a.S + 1);
  for (int i = threadIdx.x; i < a.S; i += blockDim.x) {
    const double lo = cpre[i] < 0.0 ? total : cpre[i];
    const double hi = (i + 1 == a.S || cpre[i + 1] < 0.0) ? total : cpre[i + 1];
    seg_mass_all[(int64_t)unit * a.S + i] = (float)(hi - lo);
  }
}

// Split / merge pass over the initial segments, one pass from the left (Alg. 1 step 3, the loop over segments;
// Sec. 3.3 "Mass-based adaptive segmentation").  cut(i), i = 1 .. K, is the end of initial segment i (cut(K) = T).
// A segment longer than l_max becomes ceil(L / l_max) parts whose lengths differ by at most one, the longer ones
// first; one shorter than l_min joins the segment to its left, the very first one stays open so that the next
// initial segment starts where it started; empty initial segments vanish.  Writes the ends of the final segments
// to out[0 .. n) (at most cap of them) and returns n.  A serial chain of at most K steps: one thread runs it.
template <typename Cut>
__device__ __forceinline__ int split_merge_pass(Cut cut, int K, int T, int l_min, int l_max, int cap, int32_t* out) {
  int n = 0, start = 0;
  bool have_left = false;
  for (int i = 1; i <= K; ++i) {
    const int e = cut(i);
    const int L = e - start;
    if (L == 0) continue;
    if (l_max > 0 && L > l_max) {
      const int parts = (L + l_max - 1) / l_max, base = L / parts, extra = L % parts;
      int pos = start;
      for (int j = 0; j < parts && n < cap; ++j) {
        pos += base + (j < extra ? 1 : 0);
        out[n++] = pos;
      }
      have_left = true;
      start = e;
    } else if (l_min > 0 && L < l_min) {
      if (have_left) {
        out[n - 1] = e;
        start = e;
      }
    } else {
      if (n < cap) out[n++] = e;
      have_left = true;
      start = e;
    }
  }
  if (start < T && n < cap) out[n++] = T;  // the whole sequence was one too-short segment
  if (n > 0) out[n - 1] = T;               // (only matters if the capacity cut the list short)
  return n;
}

// Delta mode, after the cut points: one pass over the initial segments from the left (Alg. 1 step 3,
// the loop over segments).  Longer than l_max: ceil(L / l_max) parts whose lengths differ by at most
// one, the longer ones first.  Shorter than l_min: joins the segment to its left; the first one
// stays open and the next initial segment starts where it started.  Empty initial segments vanish.
// The pass is a short serial chain (at most K steps) and runs on one lane per unit; the new bounds
// are staged in LDS because they overwrite the old ones.
__global__ __launch_bounds__(64) void resegment_kernel(MsArgs a) {
  __shared__ int32_t out[kMaxSegments + 1];
  __shared__ int n_out;
  const int unit = blockIdx.x;
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T = seq_len(a.d, a.seq_lens, b);
  int32_t* bounds = a.bounds + (int64_t)unit * (a.S + 1);
  if (threadIdx.x == 0) {
    const int K = a.K;
    const int n = split_merge_pass([&](int i) { return i == K ? T : bounds[i]; }, K, T, a.l_min, a.l_max, a.S, out);
    n_out = n;
  }
  __syncthreads();
  const int n = n_out;
  for (int i = threadIdx.x; i < a.S; i += 64) bounds[i + 1] = i < n ? out[i] : T;
}

// Mass of every final segment: one wave per (segment, unit), strided partial sums in double, then
// a fixed tree over the lanes.
__global__ __launch_bounds__(64) void segment_mass_kernel(MsArgs a, const float* m_all, float* seg_mass_all) {
  const int unit = blockIdx.y, seg = blockIdx.x;
  const int32_t* bounds = a.bounds + (int64_t)unit * (a.S + 1);
  const int lo = bounds[seg], hi = bounds[seg + 1];
  const float* m = m_all + (int64_t)unit * a.d.t_stride;
  double s = 0.0;
  for (int t = lo + threadIdx.x; t < hi; t += 64) s += (double)m[t];
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o);
  if (threadIdx.x == 0) seg_mass_all[(int64_t)unit * a.S + seg] = (float)s;
}

// Eq. (1), the EMA, the prefix sum with its cuts, the segment masses and the quotas of one unit in ONE
// workgroup of 1024 threads.  The unit is walked in groups of 1024*PER positions; inside a group thread
// i owns the PER consecutive positions from i*PER on, so the running prefix is a serial sum per thread,
// a scan over the lanes, an ordered sum over the 16 waves and the total of the groups before -- no
// chunk totals through memory, no second read of m_used, and the launches of the chunked kernels above
// become one.  The next group's usage and credit are requested before the current group is worked on.
// The arithmetic per position, the thresholds, the split / merge pass and the quotas are those of the
// kernels above.
//   GENERAL = false: thresholds k/S, at most 64 segments, no pooling (the headline configuration).
//   GENERAL = true:  also thresholds k*Delta with the split / merge pass, pooled usage, up to 1024
//                    segments; needs more LDS (the pooling tile, the quota scratch).
constexpr int kUnitBlock = 1024;
constexpr int kUnitMaxSeg = 64;

// Pooled usage of the whole unit (see pool_run), group by group: the group's scores and r more on either
// side are staged in LDS, consecutive threads then pool consecutive positions (no bank conflicts), store the
// result (rounded to fp32 like a stored intermediate) to out[] and add max(pooled, 0) + eps to v and the
// position's old credit to c.  The next group's scores are requested before the current group is pooled.
template <int GROUP>
__device__ __forceinline__ void pool_unit(const float* u, const float* credit, float* out, int T, int r,
                                          float* tile, double eps, double& v, double& c) {
  constexpr int kStage = (GROUP + 2 * kMaxPoolR + kUnitBlock - 1) / kUnitBlock;
  const int n_groups = (T + GROUP - 1) / GROUP;
  const double inv_full = 1.0 / (double)(2 * r + 1);
  float stage[kStage];
  auto fetch = [&](int g0) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < kStage; ++q) {
      const int e = q * kUnitBlock + (int)threadIdx.x, t = g0 - r + e;
      stage[q] = (e < GROUP + 2 * r && t >= 0 && t < T) ? u[t] : 0.f;
    }
  };
  fetch(0);
#pragma unroll 1
  for (int g = 0; g < n_groups; ++g) {
    const int g0 = g * GROUP, first = g0 - r;  // first = position of tile[0]
#pragma unroll
    for (int q = 0; q < kStage; ++q) {
      const int e = q * kUnitBlock + (int)threadIdx.x;
      if (e < GROUP + 2 * r) tile[e] = stage[q];
    }
    __syncthreads();
    if (g + 1 < n_groups) fetch(g0 + GROUP);
    for (int e = threadIdx.x; e < GROUP; e += kUnitBlock) {
      const int t = g0 + e;
      if (t < T) {
        const float cr = credit[t];
        const int lo = max(0, t - r), hi = min(T - 1, t + r);
        double sum = 0.0;
        for (int j = lo; j <= hi; ++j) sum += (double)tile[j - first];
        const int n = hi - lo + 1;
        const float p = (float)(n == 2 * r + 1 ? sum * inv_full : sum / (double)n);
        out[t] = p;
        v += fmax((double)p, 0.0) + eps;
        c += (double)cr;
      }
    }
    __syncthreads();
  }
}

template <int PER, bool GENERAL>
__global__ __launch_bounds__(kUnitBlock) void unit_mass_kernel(MsArgs a, const float* u_all, float* credit_all,
                                                                float* m_used_all, float lambda, float beta,
                                                                float eps_f, int budget, int q_min,
                                                                float* seg_mass_all, int32_t* quota_all,
                                                                int32_t* idx_all, int32_t* n_kept_all, int n_sink,
                                                                int n_last, uint32_t* flags_all, int n_words,
                                                                const int32_t* status) {
  constexpr int kW = kUnitBlock / 64, kGroup = kUnitBlock * PER;
  constexpr int kCap = GENERAL ? kMaxSegments : kUnitMaxSeg;
  __shared__ double wave_tot[2][kW];
  __shared__ double ends[2][kUnitBlock];
  __shared__ double thr[kCap + 1], cpre[kCap + 1];
  __shared__ int32_t bounds[kCap + 1];
  __shared__ float mass[kCap];
  __shared__ double2 sums;
  __shared__ float tile[GENERAL ? kGroup + 2 * kMaxPoolR : 1];
  __shared__ int32_t reseg[GENERAL ? kCap + 1 : 1];
  __shared__ int n_reseg;
  // Delta mode on caches of up to kEndGroups groups: the prefix at the end of every thread's run, from which
  // the mass of a segment that the split / merge pass has moved follows without another sum over its positions
  constexpr int kEndGroups = 4;
  __shared__ double ends_all[GENERAL ? kEndGroups * kUnitBlock : 1];
  __shared__ typename std::conditional<GENERAL, QuotaScratch, int>::type qs;
  const int unit = blockIdx.x, S = a.S;
  const int K = GENERAL ? a.K : S;  // initial segments: thresholds k = 1 .. K-1
  const bool delta_mode = GENERAL && a.delta > 0.0;
  const int pool_r = GENERAL ? a.pool_r : 0;
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T = seq_len(a.d, a.seq_lens, b);
  const float* u = u_all + (int64_t)unit * a.d.t_stride;
  float* credit = credit_all + (int64_t)unit * a.d.t_stride;
  float* m_used = m_used_all + (int64_t)unit * a.d.t_stride;
  const int n_groups = (T + kGroup - 1) / kGroup;
  // with pooling, the pooled usage passes through the m_used row: written while the normalisers are summed,
  // read back (and overwritten by m_used proper) in the main walk
  const float* u_src = pool_r > 0 ? m_used : u;
  float ux[PER], cx[PER];
  if (pool_r == 0) load_run(u, (int)threadIdx.x * PER, T, a.vec, ux, 0.f);  // in flight while the normalisers are summed
  load_run(credit, (int)threadIdx.x * PER, T, a.vec, cx, 0.f);
  for (int k = threadIdx.x; k <= S; k += kUnitBlock) {
    bounds[k] = (k == 0) ? 0 : T;
    cpre[k] = (k == 0) ? 0.0 : -1.0;
  }
  for (int k = threadIdx.x; k <= K; k += kUnitBlock) thr[k] = delta_mode ? (double)k * a.delta : (double)k / (double)S;
  const double lam = (double)lambda, bet = (double)beta, eps = (double)eps_f;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  double2 zc;
  if (a.vc_part && pool_r == 0) {  // the scorer left the sums of max(u,0)+eps and of the old credit per chunk
    const int nvc = (T + a.vc_tokens - 1) / a.vc_tokens;
    zc = ordered_sum2(a.vc_part + (int64_t)unit * a.vc_stride, nvc, &sums);
  } else {
    // no usable sums from the scorer (causal window, pooled usage): one more walk over the unit, every
    // thread its positions in order, then the lanes and the waves in a fixed order
    double v = 0.0, c = 0.0;
    if (pool_r > 0) {
      if constexpr (GENERAL) {
        pool_unit<kGroup>(u, credit, m_used, T, pool_r, tile, eps, v, c);
      }
    } else {
      for (int j = threadIdx.x * 4; j < T; j += kUnitBlock * 4) {
        float ur[4], cr[4];
        load_run(u, j, T, a.vec, ur, 0.f);
        load_run(credit, j, T, a.vec, cr, 0.f);
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (j + i < T) {
            v += fmax((double)ur[i], 0.0) + eps;
            c += (double)cr[i];
          }
      }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      v += __shfl_xor(v, o);
      c += __shfl_xor(c, o);
    }
    if (lane == 0) ends[0][wave] = v, ends[1][wave] = c;
    __syncthreads();
    zc = make_double2(0.0, 0.0);
    for (int w = 0; w < kW; ++w) {
      zc.x += ends[0][w];
      zc.y += ends[1][w];
    }
    __syncthreads();  // ends is used again below
  }
  if (pool_r > 0) load_run(u_src, (int)threadIdx.x * PER, T, a.vec, ux, 0.f);
  const double Z = zc.x, c_old = zc.y;
  const double inv_z = 1.0 / Z, inv_csum = 1.0 / (lam * c_old + (1.0 - lam));
  const double scale = delta_mode ? 1.0 / a.delta : (double)S;
  double C = 0.0;  // prefix at the end of the groups before
#pragma unroll 1
  for (int r = 0; r < n_groups; ++r) {
    const int j0 = r * kGroup + (int)threadIdx.x * PER, par = r & 1;
    float un[PER], cn_next[PER];
    if (r + 1 < n_groups) {
      load_run(u_src, j0 + kGroup, T, a.vec, un, 0.f);
      load_run(credit, j0 + kGroup, T, a.vec, cn_next, 0.f);
    }
    float mu[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      mu[i] = 0.f;
      if (j0 + i < T) {
        const float mc = (float)((fmax((double)ux[i], 0.0) + eps) * inv_z);
        float cn = mc;
        mu[i] = mc;  // lambda == 0: credit not used, the mass passes through unchanged
        if (lambda != 0.f) {
          cn = (float)(lam * (double)cx[i] + (1.0 - lam) * (double)mc);
          mu[i] = (float)(bet * (double)mc + (1.0 - bet) * ((double)cn * inv_csum));
        }
        cx[i] = cn;
      }
    }
    store_run(credit, j0, T, a.vec, cx);
    store_run(m_used, j0, T, a.vec, mu);
    // inclusive prefix: serial over the thread's run, scan over the lanes, ordered sum over the waves
    double ts = 0.0;
#pragma unroll
    for (int i = 0; i < PER; ++i) ts += (double)mu[i];
    double incl = ts;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const double v = __shfl_up(incl, o);
      if (lane >= o) incl += v;
    }
    if (lane == 63) wave_tot[par][wave] = incl;
    __syncthreads();
    double off = C;
    for (int w = 0; w < wave; ++w) off += wave_tot[par][w];
    const double start = off + (incl - ts);  // prefix of the position in front of this thread's run
    double run = start;
#pragma unroll
    for (int i = 0; i < PER; ++i) run += (double)mu[i];
    ends[par][threadIdx.x] = run;
    if constexpr (GENERAL)
      if (delta_mode && n_groups <= kEndGroups) ends_all[r * kUnitBlock + threadIdx.x] = run;
    __syncthreads();
    const double prev_end = threadIdx.x > 0 ? ends[par][threadIdx.x - 1] : C;
    C = ends[par][kUnitBlock - 1];
    int f_prev = thresholds_reached(prev_end, K, thr, scale);
    // most threads see no threshold between their neighbour's prefix and their own last one (the masses
    // are not negative, so the prefix does not fall)
    if (thresholds_reached(run, K, thr, scale) > f_prev) {
      // the walk repeats the additions that gave `run`, so its last value IS the published end of this
      // run: every threshold in (neighbour's end, run] is met by exactly one position of this thread
      double P = start;
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        P += (double)mu[i];
        if (j0 + i < T) {
          const int f_cur = thresholds_reached(P, K, thr, scale);
          for (int k = f_prev + 1; k <= f_cur; ++k) {  // position j0+i is the first to reach threshold k
            atomicMin(&bounds[k], j0 + i + 1);
            cpre[k] = P;
          }
          f_prev = max(f_prev, f_cur);
        }
      }
    }
    if (r + 1 < n_groups) {
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        ux[i] = un[i];
        cx[i] = cn_next[i];
      }
    }
  }
  __syncthreads();
  const double total = C;
  if constexpr (GENERAL) {
    if (delta_mode) {
      // the split / merge pass over the initial segments (see resegment_kernel), then the mass of every
      // final segment summed from the m_used this workgroup has just written
      if (threadIdx.x == 0) {
        const int n = split_merge_pass([&](int i) { return i == K ? T : bounds[i]; }, K, T, a.l_min, a.l_max, S, reseg);
        n_reseg = n;
      }
      __syncthreads();
      const int n = n_reseg;
      for (int i = threadIdx.x; i < S; i += kUnitBlock) bounds[i + 1] = i < n ? reseg[i] : T;
      __syncthreads();
      if (n_groups <= kEndGroups) {
        // prefix in front of every bound: the end of the run before the one the bound lies in, plus the
        // positions of that run in front of it (the scan's own order of additions)
        for (int i = threadIdx.x; i <= S; i += kUnitBlock) {
          const int bnd = bounds[i];
          double P = 0.0;
          if (bnd > 0) {
            const int q = (bnd - 1) / PER;  // run of the last position in front of the bound
            if (q > 0) P = ends_all[q - 1];
            for (int t = q * PER; t < bnd; ++t) P += (double)m_used[t];
          }
          cpre[i] = P;
        }
        __syncthreads();
        for (int i = threadIdx.x; i < S; i += kUnitBlock) mass[i] = (float)(cpre[i + 1] - cpre[i]);
      } else {
        for (int sg = wave; sg < S; sg += kW) {
          const int lo = bounds[sg], hi = bounds[sg + 1];
          double sm = 0.0;
          for (int t = lo + lane; t < hi; t += 64) sm += (double)m_used[t];
#pragma unroll
          for (int o = 32; o >= 1; o >>= 1) sm += __shfl_xor(sm, o);
          if (lane == 0) mass[sg] = (float)sm;
        }
      }
      __syncthreads();
    }
  }
  if (!delta_mode) {
    for (int i = threadIdx.x; i < S; i += kUnitBlock) {
      const double lo = cpre[i] < 0.0 ? total : cpre[i];
      const double hi = (i + 1 == S || cpre[i + 1] < 0.0) ? total : cpre[i + 1];
      mass[i] = (float)(hi - lo);
    }
    __syncthreads();
  }
  for (int i = threadIdx.x; i < S; i += kUnitBlock) seg_mass_all[(int64_t)unit * S + i] = mass[i];
  for (int i = threadIdx.x; i <= S; i += kUnitBlock) a.bounds[(int64_t)unit * (S + 1) + i] = bounds[i];
  // what the quota kernels do besides the quotas: the -1 tail of idx, the kept count, the cleared bitmap
  // of the must-keep path; sinks and the recent suffix come out of the budget first
  const int kept = min(budget, T);
  const int sinks = min(n_sink, kept);
  const int bud = kept - sinks - min(n_last, kept - sinks);
  int32_t* idx = idx_all + (int64_t)unit * budget;
  for (int j = kept + threadIdx.x; j < budget; j += kUnitBlock) idx[j] = -1;
  // a scorer whose bounded wait expired left unfinished scores: no unit reports a kept set then
  if (threadIdx.x == 0) n_kept_all[unit] = (status && *status != 0) ? -1 : kept;
  if (flags_all)
    for (int j = threadIdx.x; j < n_words; j += kUnitBlock) flags_all[(int64_t)unit * n_words + j] = 0u;
  if (S <= kUnitMaxSeg) {
    if (threadIdx.x < 64) {
      const int q = quota_wave(S, bud, q_min, bounds, mass);
      if ((int)threadIdx.x < S) quota_all[(int64_t)unit * S + threadIdx.x] = q;
    }
  } else {
    if constexpr (GENERAL) {
      if (threadIdx.x < 64) {  // one wave, no workgroup barriers
        quota_block<64>(S, bud, q_min, bounds, mass, qs);
        for (int i = threadIdx.x; i < S; i += 64) quota_all[(int64_t)unit * S + i] = qs.quo[i];
      }
    }
  }
}

MsArgs make_args(const ams_params* p, const Dims& d, const int32_t* seq_lens, char* ws, const WsLayout& wl,
                 int32_t* bounds) {
  MsArgs a;
  a.d = d;
  a.seq_lens = seq_lens;
  a.n_chunks = wl.n_chunks4k;
  a.S = p->n_segments;
  a.delta = (double)p->seg_delta;
  a.K = p->seg_delta > 0.f ? initial_segments(p->seg_delta) : p->n_segments;
  a.l_min = p->l_min;
  a.l_max = p->l_max;
  a.pool_r = p->pool_kernel > 1 ? p->pool_kernel / 2 : 0;
  a.vc_part = (double2*)(ws + wl.vc_part);
  a.vc_stride = wl.n_chunks4k;
  a.vc_tokens = kChunk;
  a.mpart = (double*)(ws + wl.mpart);
  a.cpre = (double*)(ws + wl.cpre);
  a.bounds = bounds;
  a.vec = false;  // set by the launchers once the pointers are known
  return a;
}

// Scratch of ams_mass_segment_static: device memory that belongs to the library and lives as long as the
// process, one copy per GPU.  In host code the array's name is only a handle; the address that kernels and
// copies may use comes from hipGetSymbolAddress, once per device, with that device current.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

}  // namespace

hipError_t static_scratch(char** out) {
  constexpr int kMaxDevices = 64;
  static char* ptr[kMaxDevices] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (!ptr[dev]) {
    void* p = nullptr;
    if ((e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) != hipSuccess) return e;
    ptr[dev] = (char*)p;
  }
  *out = ptr[dev];
  return hipSuccess;
}

hipError_t launch_ema(const ams_params* p, const Dims& d, const int32_t* seq_lens, const float* u,
                      float* credit, float* m_used, const VcInfo& vc, char* ws, const WsLayout& wl,
                      hipStream_t s) {
  MsArgs a = make_args(p, d, seq_lens, ws, wl, nullptr);
  a.vec = d.t_stride % 4 == 0 && (((uintptr_t)u | (uintptr_t)credit | (uintptr_t)m_used) & 15) == 0;
  const dim3 grid(a.n_chunks, d.units);
  if (vc.have && a.pool_r == 0) {  // left by the scorer (sums of the unsmoothed usage)
    a.vc_stride = vc.stride;
    a.vc_tokens = vc.tokens;
  } else {
    prof_mark("vc_sums", s);
    hipLaunchKernelGGL(vc_sums_kernel, grid, dim3(kBlock), 0, s, a, u, (const float*)credit, p->mass_eps);
  }
  prof_mark("mass_ema", s);
  hipLaunchKernelGGL(mass_ema_kernel, grid, dim3(kBlock), 0, s, a, u, credit, m_used, p->ema_lambda,
                     p->ema_beta, p->mass_eps);
  return hipGetLastError();
}

hipError_t launch_segment(const ams_params* p, const Dims& d, const int32_t* seq_lens,
                          const float* m_used, int32_t* bounds, float* seg_mass, char* ws, const WsLayout& wl,
                          hipStream_t s) {
  MsArgs a = make_args(p, d, seq_lens, ws, wl, bounds);
  a.vec = d.t_stride % 4 == 0 && ((uintptr_t)m_used & 15) == 0;
  const dim3 grid(a.n_chunks, d.units);
  prof_mark("chunk_total", s);
  hipLaunchKernelGGL(chunk_total_kernel, grid, dim3(kBlock), 0, s, a, m_used);
  prof_mark("segment_scan", s);
  hipLaunchKernelGGL(segment_scan_kernel, grid, dim3(kBlock), 0, s, a, m_used);
  if (a.delta > 0.0) {  // the cuts move, so the masses cannot come from the prefix at the cuts
    if (!seg_mass) return hipErrorInvalidValue;
    prof_mark("resegment", s);
    hipLaunchKernelGGL(resegment_kernel, dim3(d.units), dim3(64), 0, s, a);
    prof_mark("segment_mass", s);
    hipLaunchKernelGGL(segment_mass_kernel, dim3(a.S, d.units), dim3(64), 0, s, a, m_used, seg_mass);
    return hipGetLastError();
  }
  if (seg_mass) {
    prof_mark("segment_finalize", s);
    hipLaunchKernelGGL(segment_finalize_kernel, dim3(d.units), dim3(64), 0, s, a, seg_mass);
  }
  return hipGetLastError();
}

// The fused step's mass / EMA / segmentation / quota stages in one launch.
hipError_t launch_unit_mass(const ams_params* p, const Dims& d, const int32_t* seq_lens, const float* u,
                            float* credit, float* m_used, int32_t* bounds, float* seg_mass, int32_t* quota,
                            int32_t* idx, int32_t* n_kept, uint32_t* flags, int n_words, const VcInfo& vc,
                            char* ws, const WsLayout& wl, hipStream_t s) {
  if (p->n_segments > kMaxSegments) return hipErrorInvalidValue;
  MsArgs a = make_args(p, d, seq_lens, ws, wl, bounds);
  a.vec = d.t_stride % 4 == 0 && (((uintptr_t)u | (uintptr_t)credit | (uintptr_t)m_used) & 15) == 0;
  if (vc.have) {  // left by the scorer
    a.vc_stride = vc.stride;
    a.vc_tokens = vc.tokens;
  } else {
    a.vc_part = nullptr;  // the kernel sums for itself
  }
  const bool must = p->n_sink > 0 || p->n_last > 0;
  if (must && !flags) return hipErrorInvalidValue;
  prof_mark("unit_mass", s);
  const dim3 grid(d.units), blk(kUnitBlock);
  const bool general = p->seg_delta > 0.f || a.pool_r > 0 || p->n_segments > kUnitMaxSeg;
#define AMS_UNIT_MASS_LAUNCH(PER, GEN)                                                                          \
  hipLaunchKernelGGL((unit_mass_kernel<PER, GEN>), grid, blk, 0, s, a, u, credit, m_used, p->ema_lambda,         \
                     p->ema_beta, p->mass_eps, p->budget, p->q_min, seg_mass, quota, idx, n_kept, p->n_sink,    \
                     p->n_last, must ? flags : nullptr, n_words, (const int32_t*)park_status_word(ws, wl))
  if (general)
    AMS_UNIT_MASS_LAUNCH(8, true);
  else
    AMS_UNIT_MASS_LAUNCH(8, false);
#undef AMS_UNIT_MASS_LAUNCH
  return hipGetLastError();
}

}  // namespace ams
