// Eq. (1) + EMA credit (Sec. 3.2, 3.3; Alg. 1 steps 1-2) and the mass prefix sum with its cut
// points (Sec. 3.3 "Mass-based adaptive segmentation"; Alg. 1 step 3, Delta = 1/S).
//
// One workgroup owns one unit.  The vectors are a few hundred KB per unit and stay in L2
// between the passes; every normaliser and every scan carry is held in double so that the
// results are independent of T to well below the fp32 tolerance.
#include "ams_internal.h"

namespace ams {
namespace {

constexpr int kBlock = 1024;
constexpr int kWaves = kBlock / 64;

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

__global__ __launch_bounds__(kBlock) void ema_kernel(Dims d, const int32_t* seq_lens, const float* u_all,
                                                      float* credit_all, float* m_used_all, float lambda,
                                                      float beta, float eps_f) {
  __shared__ double sm[kWaves];
  const int unit = blockIdx.x;
  int l, b, h;
  unit_coords(d, unit, l, b, h);
  const int T = seq_lens[b];
  const float* u = u_all + (int64_t)unit * d.t_stride;
  float* credit = credit_all + (int64_t)unit * d.t_stride;
  float* m_used = m_used_all + (int64_t)unit * d.t_stride;
  const double eps = (double)eps_f, lam = (double)lambda, bet = (double)beta;

  double acc = 0.0;
  for (int t = threadIdx.x; t < T; t += kBlock) acc += fmax((double)u[t], 0.0) + eps;
  const double Z = block_sum(acc, sm);

  if (lambda == 0.f) {  // credit not used: the mass passes through unchanged
    for (int t = threadIdx.x; t < T; t += kBlock) {
      const float mc = (float)((fmax((double)u[t], 0.0) + eps) / Z);
      credit[t] = mc;
      m_used[t] = mc;
    }
    return;
  }
  acc = 0.0;
  for (int t = threadIdx.x; t < T; t += kBlock) {
    const float mc = (float)((fmax((double)u[t], 0.0) + eps) / Z);
    const float cn = (float)(lam * (double)credit[t] + (1.0 - lam) * (double)mc);
    credit[t] = cn;
    acc += (double)cn;
  }
  const double csum = block_sum(acc, sm);
  acc = 0.0;
  for (int t = threadIdx.x; t < T; t += kBlock) {
    const float mc = (float)((fmax((double)u[t], 0.0) + eps) / Z);
    const double ctil = csum > 0.0 ? (double)credit[t] / csum : (double)mc;
    acc += bet * (double)mc + (1.0 - bet) * ctil;
  }
  const double msum = block_sum(acc, sm);
  for (int t = threadIdx.x; t < T; t += kBlock) {
    const float mc = (float)((fmax((double)u[t], 0.0) + eps) / Z);
    const double ctil = csum > 0.0 ? (double)credit[t] / csum : (double)mc;
    m_used[t] = (float)((bet * (double)mc + (1.0 - bet) * ctil) / msum);
  }
}

// Number of thresholds k/S, k = 1..S-1, that are <= c.
__device__ __forceinline__ int thresholds_reached(double c, int S) {
  int f = (int)floor(c * (double)S);
  f = max(0, min(S - 1, f));
  while (f < S - 1 && c >= (double)(f + 1) / (double)S) ++f;
  while (f > 0 && c < (double)f / (double)S) --f;
  return f;
}

constexpr int kPerThread = 4;
constexpr int kTile = kBlock * kPerThread;
constexpr int kMaxSeg = 1024;

// Inclusive prefix P(j) of the unit's mass: every thread owns four consecutive positions of a
// 4096-position tile; P is the tile carry plus a workgroup scan of the thread sums plus the
// thread's own running sum.  Threshold k is cut at the first j whose P(j) reaches k/S.
__global__ __launch_bounds__(kBlock) void segment_kernel(Dims d, const int32_t* seq_lens,
                                                          const float* m_all, int S, int32_t* bounds_all,
                                                          float* seg_mass_all) {
  __shared__ double wave_tot[kWaves];
  __shared__ double ends[kBlock];
  __shared__ int32_t lb[kMaxSeg + 1];
  __shared__ double cpre[kMaxSeg + 1];
  const int unit = blockIdx.x;
  int l, b, h;
  unit_coords(d, unit, l, b, h);
  const int T = seq_lens[b];
  const float* m = m_all + (int64_t)unit * d.t_stride;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  for (int k = threadIdx.x; k <= S; k += kBlock) lb[k] = (k == 0) ? 0 : T;
  double total = 0.0;
  for (int phase = 0; phase < 2; ++phase) {
    double carry = 0.0;      // P of the last position of the previous tile
    double prev_tile_end = 0.0;
    __syncthreads();
    for (int base = 0; base < T; base += kTile) {
      const int j0 = base + threadIdx.x * kPerThread;
      float x[kPerThread];
#pragma unroll
      for (int i = 0; i < kPerThread; ++i) x[i] = (j0 + i < T) ? m[j0 + i] : 0.f;
      double ts = 0.0;
#pragma unroll
      for (int i = 0; i < kPerThread; ++i) ts += (double)x[i];
      double incl = ts;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const double v = __shfl_up(incl, o);
        if (lane >= o) incl += v;
      }
      if (lane == 63) wave_tot[wave] = incl;
      __syncthreads();
      double off = carry;
      for (int w = 0; w < wave; ++w) off += wave_tot[w];
      double tile_end = carry;
      for (int w = 0; w < kWaves; ++w) tile_end += wave_tot[w];
      const double excl = off + (incl - ts);
      double c[kPerThread];
      double run = excl;
#pragma unroll
      for (int i = 0; i < kPerThread; ++i) {
        run += (double)x[i];
        c[i] = run;
      }
      ends[threadIdx.x] = run;
      __syncthreads();
      const double prev_end = threadIdx.x > 0 ? ends[threadIdx.x - 1] : prev_tile_end;
      int f_prev = thresholds_reached(prev_end, S);
#pragma unroll
      for (int i = 0; i < kPerThread; ++i) {
        if (j0 + i < T) {
          const int f_cur = thresholds_reached(c[i], S);
          for (int k = f_prev + 1; k <= f_cur; ++k) {
            if (phase == 0) atomicMin(&lb[k], j0 + i + 1);          // first position that reaches k/S
            else if (lb[k] == j0 + i + 1) cpre[k] = c[i];           // prefix at the cut, for the masses
          }
          f_prev = max(f_prev, f_cur);
        }
      }
      prev_tile_end = ends[kBlock - 1];
      carry = tile_end;
      __syncthreads();
    }
    total = carry;
    if (phase == 0) {
      __syncthreads();
      for (int k = threadIdx.x; k <= S; k += kBlock) cpre[k] = (k == 0) ? 0.0 : total;
    }
  }
  __syncthreads();
  int32_t* bounds = bounds_all + (int64_t)unit * (S + 1);
  float* seg_mass = seg_mass_all + (int64_t)unit * S;
  for (int k = threadIdx.x; k <= S; k += kBlock) bounds[k] = lb[k];
  for (int i = threadIdx.x; i < S; i += kBlock) seg_mass[i] = (float)(cpre[i + 1] - cpre[i]);
}

}  // namespace

hipError_t launch_ema(const ams_params* p, const Dims& d, const int32_t* seq_lens, const float* u,
                      float* credit, float* m_used, hipStream_t s) {
  prof_mark("ema", s);
  hipLaunchKernelGGL(ema_kernel, dim3(d.units), dim3(kBlock), 0, s, d, seq_lens, u, credit, m_used,
                     p->ema_lambda, p->ema_beta, p->mass_eps);
  return hipGetLastError();
}

hipError_t launch_segment(const ams_params* p, const Dims& d, const int32_t* seq_lens,
                          const float* m_used, int32_t* bounds, float* seg_mass, hipStream_t s) {
  if (p->n_segments > kMaxSeg) return hipErrorInvalidValue;
  prof_mark("segment", s);
  hipLaunchKernelGGL(segment_kernel, dim3(d.units), dim3(kBlock), 0, s, d, seq_lens, m_used,
                     p->n_segments, bounds, seg_mass);
  return hipGetLastError();
}

}  // namespace ams
