// Usage u and the softmax-based g of a SHORT cache in one launch (Alg. 1 step 1; Sec. 3.2; Sec. 3.3;
// App. "Compression schedule": after the first event a cache is the kept rows plus the tokens decoded
// since, a few thousand positions).
//
// One workgroup owns a whole unit (at most kScoreChunk positions): it walks the unit's keys once for the
// per-query (max, sum of exp), merges them inside the workgroup, and walks the keys again for the usage --
// the second walk finds the keys in the caches they were just pulled through.  The arithmetic is that of the
// two-sweep kernels (score.hip): the same tiles, the same running statistics, the normaliser in double; what
// goes away are two launches and the trip of the statistics through memory, which is most of the scorer's
// time when an event moves only a couple of megabytes per unit.
#include "score_tile.h"

namespace ams {
namespace {

constexpr int kUnitThreads = 512, kUnitWaves = kUnitThreads / 64;

template <bool BF16, int NB, int MODE, int HD>
__global__ __launch_bounds__(kUnitThreads, 2) void score_unit_kernel(ScoreArgs a) {
  constexpr int NG = (NB % 2 == 0 && NB >= 4) ? NB / 2 : NB, QS = Tr<BF16, HD>::kQStride, NQ = NB * 32;
  constexpr int RB = Tr<BF16, HD>::kRowBytes, CPR = RB / 16;
  extern __shared__ __align__(16) char qlds[];
  __shared__ float2 xch[kUnitWaves][NQ];
  __shared__ float4 fin_s[NQ];
  __shared__ float u_sm[kScoreChunk];
  __shared__ float g_sm[MODE == MODE_LAST ? kScoreChunk : 1];
  __shared__ double2 vc_sm[kUnitWaves];
  const int unit = blockIdx.x;
  if (unit == 0 && threadIdx.x == 0 && a.status) *a.status = 0;  // no bounded wait on this path
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T = seq_len(a.d, a.seq_lens, b);
  if (T <= 0) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, hf = lane >> 5, c = lane & 31;
  uint4 av0[Tr<BF16, HD>::kAVecs], av1[Tr<BF16, HD>::kAVecs];
  constexpr int kStep = kUnitWaves * 32;  // tokens between two blocks of one wave
  if (wave * 32 < T) load_a<BF16, HD>(a, l, b, h, wave * 32, T, lane, av0);
  {  // the query window -> LDS, rows padded against bank conflicts, rows >= N zero
    const char* src = a.q + ((((int64_t)l * a.d.B + b) * a.d.H + h) * a.d.G) * (int64_t)a.d.W * RB;
    for (int ch = threadIdx.x; ch < NQ * CPR; ch += kUnitThreads) {
      const int n = ch / CPR, col = ch % CPR;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (n < a.d.N) v = *(const uint4*)(src + (int64_t)n * RB + col * 16);
      *(uint4*)(qlds + n * QS + col * 16) = v;
    }
  }
  // the old credit of the unit (for the EMA normaliser): at most 8 positions per thread, in flight during the walks
  float cr[kScoreChunk / kUnitThreads];
#pragma unroll
  for (int k = 0; k < kScoreChunk / kUnitThreads; ++k) {
    const int t = k * kUnitThreads + (int)threadIdx.x;
    cr[k] = (a.vc_part && a.credit && t < T) ? a.credit[(int64_t)unit * a.d.t_stride + t] : 0.f;
  }
  __syncthreads();
  const float c2 = a.c2;

  // ---- first walk: per query (max, sum exp2) of the scaled logits over this wave's blocks ----
  float m[NB], z[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    m[nb] = kNegInit;
    z[nb] = 0.f;
  }
  auto stats_block = [&](const uint4 (&av)[Tr<BF16, HD>::kAVecs], int t0) __attribute__((always_inline)) {
    const bool ragged = t0 + 32 > T;
    int qoff = 0;  // the query fragments are re-read from LDS per block on purpose (registers)
    asm volatile("" : "+s"(qoff));
#pragma unroll
    for (int g0 = 0; g0 < NB; g0 += NG) {
      floatx16 acc[NG];
      tile_mma<BF16, NG, HD>(av, qlds + qoff + g0 * 32 * QS, lane, acc);
#pragma unroll
      for (int k = 0; k < NG; ++k) {
        const int nb = g0 + k;
        if (ragged) {
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[k][i] = (t0 + acc_row(i, hf) >= T) ? -INFINITY : acc[k][i];
        }
        float mr = acc[k][0];
#pragma unroll
        for (int i = 1; i < 16; ++i) mr = fmaxf(mr, acc[k][i]);
        const float mx = fmaxf(m[nb], mr * c2);  // c2 > 0: the maximum commutes with the scale
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) sum += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[k][i], c2, -mx));
        z[nb] = __builtin_fmaf(z[nb], __builtin_amdgcn_exp2f(m[nb] - mx), sum);
        m[nb] = mx;
      }
    }
  };
#pragma unroll 1
  for (int t0 = wave * 32; t0 < T; t0 += 2 * kStep) {
    if (t0 + kStep < T) load_a<BF16, HD>(a, l, b, h, t0 + kStep, T, lane, av1);
    stats_block(av0, t0);
    if (t0 + kStep >= T) break;
    if (t0 + 2 * kStep < T) load_a<BF16, HD>(a, l, b, h, t0 + 2 * kStep, T, lane, av0);
    stats_block(av1, t0 + kStep);
  }
  // the second walk's first block travels during the merge
  if (wave * 32 < T) load_a<BF16, HD>(a, l, b, h, wave * 32, T, lane, av0);
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const float m2 = __shfl_xor(m[nb], 32), z2 = __shfl_xor(z[nb], 32);
    const float M = fmaxf(m[nb], m2);
    // lower half first so that both halves compute the same value
    const float zl = hf ? z2 : z[nb], ml = hf ? m2 : m[nb], zh = hf ? z[nb] : z2, mh = hf ? m[nb] : m2;
    const float Z = zl * __builtin_amdgcn_exp2f(ml - M) + zh * __builtin_amdgcn_exp2f(mh - M);
    if (hf == 0) xch[wave][nb * 32 + c] = make_float2(M, Z);
  }
  __syncthreads();
  if (threadIdx.x < NQ) {  // waves merged in index order, the normaliser in double
    const int n = threadIdx.x;
    float M = kNegInit;
#pragma unroll
    for (int w = 0; w < kUnitWaves; ++w) M = fmaxf(M, xch[w][n].x);
    double Z = 0.0;
#pragma unroll
    for (int w = 0; w < kUnitWaves; ++w) Z += (double)xch[w][n].y * (double)__builtin_amdgcn_exp2f(xch[w][n].x - M);
    const bool real = n < a.d.N;
    const bool newest = real && (n % a.d.W) == a.d.W - 1;
    fin_s[n] = make_float4(M, real ? (float)(1.0 / ((double)a.d.N * Z)) : 0.f,
                           newest ? (float)(1.0 / ((double)a.d.G * Z)) : 0.f, real ? 1.f : 0.f);
  }
  __syncthreads();

  // ---- second walk: u[t] = sum_n exp2(x[n][t] - M_n) / (N Z_n), and the last-query g ----
  float4 f[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) f[nb] = fin_s[nb * 32 + c];
  float v_part = 0.f;  // this lane's share of sum(max(u,0)+eps)
  auto usage_block = [&](const uint4 (&av)[Tr<BF16, HD>::kAVecs], int t0) __attribute__((always_inline)) {
    float pu[16], pg[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) pu[i] = pg[i] = 0.f;
    int qoff = 0;
    asm volatile("" : "+s"(qoff));
#pragma unroll
    for (int g0 = 0; g0 < NB; g0 += NG) {
      floatx16 acc[NG];
      tile_mma<BF16, NG, HD>(av, qlds + qoff + g0 * 32 * QS, lane, acc);
#pragma unroll
      for (int k = 0; k < NG; ++k) {
        const int nb = g0 + k;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[k][i], c2, -f[nb].x));
          pu[i] = __builtin_fmaf(f[nb].y, e, pu[i]);
          if (MODE == MODE_LAST) pg[i] = __builtin_fmaf(f[nb].z, e, pg[i]);
        }
      }
    }
    const int t = t0 + acc_row(c >> 1, hf);
    const float ru = reduce16_over32(pu, c);
    float rg = ru;
    if (MODE == MODE_LAST) rg = reduce16_over32(pg, c);
    if ((c & 1) == 0 && t < T) {
      u_sm[t] = ru;
      if (MODE == MODE_LAST) g_sm[t] = rg;
      v_part += fmaxf(ru, 0.f) + a.eps;
    }
  };
#pragma unroll 1
  for (int t0 = wave * 32; t0 < T; t0 += 2 * kStep) {
    if (t0 + kStep < T) load_a<BF16, HD>(a, l, b, h, t0 + kStep, T, lane, av1);
    usage_block(av0, t0);
    if (t0 + kStep >= T) break;
    if (t0 + 2 * kStep < T) load_a<BF16, HD>(a, l, b, h, t0 + 2 * kStep, T, lane, av0);
    usage_block(av1, t0 + kStep);
  }
  __syncthreads();
  float* u_row = a.u + (int64_t)unit * a.d.t_stride;
  float* g_row = a.g ? a.g + (int64_t)unit * a.d.t_stride : nullptr;
  for (int t = threadIdx.x; t < T; t += kUnitThreads) {
    u_row[t] = u_sm[t];
    if (g_row) g_row[t] = MODE == MODE_LAST ? g_sm[t] : u_sm[t];
  }
  if (a.vc_part) {  // the unit's sums of max(u,0)+eps and of the old credit: lanes, then waves, fixed order
    double v_acc = (double)v_part, c_acc = 0.0;
#pragma unroll
    for (int k = 0; k < kScoreChunk / kUnitThreads; ++k) c_acc += (double)cr[k];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      v_acc += __shfl_xor(v_acc, o);
      c_acc += __shfl_xor(c_acc, o);
    }
    if (lane == 0) vc_sm[wave] = make_double2(v_acc, c_acc);
    __syncthreads();
    if (threadIdx.x == 0) {
      double2 t = vc_sm[0];
      for (int w = 1; w < kUnitWaves; ++w) {
        t.x += vc_sm[w].x;
        t.y += vc_sm[w].y;
      }
      a.vc_part[unit] = t;
    }
  }
}

template <bool BF16, int NB, int MODE, int HD>
hipError_t launch_unit(const ScoreArgs& a, hipStream_t s) {
  const int lds = NB * 32 * Tr<BF16, HD>::kQStride;
  const hipError_t e = ensure_lds<score_unit_kernel<BF16, NB, MODE, HD>>(lds);
  if (e != hipSuccess) return e;
  prof_mark("score_unit", s);
  hipLaunchKernelGGL((score_unit_kernel<BF16, NB, MODE, HD>), dim3(a.d.units), dim3(kUnitThreads), lds, s, a);
  return hipGetLastError();
}

template <bool BF16, int HD>
hipError_t unit_by_nb(const ScoreArgs& a, int nb, int mode, hipStream_t s, bool* ran) {
  *ran = true;
#define AMS_UNIT_CASE(NBV)                                                           \
  if (nb <= NBV) {                                                                   \
    if (mode == MODE_LAST) return launch_unit<BF16, NBV, MODE_LAST, HD>(a, s);       \
    return launch_unit<BF16, NBV, MODE_MEAN, HD>(a, s);                              \
  }
  AMS_UNIT_CASE(1)
  AMS_UNIT_CASE(2)
  AMS_UNIT_CASE(4)
#undef AMS_UNIT_CASE
  *ran = false;
  return hipSuccess;
}

}  // namespace

// Runs the one-launch scorer when it applies: caches of at most kScoreChunk positions, bf16 or fp32, up to
// 128 queries per KV head, no causal window, mean-window / last-query statistics (the key-diversity scorer
// takes its usage from here too).  *ran = false: the caller uses the two sweeps.
hipError_t launch_score_unit(const ScoreArgs& a, bool bf16, int head_dim, int mode, hipStream_t s, bool* ran) {
  *ran = false;
  if (a.d.t_max > kScoreChunk || a.causal || mode == MODE_EXPECTED || a.n_pad > 128) return hipSuccess;
  const int nb = a.n_pad / 32;
  if (head_dim == 64)
    return bf16 ? unit_by_nb<true, 64>(a, nb, mode, s, ran) : unit_by_nb<false, 64>(a, nb, mode, s, ran);
  return bf16 ? unit_by_nb<true, 128>(a, nb, mode, s, ran) : unit_by_nb<false, 128>(a, nb, mode, s, ran);
}

}  // namespace ams
