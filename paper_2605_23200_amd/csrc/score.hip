// Usage u and base score g (Alg. 1 step 1; Sec. 3.2; Sec. 3.3 plug-in scorer).
//
// s[n][t] = q_n . k_t / sqrt(D) is a dense N x D by D x T contraction and runs on
// the matrix cores (32x32 MFMA tiles, token rows x query columns).  The row
// softmax needs every row's normaliser before a column can be finished, so the
// work is two sweeps over K:
//   sweep 1  per 1024-token chunk, per query: running (max, sum of exp) in the
//            log2 domain, lane-local, merged per chunk          -> part_stats
//   reduce   chunks merged in a fixed order                     -> (M_n, weights)
//   sweep 2  tiles recomputed, exp2(s - M_n) weighted by 1/(N Z_n) and summed
//            over the queries of each token                     -> u (and g)
// The score matrix itself never reaches memory.
#include "score_tile.h"

namespace ams {
namespace {

// ---------------------------------------------------------------------------------------------
// Both sweeps walk a 1024-token chunk in 32-token blocks per wave.  The keys of the next block are
// requested before the current block is multiplied (two register buffers, used alternately), and
// the query columns are processed in groups of kGroup<NB> blocks of 32 so that only that many
// accumulator tiles are live at a time: more bytes in flight per wave at the same occupancy.
// ---------------------------------------------------------------------------------------------
#ifndef AMS_SCORE_GROUP_DIV
#define AMS_SCORE_GROUP_DIV 2   // column blocks of a wave are processed in this many groups (tuning knob)
#endif
#ifndef AMS_SCORE_MIN_WAVES
#define AMS_SCORE_MIN_WAVES 3   // waves per SIMD the register allocation aims for (tuning knob)
#endif
template <int NB>
constexpr int kGroup = (NB % AMS_SCORE_GROUP_DIV == 0 && NB >= 4) ? NB / AMS_SCORE_GROUP_DIV : NB;

// ---------------------------------------------------------------------------------------------
// Sweep 1: per chunk, per query (max, sum exp2) of the scaled logits.
// ---------------------------------------------------------------------------------------------
template <bool BF16, int NB>
__global__ __launch_bounds__(kThreads, (BF16 && NB <= 4) ? AMS_SCORE_MIN_WAVES : 2) void score_stats_kernel(ScoreArgs a) {
  constexpr int NG = kGroup<NB>, QS = Tr<BF16>::kQStride, NBLK = kScoreChunk / 128;
  extern __shared__ __align__(16) char qlds[];
  __shared__ float2 xch[4][NB * 32];
  const int unit = blockIdx.y, chunk = blockIdx.x;
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T = max(a.seq_lens[b] - a.t_cut, 0);
  const int c0 = chunk * kScoreChunk;
  if (c0 >= T) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, hf = lane >> 5;
  uint4 av0[Tr<BF16>::kAVecs], av1[Tr<BF16>::kAVecs];
  if (c0 + wave * 32 < T) load_a<BF16>(a, l, b, h, c0 + wave * 32, T, lane, av0);
  load_q<BF16, NB>(a, l, b, h, qlds);
  __syncthreads();
  float m[NB], z[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    m[nb] = kNegInit;
    z[nb] = 0.f;
  }
  const float c2 = a.c2;
  auto block = [&](const uint4 (&av)[Tr<BF16>::kAVecs], int t0) __attribute__((always_inline)) {
    const bool ragged = t0 + 32 > T;
    // the query fragments are re-read from LDS for every block: keeping them in registers across
    // blocks would cost more registers than the reads cost time, so their address is made opaque
    int qoff = 0;
    asm volatile("" : "+s"(qoff));
#pragma unroll
    for (int g0 = 0; g0 < NB; g0 += NG) {
      floatx16 acc[NG];
      tile_mma<BF16, NG>(av, qlds + qoff + g0 * 32 * QS, lane, acc);
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
  for (int blk = 0; blk < NBLK; blk += 2) {
    const int t0 = c0 + (blk * 4 + wave) * 32;
    if (t0 >= T) break;
    if (t0 + 128 < T) load_a<BF16>(a, l, b, h, t0 + 128, T, lane, av1);
    block(av0, t0);
    if (t0 + 128 >= T) break;
    if (blk + 2 < NBLK && t0 + 256 < T) load_a<BF16>(a, l, b, h, t0 + 256, T, lane, av0);
    block(av1, t0 + 128);
  }
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const float m2 = __shfl_xor(m[nb], 32), z2 = __shfl_xor(z[nb], 32);
    const float M = fmaxf(m[nb], m2);
    // lower half first so that both halves compute the same value
    const float zl = hf ? z2 : z[nb], ml = hf ? m2 : m[nb], zh = hf ? z[nb] : z2, mh = hf ? m[nb] : m2;
    const float Z = zl * __builtin_amdgcn_exp2f(ml - M) + zh * __builtin_amdgcn_exp2f(mh - M);
    if (hf == 0) xch[wave][nb * 32 + (lane & 31)] = make_float2(M, Z);
  }
  __syncthreads();
  for (int n = threadIdx.x; n < NB * 32; n += kThreads) {
    float M = kNegInit;
#pragma unroll
    for (int w = 0; w < 4; ++w) M = fmaxf(M, xch[w][n].x);
    float Z = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) Z += xch[w][n].y * __builtin_amdgcn_exp2f(xch[w][n].x - M);
    a.part[((int64_t)unit * (a.n_chunks + 1) + chunk) * a.n_pad + n] = make_float2(M, Z);
  }
}

// Chunk statistics merged per query: the 1024 threads split into (query, contiguous range of
// chunks) pairs, the ranges are then combined in ascending order (fixed association) -> M_n and
// the per-query weights of the column sums.
constexpr int kReduceThreads = 1024;
__global__ __launch_bounds__(kReduceThreads) void score_reduce_kernel(ScoreArgs a) {
  __shared__ float pm[kReduceThreads];
  __shared__ double pz[kReduceThreads];
  const int unit = blockIdx.x;
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T_all = a.seq_lens[b];
  const int T = max(T_all - a.t_cut, 0);
  // with a causal window one more entry follows the chunks: the statistics over the newest keys
  const int nch = (T + kScoreChunk - 1) / kScoreChunk + (a.t_cut > 0 ? 1 : 0);
  const int parts = kReduceThreads / a.n_pad;
  const int n = threadIdx.x % a.n_pad, part = threadIdx.x / a.n_pad;
  if (part < parts) {
    const int per = (nch + parts - 1) / parts;
    const int c0 = part * per, c1 = min(nch, c0 + per);
    const float2* p = a.part + (int64_t)unit * (a.n_chunks + 1) * a.n_pad + n;
    float M = kNegInit;
    for (int c = c0; c < c1; ++c) M = fmaxf(M, p[(int64_t)c * a.n_pad].x);
    double Z = 0.0;
    for (int c = c0; c < c1; ++c) {
      const float2 s = p[(int64_t)c * a.n_pad];
      Z += (double)s.y * (double)__builtin_amdgcn_exp2f(s.x - M);
    }
    pm[threadIdx.x] = M;
    pz[threadIdx.x] = Z;
  }
  __syncthreads();
  if (threadIdx.x < a.n_pad) {
    float M = kNegInit;
    for (int q = 0; q < parts; ++q) M = fmaxf(M, pm[q * a.n_pad + n]);
    double Z = 0.0;
    for (int q = 0; q < parts; ++q) Z += pz[q * a.n_pad + n] * (double)__builtin_amdgcn_exp2f(pm[q * a.n_pad + n] - M);
    const bool real = n < a.d.N;
    // causal window on a cache shorter than the window: a query before position 0 does not exist
    const bool exists = real && (a.t_cut == 0 || T_all - a.d.W + (n % a.d.W) >= 0);
    const bool newest = exists && (n % a.d.W) == a.d.W - 1;
    float4 f;
    f.x = M;
    f.y = exists ? (float)(1.0 / ((double)a.d.N * Z)) : 0.f;
    f.z = newest ? (float)(1.0 / ((double)a.d.G * Z)) : 0.f;
    f.w = real ? 1.f : 0.f;
    a.fin[(int64_t)unit * a.n_pad + n] = f;
  }
}

// ---------------------------------------------------------------------------------------------
// Sweep 2: u[t] = sum_n exp2(x[n][t] - M_n) / (N Z_n), and g for the softmax- or moment-based scorers.
// ---------------------------------------------------------------------------------------------
template <bool BF16, int NB, int MODE>
__global__ __launch_bounds__(kThreads, (BF16 && NB <= 4) ? AMS_SCORE_MIN_WAVES : 2) void score_usage_kernel(ScoreArgs a) {
  // the moment-based scorer needs all N logits of a token twice: keep every column block live
  constexpr int NG = (MODE == MODE_EXPECTED) ? NB : kGroup<NB>;
  constexpr int QS = Tr<BF16>::kQStride, NBLK = kScoreChunk / 128;
  extern __shared__ __align__(16) char qlds[];
  const int unit = blockIdx.y, chunk = blockIdx.x;
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T = max(a.seq_lens[b] - a.t_cut, 0);
  const int c0 = chunk * kScoreChunk;
  if (c0 >= T) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, hf = lane >> 5, c = lane & 31;
  uint4 av0[Tr<BF16>::kAVecs], av1[Tr<BF16>::kAVecs];
  if (c0 + wave * 32 < T) load_a<BF16>(a, l, b, h, c0 + wave * 32, T, lane, av0);
  load_q<BF16, NB>(a, l, b, h, qlds);
  __syncthreads();
  float4 f[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) f[nb] = a.fin[(int64_t)unit * a.n_pad + nb * 32 + c];
  float* u_row = a.u + (int64_t)unit * a.d.t_stride;
  float* g_row = a.g ? a.g + (int64_t)unit * a.d.t_stride : nullptr;
  const float inv_n = 1.f / (float)a.d.N, c2 = a.c2;
  const float* c_row = a.credit ? a.credit + (int64_t)unit * a.d.t_stride : nullptr;
  float v_part = 0.f;  // this lane's share of sum(max(u,0)+eps): at most 8 terms
  auto block = [&](const uint4 (&av)[Tr<BF16>::kAVecs], int t0) __attribute__((always_inline)) {
    float pu[16], pg[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) pu[i] = pg[i] = 0.f;
    float rg = 0.f;
    int qoff = 0;  // see the first sweep: the query fragments are re-read per block on purpose
    asm volatile("" : "+s"(qoff));
#pragma unroll
    for (int g0 = 0; g0 < NB; g0 += NG) {
      floatx16 acc[NG];
      tile_mma<BF16, NG>(av, qlds + qoff + g0 * 32 * QS, lane, acc);
      if (MODE == MODE_EXPECTED) {
        // mean and centred second moment of the N logits of each token (padded queries add exact zeros)
#pragma unroll
        for (int k = 0; k < NG; ++k)
#pragma unroll
          for (int i = 0; i < 16; ++i) pg[i] += acc[k][i] * a.inv_sqrt_d;
        const float mean_mine = reduce16_over32(pg, c) * inv_n;
        float pv[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float mean_i = __shfl(mean_mine, 2 * i + 32 * hf);
          float s2 = 0.f;
#pragma unroll
          for (int k = 0; k < NG; ++k) {
            const float dlt = acc[k][i] * a.inv_sqrt_d - mean_i;
            s2 += f[g0 + k].w * dlt * dlt;
          }
          pv[i] = s2;
        }
        rg = mean_mine + 0.5f * reduce16_over32(pv, c) * inv_n;
      }
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
    const float ru = reduce16_over32(pu, c);
    if (MODE == MODE_MEAN) rg = ru;
    if (MODE == MODE_LAST) rg = reduce16_over32(pg, c);
    const int t = t0 + acc_row(c >> 1, hf);
    if ((c & 1) == 0 && t < T) {
      u_row[t] = ru;
      if (g_row) g_row[t] = rg;
      v_part += fmaxf(ru, 0.f) + a.eps;
    }
  };
#pragma unroll 1
  for (int blk = 0; blk < NBLK; blk += 2) {
    const int t0 = c0 + (blk * 4 + wave) * 32;
    if (t0 >= T) break;
    if (t0 + 128 < T) load_a<BF16>(a, l, b, h, t0 + 128, T, lane, av1);
    block(av0, t0);
    if (t0 + 128 >= T) break;
    if (blk + 2 < NBLK && t0 + 256 < T) load_a<BF16>(a, l, b, h, t0 + 256, T, lane, av0);
    block(av1, t0 + 128);
  }
  if (a.vc_part) {  // chunk sums in a fixed order: lanes, then waves
    __shared__ double2 vc_sm[4];
    double v_acc = (double)v_part, c_acc = 0.0;
    if (c_row) {  // the chunk's credit, a few consecutive positions per thread
      constexpr int PER = kScoreChunk / kThreads;
      const int j0 = c0 + threadIdx.x * PER;
#pragma unroll
      for (int i = 0; i < PER; ++i)
        if (j0 + i < T) c_acc += (double)c_row[j0 + i];
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      v_acc += __shfl_xor(v_acc, o);
      c_acc += __shfl_xor(c_acc, o);
    }
    if (lane == 0) vc_sm[wave] = make_double2(v_acc, c_acc);
    __syncthreads();
    if (threadIdx.x == 0) {
      double2 t = vc_sm[0];
      for (int w = 1; w < 4; ++w) {
        t.x += vc_sm[w].x;
        t.y += vc_sm[w].y;
      }
      a.vc_part[(int64_t)unit * a.n_chunks + chunk] = t;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Key-diversity score: g[t] = -cos(k_t, kbar), kbar the mean key of the unit.
// ---------------------------------------------------------------------------------------------
template <bool BF16>
__device__ __forceinline__ void widen8(const uint4& v, float (&x)[8], int& n) {
  if constexpr (BF16) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = __uint_as_float(w[i] << 16);
      x[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
    n = 8;
  } else {
    x[0] = __uint_as_float(v.x);
    x[1] = __uint_as_float(v.y);
    x[2] = __uint_as_float(v.z);
    x[3] = __uint_as_float(v.w);
    n = 4;
  }
}

// partial key sums per chunk: ksum[unit][chunk][D] (double)
template <bool BF16>
__global__ __launch_bounds__(kThreads) void keysum_kernel(ScoreArgs a, double* ksum) {
  constexpr int CPR = Tr<BF16>::kRowBytes / 16, EPC = BF16 ? 8 : 4, RPI = kThreads / CPR;
  __shared__ double sm[kThreads][EPC];
  const int unit = blockIdx.y, chunk = blockIdx.x;
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T = a.seq_lens[b];
  const int c0 = chunk * kScoreChunk;
  if (c0 >= T) return;
  const int col = threadIdx.x % CPR, r0 = threadIdx.x / CPR;
  double s[EPC];
#pragma unroll
  for (int e = 0; e < EPC; ++e) s[e] = 0.0;
  for (int t = c0 + r0; t < min(T, c0 + kScoreChunk); t += RPI) {
    const uint4 v = *(const uint4*)(kv_row(a.k, l, b, h, t) + col * 16);
    float x[8];
    int n;
    widen8<BF16>(v, x, n);
#pragma unroll
    for (int e = 0; e < EPC; ++e) s[e] += (double)x[e];
  }
#pragma unroll
  for (int e = 0; e < EPC; ++e) sm[threadIdx.x][e] = s[e];
  __syncthreads();
  if (threadIdx.x < CPR) {
    for (int e = 0; e < EPC; ++e) {
      double t = 0.0;
      for (int r = 0; r < RPI; ++r) t += sm[r * CPR + threadIdx.x][e];
      ksum[((int64_t)unit * a.n_chunks + chunk) * a.d.D + threadIdx.x * EPC + e] = t;
    }
  }
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void keydiff_kernel(ScoreArgs a, const double* ksum) {
  constexpr int CPR = Tr<BF16>::kRowBytes / 16, EPC = BF16 ? 8 : 4, RPI = kThreads / CPR;
  __shared__ double kbar[128];
  __shared__ double kbar_norm;
  const int unit = blockIdx.y, chunk = blockIdx.x;
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T = a.seq_lens[b];
  const int c0 = chunk * kScoreChunk;
  if (c0 >= T) return;
  const int nch = (T + kScoreChunk - 1) / kScoreChunk;
  if (threadIdx.x < a.d.D) {
    double t = 0.0;
    for (int c = 0; c < nch; ++c) t += ksum[((int64_t)unit * a.n_chunks + c) * a.d.D + threadIdx.x];
    kbar[threadIdx.x] = t / (double)T;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double n2 = 0.0;
    for (int d = 0; d < a.d.D; ++d) n2 += kbar[d] * kbar[d];
    kbar_norm = sqrt(n2);
  }
  __syncthreads();
  const int col = threadIdx.x % CPR, r0 = threadIdx.x / CPR;
  float* g_row = a.g + (int64_t)unit * a.d.t_stride;
  for (int tb = c0; tb < min(T, c0 + kScoreChunk); tb += RPI) {
    const int t = tb + r0;
    double dot = 0.0, nk = 0.0;
    if (t < T) {
      const uint4 v = *(const uint4*)(kv_row(a.k, l, b, h, t) + col * 16);
      float x[8];
      int n;
      widen8<BF16>(v, x, n);
#pragma unroll
      for (int e = 0; e < EPC; ++e) {
        dot += (double)x[e] * kbar[col * EPC + e];
        nk += (double)x[e] * (double)x[e];
      }
    }
    // the CPR lanes of a row are consecutive lanes of one wave
#pragma unroll
    for (int o = CPR / 2; o >= 1; o >>= 1) {
      dot += __shfl_xor(dot, o);
      nk += __shfl_xor(nk, o);
    }
    if (col == 0 && t < T) {
      const double den = sqrt(nk) * kbar_norm;
      g_row[t] = den > 0.0 ? (float)(-dot / den) : 0.f;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Causal window (App. A "Mass construction"): query w of the window sits at position T-W+w and sees
// the keys up to its own position.  The keys up to T-W are seen by every query and go through the
// two sweeps above; the W-1 newest keys are few, each seen by a different set of queries, and are
// handled here with one thread per query: their contribution to every query's (max, sum), and then
// their usage, where each observation a key is missing counts as the largest probability it got.
// ---------------------------------------------------------------------------------------------
template <bool BF16>
__device__ __forceinline__ void load_q_rows(const ScoreArgs& a, int l, int b, int h, char* qlds) {
  constexpr int RB = Tr<BF16>::kRowBytes, QS = Tr<BF16>::kQStride, CPR = RB / 16;
  const char* src = a.q + ((((int64_t)l * a.d.B + b) * a.d.H + h) * a.d.G) * (int64_t)a.d.W * RB;
  for (int ch = threadIdx.x; ch < a.d.N * CPR; ch += kThreads) {
    const int n = ch / CPR, col = ch % CPR;
    *(uint4*)(qlds + n * QS + col * 16) = *(const uint4*)(src + (int64_t)n * RB + col * 16);
  }
}

// q . k over the 128 channels, fp32 accumulation in four interleaved partial sums
template <bool BF16>
__device__ __forceinline__ float dot_qk(const char* qrow, const char* krow) {
  float s[4] = {0.f, 0.f, 0.f, 0.f};
  constexpr int NV = Tr<BF16>::kRowBytes / 16;
#pragma unroll 4
  for (int i = 0; i < NV; ++i) {
    const uint4 kv = *(const uint4*)(krow + i * 16), qv = *(const uint4*)(qrow + i * 16);
    float kx[8], qx[8];
    int n;
    widen8<BF16>(kv, kx, n);
    widen8<BF16>(qv, qx, n);
#pragma unroll
    for (int e = 0; e < (BF16 ? 8 : 4); ++e) s[e & 3] = __builtin_fmaf(qx[e], kx[e], s[e & 3]);
  }
  return (s[0] + s[1]) + (s[2] + s[3]);
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void score_tail_stats_kernel(ScoreArgs a) {
  extern __shared__ __align__(16) char qlds[];
  const int unit = blockIdx.x, n = threadIdx.x;
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T = a.seq_lens[b], W = a.d.W;
  const int t_first = max(T - a.t_cut, 0);
  load_q_rows<BF16>(a, l, b, h, qlds);
  __syncthreads();
  float m = kNegInit, z = 0.f;
  if (n < a.d.N) {
    const int pos = T - W + (n % W);  // newest key this query sees
    for (int t = t_first; t <= pos; ++t) {
      const float x = dot_qk<BF16>(qlds + n * Tr<BF16>::kQStride, kv_row(a.k, l, b, h, t)) * a.c2;
      const float mx = fmaxf(m, x);
      z = __builtin_fmaf(z, __builtin_amdgcn_exp2f(m - mx), __builtin_amdgcn_exp2f(x - mx));
      m = mx;
    }
  }
  const int slot = (t_first + kScoreChunk - 1) / kScoreChunk;  // right after the chunks of the sweeps
  if (n < a.n_pad) a.part[((int64_t)unit * (a.n_chunks + 1) + slot) * a.n_pad + n] = make_float2(m, z);
}

template <bool BF16, int MODE>
__global__ __launch_bounds__(kThreads) void score_tail_usage_kernel(ScoreArgs a) {
  extern __shared__ __align__(16) char qlds[];
  __shared__ float4 red[4];
  __shared__ float red2[4];
  const int unit = blockIdx.x, n = threadIdx.x, lane = n & 63, wave = n >> 6;
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T = a.seq_lens[b], W = a.d.W, N = a.d.N;
  const int t_first = max(T - a.t_cut, 0);
  load_q_rows<BF16>(a, l, b, h, qlds);
  __syncthreads();
  const bool real = n < N;
  const int pos = real ? T - W + (n % W) : -1;
  const float4 f = n < a.n_pad ? a.fin[(int64_t)unit * a.n_pad + n] : make_float4(0.f, 0.f, 0.f, 0.f);
  float* u_row = a.u + (int64_t)unit * a.d.t_stride;
  float* g_row = a.g ? a.g + (int64_t)unit * a.d.t_stride : nullptr;
  const float inv_n = 1.f / (float)N;
  for (int t = t_first; t < T; ++t) {
    const float x = real ? dot_qk<BF16>(qlds + n * Tr<BF16>::kQStride, kv_row(a.k, l, b, h, t)) : 0.f;
    const bool sees = pos >= t;
    const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(x, a.c2, -f.x));
    // x: share of this (query, key) pair in u, y: the same for the maximum, z: share in the
    // last-query score, w: logit for the moment-based score
    float4 v = make_float4(sees ? e * f.y : 0.f, sees ? e * f.y : 0.f, sees ? e * f.z : 0.f,
                           real ? x * a.inv_sqrt_d : 0.f);
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      v.x += __shfl_xor(v.x, o);
      v.y = fmaxf(v.y, __shfl_xor(v.y, o));
      v.z += __shfl_xor(v.z, o);
      v.w += __shfl_xor(v.w, o);
    }
    if (lane == 0) red[wave] = v;
    __syncthreads();
    const float sum_p = (red[0].x + red[1].x) + (red[2].x + red[3].x);
    const float max_p = fmaxf(fmaxf(red[0].y, red[1].y), fmaxf(red[2].y, red[3].y));
    const float sum_last = (red[0].z + red[1].z) + (red[2].z + red[3].z);
    const float mean = ((red[0].w + red[1].w) + (red[2].w + red[3].w)) * inv_n;
    float var = 0.f;
    if (MODE == MODE_EXPECTED) {
      const float dlt = x * a.inv_sqrt_d - mean;
      float s2 = real ? dlt * dlt : 0.f;
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) s2 += __shfl_xor(s2, o);
      if (lane == 0) red2[wave] = s2;
      __syncthreads();
      var = ((red2[0] + red2[1]) + (red2[2] + red2[3])) * inv_n;
    }
    if (n == 0) {
      const int seen = a.d.G * min(W, T - t);  // pairs that see key t
      const float ru = sum_p + (float)(N - seen) * max_p;
      u_row[t] = ru;
      if (g_row) g_row[t] = MODE == MODE_MEAN ? ru : MODE == MODE_LAST ? sum_last : mean + 0.5f * var;
    }
    __syncthreads();
  }
}

template <typename K>
hipError_t set_lds(K kernel, int bytes) {
  return hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

template <bool BF16>
hipError_t run_tail_usage(const ScoreArgs& a, int mode, hipStream_t s) {
  const int lds = a.d.N * Tr<BF16>::kQStride;
  const dim3 grid(a.d.units), blk(kThreads);
  hipError_t e;
  prof_mark("score_tail_usage", s);
  switch (mode) {
    case MODE_LAST:
      if ((e = set_lds(score_tail_usage_kernel<BF16, MODE_LAST>, lds)) != hipSuccess) return e;
      hipLaunchKernelGGL((score_tail_usage_kernel<BF16, MODE_LAST>), grid, blk, lds, s, a);
      break;
    case MODE_EXPECTED:
      if ((e = set_lds(score_tail_usage_kernel<BF16, MODE_EXPECTED>, lds)) != hipSuccess) return e;
      hipLaunchKernelGGL((score_tail_usage_kernel<BF16, MODE_EXPECTED>), grid, blk, lds, s, a);
      break;
    default:
      if ((e = set_lds(score_tail_usage_kernel<BF16, MODE_MEAN>, lds)) != hipSuccess) return e;
      hipLaunchKernelGGL((score_tail_usage_kernel<BF16, MODE_MEAN>), grid, blk, lds, s, a);
  }
  return hipGetLastError();
}

template <bool BF16, int NB>
hipError_t run_softmax_sweeps(const ScoreArgs& a, int mode, hipStream_t s) {
  const int lds = NB * 32 * Tr<BF16>::kQStride;
  const dim3 grid(a.n_chunks, a.d.units), blk(kThreads);
  hipError_t e;
  if ((e = set_lds(score_stats_kernel<BF16, NB>, lds)) != hipSuccess) return e;
  prof_mark("score_stats", s);
  hipLaunchKernelGGL((score_stats_kernel<BF16, NB>), grid, blk, lds, s, a);
  if (a.t_cut > 0) {
    const int tail_lds = a.d.N * Tr<BF16>::kQStride;
    if ((e = set_lds(score_tail_stats_kernel<BF16>, tail_lds)) != hipSuccess) return e;
    prof_mark("score_tail_stats", s);
    hipLaunchKernelGGL(score_tail_stats_kernel<BF16>, dim3(a.d.units), blk, tail_lds, s, a);
  }
  prof_mark("score_reduce", s);
  hipLaunchKernelGGL(score_reduce_kernel, dim3(a.d.units), dim3(kReduceThreads), 0, s, a);
  prof_mark("score_usage", s);
  switch (mode) {
    case MODE_LAST:
      if ((e = set_lds(score_usage_kernel<BF16, NB, MODE_LAST>, lds)) != hipSuccess) return e;
      hipLaunchKernelGGL((score_usage_kernel<BF16, NB, MODE_LAST>), grid, blk, lds, s, a);
      break;
    case MODE_EXPECTED:
      if ((e = set_lds(score_usage_kernel<BF16, NB, MODE_EXPECTED>, lds)) != hipSuccess) return e;
      hipLaunchKernelGGL((score_usage_kernel<BF16, NB, MODE_EXPECTED>), grid, blk, lds, s, a);
      break;
    default:
      if ((e = set_lds(score_usage_kernel<BF16, NB, MODE_MEAN>, lds)) != hipSuccess) return e;
      hipLaunchKernelGGL((score_usage_kernel<BF16, NB, MODE_MEAN>), grid, blk, lds, s, a);
  }
  if ((e = hipGetLastError()) != hipSuccess) return e;
  return a.t_cut > 0 ? run_tail_usage<BF16>(a, mode, s) : hipSuccess;
}

template <bool BF16>
hipError_t run_by_nb(const ScoreArgs& a, int nb, int mode, hipStream_t s) {
  if (nb <= 1) return run_softmax_sweeps<BF16, 1>(a, mode, s);
  if (nb <= 2) return run_softmax_sweeps<BF16, 2>(a, mode, s);
  if (nb <= 4) return run_softmax_sweeps<BF16, 4>(a, mode, s);
  if constexpr (BF16) {
    if (nb <= 7) return run_softmax_sweeps<BF16, 7>(a, mode, s);
    if (nb <= 8) return run_softmax_sweeps<BF16, 8>(a, mode, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_score(const ams_params* p, const Dims& d, const KvDev& k, const int32_t* seq_lens,
                        const void* q, float* u, float* g, const float* credit, VcInfo* vc, char* ws,
                        const WsLayout& wl, hipStream_t s) {
  if (vc) vc->have = false;
  ScoreArgs a;
  // with a causal window the chunk sums of the second sweep would miss the newest keys: the
  // mass kernels then form their own sums
  const bool causal = p->causal != 0 && d.W > 1;
  if (causal) vc = nullptr;
  a.t_cut = causal ? d.W - 1 : 0;
  a.vc_part = vc ? (double2*)(ws + wl.vc_part) : nullptr;
  a.credit = credit;
  a.eps = p->mass_eps;
  a.k = k;
  a.d = d;
  a.seq_lens = seq_lens;
  a.q = (const char*)q;
  a.part = (float2*)(ws + wl.part_stats);
  a.fin = (float4*)(ws + wl.fin_stats);
  a.u = u;
  a.n_chunks = wl.n_chunks;
  a.n_pad = wl.n_pad;
  a.inv_sqrt_d = (float)(1.0 / sqrt((double)d.D));
  a.c2 = (float)(1.4426950408889634 / sqrt((double)d.D));
  const bool bf16 = p->kv_dtype == AMS_BF16;
  int mode = MODE_MEAN;
  a.g = nullptr;
  if (p->scorer == AMS_SCORER_MEAN_WINDOW) a.g = (g != u) ? g : nullptr;
  if (p->scorer == AMS_SCORER_LAST_QUERY) { mode = MODE_LAST; a.g = g; }
  if (p->scorer == AMS_SCORER_EXPECTED) { mode = MODE_EXPECTED; a.g = g; }
  const int nb = wl.n_pad / 32;
  bool oneread = false;
  int vc_stride = 0, vc_tokens = 0;
  hipError_t e = hipSuccess;
  if (!causal)
    e = launch_score_oneread(p, d, k, seq_lens, q, u, g, credit, vc != nullptr, &vc_stride, &vc_tokens, ws, wl, s,
                             &oneread);
  if (e != hipSuccess) return e;
  if (!oneread) {
    e = bf16 ? run_by_nb<true>(a, nb, mode, s) : run_by_nb<false>(a, nb, mode, s);
    vc_stride = wl.n_chunks;
    vc_tokens = kScoreChunk;
  }
  if (e != hipSuccess) return e;
  if (vc) {
    vc->have = true;
    vc->stride = vc_stride;
    vc->tokens = vc_tokens;
  }
  if (p->scorer == AMS_SCORER_KEYDIFF) {
    a.g = g;
    double* ksum = (double*)(ws + wl.kbar);
    const dim3 grid(a.n_chunks, d.units), blk(kThreads);
    prof_mark("keysum", s);
    if (bf16) {
      hipLaunchKernelGGL(keysum_kernel<true>, grid, blk, 0, s, a, ksum);
      prof_mark("keydiff", s);
      hipLaunchKernelGGL(keydiff_kernel<true>, grid, blk, 0, s, a, (const double*)ksum);
    } else {
      hipLaunchKernelGGL(keysum_kernel<false>, grid, blk, 0, s, a, ksum);
      prof_mark("keydiff", s);
      hipLaunchKernelGGL(keydiff_kernel<false>, grid, blk, 0, s, a, (const double*)ksum);
    }
    e = hipGetLastError();
  }
  return e;
}

}  // namespace ams
