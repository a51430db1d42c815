// Usage u and base score g (Alg. 1 step 1; Sec. 3.2; Sec. 3.3 plug-in scorer).
//
// s[n][t] = q_n . k_t / sqrt(D) is a dense N x D by D x T contraction and runs on
// the matrix cores (32x32 MFMA tiles, token rows x query columns).  The row
// softmax needs every row's normaliser before a column can be finished, so the
// work is two sweeps over K:
//   sweep 1  per chunk of tokens, per query: running (max, sum of exp) in the
//            log2 domain, lane-local, merged per chunk          -> part_stats
//            (with the expected-attention scorers also the moment score -> g)
//   reduce   chunks merged in a fixed order                     -> (M_n, weights)
//   sweep 2  tiles recomputed, exp2(s - M_n) weighted by 1/(N Z_n) and summed
//            over the queries of each token                     -> u (and g)
// The score matrix itself never reaches memory.  The key-diversity and the
// value-weighted scorers add streaming kernels of their own at the end of the file.
#include <type_traits>

#include "score_tile.h"

namespace ams {
namespace {

// ---------------------------------------------------------------------------------------------
// Both sweeps walk a chunk of tokens (256 .. kScoreChunk, chosen on the host so that short caches
// still give the chip enough workgroups) in 32-token blocks per wave.  The keys of the next block are
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
// With five or more column blocks (bf16 caches, plain sweeps; two waves per SIMD either way) a block is
// walked as a software pipeline over its column blocks (score_tile.h: col_frags / col_mma / col_hints):
// two accumulator tiles and two sets of query fragments live instead of all accumulator tiles, the
// matrix cores and the vector ALU busy together for longer (30 % of the cycles against 17 %).  Measured
// at 224 queries per key, same machine: 1.064 + 0.938 ms for the two sweeps against 1.095 + 0.978.  With
// four column blocks it does not pay: three waves per SIMD do not fit the extra registers (and spill),
// and the two-wave moment-sum kernel is unchanged by it (0.617 ms either way).
#ifndef AMS_SCORE_PIPE_MIN_NB
#define AMS_SCORE_PIPE_MIN_NB 5
#endif
template <bool BF16, int NB, bool TAIL>
constexpr bool kPipe = BF16 && !TAIL && NB >= AMS_SCORE_PIPE_MIN_NB;

// ---------------------------------------------------------------------------------------------
// Sweep 1: per chunk, per query (max, sum exp2) of the scaled logits.
// ---------------------------------------------------------------------------------------------
//
// Causal window (App. A "Mass construction"): query w of the window sits at position T-W+w and sees
// the keys up to its own position.  The 32-token blocks that lie entirely before the newest W-1 keys
// are seen by every query and run through the plain kernels, which then stop at t_end; the few
// blocks from t_end on go through the TAIL instantiation of the same kernels (one workgroup per
// unit), where a (query, key) pair the mask hides is left out.
// Which (unit, chunk) a workgroup of the sweeps takes.  Dense caches: grid x = chunk, grid y = unit.
// Paged caches keep the rows of a position's KV heads next to each other in a slot, so there the
// heads of one (layer, sequence, chunk) are given to consecutive workgroups: they run at the same
// time and read the same slots (DRAM pages) together instead of eight separate times.
__device__ __forceinline__ void sweep_tile(const ScoreArgs& a, bool tail, bool reversed, int& unit, int& chunk) {
  int bx = blockIdx.x, by = blockIdx.y;
  if (reversed) {
    bx = gridDim.x - 1 - bx;
    by = gridDim.y - 1 - by;
  }
  if (a.k.layout != AMS_LAYOUT_PAGED || tail) {
    unit = by;
    chunk = tail ? 0 : bx;
    return;
  }
  const int lin = by * gridDim.x + bx;  // gridDim.x = chunks per unit, gridDim.y = units
  const int h = lin % a.d.H, rest = lin / a.d.H;
  chunk = rest % (int)gridDim.x;
  unit = (rest / (int)gridDim.x) * a.d.H + h;
}

__device__ __forceinline__ int causal_t_end(const ScoreArgs& a, int T) {
  return a.causal ? max(0, (T - a.d.W + 1) / 32 * 32) : T;
}

//
// MOMENTS (expected-attention score, Sec. 3.3 plug-in scorer): the log of the Gaussian moment of the
// window's queries is mean_n s + var_n s / 2 over the N logits of a token.  It needs no softmax
// statistics, so it is formed here, where few registers are live, from sums of (s - r) and (s - r)^2
// with r the token's logit against the unit's first query (a reference close to the mean keeps the
// subtraction of the squares harmless).  Raw logits are used: the causal mask does not apply.
template <bool BF16, int NB, bool TAIL, bool MOMENTS, int HD>
__global__ __launch_bounds__(kThreads, (BF16 && NB <= 4 && !MOMENTS) ? AMS_SCORE_MIN_WAVES : 2) void score_stats_kernel(ScoreArgs a) {
  constexpr int NG = kGroup<NB>, QS = Tr<BF16, HD>::kQStride;
  extern __shared__ __align__(16) char qlds[];
  __shared__ float2 xch[4][NB * 32];
  int unit, chunk;
  sweep_tile(a, TAIL, false, unit, chunk);
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T_all = seq_len(a.d, a.seq_lens, b), t_end = causal_t_end(a, T_all);
  const int T = TAIL ? T_all : t_end;
  const int c0 = TAIL ? t_end : chunk * a.chunk;
  if (c0 >= T) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, hf = lane >> 5;
  const int t_vis0 = T_all - a.d.W;  // newest key visible to the oldest query of the window
  uint4 av0[Tr<BF16, HD>::kAVecs], av1[Tr<BF16, HD>::kAVecs];
  __shared__ int32_t blk_sm[kScoreChunk / 16];
  const int32_t* blk = nullptr;  // paged caches: this chunk's block numbers, staged once
  if (a.k.layout == AMS_LAYOUT_PAGED) {
    stage_blocks(a, b, c0, min(T, c0 + a.chunk), blk_sm);
    blk = blk_sm;
  }
  if (c0 + wave * 32 < T) load_a<BF16, HD>(a, l, b, h, c0 + wave * 32, T, lane, av0, blk, c0);
  load_q<BF16, NB, HD>(a, l, b, h, qlds);
  __syncthreads();
  float m[NB], z[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    m[nb] = kNegInit;
    z[nb] = 0.f;
  }
  const float c2 = a.c2;
  float* g_row = MOMENTS ? a.g + (int64_t)unit * a.d.t_stride : nullptr;
  __shared__ float g_sm[MOMENTS ? kScoreChunk : 1];  // the chunk's moment scores, written once at the end
  auto block_of = [&](const uint4 (&av)[Tr<BF16, HD>::kAVecs], int t0, auto ragged_c) __attribute__((always_inline)) {
    constexpr bool ragged = decltype(ragged_c)::value;  // the block reaches past the end of the cache
    // the query fragments are re-read from LDS for every block: keeping them in registers across
    // blocks would cost more registers than the reads cost time, so their address is made opaque
    int qoff = 0;
    asm volatile("" : "+s"(qoff));
    float ref[16], s1[16], s2[16];
    // the vector work on one column block of logits
    auto col_moments = [&](const floatx16& acc, int nb) __attribute__((always_inline)) {
      if (nb == 0) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          // the half wave's first lane holds the logit against query 0 of the rows this lane owns
          const float r0 = __builtin_amdgcn_readlane(acc[i], 0), r1 = __builtin_amdgcn_readlane(acc[i], 32);
          ref[i] = hf ? r1 : r0;
          s1[i] = s2[i] = 0.f;
        }
      }
      const bool real = nb * 32 + (lane & 31) < a.d.N;  // padded query columns do not count
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float dlt = real ? acc[i] - ref[i] : 0.f;
        s1[i] += dlt;
        s2[i] = __builtin_fmaf(dlt, dlt, s2[i]);
      }
    };
    auto col_stats = [&](floatx16& acc, int nb) __attribute__((always_inline)) {
      if (TAIL) {
        // this column's query sees the keys up to lim (< T, so rows past the end are covered too)
        const int lim = t_vis0 + (nb * 32 + (lane & 31)) % a.d.W;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = (t0 + acc_row(i, hf) > lim) ? -INFINITY : acc[i];
      } else if (ragged) {
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = (t0 + acc_row(i, hf) >= T) ? -INFINITY : acc[i];
      }
      float mr = acc[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) mr = fmaxf(mr, acc[i]);
      const float mx = fmaxf(m[nb], mr * c2);  // c2 > 0: the maximum commutes with the scale
      float sum = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) sum += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[i], c2, -mx));
      z[nb] = __builtin_fmaf(z[nb], __builtin_amdgcn_exp2f(m[nb] - mx), sum);
      m[nb] = mx;
    };
    if constexpr (kPipe<BF16, NB, TAIL> && !ragged) {
      constexpr int NV = Tr<BF16, HD>::kAVecs;
      const char* qb = qlds + qoff + (lane & 31) * QS + (lane >> 5) * (Tr<BF16, HD>::kRowBytes / 2);
      uint4 bq[2][NV];
      floatx16 acc2[2];
      col_frags<BF16, HD>(qb, bq[0]);
      col_frags<BF16, HD>(qb + 32 * QS, bq[1]);
      __builtin_amdgcn_sched_barrier(0);
      col_mma<BF16, HD>(av, bq[0], acc2[0]);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        __builtin_amdgcn_sched_barrier(0);
        if (nb + 2 < NB) col_frags<BF16, HD>(qb + (nb + 2) * 32 * QS, bq[nb & 1]);
        if (nb + 1 < NB) col_mma<BF16, HD>(av, bq[(nb + 1) & 1], acc2[(nb + 1) & 1]);
        if (MOMENTS) col_moments(acc2[nb & 1], nb);
        col_stats(acc2[nb & 1], nb);
        if (nb + 2 < NB)
          col_hints<NV, MOMENTS ? 10 : 6, 2, true>();
        else if (nb + 1 < NB)
          col_hints<NV, MOMENTS ? 10 : 6, 2, false>();
      }
    } else {
#pragma unroll
      for (int g0 = 0; g0 < NB; g0 += NG) {
        floatx16 acc[NG];
        tile_mma<BF16, NG, HD>(av, qlds + qoff + g0 * 32 * QS, lane, acc);
        if (MOMENTS) {
#pragma unroll
          for (int k = 0; k < NG; ++k) col_moments(acc[k], g0 + k);
        }
#pragma unroll
        for (int k = 0; k < NG; ++k) col_stats(acc[k], g0 + k);
      }
    }
    if (MOMENTS) {
      const int c = lane & 31;
      float rr[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) rr[i] = c == 0 ? ref[i] : 0.f;
      const float inv_n = 1.f / (float)a.d.N;
      const float r_tok = reduce16_over32(rr, c);            // the reference of token c >> 1
      const float d_mean = reduce16_over32(s1, c) * inv_n;   // mean of s - r
      const float d_sq = reduce16_over32(s2, c) * inv_n;     // mean of (s - r)^2
      const int t = t0 + acc_row(c >> 1, hf);
      if ((c & 1) == 0 && t < T_all)
        g_sm[t - c0] = (r_tok + d_mean) * a.inv_sqrt_d + 0.5f * (d_sq - d_mean * d_mean) * (a.inv_sqrt_d * a.inv_sqrt_d);
    }
  };
  auto block = [&](const uint4 (&av)[Tr<BF16, HD>::kAVecs], int t0) __attribute__((always_inline)) {
    if (t0 + 32 > T)
      block_of(av, t0, std::true_type{});
    else
      block_of(av, t0, std::false_type{});
  };
  // this wave's blocks: every fourth block of 32 tokens up to the end of the chunk (or of the cache)
  const int t_lim = min(T, c0 + a.chunk);
#pragma unroll 1
  for (int t0 = c0 + wave * 32; t0 < t_lim; t0 += 256) {
    if (t0 + 128 < t_lim) load_a<BF16, HD>(a, l, b, h, t0 + 128, T, lane, av1, blk, c0);
    block(av0, t0);
    if (t0 + 128 >= t_lim) break;
    if (t0 + 256 < t_lim) load_a<BF16, HD>(a, l, b, h, t0 + 256, T, lane, av0, blk, c0);
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
  if (MOMENTS)
    for (int t = c0 + threadIdx.x; t < t_lim; t += kThreads) g_row[t] = g_sm[t - c0];
  for (int n = threadIdx.x; n < NB * 32; n += kThreads) {
    float M = kNegInit;
#pragma unroll
    for (int w = 0; w < 4; ++w) M = fmaxf(M, xch[w][n].x);
    float Z = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) Z += xch[w][n].y * __builtin_amdgcn_exp2f(xch[w][n].x - M);
    // the tail's entry follows those of the chunks
    const int slot = TAIL ? (t_end + a.chunk - 1) / a.chunk : chunk;
    a.part[((int64_t)unit * (a.n_chunks + 1) + slot) * a.n_pad + n] = make_float2(M, Z);
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
  if (unit == 0 && threadIdx.x == 0 && a.status) *a.status = 0;  // no bounded wait on this path
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T = seq_len(a.d, a.seq_lens, b);
  const int nch = (causal_t_end(a, T) + a.chunk - 1) / a.chunk + (a.causal ? 1 : 0);
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
  if ((int)threadIdx.x < a.n_pad) {
    float M = kNegInit;
    for (int q = 0; q < parts; ++q) M = fmaxf(M, pm[q * a.n_pad + n]);
    double Z = 0.0;
    for (int q = 0; q < parts; ++q) Z += pz[q * a.n_pad + n] * (double)__builtin_amdgcn_exp2f(pm[q * a.n_pad + n] - M);
    const bool real = n < a.d.N;
    // causal window on a cache shorter than the window: a query before position 0 does not exist
    const bool exists = real && (!a.causal || T - a.d.W + (n % a.d.W) >= 0);
    const bool newest = exists && (n % a.d.W) == a.d.W - 1;
    float4 f;
    f.x = M;
    f.y = exists ? (float)(1.0 / ((double)a.d.N * Z)) : 0.f;
    f.z = newest ? (float)(1.0 / ((double)a.d.G * Z)) : 0.f;
    f.w = real ? 1.f : 0.f;
    a.fin[(int64_t)unit * a.n_pad + n] = f;
  }
  if (a.csum) {  // sum of the credit before the update (for the EMA normaliser), strided partials in a fixed tree
    __shared__ double cs[kReduceThreads / 64];
    const float* c_row = a.credit + (int64_t)unit * a.d.t_stride;
    double c = 0.0;
    if ((a.d.t_stride & 3) == 0 && ((uintptr_t)a.credit & 15) == 0) {  // 16-byte loads, several in flight
      const float4* c4 = (const float4*)c_row;
      const int n4 = T >> 2;
#pragma unroll 8
      for (int q = threadIdx.x; q < n4; q += kReduceThreads) {
        const float4 v = c4[q];
        c += ((double)v.x + (double)v.y) + ((double)v.z + (double)v.w);
      }
      for (int t = (n4 << 2) + threadIdx.x; t < T; t += kReduceThreads) c += (double)c_row[t];
    } else {
      for (int t = threadIdx.x; t < T; t += kReduceThreads) c += (double)c_row[t];
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) c += __shfl_xor(c, o);
    if ((threadIdx.x & 63) == 0) cs[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) {
      double t = 0.0;
      for (int w = 0; w < kReduceThreads / 64; ++w) t += cs[w];
      a.csum[unit] = t;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Sweep 2: u[t] = sum_n exp2(x[n][t] - M_n) / (N Z_n), and g for the softmax-based scorers.
// ---------------------------------------------------------------------------------------------
// TAIL (causal window, blocks from t_end on): a (query, key) pair the mask hides adds nothing, and
// every observation a key is missing counts as the largest share it got.
template <bool BF16, int NB, int MODE, bool TAIL, int HD>
__global__ __launch_bounds__(kThreads, (BF16 && NB <= 4) ? AMS_SCORE_MIN_WAVES : 2) void score_usage_kernel(ScoreArgs a) {
  constexpr int NG = kGroup<NB>;
  constexpr int QS = Tr<BF16, HD>::kQStride;
  extern __shared__ __align__(16) char qlds[];
  // the second sweep walks the cache backwards: what the first sweep read last is still in the
  // memory-side cache (about a tenth of the keys at the headline size)
  int unit, chunk;
  sweep_tile(a, TAIL, true, unit, chunk);
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T_all = seq_len(a.d, a.seq_lens, b), t_end = causal_t_end(a, T_all);
  const int T = TAIL ? T_all : t_end;
  const int c0 = TAIL ? t_end : chunk * a.chunk;
  if (c0 >= T) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, hf = lane >> 5, c = lane & 31;
  const int t_vis0 = T_all - a.d.W;  // newest key visible to the oldest query of the window
  uint4 av0[Tr<BF16, HD>::kAVecs], av1[Tr<BF16, HD>::kAVecs];
  __shared__ int32_t blk_sm[kScoreChunk / 16];
  const int32_t* blk = nullptr;  // paged caches: this chunk's block numbers, staged once
  if (a.k.layout == AMS_LAYOUT_PAGED) {
    stage_blocks(a, b, c0, min(T, c0 + a.chunk), blk_sm);
    blk = blk_sm;
  }
  if (c0 + wave * 32 < T) load_a<BF16, HD>(a, l, b, h, c0 + wave * 32, T, lane, av0, blk, c0);
  load_q<BF16, NB, HD>(a, l, b, h, qlds);
  __syncthreads();
  float4 f[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) f[nb] = a.fin[(int64_t)unit * a.n_pad + nb * 32 + c];
  float* u_row = a.u + (int64_t)unit * a.d.t_stride;
  float* g_row = a.g ? a.g + (int64_t)unit * a.d.t_stride : nullptr;
  const float c2 = a.c2;
  // u (and the last-query g) of the chunk are collected in LDS and written once at the end: stores
  // scattered through the sweep cost the key stream 7 % of its rate
  constexpr bool kBufG = MODE == MODE_LAST && NB <= 7;  // (8 column blocks: LDS is needed for the query window)
  __shared__ float u_sm[kScoreChunk];
  __shared__ float g_sm[kBufG ? kScoreChunk : 1];
  float v_part = 0.f;  // this lane's share of sum(max(u,0)+eps): one term per block of 32 keys of this wave (32 blocks per chunk)
  auto block = [&](const uint4 (&av)[Tr<BF16, HD>::kAVecs], int t0) __attribute__((always_inline)) {
    float pu[16], pg[16], pm[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) pu[i] = pg[i] = pm[i] = 0.f;
    float rg = 0.f;
    constexpr bool masked = TAIL;
    int qoff = 0;  // see the first sweep: the query fragments are re-read per block on purpose
    asm volatile("" : "+s"(qoff));
    auto col_usage = [&](const floatx16& acc, int nb) __attribute__((always_inline)) {
      if (masked) {
        const int lim = t_vis0 + (nb * 32 + c) % a.d.W;  // newest key this column's query sees
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[i], c2, -f[nb].x));
          const bool sees = t0 + acc_row(i, hf) <= lim;
          const float share = sees ? f[nb].y * e : 0.f;
          pu[i] += share;
          pm[i] = fmaxf(pm[i], share);
          if (MODE == MODE_LAST) pg[i] += sees ? f[nb].z * e : 0.f;
        }
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[i], c2, -f[nb].x));
          pu[i] = __builtin_fmaf(f[nb].y, e, pu[i]);
          if (MODE == MODE_LAST) pg[i] = __builtin_fmaf(f[nb].z, e, pg[i]);
        }
      }
    };
    if constexpr (kPipe<BF16, NB, TAIL>) {
      constexpr int NV = Tr<BF16, HD>::kAVecs;
      const char* qb = qlds + qoff + (lane & 31) * QS + (lane >> 5) * (Tr<BF16, HD>::kRowBytes / 2);
      uint4 bq[2][NV];
      floatx16 acc2[2];
      col_frags<BF16, HD>(qb, bq[0]);
      col_frags<BF16, HD>(qb + 32 * QS, bq[1]);
      __builtin_amdgcn_sched_barrier(0);
      col_mma<BF16, HD>(av, bq[0], acc2[0]);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        __builtin_amdgcn_sched_barrier(0);
        if (nb + 2 < NB) col_frags<BF16, HD>(qb + (nb + 2) * 32 * QS, bq[nb & 1]);
        if (nb + 1 < NB) col_mma<BF16, HD>(av, bq[(nb + 1) & 1], acc2[(nb + 1) & 1]);
        col_usage(acc2[nb & 1], nb);
        if (nb + 2 < NB)
          col_hints<NV, MODE == MODE_LAST ? 6 : 4, 2, true>();
        else if (nb + 1 < NB)
          col_hints<NV, MODE == MODE_LAST ? 6 : 4, 2, false>();
      }
    } else {
#pragma unroll
      for (int g0 = 0; g0 < NB; g0 += NG) {
        floatx16 acc[NG];
        tile_mma<BF16, NG, HD>(av, qlds + qoff + g0 * 32 * QS, lane, acc);
#pragma unroll
        for (int k = 0; k < NG; ++k) col_usage(acc[k], g0 + k);
      }
    }
    const int t = t0 + acc_row(c >> 1, hf);
    float ru = reduce16_over32(pu, c);
    if (masked) {
      const int seen = a.d.G * min(a.d.W, T - t);  // (head, query) pairs that see key t
      ru += (float)(a.d.N - seen) * reduce16_over32<true>(pm, c);
    }
    if (MODE == MODE_MEAN) rg = ru;
    if (MODE == MODE_LAST) rg = reduce16_over32(pg, c);
    if ((c & 1) == 0 && t < T) {
      u_sm[t - c0] = ru;
      if (kBufG)
        g_sm[t - c0] = rg;
      else if (g_row)
        g_row[t] = rg;
      v_part += fmaxf(ru, 0.f) + a.eps;
    }
  };
  // this wave's blocks: every fourth block of 32 tokens up to the end of the chunk (or of the cache)
  const int t_lim = min(T, c0 + a.chunk);
#pragma unroll 1
  for (int t0 = c0 + wave * 32; t0 < t_lim; t0 += 256) {
    if (t0 + 128 < t_lim) load_a<BF16, HD>(a, l, b, h, t0 + 128, T, lane, av1, blk, c0);
    block(av0, t0);
    if (t0 + 128 >= t_lim) break;
    if (t0 + 256 < t_lim) load_a<BF16, HD>(a, l, b, h, t0 + 256, T, lane, av0, blk, c0);
    block(av1, t0 + 128);
  }
  __syncthreads();
  for (int t = c0 + threadIdx.x; t < t_lim; t += kThreads) {
    u_row[t] = u_sm[t - c0];
    if (kBufG) g_row[t] = g_sm[t - c0];
  }
  if (a.vc_part) {  // chunk sums of max(u,0)+eps in a fixed order: lanes, then waves
    __shared__ double vc_sm[4];
    double v_acc = (double)v_part;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v_acc += __shfl_xor(v_acc, o);
    if (lane == 0) vc_sm[wave] = v_acc;
    __syncthreads();
    if (threadIdx.x == 0) {
      // the unit's credit sum (formed between the sweeps) rides in the first chunk's entry
      const double c = (chunk == 0 && a.csum) ? a.csum[unit] : 0.0;
      a.vc_part[(int64_t)unit * a.n_chunks + chunk] = make_double2((vc_sm[0] + vc_sm[1]) + (vc_sm[2] + vc_sm[3]), c);
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

// partial key sums per chunk: ksum[unit][chunk][D] (double).  NORMALIZE: every key is divided by its
// length first (the redundancy-aware score needs the sum of the unit vectors; a zero key adds nothing).
template <bool BF16, int HD, bool NORMALIZE>
__global__ __launch_bounds__(kThreads) void keysum_kernel(ScoreArgs a, double* ksum) {
  constexpr int CPR = Tr<BF16, HD>::kRowBytes / 16, EPC = BF16 ? 8 : 4, RPI = kThreads / CPR;
  __shared__ double sm[kThreads][EPC];
  const int unit = blockIdx.y, chunk = blockIdx.x;
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T = seq_len(a.d, a.seq_lens, b);
  const int c0 = chunk * a.chunk;
  if (c0 >= T) return;
  const int col = threadIdx.x % CPR, r0 = threadIdx.x / CPR;
  double s[EPC];
#pragma unroll
  for (int e = 0; e < EPC; ++e) s[e] = 0.0;
  // four rows per lane in flight (a row past the end re-reads the last one and is not added)
  constexpr int kRows = 4;
  const int t_end = min(T, c0 + a.chunk);
  for (int tb = c0 + r0; tb < t_end; tb += kRows * RPI) {
    uint4 v[kRows];
#pragma unroll
    for (int j = 0; j < kRows; ++j)
      v[j] = *(const uint4*)(kv_row(a.k, l, b, h, min(tb + j * RPI, T - 1)) + col * 16);
#pragma unroll
    for (int j = 0; j < kRows; ++j) {
      float x[8];
      int n;
      widen8<BF16>(v[j], x, n);
      double scale = 1.0;
      if (NORMALIZE) {  // the CPR lanes of a row are consecutive lanes of one wave
        float n2 = 0.f;
#pragma unroll
        for (int e = 0; e < EPC; ++e) n2 = __builtin_fmaf(x[e], x[e], n2);
#pragma unroll
        for (int o = CPR / 2; o >= 1; o >>= 1) n2 += __shfl_xor(n2, o);
        scale = n2 > 0.f ? 1.0 / sqrt((double)n2) : 0.0;
      }
      if (tb + j * RPI < t_end) {
#pragma unroll
        for (int e = 0; e < EPC; ++e) s[e] += (double)x[e] * scale;
      }
    }
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

// MEAN_COS = false: g[t] = -cos(k_t, mean key).  MEAN_COS = true (ksum holds sums of unit vectors):
// g[t] = mean over s != t of cos(k_t, k_s) = (k_t / |k_t| . sum of unit vectors - 1) / (T - 1).
template <bool BF16, int HD, bool MEAN_COS>
__global__ __launch_bounds__(kThreads) void keydiff_kernel(ScoreArgs a, const double* ksum) {
  constexpr int CPR = Tr<BF16, HD>::kRowBytes / 16, EPC = BF16 ? 8 : 4, RPI = kThreads / CPR;
  __shared__ double kbar[128];
  __shared__ double kbar_norm;
  __shared__ float2 row_sums[kScoreChunk];  // per token: k . kbar and k . k
  const int unit = blockIdx.y, chunk = blockIdx.x;
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T = seq_len(a.d, a.seq_lens, b);
  const int c0 = chunk * a.chunk;
  if (c0 >= T) return;
  const int nch = (T + a.chunk - 1) / a.chunk;
  if ((int)threadIdx.x < a.d.D) {
    double t = 0.0;
    for (int c = 0; c < nch; ++c) t += ksum[((int64_t)unit * a.n_chunks + c) * a.d.D + threadIdx.x];
    kbar[threadIdx.x] = MEAN_COS ? t : t / (double)T;
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
  float kb[EPC];  // this lane's channels of the mean key
#pragma unroll
  for (int e = 0; e < EPC; ++e) kb[e] = (float)kbar[col * EPC + e];
  // four rows per lane in flight: the loads are unconditional (a row past the end re-reads the last one)
  constexpr int kRows = 4;
  const int t_end = min(T, c0 + a.chunk);
  for (int tb = c0; tb < t_end; tb += kRows * RPI) {
    uint4 v[kRows];
#pragma unroll
    for (int j = 0; j < kRows; ++j)
      v[j] = *(const uint4*)(kv_row(a.k, l, b, h, min(tb + j * RPI + r0, T - 1)) + col * 16);
#pragma unroll
    for (int j = 0; j < kRows; ++j) {
      const int t = tb + j * RPI + r0;
      // a row's 128 products are summed in fp32 (8 per lane, then 16 or 32 lanes); the ratio is formed in double
      float dot = 0.f, nk = 0.f;
      float x[8];
      int n;
      widen8<BF16>(v[j], x, n);
#pragma unroll
      for (int e = 0; e < EPC; ++e) {
        dot = __builtin_fmaf(x[e], kb[e], dot);
        nk = __builtin_fmaf(x[e], x[e], nk);
      }
      // the CPR lanes of a row are consecutive lanes of one wave
#pragma unroll
      for (int o = CPR / 2; o >= 1; o >>= 1) {
        dot += __shfl_xor(dot, o);
        nk += __shfl_xor(nk, o);
      }
      if (col == 0 && t < t_end) row_sums[t - c0] = make_float2(dot, nk);
    }
  }
  __syncthreads();
  // one token per thread for the ratio, so that every lane works
  for (int t = c0 + threadIdx.x; t < min(T, c0 + a.chunk); t += kThreads) {
    const float2 r = row_sums[t - c0];
    if (MEAN_COS) {
      g_row[t] = (r.y > 0.f && T > 1) ? (float)(((double)r.x / sqrt((double)r.y) - 1.0) / (double)(T - 1)) : 0.f;
    } else {
      const double den = sqrt((double)r.y) * kbar_norm;
      g_row[t] = den > 0.0 ? (float)(-(double)r.x / den) : 0.f;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Value-weighted expected attention (Sec. 3.3 plug-in scorer): the log-moment scores e left in g by
// the second sweep become p = softmax over the cache, and g[t] = (p[t] + eps) * ||v_t||.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void esoftmax_part_kernel(ScoreArgs a, double2* part) {
  __shared__ double2 sm[4];
  const int unit = blockIdx.y, chunk = blockIdx.x;
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T = seq_len(a.d, a.seq_lens, b);
  const int c0 = chunk * a.chunk;
  if (c0 >= T) return;
  const float* e = a.g + (int64_t)unit * a.d.t_stride;
  const int end = min(T, c0 + a.chunk);
  double m = -INFINITY, z = 0.0;
  for (int t = c0 + threadIdx.x; t < end; t += kThreads) {
    const double x = (double)e[t];
    const double mx = fmax(m, x);
    z = z * exp(m - mx) + exp(x - mx);
    m = mx;
  }
  // lanes, then waves, each in a fixed order; an empty partial is (-inf, 0)
  auto merge = [](double& m1, double& z1, double m2, double z2) __attribute__((always_inline)) {
    const double mx = fmax(m1, m2);
    if (mx == -INFINITY) return;
    z1 = z1 * exp(m1 - mx) + z2 * exp(m2 - mx);
    m1 = mx;
  };
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const double m2 = __shfl_xor(m, o), z2 = __shfl_xor(z, o);
    // both partners must arrive at the same value: combine in lane order
    double ml = (threadIdx.x & o) ? m2 : m, zl = (threadIdx.x & o) ? z2 : z;
    const double mh = (threadIdx.x & o) ? m : m2, zh = (threadIdx.x & o) ? z : z2;
    merge(ml, zl, mh, zh);
    m = ml;
    z = zl;
  }
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = make_double2(m, z);
  __syncthreads();
  if (threadIdx.x == 0) {
    double M = sm[0].x, Z = sm[0].y;
    for (int w = 1; w < 4; ++w) merge(M, Z, sm[w].x, sm[w].y);
    part[(int64_t)unit * a.n_chunks + chunk] = make_double2(M, Z);
  }
}

template <bool BF16, int HD>
__global__ __launch_bounds__(kThreads) void vweight_kernel(ScoreArgs a, KvDev v, const double2* part, float eps_f) {
  constexpr int CPR = Tr<BF16, HD>::kRowBytes / 16, EPC = BF16 ? 8 : 4, RPI = kThreads / CPR;
  __shared__ double2 stat;
  __shared__ float norm2[kScoreChunk];  // per token: v . v
  const int unit = blockIdx.y, chunk = blockIdx.x;
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T = seq_len(a.d, a.seq_lens, b);
  const int c0 = chunk * a.chunk;
  if (c0 >= T) return;
  if (threadIdx.x == 0) {  // chunk statistics merged in index order
    const int nch = (T + a.chunk - 1) / a.chunk;
    double M = -INFINITY;
    for (int c = 0; c < nch; ++c) M = fmax(M, part[(int64_t)unit * a.n_chunks + c].x);
    double Z = 0.0;
    for (int c = 0; c < nch; ++c) {
      const double2 s = part[(int64_t)unit * a.n_chunks + c];
      Z += s.y * exp(s.x - M);
    }
    stat = make_double2(M, Z);
  }
  __syncthreads();
  const double M = stat.x, inv_z = 1.0 / stat.y, eps = (double)eps_f;
  const int col = threadIdx.x % CPR, r0 = threadIdx.x / CPR;
  float* g_row = a.g + (int64_t)unit * a.d.t_stride;
  for (int tb = c0; tb < min(T, c0 + a.chunk); tb += RPI) {
    const int t = tb + r0;
    float n2 = 0.f;  // 128 squares summed in fp32, the rest in double
    if (t < T) {
      const uint4 x4 = *(const uint4*)(kv_row(v, l, b, h, t) + col * 16);
      float x[8];
      int n;
      widen8<BF16>(x4, x, n);
#pragma unroll
      for (int e = 0; e < EPC; ++e) n2 = __builtin_fmaf(x[e], x[e], n2);
    }
    // the CPR lanes of a row are consecutive lanes of one wave
#pragma unroll
    for (int o = CPR / 2; o >= 1; o >>= 1) n2 += __shfl_xor(n2, o);
    if (col == 0 && t < T) norm2[t - c0] = n2;
  }
  __syncthreads();
  // one token per thread for the exponential, so that every lane works
  for (int t = c0 + threadIdx.x; t < min(T, c0 + a.chunk); t += kThreads)
    g_row[t] = (float)((exp((double)g_row[t] - M) * inv_z + eps) * sqrt((double)norm2[t - c0]));
}

template <bool BF16, int NB, bool TAIL, int HD>
hipError_t launch_stats(const ScoreArgs& a, bool moments, dim3 grid, int lds, hipStream_t s) {
  hipError_t e;
  if (moments) {
    if ((e = ensure_lds<score_stats_kernel<BF16, NB, TAIL, true, HD>>(lds)) != hipSuccess) return e;
    hipLaunchKernelGGL((score_stats_kernel<BF16, NB, TAIL, true, HD>), grid, dim3(kThreads), lds, s, a);
  } else {
    if ((e = ensure_lds<score_stats_kernel<BF16, NB, TAIL, false, HD>>(lds)) != hipSuccess) return e;
    hipLaunchKernelGGL((score_stats_kernel<BF16, NB, TAIL, false, HD>), grid, dim3(kThreads), lds, s, a);
  }
  return hipGetLastError();
}

template <bool BF16, int NB, bool TAIL, int HD>
hipError_t launch_usage(const ScoreArgs& a, int mode, dim3 grid, int lds, hipStream_t s) {
  const dim3 blk(kThreads);
  hipError_t e;
  switch (mode) {
    case MODE_LAST:
      if ((e = ensure_lds<score_usage_kernel<BF16, NB, MODE_LAST, TAIL, HD>>(lds)) != hipSuccess) return e;
      hipLaunchKernelGGL((score_usage_kernel<BF16, NB, MODE_LAST, TAIL, HD>), grid, blk, lds, s, a);
      break;
    default:
      if ((e = ensure_lds<score_usage_kernel<BF16, NB, MODE_MEAN, TAIL, HD>>(lds)) != hipSuccess) return e;
      hipLaunchKernelGGL((score_usage_kernel<BF16, NB, MODE_MEAN, TAIL, HD>), grid, blk, lds, s, a);
  }
  return hipGetLastError();
}

template <bool BF16, int NB, int HD>
hipError_t run_softmax_sweeps(const ScoreArgs& a, int mode, hipStream_t s) {
  const int lds = NB * 32 * Tr<BF16, HD>::kQStride;
  const dim3 grid(a.n_chunks, a.d.units);
  hipError_t e;
  prof_mark("score_stats", s);
  if ((e = launch_stats<BF16, NB, false, HD>(a, mode == MODE_EXPECTED, grid, lds, s)) != hipSuccess) return e;
  if (a.causal) {
    prof_mark("score_stats_tail", s);
    if ((e = launch_stats<BF16, NB, true, HD>(a, mode == MODE_EXPECTED, dim3(1, a.d.units), lds, s)) != hipSuccess) return e;
  }
  prof_mark("score_reduce", s);
  hipLaunchKernelGGL(score_reduce_kernel, dim3(a.d.units), dim3(kReduceThreads), 0, s, a);
  // the moment-based score has been written by the first sweep: the second one leaves g alone
  ScoreArgs a2 = a;
  if (mode == MODE_EXPECTED) a2.g = nullptr;
  prof_mark("score_usage", s);
  if ((e = launch_usage<BF16, NB, false, HD>(a2, mode, grid, lds, s)) != hipSuccess) return e;
  if (a.causal) {
    prof_mark("score_usage_tail", s);
    if ((e = launch_usage<BF16, NB, true, HD>(a2, mode, dim3(1, a.d.units), lds, s)) != hipSuccess) return e;
  }
  return hipSuccess;
}

template <bool BF16, int HD>
hipError_t run_by_nb(const ScoreArgs& a, int nb, int mode, hipStream_t s) {
  if (nb <= 1) return run_softmax_sweeps<BF16, 1, HD>(a, mode, s);
  if (nb <= 2) return run_softmax_sweeps<BF16, 2, HD>(a, mode, s);
  if (nb <= 4) return run_softmax_sweeps<BF16, 4, HD>(a, mode, s);
  if constexpr (BF16) {
    if (nb <= 7) return run_softmax_sweeps<BF16, 7, HD>(a, mode, s);
    if (nb <= 8) return run_softmax_sweeps<BF16, 8, HD>(a, mode, s);
  }
  return hipErrorInvalidValue;
}

template <bool BF16, int HD>
hipError_t launch_vweight(const ScoreArgs& a, const KvDev& v, char* ws, const WsLayout& wl, float eps, hipStream_t s) {
  hipLaunchKernelGGL((vweight_kernel<BF16, HD>), dim3(a.n_chunks, a.d.units), dim3(kThreads), 0, s, a, v,
                     (const double2*)(ws + wl.kbar), eps);
  return hipGetLastError();
}

template <bool BF16, int HD>
hipError_t launch_keydiff(const ScoreArgs& a, char* ws, const WsLayout& wl, hipStream_t s) {
  double* ksum = (double*)(ws + wl.kbar);
  const dim3 grid(a.n_chunks, a.d.units), blk(kThreads);
  prof_mark("keysum", s);
  hipLaunchKernelGGL((keysum_kernel<BF16, HD, false>), grid, blk, 0, s, a, ksum);
  prof_mark("keydiff", s);
  hipLaunchKernelGGL((keydiff_kernel<BF16, HD, false>), grid, blk, 0, s, a, (const double*)ksum);
  return hipGetLastError();
}

// Redundancy-aware score (Sec. 4 "Universality across diverse base scorers"): the mean cosine similarity of
// every key to the other keys of its unit (two streams of K: the sum of the unit vectors, then one dot product
// per key), its softmax over the cache, and g = lambda * (pooled) usage - (1 - lambda) * that softmax.
__global__ __launch_bounds__(kThreads) void redundancy_combine_kernel(ScoreArgs a, const double2* part, float mix_lambda,
                                                                       int pool_r) {
  __shared__ double2 stat;
  const int unit = blockIdx.y, chunk = blockIdx.x;
  int l, b, h;
  unit_coords(a.d, unit, l, b, h);
  const int T = seq_len(a.d, a.seq_lens, b);
  const int c0 = chunk * a.chunk;
  if (c0 >= T) return;
  if (threadIdx.x == 0) {  // chunk statistics of the similarities merged in index order
    const int nch = (T + a.chunk - 1) / a.chunk;
    double M = -INFINITY;
    for (int c = 0; c < nch; ++c) M = fmax(M, part[(int64_t)unit * a.n_chunks + c].x);
    double Z = 0.0;
    for (int c = 0; c < nch; ++c) {
      const double2 s = part[(int64_t)unit * a.n_chunks + c];
      Z += s.y * exp(s.x - M);
    }
    stat = make_double2(M, Z);
  }
  __syncthreads();
  const double M = stat.x, inv_z = 1.0 / stat.y, lam = (double)mix_lambda;
  const float* u_row = a.u + (int64_t)unit * a.d.t_stride;
  float* g_row = a.g + (int64_t)unit * a.d.t_stride;
  for (int t = c0 + threadIdx.x; t < min(T, c0 + a.chunk); t += kThreads) {
    float imp = u_row[t];
    if (pool_r > 0) {  // the mean of u over the positions t - r .. t + r that exist, stored as fp32
      const int lo = max(0, t - pool_r), hi = min(T - 1, t + pool_r);
      double sum = 0.0;
      for (int j = lo; j <= hi; ++j) sum += (double)u_row[j];
      imp = (float)(sum / (double)(hi - lo + 1));
    }
    g_row[t] = (float)(lam * (double)imp - (1.0 - lam) * (exp((double)g_row[t] - M) * inv_z));
  }
}

template <bool BF16, int HD>
hipError_t launch_redundancy(const ScoreArgs& a, char* ws, const WsLayout& wl, float mix_lambda, int kernel, hipStream_t s) {
  double* ksum = (double*)(ws + wl.kbar);
  const dim3 grid(a.n_chunks, a.d.units), blk(kThreads);
  prof_mark("khat_sum", s);
  hipLaunchKernelGGL((keysum_kernel<BF16, HD, true>), grid, blk, 0, s, a, ksum);
  prof_mark("mean_cos", s);
  hipLaunchKernelGGL((keydiff_kernel<BF16, HD, true>), grid, blk, 0, s, a, (const double*)ksum);
  prof_mark("esoftmax_part", s);  // the chunk statistics take the place of the key sums, which are used up
  hipLaunchKernelGGL(esoftmax_part_kernel, grid, blk, 0, s, a, (double2*)(ws + wl.kbar));
  prof_mark("redundancy_combine", s);
  hipLaunchKernelGGL(redundancy_combine_kernel, grid, blk, 0, s, a, (const double2*)(ws + wl.kbar), mix_lambda,
                     kernel > 1 ? kernel / 2 : 0);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_score(const ams_params* p, const Dims& d, const KvDev& k, const KvDev* v,
                        const int32_t* seq_lens,
                        const void* q, float* u, float* g, const float* credit, VcInfo* vc, char* ws,
                        const WsLayout& wl, hipStream_t s) {
  if (vc) vc->have = false;
  ScoreArgs a;
  const bool causal = p->causal != 0 && d.W > 1;  // a window of one query sees everything anyway
  a.causal = causal;
  // the chunk sums of the second sweep would miss the tail blocks: the mass kernels form their own
  if (causal) vc = nullptr;
  a.vc_part = vc ? (double2*)(ws + wl.vc_part) : nullptr;
  a.credit = credit;
  a.csum = (vc && credit) ? (double*)(ws + wl.csum) : nullptr;
  a.eps = p->mass_eps;
  a.k = k;
  a.d = d;
  a.seq_lens = seq_lens;
  a.q = (const char*)q;
  a.part = (float2*)(ws + wl.part_stats);
  a.fin = (float4*)(ws + wl.fin_stats);
  a.status = park_status_word(ws, wl);
  a.u = u;
  const bool paged = k.layout != AMS_LAYOUT_DENSE;
  a.n_chunks = paged ? wl.n_chunks_paged : wl.n_chunks;
  a.chunk = paged ? wl.score_chunk_paged : wl.score_chunk;
  a.n_pad = wl.n_pad;
  a.inv_sqrt_d = (float)(1.0 / sqrt((double)d.D));
  a.c2 = (float)(1.4426950408889634 / sqrt((double)d.D));
  const bool bf16 = p->kv_dtype == AMS_BF16;
  int mode = MODE_MEAN;
  a.g = nullptr;
  if (p->scorer == AMS_SCORER_MEAN_WINDOW) a.g = (g != u) ? g : nullptr;
  if (p->scorer == AMS_SCORER_LAST_QUERY) { mode = MODE_LAST; a.g = g; }
  const bool vnorm = p->scorer == AMS_SCORER_EXPECTED_VNORM;
  if (vnorm && !v) return hipErrorInvalidValue;
  if (p->scorer == AMS_SCORER_EXPECTED || vnorm) { mode = MODE_EXPECTED; a.g = g; }
  const int nb = wl.n_pad / 32;
  bool oneread = false;
  int vc_stride = 0, vc_tokens = 0;
  hipError_t e = hipSuccess;
  // AMS_SCORE_PATH_AUTO: the two sweeps, which are the faster of the two on every workload measured so far
  if (p->score_path == AMS_SCORE_PATH_ONE_READ)
    e = launch_score_oneread(p, d, k, seq_lens, q, u, g, credit, vc != nullptr, &vc_stride, &vc_tokens, ws, wl, s,
                             &oneread);
  if (e != hipSuccess) return e;
  if (!oneread && p->score_path == AMS_SCORE_PATH_ONE_READ) return hipErrorNotSupported;
  if (!oneread) {
    // short caches with enough units to fill the chip: one workgroup per unit, one launch
    const bool want_unit = p->score_path == AMS_SCORE_PATH_ONE_LAUNCH ||
                           (p->score_path == AMS_SCORE_PATH_AUTO && d.units >= kUnitScorerMinUnits);
    if (want_unit) {
      e = launch_score_unit(a, bf16, d.D, mode, s, &oneread);
      if (e != hipSuccess) return e;
      vc_stride = 1;
      vc_tokens = kScoreChunk;
    }
    if (!oneread && p->score_path == AMS_SCORE_PATH_ONE_LAUNCH) return hipErrorNotSupported;
  }
  if (!oneread) {
    if (d.D == 64)
      e = bf16 ? run_by_nb<true, 64>(a, nb, mode, s) : run_by_nb<false, 64>(a, nb, mode, s);
    else
      e = bf16 ? run_by_nb<true, 128>(a, nb, mode, s) : run_by_nb<false, 128>(a, nb, mode, s);
    vc_stride = a.n_chunks;
    vc_tokens = a.chunk;
  }
  if (e != hipSuccess) return e;
  if (vc) {
    vc->have = true;
    vc->stride = vc_stride;
    vc->tokens = vc_tokens;
  }
  if (vnorm) {
    prof_mark("esoftmax_part", s);
    hipLaunchKernelGGL(esoftmax_part_kernel, dim3(a.n_chunks, d.units), dim3(kThreads), 0, s, a,
                       (double2*)(ws + wl.kbar));
    prof_mark("vweight", s);
    if (d.D == 64)
      e = bf16 ? launch_vweight<true, 64>(a, *v, ws, wl, p->vnorm_eps, s) : launch_vweight<false, 64>(a, *v, ws, wl, p->vnorm_eps, s);
    else
      e = bf16 ? launch_vweight<true, 128>(a, *v, ws, wl, p->vnorm_eps, s) : launch_vweight<false, 128>(a, *v, ws, wl, p->vnorm_eps, s);
  }
  if (p->scorer == AMS_SCORER_REDUNDANCY) {
    a.g = g;
    if (d.D == 64)
      e = bf16 ? launch_redundancy<true, 64>(a, ws, wl, p->mix_lambda, p->score_kernel, s)
               : launch_redundancy<false, 64>(a, ws, wl, p->mix_lambda, p->score_kernel, s);
    else
      e = bf16 ? launch_redundancy<true, 128>(a, ws, wl, p->mix_lambda, p->score_kernel, s)
               : launch_redundancy<false, 128>(a, ws, wl, p->mix_lambda, p->score_kernel, s);
  }
  if (p->scorer == AMS_SCORER_KEYDIFF) {
    a.g = g;
    if (d.D == 64)
      e = bf16 ? launch_keydiff<true, 64>(a, ws, wl, s) : launch_keydiff<false, 64>(a, ws, wl, s);
    else
      e = bf16 ? launch_keydiff<true, 128>(a, ws, wl, s) : launch_keydiff<false, 128>(a, ws, wl, s);
  }
  return e;
}

}  // namespace ams
