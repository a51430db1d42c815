// One-sweep scorer: usage u (and g) with K read from HBM exactly once
// (Alg. 1 step 1; Sec. 3.2; Sec. 3.3 plug-in scorer).
//
// u[t] = (1/N) sum_n exp(s[n][t] - M_n) / Z_n needs the softmax normaliser of every query over
// ALL tokens of the unit before any token can be finished.  Instead of sweeping K twice, every
// workgroup keeps its 256-token x N-query tile of exp2(s - m_tile) in registers (128 per lane),
// publishes the tile's per-query (max, sum), waits until the unit's normalisers are known, and
// then finishes its tokens from registers.  The kernel is persistent and launched cooperatively,
// so every workgroup is resident; tiles are taken in increasing order (tile = block + k * grid)
// and a unit never has more tiles than the grid has workgroups, which makes the wait free of
// deadlock: the workgroups a tile waits for are resident and never wait for a later unit.
//
// Per unit: `counter` counts published tiles; the workgroup that brings it to the tile count
// merges the statistics in ascending tile order (deterministic), stores the per-query
// (M_n, 1/(N Z_n), last-query weight) and raises `flag`.  Waits are bounded: a workgroup that spins
// past the limit records an error code and leaves.
#include <stdlib.h>

#include "score_tile.h"

namespace ams {
namespace {

constexpr int kTileTok = 256;  // tokens per workgroup tile: 4 waves x 2 MFMA row blocks x 32
constexpr int kSpinLimit = 1 << 22;

struct FusedArgs {
  ScoreArgs s;
  const int32_t* tiles_before;  // [B + 1] exclusive prefix over sequences of tiles per (sequence, head)
  float2* tstats;               // [units][tiles_max][n_pad]
  int32_t* counter;             // [units]
  int32_t* flag;                // [units]
  int32_t* status;              // [1] 0 = fine
  double* vsum_part;            // [units][tiles_max] sum over the tile of max(u,0)+eps
  int tiles_max;
  float eps;
};

// Cross-workgroup data travels through device-scope (agent) relaxed atomics: such loads and stores
// are coherent across the chip's L2 slices by themselves, so no cache-wide write-back or
// invalidation (a full fence) is needed on the hot path.  Ordering is by completion: a wave waits
// for its stores to complete before the workgroup announces them.
__device__ __forceinline__ void store_agent(float2* p, float2 v) {
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), __builtin_bit_cast(unsigned long long, v),
                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 load_agent(const float2* p) {
  return __builtin_bit_cast(float2, __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p),
                                                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ void wait_stores_complete() { __builtin_amdgcn_s_waitcnt(0x0F70); }  // vmcnt(0)

#ifdef AMS_FUSED_TIMING
// development aid: cycles per phase, summed per workgroup, left in the vsum_part scratch region
#define TICK(k)                                                    \
  do {                                                             \
    const long long now_ = clock64();                              \
    if (threadIdx.x == 0) tacc[k] += now_ - tprev;                 \
    tprev = now_;                                                  \
  } while (0)
#else
#define TICK(k) do {} while (0)
#endif

struct TileId {
  int unit, l, b, h, j, T;
};

__device__ __forceinline__ TileId decode_tile(const FusedArgs& a, int tile, int per_layer) {
  TileId t;
  t.l = tile / per_layer;
  const int r = tile - t.l * per_layer;
  // largest b with H * tiles_before[b] <= r
  int lo = 0, hi = a.s.d.B - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (a.s.d.H * a.tiles_before[mid] <= r) lo = mid; else hi = mid - 1;
  }
  t.b = lo;
  const int tiles_b = a.tiles_before[lo + 1] - a.tiles_before[lo];
  const int r2 = r - a.s.d.H * a.tiles_before[lo];
  t.h = r2 / tiles_b;
  t.j = r2 - t.h * tiles_b;
  t.unit = (t.l * a.s.d.B + t.b) * a.s.d.H + t.h;
  t.T = a.s.seq_lens[t.b];
  return t;
}

// Zeroes the per-unit synchronisation words and lays out the tile numbering.
__global__ void fused_init_kernel(FusedArgs a, int32_t* tiles_before_out) {
  for (int i = threadIdx.x; i < a.s.d.units; i += blockDim.x) {
    a.counter[i] = 0;
    a.flag[i] = 0;
  }
  if (threadIdx.x == 0) {
    *a.status = 0;
    int acc = 0;
    for (int b = 0; b < a.s.d.B; ++b) {
      tiles_before_out[b] = acc;
      acc += (a.s.seq_lens[b] + kTileTok - 1) / kTileTok;
    }
    tiles_before_out[a.s.d.B] = acc;
  }
}

template <int NB, int MODE>
__global__ __launch_bounds__(kThreads, 2) void score_onepass_kernel(FusedArgs a) {
  extern __shared__ __align__(16) char qlds[];
  __shared__ float2 xch[4][NB * 32];
  __shared__ int s_last, s_ok;
  __shared__ float merge_m[kThreads];
  __shared__ double merge_z[kThreads];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, hf = lane >> 5, c = lane & 31;
  const int per_layer = a.s.d.H * a.tiles_before[a.s.d.B];
  const int total = a.s.d.L * per_layer;
  const int n_pad = a.s.n_pad;
  const float c2 = a.s.c2;

  int tile = blockIdx.x;
  if (tile >= total) return;
  TileId cur = decode_tile(a, tile, per_layer);
  uint4 av0[8], av1[8];
  {
    const int t0 = cur.j * kTileTok + wave * 64;
    load_a<true>(a.s, cur.l, cur.b, cur.h, t0, cur.T, lane, av0);
    load_a<true>(a.s, cur.l, cur.b, cur.h, t0 + 32, cur.T, lane, av1);
  }
#ifdef AMS_FUSED_TIMING
  long long tacc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  long long tprev = clock64();
#endif
  bool alive = true;
  while (alive) {
    const int t0 = cur.j * kTileTok + wave * 64;
    __syncthreads();  // the previous tile's MFMAs have read the query tile in LDS
    load_q<true, NB>(a.s, cur.l, cur.b, cur.h, qlds);
    __syncthreads();
    TICK(0);
    floatx16 acc0[NB], acc1[NB];
    tile_mma<true, NB>(av0, qlds, lane, acc0);
    tile_mma<true, NB>(av1, qlds, lane, acc1);

    if (MODE == MODE_EXPECTED) {
      // moments of the N logits of every token, before the logits are overwritten by exponentials
      const float inv_n = 1.f / (float)a.s.d.N;
      float* g_row = a.s.g + (int64_t)cur.unit * a.s.d.t_stride;
#pragma unroll
      for (int blk = 0; blk < 2; ++blk) {
        floatx16* acc = blk ? acc1 : acc0;
        float ps[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          ps[i] = 0.f;
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) ps[i] += acc[nb][i] * a.s.inv_sqrt_d;
        }
        const float mean_mine = reduce16_over32(ps, c) * inv_n;
        float pv[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float mean_i = __shfl(mean_mine, 2 * i + 32 * hf);
          float s2 = 0.f;
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            const float dlt = acc[nb][i] * a.s.inv_sqrt_d - mean_i;
            s2 += ((nb * 32 + c) < a.s.d.N ? 1.f : 0.f) * dlt * dlt;
          }
          pv[i] = s2;
        }
        const float rg = mean_mine + 0.5f * reduce16_over32(pv, c) * inv_n;
        const int t = t0 + blk * 32 + acc_row(c >> 1, hf);
        if ((c & 1) == 0 && t < cur.T) g_row[t] = rg;
      }
    }

    // tile statistics of this wave, per query column, in the log2 domain
    const bool wave_has_tokens = t0 < cur.T;
    float mw[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      float mx = -INFINITY;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int r = acc_row(i, hf);
        float x0 = acc0[nb][i], x1 = acc1[nb][i];
        if (t0 + r >= cur.T) x0 = -INFINITY;
        if (t0 + 32 + r >= cur.T) x1 = -INFINITY;
        acc0[nb][i] = x0;
        acc1[nb][i] = x1;
        mx = fmaxf(mx, fmaxf(x0, x1));
      }
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m = wave_has_tokens ? mx * c2 : kNegInit;  // c2 > 0: the maximum commutes with the scale
      float z = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(acc0[nb][i], c2, -m));
        const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(acc1[nb][i], c2, -m));
        acc0[nb][i] = e0;
        acc1[nb][i] = e1;
        z += e0 + e1;
      }
      z += __shfl_xor(z, 32);
      mw[nb] = m;
      if (hf == 0) xch[wave][nb * 32 + c] = make_float2(m, wave_has_tokens ? z : 0.f);
    }
    __syncthreads();
    TICK(1);
    const int tiles_u = a.tiles_before[cur.b + 1] - a.tiles_before[cur.b];
    float2* my_stats = a.tstats + ((int64_t)cur.unit * a.tiles_max + cur.j) * n_pad;
    if (threadIdx.x < NB * 32) {
      const int n = threadIdx.x;
      float M = kNegInit;
#pragma unroll
      for (int w = 0; w < 4; ++w) M = fmaxf(M, xch[w][n].x);
      float Z = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) Z += xch[w][n].y * __builtin_amdgcn_exp2f(xch[w][n].x - M);
      store_agent(&my_stats[n], make_float2(M, Z));
    }
    wait_stores_complete();  // the statistics are in place before the tile is counted
    __syncthreads();
    TICK(2);
    if (threadIdx.x == 0) {
      const int old = __hip_atomic_fetch_add(&a.counter[cur.unit], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_last = (old == tiles_u - 1);
    }
    __syncthreads();
    TICK(3);
    if (s_last) {
      // last tile of the unit: merge all tiles' statistics.  The 256 threads split into
      // (query, contiguous range of tiles) pairs; loads go out sixteen at a time so that their
      // latencies overlap; the ranges are then combined in ascending order (fixed association).
      {
        const int parts = kThreads / n_pad;
        const int n = threadIdx.x % n_pad, part = threadIdx.x / n_pad;
        const int per = (tiles_u + parts - 1) / parts;
        const int j0 = part * per, j1 = min(tiles_u, j0 + per);
        const float2* p = a.tstats + (int64_t)cur.unit * a.tiles_max * n_pad + n;
        float M = kNegInit;
        double Z = 0.0;
        for (int j = j0; j < j1; j += 16) {
          float2 v[16];
#pragma unroll
          for (int k = 0; k < 16; ++k)
            v[k] = (j + k < j1) ? load_agent(p + (int64_t)(j + k) * n_pad) : make_float2(kNegInit, 0.f);
          float bm = M;
#pragma unroll
          for (int k = 0; k < 16; ++k) bm = fmaxf(bm, v[k].x);
          Z *= (double)__builtin_amdgcn_exp2f(M - bm);
#pragma unroll
          for (int k = 0; k < 16; ++k) Z += (double)v[k].y * (double)__builtin_amdgcn_exp2f(v[k].x - bm);
          M = bm;
        }
        merge_m[threadIdx.x] = M;
        merge_z[threadIdx.x] = Z;
        __syncthreads();
        if (threadIdx.x < n_pad) {
          float Mf = kNegInit;
          for (int q = 0; q < parts; ++q) Mf = fmaxf(Mf, merge_m[q * n_pad + n]);
          double Zf = 0.0;
          for (int q = 0; q < parts; ++q)
            Zf += merge_z[q * n_pad + n] * (double)__builtin_amdgcn_exp2f(merge_m[q * n_pad + n] - Mf);
          const bool real = n < a.s.d.N;
          const bool newest = real && (n % a.s.d.W) == a.s.d.W - 1;
          float2* fo = reinterpret_cast<float2*>(a.s.fin + (int64_t)cur.unit * n_pad + n);
          store_agent(fo, make_float2(Mf, real ? (float)(1.0 / ((double)a.s.d.N * Zf)) : 0.f));
          store_agent(fo + 1, make_float2(newest ? (float)(1.0 / ((double)a.s.d.G * Zf)) : 0.f, real ? 1.f : 0.f));
        }
      }
      wait_stores_complete();
      __syncthreads();
      if (threadIdx.x == 0) __hip_atomic_store(&a.flag[cur.unit], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    TICK(4);
    // the next tile's keys start to travel while this tile waits for its unit
    const int next = tile + gridDim.x;
    TileId nxt = cur;
    if (next < total) {
      nxt = decode_tile(a, next, per_layer);
      const int n0 = nxt.j * kTileTok + wave * 64;
      load_a<true>(a.s, nxt.l, nxt.b, nxt.h, n0, nxt.T, lane, av0);
      load_a<true>(a.s, nxt.l, nxt.b, nxt.h, n0 + 32, nxt.T, lane, av1);
    }

    if (threadIdx.x == 0) {
      int budget = kSpinLimit;
      while (__hip_atomic_load(&a.flag[cur.unit], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0 && --budget > 0)
        __builtin_amdgcn_s_sleep(8);
      s_ok = budget > 0;
      if (budget <= 0) atomicExch(a.status, 1);
    }
    __syncthreads();
    TICK(5);
    if (!s_ok) return;  // give up: the status word tells the host side
    // finish this wave's tokens from registers
    if (wave_has_tokens) {
      const float4* fin = a.s.fin + (int64_t)cur.unit * n_pad;
      float fu[NB], fg[NB];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const float2* fi = reinterpret_cast<const float2*>(fin + nb * 32 + c);
        const float2 f01 = load_agent(fi), f23 = load_agent(fi + 1);
        const float sc = __builtin_amdgcn_exp2f(mw[nb] - f01.x);
        fu[nb] = sc * f01.y;
        fg[nb] = sc * f23.x;
      }
      float* u_row = a.s.u + (int64_t)cur.unit * a.s.d.t_stride;
      float* g_row = (MODE != MODE_EXPECTED && a.s.g) ? a.s.g + (int64_t)cur.unit * a.s.d.t_stride : nullptr;
#pragma unroll
      for (int blk = 0; blk < 2; ++blk) {
        floatx16* acc = blk ? acc1 : acc0;
        float pu[16], pg[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          pu[i] = 0.f;
          pg[i] = 0.f;
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            pu[i] = __builtin_fmaf(fu[nb], acc[nb][i], pu[i]);
            if (MODE == MODE_LAST) pg[i] = __builtin_fmaf(fg[nb], acc[nb][i], pg[i]);
          }
        }
        const float ru = reduce16_over32(pu, c);
        float rg = ru;
        if (MODE == MODE_LAST) rg = reduce16_over32(pg, c);
        const int t = t0 + blk * 32 + acc_row(c >> 1, hf);
        if ((c & 1) == 0 && t < cur.T) {
          u_row[t] = ru;
          if (g_row) g_row[t] = rg;
        }
      }
    }
    TICK(6);
    tile = next;
    cur = nxt;
    alive = tile < total;
  }
#ifdef AMS_FUSED_TIMING
  if (threadIdx.x == 0)
    for (int k = 0; k < 8; ++k) reinterpret_cast<long long*>(a.vsum_part)[blockIdx.x * 8 + k] = tacc[k];
#endif
}

template <typename K>
hipError_t launch_coop(K kernel, int lds, const FusedArgs& a, int max_tiles, int tiles_per_unit_max,
                       hipStream_t s, bool* ran) {
  *ran = false;
  hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e != hipSuccess) return e;
  int dev = 0, per_cu = 0, cus = 0, coop = 0;
  if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
  if ((e = hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev)) != hipSuccess) return e;
  if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
  if ((e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kThreads, lds)) != hipSuccess) return e;
  const int resident = per_cu * cus;
  if (!coop || resident < 1 || tiles_per_unit_max > resident) return hipSuccess;  // caller falls back
  const int grid = max_tiles < resident ? max_tiles : resident;
  prof_mark("score_init", s);
  hipLaunchKernelGGL(fused_init_kernel, dim3(1), dim3(1024), 0, s, a, (int32_t*)a.tiles_before);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  FusedArgs args = a;
  void* kargs[] = {(void*)&args};
  prof_mark("score_onepass", s);
  e = hipLaunchCooperativeKernel((const void*)kernel, dim3(grid), dim3(kThreads), kargs, lds, s);
  if (e == hipSuccess) *ran = true;
  return e;
}

}  // namespace

size_t fused_score_ws_bytes(int64_t units, int t_max, int n_pad, int batch) {
  const int64_t tiles_max = (t_max + kTileTok - 1) / kTileTok;
  size_t o = 0;
  o += ((size_t)units * tiles_max * n_pad * sizeof(float2) + 255) & ~(size_t)255;
  o += ((size_t)units * tiles_max * sizeof(double) + 255) & ~(size_t)255;
  o += (((size_t)units * 2 + 64) * sizeof(int32_t) + 255) & ~(size_t)255;
  o += (((size_t)batch + 1) * sizeof(int32_t) + 255) & ~(size_t)255;
  return o;
}

// Returns hipSuccess with *ran = false when the one-sweep kernel does not apply (the caller then
// uses the two-sweep kernels).
hipError_t launch_score_onepass(const ams_params* p, const Dims& d, const KvDev& k, const int32_t* seq_lens,
                                const void* q, float* u, float* g, char* ws, const WsLayout& wl,
                                hipStream_t s, bool* ran) {
  *ran = false;
  if (p->kv_dtype != AMS_BF16 || wl.n_pad > 128) return hipSuccess;
  // Experimental: measured slower than the two-sweep kernels on MI355X (the cross-workgroup wait per
  // tile is not hidden with two resident workgroups per CU), so it only runs on request.
  const char* want = getenv("AMS_SCORER_ONEPASS");
  if (!want || want[0] != '1') return hipSuccess;
  int mode = MODE_MEAN;
  float* g_out = nullptr;
  if (p->scorer == AMS_SCORER_MEAN_WINDOW) g_out = (g != u) ? g : nullptr;
  if (p->scorer == AMS_SCORER_LAST_QUERY) { mode = MODE_LAST; g_out = g; }
  if (p->scorer == AMS_SCORER_EXPECTED) { mode = MODE_EXPECTED; g_out = g; }
  FusedArgs a;
  a.s.k = k;
  a.s.d = d;
  a.s.seq_lens = seq_lens;
  a.s.q = (const char*)q;
  a.s.part = nullptr;
  a.s.vc_part = nullptr;
  a.s.credit = nullptr;
  a.s.eps = p->mass_eps;
  a.s.fin = (float4*)(ws + wl.fin_stats);
  a.s.u = u;
  a.s.g = g_out;
  a.s.n_chunks = 0;
  a.s.n_pad = wl.n_pad;
  a.s.inv_sqrt_d = (float)(1.0 / sqrt((double)d.D));
  a.s.c2 = (float)(1.4426950408889634 / sqrt((double)d.D));
  a.tiles_max = (d.t_max + kTileTok - 1) / kTileTok;
  a.eps = p->mass_eps;
  char* w = ws + wl.fused;
  a.tstats = (float2*)w;
  w += ((size_t)d.units * a.tiles_max * wl.n_pad * sizeof(float2) + 255) & ~(size_t)255;
  a.vsum_part = (double*)w;
  w += ((size_t)d.units * a.tiles_max * sizeof(double) + 255) & ~(size_t)255;
  a.counter = (int32_t*)w;
  a.flag = a.counter + d.units;
  a.status = a.flag + d.units;
  w += (((size_t)d.units * 2 + 64) * sizeof(int32_t) + 255) & ~(size_t)255;
  int32_t* tiles_before = (int32_t*)w;
  a.tiles_before = tiles_before;

  // is the kernel usable for these shapes at all?  (decided before anything is launched)
  const int nb = wl.n_pad / 32;
  const int lds = nb * 32 * Tr<true>::kQStride;
  const int max_tiles = d.units * a.tiles_max > 0x7fffffff / 2 ? 0x3fffffff : d.units * a.tiles_max;
#define AMS_FUSED_CASE(NBV)                                                                                  \
  if (nb == NBV) {                                                                                           \
    if (mode == MODE_LAST) return launch_coop(score_onepass_kernel<NBV, MODE_LAST>, lds, a, max_tiles, a.tiles_max, s, ran); \
    if (mode == MODE_EXPECTED) return launch_coop(score_onepass_kernel<NBV, MODE_EXPECTED>, lds, a, max_tiles, a.tiles_max, s, ran); \
    return launch_coop(score_onepass_kernel<NBV, MODE_MEAN>, lds, a, max_tiles, a.tiles_max, s, ran);       \
  }
  AMS_FUSED_CASE(1)
  AMS_FUSED_CASE(2)
  AMS_FUSED_CASE(4)
#undef AMS_FUSED_CASE
  return hipSuccess;
}

}  // namespace ams
