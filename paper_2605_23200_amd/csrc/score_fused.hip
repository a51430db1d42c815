// One-read scorer: usage u (and g) with K read from HBM exactly once
// (Alg. 1 step 1; Sec. 3.2; Sec. 3.3 plug-in scorer).
//
// u[t] = (1/N) sum_n exp(s[n][t] - M_n) / Z_n needs the softmax normaliser of every query over
// ALL tokens of the unit before any token can be finished.  The two-sweep kernels read K twice
// for that.  Here every wave keeps the keys of its tokens in registers (bf16, 32 registers per
// 32-token block) across the wait: it multiplies them once for the per-query (max, sum of exp),
// the workgroup publishes its tile's statistics, waits until the unit's normalisers are known,
// and then multiplies the SAME registers again to finish its tokens.  The logits are computed
// twice (the matrix cores have the headroom), the keys cross the memory system once.
//
// The kernel is persistent and launched cooperatively, so every workgroup is resident; tiles are
// taken in increasing order (tile = block + k * grid) and a unit never has more tiles than the
// grid has workgroups, which makes the wait free of deadlock: the workgroups a tile waits for are
// resident and never wait for a later unit.
//
// Per unit: `counter` counts published tiles; the workgroup that brings it to the tile count
// merges the statistics (fixed association, deterministic), stores the per-query
// (M_n, 1/(N Z_n), last-query weight) and raises `flag`.  Waits are bounded: a workgroup that spins
// past the limit records an error code and leaves.
#include <stdlib.h>

#include "score_tile.h"

namespace ams {
namespace {

constexpr int kRB = 2;                   // 32-token blocks a wave keeps in registers
constexpr int kWaveTok = kRB * 32;       // tokens per wave and tile
constexpr int kTileTok = 4 * kWaveTok;   // tokens per workgroup tile
constexpr int kSpinLimit = 1 << 22;

struct FusedArgs {
  ScoreArgs s;
  const int32_t* tiles_before;  // [B + 1] exclusive prefix over sequences of tiles per (sequence, head)
  float2* tstats;               // [units][tiles_max][n_pad]
  int32_t* counter;             // [units]
  int32_t* flag;                // [units]
  int32_t* status;              // [1] 0 = fine
  int tiles_max;
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
  t.T = seq_len(a.s.d, a.s.seq_lens, t.b);
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
      acc += (seq_len(a.s.d, a.s.seq_lens, b) + kTileTok - 1) / kTileTok;
    }
    tiles_before_out[a.s.d.B] = acc;
  }
}

template <int NB>
constexpr int kColGroup = (NB % 2 == 0 && NB >= 4) ? NB / 2 : NB;

template <int NB, int MODE>
__global__ __launch_bounds__(kThreads, 3) void score_oneread_kernel(FusedArgs a) {
  constexpr int NG = kColGroup<NB>, QS = Tr<true>::kQStride;
  extern __shared__ __align__(16) char qlds[];
  __shared__ float2 xch[4][NB * 32];
  __shared__ float4 fin_s[NB * 32];
  __shared__ int s_last, s_ok;
  __shared__ float merge_m[kThreads];
  __shared__ double merge_z[kThreads];
  __shared__ double2 vc_sm[4];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, hf = lane >> 5, c = lane & 31;
  const int per_layer = a.s.d.H * a.tiles_before[a.s.d.B];
  const int total = a.s.d.L * per_layer;
  const int n_pad = a.s.n_pad;
  const float c2 = a.s.c2;

#pragma unroll 1
  for (int tile = blockIdx.x; tile < total; tile += gridDim.x) {
    const TileId cur = decode_tile(a, tile, per_layer);
    const int T = cur.T;
    const int t0w = cur.j * kTileTok + wave * kWaveTok;
    // the wave's keys: requested now, multiplied twice, held until the tile is finished
    uint4 kv[kRB][8];
#pragma unroll
    for (int r = 0; r < kRB; ++r)
      if (t0w + 32 * r < T) load_a<true>(a.s, cur.l, cur.b, cur.h, t0w + 32 * r, T, lane, kv[r]);
    __syncthreads();  // the previous tile is done with the LDS areas
    load_q<true, NB>(a.s, cur.l, cur.b, cur.h, qlds);
    __syncthreads();

    // ---- first product: per-query (max, sum exp2) over this wave's tokens, log2 domain ----
    float m[NB], z[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      m[nb] = kNegInit;
      z[nb] = 0.f;
    }
#pragma unroll
    for (int r = 0; r < kRB; ++r) {
      const int t0 = t0w + 32 * r;
      if (t0 < T) {
        const bool ragged = t0 + 32 > T;
        int qoff = 0;  // the query fragments are re-read from LDS per block on purpose (registers)
        asm volatile("" : "+s"(qoff));
#pragma unroll
        for (int g0 = 0; g0 < NB; g0 += NG) {
          floatx16 acc[NG];
          tile_mma<true, NG>(kv[r], qlds + qoff + g0 * 32 * QS, lane, acc);
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
            const float mx = fmaxf(m[nb], mr * c2);
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) sum += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[k][i], c2, -mx));
            z[nb] = __builtin_fmaf(z[nb], __builtin_amdgcn_exp2f(m[nb] - mx), sum);
            m[nb] = mx;
          }
        }
      }
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const float m2 = __shfl_xor(m[nb], 32), z2 = __shfl_xor(z[nb], 32);
      const float M = fmaxf(m[nb], m2);
      const float zl = hf ? z2 : z[nb], ml = hf ? m2 : m[nb], zh = hf ? z[nb] : z2, mh = hf ? m[nb] : m2;
      const float Z = zl * __builtin_amdgcn_exp2f(ml - M) + zh * __builtin_amdgcn_exp2f(mh - M);
      if (hf == 0) xch[wave][nb * 32 + c] = make_float2(M, Z);
    }
    __syncthreads();
    const int tiles_u = a.tiles_before[cur.b + 1] - a.tiles_before[cur.b];
    if (threadIdx.x < NB * 32) {
      const int n = threadIdx.x;
      float M = kNegInit;
#pragma unroll
      for (int w = 0; w < 4; ++w) M = fmaxf(M, xch[w][n].x);
      float Z = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) Z += xch[w][n].y * __builtin_amdgcn_exp2f(xch[w][n].x - M);
      store_agent(a.tstats + ((int64_t)cur.unit * a.tiles_max + cur.j) * n_pad + n, make_float2(M, Z));
    }
    wait_stores_complete();  // the statistics are in place before the tile is counted
    __syncthreads();
    if (threadIdx.x == 0) {
      const int old = __hip_atomic_fetch_add(&a.counter[cur.unit], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_last = (old == tiles_u - 1);
    }
    __syncthreads();
    if (s_last) {
      // last tile of the unit: merge all tiles' statistics.  The 256 threads split into
      // (query, contiguous range of tiles) pairs; loads go out in batches so that their latencies
      // overlap; the ranges are then combined in ascending order (fixed association).
      const int parts = kThreads / n_pad;
      const int n = threadIdx.x % n_pad, part = threadIdx.x / n_pad;
      const int per = (tiles_u + parts - 1) / parts;
      const int j0 = part * per, j1 = min(tiles_u, j0 + per);
      const float2* p = a.tstats + (int64_t)cur.unit * a.tiles_max * n_pad + n;
      float M = kNegInit;
      double Z = 0.0;
      constexpr int kBatch = 16;
      for (int j = j0; j < j1; j += kBatch) {
        float2 v[kBatch];
#pragma unroll
        for (int k = 0; k < kBatch; ++k)
          v[k] = (j + k < j1) ? load_agent(p + (int64_t)(j + k) * n_pad) : make_float2(kNegInit, 0.f);
        float bm = M;
#pragma unroll
        for (int k = 0; k < kBatch; ++k) bm = fmaxf(bm, v[k].x);
        Z *= (double)__builtin_amdgcn_exp2f(M - bm);
#pragma unroll
        for (int k = 0; k < kBatch; ++k) Z += (double)v[k].y * (double)__builtin_amdgcn_exp2f(v[k].x - bm);
        M = bm;
      }
      merge_m[threadIdx.x] = M;
      merge_z[threadIdx.x] = Z;
      __syncthreads();
      if ((int)threadIdx.x < n_pad) {
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
      wait_stores_complete();
      __syncthreads();
      if (threadIdx.x == 0) __hip_atomic_store(&a.flag[cur.unit], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (threadIdx.x == 0) {
      int budget = kSpinLimit;
      while (__hip_atomic_load(&a.flag[cur.unit], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0 && --budget > 0)
        __builtin_amdgcn_s_sleep(8);
      s_ok = budget > 0;
      if (budget <= 0) atomicExch(a.status, 1);
    }
    __syncthreads();
    if (!s_ok) return;  // give up: the status word tells the host side
    if (threadIdx.x < NB * 32) {
      const float2* fi = reinterpret_cast<const float2*>(a.s.fin + (int64_t)cur.unit * n_pad + threadIdx.x);
      const float2 f01 = load_agent(fi), f23 = load_agent(fi + 1);
      fin_s[threadIdx.x] = make_float4(f01.x, f01.y, f23.x, f23.y);
    }
    __syncthreads();

    // ---- second product from the same registers: u[t] = sum_n exp2(x - M_n) / (N Z_n) ----
    float4 f[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) f[nb] = fin_s[nb * 32 + c];
    float* u_row = a.s.u + (int64_t)cur.unit * a.s.d.t_stride;
    float* g_row = a.s.g ? a.s.g + (int64_t)cur.unit * a.s.d.t_stride : nullptr;
    float v_part = 0.f;
#pragma unroll
    for (int r = 0; r < kRB; ++r) {
      const int t0 = t0w + 32 * r;
      if (t0 < T) {
        float pu[16], pg[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) pu[i] = pg[i] = 0.f;
        int qoff = 0;
        asm volatile("" : "+s"(qoff));
#pragma unroll
        for (int g0 = 0; g0 < NB; g0 += NG) {
          floatx16 acc[NG];
          tile_mma<true, NG>(kv[r], qlds + qoff + g0 * 32 * QS, lane, acc);
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
        float rg = ru;
        if (MODE == MODE_LAST) rg = reduce16_over32(pg, c);
        const int t = t0 + acc_row(c >> 1, hf);
        if ((c & 1) == 0 && t < T) {
          u_row[t] = ru;
          if (g_row) g_row[t] = rg;
          v_part += fmaxf(ru, 0.f) + a.s.eps;
        }
      }
    }
    if (a.s.vc_part) {  // per tile: sums of max(u,0)+eps and of the old credit, fixed order
      double v_acc = (double)v_part, c_acc = 0.0;
      if (a.s.credit) {
        const int jt = cur.j * kTileTok + threadIdx.x;  // kTileTok == kThreads: one position per thread
        if (jt < T) c_acc = (double)a.s.credit[(int64_t)cur.unit * a.s.d.t_stride + jt];
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
        a.s.vc_part[(int64_t)cur.unit * a.tiles_max + cur.j] = t;
      }
    }
  }
}
static_assert(kTileTok == kThreads, "the credit sum reads one position per thread");

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
  prof_mark("score_oneread", s);
  e = hipLaunchCooperativeKernel((const void*)kernel, dim3(grid), dim3(kThreads), kargs, lds, s);
  if (e == hipSuccess) *ran = true;
  return e;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

size_t fused_score_ws_bytes(int64_t units, int t_max, int n_pad, int batch) {
  const int64_t tiles_max = (t_max + kTileTok - 1) / kTileTok;
  size_t o = 0;
  o += align256((size_t)units * tiles_max * n_pad * sizeof(float2));
  o += align256(((size_t)units * 2 + 64) * sizeof(int32_t));
  o += align256(((size_t)batch + 1) * sizeof(int32_t));
  return o;
}

// Returns hipSuccess with *ran = false when the one-read kernel does not apply (the caller then
// uses the two-sweep kernels).  On *ran = true and want_vc, the per-tile sums for Eq. (1) / EMA are
// in ws + wl.vc_part with row stride *vc_stride and one entry per *vc_tokens positions.
hipError_t launch_score_oneread(const ams_params* p, const Dims& d, const KvDev& k, const int32_t* seq_lens,
                                const void* q, float* u, float* g, const float* credit, bool want_vc,
                                int* vc_stride, int* vc_tokens, char* ws, const WsLayout& wl,
                                hipStream_t s, bool* ran) {
  *ran = false;
  if (p->kv_dtype != AMS_BF16 || wl.n_pad > 128 || d.D != 128) return hipSuccess;
  // Opt-in (AMS_SCORER=oneread).  Measured on MI355X at 32 layers x 8 heads x 32k tokens: 1.54 ms
  // against 0.92 ms for the two sweeps.  Each 32-token block costs a SIMD about 4000 cycles of
  // matrix + vector issue per product (they overlap little) against about 3400 cycles of HBM time,
  // so computing the logits twice is compute-bound, and the per-tile wait for the unit's normalisers
  // (about 13 us of a 36 us tile round) is not hidden by three resident workgroups per CU.
  const char* want = getenv("AMS_SCORER");
  if (!want || want[0] != 'o') return hipSuccess;
  int mode = MODE_MEAN;
  float* g_out = nullptr;
  if (p->scorer == AMS_SCORER_MEAN_WINDOW) g_out = (g != u) ? g : nullptr;
  if (p->scorer == AMS_SCORER_LAST_QUERY) { mode = MODE_LAST; g_out = g; }
  // the moment-based scores keep all logits of a token live
  if (p->scorer == AMS_SCORER_EXPECTED || p->scorer == AMS_SCORER_EXPECTED_VNORM) return hipSuccess;
  FusedArgs a;
  a.s.k = k;
  a.s.d = d;
  a.s.seq_lens = seq_lens;
  a.s.q = (const char*)q;
  a.s.part = nullptr;
  a.s.fin = (float4*)(ws + wl.fin_stats);
  a.s.u = u;
  a.s.g = g_out;
  a.s.n_chunks = 0;
  a.s.n_pad = wl.n_pad;
  a.s.inv_sqrt_d = (float)(1.0 / sqrt((double)d.D));
  a.s.c2 = (float)(1.4426950408889634 / sqrt((double)d.D));
  a.s.vc_part = want_vc ? (double2*)(ws + wl.vc_part) : nullptr;
  a.s.credit = credit;
  a.s.eps = p->mass_eps;
  a.tiles_max = (d.t_max + kTileTok - 1) / kTileTok;
  char* w = ws + wl.fused;
  a.tstats = (float2*)w;
  w += align256((size_t)d.units * a.tiles_max * wl.n_pad * sizeof(float2));
  a.counter = (int32_t*)w;
  a.flag = a.counter + d.units;
  a.status = a.flag + d.units;
  w += align256(((size_t)d.units * 2 + 64) * sizeof(int32_t));
  a.tiles_before = (int32_t*)w;
  w += align256(((size_t)d.B + 1) * sizeof(int32_t));
  const int nb = wl.n_pad / 32;
  const int lds = nb * 32 * Tr<true>::kQStride;
  const int64_t all_tiles = (int64_t)d.units * a.tiles_max;
  const int max_tiles = all_tiles > 0x3fffffff ? 0x3fffffff : (int)all_tiles;
  if (vc_stride) *vc_stride = a.tiles_max;
  if (vc_tokens) *vc_tokens = kTileTok;
#define AMS_FUSED_CASE(NBV)                                                                                  \
  if (nb == NBV) {                                                                                           \
    if (mode == MODE_LAST) return launch_coop(score_oneread_kernel<NBV, MODE_LAST>, lds, a, max_tiles, a.tiles_max, s, ran); \
    return launch_coop(score_oneread_kernel<NBV, MODE_MEAN>, lds, a, max_tiles, a.tiles_max, s, ran);       \
  }
  AMS_FUSED_CASE(1)
  AMS_FUSED_CASE(2)
  AMS_FUSED_CASE(4)
#undef AMS_FUSED_CASE
  return hipSuccess;
}

}  // namespace ams
