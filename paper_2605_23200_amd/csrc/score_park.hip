// One-read scorer: usage u (and the softmax-based g) with K read from memory exactly once
// (Alg. 1 step 1; Sec. 3.2; Sec. 3.3 plug-in scorer; App. "Complexity and System Efficiency":
// the base scoring function dominates the cost of an event).
//
// u[t] = (1/N) sum_n exp(s[n][t] - M_n) / Z_n needs every query's normaliser over ALL tokens of the
// unit before any token can be finished.  The two-sweep kernels read K twice for that.  Here a
// CLUSTER of C workgroups owns a whole unit for the time it takes: workgroup j of the cluster keeps
// the keys of tokens [512 j, 512 j + 512) on chip (bf16; per wave 128 tokens: three 32-token blocks
// in 96 registers, the fourth in 8 KB of LDS), multiplies them once for the per-query (max, sum of exp), publishes
// that, waits for the unit's normalisers -- ONE exchange per unit and cluster -- and multiplies the
// same registers again to finish its tokens.  The logits are computed twice (the matrix cores have
// the headroom), the keys cross the memory system once.  As soon as a pair of blocks has been used
// the second time, the keys of the cluster's NEXT unit are requested into the same registers, so
// the key stream keeps flowing through the exchange and the epilogue.
//
// The grid holds as many workgroups as are resident at once (two per CU: while one waits for its
// exchange the other one computes) and clusters walk their units in increasing order, so every
// workgroup a wait depends on is running and never waits for a later unit.  All waits are bounded:
// a workgroup that spins past the limit raises the status word and leaves; the kernels that follow
// turn a raised status word into kept counts of -1.
//
// Exchange per (cluster, unit): members store their 2 floats per query with device-scope relaxed
// atomics (coherent across the L2 slices without cache-wide fences), wait for the stores to
// complete and count in; the member that completes the count merges the C contributions in member
// order (fixed association, independent of arrival order), stores (M_n, 1/(N Z_n), last-query
// weight) and raises the cluster's flag to the unit's sequence number; the others poll the flag.
// The contribution slots alternate with the parity of the sequence number: nobody can be two units
// ahead of the merging member.
#include <type_traits>

#include "score_tile.h"

namespace ams {
namespace {

constexpr int kParkBlocks = 4;                   // 32-token blocks a wave keeps on chip
constexpr int kParkWaveTok = kParkBlocks * 32;   // tokens per wave and unit
constexpr int kParkTok = 4 * kParkWaveTok;       // tokens per workgroup and unit
constexpr int kParkSpin = 1 << 17;               // polls of a bounded wait (about 0.1 s)
#ifndef AMS_PARK_STAGGER
#define AMS_PARK_STAGGER 1   // 1: the upper half of the clusters starts half a unit late (tuning knob)
#endif

#ifdef AMS_PARK_TRACE
#define PARK_MARK(k) do { if (threadIdx.x == 0 && a.trace) a.trace[((int64_t)blockIdx.x * 64 + seq) * 8 + (k)] = wall_clock64(); } while (0)
#else
#define PARK_MARK(k) do { } while (0)
#endif

int g_wait_limit = 0;  // ams_debug_set_wait_limit: 0 = kParkSpin

struct ParkArgs {
  ScoreArgs s;
  float2* part;      // [clusters][2][C][n_pad]  per member (max, sum) in the log2 domain
  int32_t* sync;     // [clusters][2]  members counted in, units finished
  int32_t* status;   // [1]  0 = fine, 1 = a wait expired
  int C;             // workgroups per cluster
  int n_clusters;
  int vc_stride;     // entries per unit of s.vc_part (one per member)
  int spin;          // polls a bounded wait may take before it gives up
#ifdef AMS_PARK_TRACE
  long long* trace;  // [workgroups][64 units][8 marks] timestamps of a measurement build
#endif
};

__device__ __forceinline__ void store_agent(float2* p, float2 v) {
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), __builtin_bit_cast(unsigned long long, v),
                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 load_agent(const float2* p) {
  return __builtin_bit_cast(float2, __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p),
                                                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ void wait_stores_complete() { __builtin_amdgcn_s_waitcnt(0x0F70); }  // vmcnt(0)

__global__ void park_init_kernel(int32_t* sync, int n_words, int32_t* status) {
  for (int i = threadIdx.x; i < n_words; i += blockDim.x) sync[i] = 0;
  if (threadIdx.x == 0) *status = 0;
}

// Two 32x32 tiles of logits against one block of 32 queries; every query fragment feeds both products.
// QROWS = false: s = K_tile . Q^T, a lane owns one query column and 16 token rows (first product: the
// maximum and the sum of a query stay inside a lane).  QROWS = true: the operands swap places and the
// tile comes out transposed, a lane owns one token column and 16 query rows (second product: the sum
// over the queries of a token stays inside a lane).  The fragments are the same registers either way.
// The contraction runs in two halves of four steps so that the fragments of the second half can travel
// from LDS while the first half is multiplied.
template <bool QROWS>
__device__ __forceinline__ void park_mma4(const uint4* k0, const uint4* k1, const uint4* q, floatx16 (&acc)[2]) {
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const bf16x8 qf = __builtin_bit_cast(bf16x8, q[ks]);
    const bf16x8 a0 = __builtin_bit_cast(bf16x8, k0[ks]), a1 = __builtin_bit_cast(bf16x8, k1[ks]);
    if (QROWS) {
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, a0, acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, a1, acc[1], 0, 0, 0);
    } else {
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qf, acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, qf, acc[1], 0, 0, 0);
    }
  }
}

// Four 16-byte fragments, 1024 bytes apart (the LDS-parked keys) or 16 bytes apart (a query row).
template <int STRIDE>
__device__ __forceinline__ void read_frags4(const char* p, uint4 (&f)[4]) {
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) f[ks] = *(const uint4*)(p + ks * STRIDE);
}

// One column block of a pair of tiles.  LDS0: the first tile's keys are the LDS-parked block, whose
// first four fragments stay in k0_lo for the whole pair and whose last four are re-read per column
// block (registers); otherwise k0 are eight registers-parked fragments.  q_lo: the column block's first
// four query fragments (requested a block ahead); the last four are requested here and arrive while
// the first half is multiplied.
template <bool QROWS, bool LDS0>
__device__ __forceinline__ void park_block(const uint4* k0, const uint4 (&k0_lo)[4], const char* k0_lds,
                                           const uint4* k1, const uint4 (&q_lo)[4], const char* q_row,
                                           floatx16 (&acc)[2]) {
  uint4 q_hi[4], k0_hi[4];
  read_frags4<16>(q_row + 64, q_hi);
  if (LDS0) read_frags4<1024>(k0_lds + 4096, k0_hi);
#pragma unroll
  for (int r = 0; r < 2; ++r)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[r][i] = 0.f;
  park_mma4<QROWS>(LDS0 ? k0_lo : k0, k1, q_lo, acc);
  park_mma4<QROWS>(LDS0 ? k0_hi : k0 + 4, k1 + 4, q_hi, acc);
  // order for the scheduler: every fragment read of the second half is issued before the first product,
  // so that the reads travel while the first half is multiplied (left alone it issues read, wait, product)
  __builtin_amdgcn_sched_group_barrier(0x100, LDS0 ? 8 : 4, 0);
  __builtin_amdgcn_sched_group_barrier(0x008, 16, 0);
}

// max(a, b, c) in one instruction; the accumulator values need no canonicalisation first
__device__ __forceinline__ float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// (value held by the lane's counterpart in the lower half wave, value held by the one in the upper half):
// v_permlane32_swap exchanges lanes 32..63 of its first operand with lanes 0..31 of its second
__device__ __forceinline__ void both_halves(float x, float& lo, float& hi) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  lo = __uint_as_float(r[0]);
  hi = __uint_as_float(r[1]);
}


template <int NB, int MODE>
__global__ __launch_bounds__(kThreads, 2) void score_park_kernel(ParkArgs a) {
  constexpr int QS = Tr<true>::kQStride, NQ = NB * 32;
  extern __shared__ __align__(16) char qlds[];  // the query window, then 8 KB of parked keys per wave
  // one static area, used in turn (barriers in between) for: the (pair, wave) statistics of the first
  // product [8][NQ] float2; the merge scratch of the member that completes the count; u and g of the
  // workgroup's 512 tokens
  __shared__ __align__(16) char area[8 * NQ * 8 > 6144 ? 8 * NQ * 8 : 6144];
  __shared__ __align__(16) float fin_m[NQ], fin_g[MODE == MODE_LAST ? NQ : 4];
  __shared__ double2 vc_sm[4];
  __shared__ int s_last, s_ok;
  float2(*xch)[NQ] = reinterpret_cast<float2(*)[NQ]>(area);
  float* merge_m = reinterpret_cast<float*>(area + 2048);       // [kThreads], after merge_z
  double* merge_z = reinterpret_cast<double*>(area);            // [kThreads]
  float* u_sm = reinterpret_cast<float*>(area);                 // [kParkTok]
  float* g_sm = reinterpret_cast<float*>(area + 4 * kParkTok);  // [kParkTok]
  const int C = a.C;
  const int cluster = blockIdx.x / C, me = blockIdx.x - cluster * C;
  if (cluster >= a.n_clusters) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, hf = lane >> 5, c = lane & 31;
  const int n_pad = a.s.n_pad;
  const float c2 = a.s.c2;
  const int w0 = me * kParkTok, t0w = w0 + wave * kParkWaveTok;
  const char* qb = qlds + c * QS + hf * (Tr<true>::kRowBytes / 2);
  char* kl_wave = qlds + NB * 32 * QS + wave * 8192;
  const char* kl = kl_wave + lane * 16;  // this lane's fragments of the LDS-parked block
  float2* part = a.part + (int64_t)cluster * 2 * C * n_pad;
  int32_t* counter = a.sync + 2 * cluster;
  int32_t* flag = counter + 1;

  // Block 0 of the wave's 128 tokens is parked in LDS, blocks 1..3 in kv[0..2].  The LDS block is
  // written by the memory system itself (global_load_lds: lane i's 16 bytes land at base + 16 i), so
  // it needs no staging registers; such loads count in vmcnt like any other, and the code waits for
  // them explicitly before the block is read.
  uint4 kv[3][8];
  // dense caches only: row t of a unit starts at base + (unit * t_capacity + t) * 256 bytes; lane (r, hf)
  // owns the hf-th half of row t0 + r (the mapping of load_a); rows past the end re-read the last row
  auto row_ptr = [&](int unit, int T, int t0) __attribute__((always_inline)) -> const char* {
    const int t = min(t0 + c, T - 1);
    return a.s.k.base + ((int64_t)unit * a.s.k.t_capacity + t) * (int64_t)Tr<true>::kRowBytes +
           hf * (Tr<true>::kRowBytes / 2);
  };
  auto unit_len = [&](int unit) __attribute__((always_inline)) -> int {
    return seq_len(a.s.d, a.s.seq_lens, (unit / a.s.d.H) % a.s.d.B);
  };
  auto request = [&](int unit, int T, int r, uint4 (&dst)[8]) __attribute__((always_inline)) {
    if (t0w + 32 * r < T) {
      const uint4* p = (const uint4*)row_ptr(unit, T, t0w + 32 * r);
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) dst[ks] = p[ks];
    }
  };
  auto request_lds = [&](int unit, int T) __attribute__((always_inline)) {
    if (t0w < T) {
      const char* row = row_ptr(unit, T, t0w);
#pragma unroll
      for (int ks = 0; ks < 8; ++ks)
        __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(row + ks * 16),
                                         (void __attribute__((address_space(3)))*)(kl_wave + ks * 1024), 16, 0, 0);
    }
  };
  if (cluster < a.s.d.units) {
    const int T0 = unit_len(cluster);
    request_lds(cluster, T0);
    request(cluster, T0, 1, kv[0]);
    request(cluster, T0, 2, kv[1]);
    request(cluster, T0, 3, kv[2]);
  }
#if AMS_PARK_STAGGER
  // the two workgroups of a CU come from the two halves of the grid: out of phase, one computes
  // while the other one waits for its exchange
  if (cluster >= (a.n_clusters + 1) / 2 && a.n_clusters > 1) __builtin_amdgcn_s_sleep(100);
#endif

#pragma unroll 1
  for (int seq = 0, unit = cluster; unit < a.s.d.units; ++seq, unit += a.n_clusters) {
    int l, b, h;
    unit_coords(a.s.d, unit, l, b, h);
    const int T = seq_len(a.s.d, a.s.seq_lens, b);
    const int next_unit = unit + a.n_clusters;
    // the next unit's length is fetched here, far from where its keys are requested
    const int T_next = next_unit < a.s.d.units ? unit_len(next_unit) : 0;
    PARK_MARK(0);
    __syncthreads();  // the previous unit is done with the LDS areas
    load_q<true, NB>(a.s, l, b, h, qlds);
    // every load of this unit has been in flight since the previous unit's second product
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the LDS-parked block is complete
    asm volatile("" ::: "memory");
    __syncthreads();
    PARK_MARK(1);
    // the old credit of this workgroup's positions (for the EMA normaliser), in flight during the products
    float cr0 = 0.f, cr1 = 0.f;
    if (a.s.vc_part && a.s.credit) {
      const float* c_row = a.s.credit + (int64_t)unit * a.s.d.t_stride;
      if (w0 + (int)threadIdx.x < T) cr0 = c_row[w0 + threadIdx.x];
      if (w0 + kThreads + (int)threadIdx.x < T) cr1 = c_row[w0 + kThreads + threadIdx.x];
    }

    // ---- first product: per-query (max, sum exp2) over the tokens of a pair of blocks, log2 domain ----
    // lane (column c, half hf) owns query nb * 32 + c and the token rows 8 (i / 4) + 4 hf + i % 4
    auto stats_pair = [&](auto lds0, int pr, const uint4* k0, const uint4* k1) __attribute__((always_inline)) {
      constexpr bool LDS0 = decltype(lds0)::value;
      const int t0 = t0w + 64 * pr;
      const bool ragged = t0 + 64 > T;
      const int hf4 = 4 * hf;
      float2* out = xch[pr * 4 + wave];
      uint4 q_lo[4], k0_lo[4];
      read_frags4<16>(qb, q_lo);
      if (LDS0) read_frags4<1024>(kl, k0_lo);
#pragma unroll 1
      for (int nb = 0; nb < NB; ++nb) {
        floatx16 acc[2];
        park_block<false, LDS0>(k0, k0_lo, kl, k1, q_lo, qb + nb * 32 * QS, acc);
        // the next column block's first query fragments travel while this block's logits are reduced
        if (nb + 1 < NB) read_frags4<16>(qb + (nb + 1) * 32 * QS, q_lo);
        if (ragged) {
          // only the 4 hf term of a row depends on the lane: one vector value against a wave-uniform limit
#pragma unroll
          for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int i = 0; i < 16; ++i)
              acc[r][i] = (hf4 >= T - t0 - 32 * r - (8 * (i >> 2) + (i & 3))) ? -INFINITY : acc[r][i];
        }
        float mr = max3(acc[0][0], acc[1][0], acc[0][1]);
        mr = max3(mr, acc[1][1], acc[0][2]);
#pragma unroll
        for (int i = 2; i < 15; ++i) mr = max3(mr, acc[1][i], acc[0][i + 1]);
        mr = fmaxf(mr, acc[1][15]);
        const float mx = fmaxf(kNegInit, mr * c2);  // c2 > 0: the maximum commutes with the scale
        float ps[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 16; ++i)
#pragma unroll
          for (int r = 0; r < 2; ++r)
            ps[(2 * i + r) & 3] += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[r][i], c2, -mx));
        const float sum = (ps[0] + ps[1]) + (ps[2] + ps[3]);
        // the two halves of the wave hold the same query: lower half first, the same value in both
        float ml, mh, zl, zh;
        both_halves(mx, ml, mh);
        both_halves(sum, zl, zh);
        const float M = fmaxf(ml, mh);
        const float Z = zl * __builtin_amdgcn_exp2f(ml - M) + zh * __builtin_amdgcn_exp2f(mh - M);
        if (hf == 0) out[nb * 32 + c] = make_float2(M, Z);
      }
    };
    // a pair of which nothing exists leaves neutral entries
    auto stats_none = [&](int pr) __attribute__((always_inline)) {
      float2* out = xch[pr * 4 + wave];
      for (int n = lane; n < NQ; n += 64) out[n] = make_float2(kNegInit, 0.f);
    };
    if (t0w < T)
      stats_pair(std::true_type{}, 0, nullptr, kv[0]);
    else
      stats_none(0);
    if (t0w + 64 < T)
      stats_pair(std::false_type{}, 1, kv[1], kv[2]);
    else
      stats_none(1);
    __syncthreads();
    PARK_MARK(2);
    float2* slot = part + (int64_t)(seq & 1) * C * n_pad;
    if (threadIdx.x < NQ) {
      const int n = threadIdx.x;
      float M = kNegInit;
#pragma unroll
      for (int w = 0; w < 8; ++w) M = fmaxf(M, xch[w][n].x);
      float Z = 0.f;
#pragma unroll
      for (int w = 0; w < 8; ++w) Z += xch[w][n].y * __builtin_amdgcn_exp2f(xch[w][n].x - M);
      store_agent(slot + (int64_t)me * n_pad + n, make_float2(M, Z));
    }
    wait_stores_complete();  // the contribution is in place before the member counts in
    __syncthreads();
    if (threadIdx.x == 0) {
      const int old = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_last = (old == (seq + 1) * C - 1);
    }
    __syncthreads();
    PARK_MARK(3);
    if (s_last) {
      // the member that completes the count merges: the 256 threads split into (query, contiguous range
      // of members) pairs, every range loads its entries in large batches, the ranges are then combined
      // in ascending order
      const int parts = kThreads / n_pad;
      const int n = threadIdx.x % n_pad, prt = threadIdx.x / n_pad;
      const int per = (C + parts - 1) / parts;
      const int j0 = prt * per, j1 = min(C, j0 + per);
      const float2* p = slot + n;
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
        float2* fo = reinterpret_cast<float2*>(a.s.fin + (int64_t)unit * n_pad + n);
        // the weight 1 / (N Z_n) moves into the exponent: p[n][t] / N = exp2(x - (M_n + log2(N Z_n)));
        // a padded query gets +inf there and adds exp2(-inf) = 0
        const float Mp = real ? (float)((double)Mf + log2((double)a.s.d.N * Zf)) : INFINITY;
        store_agent(fo, make_float2(Mp, newest ? (float)((double)a.s.d.N / (double)a.s.d.G) : 0.f));
      }
      wait_stores_complete();
      __syncthreads();
      if (threadIdx.x == 0) __hip_atomic_store(flag, seq + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (threadIdx.x == 0) {
      int budget = a.spin;
      while (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < seq + 1 && --budget > 0)
        __builtin_amdgcn_s_sleep(2);
      s_ok = budget > 0;
      if (budget <= 0) atomicExch(a.status, 1);
    }
    __syncthreads();
    if (!s_ok) return;  // give up: the status word tells the kernels that follow
    PARK_MARK(4);
    if (threadIdx.x < NQ) {
      const float2* fi = reinterpret_cast<const float2*>(a.s.fin + (int64_t)unit * n_pad + threadIdx.x);
      const float2 f01 = load_agent(fi);
      fin_m[threadIdx.x] = f01.x;
      if (MODE == MODE_LAST) fin_g[threadIdx.x] = f01.y;
    }
    __syncthreads();

    // ---- second product from the parked keys: u[t] = sum_n exp2(x - M_n) / (N Z_n) ----
    // transposed tiles: lane (column c, half hf) owns token t0 + c and the query rows 8 (i / 4) + 4 hf + i % 4,
    // whose (M_n, weight) it reads from LDS four at a time (the whole half wave reads the same address)
    float v_part = 0.f;  // this lane's share of sum(max(u,0)+eps), at most 4 terms
    auto usage_pair = [&](auto lds0, int pr, const uint4* k0, const uint4* k1) __attribute__((always_inline)) {
      constexpr bool LDS0 = decltype(lds0)::value;
      const int t0 = t0w + 64 * pr;
      float pu[2][4], pg[MODE == MODE_LAST ? 2 : 1][4];
#pragma unroll
      for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          pu[r][j] = 0.f;
          if (MODE == MODE_LAST) pg[r][j] = 0.f;
        }
      uint4 q_lo[4], k0_lo[4];
      read_frags4<16>(qb, q_lo);
      if (LDS0) read_frags4<1024>(kl, k0_lo);
#pragma unroll 1
      for (int nb = 0; nb < NB; ++nb) {
        floatx16 acc[2];
        park_block<true, LDS0>(k0, k0_lo, kl, k1, q_lo, qb + nb * 32 * QS, acc);
        if (nb + 1 < NB) read_frags4<16>(qb + (nb + 1) * 32 * QS, q_lo);
        // references (with the weights folded in) of this lane's 16 query rows
        float4 mm[4], wg[MODE == MODE_LAST ? 4 : 1];
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          mm[q4] = *(const float4*)&fin_m[nb * 32 + 8 * q4 + 4 * hf];
          if (MODE == MODE_LAST) wg[q4] = *(const float4*)&fin_g[nb * 32 + 8 * q4 + 4 * hf];
        }
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const float mj[4] = {mm[q4].x, mm[q4].y, mm[q4].z, mm[q4].w};
#pragma unroll
          for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 2; ++r) {
              const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[r][4 * q4 + j], c2, -mj[j]));
              pu[r][j] += e;
              if (MODE == MODE_LAST) {
                const float gj[4] = {wg[q4].x, wg[q4].y, wg[q4].z, wg[q4].w};
                pg[r][j] = __builtin_fmaf(gj[j], e, pg[r][j]);
              }
            }
        }
      }
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        float lo, hi;
        both_halves((pu[r][0] + pu[r][1]) + (pu[r][2] + pu[r][3]), lo, hi);
        const float ru = lo + hi;  // the two halves own different query rows
        float rg = ru;
        if (MODE == MODE_LAST) {
          both_halves((pg[r][0] + pg[r][1]) + (pg[r][2] + pg[r][3]), lo, hi);
          rg = lo + hi;
        }
        const int t = t0 + 32 * r + c;
        if (hf == 0 && t < T) {
          u_sm[t - w0] = ru;
          if (MODE == MODE_LAST) g_sm[t - w0] = rg;
          v_part += fmaxf(ru, 0.f) + a.s.eps;
        }
      }
    };
    // as soon as a pair's keys have been used the second time, the keys of the cluster's next unit are
    // requested into their place (the products that read the LDS block have consumed its fragments)
    if (t0w < T) usage_pair(std::true_type{}, 0, nullptr, kv[0]);
    asm volatile("" ::: "memory");
    if (next_unit < a.s.d.units) {
      request_lds(next_unit, T_next);
      request(next_unit, T_next, 1, kv[0]);
    }
    if (t0w + 64 < T) usage_pair(std::false_type{}, 1, kv[1], kv[2]);
    if (next_unit < a.s.d.units) {
      request(next_unit, T_next, 2, kv[1]);
      request(next_unit, T_next, 3, kv[2]);
    }
    __syncthreads();
    PARK_MARK(5);
    {
      float* u_row = a.s.u + (int64_t)unit * a.s.d.t_stride;
      float* g_row = a.s.g ? a.s.g + (int64_t)unit * a.s.d.t_stride : nullptr;
#pragma unroll
      for (int k = 0; k < kParkTok / kThreads; ++k) {
        const int t = w0 + k * kThreads + (int)threadIdx.x;
        if (t < T) {
          u_row[t] = u_sm[t - w0];
          if (g_row) g_row[t] = MODE == MODE_LAST ? g_sm[t - w0] : u_sm[t - w0];
        }
      }
    }
    if (a.s.vc_part && w0 < T) {  // per member: sums of max(u,0)+eps and of the old credit, fixed order
      double v_acc = (double)v_part, c_acc = (double)cr0 + (double)cr1;
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
        a.s.vc_part[(int64_t)unit * a.vc_stride + me] = t;
      }
    }
    PARK_MARK(6);
  }
}

struct ParkPlan {
  bool known = false;
  int resident = 0;  // workgroups of the kernel that run at once on this device
};

template <typename K>
hipError_t plan_for(K kernel, int lds, ParkPlan& plan) {
  if (plan.known) return hipSuccess;
  hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e != hipSuccess) return e;
  int dev = 0, per_cu = 0, cus = 0;
  if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
  if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
  if ((e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kThreads, lds)) != hipSuccess) return e;
  plan.resident = (per_cu > 2 ? 2 : per_cu) * cus;
  if (plan.resident > kParkMaxWorkgroups) plan.resident = kParkMaxWorkgroups;
  plan.known = true;
  return hipSuccess;
}

template <int NB, int MODE>
hipError_t launch_park(ParkArgs a, int units, int t_max, hipStream_t s, bool force, bool* ran) {
  static ParkPlan plan;  // one device per process is assumed for the cached occupancy
  const int lds = NB * 32 * Tr<true>::kQStride + 4 * 8192;
  hipError_t e = plan_for(score_park_kernel<NB, MODE>, lds, plan);
  if (e != hipSuccess) return e;
  const int C = div_up(t_max, kParkTok);
  if (plan.resident < 1 || C > plan.resident || C > kParkMaxMembers) return hipSuccess;  // caller falls back
  int n_clusters = plan.resident / C;
  if (n_clusters > units) n_clusters = units;
  if (n_clusters > kParkMaxClusters) n_clusters = kParkMaxClusters;
  (void)force;
  a.C = C;
  a.n_clusters = n_clusters;
  a.vc_stride = div_up(t_max, kParkTok);
  prof_mark("score_init", s);
  hipLaunchKernelGGL(park_init_kernel, dim3(1), dim3(256), 0, s, a.sync, 2 * n_clusters, a.status);
  prof_mark("score_oneread", s);
  hipLaunchKernelGGL((score_park_kernel<NB, MODE>), dim3(n_clusters * C), dim3(kThreads), lds, s, a);
  e = hipGetLastError();
  if (e == hipSuccess) *ran = true;
  return e;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

size_t park_score_ws_bytes(int n_pad) {
  size_t o = 0;
  o += align256((size_t)kParkMaxWorkgroups * 2 * n_pad * sizeof(float2));  // contributions, both parities
  o += align256(((size_t)kParkMaxClusters * 2 + 64) * sizeof(int32_t));    // counters, flags, status
  return o;
}

void set_park_wait_limit(int polls) { g_wait_limit = polls > 0 ? polls : 0; }

int32_t* park_status_word(char* ws, const WsLayout& wl) {
  return (int32_t*)(ws + wl.park + align256((size_t)kParkMaxWorkgroups * 2 * wl.n_pad * sizeof(float2))) +
         2 * kParkMaxClusters;
}

// Returns hipSuccess with *ran = false when the one-read kernel does not apply (the caller then uses the
// two-sweep kernels).  On *ran = true and want_vc, the per-member sums for Eq. (1) / EMA are in
// ws + wl.vc_part with row stride *vc_stride and one entry per *vc_tokens positions.
hipError_t launch_score_oneread(const ams_params* p, const Dims& d, const KvDev& k, const int32_t* seq_lens,
                                const void* q, float* u, float* g, const float* credit, bool want_vc,
                                int* vc_stride, int* vc_tokens, char* ws, const WsLayout& wl,
                                hipStream_t s, bool* ran) {
  *ran = false;
  if (p->kv_dtype != AMS_BF16 || wl.n_pad > 128 || d.D != 128 || k.layout != AMS_LAYOUT_DENSE) return hipSuccess;
  if (p->causal != 0 && d.W > 1) return hipSuccess;  // the masked tail blocks live in the two-sweep kernels
  int mode = MODE_MEAN;
  float* g_out = nullptr;
  if (p->scorer == AMS_SCORER_MEAN_WINDOW) g_out = (g != u) ? g : nullptr;
  if (p->scorer == AMS_SCORER_LAST_QUERY) { mode = MODE_LAST; g_out = g; }
  // the moment-based scores keep all logits of a token live: they stay with the two-sweep kernels
  if (p->scorer == AMS_SCORER_EXPECTED || p->scorer == AMS_SCORER_EXPECTED_VNORM) return hipSuccess;
  ParkArgs a;
  a.s.k = k;
  a.s.d = d;
  a.s.seq_lens = seq_lens;
  a.s.q = (const char*)q;
  a.s.part = nullptr;
  a.s.fin = (float4*)(ws + wl.fin_stats);
  a.s.u = u;
  a.s.g = g_out;
  a.s.n_chunks = 0;
  a.s.chunk = 0;
  a.s.n_pad = wl.n_pad;
  a.s.inv_sqrt_d = (float)(1.0 / sqrt((double)d.D));
  a.s.c2 = (float)(1.4426950408889634 / sqrt((double)d.D));
  a.s.vc_part = want_vc ? (double2*)(ws + wl.vc_part) : nullptr;
  a.s.credit = credit;
  a.s.csum = nullptr;
  a.s.eps = p->mass_eps;
  a.s.causal = false;
  a.s.status = nullptr;
  char* w = ws + wl.park;
  a.part = (float2*)w;
  w += align256((size_t)kParkMaxWorkgroups * 2 * wl.n_pad * sizeof(float2));
  a.sync = (int32_t*)w;
  a.status = a.sync + 2 * kParkMaxClusters;
  a.C = a.n_clusters = a.vc_stride = 0;
  a.spin = g_wait_limit > 0 ? g_wait_limit : kParkSpin;
  if (vc_stride) *vc_stride = div_up(d.t_max, kParkTok);
  if (vc_tokens) *vc_tokens = kParkTok;
  const int nb = wl.n_pad / 32;
  const bool force = p->score_path == AMS_SCORE_PATH_ONE_READ;
#define AMS_PARK_CASE(NBV)                                                                              \
  if (nb == NBV) {                                                                                      \
    if (mode == MODE_LAST) return launch_park<NBV, MODE_LAST>(a, d.units, d.t_max, s, force, ran);      \
    return launch_park<NBV, MODE_MEAN>(a, d.units, d.t_max, s, force, ran);                             \
  }
  AMS_PARK_CASE(1)
  AMS_PARK_CASE(2)
  AMS_PARK_CASE(4)
#undef AMS_PARK_CASE
  return hipSuccess;
}

}  // namespace ams
