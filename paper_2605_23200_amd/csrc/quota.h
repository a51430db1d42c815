// Quota of every segment of one unit, for up to 64 segments, by one wave (Sec. 3.3 "Segment-wise
// Quota Allocation"; Alg. 1 step 4).  Shared by the stand-alone quota kernel and the per-unit mass kernel.
#ifndef AMS_QUOTA_H
#define AMS_QUOTA_H

#include "ams_internal.h"

namespace ams {

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// Quotas for S <= 64: lane i owns segment i.  Sums of masses run in index order over the active
// lanes and every share is rem * M_i / sum, the same operations in the same order as plain C.
__device__ __forceinline__ int quota_wave(int S, int bud, int q_min, const int32_t* bounds, const float* mass) {
  const int lane = threadIdx.x;
  const bool valid = lane < S;
  const int len = valid ? bounds[lane + 1] - bounds[lane] : 0;
  const double mass_d = valid ? (double)mass[lane] : 0.0;
  const int nonempty = __popcll(__ballot(len > 0));
  int floor_q = q_min;
  if (wave_sum(min(floor_q, len)) > bud) floor_q = nonempty > 0 ? bud / nonempty : 0;
  const int lo = min(floor_q, len);
  const int room = len - lo;
  bool active = room > 0;
  int quo = lo;
  int rem = bud - wave_sum(lo);
  double raw = 0.0;
  // proportional shares; a segment whose share reaches its room is filled and leaves the pool
  for (;;) {
    const uint64_t act = __ballot(active);
    const int n_active = __popcll(act);
    if (n_active == 0 || rem <= 0) break;
    double msum = 0.0;
    for (uint64_t m = act; m; m &= m - 1) msum += __shfl(mass_d, __ffsll((long long)m) - 1);
    if (active) raw = msum > 0.0 ? (double)rem * mass_d / msum : (double)rem / (double)n_active;
    const bool sat = active && raw >= (double)room;
    if (!__ballot(sat)) break;
    rem -= wave_sum(sat ? room : 0);
    if (sat) {
      quo = len;
      active = false;
    }
  }
  if (rem > 0) {
    double frac = -1.0;
    int fl_i = 0;
    if (active) {
      const double fl = floor(raw);
      frac = raw - fl;
      fl_i = (int)fl;
      quo += fl_i;
    }
    int left = rem - wave_sum(fl_i);
    // one extra each, largest fractional part first, equal parts by lower segment index
    while (left > 0) {
      const bool can = active && quo < len;
      const uint64_t cm = __ballot(can);
      if (!cm) break;
      int rank = 0;
      for (uint64_t m = cm; m; m &= m - 1) {
        const int j = __ffsll((long long)m) - 1;
        const double fj = __shfl(frac, j);
        if (fj > frac || (fj == frac && j < lane)) ++rank;
      }
      const bool take = can && rank < left;
      if (take) ++quo;
      left -= __popcll(__ballot(take));
    }
  }
  return quo;
}

// Quotas for up to 1024 segments by the first BLOCK threads of a workgroup (BLOCK == 64: its first wave
// alone; otherwise BLOCK must be the whole workgroup), the segments in LDS.  Integer
// sums are order-free; the sum of the masses of the open segments is taken by one thread in index
// order, the same order as plain C, so that every share is the same double.  The quotas are left in
// sc.quo (valid after the final barrier inside).
constexpr int kQuotaMaxSeg = 1024;
struct QuotaScratch {
  int32_t len[kQuotaMaxSeg], room[kQuotaMaxSeg], quo[kQuotaMaxSeg];
  double mass_d[kQuotaMaxSeg], raw[kQuotaMaxSeg];
  __attribute__((aligned(16))) double key[kQuotaMaxSeg];
  uint8_t active[kQuotaMaxSeg], can[kQuotaMaxSeg];
  int red[16];
  double msum;
};

// Barrier between the steps of quota_block: a workgroup barrier, or for BLOCK == 64 (one wave runs the whole
// routine, the other waves of the workgroup do not take part) only the ordering of the wave's own LDS accesses.
template <int BLOCK>
__device__ __forceinline__ void quota_sync() {
  if constexpr (BLOCK == 64) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  } else {
    __syncthreads();
  }
}

template <int BLOCK>
__device__ __forceinline__ int block_sum_int(int v, int* sm) {
  v = wave_sum(v);
  if constexpr (BLOCK == 64) {
    quota_sync<64>();  // the callers rely on a barrier's ordering of their LDS accesses here
    return v;
  }
  __syncthreads();  // sm may still be read from a previous call
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
  __syncthreads();
  int t = 0;
#pragma unroll
  for (int w = 0; w < BLOCK / 64; ++w) t += sm[w];
  return t;
}

template <int BLOCK>
__device__ __forceinline__ void quota_block(int S, int bud, int q_min, const int32_t* bounds, const float* mass,
                                            QuotaScratch& sc) {
  int c_nonempty = 0, c_need = 0;
  for (int i = threadIdx.x; i < S; i += BLOCK) {
    sc.len[i] = bounds[i + 1] - bounds[i];
    sc.mass_d[i] = (double)mass[i];
    c_nonempty += sc.len[i] > 0;
    c_need += min(q_min, sc.len[i]);
  }
  const int nonempty = block_sum_int<BLOCK>(c_nonempty, sc.red);
  const int need = block_sum_int<BLOCK>(c_need, sc.red);
  int floor_q = q_min;
  if (need > bud) floor_q = nonempty > 0 ? bud / nonempty : 0;
  int c_lo = 0;
  for (int i = threadIdx.x; i < S; i += BLOCK) {
    const int lo = min(floor_q, sc.len[i]);
    sc.room[i] = sc.len[i] - lo;
    sc.active[i] = sc.room[i] > 0;
    sc.quo[i] = lo;
    sc.raw[i] = 0.0;
    c_lo += lo;
  }
  int rem = bud - block_sum_int<BLOCK>(c_lo, sc.red);
  // proportional shares; a segment whose share reaches its room is filled and leaves the pool
  for (;;) {
    int c_act = 0;
    for (int i = threadIdx.x; i < S; i += BLOCK) c_act += sc.active[i];
    const int n_active = block_sum_int<BLOCK>(c_act, sc.red);
    if (n_active == 0 || rem <= 0) break;
    if (threadIdx.x == 0) {
      // index order; a closed segment adds an exact zero, so the loads need not wait for the flags
      double msum = 0.0;
#pragma unroll 8
      for (int i = 0; i < S; ++i) {
        const double md = sc.mass_d[i];
        const bool open = sc.active[i] != 0;
        msum += open ? md : 0.0;
      }
      sc.msum = msum;
    }
    quota_sync<BLOCK>();
    const double msum = sc.msum;
    int c_sat = 0, c_taken = 0;
    for (int i = threadIdx.x; i < S; i += BLOCK)
      if (sc.active[i]) {
        sc.raw[i] = msum > 0.0 ? (double)rem * sc.mass_d[i] / msum : (double)rem / (double)n_active;
        if (sc.raw[i] >= (double)sc.room[i]) {
          sc.quo[i] = sc.len[i];
          sc.active[i] = 0;
          ++c_sat;
          c_taken += sc.room[i];
        }
      }
    const int n_sat = block_sum_int<BLOCK>(c_sat, sc.red);
    rem -= block_sum_int<BLOCK>(c_taken, sc.red);
    if (n_sat == 0) break;
  }
  if (rem > 0) {
    int c_given = 0;
    for (int i = threadIdx.x; i < S; i += BLOCK)
      if (sc.active[i]) {
        const double fl = floor(sc.raw[i]);
        sc.raw[i] -= fl;  // now the fractional part
        sc.quo[i] += (int)fl;
        c_given += (int)fl;
      }
    int left = rem - block_sum_int<BLOCK>(c_given, sc.red);
    // one extra each, largest fractional part first, equal parts by lower segment index
    while (left > 0) {
      int c_can = 0;
      // key = the fractional part of a segment that can still take one, -1 for the others (a fraction
      // is never negative), padded to a multiple of four entries: the ranking loop then reads one array,
      // four entries at a time, without waiting for flags
      const int S4 = (S + 3) & ~3;
      for (int i = threadIdx.x; i < S4; i += BLOCK) {
        const bool c = i < S && sc.active[i] && sc.quo[i] < sc.len[i];
        if (i < S) sc.can[i] = c;
        sc.key[i] = c ? sc.raw[i] : -1.0;
        c_can += c;
      }
      const int n_can = block_sum_int<BLOCK>(c_can, sc.red);
      if (n_can == 0) break;
      int c_take = 0;
      for (int i = threadIdx.x; i < S; i += BLOCK)
        if (sc.can[i]) {
          int rank = 0;
          if (n_can > left) {  // otherwise everybody is served
            const double fi = sc.key[i];
            for (int j = 0; j < S4; j += 4) {
              const double k0 = sc.key[j], k1 = sc.key[j + 1], k2 = sc.key[j + 2], k3 = sc.key[j + 3];
              rank += (k0 > fi || (k0 == fi && j < i)) ? 1 : 0;
              rank += (k1 > fi || (k1 == fi && j + 1 < i)) ? 1 : 0;
              rank += (k2 > fi || (k2 == fi && j + 2 < i)) ? 1 : 0;
              rank += (k3 > fi || (k3 == fi && j + 3 < i)) ? 1 : 0;
            }
          }
          if (rank < left) {
            ++sc.quo[i];
            ++c_take;
          }
        }
      left -= block_sum_int<BLOCK>(c_take, sc.red);
    }
  }
  quota_sync<BLOCK>();
}

}  // namespace ams
#endif
