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

}  // namespace ams
#endif
