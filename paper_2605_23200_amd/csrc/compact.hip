// Gather-compact of the kept rows (Alg. 1 step 6: K' = K[idx], V' = V[idx]); with a paged
// destination this is the head-wise compaction copy of App. E.  Pure byte movement: a row of
// head_dim elements is moved by row_bytes/16 consecutive lanes with 16-byte accesses, so every
// row is one fully used 256- or 512-byte burst on both sides.
#include "ams_internal.h"

namespace ams {
namespace {

constexpr int kBlock = 256;
constexpr int kRowsPerBlock = 64;

__global__ __launch_bounds__(kBlock) void compact_kernel(Dims d, KvDev ks, KvDev vs, KvDev kd, KvDev vd,
                                                         int budget, const int32_t* idx_all,
                                                         const int32_t* n_kept_all,
                                                         const float* credit_src, float* credit_dst) {
  const int unit = blockIdx.y;
  int l, b, h;
  unit_coords(d, unit, l, b, h);
  // a count above the budget or an index outside the cache (a caller's mistake when the stage is
  // used on its own) must not turn into an access outside the buffers: the count is clamped and
  // such a row is skipped
  const int n = min(n_kept_all[unit], min(budget, d.t_max));
  const int j0 = blockIdx.x * kRowsPerBlock;
  if (j0 >= n) return;
  const int32_t* idx = idx_all + (int64_t)unit * budget;
  const int lanes_per_row = ks.row_bytes / 16;
  const int rows_per_pass = kBlock / lanes_per_row;
  const int sub = threadIdx.x % lanes_per_row, r = threadIdx.x / lanes_per_row;
  for (int jj = r; jj < kRowsPerBlock; jj += rows_per_pass) {
    const int j = j0 + jj;
    if (j >= n) break;
    const int t = idx[j];
    if (t < 0 || t >= d.t_max) continue;
    const uint4 kx = *(const uint4*)(kv_row(ks, l, b, h, t) + sub * 16);
    const uint4 vx = *(const uint4*)(kv_row(vs, l, b, h, t) + sub * 16);
    *(uint4*)(kv_row(kd, l, b, h, j) + sub * 16) = kx;
    *(uint4*)(kv_row(vd, l, b, h, j) + sub * 16) = vx;
  }
  if (credit_src && credit_dst && threadIdx.x < kRowsPerBlock) {
    const int j = j0 + threadIdx.x;
    if (j < n && idx[j] >= 0 && idx[j] < d.t_max)
      credit_dst[(int64_t)unit * budget + j] = credit_src[(int64_t)unit * d.t_stride + idx[j]];
  }
}

}  // namespace

hipError_t launch_compact(const ams_params* p, const Dims& d, const KvDev& ks, const KvDev& vs,
                          const KvDev& kd, const KvDev& vd, const int32_t* idx, const int32_t* n_kept,
                          const float* credit_src, float* credit_dst, hipStream_t s) {
  const int max_keep = p->budget < d.t_max ? p->budget : d.t_max;
  const dim3 grid((max_keep + kRowsPerBlock - 1) / kRowsPerBlock, d.units);
  prof_mark("compact", s);
  hipLaunchKernelGGL(compact_kernel, grid, dim3(kBlock), 0, s, d, ks, vs, kd, vd, p->budget, idx, n_kept,
                     credit_src, credit_dst);
  return hipGetLastError();
}

}  // namespace ams
