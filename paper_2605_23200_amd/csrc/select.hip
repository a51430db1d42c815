// Segment quotas, in-segment top-k and the kept set (Sec. 3.3 "Segment-wise Quota Allocation",
// "In-Segment Selection" and the must-keep rules; Alg. 1 steps 4-5).
//
// quota_kernel   one wave per unit (up to 64 segments in registers, up to 1024 in LDS); the
//                arithmetic is a handful of double operations per segment and is done in index
//                order so that it is reproducible bit for bit.
// select_kernel  one workgroup per (segment, unit): radix select (4 x 8 bits, most significant
//                digit first) of the quota-th largest score on an order-preserving integer image
//                of the floats, then an ordered compaction that keeps everything above the
//                threshold and the first few positions equal to it, ascending.
// finalize_kernel  (only with a must-keep set) one workgroup per unit.  The segment picks arrive as
//                bits of a per-unit bitmap, so the union with the must-keep positions and the removal
//                of duplicates are one OR; what the duplicates leave open is filled with the best
//                scores outside the set (another radix select, over the unset positions), and the
//                ascending index list is read off the bitmap.
#include "ams_internal.h"
#include "quota.h"

namespace ams {
namespace {

constexpr int kMaxSeg = 1024;

// What both quota kernels do before the quotas: the -1 tail of idx, the kept count, the cleared bitmap of the
// must-keep path.  Returns the budget the segments share.
__device__ __forceinline__ int quota_prologue(const Dims& d, const int32_t* seq_lens, int budget,
                                              int32_t* idx_all, int32_t* n_kept_all, int n_sink, int n_last,
                                              uint32_t* flags_all, int n_words) {
  const int unit = blockIdx.x, nthr = blockDim.x;
  int l, b, h;
  unit_coords(d, unit, l, b, h);
  const int T = seq_len(d, seq_lens, b);
  // must-keep positions go in first: sinks always, the recent suffix as far as it fits; the segments
  // share what is left
  const int kept = min(budget, T);
  const int sinks = min(n_sink, kept);
  const int bud = kept - sinks - min(n_last, kept - sinks);
  int32_t* idx = idx_all + (int64_t)unit * budget;
  // entries of idx beyond the kept count are -1
  for (int j = kept + threadIdx.x; j < budget; j += nthr) idx[j] = -1;
  if (threadIdx.x == 0) n_kept_all[unit] = kept;
  if (flags_all)
    for (int j = threadIdx.x; j < n_words; j += nthr) flags_all[(int64_t)unit * n_words + j] = 0u;
  return bud;
}

// Up to 64 segments: one wave per unit.
__global__ __launch_bounds__(64) void quota_kernel(Dims d, const int32_t* seq_lens, int S, int budget,
                                                   int q_min, const int32_t* bounds_all,
                                                   float* seg_mass_all, int32_t* quota_all,
                                                   int32_t* idx_all, int32_t* n_kept_all, int n_sink, int n_last,
                                                   uint32_t* flags_all, int n_words) {
  const int unit = blockIdx.x;
  const int bud = quota_prologue(d, seq_lens, budget, idx_all, n_kept_all, n_sink, n_last, flags_all, n_words);
  const int q = quota_wave(S, bud, q_min, bounds_all + (int64_t)unit * (S + 1), seg_mass_all + (int64_t)unit * S);
  if ((int)threadIdx.x < S) quota_all[(int64_t)unit * S + threadIdx.x] = q;
}

// More than 64 segments (up to 1024): one wave per unit as well, the segments in LDS.
constexpr int kQuotaBlock = 64;

__global__ __launch_bounds__(kQuotaBlock) void quota_block_kernel(Dims d, const int32_t* seq_lens, int S,
                                                                  int budget, int q_min,
                                                                  const int32_t* bounds_all, float* seg_mass_all,
                                                                  int32_t* quota_all, int32_t* idx_all,
                                                                  int32_t* n_kept_all, int n_sink, int n_last,
                                                                  uint32_t* flags_all, int n_words) {
  __shared__ QuotaScratch sc;
  const int unit = blockIdx.x;
  const int bud = quota_prologue(d, seq_lens, budget, idx_all, n_kept_all, n_sink, n_last, flags_all, n_words);
  quota_block<kQuotaBlock>(S, bud, q_min, bounds_all + (int64_t)unit * (S + 1), seg_mass_all + (int64_t)unit * S, sc);
  for (int i = threadIdx.x; i < S; i += kQuotaBlock) quota_all[(int64_t)unit * S + i] = sc.quo[i];
}

// Order-preserving image of a score: larger float <-> larger unsigned; -0 and +0 coincide and
// NaN ranks with -infinity.
__device__ __forceinline__ uint32_t score_key(float x) {
  if (x != x) x = -INFINITY;
  if (x == 0.f) x = 0.f;
  const uint32_t b = __float_as_uint(x);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Where a selected position goes: slot `slot` of the ascending index list, or its bit of the bitmap.
template <bool FLAGS>
struct Emit {
  int32_t* out;
  uint32_t* flags;
  __device__ __forceinline__ void operator()(int slot, int t) const {
    if (FLAGS)
      atomicOr(&flags[t >> 5], 1u << (t & 31));
    else
      out[slot] = t;
  }
};

// 3968 keys + the four histograms come to 19.6 KB: eight workgroups fit the LDS of a CU (4096 keys: seven,
// and the 4096 workgroups of the headline workload then need three rounds instead of two)
constexpr int kSelectCap = 3968;

// The selection kernel comes in two shapes: 256 threads with room for 3968 keys in LDS (segments of
// thousands of positions) and one wave with room for 1024 keys (many short segments: more workgroups
// per compute unit and no barriers between waves).  BLOCK = threads, CAP = segment lengths up to
// which the keys are selected from a copy in LDS.

// Segment longer than the LDS staging area: the scores are re-read from memory for every pass.
template <bool FLAGS, int BLOCK>
__device__ void select_from_memory(const float* g, int a, int b, int q, const Emit<FLAGS>& emit, int* hist,
                                   uint32_t* sel_prefix, int* sel_rem, int2* wave_cnt) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // radix select of the q-th largest key, 8 bits at a time from the top
  uint32_t prefix = 0, mask = 0;
  int rem = q;
  for (int shift = 24; shift >= 0; shift -= 8) {
    for (int i = threadIdx.x; i < 256; i += BLOCK) hist[i] = 0;
    __syncthreads();
    for (int t = a + threadIdx.x; t < b; t += BLOCK) {
      const uint32_t k = score_key(g[t]);
      if ((k & mask) == prefix) atomicAdd(&hist[(k >> shift) & 255], 1);
    }
    __syncthreads();
    if (wave == 0) {
      int hb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) hb[i] = hist[lane * 4 + i];
      const int s = hb[0] + hb[1] + hb[2] + hb[3];
      int incl = s;  // sum over lanes >= this one
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_down(incl, o);
        if (lane + o < 64) incl += v;
      }
      int cum = incl - s;  // keys in bins above this lane's
#pragma unroll
      for (int i = 3; i >= 0; --i) {
        if (cum < rem && rem <= cum + hb[i]) {
          *sel_prefix = prefix | ((uint32_t)(lane * 4 + i) << shift);
          *sel_rem = rem - cum;
        }
        cum += hb[i];
      }
    }
    __syncthreads();
    prefix = *sel_prefix;
    rem = *sel_rem;
    mask |= 0xFFu << shift;
    __syncthreads();
  }
  // prefix = key of the q-th largest score; rem = how many of the keys equal to it are kept
  const uint32_t thr = prefix;
  int base_gt = 0, base_eq = 0;  // counts over the positions before the current tile
  for (int t0 = a; t0 < b; t0 += BLOCK) {
    const int t = t0 + threadIdx.x;
    uint32_t k = 0;
    const bool in = t < b;
    if (in) k = score_key(g[t]);
    const bool gt = in && k > thr, eq = in && k == thr;
    const uint64_t bgt = __ballot(gt), beq = __ballot(eq);
    const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    if (lane == 0) wave_cnt[wave] = make_int2(__popcll(bgt), __popcll(beq));
    __syncthreads();
    int n_gt = base_gt + __popcll(bgt & below), n_eq = base_eq + __popcll(beq & below);
    int tot_gt = 0, tot_eq = 0;
#pragma unroll
    for (int w = 0; w < (BLOCK / 64); ++w) {
      const int2 c = wave_cnt[w];
      if (w < wave) {
        n_gt += c.x;
        n_eq += c.y;
      }
      tot_gt += c.x;
      tot_eq += c.y;
    }
    if (gt || (eq && n_eq < rem)) emit(n_gt + min(n_eq, rem), t);
    base_gt += tot_gt;
    base_eq += tot_eq;
    __syncthreads();
  }
}

template <bool FLAGS, int BLOCK, int CAP>
__global__ __launch_bounds__(BLOCK) void select_kernel(Dims d, int S, int budget, const float* g_all,
                                                           const int32_t* bounds_all,
                                                           const int32_t* quota_all, int32_t* idx_all,
                                                           uint32_t* flags_all, int n_words) {
  __shared__ uint32_t keys[CAP];
  __shared__ int hist[(BLOCK / 64)][256];
  __shared__ uint32_t sel_prefix;
  __shared__ int sel_rem;
  __shared__ int2 wave_cnt[(BLOCK / 64)];
  __shared__ uint32_t red_and[(BLOCK / 64)], red_or[(BLOCK / 64)];
  const int unit = blockIdx.y, seg = blockIdx.x;
  const int32_t* bounds = bounds_all + (int64_t)unit * (S + 1);
  const int32_t* quota = quota_all + (int64_t)unit * S;
  const int a = bounds[seg], b = bounds[seg + 1], q = quota[seg];
  if (q <= 0) return;
  int out0 = 0;  // place of this segment's picks in the index list: the quotas before it
  if (!FLAGS) {
    for (int i = threadIdx.x; i < seg; i += BLOCK) out0 += quota[i];
    out0 = wave_sum(out0);
    if ((threadIdx.x & 63) == 0) wave_cnt[threadIdx.x >> 6].x = out0;
    __syncthreads();
    out0 = 0;
#pragma unroll
    for (int w = 0; w < BLOCK / 64; ++w) out0 += wave_cnt[w].x;
    __syncthreads();
  }
  const float* g = g_all + (int64_t)unit * d.t_stride;
  const Emit<FLAGS> emit{idx_all + (int64_t)unit * budget + out0,
                         FLAGS ? flags_all + (int64_t)unit * n_words : nullptr};
  const int L = b - a;
  if (q >= L) {  // whole segment kept
    for (int j = threadIdx.x; j < L; j += BLOCK) emit(j, a + j);
    return;
  }
  if (L > CAP) {
    select_from_memory<FLAGS, BLOCK>(g, a, b, q, emit, &hist[0][0], &sel_prefix, &sel_rem, wave_cnt);
    return;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  // keys of the segment -> LDS; bits that are the same in every key need no radix pass
  uint32_t k_and = 0xFFFFFFFFu, k_or = 0;
  for (int e = threadIdx.x; e < L; e += BLOCK) {
    const uint32_t k = score_key(g[a + e]);
    keys[e] = k;
    k_and &= k;
    k_or |= k;
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    k_and &= __shfl_xor(k_and, o);
    k_or |= __shfl_xor(k_or, o);
  }
  if (lane == 0) {
    red_and[wave] = k_and;
    red_or[wave] = k_or;
  }
  __syncthreads();
  k_and = red_and[0];
  k_or = red_or[0];
#pragma unroll
  for (int w = 1; w < BLOCK / 64; ++w) {
    k_and &= red_and[w];
    k_or |= red_or[w];
  }
  const uint32_t diff = k_and ^ k_or;
  uint32_t thr = k_and;  // all keys equal: the threshold is that key
  int rem = q;
  if (diff != 0) {
    const int hb = 31 - __clz(diff);  // highest bit in which two keys differ
    uint32_t mask = hb == 31 ? 0u : ~((2u << hb) - 1u);  // bits known so far
    uint32_t prefix = k_and & mask;
    int shift = max(hb - 7, 0);
    for (;;) {
      for (int i = threadIdx.x; i < (BLOCK / 64) * 256; i += BLOCK) (&hist[0][0])[i] = 0;
      __syncthreads();
      for (int e = threadIdx.x; e < L; e += BLOCK) {
        const uint32_t k = keys[e];
        if ((k & mask) == prefix) atomicAdd(&hist[wave][(k >> shift) & 255], 1);
      }
      __syncthreads();
      if (wave == 0) {
        int hbin[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          hbin[i] = 0;
#pragma unroll
          for (int w = 0; w < (BLOCK / 64); ++w) hbin[i] += hist[w][lane * 4 + i];
        }
        const int s = hbin[0] + hbin[1] + hbin[2] + hbin[3];
        int incl = s;  // sum over lanes >= this one
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          const int v = __shfl_down(incl, o);
          if (lane + o < 64) incl += v;
        }
        int cum = incl - s;  // keys in bins above this lane's
#pragma unroll
        for (int i = 3; i >= 0; --i) {
          if (cum < rem && rem <= cum + hbin[i]) {
            sel_prefix = (uint32_t)(lane * 4 + i);
            sel_rem = rem - cum;
          }
          cum += hbin[i];
        }
      }
      __syncthreads();
      // the digit may overlap bits that are already known; OR-ing it in is then a no-op for those bits
      prefix |= sel_prefix << shift;
      rem = sel_rem;
      mask = shift == 0 ? 0xFFFFFFFFu : ~((1u << shift) - 1u);
      __syncthreads();
      if (shift == 0) break;
      shift = max(shift - 8, 0);
    }
    thr = prefix;
  }
  // thr = key of the q-th largest score; rem = how many of the keys equal to it are kept (the first
  // rem in position order).  Every thread takes a contiguous run of positions, so one workgroup scan
  // of the per-thread counts gives every kept position its place in the ascending output.
  const int per = (L + BLOCK - 1) / BLOCK;
  const int e0 = min(L, (int)threadIdx.x * per), e1 = min(L, e0 + per);
  int c_gt = 0, c_eq = 0;
  for (int e = e0; e < e1; ++e) {
    const uint32_t k = keys[e];
    c_gt += k > thr;
    c_eq += k == thr;
  }
  int i_gt = c_gt, i_eq = c_eq;  // inclusive scans within the wave
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int vg = __shfl_up(i_gt, o), ve = __shfl_up(i_eq, o);
    if (lane >= o) {
      i_gt += vg;
      i_eq += ve;
    }
  }
  if (lane == 63) wave_cnt[wave] = make_int2(i_gt, i_eq);
  __syncthreads();
  int n_gt = i_gt - c_gt, n_eq = i_eq - c_eq;
  for (int w = 0; w < wave; ++w) {
    n_gt += wave_cnt[w].x;
    n_eq += wave_cnt[w].y;
  }
  for (int e = e0; e < e1; ++e) {
    const uint32_t k = keys[e];
    if (k > thr) {
      emit(n_gt + min(n_eq, rem), a + e);
      ++n_gt;
    } else if (k == thr) {
      if (n_eq < rem) emit(n_gt + n_eq, a + e);
      ++n_eq;
    }
  }
}

// Bits of word w (positions 32w .. 32w+31) that lie in [lo, hi).
__device__ __forceinline__ uint32_t range_bits(int w, int lo, int hi) {
  const int a = max(lo - w * 32, 0), b = min(hi - w * 32, 32);
  if (a >= b) return 0u;
  const uint32_t upto_b = b == 32 ? 0xFFFFFFFFu : (1u << b) - 1u;
  return upto_b & ~((1u << a) - 1u);
}

constexpr int kFinBlock = 1024;
constexpr int kFinWaves = kFinBlock / 64;
constexpr int kFinPer = 32;  // positions per thread whose keys stay in registers (T <= 32768)

__global__ __launch_bounds__(kFinBlock) void finalize_kernel(Dims d, const int32_t* seq_lens, int budget,
                                                             int n_sink, int n_last, const float* g_all,
                                                             uint32_t* flags_all, int n_words,
                                                             int32_t* idx_all) {
  __shared__ int hist[kFinWaves][256];
  __shared__ uint32_t sel_digit;
  __shared__ int sel_rem;
  __shared__ int red[kFinWaves];
  __shared__ uint32_t red_and[kFinWaves], red_or[kFinWaves];
  __shared__ int2 wave_cnt[kFinWaves];
  __shared__ uint32_t bm[kFinBlock];  // the bitmap of a sequence of up to 32768 positions
  const int unit = blockIdx.x;
  int l, b, h;
  unit_coords(d, unit, l, b, h);
  const int T = seq_len(d, seq_lens, b);
  const int kept = min(budget, T);
  const int sinks = min(n_sink, kept);
  const int last = min(n_last, kept - sinks);
  const float* g = g_all + (int64_t)unit * d.t_stride;
  uint32_t* flags = flags_all + (int64_t)unit * n_words;
  int32_t* idx = idx_all + (int64_t)unit * budget;
  const int nw = (T + 31) >> 5;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // Up to 32768 positions the bitmap is worked on in LDS and the keys are read once into registers;
  // longer sequences keep the bitmap in memory and re-read the scores in every pass.
  const bool inreg = T <= kFinBlock * kFinPer;

  // union with the must-keep positions; size of the union
  int cnt = 0;
  if (inreg) bm[threadIdx.x] = 0u;
  for (int w = threadIdx.x; w < nw; w += kFinBlock) {
    const uint32_t f = flags[w] | range_bits(w, 0, sinks) | range_bits(w, T - last, T);
    if (inreg)
      bm[w] = f;
    else
      flags[w] = f;
    cnt += __popc(f);
  }
  cnt = wave_sum(cnt);
  if (lane == 0) red[wave] = cnt;
  __syncthreads();  // also orders the flag stores before the reads below
  cnt = 0;
#pragma unroll
  for (int w = 0; w < kFinWaves; ++w) cnt += red[w];
  const int deficit = kept - cnt;  // positions the duplicates left open; never negative
  const bool fill = deficit > 0;

  // Keys of the positions outside the set (0 = in the set or past the end; no score maps to 0).
  uint32_t kreg[kFinPer];
  auto key_at = [&](int t) __attribute__((always_inline)) -> uint32_t {
    if (t >= T) return 0u;
    const uint32_t word = inreg ? bm[t >> 5] : flags[t >> 5];
    return ((word >> (t & 31)) & 1u) ? 0u : score_key(g[t]);
  };
  if (fill && inreg) {
#pragma unroll
    for (int j = 0; j < kFinPer; ++j) kreg[j] = key_at(threadIdx.x + j * kFinBlock);
  }

  // key of the deficit-th largest score among the positions outside the set
  uint32_t thr = 0xFFFFFFFFu;
  int rem = 0;
  if (fill) {
    // bits that are the same in every key need no radix pass
    uint32_t k_and = 0xFFFFFFFFu, k_or = 0u;
    if (inreg) {
#pragma unroll
      for (int j = 0; j < kFinPer; ++j)
        if (kreg[j]) {
          k_and &= kreg[j];
          k_or |= kreg[j];
        }
    } else {
      for (int t = threadIdx.x; t < T; t += kFinBlock) {
        const uint32_t k = key_at(t);
        if (k) {
          k_and &= k;
          k_or |= k;
        }
      }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      k_and &= __shfl_xor(k_and, o);
      k_or |= __shfl_xor(k_or, o);
    }
    if (lane == 0) {
      red_and[wave] = k_and;
      red_or[wave] = k_or;
    }
    __syncthreads();
    k_and = 0xFFFFFFFFu;
    k_or = 0u;
#pragma unroll
    for (int w = 0; w < kFinWaves; ++w) {
      k_and &= red_and[w];
      k_or |= red_or[w];
    }
    const uint32_t diff = k_and ^ k_or;
    thr = k_and;  // all keys equal: the threshold is that key
    rem = deficit;
    if (diff != 0) {
      const int hb = 31 - __clz(diff);  // highest bit in which two keys differ
      uint32_t mask = hb == 31 ? 0u : ~((2u << hb) - 1u);  // bits known so far
      uint32_t prefix = k_and & mask;
      int shift = max(hb - 7, 0);
      for (;;) {
        for (int i = threadIdx.x; i < kFinWaves * 256; i += kFinBlock) (&hist[0][0])[i] = 0;
        __syncthreads();
        if (inreg) {
#pragma unroll
          for (int j = 0; j < kFinPer; ++j) {
            const uint32_t k = kreg[j];
            if (k && (k & mask) == prefix) atomicAdd(&hist[wave][(k >> shift) & 255], 1);
          }
        } else {
          for (int t = threadIdx.x; t < T; t += kFinBlock) {
            const uint32_t k = key_at(t);
            if (k && (k & mask) == prefix) atomicAdd(&hist[wave][(k >> shift) & 255], 1);
          }
        }
        __syncthreads();
        if (wave == 0) {
          int hbin[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            hbin[i] = 0;
#pragma unroll
            for (int w = 0; w < kFinWaves; ++w) hbin[i] += hist[w][lane * 4 + i];
          }
          const int s = hbin[0] + hbin[1] + hbin[2] + hbin[3];
          int incl = s;  // sum over lanes >= this one
#pragma unroll
          for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_down(incl, o);
            if (lane + o < 64) incl += v;
          }
          int cum = incl - s;  // keys in bins above this lane's
#pragma unroll
          for (int i = 3; i >= 0; --i) {
            if (cum < rem && rem <= cum + hbin[i]) {
              sel_digit = (uint32_t)(lane * 4 + i);
              sel_rem = rem - cum;
            }
            cum += hbin[i];
          }
        }
        __syncthreads();
        // the digit may overlap bits that are already known; OR-ing it in is then a no-op for those bits
        prefix |= sel_digit << shift;
        rem = sel_rem;
        mask = shift == 0 ? 0xFFFFFFFFu : ~((1u << shift) - 1u);
        __syncthreads();
        if (shift == 0) break;
        shift = max(shift - 8, 0);
      }
      thr = prefix;
    }
  }

  const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  if (inreg) {
    // the positions that fill the gap get their bits: everything above the threshold, and of the
    // positions equal to it the first rem in index order
    if (fill) {
      int c_eq = 0;
#pragma unroll
      for (int j = 0; j < kFinPer; ++j) c_eq += kreg[j] == thr;
      c_eq = wave_sum(c_eq);
      if (lane == 0) red[wave] = c_eq;
      __syncthreads();
      c_eq = 0;
#pragma unroll
      for (int w = 0; w < kFinWaves; ++w) c_eq += red[w];
      __syncthreads();  // red[] is written again below: every wave has read it first
      const bool all_eq = c_eq == rem;  // no choice to make among equal scores
#pragma unroll
      for (int j = 0; j < kFinPer; ++j) {
        const int t = threadIdx.x + j * kFinBlock;
        if (kreg[j] > thr || (all_eq && kreg[j] == thr)) atomicOr(&bm[t >> 5], 1u << (t & 31));
      }
      if (!all_eq) {
        int base_eq = 0;  // equal scores met so far, in index order (round j covers 1024 consecutive positions)
#pragma unroll
        for (int j = 0; j < kFinPer; ++j) {
          if (j * kFinBlock < T && base_eq < rem) {
            const int t = threadIdx.x + j * kFinBlock;
            const bool eq = kreg[j] == thr;
            const uint64_t be = __ballot(eq);
            if (lane == 0) red[wave] = __popcll(be);
            __syncthreads();
            int n_eq = base_eq + __popcll(be & below), tot = 0;
#pragma unroll
            for (int v = 0; v < kFinWaves; ++v) {
              if (v < wave) n_eq += red[v];
              tot += red[v];
            }
            if (eq && n_eq < rem) atomicOr(&bm[t >> 5], 1u << (t & 31));
            base_eq += tot;
            __syncthreads();
          }
        }
      }
      __syncthreads();
    }
    // ascending index list read off the bitmap: one word per thread
    const uint32_t f = bm[threadIdx.x];
    const int c = __popc(f);
    int incl = c;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int v = __shfl_up(incl, o);
      if (lane >= o) incl += v;
    }
    if (lane == 63) wave_cnt[wave].x = incl;
    __syncthreads();
    int slot = incl - c;
    for (int v = 0; v < wave; ++v) slot += wave_cnt[v].x;
    for (uint32_t m = f; m; m &= m - 1) idx[slot++] = threadIdx.x * 32 + __ffs((int)m) - 1;
    return;
  }

  // long sequences: one position per thread and round; a position is kept when its bit is set or its
  // score is above the threshold, and the first rem positions equal to the threshold join
  int base_keep = 0, base_eq = 0;
  for (int t0 = 0; t0 < T; t0 += kFinBlock) {
    const int t = t0 + threadIdx.x;
    bool keep = false, eq = false;
    if (t < T) {
      keep = (flags[t >> 5] >> (t & 31)) & 1u;
      if (fill && !keep) {
        const uint32_t k = score_key(g[t]);
        keep = k > thr;
        eq = k == thr;
      }
    }
    const uint64_t bk = __ballot(keep), be = __ballot(eq);
    if (lane == 0) wave_cnt[wave] = make_int2(__popcll(bk), __popcll(be));
    __syncthreads();
    int n_keep = base_keep + __popcll(bk & below), n_eq = base_eq + __popcll(be & below);
    int tot_keep = 0, tot_eq = 0;
#pragma unroll
    for (int v = 0; v < kFinWaves; ++v) {
      const int2 c = wave_cnt[v];
      if (v < wave) {
        n_keep += c.x;
        n_eq += c.y;
      }
      tot_keep += c.x;
      tot_eq += c.y;
    }
    if (keep)
      idx[n_keep + min(n_eq, rem)] = t;
    else if (eq && n_eq < rem)
      idx[n_keep + n_eq] = t;
    base_keep += tot_keep;
    base_eq += tot_eq;
    __syncthreads();
  }
}

}  // namespace

hipError_t launch_select(const ams_params* p, const Dims& d, const int32_t* seq_lens, const float* g,
                         const int32_t* bounds, float* seg_mass, int32_t* quota, int32_t* idx,
                         int32_t* n_kept, uint32_t* flags, int n_words, hipStream_t s, bool quota_done) {
  const int S = p->n_segments;
  if (S > kMaxSeg) return hipErrorInvalidValue;
  const bool must = p->n_sink > 0 || p->n_last > 0;
  if (must && !flags) return hipErrorInvalidValue;
  if (!quota_done) prof_mark("quota", s);
  if (quota_done) {
    // quotas, the tail of idx, the kept count and the cleared bitmap are already in place
  } else if (S <= 64)
    hipLaunchKernelGGL(quota_kernel, dim3(d.units), dim3(64), 0, s, d, seq_lens, S, p->budget, p->q_min,
                       bounds, seg_mass, quota, idx, n_kept, p->n_sink, p->n_last,
                       must ? flags : nullptr, n_words);
  else
    hipLaunchKernelGGL(quota_block_kernel, dim3(d.units), dim3(kQuotaBlock), 0, s, d, seq_lens, S, p->budget,
                       p->q_min, bounds, seg_mass, quota, idx, n_kept, p->n_sink,
                       p->n_last, must ? flags : nullptr, n_words);
  prof_mark("select", s);
  // expected segment length decides the shape of the selection workgroups
  const double expect = p->seg_delta > 0.f
                            ? (p->l_max > 0 ? (double)p->l_max : (double)p->t_max * (double)p->seg_delta)
                            : (double)p->t_max / (double)S;
  const bool small = expect <= 512.0;
  const dim3 grid(S, d.units);
  if (!must) {
    if (small)
      hipLaunchKernelGGL((select_kernel<false, 64, 1024>), grid, dim3(64), 0, s, d, S, p->budget, g, bounds, quota,
                         idx, nullptr, 0);
    else
      hipLaunchKernelGGL((select_kernel<false, 256, kSelectCap>), grid, dim3(256), 0, s, d, S, p->budget, g, bounds,
                         quota, idx, nullptr, 0);
    return hipGetLastError();
  }
  if (small)
    hipLaunchKernelGGL((select_kernel<true, 64, 1024>), grid, dim3(64), 0, s, d, S, p->budget, g, bounds, quota,
                       idx, flags, n_words);
  else
    hipLaunchKernelGGL((select_kernel<true, 256, kSelectCap>), grid, dim3(256), 0, s, d, S, p->budget, g, bounds, quota,
                       idx, flags, n_words);
  prof_mark("finalize", s);
  hipLaunchKernelGGL(finalize_kernel, dim3(d.units), dim3(kFinBlock), 0, s, d, seq_lens, p->budget, p->n_sink,
                     p->n_last, g, flags, n_words, idx);
  return hipGetLastError();
}

}  // namespace ams
