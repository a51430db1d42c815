// Building blocks of the scoring kernels: the MFMA tile s = K_tile . Q^T of one wave, the staging
// of the query window in LDS, and the cross-lane sum over the queries of a token.
// (Alg. 1 step 1: "aggregate usage of each cached position from the last W queries".)
#ifndef AMS_SCORE_TILE_H
#define AMS_SCORE_TILE_H

#include "ams_internal.h"

namespace ams {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

static constexpr float kNegInit = -3.0e38f;  // finite "minus infinity" for running maxima
static constexpr int kThreads = 256;

enum { MODE_MEAN = 0, MODE_LAST = 1, MODE_EXPECTED = 2 };

struct ScoreArgs {
  KvDev k;
  Dims d;
  const int32_t* seq_lens;
  const char* q;
  float2* part;  // [units][n_chunks + 1][n_pad]  (max, sum) in the log2 domain; the last entry of a
                 // unit takes the tail blocks of a causal window
  float4* fin;   // [units][n_pad]  (M, weight for u, weight for g, query is real)
  float* u;
  float* g;
  int n_chunks, n_pad;
  int chunk;         // tokens per workgroup: a multiple of 256, at most kScoreChunk
  float c2;          // log2(e) / sqrt(D)
  float inv_sqrt_d;  // 1 / sqrt(D)
  // optional by-products for Eq. (1) and the EMA (NULL: not wanted): per chunk the sum of
  // max(u,0)+eps from the second sweep; the unit's sum of the credit before the update, formed by the
  // kernel that merges the statistics and carried in the first chunk's entry
  double2* vc_part;     // [units][n_chunks]
  const float* credit;  // [units][t_stride]
  double* csum;         // [units]
  float eps;
  bool causal;  // causal window (App. A): query w of the window sees keys 0 .. T-W+w
  int32_t* status;  // word the one-read scorer raises when a bounded wait expires; the two-sweep path clears it
};

// Raises a kernel's dynamic LDS limit once per kernel and device (not before every launch).
template <auto Kernel>
inline hipError_t ensure_lds(int bytes) {
  constexpr int kMaxDevices = 64;
  static int granted[kMaxDevices] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (granted[dev] >= bytes) return hipSuccess;
  e = hipFuncSetAttribute((const void*)Kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) granted[dev] = bytes;
  return e;
}

// Row geometry of a cache of HD channels: bytes per row, stride of a query row in LDS (padded by
// 16 bytes against bank conflicts), 16-byte vectors per half row (what one lane feeds the MFMA).
template <bool BF16, int HD = 128>
struct Tr {
  static_assert(HD == 64 || HD == 128, "head dimensions the tiles are written for");
  static constexpr int kRowBytes = HD * (BF16 ? 2 : 4), kQStride = kRowBytes + 16, kAVecs = kRowBytes / 32;
};

// Query window of the unit -> LDS, rows padded against bank conflicts, rows >= N zero.
template <bool BF16, int NB, int HD = 128>
__device__ __forceinline__ void load_q(const ScoreArgs& a, int l, int b, int h, char* qlds) {
  constexpr int RB = Tr<BF16, HD>::kRowBytes, QS = Tr<BF16, HD>::kQStride, CPR = RB / 16;
  const char* src = a.q + ((((int64_t)l * a.d.B + b) * a.d.H + h) * a.d.G) * (int64_t)a.d.W * RB;
  for (int ch = threadIdx.x; ch < NB * 32 * CPR; ch += kThreads) {
    const int n = ch / CPR, col = ch % CPR;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (n < a.d.N) v = *(const uint4*)(src + (int64_t)n * RB + col * 16);
    *(uint4*)(qlds + n * QS + col * 16) = v;
  }
}

// Lane (r = lane % 32, hf = lane / 32) reads the hf-th half of row t0 + r: one contiguous piece
// (128 bytes for bf16 rows of 128 channels).  The contraction index is permuted the same way on
// the query side, which leaves the dot products unchanged.
template <bool BF16, int HD = 128>
__device__ __forceinline__ void load_a(const ScoreArgs& a, int l, int b, int h, int t0, int T,
                                       int lane, uint4 (&av)[Tr<BF16, HD>::kAVecs],
                                       const int32_t* blk_lds = nullptr, int blk_t0 = 0) {
  constexpr int NV = Tr<BF16, HD>::kAVecs;
  // rows past the end re-read the last row (no divergent branch); their logits are masked later
  const int t = min(t0 + (lane & 31), T - 1);
  const char* row;
  if (blk_lds) {
    // paged cache: the physical block numbers of the positions from blk_t0 (a multiple of 16) on
    // were staged in LDS, so the row address does not wait for a table entry from memory
    int64_t slot = (int64_t)blk_lds[(t - blk_t0) >> 4] * 16 + (t & 15);
    slot = slot < 0 ? 0 : (slot >= a.k.n_slots ? a.k.n_slots - 1 : slot);
    row = a.k.base + (((int64_t)l * a.k.n_slots + slot) * a.k.H + h) * (int64_t)a.k.row_bytes;
  } else {
    row = kv_row(a.k, l, b, h, t);
  }
  const uint4* p = (const uint4*)(row + (lane >> 5) * (Tr<BF16, HD>::kRowBytes / 2));
#pragma unroll
  for (int i = 0; i < NV; ++i) av[i] = p[i];
}

// Paged cache: block numbers of the positions [c0, t_lim) of sequence b -> LDS (c0 a multiple of 16).
__device__ __forceinline__ void stage_blocks(const ScoreArgs& a, int b, int c0, int t_lim, int32_t* blk_lds) {
  const int n = (t_lim - c0 + 15) >> 4;
  for (int i = threadIdx.x; i < n; i += kThreads)
    blk_lds[i] = a.k.block_table[(int64_t)b * a.k.max_blocks + (c0 >> 4) + i];
  __syncthreads();
}

// acc[nb][i] = s_raw[token 8*(i/4) + 4*hf + i%4][query nb*32 + lane%32]
template <bool BF16, int NB, int HD = 128>
__device__ __forceinline__ void tile_mma(const uint4 (&av)[Tr<BF16, HD>::kAVecs], const char* qlds,
                                         int lane, floatx16 (&acc)[NB]) {
  constexpr int QS = Tr<BF16, HD>::kQStride, NV = Tr<BF16, HD>::kAVecs;
  const char* qb = qlds + (lane & 31) * QS + (lane >> 5) * (Tr<BF16, HD>::kRowBytes / 2);
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[nb][i] = 0.f;
  if constexpr (BF16) {
#pragma unroll
    for (int ks = 0; ks < NV; ++ks) {
      const bf16x8 A = __builtin_bit_cast(bf16x8, av[ks]);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const uint4 bv = *(const uint4*)(qb + nb * 32 * QS + ks * 16);
        acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, __builtin_bit_cast(bf16x8, bv), acc[nb], 0, 0, 0);
      }
    }
  } else {
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const float4 A = __builtin_bit_cast(float4, av[j]);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const float4 bv = *(const float4*)(qb + nb * 32 * QS + j * 16);
        acc[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(A.x, bv.x, acc[nb], 0, 0, 0);
        acc[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(A.y, bv.y, acc[nb], 0, 0, 0);
        acc[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(A.z, bv.z, acc[nb], 0, 0, 0);
        acc[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(A.w, bv.w, acc[nb], 0, 0, 0);
      }
    }
  }
}

__device__ __forceinline__ int acc_row(int i, int hf) { return 8 * (i >> 2) + 4 * hf + (i & 3); }

// Software pipeline over the column blocks of a tile (bf16 caches): the query fragments of a column
// block are read from LDS a whole column block before the matrix instructions that use them, and the
// matrix instructions of column block nb + 1 are issued between the vector instructions that consume
// column block nb.  A wave then neither waits for LDS in front of every MFMA nor leaves one of the
// two pipes idle while it uses the other.
//   col_frags   this lane's 16-byte query fragments of one column block -> registers
//   col_mma     acc = K_block . Q_col^T from fragments in registers
//   col_hints   scheduling hints for one step of the pipeline (STEPS matrix instructions, each
//               followed by VALU_PER vector and TRANS_PER transcendental instructions)
template <bool BF16, int HD = 128>
__device__ __forceinline__ void col_frags(const char* qb, uint4 (&bq)[Tr<BF16, HD>::kAVecs]) {
#pragma unroll
  for (int ks = 0; ks < Tr<BF16, HD>::kAVecs; ++ks) bq[ks] = *(const uint4*)(qb + ks * 16);
}
template <bool BF16, int HD = 128>
__device__ __forceinline__ void col_mma(const uint4 (&av)[Tr<BF16, HD>::kAVecs],
                                        const uint4 (&bq)[Tr<BF16, HD>::kAVecs], floatx16& acc) {
  static_assert(BF16, "the pipelined walk is written for bf16 caches");
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
  for (int ks = 0; ks < Tr<BF16, HD>::kAVecs; ++ks)
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av[ks]), __builtin_bit_cast(bf16x8, bq[ks]),
                                                  acc, 0, 0, 0);
}
template <int STEPS, int VALU_PER, int TRANS_PER, bool READS>
__device__ __forceinline__ void col_hints() {
  if (READS) __builtin_amdgcn_sched_group_barrier(0x100, STEPS, 0);  // the LDS reads of the column block after next, first
#pragma unroll
  for (int i = 0; i < STEPS; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);         // MFMA
    __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER, 0);  // vector ALU
    if (TRANS_PER > 0) __builtin_amdgcn_sched_group_barrier(0x400, TRANS_PER, 0);  // exp2
  }
}

// Sum (or maximum) of 16 per-lane values over the 32 lanes of a half wave, halving the number of live values
// at every exchange.  Lane c ends up with the total of value index c >> 1.
// Exchanges: rows of 16 lanes swap through v_permlane16_swap (bit 4 of the lane), then DPP
// row_ror:8 (bit 3), row_half_mirror (lane <-> 7 - lane inside groups of 8: the partner has the
// opposite bit 2), quad_perm xor 2 (bit 1) and xor 1; no LDS traffic.
__device__ __forceinline__ float dpp_ror8(float x) {
  return __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), 0x128, 0xf, 0xf, true));
}
__device__ __forceinline__ float dpp_half_mirror(float x) {
  return __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), 0x141, 0xf, 0xf, true));
}
__device__ __forceinline__ float dpp_xor2(float x) {
  return __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), 0x4E, 0xf, 0xf, true));
}
__device__ __forceinline__ float dpp_xor1(float x) {
  return __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), 0xB1, 0xf, 0xf, true));
}
template <bool MAX = false>
__device__ __forceinline__ float reduce16_over32(const float (&v)[16], int c) {
  auto op = [](float x, float y) __attribute__((always_inline)) { return MAX ? fmaxf(x, y) : x + y; };
  float w8[8], w4[4], w2[2];
  const bool b3 = c & 8, b2 = c & 4, b1 = c & 2;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    // even rows receive the partner row's v[j], odd rows the partner row's v[j + 8]
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v[j]), __float_as_uint(v[j + 8]), false, false);
    w8[j] = op(__uint_as_float(r[0]), __uint_as_float(r[1]));
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float keep = b3 ? w8[j + 4] : w8[j], send = b3 ? w8[j] : w8[j + 4];
    w4[j] = op(keep, dpp_ror8(send));
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const float keep = b2 ? w4[j + 2] : w4[j], send = b2 ? w4[j] : w4[j + 2];
    w2[j] = op(keep, dpp_half_mirror(send));
  }
  const float keep = b1 ? w2[1] : w2[0], send = b1 ? w2[0] : w2[1];
  const float w1 = op(keep, dpp_xor2(send));
  return op(w1, dpp_xor1(w1));
}

}  // namespace ams
#endif
