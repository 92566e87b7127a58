// Device helpers shared by the bf16 scoring kernels (one kernel per stage, and one
// workgroup per problem).
#pragma once

#include "finch_internal.h"

namespace finch {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr float kInf = __builtin_inff();

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

__device__ __forceinline__ int round_up32(int x) { return (x + 31) & ~31; }

// Merge two (max, sum) pairs of a running softmax in the log2 domain.
__device__ __forceinline__ void merge_stats(float& m, float& z, float m2, float z2) {
  const float mm = fmaxf(m, m2);
  if (mm == -kInf) {
    z = 0.f;
  } else {
    z = z * fast_exp2(m - mm) + z2 * fast_exp2(m2 - mm);
  }
  m = mm;
}

// log2-domain log-sum-exp of a row widened by keys outside the candidates whose
// natural-log log-sum-exp is extra_ln (-inf: none).
__device__ __forceinline__ float widen_lse(float lse2, float extra_ln) {
  const float e2 = extra_ln * 1.4426950408889634f;
  const float mx = fmaxf(lse2, e2);
  if (mx == -kInf) return lse2;
  return mx + fast_log2(fast_exp2(lse2 - mx) + fast_exp2(e2 - mx));
}

// Key (row of the 32x32 logit block) held in accumulator register v of a lane in
// lane-half h.
__device__ __forceinline__ int acc_key(int v, int h) { return 8 * (v >> 2) + 4 * h + (v & 3); }

// One 32-key block of K as MFMA A operands: lane (t, h) holds row kbase + t,
// elements 16*s + 8*h .. +7 of it for k-step s.  Rows at or past N are zeros.
template <int D>
__device__ __forceinline__ void load_k_block(const finch_problem& pb, int N, int kbase, int lane,
                                             bf16x8 (&kf)[D / 16]) {
  const int key = kbase + (lane & 31);
  const int h = lane >> 5;
  if (key < N) {
    const char* row = key < pb.c
                          ? static_cast<const char*>(pb.k_cache) + static_cast<size_t>(key) * (D * 2)
                          : static_cast<const char*>(pb.k_chunk) +
                                static_cast<size_t>(key - pb.c) * (D * 2);
    const FINCH_GLOBAL u32x4* rp = as_global<u32x4>(row);
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      const u32x4 raw = rp[2 * s + h];
      kf[s] = __builtin_bit_cast(bf16x8, raw);
    }
  } else {
    const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int s = 0; s < D / 16; ++s) kf[s] = __builtin_bit_cast(bf16x8, zero);
  }
}

// Values that are the same in every lane, moved into scalar registers (used where
// the compiler cannot see the uniformity, e.g. arguments of non-inlined functions).
__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ float uni(float x) {
  return __uint_as_float(static_cast<unsigned>(__builtin_amdgcn_readfirstlane(static_cast<int>(__float_as_uint(x)))));
}
template <typename T>
__device__ __forceinline__ T* uni(T* p) {
  const unsigned long long v = reinterpret_cast<unsigned long long>(p);
  const unsigned lo = static_cast<unsigned>(__builtin_amdgcn_readfirstlane(static_cast<int>(v)));
  const unsigned hi = static_cast<unsigned>(__builtin_amdgcn_readfirstlane(static_cast<int>(v >> 32)));
  return reinterpret_cast<T*>((static_cast<unsigned long long>(hi) << 32) | lo);
}

// Where the keys of a problem live: rows [0, c) in `cache`, the rest in `chunk`.
struct KeySource {
  const char* cache;
  const char* chunk;
  int c;
};

// load_k_block with the three descriptor fields it needs passed directly.
template <int D>
__device__ __forceinline__ void load_k_block(const KeySource& ks, int N, int kbase, int lane,
                                             bf16x8 (&kf)[D / 16]) {
  const int key = kbase + (lane & 31);
  const int h = lane >> 5;
  if (key < N) {
    const char* row = key < ks.c ? ks.cache + static_cast<size_t>(key) * (D * 2)
                                 : ks.chunk + static_cast<size_t>(key - ks.c) * (D * 2);
    const FINCH_GLOBAL u32x4* rp = as_global<u32x4>(row);
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      const u32x4 raw = rp[2 * s + h];
      kf[s] = __builtin_bit_cast(bf16x8, raw);
    }
  } else {
    const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int s = 0; s < D / 16; ++s) kf[s] = __builtin_bit_cast(bf16x8, zero);
  }
}

// Copy prompt rows [row0, row0+rows) into LDS, rows past R as zeros.  Row stride
// D*2+16 bytes keeps the 16-byte B-operand reads of 8 consecutive lanes on
// distinct banks.  NT = threads of the workgroup.
template <int D, int NT>
__device__ __forceinline__ void stage_q(const void* q, int R, int row0, int rows, char* lds_q,
                                        int tid) {
  constexpr int kSegs = D / 8;
  constexpr int kStride = D * 2 + 16;
  constexpr int kBatch = 4;  // loads in flight per thread
  const FINCH_GLOBAL u32x4* src = as_global<u32x4>(q);
  const int total = rows * kSegs;
  for (int i0 = tid; i0 < total; i0 += NT * kBatch) {
    u32x4 val[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int i = i0 + u * NT;
      const int row = i / kSegs;
      const int seg = i - row * kSegs;
      const u32x4 zero = {0u, 0u, 0u, 0u};
      val[u] = zero;
      if (i < total && row0 + row < R) val[u] = src[static_cast<size_t>(row0 + row) * kSegs + seg];
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int i = i0 + u * NT;
      const int row = i / kSegs;
      const int seg = i - row * kSegs;
      if (i < total) *reinterpret_cast<u32x4*>(lds_q + row * kStride + seg * 16) = val[u];
    }
  }
}

// B operands (prompt rows qb*32 .. +31) from LDS.
template <int D>
__device__ __forceinline__ void load_q_frags(const char* lds_q, int qb, int lane,
                                             bf16x8 (&qf)[D / 16]) {
  constexpr int kStride = D * 2 + 16;
  const char* qrow = lds_q + (qb * 32 + (lane & 31)) * kStride + 16 * (lane >> 5);
#pragma unroll
  for (int s = 0; s < D / 16; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(qrow + 32 * s);
}

// 32 keys x 32 rows of raw dot products: out[key][row], one prompt row per lane.
template <int D>
__device__ __forceinline__ f32x16 mfma_block(const bf16x8 (&kf)[D / 16], const bf16x8 (&qf)[D / 16]) {
  f32x16 a = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < D / 16; ++s) a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[s], a, 0, 0, 0);
  return a;
}

// Two 32x32 logit blocks of the same 32 keys against two blocks of 32 prompt rows,
// as two independent accumulation chains issued alternately (a chain's next
// instruction needs its previous result; two chains keep the matrix pipe fed).
template <int D>
__device__ __forceinline__ void mfma_block_pair(const bf16x8 (&kf)[D / 16], const bf16x8 (&qf0)[D / 16],
                                                const bf16x8 (&qf1)[D / 16], f32x16& a0, f32x16& a1) {
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  a0 = zero;
  a1 = zero;
#pragma unroll
  for (int s = 0; s < D / 16; ++s) {
    a0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf0[s], a0, 0, 0, 0);
    a1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf1[s], a1, 0, 0, 0);
  }
}

// The same with the prompt rows read from LDS inside the chain, one k-step ahead of
// the matrix instructions that use them (two 16-byte reads in flight while two
// matrix instructions run), so that the LDS latency is hidden without holding all
// sixteen operands in registers.  Row blocks qb and qb + 1.
template <int D>
__device__ __forceinline__ void mfma_block_pair_lds(const bf16x8 (&kf)[D / 16], const char* lds_q, int qb,
                                                    int lane, f32x16& a0, f32x16& a1) {
  constexpr int kStride = D * 2 + 16;
  const char* r0 = lds_q + (qb * 32 + (lane & 31)) * kStride + 16 * (lane >> 5);
  const char* r1 = r0 + 32 * kStride;
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  a0 = zero;
  a1 = zero;
  bf16x8 c0 = *reinterpret_cast<const bf16x8*>(r0);
  bf16x8 c1 = *reinterpret_cast<const bf16x8*>(r1);
#pragma unroll
  for (int s = 0; s < D / 16; ++s) {
    bf16x8 n0 = c0, n1 = c1;
    if (s + 1 < D / 16) {
      n0 = *reinterpret_cast<const bf16x8*>(r0 + 32 * (s + 1));
      n1 = *reinterpret_cast<const bf16x8*>(r1 + 32 * (s + 1));
    }
    a0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], c0, a0, 0, 0, 0);
    a1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], c1, a1, 0, 0, 0);
    // keep this order in the schedule: two LDS reads, then two matrix instructions
    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
    c0 = n0;
    c1 = n1;
  }
}

// A value of the lane that a DPP control names (row_ror:8 = lane ^ 8, row_half_mirror =
// lane ^ 7, quad_perm [2,3,0,1] = lane ^ 2, quad_perm [1,0,3,2] = lane ^ 1).
template <int CTRL>
__device__ __forceinline__ float from_lane_dpp(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}

// Sum each of 16 per-lane values over the 32 lanes of a lane-half.  On return the
// lane with in-half index t holds the total of value index t >> 1.  Fixed order.
// Five halving rounds: a lane keeps the half of its values that its own lane bit
// selects and adds the partner's sums of the same values.  The partners are lane ^ 16
// (one permlane16_swap per pair of values: the odd 16-lane rows of the first change
// places with the even rows of the second, after which the two registers hold exactly
// the two addends), then lane ^ 8, lane ^ 7, lane ^ 2, lane ^ 1 through DPP - no trip
// through the LDS crossbar, which the matrix operands keep busy.  (Any partner with the
// same higher bits and the opposite bit of the round will do: lane ^ 7 is what a
// single DPP control offers for the third round.)
__device__ __forceinline__ float fold16_over32(const float (&u)[16], int t) {
  float w8[8], w4[4], w2[2];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(u[i]), __float_as_uint(u[i + 8]), false, false);
    w8[i] = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
  }
  const bool b3 = (t & 8) != 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float keep = b3 ? w8[i + 4] : w8[i];
    const float send = b3 ? w8[i] : w8[i + 4];
    w4[i] = keep + from_lane_dpp<0x128>(send);
  }
  const bool b2 = (t & 4) != 0;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const float keep = b2 ? w4[i + 2] : w4[i];
    const float send = b2 ? w4[i] : w4[i + 2];
    w2[i] = keep + from_lane_dpp<0x141>(send);
  }
  const bool b1 = (t & 2) != 0;
  const float keep = b1 ? w2[1] : w2[0];
  const float send = b1 ? w2[0] : w2[1];
  float w1 = keep + from_lane_dpp<0x4E>(send);
  w1 += from_lane_dpp<0xB1>(w1);
  return w1;
}

}  // namespace finch
