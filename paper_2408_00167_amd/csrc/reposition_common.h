// Device helpers of the re-positioning of kept keys (Method: Managing the Cache -
// the rotary embedding of a kept key is turned to the position it moves to),
// shared by the compaction kernel and the one-workgroup-per-problem step kernel.
#pragma once

#include "finch_internal.h"

namespace finch {

typedef unsigned int rp_u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_to_f32(unsigned bits16) { return __uint_as_float(bits16 << 16); }
__device__ __forceinline__ unsigned f32_to_bf16(float x) {  // round to nearest even; finite inputs
  const unsigned u = __float_as_uint(x);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Element e of a 16-byte piece as float, and back.  E = elements per piece.
template <int E>
__device__ __forceinline__ float piece_get(const rp_u32x4& v, int e) {
  if (E == 4) return __uint_as_float(v[e]);
  const unsigned w = v[e >> 1];
  return bf16_to_f32((e & 1) ? (w >> 16) : (w & 0xFFFFu));
}
template <int E>
__device__ __forceinline__ void piece_set(rp_u32x4& v, int e, float x) {
  if (E == 4) {
    v[e] = __float_as_uint(x);
  } else {
    const unsigned b = f32_to_bf16(x);
    unsigned w = v[e >> 1];
    w = (e & 1) ? ((w & 0x0000FFFFu) | (b << 16)) : ((w & 0xFFFF0000u) | b);
    v[e >> 1] = w;
  }
}

// (cos, sin) of shift * theta, theta in radians per position: the angle is reduced
// to a fraction of a turn in fp64 before the fp32 sine and cosine.
__device__ __forceinline__ void turn(double theta, int shift, float& c, float& s) {
  const double rev = static_cast<double>(shift) * theta * 0.15915494309189535;  // turns
  const double frac = rev - rint(rev);                                           // [-0.5, 0.5]
  sincospif(static_cast<float>(2.0 * frac), &s, &c);
}

// theta of the E channel pairs owned by the thread that holds pieces `seg` and
// `seg + HALF` (HALF = pieces per half row) of a row of D = 2 * HALF * E channels.
template <int E, int HALF>
__device__ __forceinline__ void pair_thetas(int pairing, int seg, double log2_base, double (&th)[E]) {
  constexpr int D = 2 * HALF * E;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    int u;
    if (pairing == FINCH_ROPE_INTERLEAVED) {
      u = e < E / 2 ? (E / 2) * seg + e : (E / 2) * (seg + HALF) + (e - E / 2);
    } else {
      u = E * seg + e;
    }
    th[e] = exp2(-2.0 * static_cast<double>(u) / static_cast<double>(D) * log2_base);
  }
}

// Turns the pairs held in pieces a (piece seg) and b (piece seg + HALF) by `shift`
// positions.
template <int E>
__device__ __forceinline__ void rotate_pieces(int pairing, const double (&th)[E], int shift, rp_u32x4& a,
                                              rp_u32x4& b) {
#pragma unroll
  for (int e = 0; e < E; ++e) {
    float c, s;
    turn(th[e], shift, c, s);
    if (pairing == FINCH_ROPE_INTERLEAVED) {
      // pairs (2e', 2e'+1) inside a piece: the first E/2 in piece a, the rest in b
      const int e2 = 2 * (e % (E / 2));
      if (e < E / 2) {
        const float x = piece_get<E>(a, e2), y = piece_get<E>(a, e2 + 1);
        piece_set<E>(a, e2, x * c - y * s);
        piece_set<E>(a, e2 + 1, y * c + x * s);
      } else {
        const float x = piece_get<E>(b, e2), y = piece_get<E>(b, e2 + 1);
        piece_set<E>(b, e2, x * c - y * s);
        piece_set<E>(b, e2 + 1, y * c + x * s);
      }
    } else {
      // pair (u, u + d/2): element e of piece a with element e of piece b
      const float x = piece_get<E>(a, e), y = piece_get<E>(b, e);
      piece_set<E>(a, e, x * c - y * s);
      piece_set<E>(b, e, y * c + x * s);
    }
  }
}

}  // namespace finch
