// Exact top-r of the per-key scores of one problem by one workgroup of NT = 512 or
// 1024 threads (Method: t = top-r(A_agg, r)): ties to the lower index, output in
// ascending index order.  Shared by the selection kernel and the
// one-workgroup-per-problem step kernel.
//
// The r-th largest value T is found by a radix select over order-preserving 32-bit
// keys, 8 bits per round, histogramming in LDS.  The kept set is { key > T } plus
// the first (r - #greater) candidates with key == T in index order, and an ordered
// scan gives each kept index its output slot, so nothing is sorted.
#pragma once

#include "finch_internal.h"

namespace finch {

constexpr int kSelThreads = 1024;          // threads of the selection kernel
constexpr int kSelMaxWaves = 16;           // most waves of any workgroup that selects
// select_regs keeps up to this many candidates per thread in registers
constexpr int kSelRegKeys = 16;

// Monotone map float -> uint32 (larger float <=> larger key); -0 counts as +0.
__device__ __forceinline__ unsigned order_key(float f) {
  const unsigned u = __float_as_uint(f + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Inclusive prefix sum over the 64 lanes of a wave without a trip through LDS: shifts
// by 1, 2, 4, 8 inside each row of 16 lanes (zeros shifted in), then lane 15 of every
// even row is added to the row above it and lane 31 to the upper half.
__device__ __forceinline__ int wave_inclusive_scan(int x) {
  int v = x;
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, true);   // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, true);   // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, true);   // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, true);   // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);  // row_bcast:15 into rows 1, 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);  // row_bcast:31 into rows 2, 3
  return v;
}

constexpr int kSelMaxLayer = 16;  // most score vectors a selection inside a workgroup adds up

struct SelLds {  // LDS scratch of a selection
  int hist[4][256];
  int wave_tot[2][kSelMaxWaves];
  int digit[4], remaining[4];
  const float* layer_src[kSelMaxLayer];  // LayerScores: the score vectors of a layer's heads
  int layer_gave_up;                     // the wait for the layer's other workgroups expired
};

// Where a selection takes the score of candidate i from: one vector ...
struct OneScoreVector {
  const FINCH_GLOBAL float* p;
  __device__ __forceinline__ float operator()(int i) const { return p[i]; }
};
// ... or the sum of the L vectors of a layer's heads, added head by head in fp32 (Method:
// "Sum over heads"; the order is that of select_layer, so both give the same bits).  The
// vectors come from other workgroups: they are read past this compute unit's caches.
struct LayerScores {
  const float* const* src;  // LDS table of L pointers
  int L;
  __device__ __forceinline__ float operator()(int i) const {
    // all loads first (they come from far away), then the sum in head order
    float v[kSelMaxLayer];
#pragma unroll
    for (int g = 0; g < kSelMaxLayer; ++g)
      v[g] = g < L ? __hip_atomic_load(src[g] + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.f;
    float t = v[0];
#pragma unroll
    for (int g = 1; g < kSelMaxLayer; ++g)
      if (g < L) t = t + v[g];
    return t;
  }
};

// Wave 0 only: lane L owns bins 4L..4L+3 of `hist`; finds the bin where the count
// from the top reaches `remaining` and writes that bin and the rank left inside it.
__device__ __forceinline__ void sel_pick_digit(const int* hist, int remaining, int lane, int* digit_out,
                                               int* left_out) {
  const int h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2], h3 = hist[4 * lane + 3];
  const int mine = h0 + h1 + h2 + h3;
  const int prefix = wave_inclusive_scan(mine);
  const int total = __builtin_amdgcn_readlane(prefix, 63);
  const int suffix = total - prefix + mine;  // inclusive sum over lanes >= this one
  const int above = suffix - mine;  // keys in bins of higher lanes
  if (above < remaining && remaining <= suffix) {
    int left = remaining - above;  // >= 1
    int digit;
    if (left <= h3) {
      digit = 3;
    } else if (left <= h3 + h2) {
      digit = 2;
      left -= h3;
    } else if (left <= h3 + h2 + h1) {
      digit = 1;
      left -= h3 + h2;
    } else {
      digit = 0;
      left -= h3 + h2 + h1;
    }
    *digit_out = 4 * lane + digit;
    *left_out = left;
  }
}

// The same by every wave for itself (all waves read the same histogram and get the same
// answer, so nothing has to be handed round through LDS and no barrier follows): the bin
// where the count from the top reaches `remaining`, and the rank left inside it.
__device__ __forceinline__ void sel_pick_digit_wave(const int* hist, int remaining, int lane, int& digit_out,
                                                    int& left_out) {
  const int h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2], h3 = hist[4 * lane + 3];
  const int mine = h0 + h1 + h2 + h3;
  const int prefix = wave_inclusive_scan(mine);
  const int total = __builtin_amdgcn_readlane(prefix, 63);
  const int suffix = total - prefix + mine;  // inclusive sum over lanes >= this one
  const int above = suffix - mine;           // keys in bins of higher lanes
  const bool found = above < remaining && remaining <= suffix;
  int left = remaining - above, digit = 3;
  if (left > h3) {
    if (left <= h3 + h2) {
      digit = 2;
      left -= h3;
    } else if (left <= h3 + h2 + h1) {
      digit = 1;
      left -= h3 + h2;
    } else {
      digit = 0;
      left -= h3 + h2 + h1;
    }
  }
  // (exactly one lane finds it when 0 < remaining <= total; lane 0's values otherwise)
  const unsigned long long m = __ballot(found);
  const int src = m ? __ffsll(static_cast<long long>(m)) - 1 : 0;
  digit_out = __shfl(4 * lane + digit, src);
  left_out = __shfl(left, src);
}

// Exclusive rank of `flag` among the workgroup's threads in thread order, and the
// total.  Two barriers; every thread must call it.
template <int NT>
__device__ __forceinline__ int sel_block_rank(bool flag, int* wave_tot, int lane, int wave, int& total) {
  const unsigned long long b = __ballot(flag);
  const int below = __popcll(b & ((1ull << lane) - 1ull));
  if (lane == 0) wave_tot[wave] = __popcll(b);
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < NT / 64; ++w) {
    const int x = wave_tot[w];
    if (w < wave) base += x;
    tot += x;
  }
  __syncthreads();
  total = tot;
  return base + below;
}

// Exclusive prefix sum of `v` over the workgroup's threads in thread order.  One
// barrier; `wave_tot` must not be reused before another barrier.
template <int NT>
__device__ __forceinline__ int sel_block_scan(int v, int* wave_tot, int lane, int wave) {
  const int incl = wave_inclusive_scan(v);
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  int base = 0;
#pragma unroll
  for (int w = 0; w < NT / 64; ++w) {
    const int x = wave_tot[w];
    if (w < wave) base += x;
  }
  return base + incl - v;
}

// Any N.  `keys` is LDS (order keys staged there) or nullptr (scores taken from
// `score_of` again each round).  Writes idx to `gidx` and, if `lidx` is not null, also to
// LDS.  0 < r < N.  Whole workgroup; starts and ends without a barrier.
template <int NT, class Src = OneScoreVector>
__device__ __forceinline__ void select_generic(const unsigned* keys, const Src& score_of,
                                               int N, int r, FINCH_GLOBAL int* gidx, int* lidx, SelLds* f,
                                               int tid, int lane, int wave) {
  auto key_at = [&](int i) -> unsigned { return keys ? keys[i] : order_key(score_of(i)); };
  unsigned prefix = 0, mask = 0;
  int remaining = r;
  int* hist = f->hist[0];
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int i = tid; i < N; i += NT) {
      const unsigned key = key_at(i);
      if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
    }
    __syncthreads();
    if (wave == 0) sel_pick_digit(hist, remaining, lane, &f->digit[0], &f->remaining[0]);
    __syncthreads();
    prefix |= static_cast<unsigned>(f->digit[0]) << shift;
    mask |= 255u << shift;
    remaining = f->remaining[0];
    __syncthreads();
  }
  const unsigned T = prefix;
  const int need_eq = remaining;  // candidates equal to T that are kept (>= 1)
  int carry_eq = 0, carry_keep = 0;
  for (int base = 0; base < N; base += NT) {
    const int i = base + tid;
    const bool valid = i < N;
    const unsigned key = valid ? key_at(i) : 0u;
    const bool gt = valid && key > T;
    const bool eq = valid && key == T;
    int tot_eq, tot_keep;
    const int eq_rank = carry_eq + sel_block_rank<NT>(eq, f->wave_tot[0], lane, wave, tot_eq);
    const bool keep = gt || (eq && eq_rank < need_eq);
    const int pos = carry_keep + sel_block_rank<NT>(keep, f->wave_tot[0], lane, wave, tot_keep);
    // (pos < r always when the scores hold still; if another workgroup is overwriting them -
    // a layer's workgroup whose bounded wait has expired - the rounds may have counted
    // different values, and nothing may be written past the r places of the output)
    if (keep && pos < r) {
      gidx[pos] = i;
      if (lidx) lidx[pos] = i;
    }
    carry_eq += tot_eq;
    carry_keep += tot_keep;
  }
}

// N <= NT * kSelRegKeys: thread t owns the candidates [t*K, t*K+K),
// K = ceil(N / NT), and keeps their order keys in registers, so the four radix
// rounds touch LDS only for the histograms (lanes of a wave that hit the same bin
// as the wave's first active lane are counted with one atomic) and the ordered
// output needs two workgroup scans.  0 < r < N.  Whole workgroup; starts with a
// barrier of its own and ends without one.
template <int NT, class Src = OneScoreVector>
__device__ __forceinline__ void select_regs(const Src& score_of, int N, int r,
                                            FINCH_GLOBAL int* gidx, int* lidx, SelLds* f, int tid,
                                            int lane, int wave) {
  const int K = (N + NT - 1) / NT;
  const int i0 = tid * K;
  const int nk = max(0, min(K, N - i0));  // candidates of this thread
  unsigned key[kSelRegKeys];
#pragma unroll
  for (int k = 0; k < kSelRegKeys; ++k) key[k] = k < nk ? order_key(score_of(i0 + k)) : 0u;
  for (int i = tid; i < 4 * 256; i += NT) (&f->hist[0][0])[i] = 0;
  __syncthreads();
  unsigned prefix = 0, mask = 0;
  int remaining = r;
#pragma unroll
  for (int round = 0; round < 4; ++round) {
    const int shift = 24 - 8 * round;
    int* hist = f->hist[round];
#pragma unroll
    for (int k = 0; k < kSelRegKeys; ++k) {
      const bool act = k < nk && (key[k] & mask) == prefix;
      const unsigned long long am = __ballot(act);
      if (am) {  // uniform
        const unsigned d = (key[k] >> shift) & 255u;
        const int leader = __ffsll(static_cast<long long>(am)) - 1;
        const unsigned dl = static_cast<unsigned>(__shfl(static_cast<int>(d), leader));
        const unsigned long long same = __ballot(act && d == dl);
        if (lane == leader) atomicAdd(&hist[dl], __popcll(same));
        if (act && d != dl) atomicAdd(&hist[d], 1);
      }
    }
    __syncthreads();
    int digit;
    sel_pick_digit_wave(hist, remaining, lane, digit, remaining);
    prefix |= static_cast<unsigned>(digit) << shift;
    mask |= 255u << shift;
  }
  const unsigned T = prefix;
  const int need_eq = remaining;  // candidates equal to T that are kept (>= 1)
  int c_eq = 0;
#pragma unroll
  for (int k = 0; k < kSelRegKeys; ++k) c_eq += (k < nk && key[k] == T) ? 1 : 0;
  int eq_rank = sel_block_scan<NT>(c_eq, f->wave_tot[0], lane, wave);
  unsigned keep_bits = 0;
  int c_keep = 0;
#pragma unroll
  for (int k = 0; k < kSelRegKeys; ++k) {
    if (k < nk) {
      bool keep = key[k] > T;
      if (key[k] == T) keep = eq_rank++ < need_eq;
      if (keep) {
        keep_bits |= 1u << k;
        ++c_keep;
      }
    }
  }
  int pos = sel_block_scan<NT>(c_keep, f->wave_tot[1], lane, wave);
#pragma unroll
  for (int k = 0; k < kSelRegKeys; ++k) {
    if (keep_bits & (1u << k)) {
      gidx[pos] = i0 + k;
      if (lidx) lidx[pos] = i0 + k;
      ++pos;
    }
  }
}

}  // namespace finch
