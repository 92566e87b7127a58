// Selection kernel: exact top-r of the per-key scores of one problem (Method:
// t = top-r(A_agg, r)), ties to the lower index, output in ascending index order.
//
// One workgroup per problem.  The r-th largest value is found by a radix select
// over order-preserving 32-bit keys, 8 bits per round, histogramming in LDS; the
// scores (a few tens of KB per problem) are re-read from L2 each round.  The kept
// set is then { key > T } plus the first (r - #greater) candidates with key == T
// in index order, and an ordered block scan of the keep flags gives each kept
// index its output slot, so no sort is needed.
#include "finch_internal.h"

namespace finch {
namespace {

constexpr int kThreads = 1024;
constexpr int kSelWaves = kThreads / 64;

// Monotone map float -> uint32 (larger float <=> larger key); -0 counts as +0.
__device__ __forceinline__ uint32_t order_key(float f) {
  const uint32_t u = __float_as_uint(f + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Exclusive prefix count of `flag` over the workgroup in thread order, plus the
// workgroup total.  `wave_tot` is LDS scratch of kSelWaves ints.  Contains two
// barriers; every thread must call it.
__device__ __forceinline__ int block_rank(bool flag, int* wave_tot, int lane, int wave, int& total) {
  const unsigned long long b = __ballot(flag);
  const int below = __popcll(b & ((1ull << lane) - 1ull));
  if (lane == 0) wave_tot[wave] = __popcll(b);
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    const int x = wave_tot[w];
    if (w < wave) base += x;
    tot += x;
  }
  __syncthreads();
  total = tot;
  return base + below;
}

}  // namespace

__global__ __launch_bounds__(kThreads) void select_topr(LaunchParams prm) {
  __shared__ int hist[256];
  __shared__ int wave_tot[kSelWaves];
  __shared__ int sh_digit, sh_remaining;

  const int p = blockIdx.x;
  const finch_problem pb = prm.probs[p];
  const int N = pb.c + pb.m;
  const int r = min(pb.r, N);
  if (r <= 0) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const FINCH_GLOBAL float* scores = as_global<float>(
      pb.scores ? pb.scores : prm.ws_scores + static_cast<size_t>(p) * prm.score_stride);
  FINCH_GLOBAL int32_t* idx = as_global_mut<int32_t>(pb.idx);

  if (r >= N) {  // nothing to decide: keep every candidate
    for (int i = tid; i < N; i += kThreads) idx[i] = i;
    return;
  }

  // ---- radix select: T = key of the r-th largest score ----
  uint32_t prefix = 0, mask = 0;
  int remaining = r;  // rank still to be located among keys matching prefix
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int i = tid; i < N; i += kThreads) {
      const uint32_t key = order_key(scores[i]);
      if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
    }
    __syncthreads();
    if (wave == 0) {
      // lane L owns bins 4L..4L+3; find the bin where the count from the top
      // reaches `remaining`.
      const int h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2],
                h3 = hist[4 * lane + 3];
      const int mine = h0 + h1 + h2 + h3;
      int suffix = mine;  // inclusive sum over lanes >= this one
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int x = __shfl_down(suffix, o);
        if (lane + o < 64) suffix += x;
      }
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
        sh_digit = 4 * lane + digit;
        sh_remaining = left;
      }
    }
    __syncthreads();
    prefix |= static_cast<uint32_t>(sh_digit) << shift;
    mask |= 255u << shift;
    remaining = sh_remaining;
    __syncthreads();
  }
  const uint32_t T = prefix;
  const int need_eq = remaining;  // candidates equal to T that are kept (>= 1)

  // ---- ordered output ----
  int carry_eq = 0, carry_keep = 0;
  for (int base = 0; base < N; base += kThreads) {
    const int i = base + tid;
    const bool valid = i < N;
    const uint32_t key = valid ? order_key(scores[i]) : 0u;
    const bool gt = valid && key > T;
    const bool eq = valid && key == T;
    int tot_eq, tot_keep;
    const int eq_rank = carry_eq + block_rank(eq, wave_tot, lane, wave, tot_eq);
    const bool keep = gt || (eq && eq_rank < need_eq);
    const int pos = carry_keep + block_rank(keep, wave_tot, lane, wave, tot_keep);
    if (keep) idx[pos] = i;
    carry_eq += tot_eq;
    carry_keep += tot_keep;
  }
}

hipError_t launch_select(const LaunchParams& p, hipStream_t s) {
  if (p.n_problems == 0) return hipSuccess;
  hipLaunchKernelGGL(select_topr, dim3(p.n_problems), dim3(kThreads), 0, s, p);
  return hipGetLastError();
}

}  // namespace finch
