// Compaction with re-positioning (Method: Managing the Cache): the kept K, V pairs
// move to their slots in the new cache and the positional embedding of each kept
// key is adjusted to the slot it lands in.  For rotary embeddings that is a
// rotation of every channel pair u of the key by (slot - old position) * theta_u,
// theta_u = base^(-2u/d); a candidate's old position is its index in
// [cache ; chunk].  Slots are either the ascending order of the kept indices or,
// as in the paper's worked example, the rank of the score among the kept ones
// (highest first, equal scores by index).  Values are copied bit for bit.
//
// One workgroup moves kGatherRows kept rows of one problem; a thread owns two
// 16-byte pieces of a row, d/2 channels apart, so that it holds both partners of
// its pairs in either pairing.  Angles are formed and reduced to a fraction of a
// turn in fp64 (the shift can be 10^5 positions or more), sine and cosine of the
// reduced angle and the rotation itself are fp32; bf16 results are rounded to
// nearest even.
#include <cmath>

#include "finch_internal.h"
#include "reposition_common.h"
#include "select_common.h"

namespace finch {

namespace {

typedef rp_u32x4 u32x4;
constexpr int kRepThreads = 256;

}  // namespace

// SEGS = 16-byte pieces per row, E = elements per piece (8: bf16, 4: fp32).
// pairing: FINCH_ROPE_OFF / _HALF / _INTERLEAVED.  RANK: slots by score rank; needs
// r * 4 bytes of dynamic LDS.
template <int SEGS, int E, bool RANK>
__global__ __launch_bounds__(kRepThreads) void reposition_rows(LaunchParams prm, int blocks_per_problem,
                                                               int pairing, double log2_base) {
  extern __shared__ __align__(16) char smem[];
  __shared__ int sh_slot[kGatherRows];
  const int p = blockIdx.x / blocks_per_problem;
  const finch_problem pb = prm.probs[p];
  const int N = pb.c + pb.m;
  const int r = min(pb.r, N);
  const int row0 = (blockIdx.x - p * blocks_per_problem) * kGatherRows;
  if (row0 >= r) return;
  const int tid = threadIdx.x;
  const FINCH_GLOBAL int* idx = as_global<int>(pb.idx);
  constexpr int kHalf = SEGS / 2;                      // threads per row
  constexpr int kRowsPerIter = kRepThreads / kHalf;
  constexpr int kIters = kGatherRows / kRowsPerIter;
  const int seg = tid % kHalf;
  const int sub = tid / kHalf;

  if (RANK) {
    // order keys of all kept candidates, then the rank of each of this workgroup's rows
    unsigned* ks = reinterpret_cast<unsigned*>(smem);
    const FINCH_GLOBAL float* scores = as_global<float>(
        pb.scores ? pb.scores : prm.ws_scores + static_cast<size_t>(p) * prm.score_stride);
    for (int u = tid; u < r; u += kRepThreads) ks[u] = order_key(scores[min(max(idx[u], 0), N - 1)]);
    __syncthreads();
    // four consecutive lanes share a row and split the candidates among them
    const int row = row0 + (tid >> 2);
    int above = 0;
    if (row < r) {
      const unsigned mine = ks[row];
      for (int u = tid & 3; u < r; u += 4) above += (ks[u] > mine || (ks[u] == mine && u < row)) ? 1 : 0;
    }
    above += __shfl_xor(above, 1);
    above += __shfl_xor(above, 2);
    if ((tid & 3) == 0) sh_slot[tid >> 2] = above;
    __syncthreads();
  }

  // theta of this thread's E channel pairs
  double th[E];
  pair_thetas<E, kHalf>(pairing, seg, log2_base, th);

  const FINCH_GLOBAL u32x4* kc = as_global<u32x4>(pb.k_cache);
  const FINCH_GLOBAL u32x4* kk = as_global<u32x4>(pb.k_chunk);
  const FINCH_GLOBAL u32x4* vc = as_global<u32x4>(pb.v_cache);
  const FINCH_GLOBAL u32x4* vk = as_global<u32x4>(pb.v_chunk);
  FINCH_GLOBAL u32x4* ko = as_global_mut<u32x4>(pb.k_out);
  FINCH_GLOBAL u32x4* vo = as_global_mut<u32x4>(pb.v_out);
  u32x4 ka[kIters], kb[kIters], va[kIters], vb[kIters];
  int shift[kIters], slot[kIters];
#pragma unroll
  for (int it = 0; it < kIters; ++it) {
    const int local = it * kRowsPerIter + sub;
    const int t = min(row0 + local, r - 1);
    const int j = min(max(idx[t], 0), N - 1);
    slot[it] = RANK ? sh_slot[min(local, r - 1 - row0)] : t;
    shift[it] = slot[it] - j;
    const bool cached = j < pb.c;
    const size_t off = static_cast<size_t>(cached ? j : j - pb.c) * SEGS + seg;
    ka[it] = (cached ? kc : kk)[off];
    kb[it] = (cached ? kc : kk)[off + kHalf];
    va[it] = (cached ? vc : vk)[off];
    vb[it] = (cached ? vc : vk)[off + kHalf];
  }
#pragma unroll
  for (int it = 0; it < kIters; ++it) {
    const int t = row0 + it * kRowsPerIter + sub;
    if (t < r) {
      if (pairing != FINCH_ROPE_OFF && shift[it] != 0) rotate_pieces<E>(pairing, th, shift[it], ka[it], kb[it]);
      const size_t o = static_cast<size_t>(slot[it]) * SEGS + seg;
      ko[o] = ka[it];
      ko[o + kHalf] = kb[it];
      vo[o] = va[it];
      vo[o + kHalf] = vb[it];
    }
  }
}

namespace {

template <int SEGS, int E>
void launch_rep(bool rank, dim3 grid, size_t lds, hipStream_t s, const LaunchParams& p, int bpp, int pairing,
                double log2_base) {
  const dim3 block(kRepThreads);
  if (rank) {
    hipLaunchKernelGGL((reposition_rows<SEGS, E, true>), grid, block, lds, s, p, bpp, pairing, log2_base);
  } else {
    hipLaunchKernelGGL((reposition_rows<SEGS, E, false>), grid, block, 0, s, p, bpp, pairing, log2_base);
  }
}

}  // namespace

// rank: slots by score rank (dynamic LDS r_max * 4 bytes, r_max <= kRankMaxRows).
hipError_t launch_reposition(const LaunchParams& p, int row_bytes, bool bf16, int r_max, int pairing,
                             bool rank, double base, hipStream_t s) {
  if (p.n_problems == 0 || r_max <= 0) return hipSuccess;
  const int bpp = (r_max + kGatherRows - 1) / kGatherRows;
  const dim3 grid(static_cast<unsigned>(bpp) * static_cast<unsigned>(p.n_problems));
  const size_t lds = rank ? static_cast<size_t>(r_max) * 4 : 0;
  const double l2b = std::log2(base);
  const int segs = row_bytes / 16;
  if (bf16 && segs == 16) {
    launch_rep<16, 8>(rank, grid, lds, s, p, bpp, pairing, l2b);
  } else if (bf16 && segs == 8) {
    launch_rep<8, 8>(rank, grid, lds, s, p, bpp, pairing, l2b);
  } else if (!bf16 && segs == 32) {
    launch_rep<32, 4>(rank, grid, lds, s, p, bpp, pairing, l2b);
  } else if (!bf16 && segs == 16) {
    launch_rep<16, 4>(rank, grid, lds, s, p, bpp, pairing, l2b);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t set_max_lds_reposition(size_t bytes) {
  const void* fns[4] = {reinterpret_cast<const void*>(&reposition_rows<16, 8, true>),
                        reinterpret_cast<const void*>(&reposition_rows<8, 8, true>),
                        reinterpret_cast<const void*>(&reposition_rows<32, 4, true>),
                        reinterpret_cast<const void*>(&reposition_rows<16, 4, true>)};
  for (int i = 0; i < 4; ++i) {
    const hipError_t e = hipFuncSetAttribute(fns[i], hipFuncAttributeMaxDynamicSharedMemorySize,
                                             static_cast<int>(bytes));
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace finch
