// Compaction kernel (Method: Managing the Cache): the K and V rows of the selected
// positions are copied, in ascending position order, into the destination cache
// that the next chunk is appended to.  A pure copy in 16-byte pieces; each
// workgroup moves kGatherRows rows of K and of V of one problem.
#include "finch_internal.h"

namespace finch {

// A native 16-byte vector (keeps copies in registers).
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <int SEGS>  // 16-byte pieces per row
__global__ __launch_bounds__(256) void gather_rows(LaunchParams prm, int blocks_per_problem) {
  const int p = blockIdx.x / blocks_per_problem;
  const finch_problem pb = prm.probs[p];
  const int N = pb.c + pb.m;
  const int r = min(pb.r, N);
  const int row0 = (blockIdx.x - p * blocks_per_problem) * kGatherRows;
  if (row0 >= r) return;
  constexpr int kRowsPerIter = 256 / SEGS;
  const int seg = threadIdx.x % SEGS;
  const int sub = threadIdx.x / SEGS;
  const FINCH_GLOBAL u32x4* kc = as_global<u32x4>(pb.k_cache);
  const FINCH_GLOBAL u32x4* kk = as_global<u32x4>(pb.k_chunk);
  const FINCH_GLOBAL u32x4* vc = as_global<u32x4>(pb.v_cache);
  const FINCH_GLOBAL u32x4* vk = as_global<u32x4>(pb.v_chunk);
  FINCH_GLOBAL u32x4* ko = as_global_mut<u32x4>(pb.k_out);
  FINCH_GLOBAL u32x4* vo = as_global_mut<u32x4>(pb.v_out);
  constexpr int kIters = kGatherRows / kRowsPerIter;
  // Loads first, stores after: every thread has 2*kIters 16-byte loads in flight.
  // Threads past the last kept row re-read row r-1 (in bounds) and store nothing.
  u32x4 kv[kIters], vv[kIters];
#pragma unroll
  for (int it = 0; it < kIters; ++it) {
    const int t = min(row0 + it * kRowsPerIter + sub, r - 1);
    // idx normally comes from the selection kernel; clamp so that a caller-supplied
    // index can never read outside the candidates
    const int j = min(max(as_global<int32_t>(pb.idx)[t], 0), N - 1);
    const bool cached = j < pb.c;
    const size_t off = static_cast<size_t>(cached ? j : j - pb.c) * SEGS + seg;
    kv[it] = (cached ? kc : kk)[off];
    vv[it] = (cached ? vc : vk)[off];
  }
#pragma unroll
  for (int it = 0; it < kIters; ++it) {
    const int t = row0 + it * kRowsPerIter + sub;
    if (t < r) {
      ko[static_cast<size_t>(t) * SEGS + seg] = kv[it];
      vo[static_cast<size_t>(t) * SEGS + seg] = vv[it];
    }
  }
}

hipError_t launch_gather(const LaunchParams& p, int row_bytes, int r_max, hipStream_t s) {
  if (p.n_problems == 0 || r_max <= 0) return hipSuccess;
  const int bpp = (r_max + kGatherRows - 1) / kGatherRows;
  const dim3 grid(static_cast<unsigned>(bpp) * static_cast<unsigned>(p.n_problems)), block(256);
  switch (row_bytes / 16) {
    case 8:
      hipLaunchKernelGGL(gather_rows<8>, grid, block, 0, s, p, bpp);
      break;
    case 16:
      hipLaunchKernelGGL(gather_rows<16>, grid, block, 0, s, p, bpp);
      break;
    case 32:
      hipLaunchKernelGGL(gather_rows<32>, grid, block, 0, s, p, bpp);
      break;
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

namespace {
__global__ void zero_words(int32_t* w, int n, int32_t* one_more) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) w[i] = 0;
  if (i == 0 && one_more) *one_more = 0;
}
}  // namespace

// Clears `n` words at `words` and the word at `one_more` (may be null) with a small kernel
// (a plain fill: safe inside a captured graph, where memset nodes are not).
hipError_t launch_zero_words(int32_t* words, int n, int32_t* one_more, hipStream_t s) {
  if (n <= 0 && !one_more) return hipSuccess;
  const int blocks = n > 0 ? (n + 255) / 256 : 1;
  hipLaunchKernelGGL(zero_words, dim3(blocks), dim3(256), 0, s, words, n, one_more);
  return hipGetLastError();
}

}  // namespace finch
