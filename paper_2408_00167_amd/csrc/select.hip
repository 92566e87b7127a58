// Selection kernel: exact top-r of the per-key scores of one problem (Method:
// t = top-r(A_agg, r)), ties to the lower index, output in ascending index order.
//
// One workgroup per problem; the algorithm is in select_common.h.  Up to 8192
// candidates are held in registers; larger problems re-read their scores (L2) in
// every round.
#include "select_common.h"

namespace finch {

__global__ __launch_bounds__(kSelThreads) void select_topr(LaunchParams prm) {
  __shared__ SelLds lds;
  const int p = blockIdx.x;
  const finch_problem pb = prm.probs[p];
  const int N = pb.c + pb.m;
  const int r = min(pb.r, N);
  if (r <= 0) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const FINCH_GLOBAL float* scores = as_global<float>(
      pb.scores ? pb.scores : prm.ws_scores + static_cast<size_t>(p) * prm.score_stride);
  FINCH_GLOBAL int* idx = as_global_mut<int>(pb.idx);
  if (r >= N) {  // nothing to decide: keep every candidate
    for (int i = tid; i < N; i += kSelThreads) idx[i] = i;
    return;
  }
  if (N <= kSelThreads * kSelRegKeys) {
    select_regs(scores, N, r, idx, nullptr, &lds, tid, lane, wave);
  } else {
    select_generic(nullptr, scores, N, r, idx, nullptr, &lds, tid, lane, wave);
  }
}

hipError_t launch_select(const LaunchParams& p, hipStream_t s) {
  if (p.n_problems == 0) return hipSuccess;
  hipLaunchKernelGGL(select_topr, dim3(p.n_problems), dim3(kSelThreads), 0, s, p);
  return hipGetLastError();
}

}  // namespace finch
