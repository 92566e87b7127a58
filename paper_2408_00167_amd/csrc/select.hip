// Selection kernel: exact top-r of the per-key scores of one problem (Method:
// t = top-r(A_agg, r)), ties to the lower index, output in ascending index order.
//
// One workgroup per problem; the algorithm is in select_common.h.  Up to 16384
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
    select_regs<kSelThreads>(OneScoreVector{scores}, N, r, idx, nullptr, &lds, tid, lane, wave);
  } else {
    select_generic<kSelThreads>(nullptr, OneScoreVector{scores}, N, r, idx, nullptr, &lds, tid, lane, wave);
  }
}

// Layer-wise selection (Method: "Sum over heads" - the scores of all heads of a layer
// are added before ONE top-r per layer): the problems of a batch come in runs of
// `group` consecutive descriptors, the KV heads of one layer, with the same c, m
// and r.  One workgroup per run adds the run's score vectors head by head (a
// fixed order), keeps the sum in `layer_scores` (one slot of prm.score_stride floats
// per run), selects on it and writes the same indices to every problem of the run.
__global__ __launch_bounds__(kSelThreads) void select_layer(LaunchParams prm, int group,
                                                            float* layer_scores) {
  __shared__ SelLds lds;
  const int run = blockIdx.x;
  const int p0 = run * group;
  const finch_problem pb0 = prm.probs[p0];
  const int N = pb0.c + pb0.m;
  const int r = min(pb0.r, N);
  if (r <= 0) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (r >= N) {  // nothing to decide: every head keeps every candidate
    for (int g = 0; g < group; ++g) {
      FINCH_GLOBAL int* idx = as_global_mut<int>(prm.probs[p0 + g].idx);
      for (int i = tid; i < N; i += kSelThreads) idx[i] = i;
    }
    return;
  }
  FINCH_GLOBAL float* total = as_global_mut<float>(layer_scores + static_cast<size_t>(run) * prm.score_stride);
  for (int g = 0; g < group; ++g) {  // head by head; a thread only ever touches its own elements
    const finch_problem pb = prm.probs[p0 + g];
    const FINCH_GLOBAL float* sc = as_global<float>(
        pb.scores ? pb.scores : prm.ws_scores + static_cast<size_t>(p0 + g) * prm.score_stride);
    for (int i = tid; i < N; i += kSelThreads) total[i] = g == 0 ? sc[i] : total[i] + sc[i];
  }
  __syncthreads();  // the sums this workgroup wrote are read back by other threads below
  FINCH_GLOBAL int* idx0 = as_global_mut<int>(pb0.idx);
  if (N <= kSelThreads * kSelRegKeys) {
    select_regs<kSelThreads>(OneScoreVector{total}, N, r, idx0, nullptr, &lds, tid, lane, wave);
  } else {
    select_generic<kSelThreads>(nullptr, OneScoreVector{total}, N, r, idx0, nullptr, &lds, tid, lane, wave);
  }
  __syncthreads();
  for (int g = 1; g < group; ++g) {
    FINCH_GLOBAL int* idx = as_global_mut<int>(prm.probs[p0 + g].idx);
    for (int t = tid; t < r; t += kSelThreads) idx[t] = idx0[t];
  }
}

hipError_t launch_select_layer(const LaunchParams& p, int group, float* layer_scores, hipStream_t s) {
  if (p.n_problems == 0) return hipSuccess;
  hipLaunchKernelGGL(select_layer, dim3(p.n_problems / group), dim3(kSelThreads), 0, s, p, group,
                     layer_scores);
  return hipGetLastError();
}

hipError_t launch_select(const LaunchParams& p, hipStream_t s) {
  if (p.n_problems == 0) return hipSuccess;
  hipLaunchKernelGGL(select_topr, dim3(p.n_problems), dim3(kSelThreads), 0, s, p);
  return hipGetLastError();
}

}  // namespace finch
