// Kernels with one workgroup per problem, rows from the prompt only (the method's
// own conditioning; Method: prompt-guided sub-matrix).  The code is in owner_body.h.
#include "owner_body.h"

namespace finch {

// Dynamic LDS the kernels need for `row_chunk` staged prompt rows (a multiple of 32,
// at most kOwnerMaxRowChunk).
size_t owner_lds_bytes(int head_dim, int row_chunk) {
  // staged prompt rows, then the larger of {pass-1 statistics + lse + block counter}
  // and the selection scratch with room for about 6000 kept indices
  const size_t q = static_cast<size_t>(row_chunk) * (head_dim * 2 + 16);
  const size_t scoring = static_cast<size_t>(row_chunk) * (kOwnWaves * 8 + 4) + 16;
  const size_t selection = sizeof(SelLds) + kOwnerSelectBytes;
  return q + (scoring > selection ? scoring : selection);
}

hipError_t launch_owner_bf16(int head_dim, const LaunchParams& p, int stages, hipStream_t s) {
  return launch_owner_impl<false>(head_dim, p, stages, s);
}

hipError_t launch_owner_loop_bf16(int head_dim, const LaunchParams& p, const int* step_first, int n_steps,
                                  int n_slots, hipStream_t s) {
  return launch_owner_loop_impl<false>(head_dim, p, step_first, n_steps, n_slots, s);
}

hipError_t set_max_lds_owner(size_t bytes) { return set_max_lds_owner_impl<false>(bytes); }

}  // namespace finch

#ifdef FINCH_PHASE_TIMERS
// Phase-timer build only: the totals of the kernels of this file (prompt rows only) on the
// current device, 8 words of wall-clock ticks (10 ns); reset != 0 clears them instead.
extern "C" int finch_debug_phases(unsigned long long* out, int reset) {
  if (reset) {
    const unsigned long long zero[8] = {0};
    return static_cast<int>(hipMemcpyToSymbol(HIP_SYMBOL(finch::finch_phase_ticks), zero, sizeof(zero)));
  }
  return static_cast<int>(hipMemcpyFromSymbol(out, HIP_SYMBOL(finch::finch_phase_ticks), sizeof(unsigned long long) * 8));
}
#endif
