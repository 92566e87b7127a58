// Kernels with one workgroup per problem whose rows include the chunk's own tokens
// (the paper's ablation of the conditioning: document-only or document + prompt
// self-attention, with the causal mask and the Method's normalisation step).  The
// code is in owner_body.h.
#include "owner_body.h"

namespace finch {

hipError_t launch_owner_doc_bf16(int head_dim, const LaunchParams& p, int stages, hipStream_t s) {
  return launch_owner_impl<true>(head_dim, p, stages, s);
}

hipError_t launch_owner_loop_doc_bf16(int head_dim, const LaunchParams& p, const int* step_first,
                                      int n_steps, int n_slots, hipStream_t s) {
  return launch_owner_loop_impl<true>(head_dim, p, step_first, n_steps, n_slots, s);
}

hipError_t set_max_lds_owner_doc(size_t bytes) { return set_max_lds_owner_impl<true>(bytes); }

}  // namespace finch
