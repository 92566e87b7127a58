// Internal declarations shared by the host driver and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "finch.h"

namespace finch {

// Keys handled by one workgroup of the fp32 scoring kernels.
constexpr int kTileKeys = 256;
// Prompt rows staged in LDS at a time (larger R is processed in several chunks).
constexpr int kMaxRowChunk = 512;
// bf16 two-pass scoring: threads per workgroup, and the number of slices the keys
// of a problem are cut into (one workgroup streams one slice of about 2400 keys).
constexpr int kStreamThreads = 512;
constexpr int kDefaultSliceKeys = 2400;
__host__ __device__ inline int stream_slices(int n_keys, int slice_keys) {
  const int s = (n_keys + slice_keys / 2) / slice_keys;
  return s < 1 ? 1 : s;
}
// One-workgroup-per-problem path: most prompt rows staged per pass over the keys.
constexpr int kOwnerMaxRowChunk = 256;
// LDS the one-workgroup-per-problem kernels keep behind their selection scratch (kept indices etc.).
constexpr size_t kOwnerSelectBytes = 24 * 1024;
// Most problems per layer run that the one-workgroup-per-problem kernels select for together.
constexpr int kOwnerMaxLayer = 16;
// Rows copied by one workgroup of the compaction kernels.
constexpr int kGatherRows = 64;
// Most kept rows per problem when slots go by score rank (their order keys are held
// in LDS by every workgroup of the problem).
constexpr int kRankMaxRows = 32768;

// Everything the scoring / selection / compaction kernels need besides the
// descriptors.  Passed by value.
struct LaunchParams {
  const finch_problem* probs;  // device descriptors
  int32_t n_problems;
  int32_t group;               // G
  int32_t tiles_max;           // most partial-statistics records of any problem:
                               // ceil(max_p (c+m) / tile_keys), or stream_slices(max) if
                               // tile_keys == 0
  int32_t tile_keys;           // kTileKeys for the fp32 kernels, 0 for the bf16 ones
  int32_t slice_keys;          // target keys per slice of the bf16 kernels
  int32_t merge_in_pass2;      // bf16: pass 2 merges the slice statistics itself (no lse kernel)
  int32_t rpad_max;            // max_p round_up(G*n_que, 32)
  int32_t row_chunk;           // rows staged per pass over the keys (multiple of 32)
  int32_t score_stride;        // floats per problem in ws_scores
  float scale_log2;            // log2(e) / sqrt(d_k)
  float2* stats;               // [P][tiles_max][rpad_max] partial (max, sum) per tile
  float* lse;                  // [P][rpad_max] log2-domain log-sum-exp per prompt row
  float* ws_scores;            // [P][score_stride] used when desc.scores == NULL
  uint32_t lds_bytes;          // dynamic LDS of the launch
  // re-positioning inside the one-workgroup-per-problem kernels (ascending slots)
  int32_t rope_pairing;        // FINCH_ROPE_OFF / _HALF / _INTERLEAVED
  int32_t rank_order;          // kept rows go to the slot of their score's rank (else ascending slots)
  double rope_log2_base;       // log2 of the rotary base
  // layer-wise selection inside the one-workgroup-per-problem kernels: the L workgroups of
  // a run of problems meet through two counters per run (scores out / scores read) and
  // share one error word behind them; zeroed before the launch
  int32_t layer_group;         // L (1: every problem selects for itself)
  int32_t* layer_sync;         // [2 * runs]
  int32_t* layer_err;          // one word behind them
  int64_t spin_ticks;          // longest wait for the other workgroups, in 100 MHz ticks
};

// Launchers; each returns hipGetLastError() after the launch.
unsigned score_grid(const LaunchParams& p);
hipError_t launch_rowstats_bf16(int head_dim, const LaunchParams& p, size_t lds, hipStream_t s);
hipError_t launch_colsum_bf16(int head_dim, const LaunchParams& p, size_t lds, hipStream_t s);
hipError_t launch_rowstats_f32(int head_dim, const LaunchParams& p, size_t lds, hipStream_t s);
hipError_t launch_colsum_f32(int head_dim, const LaunchParams& p, size_t lds, hipStream_t s);
hipError_t launch_lse(const LaunchParams& p, hipStream_t s);
hipError_t launch_select(const LaunchParams& p, hipStream_t s);
hipError_t launch_select_layer(const LaunchParams& p, int group, float* layer_scores, hipStream_t s);
hipError_t launch_gather(const LaunchParams& p, int row_bytes, int r_max, hipStream_t s);
size_t owner_lds_bytes(int head_dim, int row_chunk);
hipError_t launch_prompt_lse(const LaunchParams& p, int head_dim, bool bf16, int rows_max, hipStream_t s);
hipError_t launch_reposition(const LaunchParams& p, int row_bytes, bool bf16, int r_max, int pairing,
                             bool rank, double base, hipStream_t s);
hipError_t set_max_lds_reposition(size_t bytes);
hipError_t launch_owner_bf16(int head_dim, const LaunchParams& p, int stages, hipStream_t s);
hipError_t launch_owner_loop_bf16(int head_dim, const LaunchParams& p, const int* step_first,
                                  int n_steps, int n_slots, hipStream_t s);
hipError_t set_max_lds_owner(size_t bytes);
// one workgroup per problem for fp32 inputs (prompt rows and rows of the chunk's own tokens)
size_t owner_f32_lds_bytes(int head_dim);
hipError_t launch_owner_f32(int head_dim, const LaunchParams& p, int stages, hipStream_t s);
hipError_t launch_owner_loop_f32(int head_dim, const LaunchParams& p, const int* step_first, int n_steps,
                                 int n_slots, hipStream_t s);
hipError_t set_max_lds_owner_f32(size_t bytes);
hipError_t launch_zero_words(int32_t* words, int n, int32_t* one_more, hipStream_t s);
// the same with rows of the chunk's own tokens (desc.q_doc)
hipError_t launch_owner_doc_bf16(int head_dim, const LaunchParams& p, int stages, hipStream_t s);
hipError_t launch_owner_loop_doc_bf16(int head_dim, const LaunchParams& p, const int* step_first,
                                      int n_steps, int n_slots, hipStream_t s);
hipError_t set_max_lds_owner_doc(size_t bytes);
// Raise the dynamic-LDS limit of the scoring kernels of one dtype to `bytes`.
hipError_t set_max_lds_bf16(size_t bytes);
hipError_t set_max_lds_f32(size_t bytes);


// Descriptor pointers are generic; telling the compiler they are global memory
// turns flat loads/stores into global ones (which do not tie up the LDS counter).
#define FINCH_GLOBAL __attribute__((address_space(1)))
template <typename T>
__device__ __forceinline__ const FINCH_GLOBAL T* as_global(const void* p) {
  return (const FINCH_GLOBAL T*)(p);
}
template <typename T>
__device__ __forceinline__ FINCH_GLOBAL T* as_global_mut(void* p) {
  return (FINCH_GLOBAL T*)(p);
}

}  // namespace finch
