// One workgroup per problem for fp32 Q/K/V: both scoring passes on the vector ALU
// (Background, attention equation; Method: prompt-guided sub-matrix, sum over heads and
// prompt rows), then the top-r and the compaction of owner_body.h, for one step or for
// the whole chunk loop in one launch (Method: Document Segmentation).  Rows come from the
// prompt and, with desc.q_doc, from the chunk's own tokens under the causal mask with the
// Method's normalisation step read per row.
//
// One thread owns one key at a time and keeps its K row in registers; the rows of a
// chunk of kRowChunk rows are broadcast from LDS.  Dot products accumulate in fp64
// (every fp32 product is exact there), the softmax runs in fp32 in the log2 domain with
// a running (maximum, sum) per row and thread, merged over the workgroup.  This serves
// fp32 problems of modest size (C1: 16 prompt rows, a few hundred keys); it is not
// tuned for large ones, which the kernels per stage spread over the chip.
#include "owner_body.h"

namespace finch {

namespace {

constexpr int kRowChunk = 16;  // rows staged at a time

struct F32Lds {
  float* rows;     // [kRowChunk][D]
  int* lim;        // [kRowChunk] a row sees the keys below its limit
  float* lse;      // [kRowChunk]
  float2* wred;    // [waves][kRowChunk]
  char* sel;       // selection scratch
};

template <int D>
__device__ __forceinline__ F32Lds f32_lds(char* smem) {
  F32Lds l;
  size_t off = 0;
  l.rows = reinterpret_cast<float*>(smem);
  off += sizeof(float) * kRowChunk * D;
  l.lim = reinterpret_cast<int*>(smem + off);
  off += sizeof(int) * kRowChunk;
  l.lse = reinterpret_cast<float*>(smem + off);
  off += sizeof(float) * kRowChunk;
  l.wred = reinterpret_cast<float2*>(smem + off);
  off += sizeof(float2) * kOwnWaves * kRowChunk;
  l.sel = smem + ((off + 15) & ~size_t{15});
  return l;
}

template <int D>
__device__ __forceinline__ void f32_load_k_row(const finch_problem& pb, int key, float (&k)[D]) {
  const float* row = key < pb.c ? static_cast<const float*>(pb.k_cache) + static_cast<size_t>(key) * D
                                : static_cast<const float*>(pb.k_chunk) + static_cast<size_t>(key - pb.c) * D;
  const FINCH_GLOBAL u32x4* rp = as_global<u32x4>(row);
#pragma unroll
  for (int s = 0; s < D / 4; ++s) {
    const u32x4 x = rp[s];
    k[4 * s] = __uint_as_float(x.x);
    k[4 * s + 1] = __uint_as_float(x.y);
    k[4 * s + 2] = __uint_as_float(x.z);
    k[4 * s + 3] = __uint_as_float(x.w);
  }
}

template <int D>
__device__ __forceinline__ float f32_dot(const float* qrow, const float (&k)[D]) {
  double acc = 0.0;
#pragma unroll
  for (int s = 0; s < D; ++s) acc = __builtin_fma(static_cast<double>(qrow[s]), static_cast<double>(k[s]), acc);
  return static_cast<float>(acc);
}

// One step of one problem by the whole workgroup; see own_step_body for `step_probs`,
// `epoch` and the return value.
template <int D, bool ROT>
__device__ __forceinline__ bool own_step_body_f32(const LaunchParams& prm, const finch_problem& pb, int slot,
                                                  int stages, char* smem, const finch_problem* step_probs,
                                                  int epoch) {
  const int N = pb.c + pb.m;
  if (N == 0) return false;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const F32Lds l = f32_lds<D>(smem);
  const float sc = prm.scale_log2;
  float* gscores = pb.scores ? pb.scores : prm.ws_scores + static_cast<size_t>(slot) * prm.score_stride;
  FINCH_GLOBAL float* dst = as_global_mut<float>(gscores);
  const int L = prm.layer_group;
  const bool layered = stages && L > 1 && pb.r > 0 && pb.r < N;
  int* const sync_words = (stages && L > 1) ? prm.layer_sync + 2 * (slot / L) : nullptr;
  if (sync_words && epoch > 0) {
    // (see own_step_body: the scores of the step before may still be read by the layer's other workgroups)
    if (tid == 0) {
      const long long t0 = wall_clock64();
      while (__hip_atomic_load(sync_words + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < L * epoch) {
        __builtin_amdgcn_s_sleep(8);
        if (wall_clock64() - t0 > prm.spin_ticks) {
          atomicOr(prm.layer_err, 1);
          break;
        }
      }
    }
    __syncthreads();
  }
  // rows: the prompt's (they see every key), then those of the chunk's own tokens, head by head
  const int Rp = pb.q ? prm.group * pb.n_que : 0;
  const int Rd = (pb.q_doc && pb.m > 0) ? prm.group * pb.m : 0;
  const int n_rows = Rp + Rd;
  for (int row0 = 0; row0 < n_rows; row0 += kRowChunk) {
    const int rows = min(kRowChunk, n_rows - row0);
    // stage the rows, their limits and what is added to their denominators
    for (int i = tid; i < rows * (D / 4); i += kOwnThreads) {
      const int ri = i / (D / 4), seg = i - ri * (D / 4);
      const int row = row0 + ri;
      const float* src = row < Rp ? static_cast<const float*>(pb.q) + static_cast<size_t>(row) * D
                                  : static_cast<const float*>(pb.q_doc) + static_cast<size_t>(row - Rp) * D;
      reinterpret_cast<u32x4*>(l.rows)[i] = as_global<u32x4>(src)[seg];
    }
    if (tid < kRowChunk) {
      const int row = row0 + tid;
      int lim = 0;  // rows past the end see nothing
      if (tid < rows) lim = row < Rp ? N : min(N, pb.c + (row - Rp) % pb.m + 1);
      l.lim[tid] = lim;
    }
    __syncthreads();
    // ---- pass 1: running (maximum, sum exp2) per row over this thread's keys
    float m_run[kRowChunk], z_run[kRowChunk];
#pragma unroll
    for (int i = 0; i < kRowChunk; ++i) {
      m_run[i] = -kInf;
      z_run[i] = 0.f;
    }
    for (int key = tid; key < N; key += kOwnThreads) {
      float k[D];
      f32_load_k_row<D>(pb, key, k);
#pragma unroll
      for (int i = 0; i < kRowChunk; ++i) {
        if (key < l.lim[i]) {
          const float s = f32_dot<D>(l.rows + i * D, k) * sc;
          const float mn = fmaxf(m_run[i], s);
          z_run[i] = z_run[i] * fast_exp2(m_run[i] - mn) + fast_exp2(s - mn);
          m_run[i] = mn;
        }
      }
    }
#pragma unroll
    for (int i = 0; i < kRowChunk; ++i) {
      float m = m_run[i], z = z_run[i];
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) {
        const float m2 = __shfl_xor(m, o);
        const float z2 = __shfl_xor(z, o);
        merge_stats(m, z, m2, z2);
      }
      if (lane == 0) l.wred[wave * kRowChunk + i] = make_float2(m, z);
    }
    __syncthreads();
    if (tid < kRowChunk) {
      float lse = kInf;  // rows past the end add exp2(-inf) = 0
      if (tid < rows) {
        float2 a = l.wred[tid];
#pragma unroll
        for (int w = 1; w < kOwnWaves; ++w) {
          const float2 c = l.wred[w * kRowChunk + tid];
          merge_stats(a.x, a.y, c.x, c.y);
        }
        lse = a.x + fast_log2(a.y);
        const int row = row0 + tid;
        if (row < Rp) {
          if (pb.lse_extra) lse = widen_lse(lse, as_global<float>(pb.lse_extra)[row]);
        } else {
          // normalisation step: the row's weights times (keys it sees) / (c + m)
          lse -= fast_log2(static_cast<float>(l.lim[tid]) / static_cast<float>(N));
        }
      }
      l.lse[tid] = lse;
    }
    __syncthreads();
    // ---- pass 2: this chunk's rows added to the scores of this thread's keys
    for (int key = tid; key < N; key += kOwnThreads) {
      float k[D];
      f32_load_k_row<D>(pb, key, k);
      float u = 0.f;
#pragma unroll
      for (int i = 0; i < kRowChunk; ++i) {
        if (key < l.lim[i]) u += fast_exp2(__builtin_fmaf(f32_dot<D>(l.rows + i * D, k), sc, -l.lse[i]));
      }
      const float val = row0 == 0 ? u : dst[key] + u;
      if (layered) __hip_atomic_store(gscores + key, val, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      else dst[key] = val;
    }
    __syncthreads();  // the staged rows may be replaced; after the last chunk: the scores are out
  }
  if (!stages) return false;
  own_finish_step<D / 4, 4, ROT>(prm, pb, slot, N, dst, l.sel, prm.lds_bytes - static_cast<size_t>(l.sel - smem),
                                 step_probs, epoch, layered, sync_words, tid);
  return layered;
}

template <int D, bool ROT>
__global__ __launch_bounds__(kOwnThreads) void owner_step_f32(LaunchParams prm, int stages) {
  extern __shared__ __align__(16) char smem[];
  const int p = own_slot_of(blockIdx.x, gridDim.x, stages ? prm.layer_group : 1);
  const finch_problem pb = prm.probs[p];
  own_step_body_f32<D, ROT>(prm, pb, p, stages, smem, prm.probs, 0);
}

template <int D, bool ROT>
__global__ __launch_bounds__(kOwnThreads) void owner_loop_f32(LaunchParams prm, const int* step_first, int n_steps) {
  extern __shared__ __align__(16) char smem[];
  const int slot = own_slot_of(blockIdx.x, gridDim.x, prm.layer_group);
  int epoch = 0;
  for (int s = 0; s < n_steps; ++s) {
    const int first = step_first[s];
    if (slot >= step_first[s + 1] - first) break;  // slots are filled from the front
    const finch_problem pb = prm.probs[first + slot];
    if (own_step_body_f32<D, ROT>(prm, pb, slot, /*stages=*/1, smem, prm.probs + first, epoch)) ++epoch;
    // the rows this step wrote are the next step's cache: complete before it reads
    __syncthreads();
  }
}

template <typename F>
bool with_f32_step_kernel(int head_dim, bool rot, F f) {
  if (head_dim == 128) rot ? f(&owner_step_f32<128, true>) : f(&owner_step_f32<128, false>);
  else if (head_dim == 64) rot ? f(&owner_step_f32<64, true>) : f(&owner_step_f32<64, false>);
  else return false;
  return true;
}
template <typename F>
bool with_f32_loop_kernel(int head_dim, bool rot, F f) {
  if (head_dim == 128) rot ? f(&owner_loop_f32<128, true>) : f(&owner_loop_f32<128, false>);
  else if (head_dim == 64) rot ? f(&owner_loop_f32<64, true>) : f(&owner_loop_f32<64, false>);
  else return false;
  return true;
}

}  // namespace

size_t owner_f32_lds_bytes(int head_dim) {
  const size_t fixed = sizeof(float) * kRowChunk * head_dim + (sizeof(int) + sizeof(float)) * kRowChunk +
                       sizeof(float2) * kOwnWaves * kRowChunk + 16;
  return fixed + sizeof(SelLds) + kOwnerSelectBytes;
}

hipError_t launch_owner_f32(int head_dim, const LaunchParams& p, int stages, hipStream_t s) {
  if (p.n_problems <= 0) return hipSuccess;
  const dim3 grid(static_cast<unsigned>(p.n_problems)), block(kOwnThreads);
  const bool ok = with_f32_step_kernel(head_dim, p.rope_pairing != FINCH_ROPE_OFF || p.rank_order, [&](auto kern) {
    hipLaunchKernelGGL(kern, grid, block, p.lds_bytes, s, p, stages);
  });
  return ok ? hipGetLastError() : hipErrorInvalidValue;
}

hipError_t launch_owner_loop_f32(int head_dim, const LaunchParams& p, const int* step_first, int n_steps,
                                 int n_slots, hipStream_t s) {
  if (n_slots <= 0 || n_steps <= 0) return hipSuccess;
  const dim3 grid(static_cast<unsigned>(n_slots)), block(kOwnThreads);
  const bool ok = with_f32_loop_kernel(head_dim, p.rope_pairing != FINCH_ROPE_OFF || p.rank_order, [&](auto kern) {
    hipLaunchKernelGGL(kern, grid, block, p.lds_bytes, s, p, step_first, n_steps);
  });
  return ok ? hipGetLastError() : hipErrorInvalidValue;
}

hipError_t set_max_lds_owner_f32(size_t bytes) {
  hipError_t err = hipSuccess;
  auto set = [&](auto kern) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes));
    if (e != hipSuccess) err = e;
  };
  for (int d = 0; d < 2; ++d)
    for (int rot = 0; rot < 2; ++rot) {
      with_f32_step_kernel(d ? 128 : 64, rot != 0, set);
      with_f32_loop_kernel(d ? 128 : 64, rot != 0, set);
    }
  return err;
}

}  // namespace finch
