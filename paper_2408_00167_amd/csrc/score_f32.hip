// Scoring kernels for fp32 Q/K: same two passes and the same statistics layout as
// the bf16 path, on the vector ALU.  One thread owns one key and keeps its K row
// in registers; prompt rows are broadcast from LDS.  Dot products accumulate in
// fp64 (every fp32 product is exact there), the softmax runs in fp32.  This path
// serves small fp32 problems and is not tuned.
#include "finch_internal.h"

namespace finch {

typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr float kInf = __builtin_inff();

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ bool decode_tile(const LaunchParams& prm, int& p, int& tile) {
  const int bid = blockIdx.x;
  const int xcd = bid & 7;
  const int slot = bid >> 3;
  const int pg = slot / prm.tiles_max;
  tile = slot - pg * prm.tiles_max;
  p = pg * 8 + xcd;
  return p < prm.n_problems;
}

__device__ __forceinline__ void merge_stats(float& m, float& z, float m2, float z2) {
  const float mm = fmaxf(m, m2);
  if (mm == -kInf) {
    z = 0.f;
  } else {
    z = z * fast_exp2(m - mm) + z2 * fast_exp2(m2 - mm);
  }
  m = mm;
}

template <int D>
__device__ __forceinline__ void load_k_row(const finch_problem& pb, int N, int key, float (&k)[D]) {
  if (key < N) {
    const float* row = key < pb.c
                           ? static_cast<const float*>(pb.k_cache) + static_cast<size_t>(key) * D
                           : static_cast<const float*>(pb.k_chunk) + static_cast<size_t>(key - pb.c) * D;
    const FINCH_GLOBAL f32x4* rp = as_global<f32x4>(row);
#pragma unroll
    for (int s = 0; s < D / 4; ++s) {
      const f32x4 x = rp[s];
      k[4 * s] = x.x;
      k[4 * s + 1] = x.y;
      k[4 * s + 2] = x.z;
      k[4 * s + 3] = x.w;
    }
  } else {
#pragma unroll
    for (int s = 0; s < D; ++s) k[s] = 0.f;
  }
}

template <int D>
__device__ __forceinline__ void stage_q(const void* q, int R, int row0, int rows, float* lds_q,
                                        int tid) {
  const FINCH_GLOBAL f32x4* src =
      as_global<f32x4>(static_cast<const float*>(q) + static_cast<size_t>(row0) * D);
  f32x4* dst = reinterpret_cast<f32x4*>(lds_q);
  const int total = rows * (D / 4);
  for (int i = tid; i < total; i += 256) dst[i] = src[i];
  (void)R;
}

template <int D>
__device__ __forceinline__ float dot_row(const float* qrow, const float (&k)[D]) {
  double acc = 0.0;
#pragma unroll
  for (int s = 0; s < D; ++s) acc = __builtin_fma(static_cast<double>(qrow[s]), static_cast<double>(k[s]), acc);
  return static_cast<float>(acc);
}

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

}  // namespace

template <int D>
__global__ __launch_bounds__(256) void rowstats_f32(LaunchParams prm) {
  extern __shared__ __align__(16) char smem[];
  int p, tile;
  if (!decode_tile(prm, p, tile)) return;
  const finch_problem pb = prm.probs[p];
  const int N = pb.c + pb.m;
  const int key0 = tile * kTileKeys;
  if (key0 >= N) return;
  const int R = prm.group * pb.n_que;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float* lds_q = reinterpret_cast<float*>(smem);
  float2* wstats = reinterpret_cast<float2*>(smem + static_cast<size_t>(prm.row_chunk) * D * 4);
  const int key = key0 + tid;
  float k[D];
  load_k_row<D>(pb, N, key, k);
  float2* out = prm.stats + (static_cast<size_t>(p) * prm.tiles_max + tile) * prm.rpad_max;
  const float sc = prm.scale_log2;

  for (int row0 = 0; row0 < R; row0 += prm.row_chunk) {
    const int rows = min(prm.row_chunk, R - row0);
    stage_q<D>(pb.q, R, row0, rows, lds_q, tid);
    __syncthreads();
    for (int i = 0; i < rows; ++i) {
      float s = dot_row<D>(lds_q + i * D, k);
      if (key >= N) s = -kInf;
      const float mx = wave_max(s);
      const float ms = (mx == -kInf) ? 0.f : mx * sc;
      const float z = wave_sum(fast_exp2(__builtin_fmaf(s, sc, -ms)));
      if (lane == 0) wstats[wave * prm.row_chunk + i] = make_float2((mx == -kInf) ? -kInf : ms, z);
    }
    __syncthreads();
    for (int i = tid; i < rows; i += 256) {
      float2 a = wstats[i];
#pragma unroll
      for (int w = 1; w < 4; ++w) {
        const float2 b = wstats[w * prm.row_chunk + i];
        merge_stats(a.x, a.y, b.x, b.y);
      }
      out[row0 + i] = a;
    }
    __syncthreads();
  }
}

template <int D>
__global__ __launch_bounds__(256) void colsum_f32(LaunchParams prm) {
  extern __shared__ __align__(16) char smem[];
  int p, tile;
  if (!decode_tile(prm, p, tile)) return;
  const finch_problem pb = prm.probs[p];
  const int N = pb.c + pb.m;
  const int key0 = tile * kTileKeys;
  if (key0 >= N) return;
  const int R = prm.group * pb.n_que;
  const int tid = threadIdx.x;
  float* lds_q = reinterpret_cast<float*>(smem);
  float* lds_lse = reinterpret_cast<float*>(smem + static_cast<size_t>(prm.row_chunk) * D * 4);
  const int key = key0 + tid;
  float k[D];
  load_k_row<D>(pb, N, key, k);
  const float* lse = prm.lse + static_cast<size_t>(p) * prm.rpad_max;
  const float sc = prm.scale_log2;
  float u = 0.f;

  for (int row0 = 0; row0 < R; row0 += prm.row_chunk) {
    const int rows = min(prm.row_chunk, R - row0);
    stage_q<D>(pb.q, R, row0, rows, lds_q, tid);
    for (int i = tid; i < rows; i += 256) lds_lse[i] = lse[row0 + i];
    __syncthreads();
    for (int i = 0; i < rows; ++i) {
      const float s = dot_row<D>(lds_q + i * D, k);
      u += fast_exp2(__builtin_fmaf(s, sc, -lds_lse[i]));
    }
    __syncthreads();
  }
  FINCH_GLOBAL float* dst = as_global_mut<float>(
      pb.scores ? pb.scores : prm.ws_scores + static_cast<size_t>(p) * prm.score_stride);
  if (key < N) dst[key] = u;
}

unsigned score_grid(const LaunchParams& p);

hipError_t launch_rowstats_f32(int head_dim, const LaunchParams& p, size_t lds, hipStream_t s) {
  const dim3 grid(score_grid(p)), block(256);
  if (head_dim == 128) {
    hipLaunchKernelGGL(rowstats_f32<128>, grid, block, lds, s, p);
  } else {
    hipLaunchKernelGGL(rowstats_f32<64>, grid, block, lds, s, p);
  }
  return hipGetLastError();
}

hipError_t launch_colsum_f32(int head_dim, const LaunchParams& p, size_t lds, hipStream_t s) {
  const dim3 grid(score_grid(p)), block(256);
  if (head_dim == 128) {
    hipLaunchKernelGGL(colsum_f32<128>, grid, block, lds, s, p);
  } else {
    hipLaunchKernelGGL(colsum_f32<64>, grid, block, lds, s, p);
  }
  return hipGetLastError();
}

hipError_t set_max_lds_f32(size_t bytes) {
  hipError_t e;
  const int b = static_cast<int>(bytes);
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(&rowstats_f32<128>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, b);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(&rowstats_f32<64>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, b);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(&colsum_f32<128>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, b);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&colsum_f32<64>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, b);
}

}  // namespace finch
