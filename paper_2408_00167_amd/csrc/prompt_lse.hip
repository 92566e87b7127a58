// The prompt's share of the softmax denominator (Method: in the model's input the
// prompt follows the context, so a prompt token attends to the context keys and,
// causally, to the prompt tokens up to itself; Background, attention equation).
// For every prompt row i = g*n_que + t of a problem this kernel writes
//   lse_extra[i] = log sum_{j <= t} exp(q_i . kq_j / sqrt(d_k))
// over the prompt's own keys kq, which the scoring kernels add to the row's
// denominator over the context keys.  The work is tiny (R * n_que / 2 dot
// products per problem): four lanes per row, each with a quarter of the channels,
// dot products accumulated in fp64.
#include "finch_internal.h"

namespace finch {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Dot product of two runs of D elements stored as 16-byte pieces; E = elements per piece.
template <int D, int E, typename PA, typename PB>
__device__ __forceinline__ double row_dot(PA a, PB b) {
  double acc[4] = {0.0, 0.0, 0.0, 0.0};  // independent chains; summed in a fixed order
#pragma unroll 4
  for (int s = 0; s < D / E; ++s) {
    const u32x4 x = a[s], y = b[s];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      if (E == 4) {
        acc[w] += static_cast<double>(__uint_as_float(x[w])) * static_cast<double>(__uint_as_float(y[w]));
      } else {
        acc[w] += static_cast<double>(__uint_as_float(x[w] << 16)) * static_cast<double>(__uint_as_float(y[w] << 16));
        acc[w] += static_cast<double>(__uint_as_float(x[w] & 0xFFFF0000u)) *
                  static_cast<double>(__uint_as_float(y[w] & 0xFFFF0000u));
      }
    }
  }
  return (acc[0] + acc[1]) + (acc[2] + acc[3]);
}

}  // namespace

// lds_rows = prompt keys that fit in the launch's dynamic LDS; problems with at most
// that many stage them there, longer prompts read them from memory.
constexpr int kRowsPerGroup = 64;  // rows per workgroup of 256 threads

template <int D, int E>
__global__ __launch_bounds__(256) void prompt_lse_rows(LaunchParams prm, int blocks_per_problem,
                                                       int lds_rows) {
  extern __shared__ __align__(16) char smem[];
  const int p = blockIdx.x / blocks_per_problem;
  const finch_problem pb = prm.probs[p];
  const int n_que = pb.n_que;
  const int R = prm.group * n_que;
  const int row0 = (blockIdx.x - p * blocks_per_problem) * kRowsPerGroup;
  if (row0 >= R) return;
  const FINCH_GLOBAL u32x4* kq = as_global<u32x4>(pb.k_que);
  const bool staged = n_que <= lds_rows;
  u32x4* lkq = reinterpret_cast<u32x4*>(smem);
  if (staged) {
    for (int i = threadIdx.x; i < n_que * (D / E); i += 256) lkq[i] = kq[i];
    __syncthreads();
  }
  // lanes 4i .. 4i+3 share row row0 + i; clamped rows compute and store nothing
  const int row = min(row0 + (static_cast<int>(threadIdx.x) >> 2), R - 1);
  const int part = threadIdx.x & 3;
  constexpr int kPieces = D / E / 4;  // 16-byte pieces per lane
  const int t = row % n_que;
  const FINCH_GLOBAL u32x4* q = as_global<u32x4>(pb.q) + static_cast<size_t>(row) * (D / E) + part * kPieces;
  const double scale = 1.0 / sqrt(static_cast<double>(D));
  double m = -__builtin_inf(), z = 0.0;
  for (int j = 0; j <= t; ++j) {
    const size_t off = static_cast<size_t>(j) * (D / E) + part * kPieces;
    double dot = staged ? row_dot<D / 4, E>(q, lkq + off) : row_dot<D / 4, E>(q, kq + off);
    dot += __shfl_xor(dot, 1);
    dot += __shfl_xor(dot, 2);
    const double s = dot * scale;
    if (s > m) {
      z = z * exp(m - s) + 1.0;   // exp(-inf) = 0 on the first key
      m = s;
    } else {
      z += exp(s - m);
    }
  }
  if (part == 0 && row0 + (static_cast<int>(threadIdx.x) >> 2) < R)
    as_global_mut<float>(pb.lse_extra)[row] = static_cast<float>(m + log(z));
}

hipError_t launch_prompt_lse(const LaunchParams& p, int head_dim, bool bf16, int rows_max, hipStream_t s) {
  if (p.n_problems == 0 || rows_max <= 0) return hipSuccess;
  const int bpp = (rows_max + kRowsPerGroup - 1) / kRowsPerGroup;
  const dim3 grid(static_cast<unsigned>(bpp) * static_cast<unsigned>(p.n_problems)), block(256);
  // prompt keys in LDS: as many as the longest prompt has, up to 48 KB (no opt-in needed)
  const int row_bytes = head_dim * (bf16 ? 2 : 4);
  int lds_rows = rows_max / (p.group > 0 ? p.group : 1);
  if (lds_rows * row_bytes > 48 * 1024) lds_rows = 48 * 1024 / row_bytes;
  const size_t lds = static_cast<size_t>(lds_rows) * row_bytes;
  if (bf16 && head_dim == 128) {
    hipLaunchKernelGGL((prompt_lse_rows<128, 8>), grid, block, lds, s, p, bpp, lds_rows);
  } else if (bf16 && head_dim == 64) {
    hipLaunchKernelGGL((prompt_lse_rows<64, 8>), grid, block, lds, s, p, bpp, lds_rows);
  } else if (!bf16 && head_dim == 128) {
    hipLaunchKernelGGL((prompt_lse_rows<128, 4>), grid, block, lds, s, p, bpp, lds_rows);
  } else if (!bf16 && head_dim == 64) {
    hipLaunchKernelGGL((prompt_lse_rows<64, 4>), grid, block, lds, s, p, bpp, lds_rows);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace finch
