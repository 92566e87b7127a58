// Scoring kernels for bf16 Q/K on gfx950: the attention weights of the stacked
// prompt rows over the context keys (Background, attention equation; Method,
// "sum over heads" / "prompt-guided sub-matrix" / aggregation over prompt rows),
// never materialised: only per-row softmax statistics and per-key column sums
// leave the chip.
//
// Layout of the contraction.  One workgroup owns a tile of kTileKeys = 256
// consecutive keys of one problem; each of its 4 waves owns two 32-key blocks
// whose rows it loads once from HBM straight into MFMA A-operand registers (a
// K row is contiguous along d, which is exactly what the A operand wants).  The
// prompt rows are staged once per workgroup in LDS and read as B operands, 32
// rows at a time.  v_mfma_f32_32x32x16_bf16 then yields a 32 keys x 32 rows
// block of logits with one prompt row per lane column: row statistics are
// lane-local, and the per-key sums over rows accumulate lane-locally across
// row blocks and are folded across lanes once per key block.
//
// Pass 1 (rowstats) : per (tile, prompt row) the pair (max, sum exp2) in the
//                     log2 domain; a small kernel merges tiles into lse[row].
// Pass 2 (colsum)   : recomputes the logits and adds exp2(s - lse[row]) into the
//                     per-key sums, i.e. the probabilities themselves in fp32.
#include "score_common.h"

namespace finch {

namespace {

constexpr int kWaves = 4;
constexpr int kKB = 2;  // 32-key blocks per wave: kWaves * kKB * 32 == kTileKeys
static_assert(kWaves * kKB * 32 == kTileKeys, "tile shape");

// Workgroup -> (problem, tile).  Consecutive tiles of one problem get block ids
// that are congruent mod 8, so that under round-robin dispatch they land on one
// XCD and share its L2 (the staged prompt rows, the row statistics).
__device__ __forceinline__ bool decode_tile(const LaunchParams& prm, int& p, int& tile) {
  const int bid = blockIdx.x;
  const int xcd = bid & 7;
  const int slot = bid >> 3;
  const int pg = slot / prm.tiles_max;
  tile = slot - pg * prm.tiles_max;
  p = pg * 8 + xcd;
  return p < prm.n_problems;
}

// logits[key][row] for the wave's key blocks against row block qb, raw dot
// products (not yet scaled).
template <int D>
__device__ __forceinline__ void logits_block(const bf16x8 (&kf)[kKB][D / 16], const char* lds_q,
                                             int qb, int lane, f32x16 (&acc)[kKB]) {
  bf16x8 qf[D / 16];
  load_q_frags<D>(lds_q, qb, lane, qf);
#pragma unroll
  for (int j = 0; j < kKB; ++j) acc[j] = mfma_block<D>(kf[j], qf);
}

}  // namespace

template <int D>
__global__ __launch_bounds__(256) void rowstats_bf16(LaunchParams prm) {
  extern __shared__ __align__(16) char smem[];
  int p, tile;
  if (!decode_tile(prm, p, tile)) return;
  const finch_problem pb = prm.probs[p];
  const int N = pb.c + pb.m;
  const int key0 = tile * kTileKeys;
  if (key0 >= N) return;
  const int R = prm.group * pb.n_que;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t = lane & 31, h = lane >> 5;
  constexpr int kStride = D * 2 + 16;
  char* lds_q = smem;
  float2* wstats = reinterpret_cast<float2*>(smem + prm.row_chunk * kStride);

  bf16x8 kf[kKB][D / 16];
  int kbase[kKB];
#pragma unroll
  for (int j = 0; j < kKB; ++j) {
    kbase[j] = key0 + (wave * kKB + j) * 32;
    load_k_block<D>(pb, N, kbase[j], lane, kf[j]);
  }
  float2* out = prm.stats + (static_cast<size_t>(p) * prm.tiles_max + tile) * prm.rpad_max;
  const float sc = prm.scale_log2;

  for (int row0 = 0; row0 < R; row0 += prm.row_chunk) {
    const int rows = min(prm.row_chunk, round_up32(R - row0));
    stage_q<D, kWaves * 64>(pb.q, R, row0, rows, lds_q, tid);
    __syncthreads();
    for (int qb = 0; qb < rows / 32; ++qb) {
      f32x16 acc[kKB];
      logits_block<D>(kf, lds_q, qb, lane, acc);
      float mx = -kInf;
#pragma unroll
      for (int j = 0; j < kKB; ++j) {
        const bool ragged = kbase[j] + 32 > N;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float s = acc[j][v];
          if (ragged && kbase[j] + acc_key(v, h) >= N) s = -kInf;
          acc[j][v] = s;
          mx = fmaxf(mx, s);
        }
      }
      const float ms = (mx == -kInf) ? 0.f : mx * sc;
      float z = 0.f;
#pragma unroll
      for (int j = 0; j < kKB; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) z += fast_exp2(__builtin_fmaf(acc[j][v], sc, -ms));
      float m = (mx == -kInf) ? -kInf : ms;
      const float m2 = __shfl_xor(m, 32);
      const float z2 = __shfl_xor(z, 32);
      merge_stats(m, z, m2, z2);
      if (h == 0) wstats[wave * prm.row_chunk + qb * 32 + t] = make_float2(m, z);
    }
    __syncthreads();
    for (int i = tid; i < rows; i += kWaves * 64) {
      float2 a = wstats[i];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) {
        const float2 b = wstats[w * prm.row_chunk + i];
        merge_stats(a.x, a.y, b.x, b.y);
      }
      out[row0 + i] = a;
    }
    __syncthreads();
  }
}

template <int D>
__global__ __launch_bounds__(256) void colsum_bf16(LaunchParams prm) {
  extern __shared__ __align__(16) char smem[];
  int p, tile;
  if (!decode_tile(prm, p, tile)) return;
  const finch_problem pb = prm.probs[p];
  const int N = pb.c + pb.m;
  const int key0 = tile * kTileKeys;
  if (key0 >= N) return;
  const int R = prm.group * pb.n_que;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t = lane & 31, h = lane >> 5;
  constexpr int kStride = D * 2 + 16;
  char* lds_q = smem;
  float* lds_lse = reinterpret_cast<float*>(smem + prm.row_chunk * kStride);

  bf16x8 kf[kKB][D / 16];
  int kbase[kKB];
#pragma unroll
  for (int j = 0; j < kKB; ++j) {
    kbase[j] = key0 + (wave * kKB + j) * 32;
    load_k_block<D>(pb, N, kbase[j], lane, kf[j]);
  }
  const float* lse = prm.lse + static_cast<size_t>(p) * prm.rpad_max;
  const float sc = prm.scale_log2;
  float u[kKB][16];
#pragma unroll
  for (int j = 0; j < kKB; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) u[j][v] = 0.f;

  for (int row0 = 0; row0 < R; row0 += prm.row_chunk) {
    const int rows = min(prm.row_chunk, round_up32(R - row0));
    stage_q<D, kWaves * 64>(pb.q, R, row0, rows, lds_q, tid);
    for (int i = tid; i < rows; i += kWaves * 64) lds_lse[i] = lse[row0 + i];
    __syncthreads();
    for (int qb = 0; qb < rows / 32; ++qb) {
      f32x16 acc[kKB];
      logits_block<D>(kf, lds_q, qb, lane, acc);
      const float L = lds_lse[qb * 32 + t];  // +inf for padding rows: they add 0
#pragma unroll
      for (int j = 0; j < kKB; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) u[j][v] += fast_exp2(__builtin_fmaf(acc[j][v], sc, -L));
    }
    __syncthreads();
  }

  FINCH_GLOBAL float* dst = as_global_mut<float>(
      pb.scores ? pb.scores : prm.ws_scores + static_cast<size_t>(p) * prm.score_stride);
#pragma unroll
  for (int j = 0; j < kKB; ++j) {
    const float tot = fold16_over32(u[j], t);
    const int key = kbase[j] + acc_key(t >> 1, h);
    if ((t & 1) == 0 && key < N) dst[key] = tot;
  }
}

// Merge the per-tile statistics of every prompt row into its log2-domain
// log-sum-exp.  Padding rows (>= R) get +inf so that they contribute exp2(-inf)=0.
__global__ __launch_bounds__(256) void lse_merge(LaunchParams prm) {
  const int p = blockIdx.x;
  const finch_problem pb = prm.probs[p];
  const int N = pb.c + pb.m;
  const int R = prm.group * pb.n_que;
  const int tiles = (N + kTileKeys - 1) / kTileKeys;
  const int rpad = round_up32(R);
  const float2* st = prm.stats + static_cast<size_t>(p) * prm.tiles_max * prm.rpad_max;
  float* lse = prm.lse + static_cast<size_t>(p) * prm.rpad_max;
  for (int row = threadIdx.x; row < rpad; row += blockDim.x) {
    float out = kInf;
    if (row < R && tiles > 0) {
      float m = -kInf, z = 0.f;
      for (int tl = 0; tl < tiles; ++tl) {
        const float2 s = st[static_cast<size_t>(tl) * prm.rpad_max + row];
        merge_stats(m, z, s.x, s.y);
      }
      out = m + fast_log2(z);
    }
    lse[row] = out;
  }
}

hipError_t launch_lse(const LaunchParams& p, hipStream_t s) {
  if (p.n_problems == 0) return hipSuccess;
  hipLaunchKernelGGL(lse_merge, dim3(p.n_problems), dim3(256), 0, s, p);
  return hipGetLastError();
}

unsigned score_grid(const LaunchParams& p) {
  return 8u * static_cast<unsigned>((p.n_problems + 7) / 8) * static_cast<unsigned>(p.tiles_max);
}

hipError_t launch_rowstats_bf16(int head_dim, const LaunchParams& p, size_t lds, hipStream_t s) {
  const dim3 grid(score_grid(p)), block(256);
  if (head_dim == 128) {
    hipLaunchKernelGGL(rowstats_bf16<128>, grid, block, lds, s, p);
  } else {
    hipLaunchKernelGGL(rowstats_bf16<64>, grid, block, lds, s, p);
  }
  return hipGetLastError();
}

hipError_t launch_colsum_bf16(int head_dim, const LaunchParams& p, size_t lds, hipStream_t s) {
  const dim3 grid(score_grid(p)), block(256);
  if (head_dim == 128) {
    hipLaunchKernelGGL(colsum_bf16<128>, grid, block, lds, s, p);
  } else {
    hipLaunchKernelGGL(colsum_bf16<64>, grid, block, lds, s, p);
  }
  return hipGetLastError();
}

hipError_t set_max_lds_bf16(size_t bytes) {
  hipError_t e;
  const int b = static_cast<int>(bytes);
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(&rowstats_bf16<128>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, b);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(&rowstats_bf16<64>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, b);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(&colsum_bf16<128>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, b);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&colsum_bf16<64>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, b);
}

}  // namespace finch
