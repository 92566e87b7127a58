// Two-pass scoring for bf16 Q/K on gfx950: the attention weights of the stacked
// prompt rows over the context keys (Background, attention equation; Method,
// "sum over heads" / "prompt-guided sub-matrix" / aggregation over prompt rows),
// never materialised: only per-row softmax statistics and per-key column sums
// leave the chip.
//
// Work split.  The keys of one problem are cut into a few long slices (about 2400
// keys each); one workgroup of 8 waves streams one slice.  Each wave walks over
// 32-key blocks of the slice, loading a block's rows from HBM straight into MFMA
// A-operand registers (a K row is contiguous along d, which is what the A operand
// wants) while the previous block is being processed, so the load latency is
// hidden behind arithmetic.  The prompt rows are staged once per workgroup in LDS
// and read as B operands, 32 rows at a time.  v_mfma_f32_32x32x16_bf16 then yields
// 32 keys x 32 rows of logits with one prompt row per lane: row statistics are
// lane-local, and per-key sums accumulate lane-locally over the row blocks and are
// folded across lanes once per key block.
//
// Pass 1 (rowstats) : running (max, sum exp2) per prompt row in the log2 domain,
//                     per slice; lse_merge merges the slices into lse[row].
// Pass 2 (colsum)   : recomputes the logits and adds exp2(s - lse[row]) into the
//                     per-key sums, i.e. the probabilities themselves in fp32.
#include "score_common.h"

namespace finch {

namespace {

constexpr int kThreads = kStreamThreads;
constexpr int kWaves = kThreads / 64;

// Workgroup -> (problem, slice).  All slices of one problem get block ids that
// are congruent mod 8, so that under round-robin dispatch they land on one XCD
// and share its L2 (the staged prompt rows; the keys again in pass 2).
__device__ __forceinline__ bool decode_slice(const LaunchParams& prm, int& p, int& slice) {
  const int bid = blockIdx.x;
  const int xcd = bid & 7;
  const int slot = bid >> 3;
  const int pg = slot / prm.tiles_max;
  slice = slot - pg * prm.tiles_max;
  p = pg * 8 + xcd;
  return p < prm.n_problems;
}

// Key blocks [b0, b1) of slice `slice` of a problem with N keys.
__device__ __forceinline__ void slice_blocks(int N, int S, int slice, int& b0, int& b1) {
  const int nb = (N + 31) >> 5;
  const int per = (nb + S - 1) / S;
  b0 = slice * per;
  b1 = min(nb, b0 + per);
}

// Next key block of the slice for this wave: the waves of a workgroup take blocks
// from a shared LDS counter, so a wave that falls behind simply takes fewer.
__device__ __forceinline__ int next_block(int* counter, int lane) {
  int v = 0;
  if (lane == 0) v = atomicAdd(counter, 1);
  return __builtin_amdgcn_readfirstlane(v);
}

}  // namespace

// ---------------------------------------------------------------- pass 1
// QBT = row blocks (of 32 prompt rows) the kernel is compiled for.
template <int D, int QBT>
__global__ __launch_bounds__(kThreads, 4) void rowstats_bf16(LaunchParams prm) {
  extern __shared__ __align__(16) char smem[];
  int p, slice;
  if (!decode_slice(prm, p, slice)) return;
  const finch_problem pb = prm.probs[p];
  const int N = pb.c + pb.m;
  if (N == 0 || slice >= stream_slices(N, prm.slice_keys)) return;
  int b0, b1;
  slice_blocks(N, stream_slices(N, prm.slice_keys), slice, b0, b1);
  const int R = prm.group * pb.n_que;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t = lane & 31, h = lane >> 5;
  constexpr int kStride = D * 2 + 16;
  char* lds_q = smem;
  float2* wstats = reinterpret_cast<float2*>(smem + prm.row_chunk * kStride);  // [kWaves][rows]
  float2* out = prm.stats + (static_cast<size_t>(p) * prm.tiles_max + slice) * prm.rpad_max;
  const float sc = prm.scale_log2;

  for (int row0 = 0; row0 < R; row0 += prm.row_chunk) {
    const int rows = min(prm.row_chunk, round_up32(R - row0));
    const int QB = rows >> 5;
    stage_q<D, kThreads>(pb.q, R, row0, rows, lds_q, tid);
    __syncthreads();

    float m_run[QBT], z_run[QBT];
#pragma unroll
    for (int q = 0; q < QBT; ++q) {
      m_run[q] = -kInf;
      z_run[q] = 0.f;
    }

    // The running reference m_run of a row only has to keep exp2 in range, so it is
    // taken from the wave's first key block and moved (with the sum rescaled) only
    // when a block's sum shows that its logits lie far above it.
    bool seeded = false;
    auto process = [&](const bf16x8(&kf)[D / 16], int b) {
      const int kbase = b << 5;
      const bool ragged = kbase + 32 > N;
#pragma unroll
      for (int q = 0; q < QBT; ++q) {
        if (q < QB) {
          bf16x8 qf[D / 16];
          load_q_frags<D>(lds_q, q, lane, qf);
          f32x16 a = mfma_block<D>(kf, qf);
          if (ragged) {
#pragma unroll
            for (int v = 0; v < 16; ++v)
              if (kbase + acc_key(v, h) >= N) a[v] = -kInf;
          }
          float z = 0.f;
          bool move = !seeded;
          if (seeded) {
            const float mu = (m_run[q] == -kInf) ? 0.f : m_run[q];
#pragma unroll
            for (int v = 0; v < 16; ++v) z += fast_exp2(__builtin_fmaf(a[v], sc, -mu));
            // (A lane without a reference - every key it has seen was masked - never meets a
            // key it sees later on: masked keys are the ones past a limit, a wave's blocks come
            // in ascending key order, and inside a block a lane's keys ascend too.)
            move = __any(!(z <= 0x1p64f));
          }
          if (move) {
            float bm = fmaxf(a[0], a[1]);
#pragma unroll
            for (int v = 2; v < 16; v += 2) bm = fmaxf(fmaxf(bm, a[v]), a[v + 1]);
            const float mn = fmaxf(m_run[q], bm * sc);
            // a lane half that has seen only masked keys so far (mn still -inf) keeps
            // its empty sum
            z_run[q] = (mn == -kInf) ? 0.f : z_run[q] * fast_exp2(m_run[q] - mn);
            m_run[q] = mn;
            const float mu = (mn == -kInf) ? 0.f : mn;
            z = 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) z += fast_exp2(__builtin_fmaf(a[v], sc, -mu));
          }
          z_run[q] += z;
        }
      }
      seeded = true;
    };

    // key blocks of this wave (a fixed assignment: the order in which a row's sums
    // are added up must not depend on timing), two register sets in ping-pong
    bf16x8 ka[D / 16], kb[D / 16];
    int b = b0 + wave;
    if (b < b1) {
      load_k_block<D>(pb, N, b << 5, lane, ka);
      while (true) {
        if (b + kWaves < b1) load_k_block<D>(pb, N, (b + kWaves) << 5, lane, kb);
        process(ka, b);
        b += kWaves;
        if (b >= b1) break;
        if (b + kWaves < b1) load_k_block<D>(pb, N, (b + kWaves) << 5, lane, ka);
        process(kb, b);
        b += kWaves;
        if (b >= b1) break;
      }
    }

    // lane halves -> wave -> workgroup -> global
#pragma unroll
    for (int q = 0; q < QBT; ++q) {
      if (q < QB) {
        float m = m_run[q], z = z_run[q];
        const float m2 = __shfl_xor(m, 32);
        const float z2 = __shfl_xor(z, 32);
        merge_stats(m, z, m2, z2);
        if (h == 0) wstats[wave * prm.row_chunk + q * 32 + t] = make_float2(m, z);
      }
    }
    __syncthreads();
    for (int i = tid; i < rows; i += kThreads) {
      float2 a = wstats[i];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) {
        const float2 c = wstats[w * prm.row_chunk + i];
        merge_stats(a.x, a.y, c.x, c.y);
      }
      out[row0 + i] = a;
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------- pass 2
template <int D>
__global__ __launch_bounds__(kThreads, 4) void colsum_bf16(LaunchParams prm) {
  extern __shared__ __align__(16) char smem[];
  int p, slice;
  if (!decode_slice(prm, p, slice)) return;
  const finch_problem pb = prm.probs[p];
  const int N = pb.c + pb.m;
  if (N == 0 || slice >= stream_slices(N, prm.slice_keys)) return;
  int b0, b1;
  slice_blocks(N, stream_slices(N, prm.slice_keys), slice, b0, b1);
  const int R = prm.group * pb.n_que;
  const int tid = threadIdx.x, lane = tid & 63;
  const int t = lane & 31, h = lane >> 5;
  constexpr int kStride = D * 2 + 16;
  char* lds_q = smem;
  float* lds_lse = reinterpret_cast<float*>(smem + prm.row_chunk * kStride);
  int* sh_next = reinterpret_cast<int*>(smem + prm.row_chunk * (kStride + kWaves * 8));
  const float* lse = prm.lse + static_cast<size_t>(p) * prm.rpad_max;
  const float sc = prm.scale_log2;
  FINCH_GLOBAL float* dst = as_global_mut<float>(
      pb.scores ? pb.scores : prm.ws_scores + static_cast<size_t>(p) * prm.score_stride);

  for (int row0 = 0; row0 < R; row0 += prm.row_chunk) {
    const int rows = min(prm.row_chunk, round_up32(R - row0));
    const int QB = rows >> 5;
    const bool first_chunk = row0 == 0;
    stage_q<D, kThreads>(pb.q, R, row0, rows, lds_q, tid);
    if (tid == 0) *sh_next = 0;
    if (prm.merge_in_pass2) {
      // few slices: merge their statistics here (same order as lse_merge) instead
      // of spending a kernel launch on it
      const int S = stream_slices(N, prm.slice_keys);
      const float2* st = prm.stats + static_cast<size_t>(p) * prm.tiles_max * prm.rpad_max;
      for (int i = tid; i < rows; i += kThreads) {
        float l = kInf;
        if (row0 + i < R) {
          float m = -kInf, z = 0.f;
          for (int sl = 0; sl < S; ++sl) {
            const float2 s2 = st[static_cast<size_t>(sl) * prm.rpad_max + row0 + i];
            merge_stats(m, z, s2.x, s2.y);
          }
          l = m + fast_log2(z);
          if (pb.lse_extra) l = widen_lse(l, as_global<float>(pb.lse_extra)[row0 + i]);
        }
        lds_lse[i] = l;
      }
    } else {
      for (int i = tid; i < rows; i += kThreads) lds_lse[i] = lse[row0 + i];
    }
    __syncthreads();

    auto process = [&](const bf16x8(&kf)[D / 16], int b) {
      const int kbase = b << 5;
      float u[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) u[v] = 0.f;
      for (int q = 0; q < QB; ++q) {
        bf16x8 qf[D / 16];
        load_q_frags<D>(lds_q, q, lane, qf);
        const f32x16 a = mfma_block<D>(kf, qf);
        const float L = lds_lse[q * 32 + t];  // +inf for padding rows: they add 0
#pragma unroll
        for (int v = 0; v < 16; ++v) u[v] += fast_exp2(__builtin_fmaf(a[v], sc, -L));
      }
      const float tot = fold16_over32(u, t);
      const int key = kbase + acc_key(t >> 1, h);
      if ((t & 1) == 0 && key < N) dst[key] = first_chunk ? tot : dst[key] + tot;
    };

    // key blocks are handed out by the workgroup's counter (each key's sum is
    // computed by one wave, so the result does not depend on who takes which)
    // The slice is walked from its end: pass 1 read it front to back, so its tail is
    // what the memory-side cache is most likely to still hold.
    bf16x8 ka[D / 16], kb[D / 16];
    int b = b1 - 1 - next_block(sh_next, lane);
    if (b >= b0) {
      load_k_block<D>(pb, N, b << 5, lane, ka);
      while (true) {
        int bn = b1 - 1 - next_block(sh_next, lane);
        if (bn >= b0) load_k_block<D>(pb, N, bn << 5, lane, kb);
        process(ka, b);
        b = bn;
        if (b < b0) break;
        bn = b1 - 1 - next_block(sh_next, lane);
        if (bn >= b0) load_k_block<D>(pb, N, bn << 5, lane, ka);
        process(kb, b);
        b = bn;
        if (b < b0) break;
      }
    }
    __syncthreads();
  }
}

// Merge the per-slice statistics of every prompt row into its log2-domain
// log-sum-exp.  Padding rows (>= R) get +inf so that they contribute exp2(-inf)=0.
__global__ __launch_bounds__(256) void lse_merge(LaunchParams prm) {
  const int p = blockIdx.x;
  const finch_problem pb = prm.probs[p];
  const int N = pb.c + pb.m;
  const int R = prm.group * pb.n_que;
  const int slices = N == 0 ? 0
                     : prm.tile_keys ? (N + prm.tile_keys - 1) / prm.tile_keys
                                     : stream_slices(N, prm.slice_keys);
  const int rpad = round_up32(R);
  const float2* st = prm.stats + static_cast<size_t>(p) * prm.tiles_max * prm.rpad_max;
  float* lse = prm.lse + static_cast<size_t>(p) * prm.rpad_max;
  for (int row = threadIdx.x; row < rpad; row += blockDim.x) {
    float out = kInf;
    if (row < R && slices > 0) {
      float m = -kInf, z = 0.f;
      for (int sl = 0; sl < slices; ++sl) {
        const float2 s = st[static_cast<size_t>(sl) * prm.rpad_max + row];
        merge_stats(m, z, s.x, s.y);
      }
      out = m + fast_log2(z);
      if (pb.lse_extra) out = widen_lse(out, as_global<float>(pb.lse_extra)[row]);
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

namespace {

template <int D>
const void* rowstats_ptr(int qbt) {
  switch (qbt) {
    case 2: return reinterpret_cast<const void*>(&rowstats_bf16<D, 2>);
    case 4: return reinterpret_cast<const void*>(&rowstats_bf16<D, 4>);
    case 6: return reinterpret_cast<const void*>(&rowstats_bf16<D, 6>);
    case 8: return reinterpret_cast<const void*>(&rowstats_bf16<D, 8>);
    case 12: return reinterpret_cast<const void*>(&rowstats_bf16<D, 12>);
    default: return reinterpret_cast<const void*>(&rowstats_bf16<D, 16>);
  }
}

template <int D>
void launch_rowstats_d(int qbt, dim3 grid, size_t lds, hipStream_t s, const LaunchParams& p) {
  const dim3 block(kThreads);
  switch (qbt) {
    case 2: hipLaunchKernelGGL((rowstats_bf16<D, 2>), grid, block, lds, s, p); break;
    case 4: hipLaunchKernelGGL((rowstats_bf16<D, 4>), grid, block, lds, s, p); break;
    case 6: hipLaunchKernelGGL((rowstats_bf16<D, 6>), grid, block, lds, s, p); break;
    case 8: hipLaunchKernelGGL((rowstats_bf16<D, 8>), grid, block, lds, s, p); break;
    case 12: hipLaunchKernelGGL((rowstats_bf16<D, 12>), grid, block, lds, s, p); break;
    default: hipLaunchKernelGGL((rowstats_bf16<D, 16>), grid, block, lds, s, p); break;
  }
}

// Smallest compiled row-block count that covers `row_chunk` staged rows.
int pick_qbt(int row_chunk) {
  const int qb = (row_chunk + 31) / 32;
  const int have[6] = {2, 4, 6, 8, 12, 16};
  for (int i = 0; i < 6; ++i)
    if (qb <= have[i]) return have[i];
  return 16;
}

}  // namespace

hipError_t launch_rowstats_bf16(int head_dim, const LaunchParams& p, size_t lds, hipStream_t s) {
  const dim3 grid(score_grid(p));
  const int qbt = pick_qbt(p.row_chunk);
  if (head_dim == 128) {
    launch_rowstats_d<128>(qbt, grid, lds, s, p);
  } else {
    launch_rowstats_d<64>(qbt, grid, lds, s, p);
  }
  return hipGetLastError();
}

hipError_t launch_colsum_bf16(int head_dim, const LaunchParams& p, size_t lds, hipStream_t s) {
  const dim3 grid(score_grid(p)), block(kThreads);
  if (head_dim == 128) {
    hipLaunchKernelGGL(colsum_bf16<128>, grid, block, lds, s, p);
  } else {
    hipLaunchKernelGGL(colsum_bf16<64>, grid, block, lds, s, p);
  }
  return hipGetLastError();
}

hipError_t set_max_lds_bf16(size_t bytes) {
  const int b = static_cast<int>(bytes);
  const int qbts[6] = {2, 4, 6, 8, 12, 16};
  for (int i = 0; i < 6; ++i) {
    hipError_t e = hipFuncSetAttribute(rowstats_ptr<128>(qbts[i]),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, b);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(rowstats_ptr<64>(qbts[i]), hipFuncAttributeMaxDynamicSharedMemorySize, b);
    if (e != hipSuccess) return e;
  }
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&colsum_bf16<128>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, b);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&colsum_bf16<64>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, b);
}

}  // namespace finch
