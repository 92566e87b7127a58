// Single-pass scoring for bf16 Q/K on gfx950 (Background, attention equation;
// Method, sum over heads / prompt-guided sub-matrix / aggregation over prompt rows).
//
// The per-key score  sum_i exp(s_ij - lse_i)  needs lse_i over ALL keys of the
// problem before any column sum can be finished.  Instead of a second pass over K
// (a second contraction and a second exp per logit), every workgroup keeps its
// tile's  E_ij = exp2(s'_ij - m_i)  (m_i = a tile-local row maximum) in registers,
// publishes the tile's per-row (max, sum) pairs and bumps its problem's arrival
// counter.  The tile that arrives last merges all pairs into lse_i and hands it to
// the others, which wait for it; every tile then finishes with
// score_j = sum_i E_ij * exp2(m_i - lse_i): one contraction and one exp per logit.
//
// Workgroup = 512 threads = 8 waves on a tile of 128 keys: wave (kb, rh) owns key
// block kb (32 keys, loaded from HBM straight into MFMA A registers) and the
// row-block half rh of the prompt rows (read from LDS as B operands), so its
// share of E is at most 4 x 16 registers and four waves fit on a SIMD.
//
// Forward progress.  Waiting workgroups need the other tiles of their problem to
// be resident.  Tiles are handed out by atomic tickets in the order workgroups
// actually start (one queue per block-id residue mod 8, i.e. per XCD under
// round-robin dispatch), so at most one problem per queue can be partly started;
// the host only chooses this kernel when 8 * (tiles_per_problem - 1) is below the
// number of workgroups the device holds at once.  The wait is bounded anyway: a
// workgroup that spins past the limit raises the context's error word and goes
// on, so every wave always exits.
#include "score_common.h"

namespace finch {

namespace {

constexpr int kThreads = kFusedThreads;

__device__ __forceinline__ void store_stat(float2* p, float m, float z) {
  const unsigned long long bits =
      (static_cast<unsigned long long>(__float_as_uint(z)) << 32) | __float_as_uint(m);
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), bits, __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ float2 load_stat(const float2* p) {
  const unsigned long long bits =
      __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED,
                        __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float(static_cast<unsigned>(bits)),
                     __uint_as_float(static_cast<unsigned>(bits >> 32)));
}

}  // namespace

template <int D, int NQ>
__global__ __launch_bounds__(kThreads, 4) void score_fused_bf16(LaunchParams prm) {
  extern __shared__ __align__(16) char smem[];
  __shared__ int sh_slot;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t = lane & 31, h = lane >> 5;
  const int kb = wave & 3, rh = wave >> 2;
  unsigned* sync = prm.sync;
  const int cls = blockIdx.x & 7;
  unsigned long long* tlog = prm.timing ? prm.timing + static_cast<size_t>(blockIdx.x) * 8 : nullptr;
#define FINCH_STAMP(i) if (tlog && tid == 0) tlog[i] = wall_clock64()
  FINCH_STAMP(0);
  if (tid == 0)
    sh_slot = static_cast<int>(__hip_atomic_fetch_add(&sync[kSyncTicket + cls * 16], 1u,
                                                      __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
  __syncthreads();
  const int slot = __builtin_amdgcn_readfirstlane(sh_slot);  // uniform: scalar descriptor loads
  const int pg = slot / prm.tiles_fused;
  const int tile = slot - pg * prm.tiles_fused;
  const int p = pg * 8 + cls;
  const int key0 = tile * kFusedKeys;
  bool active = p < prm.n_problems;
  int N = 0;
  if (active) {
    N = prm.probs[p].c + prm.probs[p].m;
    active = key0 < N;
  }

  if (active) {
    const finch_problem pb = prm.probs[p];
    const int R = prm.group * pb.n_que;
    const int rpad = round_up32(R);
    const int QB = rpad >> 5;
    const int tiles_p = (N + kFusedKeys - 1) / kFusedKeys;
    constexpr int kStride = D * 2 + 16;
    const int rows_lds = prm.rpad_max;
    char* lds_q = smem;
    float2* lds_st = reinterpret_cast<float2*>(smem + rows_lds * kStride);  // [4][rows_lds]
    float* lds_lse = reinterpret_cast<float*>(lds_st + 4 * rows_lds);       // [rows_lds]
    float* lds_col = lds_lse + rows_lds;                                    // [2][128]

    bf16x8 kf[D / 16];
    const int kbase = key0 + kb * 32;
    load_k_block<D>(pb, N, kbase, lane, kf);
    stage_q<D, kThreads>(pb.q, R, 0, rpad, lds_q, tid);
    __syncthreads();
    FINCH_STAMP(1);

    const float sc = prm.scale_log2;
    const bool ragged = kbase + 32 > N;
    float E[NQ][16];
    float mref[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const int qb = rh * NQ + q;
      if (qb < QB) {
        bf16x8 qf[D / 16];
        load_q_frags<D>(lds_q, qb, lane, qf);
        f32x16 a = mfma_block<D>(kf, qf);
        float mx = -kInf;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float s = a[v];
          if (ragged && kbase + acc_key(v, h) >= N) s = -kInf;
          a[v] = s;
          mx = fmaxf(mx, s);
        }
        const float ms = (mx == -kInf) ? 0.f : mx * sc;
        float z = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float e = fast_exp2(__builtin_fmaf(a[v], sc, -ms));
          E[q][v] = e;
          z += e;
        }
        float m = (mx == -kInf) ? -kInf : ms;
        mref[q] = m;  // reference of this lane-half's 16 keys
        const float m2 = __shfl_xor(m, 32);
        const float z2 = __shfl_xor(z, 32);
        merge_stats(m, z, m2, z2);
        if (h == 0) lds_st[kb * rows_lds + qb * 32 + t] = make_float2(m, z);
      } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) E[q][v] = 0.f;
        mref[q] = -kInf;
      }
    }
    __syncthreads();
    FINCH_STAMP(2);

    // Publish this tile's row statistics.  Shared words are written and read with
    // device-scope atomics (they bypass the per-CU cache and are coherent between
    // the L2s); ordering comes from waiting for the stores to complete before the
    // arrival counter is bumped, not from cache write-backs or invalidations.
    float2* gst = prm.stats + (static_cast<size_t>(p) * prm.tiles_fused + tile) * prm.rpad_max;
    if (tid < rpad) {
      float2 a = lds_st[tid];
#pragma unroll
      for (int w = 1; w < 4; ++w) {
        const float2 b = lds_st[w * rows_lds + tid];
        merge_stats(a.x, a.y, b.x, b.y);
      }
      store_stat(gst + tid, a.x, a.y);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // s_waitcnt: stores done
    __syncthreads();
    unsigned* arrive = sync + kSyncProblems + 2 * p;
    float* glse = prm.lse + static_cast<size_t>(p) * prm.rpad_max;
    if (tid == 0) {
      const unsigned old =
          __hip_atomic_fetch_add(arrive, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      sh_slot = (old == static_cast<unsigned>(tiles_p) - 1u) ? 1 : 0;  // 1: all tiles are in
    }
    __syncthreads();
    FINCH_STAMP(3);
    const bool combiner = __builtin_amdgcn_readfirstlane(sh_slot) != 0;
    if (tlog && tid == 0) tlog[7] = (static_cast<unsigned long long>(p) << 32) | (tile << 1) | (combiner ? 1 : 0);
    if (combiner) {
      // The last tile to arrive merges all tiles' statistics into lse per prompt
      // row (thread (row, part) takes every second tile, fixed order), hands the
      // result to the waiting tiles and bumps the counter once more.
      const int row = tid & 255, part = tid >> 8;
      if (row < rpad) {
        float m = -kInf, z = 0.f;
        if (row < R) {
          const float2* st =
              prm.stats + static_cast<size_t>(p) * prm.tiles_fused * prm.rpad_max + row;
          constexpr int kBatch = NQ >= 4 ? 4 : 8;  // loads in flight per thread
          for (int tl0 = part; tl0 < tiles_p; tl0 += 2 * kBatch) {
            float2 sv[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
              const int tl = tl0 + 2 * j;
              sv[j] = tl < tiles_p ? load_stat(st + static_cast<size_t>(tl) * prm.rpad_max)
                                   : make_float2(-kInf, 0.f);
            }
#pragma unroll
            for (int j = 0; j < kBatch; ++j) merge_stats(m, z, sv[j].x, sv[j].y);
          }
        }
        lds_st[part * rows_lds + row] = make_float2(m, z);
      }
      __syncthreads();
      if (tid < rpad) {
        float2 a = lds_st[tid];
        const float2 b = lds_st[rows_lds + tid];
        merge_stats(a.x, a.y, b.x, b.y);
        const float l = (tid < R) ? a.x + fast_log2(a.y) : kInf;
        lds_lse[tid] = l;
        __hip_atomic_store(glse + tid, l, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      __syncthreads();
      if (tid == 0)
        __hip_atomic_fetch_add(arrive, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
      if (tid == 0) {
        unsigned spins = 0;
        while (__hip_atomic_load(arrive, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) <=
               static_cast<unsigned>(tiles_p)) {
          __builtin_amdgcn_s_sleep(4);
          if (++spins > prm.spin_limit) {
            __hip_atomic_fetch_or(&sync[kSyncError], 1u, __ATOMIC_RELAXED,
                                  __HIP_MEMORY_SCOPE_AGENT);
            break;
          }
        }
      }
      __syncthreads();
      if (tid < rpad)
        lds_lse[tid] = __hip_atomic_load(glse + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __syncthreads();
    }

    FINCH_STAMP(4);
    // per-key sums over this wave's rows, folded over lanes, then over row halves
    float u[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) u[v] = 0.f;
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const int qb = rh * NQ + q;
      if (qb < QB) {
        const float w = fast_exp2(mref[q] - lds_lse[qb * 32 + t]);
#pragma unroll
        for (int v = 0; v < 16; ++v) u[v] = __builtin_fmaf(E[q][v], w, u[v]);
      }
    }
    const float tot = fold16_over32(u, t);
    if ((t & 1) == 0) lds_col[rh * kFusedKeys + kb * 32 + acc_key(t >> 1, h)] = tot;
    __syncthreads();
    if (tid < kFusedKeys) {
      const int key = key0 + tid;
      FINCH_GLOBAL float* dst = as_global_mut<float>(
          pb.scores ? pb.scores : prm.ws_scores + static_cast<size_t>(p) * prm.score_stride);
      if (key < N) dst[key] = lds_col[tid] + lds_col[kFusedKeys + tid];
    }

    // leave: the last tile of the problem clears its counters for the next launch
    __syncthreads();
    FINCH_STAMP(5);
    if (tid == 0) {
      const unsigned d =
          __hip_atomic_fetch_add(arrive + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (d == static_cast<unsigned>(tiles_p) - 1u) {
        __hip_atomic_store(arrive, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(arrive + 1, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }

  // retire: the last workgroup of the grid clears the ticket queues
  if (tid == 0) {
    const unsigned d = __hip_atomic_fetch_add(&sync[kSyncDone], 1u, __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_AGENT);
    if (d == gridDim.x - 1u) {
      for (int c = 0; c < 8; ++c)
        __hip_atomic_store(&sync[kSyncTicket + c * 16], 0u, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(&sync[kSyncDone], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

unsigned fused_grid(const LaunchParams& p) {
  return 8u * static_cast<unsigned>((p.n_problems + 7) / 8) * static_cast<unsigned>(p.tiles_fused);
}

size_t fused_lds_bytes(int head_dim, int rpad_max) {
  return static_cast<size_t>(rpad_max) * (head_dim * 2 + 16 + 4 * sizeof(float2) + sizeof(float)) +
         2 * kFusedKeys * sizeof(float);
}

namespace {

template <int D, int NQ>
hipError_t launch_one(const LaunchParams& p, size_t lds, hipStream_t s) {
  hipLaunchKernelGGL((score_fused_bf16<D, NQ>), dim3(fused_grid(p)), dim3(kThreads), lds, s, p);
  return hipGetLastError();
}

template <int D, int NQ>
const void* kernel_ptr() {
  return reinterpret_cast<const void*>(&score_fused_bf16<D, NQ>);
}

const void* fused_kernel(int head_dim, int nq) {
  if (head_dim == 128) {
    switch (nq) {
      case 1: return kernel_ptr<128, 1>();
      case 2: return kernel_ptr<128, 2>();
      case 3: return kernel_ptr<128, 3>();
      case 4: return kernel_ptr<128, 4>();
    }
  } else {
    switch (nq) {
      case 1: return kernel_ptr<64, 1>();
      case 2: return kernel_ptr<64, 2>();
      case 3: return kernel_ptr<64, 3>();
      case 4: return kernel_ptr<64, 4>();
    }
  }
  return nullptr;
}

}  // namespace

hipError_t launch_fused_bf16(int head_dim, int nq, const LaunchParams& p, size_t lds,
                             hipStream_t s) {
  if (head_dim == 128) {
    switch (nq) {
      case 1: return launch_one<128, 1>(p, lds, s);
      case 2: return launch_one<128, 2>(p, lds, s);
      case 3: return launch_one<128, 3>(p, lds, s);
      case 4: return launch_one<128, 4>(p, lds, s);
    }
  } else if (head_dim == 64) {
    switch (nq) {
      case 1: return launch_one<64, 1>(p, lds, s);
      case 2: return launch_one<64, 2>(p, lds, s);
      case 3: return launch_one<64, 3>(p, lds, s);
      case 4: return launch_one<64, 4>(p, lds, s);
    }
  }
  return hipErrorInvalidValue;
}

hipError_t set_max_lds_fused(size_t bytes) {
  for (int d = 64; d <= 128; d += 64)
    for (int nq = 1; nq <= 4; ++nq) {
      const hipError_t e = hipFuncSetAttribute(fused_kernel(d, nq),
                                               hipFuncAttributeMaxDynamicSharedMemorySize,
                                               static_cast<int>(bytes));
      if (e != hipSuccess) return e;
    }
  return hipSuccess;
}

// Workgroups of the fused kernel one compute unit holds at once for this LDS size.
hipError_t fused_blocks_per_cu(int head_dim, int nq, size_t lds, int* blocks) {
  return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks, fused_kernel(head_dim, nq), kThreads,
                                                      lds);
}

}  // namespace finch
