// One kernel per prefill step for bf16 Q/K/V on gfx950: scoring pass 1, the merge
// of the row statistics, scoring pass 2, top-r and compaction (Method: attention
// of the prompt rows over cache + chunk keys, sum over heads and prompt rows,
// t = top-r(A_agg, r), Managing the Cache), without returning to the host and
// without kernel boundaries between the stages.
//
// The launch is a queue of work items taken by atomic ticket in the order
// workgroups start:
//     items [0, n1)      pass 1 of (problem, slice): running (max, sum exp2) per
//                        prompt row over the slice's keys -> stats[p][slice][row]
//     items [n1, 2*n1)   pass 2 of (problem, slice): per-key sums of
//                        exp2(s - lse[row]) -> scores
// The workgroup that finishes the LAST pass-1 slice of a problem merges the
// slices into lse[p][row] and publishes it; a pass-2 item polls for that (it only
// ever waits for items with smaller tickets, which have all started, so the wait
// cannot deadlock, and it is bounded anyway).  The workgroup that finishes the
// LAST pass-2 slice of a problem then selects the top r of the problem's scores;
// the copies of the kept K/V rows are further items (a few per problem, after all
// pass-2 items in the queue) that poll for their problem's indices.  Because items are handed out dynamically,
// workgroups that finish early move on to the next stage while slower ones are
// still busy, and the HBM-bound copies of early problems overlap the
// arithmetic-bound scoring of later ones.
//
// Words shared between workgroups (statistics, lse, scores, counters) are written
// and read with device-scope atomics, which bypass the per-CU cache and are
// coherent across the L2s; a producer waits for its stores to complete before it
// bumps the counter a consumer polls.
#include "score_common.h"

namespace finch {

namespace {

constexpr int kThreads = kStreamThreads;
constexpr int kWaves = kThreads / 64;

__device__ __forceinline__ void st_stat(float2* p, float m, float z) {
  const unsigned long long bits =
      (static_cast<unsigned long long>(__float_as_uint(z)) << 32) | __float_as_uint(m);
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), bits, __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 ld_stat(const float2* p) {
  const unsigned long long bits =
      __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED,
                        __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float(static_cast<unsigned>(bits)),
                     __uint_as_float(static_cast<unsigned>(bits >> 32)));
}
__device__ __forceinline__ void st_f32(float* p, float x) {
  __hip_atomic_store(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_f32(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned ld_u32(const unsigned* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned add_u32(unsigned* p, unsigned x) {
  return __hip_atomic_fetch_add(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// All earlier stores of this thread have completed (and the compiler keeps later
// memory operations after this point).
__device__ __forceinline__ void stores_done() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup"); }

// Monotone map float -> uint32 (larger float <=> larger key); -0 counts as +0.
__device__ __forceinline__ unsigned order_key(float f) {
  const unsigned u = __float_as_uint(f + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Exclusive rank of `flag` among the workgroup's threads in thread order, and the
// total.  Two barriers; every thread must call it.
__device__ __forceinline__ int block_rank(bool flag, int* wave_tot, int lane, int wave, int& total) {
  const unsigned long long b = __ballot(flag);
  const int below = __popcll(b & ((1ull << lane) - 1ull));
  if (lane == 0) wave_tot[wave] = __popcll(b);
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const int x = wave_tot[w];
    if (w < wave) base += x;
    tot += x;
  }
  __syncthreads();
  total = tot;
  return base + below;
}

// Key blocks [b0, b1) of slice `slice` of a problem with N keys.
__device__ __forceinline__ void slice_blocks(int N, int S, int slice, int& b0, int& b1) {
  const int nb = (N + 31) >> 5;
  const int per = (nb + S - 1) / S;
  b0 = slice * per;
  b1 = min(nb, b0 + per);
}

struct FinLds {            // layout of the LDS scratch of the selection stage
  int hist[256];
  int wave_tot[kWaves];
  int digit, remaining;
};

// Top-r of scores[0..N) -> idx (ascending), ties to the lower index.  `keys` is
// either LDS (the scores were staged there as order keys) or nullptr, in which
// case they are re-read from `gscores` each round.  Writes idx to `gidx` and, if
// `lidx` is not null, also to LDS.  Whole workgroup; r in (0, N).
__device__ __forceinline__ void select_stage(const unsigned* keys, const float* gscores, int N, int r, int* gidx,
                             int* lidx, FinLds* f, int tid, int lane, int wave) {
  auto key_at = [&](int i) -> unsigned { return keys ? keys[i] : order_key(ld_f32(gscores + i)); };
  unsigned prefix = 0, mask = 0;
  int remaining = r;
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) f->hist[tid] = 0;
    __syncthreads();
    for (int i = tid; i < N; i += kThreads) {
      const unsigned key = key_at(i);
      if ((key & mask) == prefix) atomicAdd(&f->hist[(key >> shift) & 255u], 1);
    }
    __syncthreads();
    if (wave == 0) {
      const int h0 = f->hist[4 * lane], h1 = f->hist[4 * lane + 1], h2 = f->hist[4 * lane + 2],
                h3 = f->hist[4 * lane + 3];
      const int mine = h0 + h1 + h2 + h3;
      int suffix = mine;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int x = __shfl_down(suffix, o);
        if (lane + o < 64) suffix += x;
      }
      const int above = suffix - mine;
      if (above < remaining && remaining <= suffix) {
        int left = remaining - above;
        int digit;
        if (left <= h3) {
          digit = 3;
        } else if (left <= h3 + h2) {
          digit = 2;
          left -= h3;
        } else if (left <= h3 + h2 + h1) {
          digit = 1;
          left -= h3 + h2;
        } else {
          digit = 0;
          left -= h3 + h2 + h1;
        }
        f->digit = 4 * lane + digit;
        f->remaining = left;
      }
    }
    __syncthreads();
    prefix |= static_cast<unsigned>(f->digit) << shift;
    mask |= 255u << shift;
    remaining = f->remaining;
    __syncthreads();
  }
  const unsigned T = prefix;
  const int need_eq = remaining;
  int carry_eq = 0, carry_keep = 0;
  for (int base = 0; base < N; base += kThreads) {
    const int i = base + tid;
    const bool valid = i < N;
    const unsigned key = valid ? key_at(i) : 0u;
    const bool gt = valid && key > T;
    const bool eq = valid && key == T;
    int tot_eq, tot_keep;
    const int eq_rank = carry_eq + block_rank(eq, f->wave_tot, lane, wave, tot_eq);
    const bool keep = gt || (eq && eq_rank < need_eq);
    const int pos = carry_keep + block_rank(keep, f->wave_tot, lane, wave, tot_keep);
    if (keep) {
      __hip_atomic_store(gidx + pos, i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (lidx) lidx[pos] = i;
    }
    carry_eq += tot_eq;
    carry_keep += tot_keep;
  }
}

// Copy rows idx[t0..t1) of [cache ; chunk] of K and V into k_out / v_out.  idx
// was written by another workgroup: device-scope loads.
template <int SEGS>
__device__ __forceinline__ void gather_stage(const finch_problem& pb, int N, int t0, int t1,
                                             const int* idx, int tid) {
  const FINCH_GLOBAL u32x4* kc = as_global<u32x4>(pb.k_cache);
  const FINCH_GLOBAL u32x4* kk = as_global<u32x4>(pb.k_chunk);
  const FINCH_GLOBAL u32x4* vc = as_global<u32x4>(pb.v_cache);
  const FINCH_GLOBAL u32x4* vk = as_global<u32x4>(pb.v_chunk);
  FINCH_GLOBAL u32x4* ko = as_global_mut<u32x4>(pb.k_out);
  FINCH_GLOBAL u32x4* vo = as_global_mut<u32x4>(pb.v_out);
  constexpr int kRowsPerIter = kThreads / SEGS;
  constexpr int kUnroll = 4;
  const int seg = tid % SEGS, sub = tid / SEGS;
  for (int row0 = t0; row0 < t1; row0 += kRowsPerIter * kUnroll) {
    u32x4 kv[kUnroll], vv[kUnroll];
#pragma unroll
    for (int it = 0; it < kUnroll; ++it) {
      const int t = min(row0 + it * kRowsPerIter + sub, t1 - 1);
      const int j = min(max(__hip_atomic_load(idx + t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT), 0),
                        N - 1);
      const bool cached = j < pb.c;
      const size_t off = static_cast<size_t>(cached ? j : j - pb.c) * SEGS + seg;
      kv[it] = (cached ? kc : kk)[off];
      vv[it] = (cached ? vc : vk)[off];
    }
#pragma unroll
    for (int it = 0; it < kUnroll; ++it) {
      const int t = row0 + it * kRowsPerIter + sub;
      if (t < t1) {
        ko[static_cast<size_t>(t) * SEGS + seg] = kv[it];
        vo[static_cast<size_t>(t) * SEGS + seg] = vv[it];
      }
    }
  }
}

}  // namespace

// Per-item context shared by the stage functions.
struct ItemCtx {
  int p, slice, N, S, R, rows, QB, b0, b1;
  unsigned* arr;    // {pass-1 arrivals (+1 once lse is out), pass-2 arrivals} of the problem
  float* glse;      // lse[p][.]
  float2* gstats;   // stats[p][.][.]
  float* gscores;   // scores of the problem
};

// The stage bodies are separate (non-inlined) functions so that each gets its own
// register allocation; they are called once per workgroup.
template <int D, int QBT>
__device__ __attribute__((noinline)) void pass1_item(const LaunchParams& prm, const finch_problem& pb,
                                                     const ItemCtx& c) {
  extern __shared__ __align__(16) char smem[];  // named here so that accesses stay LDS accesses
  __shared__ int sh_flag;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t = lane & 31, h = lane >> 5;
  constexpr int kStride = D * 2 + 16;
  // arguments arrive through memory: pull what the loops use into scalar registers
  const int rpad_max = uni(prm.rpad_max);
  const float sc = uni(prm.scale_log2);
  const int N = uni(c.N), QB = uni(c.QB), b1 = uni(c.b1), S = uni(c.S), R = uni(c.R),
            rows = uni(c.rows), slice = uni(c.slice);
  const KeySource ks = {uni(static_cast<const char*>(pb.k_cache)),
                        uni(static_cast<const char*>(pb.k_chunk)), uni(pb.c)};
  unsigned* arr = uni(c.arr);
  float* glse = uni(c.glse);
  float2* gstats = uni(c.gstats);
  char* lds_q = smem;
  float2* wstats = reinterpret_cast<float2*>(smem + rpad_max * kStride);  // [kWaves][rpad_max]
  bf16x8 ka[D / 16], kb[D / 16];
  int b = uni(c.b0) + wave;
  if (b < b1) load_k_block<D>(ks, N, b << 5, lane, ka);  // requested before Q is staged
  stage_q<D, kThreads>(uni(pb.q), R, 0, rows, lds_q, tid);
  __syncthreads();
  float m_run[QBT], z_run[QBT];
#pragma unroll
  for (int q = 0; q < QBT; ++q) {
    m_run[q] = -kInf;
    z_run[q] = 0.f;
  }
  auto process = [&](const bf16x8(&kf)[D / 16], int blk) {
    const int kbase = blk << 5;
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
        float bm = fmaxf(a[0], a[1]);
#pragma unroll
        for (int v = 2; v < 16; v += 2) bm = fmaxf(fmaxf(bm, a[v]), a[v + 1]);
        const float bms = bm * sc;
        if (__any(bms > m_run[q])) {  // rare after the first blocks: rescale the running sum
          const float mn = fmaxf(m_run[q], bms);
          z_run[q] = (mn == -kInf) ? 0.f : z_run[q] * fast_exp2(m_run[q] - mn);
          m_run[q] = mn;
        }
        const float mu = (m_run[q] == -kInf) ? 0.f : m_run[q];
        float z = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) z += fast_exp2(__builtin_fmaf(a[v], sc, -mu));
        z_run[q] += z;
      }
    }
  };
  if (b < b1) {
    while (true) {
      if (b + kWaves < b1) load_k_block<D>(ks, N, (b + kWaves) << 5, lane, kb);
      process(ka, b);
      b += kWaves;
      if (b >= b1) break;
      if (b + kWaves < b1) load_k_block<D>(ks, N, (b + kWaves) << 5, lane, ka);
      process(kb, b);
      b += kWaves;
      if (b >= b1) break;
    }
  }
#pragma unroll
  for (int q = 0; q < QBT; ++q) {
    if (q < QB) {
      float m = m_run[q], z = z_run[q];
      const float m2 = __shfl_xor(m, 32);
      const float z2 = __shfl_xor(z, 32);
      merge_stats(m, z, m2, z2);
      if (h == 0) wstats[wave * rpad_max + q * 32 + t] = make_float2(m, z);
    }
  }
  __syncthreads();
  float2* out = gstats + static_cast<size_t>(slice) * rpad_max;
  for (int i = tid; i < rows; i += kThreads) {
    float2 a = wstats[i];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) {
      const float2 x = wstats[w * rpad_max + i];
      merge_stats(a.x, a.y, x.x, x.y);
    }
    st_stat(out + i, a.x, a.y);
  }
  stores_done();
  __syncthreads();
  if (tid == 0) sh_flag = (add_u32(arr, 1u) == static_cast<unsigned>(S) - 1u) ? 1 : 0;
  __syncthreads();
  if (__builtin_amdgcn_readfirstlane(sh_flag)) {
    // last slice of the problem: merge the slices (fixed order) and publish lse
    for (int i = tid; i < rows; i += kThreads) {
      float l = kInf;  // padding rows add exp2(-inf) = 0 in pass 2
      if (i < R) {
        float m = -kInf, z = 0.f;
        for (int sl = 0; sl < S; ++sl) {
          const float2 s2 = ld_stat(gstats + static_cast<size_t>(sl) * rpad_max + i);
          merge_stats(m, z, s2.x, s2.y);
        }
        l = m + fast_log2(z);
      }
      st_f32(glse + i, l);
    }
    stores_done();
    __syncthreads();
    if (tid == 0) add_u32(arr, 1u);  // S + 1: lse is out
  }
}

// Returns (uniformly) whether this workgroup finished the last pass-2 slice.
template <int D>
__device__ __attribute__((noinline)) int pass2_item(const LaunchParams& prm, const finch_problem& pb,
                                                    const ItemCtx& c) {
  extern __shared__ __align__(16) char smem[];
  __shared__ int sh_flag;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t = lane & 31, h = lane >> 5;
  constexpr int kStride = D * 2 + 16;
  // arguments arrive through memory: pull what the loops use into scalar registers
  const int rpad_max = uni(prm.rpad_max);
  const float sc = uni(prm.scale_log2);
  const unsigned spin_limit = static_cast<unsigned>(uni(static_cast<int>(prm.spin_limit)));
  const int N = uni(c.N), QB = uni(c.QB), b1 = uni(c.b1), S = uni(c.S), R = uni(c.R),
            rows = uni(c.rows);
  const KeySource ks = {uni(static_cast<const char*>(pb.k_cache)),
                        uni(static_cast<const char*>(pb.k_chunk)), uni(pb.c)};
  unsigned* arr = uni(c.arr);
  float* glse = uni(c.glse);
  float* gscores = uni(c.gscores);
  unsigned* sync = uni(prm.sync);
  char* lds_q = smem;
  float* lds_lse = reinterpret_cast<float*>(smem + rpad_max * kStride);
  bf16x8 ka[D / 16], kb[D / 16];
  int b = uni(c.b0) + wave;
  if (b < b1) load_k_block<D>(ks, N, b << 5, lane, ka);
  stage_q<D, kThreads>(uni(pb.q), R, 0, rows, lds_q, tid);
  if (tid == 0) {  // wait for the problem's lse (written by items with smaller tickets)
    unsigned spins = 0;
    while (ld_u32(arr) <= static_cast<unsigned>(S)) {
      __builtin_amdgcn_s_sleep(4);
      if (++spins > spin_limit) {
        __hip_atomic_fetch_or(&sync[kSyncError], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
    }
  }
  __syncthreads();
  for (int i = tid; i < rows; i += kThreads) lds_lse[i] = ld_f32(glse + i);
  __syncthreads();
  auto process = [&](const bf16x8(&kf)[D / 16], int blk) {
    const int kbase = blk << 5;
    float u[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) u[v] = 0.f;
    for (int q = 0; q < QB; ++q) {
      bf16x8 qf[D / 16];
      load_q_frags<D>(lds_q, q, lane, qf);
      const f32x16 a = mfma_block<D>(kf, qf);
      const float L = lds_lse[q * 32 + t];
#pragma unroll
      for (int v = 0; v < 16; ++v) u[v] += fast_exp2(__builtin_fmaf(a[v], sc, -L));
    }
    const float tot = fold16_over32(u, t);
    const int key = kbase + acc_key(t >> 1, h);
    if ((t & 1) == 0 && key < N) st_f32(gscores + key, tot);
  };
  if (b < b1) {
    while (true) {
      if (b + kWaves < b1) load_k_block<D>(ks, N, (b + kWaves) << 5, lane, kb);
      process(ka, b);
      b += kWaves;
      if (b >= b1) break;
      if (b + kWaves < b1) load_k_block<D>(ks, N, (b + kWaves) << 5, lane, ka);
      process(kb, b);
      b += kWaves;
      if (b >= b1) break;
    }
  }
  stores_done();
  __syncthreads();
  if (tid == 0) sh_flag = (add_u32(arr + 1, 1u) == static_cast<unsigned>(S) - 1u) ? 1 : 0;
  __syncthreads();
  return __builtin_amdgcn_readfirstlane(sh_flag);
}

// Top-r of one problem whose scores are all out; idx goes to memory.
__device__ __attribute__((noinline)) void select_item(const LaunchParams& prm, const finch_problem& pb,
                                                      const ItemCtx& c) {
  extern __shared__ __align__(16) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int N = c.N;
  const int r = min(pb.r, N);
  if (r <= 0) return;
  int* gidx = pb.idx;
  if (r >= N) {
    for (int i = tid; i < N; i += kThreads)
      __hip_atomic_store(gidx + i, i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return;
  }
  // LDS: [order keys N][FinLds] if it fits, else the keys are re-read from memory
  const size_t need = static_cast<size_t>(N) * 4 + sizeof(FinLds);
  const bool in_lds = need <= prm.lds_bytes;
  unsigned* lkeys = in_lds ? reinterpret_cast<unsigned*>(smem) : nullptr;
  FinLds* fl = in_lds ? reinterpret_cast<FinLds*>(smem + static_cast<size_t>(N) * 4)
                      : reinterpret_cast<FinLds*>(smem);
  if (in_lds)
    for (int i = tid; i < N; i += kThreads) lkeys[i] = order_key(ld_f32(c.gscores + i));
  __syncthreads();
  select_stage(lkeys, c.gscores, N, r, gidx, nullptr, fl, tid, lane, wave);
}

// One part of the compaction of one problem: waits (bounded) for the problem's
// indices, copies its share of the kept rows, and the last part to finish clears
// the problem's counters.
template <int D>
__device__ __attribute__((noinline)) void gather_item(const LaunchParams& prm, const finch_problem& pb,
                                                      const ItemCtx& c, int part, int parts) {
  const int tid = threadIdx.x;
  if (tid == 0) {
    unsigned spins = 0;
    while (ld_u32(c.arr + 1) <= static_cast<unsigned>(c.S)) {
      __builtin_amdgcn_s_sleep(4);
      if (++spins > prm.spin_limit) {
        __hip_atomic_fetch_or(&prm.sync[kSyncError], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
    }
  }
  __syncthreads();
  const int r = min(pb.r, c.N);
  const int per = (r + parts - 1) / parts;
  const int t0 = part * per, t1 = min(r, t0 + per);
  if (t0 < t1) gather_stage<D / 8>(pb, c.N, t0, t1, pb.idx, tid);
  __syncthreads();
  if (tid == 0) {
    // pass-1 word: S + 1 since lse went out; each finished part adds one more
    if (add_u32(c.arr, 1u) == static_cast<unsigned>(c.S + parts)) {
      __hip_atomic_store(c.arr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(c.arr + 1, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

// n1 = problems * slices per problem (pass-1 items = pass-2 items); parts = copy
// items per problem (0: scoring only, nothing after pass 2).
template <int D, int QBT>
__global__ __launch_bounds__(kThreads, 4) void step_bf16(LaunchParams prm, int n1, int parts) {
  __shared__ int sh_word;
  const int tid = threadIdx.x;
  unsigned* sync = prm.sync;

  if (tid == 0) sh_word = static_cast<int>(add_u32(&sync[kSyncTicket], 1u));
  __syncthreads();
  const int item = __builtin_amdgcn_readfirstlane(sh_word);
  __syncthreads();  // sh_word is reused by the stages
  const int phase = item < n1 ? 0 : item < 2 * n1 ? 1 : 2;
  const int sub = item - (phase == 0 ? 0 : phase == 1 ? n1 : 2 * n1);
  const int per_problem = phase == 2 ? parts : prm.tiles_max;
  ItemCtx c;
  c.p = sub / per_problem;
  c.slice = sub - c.p * per_problem;  // slice of the keys, or part of the kept rows
  bool active = c.p < prm.n_problems;
  c.N = 0;
  c.S = 1;
  if (active) {
    c.N = prm.probs[c.p].c + prm.probs[c.p].m;
    c.S = stream_slices(c.N, prm.slice_keys);
    active = c.N > 0 && (phase == 2 || c.slice < c.S);
  }

  if (active) {
    const finch_problem pb = prm.probs[c.p];
    c.R = prm.group * pb.n_que;
    c.rows = round_up32(c.R);
    c.QB = c.rows >> 5;
    c.arr = sync + kSyncProblems + 2 * c.p;
    c.glse = prm.lse + static_cast<size_t>(c.p) * prm.rpad_max;
    c.gstats = prm.stats + static_cast<size_t>(c.p) * prm.tiles_max * prm.rpad_max;
    c.gscores = pb.scores ? pb.scores : prm.ws_scores + static_cast<size_t>(c.p) * prm.score_stride;
    if (phase == 0) {
      slice_blocks(c.N, c.S, c.slice, c.b0, c.b1);
      pass1_item<D, QBT>(prm, pb, c);
    } else if (phase == 1) {
      slice_blocks(c.N, c.S, c.slice, c.b0, c.b1);
      if (pass2_item<D>(prm, pb, c)) {
        // last slice of the problem: every score of the problem is out
        if (parts > 0) {
          select_item(prm, pb, c);
          stores_done();
          __syncthreads();
          if (tid == 0) add_u32(c.arr + 1, 1u);  // S + 1: the indices are out
        } else if (tid == 0) {  // scoring only: the problem is finished, clear its counters
          __hip_atomic_store(c.arr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_store(c.arr + 1, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
    } else {
      gather_item<D>(prm, pb, c, c.slice, parts);
    }
  }

  // retire: the last workgroup of the launch clears the ticket
  if (tid == 0) {
    if (add_u32(&sync[kSyncDone], 1u) == gridDim.x - 1u) {
      __hip_atomic_store(&sync[kSyncTicket], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(&sync[kSyncDone], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

namespace {

template <int D>
const void* step_ptr(int qbt) {
  switch (qbt) {
    case 2: return reinterpret_cast<const void*>(&step_bf16<D, 2>);
    case 4: return reinterpret_cast<const void*>(&step_bf16<D, 4>);
    case 6: return reinterpret_cast<const void*>(&step_bf16<D, 6>);
    case 8: return reinterpret_cast<const void*>(&step_bf16<D, 8>);
    default: return reinterpret_cast<const void*>(&step_bf16<D, 14>);
  }
}

template <int D>
void launch_step_d(int qbt, dim3 grid, size_t lds, hipStream_t s, const LaunchParams& p, int n1,
                   int parts) {
  const dim3 block(kThreads);
  switch (qbt) {
    case 2: hipLaunchKernelGGL((step_bf16<D, 2>), grid, block, lds, s, p, n1, parts); break;
    case 4: hipLaunchKernelGGL((step_bf16<D, 4>), grid, block, lds, s, p, n1, parts); break;
    case 6: hipLaunchKernelGGL((step_bf16<D, 6>), grid, block, lds, s, p, n1, parts); break;
    case 8: hipLaunchKernelGGL((step_bf16<D, 8>), grid, block, lds, s, p, n1, parts); break;
    default: hipLaunchKernelGGL((step_bf16<D, 14>), grid, block, lds, s, p, n1, parts); break;
  }
}

int step_qbt(int rpad_max) {
  const int qb = (rpad_max + 31) / 32;
  const int have[4] = {2, 4, 6, 8};
  for (int i = 0; i < 4; ++i)
    if (qb <= have[i]) return have[i];
  return 14;
}

}  // namespace

// Scoring (and, if parts > 0, selection and compaction in `parts` copy items per
// problem) of the whole batch in one
// launch.  Needs every problem's padded row count <= kStepMaxRows.
hipError_t launch_step_bf16(int head_dim, const LaunchParams& p, size_t lds, int parts,
                            hipStream_t s) {
  const int n1 = p.n_problems * p.tiles_max;
  if (n1 <= 0) return hipSuccess;
  const dim3 grid(2u * static_cast<unsigned>(n1) +
                  static_cast<unsigned>(p.n_problems) * static_cast<unsigned>(parts));
  const int qbt = step_qbt(p.rpad_max);
  if (head_dim == 128) {
    launch_step_d<128>(qbt, grid, lds, s, p, n1, parts);
  } else {
    launch_step_d<64>(qbt, grid, lds, s, p, n1, parts);
  }
  return hipGetLastError();
}

hipError_t set_max_lds_step(size_t bytes) {
  const int qbts[5] = {2, 4, 6, 8, 14};
  for (int i = 0; i < 5; ++i) {
    hipError_t e = hipFuncSetAttribute(step_ptr<128>(qbts[i]),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       static_cast<int>(bytes));
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(step_ptr<64>(qbts[i]), hipFuncAttributeMaxDynamicSharedMemorySize,
                            static_cast<int>(bytes));
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace finch
