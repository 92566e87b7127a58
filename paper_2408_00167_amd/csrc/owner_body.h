// One workgroup per problem for a whole prefill step, bf16 Q/K/V on gfx950: scoring
// pass 1, the merge of the row statistics, scoring pass 2, top-r and compaction
// (Method: attention of the prompt rows over cache + chunk keys, sum over heads and
// prompt rows, t = top-r(A_agg, r), Managing the Cache) run back to back inside the
// workgroup that owns the problem.
//
// Nothing is exchanged between workgroups, so there are no kernel boundaries, no
// atomics on device memory and no waits: the row statistics are merged in LDS, the
// scores a workgroup wrote are read back by itself (top-r), and so are the indices
// (compaction).  The keys are read a second time right after the first pass, while
// the memory-side cache still holds most of them.  Workgroups are 8 waves (two per
// SIMD, up to 256 registers each), one per CU; the batch should have about as many problems as the chip has CUs (or a
// multiple), which the host checks before it picks this path.
//
// The arithmetic (and therefore every output bit of scores given the same block
// assignment rules) follows the two-pass kernels: MFMA 32x32x16 bf16 with one
// prompt row per lane, log2-domain softmax, pass 1 with a fixed assignment of key
// blocks to waves, pass 2 with key blocks handed out by an LDS counter.
//
// Templates of the one-workgroup-per-problem kernels; instantiated by
// owner_bf16.hip (prompt rows only) and owner_doc_bf16.hip (rows of the chunk's own
// tokens as well).
#pragma once

#include "reposition_common.h"
#include "score_common.h"
#include "select_common.h"

namespace finch {

namespace {

// Phase timers, compiled in only with -DFINCH_PHASE_TIMERS (the build script's --phase-timers
// writes that variant to a library of its own; the normal library has none of this).  Thread 0
// of every workgroup adds the ticks of the 100 MHz wall clock it spent between two marks to
// the phase's total: 0 staging of the prompt rows, 1 pass 1 of wave 0, 2 wave 0's wait at the
// barrier after pass 1, 3 merge of the row statistics, 4 pass 2 of wave 0, 5 its wait at the
// barrier after pass 2, 6 top-r, 7 compaction.  Each translation unit has its own totals.
#ifdef FINCH_PHASE_TIMERS
static __device__ unsigned long long finch_phase_ticks[8];
#define FINCH_PHASE_BEGIN() unsigned long long phase_last_ = wall_clock64()
#define FINCH_PHASE(i)                                        \
  do {                                                        \
    if (threadIdx.x == 0) {                                   \
      const unsigned long long now_ = wall_clock64();         \
      atomicAdd(&finch_phase_ticks[i], now_ - phase_last_);   \
      phase_last_ = now_;                                     \
    }                                                         \
  } while (0)
#else
#define FINCH_PHASE_BEGIN() do { } while (0)
#define FINCH_PHASE(i) do { } while (0)
#endif

constexpr int kOwnThreads = 512;
constexpr int kOwnWaves = kOwnThreads / 64;

__device__ __forceinline__ int own_next_block(int* counter, int lane) {
  int v = 0;
  if (lane == 0) v = atomicAdd(counter, 1);
  return __builtin_amdgcn_readfirstlane(v);
}

// Copy rows idx[0..r) of [cache ; chunk] of K and V into k_out / v_out by NT threads
// (`tid` = index among them).  `lidx` (LDS) or `gidx` (memory, written by this
// workgroup) holds the indices; with `identity` row t is simply candidate t.
template <int SEGS, int NT = kOwnThreads>
__device__ __forceinline__ void own_gather(const finch_problem& pb, int N, int r, const int* lidx,
                                           const FINCH_GLOBAL int* gidx, bool identity, int tid) {
  const FINCH_GLOBAL u32x4* kc = as_global<u32x4>(pb.k_cache);
  const FINCH_GLOBAL u32x4* kk = as_global<u32x4>(pb.k_chunk);
  const FINCH_GLOBAL u32x4* vc = as_global<u32x4>(pb.v_cache);
  const FINCH_GLOBAL u32x4* vk = as_global<u32x4>(pb.v_chunk);
  FINCH_GLOBAL u32x4* ko = as_global_mut<u32x4>(pb.k_out);
  FINCH_GLOBAL u32x4* vo = as_global_mut<u32x4>(pb.v_out);
  constexpr int kRowsPerIter = NT / SEGS;
  constexpr int kUnroll = 8;
  const int seg = tid % SEGS, sub = tid / SEGS;
  for (int row0 = 0; row0 < r; row0 += kRowsPerIter * kUnroll) {
    u32x4 kv[kUnroll], vv[kUnroll];
#pragma unroll
    for (int it = 0; it < kUnroll; ++it) {
      const int t = min(row0 + it * kRowsPerIter + sub, r - 1);
      int j = identity ? t : (lidx ? lidx[t] : gidx[t]);
      j = min(max(j, 0), N - 1);
      const bool cached = j < pb.c;
      const size_t off = static_cast<size_t>(cached ? j : j - pb.c) * SEGS + seg;
      kv[it] = (cached ? kc : kk)[off];
      vv[it] = (cached ? vc : vk)[off];
    }
#pragma unroll
    for (int it = 0; it < kUnroll; ++it) {
      const int t = row0 + it * kRowsPerIter + sub;
      if (t < r) {
        ko[static_cast<size_t>(t) * SEGS + seg] = kv[it];
        vo[static_cast<size_t>(t) * SEGS + seg] = vv[it];
      }
    }
  }
}

// The same with the kept keys re-positioned: slot p takes kept row t = p (the ascending
// order), or, with `ranked` (LDS; see own_rank_kept), the kept row whose record stands
// at place p of the sorted records; the key is turned by p - idx[t] positions while it
// is copied (not at all with pairing FINCH_ROPE_OFF).  A thread owns two pieces of a
// row, d/2 channels apart, i.e. both partners of its channel pairs.
template <int SEGS, int NT = kOwnThreads, int E = 8>
__device__ __forceinline__ void own_gather_rot(const finch_problem& pb, int N, int r, const int* lidx,
                                               const FINCH_GLOBAL int* gidx, bool identity, int pairing,
                                               double log2_base, int tid,
                                               const unsigned long long* ranked = nullptr) {
  constexpr int kHalf = SEGS / 2;
  const FINCH_GLOBAL u32x4* kc = as_global<u32x4>(pb.k_cache);
  const FINCH_GLOBAL u32x4* kk = as_global<u32x4>(pb.k_chunk);
  const FINCH_GLOBAL u32x4* vc = as_global<u32x4>(pb.v_cache);
  const FINCH_GLOBAL u32x4* vk = as_global<u32x4>(pb.v_chunk);
  FINCH_GLOBAL u32x4* ko = as_global_mut<u32x4>(pb.k_out);
  FINCH_GLOBAL u32x4* vo = as_global_mut<u32x4>(pb.v_out);
  constexpr int kRowsPerIter = NT / kHalf;
  constexpr int kUnroll = 4;
  const int seg = tid % kHalf, sub = tid / kHalf;
  double th[E];
  pair_thetas<E, kHalf>(pairing, seg, log2_base, th);
  for (int row0 = 0; row0 < r; row0 += kRowsPerIter * kUnroll) {
    u32x4 ka[kUnroll], kb[kUnroll], va[kUnroll], vb[kUnroll];
    int shift[kUnroll], slot[kUnroll];
#pragma unroll
    for (int it = 0; it < kUnroll; ++it) {
      const int p = min(row0 + it * kRowsPerIter + sub, r - 1);
      const int t = ranked ? min(static_cast<int>(~static_cast<unsigned>(ranked[p])), r - 1) : p;
      int j = identity ? t : (lidx ? lidx[t] : gidx[t]);
      j = min(max(j, 0), N - 1);
      slot[it] = p;
      shift[it] = p - j;
      const bool cached = j < pb.c;
      const size_t off = static_cast<size_t>(cached ? j : j - pb.c) * SEGS + seg;
      ka[it] = (cached ? kc : kk)[off];
      kb[it] = (cached ? kc : kk)[off + kHalf];
      va[it] = (cached ? vc : vk)[off];
      vb[it] = (cached ? vc : vk)[off + kHalf];
    }
#pragma unroll
    for (int it = 0; it < kUnroll; ++it) {
      if (row0 + it * kRowsPerIter + sub < r) {
        if (pairing != FINCH_ROPE_OFF && shift[it] != 0) rotate_pieces<E>(pairing, th, shift[it], ka[it], kb[it]);
        const size_t o = static_cast<size_t>(slot[it]) * SEGS + seg;
        ko[o] = ka[it];
        ko[o + kHalf] = kb[it];
        vo[o] = va[it];
        vo[o + kHalf] = vb[it];
      }
    }
  }
}

}  // namespace

// Kept rows by relevance: one 64-bit record per kept row t < r - order key of its score
// in the upper half, ~t in the lower - sorted in descending order by a bitonic network
// over npad = max(64, next power of two) records (padding records are zero and end up
// last), so that place p holds the row with the p-th highest score, equal scores in index
// order.  `ranked` needs 8 * npad bytes of LDS.  Whole workgroup; ends with a barrier.
// A wave owns a part of max(64, npad / 8) consecutive records and keeps them in registers,
// record lane + 64 s of the part in slot s of the lane: partners less than 64 apart are
// exchanged by lane shuffles, partners 64 or 128 apart sit in the same lane, and only the
// stages whose partners lie in different parts go through LDS and workgroup barriers.
constexpr int kRankSlots = 4;  // records per lane: parts of at most 256 records = 2048 kept rows
__device__ __forceinline__ int own_rank_pad(int r) {
  int npad = 64;
  while (npad < r) npad <<= 1;
  return npad;
}
__device__ __forceinline__ void own_rank_kept(unsigned long long* ranked, int r, const FINCH_GLOBAL float* scores,
                                              const int* lidx, bool identity, int tid) {
  const int npad = own_rank_pad(r);
  const int lane = tid & 63, wave = tid >> 6;
  const int part = max(64, npad / kOwnWaves);
  const int slots = part >> 6;  // 1, 2 or 4
  const bool active = wave * part < npad;
  const int e0 = wave * part + lane;  // slot s holds record e0 + 64 s
  unsigned long long rec[kRankSlots];
#pragma unroll
  for (int sl = 0; sl < kRankSlots; ++sl) {
    rec[sl] = 0ull;
    const int u = e0 + 64 * sl;
    if (active && sl < slots && u < r)
      rec[sl] = (static_cast<unsigned long long>(order_key(scores[identity ? u : lidx[u]])) << 32) | static_cast<unsigned>(~u);
  }
  // the record that stays at position e after the exchange with position e ^ j in the stage (k, j)
  auto keep = [](unsigned long long mine, unsigned long long other, int e, int j, int k) {
    const bool want_max = ((e & k) == 0) == ((e & j) == 0);
    return want_max ? (mine > other ? mine : other) : (mine < other ? mine : other);
  };
  bool in_lds = false;  // the current order is in `ranked`, not in the registers
  for (int k = 2; k <= npad; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      if (j >= part) {
        if (!in_lds) {
#pragma unroll
          for (int sl = 0; sl < kRankSlots; ++sl)
            if (active && sl < slots) ranked[e0 + 64 * sl] = rec[sl];
        }
        __syncthreads();
        for (int q = tid; q < (npad >> 1); q += kOwnThreads) {
          const int i = ((q & ~(j - 1)) << 1) | (q & (j - 1));
          const unsigned long long a = ranked[i], b = ranked[i + j];
          if (((i & k) == 0) ? a < b : a > b) {
            ranked[i] = b;
            ranked[i + j] = a;
          }
        }
        in_lds = true;
        continue;
      }
      if (in_lds) {
        __syncthreads();
#pragma unroll
        for (int sl = 0; sl < kRankSlots; ++sl)
          if (active && sl < slots) rec[sl] = ranked[e0 + 64 * sl];
        in_lds = false;
      }
      if (j >= 64) {
        // partner in the same lane, j / 64 slots away (1 or 2)
        unsigned long long nxt[kRankSlots];
#pragma unroll
        for (int sl = 0; sl < kRankSlots; ++sl) {
          const unsigned long long other = (j == 64) ? rec[sl ^ 1] : rec[sl ^ 2];
          nxt[sl] = keep(rec[sl], other, e0 + 64 * sl, j, k);
        }
#pragma unroll
        for (int sl = 0; sl < kRankSlots; ++sl)
          if (sl < slots) rec[sl] = nxt[sl];
      } else {
#pragma unroll
        for (int sl = 0; sl < kRankSlots; ++sl) {
          const unsigned long long other = __shfl_xor(rec[sl], j);
          rec[sl] = keep(rec[sl], other, e0 + 64 * sl, j, k);
        }
      }
    }
  }
  if (in_lds) {
    __syncthreads();
  } else {
    // (nobody reads `ranked` before the barrier below, and the last stage that wrote it
    // was followed by a barrier and a reload)
#pragma unroll
    for (int sl = 0; sl < kRankSlots; ++sl)
      if (active && sl < slots) ranked[e0 + 64 * sl] = rec[sl];
    __syncthreads();
  }
}

// The rest of a step once this workgroup's scores are in memory (and a barrier has been
// passed since): top-r (Method: t = top-r(A_agg, r); with `layered` on the sum over the
// layer's heads) and compaction (Method: Managing the Cache) of rows of SEGS 16-byte
// pieces with E elements each.  `sel` is LDS scratch of sel_bytes (>= sizeof(SelLds) +
// kOwnerSelectBytes); `dst` the scores of this problem.
template <int SEGS, int E, bool ROT>
__device__ __forceinline__ void own_finish_step(const LaunchParams& prm, const finch_problem& pb, int slot, int N,
                                                FINCH_GLOBAL float* dst, char* sel, size_t sel_bytes,
                                                const finch_problem* step_probs, int epoch, bool layered,
                                                int* sync_words, int tid) {
  const int lane = tid & 63, wave = tid >> 6;
  const int L = prm.layer_group;
  FINCH_PHASE_BEGIN();
  // ---- top-r on the scores this workgroup has just written
  const int r = min(pb.r, N);
  if (r <= 0) return;
  FINCH_GLOBAL int* gidx = as_global_mut<int>(pb.idx);
  const bool identity = r >= N;
  SelLds* fl = reinterpret_cast<SelLds*>(sel);
  int* lidx = nullptr;
  if (identity) {
    for (int i = tid; i < N; i += kOwnThreads) gidx[i] = i;
  } else {
    size_t used = sizeof(SelLds);
    if (used + static_cast<size_t>(r) * 4 <= sel_bytes) {
      lidx = reinterpret_cast<int*>(sel + used);
      used += static_cast<size_t>(r) * 4;
    }
    if (layered) {
      // this workgroup's scores are out (stored past the caches, and every thread has waited
      // for its own stores at the barrier after pass 2); wait until all L workgroups of the
      // run say the same
      const int run = slot / L;
      if (tid == 0) {
        __hip_atomic_fetch_add(sync_words, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const long long t0 = wall_clock64();
        int gave_up = 0;
        while (__hip_atomic_load(sync_words, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < L * (epoch + 1)) {
          __builtin_amdgcn_s_sleep(8);
          if (wall_clock64() - t0 > prm.spin_ticks) {
            atomicOr(prm.layer_err, 1);
            gave_up = 1;
            break;
          }
        }
        fl->layer_gave_up = gave_up;
      }
      if (tid < L) {
        const finch_problem pg = step_probs[run * L + tid];
        fl->layer_src[tid] = pg.scores ? pg.scores
                                       : prm.ws_scores + static_cast<size_t>(run * L + tid) * prm.score_stride;
      }
      __syncthreads();
      if (fl->layer_gave_up) {
        // Scores that other workgroups are still writing must not be selected on (a
        // selection that reads them twice could count differently each time): this
        // workgroup leaves the step's indices and cache rows unwritten.  It still says
        // that it will not read the others' scores any more.
        if (tid == 0) __hip_atomic_fetch_add(sync_words + 1, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
      }
    }
    const LayerScores layer_sum = {fl->layer_src, L};
    const OneScoreVector own = {dst};
    if (N <= kOwnThreads * kSelRegKeys) {
      if (layered) select_regs<kOwnThreads>(layer_sum, N, r, gidx, lidx, fl, tid, lane, wave);
      else select_regs<kOwnThreads>(own, N, r, gidx, lidx, fl, tid, lane, wave);
    } else {
      unsigned* lkeys = nullptr;
      if (used + static_cast<size_t>(N) * 4 <= sel_bytes) {
        lkeys = reinterpret_cast<unsigned*>(sel + used);
        for (int i = tid; i < N; i += kOwnThreads) lkeys[i] = order_key(layered ? layer_sum(i) : own(i));
      }
      __syncthreads();
      if (layered) select_generic<kOwnThreads>(lkeys, layer_sum, N, r, gidx, lidx, fl, tid, lane, wave);
      else select_generic<kOwnThreads>(lkeys, own, N, r, gidx, lidx, fl, tid, lane, wave);
    }
    __syncthreads();  // idx (LDS and memory) complete
    // (the other workgroups' scores have been read for the last time)
    if (layered && tid == 0) __hip_atomic_fetch_add(sync_words + 1, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  FINCH_PHASE(6);

  // ---- compaction
  if (ROT) {
    // slots by relevance (Method: Managing the Cache, the worked example): the rank of a kept
    // row's score among the kept ones, highest first, equal scores by index.  The host
    // sends such batches here only if the indices and the records of all kept rows fit
    // behind the selection scratch.
    unsigned long long* ranked = nullptr;
    if (prm.rank_order) {
      __syncthreads();  // (the identity case has not been through a barrier since the scores)
      ranked = reinterpret_cast<unsigned long long*>(sel + sizeof(SelLds) + ((static_cast<size_t>(r) * 4 + 7) & ~size_t{7}));
      own_rank_kept(ranked, r, dst, lidx, identity, tid);
    }
    own_gather_rot<SEGS, kOwnThreads, E>(pb, N, r, lidx, gidx, identity, prm.rope_pairing, prm.rope_log2_base, tid, ranked);
  } else {
    own_gather<SEGS>(pb, N, r, lidx, gidx, identity, tid);
  }
  FINCH_PHASE(7);
}

// One step of one problem by the whole workgroup.  QBT = row blocks (of 32 prompt
// rows) per pass over the keys the code is compiled for; prm.row_chunk <= 32 * QBT.
// stages: 0 = scores only, 1 = scores, top-r and compaction.  `staged_q` names the
// prompt block whose rows are in LDS from the previous step of the same launch (or
// nullptr); inputs do not change during a launch, so the same pointer and row
// count mean the same rows and the copy is skipped.  Ends with every thread past
// its last access to LDS only after the next barrier: callers that go on to
// another step must put a barrier in between.
// With prm.layer_group = L > 1 the L workgroups of a run of slots (a layer's KV heads)
// select together (Method: "Sum over heads", then one top-r per layer): each publishes
// its scores, waits for the others (bounded: a wait that runs out sets the error word
// and the workgroup goes on with what it finds), adds the L vectors up in the same order
// and selects on the sum, so that all L arrive at the same indices on their own.
// `step_probs` are the descriptors of this step, `epoch` counts the exchanges this
// workgroup has been through in this launch; returns true if the step made one.
template <int D, int QBT, bool ROT, bool DOC>
__device__ __forceinline__ bool own_step_body(const LaunchParams& prm, const finch_problem& pb, int slot,
                                              int stages, char* smem, const void*& staged_q,
                                              int& staged_rows, const finch_problem* step_probs = nullptr,
                                              int epoch = 0) {
  const int N = pb.c + pb.m;
  if (N == 0) return false;
  FINCH_PHASE_BEGIN();
  const int Rp = (DOC && !pb.q) ? 0 : prm.group * pb.n_que;  // prompt rows
  // (the thread index goes through an empty asm: in the whole-loop kernel the compiler
  // would otherwise compute everything that depends only on it once for all steps and
  // keep it in registers through every phase)
  int tid_ = threadIdx.x;
  asm volatile("" : "+v"(tid_));
  const int tid = tid_, lane = tid & 63, wave = tid >> 6;
  const int t = lane & 31, h = lane >> 5;
  constexpr int kStride = D * 2 + 16;
  const int RC = prm.row_chunk;
  char* lds_q = smem;
  float2* wstats = reinterpret_cast<float2*>(smem + RC * kStride);                 // [waves][RC]
  float* lds_lse = reinterpret_cast<float*>(smem + RC * (kStride + kOwnWaves * 8));  // [RC]
  int* sh_next = reinterpret_cast<int*>(smem + RC * (kStride + kOwnWaves * 8 + 4));
  const KeySource ks = {static_cast<const char*>(pb.k_cache), static_cast<const char*>(pb.k_chunk), pb.c};
  const int nb = (N + 31) >> 5;
  const float sc = prm.scale_log2;
  float* gscores = pb.scores ? pb.scores : prm.ws_scores + static_cast<size_t>(slot) * prm.score_stride;
  FINCH_GLOBAL float* dst = as_global_mut<float>(gscores);
  const int L = prm.layer_group;
  const bool layered = stages && L > 1 && pb.r > 0 && pb.r < N;  // the same in every workgroup of the run
  int* const sync_words = (stages && L > 1) ? prm.layer_sync + 2 * (slot / L) : nullptr;
  if (sync_words && epoch > 0) {
    // nobody of the run may still be adding up the scores of the step before when this
    // step's scores start to overwrite them
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

  // Row chunks: the prompt rows first (they see every key, so they initialise all
  // scores), then, in DOC kernels, the rows of the chunk's own tokens, head by head
  // and from the last tokens to the first (the last ones see every key as well).
  const int n_pchunks = (Rp + RC - 1) / RC;
  const int dper = (DOC && pb.q_doc && pb.m > 0) ? (pb.m + RC - 1) / RC : 0;
  const int n_chunks = n_pchunks + prm.group * dper;
  for (int ch = 0; ch < n_chunks; ++ch) {
    // rows [row0, row0 + rows) of `qsrc` (R rows in all); row i of the chunk sees the
    // keys below lim0 + lim_step * i
    const void* qsrc = pb.q;
    int R = Rp, row0 = ch * RC, lim0 = N, lim_step = 0;
    if (DOC && ch >= n_pchunks) {
      const int dc = ch - n_pchunks;
      const int g = dc / dper;
      row0 = (dper - 1 - (dc - g * dper)) * RC;
      qsrc = static_cast<const char*>(pb.q_doc) + static_cast<size_t>(g) * pb.m * (D * 2);
      R = pb.m;
      lim0 = pb.c + row0 + 1;
      lim_step = 1;
    }
    const int rows = min(RC, round_up32(R - row0));
    const int QB = rows >> 5;
    const bool first_chunk = ch == 0;
    // key blocks any row of the chunk sees
    const int nbc = DOC ? (min(N, lim0 + lim_step * (min(row0 + rows, R) - 1 - row0)) + 31) >> 5 : nb;
    // smallest and largest limit of row block q, and this lane's own in it
    auto lim_lo = [&](int q) { return lim0 + lim_step * (q * 32); };
    auto lim_hi = [&](int q) { return lim0 + lim_step * (q * 32 + 31); };
    auto lim_mine = [&](int q) { return min(N, lim0 + lim_step * (q * 32 + t)); };
    bf16x8 ka[D / 16], kb[D / 16];
    int b = wave;
    if (b < nbc) load_k_block<D>(ks, N, b << 5, lane, ka);  // requested before Q is staged
    if (!(R <= RC && staged_q == qsrc && staged_rows == R)) {
      stage_q<D, kOwnThreads>(qsrc, R, row0, rows, lds_q, tid);
      __syncthreads();
    }
    staged_q = nullptr;
    FINCH_PHASE(0);

    // ---- pass 1: running (reference, sum exp2) per prompt row, fixed block assignment
    {
      float m_run[QBT], z_run[QBT];
#pragma unroll
      for (int q = 0; q < QBT; ++q) {
        m_run[q] = -kInf;
        z_run[q] = 0.f;
      }
      // The reference of a row only has to keep exp2 in range: it is taken from the
      // wave's first key block and moved (sum rescaled) only when a block's sum shows
      // that its logits lie far above it.
      // (bit q: row block q has been through at least one visible key block)
      unsigned seeded = 0;
      // statistics of one 32 x 32 logit block
      auto tile_stats = [&](f32x16 a, int q, int kbase) {
        if (kbase + 32 > (DOC ? min(N, lim_lo(q)) : N)) {  // keys this row does not see, or past the end
          const int lim = DOC ? lim_mine(q) : N;
#pragma unroll
          for (int v = 0; v < 16; ++v)
            if (kbase + acc_key(v, h) >= lim) a[v] = -kInf;
        }
        float z = 0.f;
        const bool was_seeded = (seeded >> q) & 1u;
        bool move = !was_seeded;
        if (was_seeded) {
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
          z_run[q] = (mn == -kInf) ? 0.f : z_run[q] * fast_exp2(m_run[q] - mn);
          m_run[q] = mn;
          const float mu = (mn == -kInf) ? 0.f : mn;
          z = 0.f;
#pragma unroll
          for (int v = 0; v < 16; ++v) z += fast_exp2(__builtin_fmaf(a[v], sc, -mu));
        }
        z_run[q] += z;
        seeded |= 1u << q;
      };
      // Row blocks go through in pairs, one pair behind: while the matrix pipe works
      // on the logits of pair i, the vector units take the exponentials of pair i - 1.
      // In DOC kernels a pair none of whose rows sees the key block is left out (the
      // limits grow with the row, and a wave's key blocks come in ascending order, so a
      // row block that is left out once stays out).
      auto process = [&](const bf16x8(&kf)[D / 16], int blk) {
        const int kbase = blk << 5;
        auto pair_visible = [&](int q) { return !DOC || kbase < lim_hi(q + 1 < QB ? q + 1 : q); };
        f32x16 acc[QBT];
#pragma unroll
        for (int q = 0; q < QBT + 2; q += 2) {
          if (q < QBT && q < QB && pair_visible(q)) {
            if (q + 1 < QB) {
              mfma_block_pair_lds<D>(kf, lds_q, q, lane, acc[q], acc[q + 1]);
            } else {
              bf16x8 qf0[D / 16];
              load_q_frags<D>(lds_q, q, lane, qf0);
              acc[q] = mfma_block<D>(kf, qf0);
            }
          }
          if (q >= 2 && q - 2 < QB && pair_visible(q - 2)) {
            tile_stats(acc[q - 2], q - 2, kbase);
            if (q - 1 < QB) tile_stats(acc[q - 1], q - 1, kbase);
          }
        }
      };
      if (b < nbc) {
        while (true) {
          if (b + kOwnWaves < nbc) load_k_block<D>(ks, N, (b + kOwnWaves) << 5, lane, kb);
          process(ka, b);
          b += kOwnWaves;
          if (b >= nbc) break;
          if (b + kOwnWaves < nbc) load_k_block<D>(ks, N, (b + kOwnWaves) << 5, lane, ka);
          process(kb, b);
          b += kOwnWaves;
          if (b >= nbc) break;
        }
      }
#pragma unroll
      for (int q = 0; q < QBT; ++q) {
        if (q < QB) {
          float m = m_run[q], z = z_run[q];
          const float m2 = __shfl_xor(m, 32);
          const float z2 = __shfl_xor(z, 32);
          merge_stats(m, z, m2, z2);
          if (h == 0) wstats[wave * RC + q * 32 + t] = make_float2(m, z);
        }
      }
    }

    FINCH_PHASE(1);
    // ---- pass 2 walks the keys from the end (what pass 1 read last is what the
    // caches most likely still hold); its first block is requested before the merge
    b = nbc - 1 - wave;
    if (b >= 0) load_k_block<D>(ks, N, b << 5, lane, ka);
    if (tid == 0) *sh_next = kOwnWaves;
    __syncthreads();
    FINCH_PHASE(2);
    for (int i = tid; i < rows; i += kOwnThreads) {
      float l = kInf;  // padding rows add exp2(-inf) = 0
      if (row0 + i < R) {
        float2 a = wstats[i];
#pragma unroll
        for (int w = 1; w < kOwnWaves; ++w) {
          const float2 c = wstats[w * RC + i];
          merge_stats(a.x, a.y, c.x, c.y);
        }
        l = a.x + fast_log2(a.y);
        if (lim_step == 0) {
          if (pb.lse_extra) l = widen_lse(l, as_global<float>(pb.lse_extra)[row0 + i]);
        } else {
          // normalisation step: the row's weights times (keys it sees) / (c + m)
          l -= fast_log2(static_cast<float>(lim0 + i) / static_cast<float>(N));
        }
      }
      lds_lse[i] = l;
    }
    __syncthreads();
    FINCH_PHASE(3);
    {
      auto process = [&](const bf16x8(&kf)[D / 16], int blk) {
        const int kbase = blk << 5;
        float u[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) u[v] = 0.f;
        auto tile_sums = [&](f32x16 a, int q) {
          const float L = lds_lse[q * 32 + t];
          if (DOC && kbase + 32 > lim_lo(q)) {  // keys this row does not see add nothing
            const int lim = lim_mine(q);
#pragma unroll
            for (int v = 0; v < 16; ++v)
              if (kbase + acc_key(v, h) >= lim) a[v] = -kInf;
          }
#pragma unroll
          for (int v = 0; v < 16; ++v) u[v] += fast_exp2(__builtin_fmaf(a[v], sc, -L));
        };
        auto pair_visible = [&](int q) { return !DOC || kbase < lim_hi(q + 1 < QB ? q + 1 : q); };
        // pairs of row blocks, the vector work one pair behind the matrix work
        f32x16 acc[QBT];
#pragma unroll
        for (int q = 0; q < QBT + 2; q += 2) {
          if (q < QBT && q < QB && pair_visible(q)) {
            if (q + 1 < QB) {
              mfma_block_pair_lds<D>(kf, lds_q, q, lane, acc[q], acc[q + 1]);
            } else {
              bf16x8 qf0[D / 16];
              load_q_frags<D>(lds_q, q, lane, qf0);
              acc[q] = mfma_block<D>(kf, qf0);
            }
          }
          if (q >= 2 && q - 2 < QB && pair_visible(q - 2)) {
            tile_sums(acc[q - 2], q - 2);
            if (q - 1 < QB) tile_sums(acc[q - 1], q - 1);
          }
        }
        const float tot = fold16_over32(u, t);
        const int key = kbase + acc_key(t >> 1, h);
        if ((t & 1) == 0 && key < N) {
          const float val = first_chunk ? tot : dst[key] + tot;
          // (scores other workgroups will read go out past this compute unit's caches)
          if (layered) __hip_atomic_store(gscores + key, val, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          else dst[key] = val;
        }
      };
      if (b >= 0) {
        while (true) {
          int bn = nbc - 1 - own_next_block(sh_next, lane);
          if (bn >= 0) load_k_block<D>(ks, N, bn << 5, lane, kb);
          process(ka, b);
          b = bn;
          if (b < 0) break;
          bn = nbc - 1 - own_next_block(sh_next, lane);
          if (bn >= 0) load_k_block<D>(ks, N, bn << 5, lane, ka);
          process(kb, b);
          b = bn;
          if (b < 0) break;
        }
      }
    }
    FINCH_PHASE(4);
    __syncthreads();  // scores of this row chunk are out; LDS may be restaged
    FINCH_PHASE(5);
  }
  // what the prompt-row region of LDS holds now (selection scratch lies behind it)
  staged_q = (n_chunks == 1) ? pb.q : nullptr;
  staged_rows = Rp;
  if (!stages) return false;

  // ---- top-r and compaction; selection scratch behind the staged prompt rows (the pass-1
  // statistics are dead)
  own_finish_step<D / 8, 8, ROT>(prm, pb, slot, N, dst, smem + RC * kStride,
                                 prm.lds_bytes - static_cast<size_t>(RC) * kStride, step_probs, epoch, layered,
                                 sync_words, tid);
  return layered;
}

// Which slot workgroup b of n takes.  Normally b itself.  With layer groups the L
// workgroups of a run exchange their scores, so runs are kept on one of the chip's eight
// dies (workgroups go to the dies in turn: b % 8) and the exchange stays in that die's L2:
// die x takes the slots [x * (n / 8) + min(x, n % 8), ...) in the order of its workgroups.
__device__ __forceinline__ int own_slot_of(int b, int n, int L) {
  if (L <= 1) return b;
  const int x = b & 7, j = b >> 3;
  return x * (n >> 3) + min(x, n & 7) + j;
}

// One launch = one step of every problem of a batch; workgroup b owns problem b.
// ROT: the compaction re-positions the kept keys (prm.rope_pairing, ascending slots).
template <int D, int QBT, bool ROT, bool DOC>
__global__ __launch_bounds__(kOwnThreads) void owner_step_bf16(LaunchParams prm, int stages) {
  extern __shared__ __align__(16) char smem[];
  const int p = own_slot_of(blockIdx.x, gridDim.x, stages ? prm.layer_group : 1);
  const finch_problem pb = prm.probs[p];
  const void* staged_q = nullptr;
  int staged_rows = 0;
  own_step_body<D, QBT, ROT, DOC>(prm, pb, p, stages, smem, staged_q, staged_rows, prm.probs, 0);
}

// One launch = the whole chunk loop (Method: Document Segmentation): workgroup b
// owns slot b and runs its steps one after the other; the descriptors of step s
// are prm.probs[step_first[s] + slot] for slot < step_first[s+1] - step_first[s].
// Slots do not depend on each other, so workgroups drift apart and the copy-bound
// and arithmetic-bound stages of different problems overlap.
template <int D, int QBT, bool ROT, bool DOC>
__global__ __launch_bounds__(kOwnThreads) void owner_loop_bf16(LaunchParams prm, const int* step_first,
                                                               int n_steps) {
  extern __shared__ __align__(16) char smem[];
  const int slot = own_slot_of(blockIdx.x, gridDim.x, prm.layer_group);
  const void* staged_q = nullptr;
  int staged_rows = 0;
  int epoch = 0;
  for (int s = 0; s < n_steps; ++s) {
    const int first = step_first[s];
    if (slot >= step_first[s + 1] - first) break;  // slots are filled from the front
    const finch_problem pb = prm.probs[first + slot];
    if (own_step_body<D, QBT, ROT, DOC>(prm, pb, slot, /*stages=*/1, smem, staged_q, staged_rows, prm.probs + first,
                                        epoch))
      ++epoch;
    // the rows this step wrote are the next step's cache: complete before it reads
    __syncthreads();
  }
}

namespace {

int own_qbt(int row_chunk) {
  const int qb = (row_chunk + 31) / 32;
  const int have[4] = {2, 4, 6, 8};
  for (int i = 0; i < 4; ++i)
    if (qb <= have[i]) return have[i];
  return 0;
}

// Calls f(kernel) for the instantiation that matches (head_dim, qbt, rot); `loop`
// picks the whole-loop kernel.  Returns false for a combination that is not built.
template <bool DOC, typename F>
bool with_step_kernel(int head_dim, int qbt, bool rot, F f) {
#define FINCH_OWN_CASE(DD, QQ)                                           \
  if (head_dim == DD && qbt == QQ) {                                     \
    if (rot) f(&owner_step_bf16<DD, QQ, true, DOC>);                     \
    else f(&owner_step_bf16<DD, QQ, false, DOC>);                        \
    return true;                                                         \
  }
  FINCH_OWN_CASE(128, 2) FINCH_OWN_CASE(128, 4) FINCH_OWN_CASE(128, 6) FINCH_OWN_CASE(128, 8)
  FINCH_OWN_CASE(64, 2) FINCH_OWN_CASE(64, 4) FINCH_OWN_CASE(64, 6) FINCH_OWN_CASE(64, 8)
#undef FINCH_OWN_CASE
  return false;
}
template <bool DOC, typename F>
bool with_loop_kernel(int head_dim, int qbt, bool rot, F f) {
#define FINCH_OWN_CASE(DD, QQ)                                           \
  if (head_dim == DD && qbt == QQ) {                                     \
    if (rot) f(&owner_loop_bf16<DD, QQ, true, DOC>);                     \
    else f(&owner_loop_bf16<DD, QQ, false, DOC>);                        \
    return true;                                                         \
  }
  FINCH_OWN_CASE(128, 2) FINCH_OWN_CASE(128, 4) FINCH_OWN_CASE(128, 6) FINCH_OWN_CASE(128, 8)
  FINCH_OWN_CASE(64, 2) FINCH_OWN_CASE(64, 4) FINCH_OWN_CASE(64, 6) FINCH_OWN_CASE(64, 8)
#undef FINCH_OWN_CASE
  return false;
}

// p.row_chunk and p.lds_bytes must describe this kernel's layout (owner_lds_bytes).
template <bool DOC>
hipError_t launch_owner_impl(int head_dim, const LaunchParams& p, int stages, hipStream_t s) {
  if (p.n_problems <= 0) return hipSuccess;
  const dim3 grid(static_cast<unsigned>(p.n_problems)), block(kOwnThreads);
  const bool ok = with_step_kernel<DOC>(head_dim, own_qbt(p.row_chunk), p.rope_pairing != FINCH_ROPE_OFF || p.rank_order,
                                        [&](auto kern) {
                                          hipLaunchKernelGGL(kern, grid, block, p.lds_bytes, s, p, stages);
                                        });
  return ok ? hipGetLastError() : hipErrorInvalidValue;
}

// The whole loop: n_slots workgroups; step_first is a DEVICE array of n_steps + 1
// offsets into p.probs.
template <bool DOC>
hipError_t launch_owner_loop_impl(int head_dim, const LaunchParams& p, const int* step_first, int n_steps,
                                  int n_slots, hipStream_t s) {
  if (n_slots <= 0 || n_steps <= 0) return hipSuccess;
  const dim3 grid(static_cast<unsigned>(n_slots)), block(kOwnThreads);
  const bool ok = with_loop_kernel<DOC>(head_dim, own_qbt(p.row_chunk), p.rope_pairing != FINCH_ROPE_OFF || p.rank_order,
                                        [&](auto kern) {
                                          hipLaunchKernelGGL(kern, grid, block, p.lds_bytes, s, p, step_first,
                                                             n_steps);
                                        });
  return ok ? hipGetLastError() : hipErrorInvalidValue;
}

template <bool DOC>
hipError_t set_max_lds_owner_impl(size_t bytes) {
  hipError_t err = hipSuccess;
  const int dims[2] = {128, 64}, qbts[4] = {2, 4, 6, 8};
  for (int d = 0; d < 2; ++d)
    for (int q = 0; q < 4; ++q)
      for (int rot = 0; rot < 2; ++rot) {
        auto set = [&](auto kern) {
          const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize,
                                                   static_cast<int>(bytes));
          if (e != hipSuccess) err = e;
        };
        with_step_kernel<DOC>(dims[d], qbts[q], rot != 0, set);
        with_loop_kernel<DOC>(dims[d], qbts[q], rot != 0, set);
      }
  return err;
}

}  // namespace

}  // namespace finch
