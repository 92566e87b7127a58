// Host driver behind the C ABI: argument checks, launch sizing, workspace layout,
// stream-ordered launches.  No allocation and no synchronisation after
// finch_create.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <algorithm>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "finch_internal.h"

struct finch_ctx {
  finch_config cfg;
  int device;
  size_t max_lds;   // largest dynamic LDS a workgroup may ask for
  int last_hip;     // hipError_t of the last failed HIP call
  int row_bytes;    // bytes of one K or V row
  // optional per-kernel timing (finch_profile): pairs of events around launches
  bool prof_on;
  int prof_used;
  hipEvent_t* prof_ev;   // 2 * kProfPairs events, or nullptr
  int* prof_kind;        // kernel class of each pair
  int n_cu;              // compute units of the device
  int step_path;         // FINCH_PATH_AUTO / _SEPARATE / _OWNER
  int slice_keys;        // target keys per workgroup slice of the bf16 scoring kernels
  finch_reposition repos;  // {OFF, ASCENDING}: plain copies
  int layer_group;         // > 1: runs of that many problems share one selection
  int64_t layer_wait_ticks;  // bound of a workgroup's wait for its layer, 100 MHz ticks
  void* static_scratch;    // this device's copy of the file-scope scratch array (finch_step_static)
  // finch_loop: fingerprint of the last descriptor set whose slots were found free of
  // overlaps (the check is repeated only when the descriptors change)
  uint64_t loop_checked_hash;
  bool loop_checked;
};

// Scratch of finch_step_static: the workspace of a step, held by the library itself so
// that the call neither takes a workspace nor allocates.  Every GPU the library runs on
// holds its own copy of the array, at its own address, until the process ends.
constexpr size_t kStaticScratchBytes = size_t{16} << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

using finch::LaunchParams;

enum Need : unsigned {
  kNeedQK = 1u,      // q, k_cache, k_chunk are read
  kNeedScoresOut = 2u,  // desc.scores must be non-NULL
  kNeedIdx = 4u,     // desc.idx is written or read
  kNeedGather = 8u,  // v_*, k_out, v_out are used
};

struct Plan {
  int32_t n_max = 0, rows_max = 0, rpad_max = 0, r_max = 0, tiles_max = 0, row_chunk = 32;
  int32_t score_stride = 0;
  bool own_ok = false;    // the batch can run with one workgroup per problem
  bool has_doc = false;   // some problem takes rows from the chunk's own tokens (q_doc)
  int32_t own_row_chunk = 32;
  size_t own_lds = 0;
  size_t lds_bytes = 0;
  size_t off_stats = 0, off_lse = 0, off_scores = 0, off_layer = 0, off_sync = 0, total = 0;
  int32_t sync_words = 0;  // counters of the layer runs (workspace word 0 is the status word)
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

inline bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
  if (!a || !b || na == 0 || nb == 0) return false;
  const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
  return a0 < b0 + nb && b0 < a0 + na;
}

size_t score_lds(const finch_ctx* ctx, int row_chunk) {
  const size_t d = static_cast<size_t>(ctx->cfg.head_dim);
  // per staged row: the row itself + one (max,sum) pair per wave (pass 1), which
  // also covers the 4-byte lse entry of pass 2; then 16 bytes for the key-block counter
  if (ctx->cfg.dtype == FINCH_BF16)
    return static_cast<size_t>(row_chunk) * (d * 2 + 16 + (finch::kStreamThreads / 64) * sizeof(float2)) + 16;
  return static_cast<size_t>(row_chunk) * (d * 4 + 4 * sizeof(float2));
}

// Sizes launches for the n descriptors of `hd`; the workspace is laid out for
// n_alloc problems (n itself unless the descriptors are several steps of n_alloc
// slots, which reuse their slot's part of the workspace).
finch_status make_plan(const finch_ctx* ctx, const finch_problem* hd, int32_t n_desc, Plan& pl,
                       int32_t n_alloc = -1) {
  const int32_t n = n_desc;
  if (n_alloc < 0) n_alloc = n_desc;
  const int G = ctx->cfg.group_size;
  int64_t n_max = 0, rows_max = 0, r_max = 0;
  for (int32_t i = 0; i < n; ++i) {
    const finch_problem& pb = hd[i];
    // prompt rows are optional when the chunk's own rows are given
    const bool prompt_rows = pb.q != nullptr || pb.q_doc == nullptr;
    if ((prompt_rows && pb.n_que < 1) || pb.n_que < 0 || pb.c < 0 || pb.m < 0 || pb.r < 0)
      return FINCH_ERR_INVALID_ARG;
    const int64_t N = static_cast<int64_t>(pb.c) + pb.m;
    int64_t R = prompt_rows ? static_cast<int64_t>(G) * pb.n_que : 0;
    if (N > (1 << 24) || R > (1 << 20)) return FINCH_ERR_CAPACITY;
    if (pb.q_doc) {
      // staged a chunk of at most kOwnerMaxRowChunk rows at a time
      pl.has_doc = true;
      const int64_t dr = pb.m < finch::kOwnerMaxRowChunk ? pb.m : finch::kOwnerMaxRowChunk;
      if (dr > R) R = dr;
    }
    if (N > n_max) n_max = N;
    if (R > rows_max) rows_max = R;
    const int64_t rr = pb.r < N ? pb.r : N;
    if (rr > r_max) r_max = rr;
  }
  pl.n_max = static_cast<int32_t>(n_max);
  pl.rows_max = static_cast<int32_t>(rows_max);
  pl.rpad_max = static_cast<int32_t>((rows_max + 31) / 32 * 32);
  pl.r_max = static_cast<int32_t>(r_max);
  pl.tiles_max = ctx->cfg.dtype == FINCH_BF16
                     ? finch::stream_slices(static_cast<int>(n_max), ctx->slice_keys)
                     : static_cast<int32_t>((n_max + finch::kTileKeys - 1) / finch::kTileKeys);
  if (n_max == 0) pl.tiles_max = 0;
  pl.score_stride = static_cast<int32_t>((n_max + 63) / 64 * 64);
  int rc = pl.rpad_max < finch::kMaxRowChunk ? pl.rpad_max : finch::kMaxRowChunk;
  if (rc < 32) rc = 32;
  while (rc > 32 && score_lds(ctx, rc) > ctx->max_lds) rc -= 32;
  if (score_lds(ctx, rc) > ctx->max_lds) return FINCH_ERR_UNSUPPORTED;
  pl.row_chunk = rc;
  pl.lds_bytes = score_lds(ctx, rc);
  // grids are 1-D: keep them below 2^31
  const int64_t pg = (static_cast<int64_t>(n) + 7) / 8 * 8;
  if (pg * (pl.tiles_max > 0 ? pl.tiles_max : 1) >= (int64_t{1} << 31)) return FINCH_ERR_CAPACITY;
  const int64_t gb = (static_cast<int64_t>(pl.r_max) + finch::kGatherRows - 1) / finch::kGatherRows;
  if (gb * n >= (int64_t{1} << 31)) return FINCH_ERR_CAPACITY;
  if (ctx->cfg.dtype == FINCH_BF16 && n_max > 0) {
    int orc = pl.rpad_max < finch::kOwnerMaxRowChunk ? pl.rpad_max : finch::kOwnerMaxRowChunk;
    while (orc > 32 && finch::owner_lds_bytes(ctx->cfg.head_dim, orc) > ctx->max_lds) orc -= 32;
    pl.own_row_chunk = orc;
    pl.own_lds = finch::owner_lds_bytes(ctx->cfg.head_dim, orc);
    pl.own_ok = pl.own_lds <= ctx->max_lds;
  }
  if (ctx->cfg.dtype == FINCH_F32 && n_max > 0) {
    pl.own_lds = finch::owner_f32_lds_bytes(ctx->cfg.head_dim);
    pl.own_ok = pl.own_lds <= ctx->max_lds;
  }
  size_t off = 256;  // the first word of the workspace is the status word of the launches (finch_workspace_status)
  pl.off_stats = off;
  const size_t na = static_cast<size_t>(n_alloc);
  off = align_up(off + na * pl.tiles_max * pl.rpad_max * sizeof(float2), 256);
  pl.off_lse = off;
  off = align_up(off + na * pl.rpad_max * sizeof(float), 256);
  pl.off_scores = off;
  off = align_up(off + na * pl.score_stride * sizeof(float), 256);
  pl.off_layer = off;
  if (ctx->layer_group > 1)
    off = align_up(off + (na / ctx->layer_group + 1) * pl.score_stride * sizeof(float), 256);
  pl.off_sync = off;
  if (ctx->layer_group > 1) {
    pl.sync_words = static_cast<int32_t>(2 * (na / ctx->layer_group + 1));
    off = align_up(off + static_cast<size_t>(pl.sync_words) * sizeof(int32_t), 256);
  }
  pl.total = off;
  return FINCH_OK;
}

finch_status validate(const finch_ctx* ctx, const finch_problem* hd, int32_t n, unsigned need) {
  const size_t rb = static_cast<size_t>(ctx->row_bytes);
  for (int32_t i = 0; i < n; ++i) {
    const finch_problem& pb = hd[i];
    const int64_t N = static_cast<int64_t>(pb.c) + pb.m;
    const int64_t rr = pb.r < N ? pb.r : N;
    if (need & kNeedQK) {
      if (N > 0) {
        if (!pb.q && !pb.q_doc) return FINCH_ERR_INVALID_ARG;
        if (pb.q && !aligned(pb.q, 16)) return FINCH_ERR_INVALID_ARG;
        if (pb.q_doc && !aligned(pb.q_doc, 16)) return FINCH_ERR_INVALID_ARG;
        if (pb.c > 0 && (!pb.k_cache || !aligned(pb.k_cache, 16))) return FINCH_ERR_INVALID_ARG;
        if (pb.m > 0 && (!pb.k_chunk || !aligned(pb.k_chunk, 16))) return FINCH_ERR_INVALID_ARG;
      }
    }
    if ((need & kNeedScoresOut) && N > 0) {
      if (!pb.scores) return FINCH_ERR_INVALID_ARG;
    }
    if (pb.scores && !aligned(pb.scores, 4)) return FINCH_ERR_INVALID_ARG;
    if (pb.lse_extra && !aligned(pb.lse_extra, 4)) return FINCH_ERR_INVALID_ARG;
    if ((need & kNeedIdx) && rr > 0) {
      if (!pb.idx || !aligned(pb.idx, 4)) return FINCH_ERR_INVALID_ARG;
    }
    if ((need & kNeedGather) && rr > 0) {
      if (!pb.k_out || !pb.v_out || !aligned(pb.k_out, 16) || !aligned(pb.v_out, 16))
        return FINCH_ERR_INVALID_ARG;
      if (pb.c > 0 && (!pb.k_cache || !pb.v_cache || !aligned(pb.k_cache, 16) ||
                       !aligned(pb.v_cache, 16)))
        return FINCH_ERR_INVALID_ARG;
      if (pb.m > 0 && (!pb.k_chunk || !pb.v_chunk || !aligned(pb.k_chunk, 16) ||
                       !aligned(pb.v_chunk, 16)))
        return FINCH_ERR_INVALID_ARG;
      const size_t ob = static_cast<size_t>(rr) * rb;
      const void* srcs[4] = {pb.k_cache, pb.v_cache, pb.k_chunk, pb.v_chunk};
      const size_t lens[4] = {static_cast<size_t>(pb.c) * rb, static_cast<size_t>(pb.c) * rb,
                              static_cast<size_t>(pb.m) * rb, static_cast<size_t>(pb.m) * rb};
      for (int s = 0; s < 4; ++s) {
        if (overlaps(pb.k_out, ob, srcs[s], lens[s]) || overlaps(pb.v_out, ob, srcs[s], lens[s]))
          return FINCH_ERR_INVALID_ARG;
      }
      if (overlaps(pb.k_out, ob, pb.v_out, ob)) return FINCH_ERR_INVALID_ARG;
    }
  }
  return FINCH_OK;
}

finch_status check_common(const finch_ctx* ctx, const finch_problem* hd, const finch_problem* dd,
                          int32_t n) {
  if (!ctx || n < 0) return FINCH_ERR_INVALID_ARG;
  if (n > 0 && (!hd || !dd)) return FINCH_ERR_INVALID_ARG;
  if (n > 0 && !aligned(dd, 8)) return FINCH_ERR_INVALID_ARG;
  return FINCH_OK;
}

finch_status check_workspace(const Plan& pl, const void* ws, size_t ws_bytes) {
  if (pl.total <= 256) return FINCH_OK;
  if (!ws || !aligned(ws, 256) || ws_bytes < pl.total) return FINCH_ERR_WORKSPACE;
  return FINCH_OK;
}

LaunchParams make_params(const finch_ctx* ctx, const finch_problem* dd, int32_t n, const Plan& pl,
                         void* ws) {
  LaunchParams p;
  std::memset(&p, 0, sizeof(p));
  p.probs = dd;
  p.n_problems = n;
  p.group = ctx->cfg.group_size;
  p.tiles_max = pl.tiles_max;
  p.tile_keys = ctx->cfg.dtype == FINCH_BF16 ? 0 : finch::kTileKeys;
  p.slice_keys = ctx->slice_keys;
  p.merge_in_pass2 = (ctx->cfg.dtype == FINCH_BF16 && pl.tiles_max <= 16) ? 1 : 0;
  p.rpad_max = pl.rpad_max;
  p.row_chunk = pl.row_chunk;
  p.score_stride = pl.score_stride;
  p.scale_log2 = static_cast<float>(1.4426950408889634 / std::sqrt(static_cast<double>(ctx->cfg.head_dim)));
  char* base = static_cast<char*>(ws);
  p.stats = reinterpret_cast<float2*>(base + pl.off_stats);
  p.lse = reinterpret_cast<float*>(base + pl.off_lse);
  p.ws_scores = reinterpret_cast<float*>(base + pl.off_scores);
  p.lds_bytes = static_cast<uint32_t>(pl.lds_bytes);
  p.rope_pairing = ctx->repos.pairing;
  p.rank_order = ctx->repos.order == FINCH_ORDER_RANK ? 1 : 0;
  p.rope_log2_base = std::log2(ctx->repos.base);
  p.layer_group = ctx->layer_group;
  p.layer_sync = base ? reinterpret_cast<int32_t*>(base + pl.off_sync) : nullptr;
  p.layer_err = reinterpret_cast<int32_t*>(base);
  p.spin_ticks = ctx->layer_wait_ticks;
  return p;
}

finch_status hip_fail(finch_ctx* ctx, hipError_t e) {
  ctx->last_hip = static_cast<int>(e);
  return FINCH_ERR_HIP;
}

// Device address of `scratch` on each GPU.  In host code the array's name only stands
// for the symbol; the address kernels can use comes from hipGetSymbolAddress, asked once
// per device with that device current.
constexpr int kMaxDevices = 64;
void* g_scratch_addr[kMaxDevices];
std::mutex g_scratch_mutex;

hipError_t static_scratch_address(int device, void** out) {
  *out = nullptr;
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_addr[device]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_addr[device] = p;
  }
  *out = g_scratch_addr[device];
  return hipSuccess;
}

constexpr int kProfPairs = 8192;

// Brackets one kernel launch with two events on the launch stream when profiling
// is on; does nothing otherwise.
struct ProfScope {
  finch_ctx* ctx;
  hipStream_t s;
  int slot;
  ProfScope(finch_ctx* c, int kind, hipStream_t st) : ctx(c), s(st), slot(-1) {
    if (c->prof_on && c->prof_used < kProfPairs) {
      slot = c->prof_used++;
      c->prof_kind[slot] = kind;
      (void)hipEventRecord(c->prof_ev[2 * slot], s);
    }
  }
  ~ProfScope() {
    if (slot >= 0) (void)hipEventRecord(ctx->prof_ev[2 * slot + 1], s);
  }
};

// One workgroup per problem pays when the problems fill the chip's CUs in whole
// rounds (one 16-wave workgroup per CU at a time): AUTO takes that path when the
// last round would be at least 85 % full.
bool repositioning(const finch_ctx* ctx) {
  return ctx->repos.pairing != FINCH_ROPE_OFF || ctx->repos.order != FINCH_ORDER_ASCENDING;
}

bool owner_wanted(const finch_ctx* ctx, const Plan& pl, int32_t n) {
  if (!pl.own_ok || n <= 0) return false;
  // slots by score rank: the workgroup sorts its kept rows in LDS (their indices and one
  // 64-bit record each, padded to a power of two of at least 64, behind the selection scratch), and a
  // layer's heads would have to share the slots
  if (ctx->repos.order == FINCH_ORDER_RANK) {
    size_t npad = 64;
    while (npad < static_cast<size_t>(pl.r_max)) npad <<= 1;
    if (static_cast<size_t>(pl.r_max) * 4 + 8 + npad * 8 > finch::kOwnerSelectBytes || ctx->layer_group > 1)
      return false;
  }
  // the workgroups of a layer wait for each other: all of them must be on the chip at once
  // (one workgroup per compute unit), and a run's score vectors are added up by every one of them
  if (ctx->layer_group > 1 &&
      (ctx->layer_group > finch::kOwnerMaxLayer || n > (ctx->n_cu > 0 ? ctx->n_cu : 256)))
    return false;
  if (ctx->step_path == FINCH_PATH_OWNER) return true;
  if (pl.has_doc) return ctx->step_path == FINCH_PATH_AUTO;  // the only kernels with those rows
  if (ctx->step_path != FINCH_PATH_AUTO) return false;
  // fp32 (vector ALU): one workgroup per problem saves launches while problems are small;
  // large ones are better spread over the chip by the kernels per stage
  if (ctx->cfg.dtype == FINCH_F32) return pl.n_max <= 4096 && pl.rows_max <= 64;
  const int64_t cu = ctx->n_cu > 0 ? ctx->n_cu : 256;
  const int64_t rounds = (n + cu - 1) / cu;
  return static_cast<int64_t>(n) * 100 >= rounds * cu * 85;
}

finch_status run_owner(finch_ctx* ctx, LaunchParams p, const Plan& pl, int stages, hipStream_t s) {
  p.row_chunk = pl.own_row_chunk;
  p.lds_bytes = static_cast<uint32_t>(pl.own_lds);
  hipError_t e;
  if (stages && ctx->layer_group > 1) {
    if ((e = finch::launch_zero_words(p.layer_sync, pl.sync_words, p.layer_err, s)) != hipSuccess) return hip_fail(ctx, e);
  }
  {
    ProfScope ps(ctx, FINCH_KERNEL_OWNER, s);
    if (ctx->cfg.dtype == FINCH_F32) e = finch::launch_owner_f32(ctx->cfg.head_dim, p, stages, s);
    else e = pl.has_doc ? finch::launch_owner_doc_bf16(ctx->cfg.head_dim, p, stages, s)
                        : finch::launch_owner_bf16(ctx->cfg.head_dim, p, stages, s);
  }
  return e == hipSuccess ? FINCH_OK : hip_fail(ctx, e);
}

finch_status run_score(finch_ctx* ctx, const LaunchParams& p, const Plan& pl, hipStream_t s) {
  if (p.n_problems == 0 || pl.tiles_max == 0) return FINCH_OK;
  hipError_t e = hipSuccess;
  const int d = ctx->cfg.head_dim;
  const bool bf16 = ctx->cfg.dtype == FINCH_BF16;
  if (owner_wanted(ctx, pl, p.n_problems)) return run_owner(ctx, p, pl, /*stages=*/0, s);
  if (ctx->step_path == FINCH_PATH_OWNER || pl.has_doc) return FINCH_ERR_UNSUPPORTED;
  {
    ProfScope ps(ctx, FINCH_KERNEL_ROWSTATS, s);
    e = bf16 ? finch::launch_rowstats_bf16(d, p, pl.lds_bytes, s)
             : finch::launch_rowstats_f32(d, p, pl.lds_bytes, s);
  }
  if (e != hipSuccess) return hip_fail(ctx, e);
  if (!p.merge_in_pass2) {
    ProfScope ps(ctx, FINCH_KERNEL_LSE, s);
    e = finch::launch_lse(p, s);
  }
  if (e != hipSuccess) return hip_fail(ctx, e);
  {
    ProfScope ps(ctx, FINCH_KERNEL_COLSUM, s);
    e = bf16 ? finch::launch_colsum_bf16(d, p, pl.lds_bytes, s)
             : finch::launch_colsum_f32(d, p, pl.lds_bytes, s);
  }
  if (e != hipSuccess) return hip_fail(ctx, e);
  return FINCH_OK;
}

// Layer groups: the batch must be whole runs of problems with the same c, m and r.
finch_status check_layer_runs(const finch_ctx* ctx, const finch_problem* hd, int32_t n) {
  const int L = ctx->layer_group;
  if (L <= 1) return FINCH_OK;
  if (n % L != 0) return FINCH_ERR_INVALID_ARG;
  for (int32_t i = 0; i < n; ++i) {
    const finch_problem& a = hd[i - i % L];
    if (hd[i].c != a.c || hd[i].m != a.m || hd[i].r != a.r) return FINCH_ERR_INVALID_ARG;
  }
  return FINCH_OK;
}

finch_status run_select(finch_ctx* ctx, const LaunchParams& p, const Plan& pl, void* ws, hipStream_t s) {
  hipError_t e;
  {
    ProfScope ps(ctx, FINCH_KERNEL_SELECT, s);
    e = ctx->layer_group > 1
            ? finch::launch_select_layer(p, ctx->layer_group,
                                         reinterpret_cast<float*>(static_cast<char*>(ws) + pl.off_layer), s)
            : finch::launch_select(p, s);
  }
  return e == hipSuccess ? FINCH_OK : hip_fail(ctx, e);
}

finch_status run_gather(finch_ctx* ctx, const LaunchParams& p, int r_max, hipStream_t s) {
  hipError_t e;
  const bool rank = ctx->repos.order == FINCH_ORDER_RANK;
  if (rank && r_max > finch::kRankMaxRows) return FINCH_ERR_CAPACITY;
  // rank-order slots come from each problem's own scores; a layer's heads must share slots
  if (rank && ctx->layer_group > 1) return FINCH_ERR_UNSUPPORTED;
  {
    ProfScope ps(ctx, FINCH_KERNEL_GATHER, s);
    e = repositioning(ctx)
            ? finch::launch_reposition(p, ctx->row_bytes, ctx->cfg.dtype == FINCH_BF16, r_max,
                                       ctx->repos.pairing, rank, ctx->repos.base, s)
            : finch::launch_gather(p, ctx->row_bytes, r_max, s);
  }
  return e == hipSuccess ? FINCH_OK : hip_fail(ctx, e);
}

// Checks the step table of finch_loop; *n_desc = descriptors in all steps, *n_slots =
// problems of step 0.
finch_status check_steps(const int32_t* first, int32_t n_steps, int32_t* n_desc, int32_t* n_slots) {
  if (n_steps < 0 || (n_steps > 0 && !first)) return FINCH_ERR_INVALID_ARG;
  *n_desc = 0;
  *n_slots = 0;
  if (n_steps == 0) return FINCH_OK;
  if (first[0] != 0) return FINCH_ERR_INVALID_ARG;
  int32_t prev = INT32_MAX;
  for (int32_t s = 0; s < n_steps; ++s) {
    const int64_t cnt = static_cast<int64_t>(first[s + 1]) - first[s];
    if (cnt < 0 || cnt > prev) return FINCH_ERR_INVALID_ARG;
    prev = static_cast<int32_t>(cnt);
  }
  *n_desc = first[n_steps];
  *n_slots = first[1] - first[0];
  return FINCH_OK;
}

// ---- finch_loop: slots must not touch each other's memory
struct Span {
  uintptr_t lo, hi;  // [lo, hi)
  int32_t slot;
};

void add_span(std::vector<Span>& v, const void* p, size_t bytes, int32_t slot) {
  if (!p || bytes == 0) return;
  const uintptr_t a = reinterpret_cast<uintptr_t>(p);
  v.push_back(Span{a, a + bytes, slot});
}

// Sorts by start and merges spans of one slot that touch or overlap (the ping-pong
// slabs of a chunk loop repeat every other step).
void merge_own(std::vector<Span>& v) {
  std::sort(v.begin(), v.end(), [](const Span& a, const Span& b) { return a.lo < b.lo; });
  size_t out = 0;
  for (size_t i = 0; i < v.size(); ++i) {
    if (out > 0 && v[i].lo <= v[out - 1].hi) {
      if (v[i].hi > v[out - 1].hi) v[out - 1].hi = v[i].hi;
    } else {
      v[out++] = v[i];
    }
  }
  v.resize(out);
}

uint64_t fingerprint(const void* data, size_t bytes, uint64_t seed) {
  const unsigned char* p = static_cast<const unsigned char*>(data);
  uint64_t h[4] = {seed ^ 0x9e3779b97f4a7c15ull, seed + 0xbf58476d1ce4e5b9ull, seed ^ 0x94d049bb133111ebull,
                   seed + 0x2545f4914f6cdd1dull};
  size_t i = 0;
  for (; i + 32 <= bytes; i += 32) {
    uint64_t w[4];
    std::memcpy(w, p + i, 32);
    for (int k = 0; k < 4; ++k) h[k] = (h[k] ^ w[k]) * 0xff51afd7ed558ccdull + (h[k] >> 29);
  }
  uint64_t tail = 0;
  if (i < bytes) std::memcpy(&tail, p + i, bytes - i < 8 ? bytes - i : 8);
  uint64_t r = tail ^ (static_cast<uint64_t>(bytes) << 1);
  for (int k = 0; k < 4; ++k) r = (r ^ h[k]) * 0xc4ceb9fe1a85ec53ull + (r >> 31);
  return r;
}

// The rule of finch_loop: a slot runs through its steps without regard to the other
// slots, so nothing a slot writes (k_out, v_out, scores, idx of any of its steps) may
// overlap what another slot writes or reads (q, q_doc, k_*, v_*, lse_extra, scores).
finch_status check_slot_overlaps(const finch_ctx* ctx, const finch_problem* hd, const int32_t* first,
                                 int32_t n_steps, int32_t n_slots) {
  if (n_slots <= 1) return FINCH_OK;
  const size_t rb = static_cast<size_t>(ctx->row_bytes);
  const int G = ctx->cfg.group_size;
  std::vector<Span> writes, reads, own_w, own_r;
  for (int32_t slot = 0; slot < n_slots; ++slot) {
    own_w.clear();
    own_r.clear();
    for (int32_t s = 0; s < n_steps; ++s) {
      if (slot >= first[s + 1] - first[s]) break;
      const finch_problem& pb = hd[first[s] + slot];
      const size_t N = static_cast<size_t>(pb.c) + static_cast<size_t>(pb.m);
      const size_t rr = static_cast<size_t>(pb.r) < N ? static_cast<size_t>(pb.r) : N;
      add_span(own_w, pb.k_out, rr * rb, slot);
      add_span(own_w, pb.v_out, rr * rb, slot);
      add_span(own_w, pb.scores, N * sizeof(float), slot);
      add_span(own_w, pb.idx, rr * sizeof(int32_t), slot);
      add_span(own_r, pb.q, static_cast<size_t>(G) * pb.n_que * rb, slot);
      add_span(own_r, pb.q_doc, static_cast<size_t>(G) * pb.m * rb, slot);
      add_span(own_r, pb.k_cache, static_cast<size_t>(pb.c) * rb, slot);
      add_span(own_r, pb.v_cache, static_cast<size_t>(pb.c) * rb, slot);
      add_span(own_r, pb.k_chunk, static_cast<size_t>(pb.m) * rb, slot);
      add_span(own_r, pb.v_chunk, static_cast<size_t>(pb.m) * rb, slot);
      add_span(own_r, pb.lse_extra, static_cast<size_t>(G) * pb.n_que * sizeof(float), slot);
    }
    merge_own(own_w);
    merge_own(own_r);
    writes.insert(writes.end(), own_w.begin(), own_w.end());
    reads.insert(reads.end(), own_r.begin(), own_r.end());
  }
  std::sort(writes.begin(), writes.end(), [](const Span& a, const Span& b) { return a.lo < b.lo; });
  // spans of one slot are disjoint now, so two neighbours that overlap belong to two slots;
  // `reach` carries the furthest end seen so far and the slot it belongs to
  uintptr_t reach = 0;
  for (size_t i = 0; i < writes.size(); ++i) {
    if (i > 0 && writes[i].lo < reach) return FINCH_ERR_INVALID_ARG;
    if (writes[i].hi > reach) reach = writes[i].hi;
  }
  // the write spans are disjoint and sorted: look each read span up
  for (const Span& r : reads) {
    auto it = std::upper_bound(writes.begin(), writes.end(), r.lo,
                               [](uintptr_t x, const Span& w) { return x < w.hi; });  // first span ending after r.lo
    for (; it != writes.end() && it->lo < r.hi; ++it)
      if (it->slot != r.slot) return FINCH_ERR_INVALID_ARG;
  }
  return FINCH_OK;
}

// One step with its launches sized by `pl` (finch_step and finch_step_static).
finch_status step_planned(finch_ctx* ctx, const finch_problem* host_desc, const finch_problem* dev_desc,
                          int32_t n, const Plan& pl, void* ws, size_t ws_bytes, void* stream) {
  finch_status st;
  if ((st = validate(ctx, host_desc, n, kNeedQK | kNeedIdx | kNeedGather)) != FINCH_OK) return st;
  if ((st = check_layer_runs(ctx, host_desc, n)) != FINCH_OK) return st;
  if ((st = check_workspace(pl, ws, ws_bytes)) != FINCH_OK) return st;
  if (n == 0) return FINCH_OK;
  const LaunchParams p = make_params(ctx, dev_desc, n, pl, ws);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (ctx->layer_group > 1) {  // the status word starts every such call at zero, whatever path it takes
    const hipError_t e = finch::launch_zero_words(nullptr, 0, p.layer_err, s);
    if (e != hipSuccess) return hip_fail(ctx, e);
  }
  if (pl.tiles_max > 0 && owner_wanted(ctx, pl, n)) return run_owner(ctx, p, pl, /*stages=*/1, s);
  if ((ctx->step_path == FINCH_PATH_OWNER || pl.has_doc) && pl.tiles_max > 0) return FINCH_ERR_UNSUPPORTED;
  if ((st = run_score(ctx, p, pl, s)) != FINCH_OK) return st;
  if (pl.r_max == 0) return FINCH_OK;
  if ((st = run_select(ctx, p, pl, ws, s)) != FINCH_OK) return st;
  return run_gather(ctx, p, pl.r_max, s);
}

}  // namespace

extern "C" {

finch_status finch_create(const finch_config* cfg, finch_ctx** out) {
  if (!cfg || !out) return FINCH_ERR_INVALID_ARG;
  *out = nullptr;
  if (cfg->reserved != 0) return FINCH_ERR_INVALID_ARG;
  if (cfg->dtype != FINCH_F32 && cfg->dtype != FINCH_BF16) return FINCH_ERR_UNSUPPORTED;
  if (cfg->head_dim != 64 && cfg->head_dim != 128) return FINCH_ERR_UNSUPPORTED;
  if (cfg->group_size < 1 || cfg->group_size > 64) return FINCH_ERR_UNSUPPORTED;
  finch_ctx* ctx = new (std::nothrow) finch_ctx;
  if (!ctx) return FINCH_ERR_INVALID_ARG;
  ctx->cfg = *cfg;
  ctx->last_hip = 0;
  ctx->device = -1;
  ctx->max_lds = 64 * 1024;
  ctx->row_bytes = cfg->head_dim * (cfg->dtype == FINCH_BF16 ? 2 : 4);
  ctx->prof_on = false;
  ctx->prof_used = 0;
  ctx->prof_ev = nullptr;
  ctx->prof_kind = nullptr;
  ctx->n_cu = 0;
  ctx->step_path = FINCH_PATH_AUTO;
  ctx->slice_keys = finch::kDefaultSliceKeys;
  ctx->layer_group = 1;
  ctx->layer_wait_ticks = 20 * 1000 * 1000;  // 0.2 s
  ctx->repos.pairing = FINCH_ROPE_OFF;
  ctx->repos.order = FINCH_ORDER_ASCENDING;
  ctx->repos.base = 10000.0;
  ctx->static_scratch = nullptr;
  ctx->loop_checked = false;
  ctx->loop_checked_hash = 0;
  hipError_t e = hipGetDevice(&ctx->device);
  if (e == hipSuccess) e = static_scratch_address(ctx->device, &ctx->static_scratch);
  if (e == hipSuccess) {
    int v = 0;
    e = hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, ctx->device);
    if (e == hipSuccess && v > 0) ctx->max_lds = static_cast<size_t>(v);
  }
  if (e == hipSuccess) {
    e = hipDeviceGetAttribute(&ctx->n_cu, hipDeviceAttributeMultiprocessorCount, ctx->device);
  }
  if (e == hipSuccess) {
    e = cfg->dtype == FINCH_BF16 ? finch::set_max_lds_bf16(ctx->max_lds)
                                 : finch::set_max_lds_f32(ctx->max_lds);
  }
  if (e == hipSuccess && cfg->dtype == FINCH_BF16) e = finch::set_max_lds_owner(ctx->max_lds);
  if (e == hipSuccess && cfg->dtype == FINCH_BF16) e = finch::set_max_lds_owner_doc(ctx->max_lds);
  if (e == hipSuccess && cfg->dtype == FINCH_F32) e = finch::set_max_lds_owner_f32(ctx->max_lds);
  // the re-positioning kernel also has a little static LDS
  if (e == hipSuccess) e = finch::set_max_lds_reposition(ctx->max_lds - 1024);
  if (e != hipSuccess) {
    // No usable GPU: there is no fallback path.  Report and hand nothing out.
    std::fprintf(stderr, "finch_create: HIP error %d (%s)\n", static_cast<int>(e),
                 hipGetErrorString(e));
    (void)hipGetLastError();
    delete ctx;
    return FINCH_ERR_HIP;
  }
  *out = ctx;
  return FINCH_OK;
}

finch_status finch_destroy(finch_ctx* ctx) {
  if (ctx) (void)finch_profile(ctx, 0);
  delete ctx;
  return FINCH_OK;
}

finch_status finch_set_option(finch_ctx* ctx, int32_t option, int64_t value) {
  if (!ctx) return FINCH_ERR_INVALID_ARG;
  switch (option) {
    case FINCH_OPT_STEP_PATH:
      if (value != FINCH_PATH_AUTO && value != FINCH_PATH_SEPARATE && value != FINCH_PATH_OWNER)
        return FINCH_ERR_INVALID_ARG;
      ctx->step_path = static_cast<int>(value);
      return FINCH_OK;
    case FINCH_OPT_LAYER_GROUP:
      if (value < 1 || value > 4096) return FINCH_ERR_INVALID_ARG;
      ctx->layer_group = static_cast<int>(value);
      return FINCH_OK;
    case FINCH_OPT_LAYER_WAIT_TICKS:
      if (value < 0 || value > 1000000000) return FINCH_ERR_INVALID_ARG;
      ctx->layer_wait_ticks = value;
      return FINCH_OK;
    case FINCH_OPT_SLICE_KEYS:
      if (value < 256 || value > (1 << 24)) return FINCH_ERR_INVALID_ARG;
      ctx->slice_keys = static_cast<int>(value);
      return FINCH_OK;
    default:
      return FINCH_ERR_INVALID_ARG;
  }
}

finch_status finch_set_reposition(finch_ctx* ctx, const finch_reposition* how) {
  if (!ctx) return FINCH_ERR_INVALID_ARG;
  finch_reposition v = {FINCH_ROPE_OFF, FINCH_ORDER_ASCENDING, 10000.0};
  if (how) v = *how;
  if (v.pairing != FINCH_ROPE_OFF && v.pairing != FINCH_ROPE_HALF && v.pairing != FINCH_ROPE_INTERLEAVED)
    return FINCH_ERR_INVALID_ARG;
  if (v.order != FINCH_ORDER_ASCENDING && v.order != FINCH_ORDER_RANK) return FINCH_ERR_INVALID_ARG;
  if (v.pairing != FINCH_ROPE_OFF && !(v.base > 1.0 && v.base < 1e30)) return FINCH_ERR_INVALID_ARG;
  if (static_cast<size_t>(finch::kRankMaxRows) * 4 + 1024 > ctx->max_lds && v.order == FINCH_ORDER_RANK)
    return FINCH_ERR_UNSUPPORTED;
  ctx->repos = v;
  return FINCH_OK;
}

finch_status finch_profile(finch_ctx* ctx, int32_t enable) {
  if (!ctx) return FINCH_ERR_INVALID_ARG;
  if (enable && !ctx->prof_ev) {
    ctx->prof_ev = new (std::nothrow) hipEvent_t[2 * kProfPairs];
    ctx->prof_kind = new (std::nothrow) int[kProfPairs];
    if (!ctx->prof_ev || !ctx->prof_kind) return FINCH_ERR_INVALID_ARG;
    for (int i = 0; i < 2 * kProfPairs; ++i) {
      const hipError_t e = hipEventCreate(&ctx->prof_ev[i]);
      if (e != hipSuccess) return hip_fail(ctx, e);
    }
    ctx->prof_used = 0;
  }
  if (!enable && ctx->prof_ev) {
    for (int i = 0; i < 2 * kProfPairs; ++i) (void)hipEventDestroy(ctx->prof_ev[i]);
    delete[] ctx->prof_ev;
    delete[] ctx->prof_kind;
    ctx->prof_ev = nullptr;
    ctx->prof_kind = nullptr;
    ctx->prof_used = 0;
  }
  ctx->prof_on = enable != 0;
  return FINCH_OK;
}

finch_status finch_profile_read(finch_ctx* ctx, float* ms, int32_t* launches) {
  if (!ctx || !ms || !launches) return FINCH_ERR_INVALID_ARG;
  for (int k = 0; k < FINCH_KERNEL_COUNT; ++k) {
    ms[k] = 0.f;
    launches[k] = 0;
  }
  if (!ctx->prof_ev) return FINCH_OK;
  for (int i = 0; i < ctx->prof_used; ++i) {
    hipError_t e = hipEventSynchronize(ctx->prof_ev[2 * i + 1]);
    if (e != hipSuccess) return hip_fail(ctx, e);
    float t = 0.f;
    e = hipEventElapsedTime(&t, ctx->prof_ev[2 * i], ctx->prof_ev[2 * i + 1]);
    if (e != hipSuccess) return hip_fail(ctx, e);
    ms[ctx->prof_kind[i]] += t;
    launches[ctx->prof_kind[i]] += 1;
  }
  ctx->prof_used = 0;
  return FINCH_OK;
}

finch_status finch_workspace_size(const finch_ctx* ctx, const finch_problem* host_desc,
                                  int32_t n_problems, size_t* bytes) {
  if (!ctx || !bytes || n_problems < 0 || (n_problems > 0 && !host_desc))
    return FINCH_ERR_INVALID_ARG;
  Plan pl;
  const finch_status st = make_plan(ctx, host_desc, n_problems, pl);
  if (st != FINCH_OK) return st;
  *bytes = pl.total;
  return FINCH_OK;
}

finch_status finch_score(finch_ctx* ctx, const finch_problem* host_desc,
                         const finch_problem* dev_desc, int32_t n, void* ws, size_t ws_bytes,
                         void* stream) {
  finch_status st = check_common(ctx, host_desc, dev_desc, n);
  if (st != FINCH_OK) return st;
  Plan pl;
  if ((st = make_plan(ctx, host_desc, n, pl)) != FINCH_OK) return st;
  if ((st = validate(ctx, host_desc, n, kNeedQK | kNeedScoresOut)) != FINCH_OK) return st;
  if ((st = check_workspace(pl, ws, ws_bytes)) != FINCH_OK) return st;
  const LaunchParams p = make_params(ctx, dev_desc, n, pl, ws);
  return run_score(ctx, p, pl, static_cast<hipStream_t>(stream));
}

finch_status finch_prompt_lse(finch_ctx* ctx, const finch_problem* host_desc,
                              const finch_problem* dev_desc, int32_t n, void* stream) {
  finch_status st = check_common(ctx, host_desc, dev_desc, n);
  if (st != FINCH_OK) return st;
  Plan pl;
  if ((st = make_plan(ctx, host_desc, n, pl)) != FINCH_OK) return st;
  for (int32_t i = 0; i < n; ++i) {
    const finch_problem& pb = host_desc[i];
    if (!pb.q || !aligned(pb.q, 16) || !pb.k_que || !aligned(pb.k_que, 16) || !pb.lse_extra ||
        !aligned(pb.lse_extra, 4))
      return FINCH_ERR_INVALID_ARG;
  }
  if (n == 0) return FINCH_OK;
  if (static_cast<int64_t>(n) * ((pl.rows_max + 63) / 64) >= (int64_t{1} << 31)) return FINCH_ERR_CAPACITY;
  const LaunchParams p = make_params(ctx, dev_desc, n, pl, nullptr);
  hipError_t e;
  {
    ProfScope ps(ctx, FINCH_KERNEL_PROMPT_LSE, static_cast<hipStream_t>(stream));
    e = finch::launch_prompt_lse(p, ctx->cfg.head_dim, ctx->cfg.dtype == FINCH_BF16, pl.rows_max,
                                 static_cast<hipStream_t>(stream));
  }
  return e == hipSuccess ? FINCH_OK : hip_fail(ctx, e);
}

finch_status finch_topk(finch_ctx* ctx, const finch_problem* host_desc,
                        const finch_problem* dev_desc, int32_t n, void* ws, size_t ws_bytes,
                        void* stream) {
  finch_status st = check_common(ctx, host_desc, dev_desc, n);
  if (st != FINCH_OK) return st;
  Plan pl;
  if ((st = make_plan(ctx, host_desc, n, pl)) != FINCH_OK) return st;
  if ((st = validate(ctx, host_desc, n, kNeedScoresOut | kNeedIdx)) != FINCH_OK) return st;
  if ((st = check_layer_runs(ctx, host_desc, n)) != FINCH_OK) return st;
  if ((st = check_workspace(pl, ws, ws_bytes)) != FINCH_OK) return st;
  if (n == 0 || pl.r_max == 0) return FINCH_OK;
  const LaunchParams p = make_params(ctx, dev_desc, n, pl, ws);
  return run_select(ctx, p, pl, ws, static_cast<hipStream_t>(stream));
}

finch_status finch_compact(finch_ctx* ctx, const finch_problem* host_desc,
                           const finch_problem* dev_desc, int32_t n, void* ws, size_t ws_bytes,
                           void* stream) {
  finch_status st = check_common(ctx, host_desc, dev_desc, n);
  if (st != FINCH_OK) return st;
  Plan pl;
  if ((st = make_plan(ctx, host_desc, n, pl)) != FINCH_OK) return st;
  const unsigned need_scores = ctx->repos.order == FINCH_ORDER_RANK ? kNeedScoresOut : 0u;
  if ((st = validate(ctx, host_desc, n, kNeedIdx | kNeedGather | need_scores)) != FINCH_OK) return st;
  if ((st = check_workspace(pl, ws, ws_bytes)) != FINCH_OK) return st;
  if (n == 0 || pl.r_max == 0) return FINCH_OK;
  const LaunchParams p = make_params(ctx, dev_desc, n, pl, ws);
  return run_gather(ctx, p, pl.r_max, static_cast<hipStream_t>(stream));
}

finch_status finch_step(finch_ctx* ctx, const finch_problem* host_desc,
                        const finch_problem* dev_desc, int32_t n, void* ws, size_t ws_bytes,
                        void* stream) {
  finch_status st = check_common(ctx, host_desc, dev_desc, n);
  if (st != FINCH_OK) return st;
  Plan pl;
  if ((st = make_plan(ctx, host_desc, n, pl)) != FINCH_OK) return st;
  return step_planned(ctx, host_desc, dev_desc, n, pl, ws, ws_bytes, stream);
}

finch_status finch_step_static(finch_ctx* ctx, const finch_problem* host_desc,
                               const finch_problem* dev_desc, int32_t n, void* stream) {
  finch_status st = check_common(ctx, host_desc, dev_desc, n);
  if (st != FINCH_OK) return st;
  Plan pl;
  if ((st = make_plan(ctx, host_desc, n, pl)) != FINCH_OK) return st;
  if (pl.total > kStaticScratchBytes) {
    std::fprintf(stderr,
                 "finch_step_static: this batch needs %zu bytes of scratch, the library holds %zu; "
                 "use finch_step with a workspace\n",
                 pl.total, kStaticScratchBytes);
    return FINCH_ERR_CAPACITY;
  }
  if (!ctx->static_scratch) return FINCH_ERR_WORKSPACE;
  // No part of the scratch has to start at zero: each region (row statistics, row
  // log-sum-exps, scores, layer sums) is written by the step before it is read.
  return step_planned(ctx, host_desc, dev_desc, n, pl, ctx->static_scratch, kStaticScratchBytes, stream);
}

size_t finch_static_scratch_bytes(void) { return kStaticScratchBytes; }

finch_status finch_loop_workspace_size(const finch_ctx* ctx, const finch_problem* host_desc,
                                       const int32_t* host_step_first, int32_t n_steps, size_t* bytes) {
  if (!ctx || !bytes) return FINCH_ERR_INVALID_ARG;
  int32_t n_desc, n_slots;
  finch_status st = check_steps(host_step_first, n_steps, &n_desc, &n_slots);
  if (st != FINCH_OK) return st;
  if (n_desc > 0 && !host_desc) return FINCH_ERR_INVALID_ARG;
  Plan pl;
  if ((st = make_plan(ctx, host_desc, n_desc, pl, n_slots)) != FINCH_OK) return st;
  *bytes = pl.total;
  return FINCH_OK;
}

finch_status finch_loop(finch_ctx* ctx, const finch_problem* host_desc, const finch_problem* dev_desc,
                        const int32_t* host_step_first, const int32_t* dev_step_first, int32_t n_steps,
                        void* ws, size_t ws_bytes, void* stream) {
  if (!ctx) return FINCH_ERR_INVALID_ARG;
  int32_t n_desc, n_slots;
  finch_status st = check_steps(host_step_first, n_steps, &n_desc, &n_slots);
  if (st != FINCH_OK) return st;
  if ((st = check_common(ctx, host_desc, dev_desc, n_desc)) != FINCH_OK) return st;
  if (n_steps > 0 && (!dev_step_first || !aligned(dev_step_first, 4))) return FINCH_ERR_INVALID_ARG;
  Plan pl;
  if ((st = make_plan(ctx, host_desc, n_desc, pl, n_slots)) != FINCH_OK) return st;
  if ((st = validate(ctx, host_desc, n_desc, kNeedQK | kNeedIdx | kNeedGather)) != FINCH_OK) return st;
  for (int32_t i = 0; i < n_steps && ctx->layer_group > 1; ++i) {
    const int32_t f = host_step_first[i];
    if ((st = check_layer_runs(ctx, host_desc + f, host_step_first[i + 1] - f)) != FINCH_OK) return st;
  }
  {
    // overlaps between slots: checked once per descriptor set
    uint64_t h = fingerprint(host_desc, static_cast<size_t>(n_desc) * sizeof(finch_problem), 1);
    h = fingerprint(host_step_first, static_cast<size_t>(n_steps + 1) * sizeof(int32_t), h);
    if (!ctx->loop_checked || ctx->loop_checked_hash != h) {
      if ((st = check_slot_overlaps(ctx, host_desc, host_step_first, n_steps, n_slots)) != FINCH_OK) return st;
      ctx->loop_checked = true;
      ctx->loop_checked_hash = h;
    }
  }
  if ((st = check_workspace(pl, ws, ws_bytes)) != FINCH_OK) return st;
  if (n_desc == 0 || pl.tiles_max == 0) return FINCH_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (ctx->layer_group > 1) {
    const hipError_t e = finch::launch_zero_words(nullptr, 0, static_cast<int32_t*>(ws), s);
    if (e != hipSuccess) return hip_fail(ctx, e);
  }
  if (owner_wanted(ctx, pl, n_slots)) {
    LaunchParams p = make_params(ctx, dev_desc, n_desc, pl, ws);
    p.row_chunk = pl.own_row_chunk;
    p.lds_bytes = static_cast<uint32_t>(pl.own_lds);
    hipError_t e;
    if (ctx->layer_group > 1) {
      if ((e = finch::launch_zero_words(p.layer_sync, pl.sync_words, p.layer_err, s)) != hipSuccess) return hip_fail(ctx, e);
    }
    {
      ProfScope ps(ctx, FINCH_KERNEL_OWNER, s);
      if (ctx->cfg.dtype == FINCH_F32)
        e = finch::launch_owner_loop_f32(ctx->cfg.head_dim, p, dev_step_first, n_steps, n_slots, s);
      else
        e = pl.has_doc
                ? finch::launch_owner_loop_doc_bf16(ctx->cfg.head_dim, p, dev_step_first, n_steps, n_slots, s)
                : finch::launch_owner_loop_bf16(ctx->cfg.head_dim, p, dev_step_first, n_steps, n_slots, s);
    }
    return e == hipSuccess ? FINCH_OK : hip_fail(ctx, e);
  }
  if (ctx->step_path == FINCH_PATH_OWNER || pl.has_doc) return FINCH_ERR_UNSUPPORTED;
  // one finch_step per step; a step's plan never needs more workspace than the loop's
  for (int32_t i = 0; i < n_steps; ++i) {
    const int32_t f = host_step_first[i], cnt = host_step_first[i + 1] - f;
    if ((st = finch_step(ctx, host_desc + f, dev_desc + f, cnt, ws, ws_bytes, stream)) != FINCH_OK)
      return st;
  }
  return FINCH_OK;
}

finch_status finch_workspace_status(finch_ctx* ctx, const void* workspace, void* stream, int32_t* flags) {
  if (!ctx || !workspace || !flags) return FINCH_ERR_INVALID_ARG;
  *flags = 0;
  if (ctx->layer_group <= 1) return FINCH_OK;  // nothing sets the word then (and nothing has cleared it)
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = hipMemcpyAsync(flags, workspace, sizeof(int32_t), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return hip_fail(ctx, e);
  return *flags == 0 ? FINCH_OK : FINCH_ERR_TIMEOUT;
}

finch_status finch_loop_check(const finch_config* cfg, const finch_problem* host_desc,
                              const int32_t* host_step_first, int32_t n_steps) {
  if (!cfg) return FINCH_ERR_INVALID_ARG;
  if (cfg->dtype != FINCH_F32 && cfg->dtype != FINCH_BF16) return FINCH_ERR_UNSUPPORTED;
  if (cfg->head_dim != 64 && cfg->head_dim != 128) return FINCH_ERR_UNSUPPORTED;
  if (cfg->group_size < 1 || cfg->group_size > 64) return FINCH_ERR_UNSUPPORTED;
  int32_t n_desc, n_slots;
  finch_status st = check_steps(host_step_first, n_steps, &n_desc, &n_slots);
  if (st != FINCH_OK) return st;
  if (n_desc > 0 && !host_desc) return FINCH_ERR_INVALID_ARG;
  // a context on the stack that only carries the settings the checks read (no GPU is touched)
  finch_ctx tmp;
  std::memset(&tmp, 0, sizeof(tmp));
  tmp.cfg = *cfg;
  tmp.row_bytes = cfg->head_dim * (cfg->dtype == FINCH_BF16 ? 2 : 4);
  tmp.layer_group = 1;
  for (int32_t i = 0; i < n_desc; ++i) {
    const finch_problem& pb = host_desc[i];
    if (pb.n_que < 0 || pb.c < 0 || pb.m < 0 || pb.r < 0) return FINCH_ERR_INVALID_ARG;
    if (static_cast<int64_t>(pb.c) + pb.m > (1 << 24)) return FINCH_ERR_CAPACITY;
  }
  if ((st = validate(&tmp, host_desc, n_desc, kNeedQK | kNeedIdx | kNeedGather)) != FINCH_OK) return st;
  return check_slot_overlaps(&tmp, host_desc, host_step_first, n_steps, n_slots);
}

finch_status finch_schedule(int64_t n_cont, int32_t m, int64_t k, int32_t* r_out, int32_t r_len) {
  return finch_schedule_mode(n_cont, m, k, FINCH_SCHEDULE_PROPORTIONAL, r_out, r_len);
}

finch_status finch_schedule_mode(int64_t n_cont, int32_t m, int64_t k, int32_t mode, int32_t* r_out,
                                 int32_t r_len) {
  if (mode != FINCH_SCHEDULE_PROPORTIONAL && mode != FINCH_SCHEDULE_CONSTANT) return FINCH_ERR_INVALID_ARG;
  if (n_cont < 0 || m < 1 || k < 0 || r_len < 0) return FINCH_ERR_INVALID_ARG;
  if (n_cont > (int64_t{1} << 40)) return FINCH_ERR_CAPACITY;
  const int64_t steps = (n_cont + m - 1) / m;
  if (steps > r_len) return FINCH_ERR_CAPACITY;
  if (steps > 0 && !r_out) return FINCH_ERR_INVALID_ARG;
  const int64_t budget = k < n_cont ? k : n_cont;
  int64_t kept = 0, seen = 0;
  for (int64_t i = 0; i < steps; ++i) {
    const int64_t mi = (n_cont - seen) < m ? (n_cont - seen) : m;
    seen += mi;
    // floor(budget * seen / n_cont) without overflow: both factors are < 2^41
    const __int128 prod = static_cast<__int128>(budget) * seen;
    int64_t r = mode == FINCH_SCHEDULE_CONSTANT ? budget : static_cast<int64_t>(prod / n_cont);
    if (r > kept + mi) r = kept + mi;
    if (r > INT32_MAX) return FINCH_ERR_CAPACITY;
    r_out[i] = static_cast<int32_t>(r);
    kept = r;
  }
  return FINCH_OK;
}

int32_t finch_last_hip_error(const finch_ctx* ctx) { return ctx ? ctx->last_hip : 0; }

const char* finch_status_string(finch_status s) {
  switch (s) {
    case FINCH_OK: return "ok";
    case FINCH_ERR_INVALID_ARG: return "invalid argument";
    case FINCH_ERR_UNSUPPORTED: return "unsupported configuration";
    case FINCH_ERR_CAPACITY: return "size exceeds capacity";
    case FINCH_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case FINCH_ERR_HIP: return "HIP call failed";
    case FINCH_ERR_TIMEOUT: return "workgroups of a layer waited for each other in vain";
  }
  return "unknown status";
}

int32_t finch_version(void) { return 100; }

}  // extern "C"
