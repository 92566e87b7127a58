/*
 * finch.h - C ABI of the MI355X (gfx950) library for Finch's prompt-guided
 * KV-cache selection step (arxiv 2408.00167, Method section).
 *
 * One *problem* is one (request, layer, KV head).  At a prefill step the problem
 * has c rows already in its compressed cache and m rows in the new document
 * chunk; N = c + m candidate keys, ordered cache rows first, then chunk rows
 * (the column order of the paper's prompt-guided sub-matrix A^cont, whose columns
 * run over the chunk and the tokens accumulated in the cache).  Its query block
 * stacks the n_que prompt rows of each of the G query heads that share the KV
 * head: R = G * n_que rows.
 *
 * All data pointers inside finch_problem are DEVICE pointers owned by the caller.
 * Descriptor arrays are passed twice: `host_desc` (host memory, read during the
 * call for validation and launch sizing) and `dev_desc` (device memory holding the
 * same bytes, read by the kernels).  Every entry point enqueues work on `stream`
 * (a hipStream_t passed as void*, NULL = the null stream) and returns without
 * synchronising; nothing is allocated after finch_create.  Outputs are valid once
 * the caller has synchronised the stream.  Results are bit-identical run to run.
 *
 * Threads and streams: one context is for one host thread and one stream at a time (it
 * holds settings, the last HIP error, the profiling pool and the memo of finch_loop's
 * checks, none of them synchronised).  Concurrent use - several host threads, or work in
 * flight on several streams - takes one context per thread or stream, each with its own
 * workspace.  Calls that share a workspace, or descriptors whose outputs overlap, must
 * be ordered by the caller (same stream, or events).
 *
 * Errors: every function returns a finch_status.  Argument errors are detected on
 * the host before anything is launched.  Non-finite inputs are undefined
 * behaviour (not checked).
 */
#ifndef FINCH_H
#define FINCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FINCH_OK = 0,
  FINCH_ERR_INVALID_ARG = -1, /* null/misaligned pointer, negative size, aliasing */
  FINCH_ERR_UNSUPPORTED = -2, /* dtype / head_dim / group size not built          */
  FINCH_ERR_CAPACITY = -3,    /* a size exceeds what one launch can index         */
  FINCH_ERR_WORKSPACE = -4,   /* workspace missing, misaligned or too small       */
  FINCH_ERR_HIP = -5,         /* a HIP call failed; see finch_last_hip_error      */
  FINCH_ERR_TIMEOUT = -6      /* finch_workspace_status: workgroups waited in vain */
} finch_status;

typedef enum { FINCH_F32 = 0, FINCH_BF16 = 1 } finch_dtype;

typedef struct finch_ctx finch_ctx; /* opaque; bound to the device current at finch_create */

typedef struct {
  int32_t dtype;      /* finch_dtype of Q, K, V.  Scores are always fp32.          */
  int32_t head_dim;   /* d_k: 64 or 128                                            */
  int32_t group_size; /* G = query heads per KV head (1 = MHA), 1..64              */
  int32_t reserved;   /* must be 0                                                 */
} finch_config;

typedef struct {
  const void* q;       /* [G*n_que][d] row-major: head 0's prompt rows, head 1's, ... */
  const void* k_cache; /* [c][d] keys kept so far (may be NULL when c == 0)           */
  const void* v_cache; /* [c][d]                                                      */
  const void* k_chunk; /* [m][d] keys of the new chunk (may be NULL when m == 0)      */
  const void* v_chunk; /* [m][d]                                                      */
  void* k_out;         /* [>= min(r, c+m)][d]; must not overlap any source above      */
  void* v_out;         /* [>= min(r, c+m)][d]                                         */
  float* scores;       /* [c+m] out.  finch_step accepts NULL (kept in workspace)     */
  int32_t* idx;        /* [min(r, c+m)] out: kept candidates, ascending, in [0, c+m)  */
  int32_t n_que;       /* prompt rows per query head, >= 1                            */
  int32_t c;           /* cache rows, >= 0                                            */
  int32_t m;           /* chunk rows, >= 0 (m == 0: a cache-only step)                */
  int32_t r;           /* rows to keep, >= 0; values above c+m mean "keep all"        */
  const void* k_que;   /* [n_que][d] the prompt's own keys for this KV head; read only
                          by finch_prompt_lse, may be NULL everywhere else            */
  float* lse_extra;    /* [G*n_que] natural-log log-sum-exp, per prompt row, of logits
                          over keys that are not candidates; NULL = none.  Written by
                          finch_prompt_lse, read by the scoring of every other call   */
  const void* q_doc;   /* [G*m][d] queries of the chunk's own tokens, head 0's m rows,
                          head 1's, ...; NULL = rows from the prompt only (see
                          "Conditioning on the chunk's own rows" below)               */
} finch_problem;

/* Row bases (q, k_*, v_*, *_out) must be 16-byte aligned, scores and idx 4-byte. */

finch_status finch_create(const finch_config* cfg, finch_ctx** out);
finch_status finch_destroy(finch_ctx* ctx);

/* Bytes of device workspace that any of the four calls below needs for this batch
 * (an upper bound valid for every call whose per-problem n_que, c+m and r do not
 * exceed the maxima of `host_desc`).  The workspace must be 256-byte aligned. */
finch_status finch_workspace_size(const finch_ctx* ctx, const finch_problem* host_desc,
                                  int32_t n_problems, size_t* bytes);

/* Scoring (Method: attention of the prompt rows over the context keys, summed
 * over the heads of the group and over the prompt rows):
 *   scores[j] = sum_{i<R} softmax_j( q_i . k_j / sqrt(d_k) ),  j < c+m,
 * the softmax running over the c+m context keys, so sum_j scores[j] == R.
 * Writes desc.scores (must be non-NULL here).  (See below for desc.lse_extra.) */
finch_status finch_score(finch_ctx* ctx, const finch_problem* host_desc,
                         const finch_problem* dev_desc, int32_t n_problems,
                         void* workspace, size_t workspace_bytes, void* stream);

/* The paper-exact denominator.  With desc.lse_extra the denominator of row i is widened to
 *   sum_j exp(s_ij) + exp(lse_extra[i]):
 * the weights of the prompt-guided sub-matrix exactly as the model forms them, where
 * (Method: the prompt follows the chunk in the input) a prompt token also attends to
 * the prompt tokens up to itself.  Then sum_j scores[j] < R.  finch_prompt_lse
 * computes that term: lse_extra[g*n_que + t] = log sum_{j<=t} exp(q_{g,t} . kq_j /
 * sqrt(d_k)) over the prompt keys desc.k_que (causal).  It reads desc.q, desc.k_que
 * and n_que and writes desc.lse_extra (all three required); no workspace. */
finch_status finch_prompt_lse(finch_ctx* ctx, const finch_problem* host_desc,
                              const finch_problem* dev_desc, int32_t n_problems, void* stream);

/* Conditioning on the chunk's own rows (the paper's ablation of the conditioning:
 * self-attention of the document chunk, alone or together with the prompt, in
 * place of the prompt-guided sub-matrix, with the Method's normalisation step).
 * With desc.q_doc the scoring of finch_score, finch_step and finch_loop adds, for
 * every head g and chunk token i, the row q_doc[g*m + i]: it sees the cache and the
 * chunk keys up to itself (the c + i + 1 first candidates; the model's input is
 * [cache ; chunk ; prompt] under the causal mask), its weights are a softmax over
 * those, and the normalisation step multiplies them by (c + i + 1) / (c + m) - read
 * per row: the factor offsets the thinner spread of rows that see more keys and is
 * 1 for prompt rows.  scores[j] is the sum over all rows that see key j.  desc.q
 * may then be NULL (document rows only; n_que is ignored).  Always through the
 * one-workgroup-per-problem kernels whatever the batch size (FINCH_PATH_SEPARATE:
 * FINCH_ERR_UNSUPPORTED); the work grows from G*n_que to G*(n_que + m) rows per problem. */

/* Selection (Method: t = top-r(A_agg, r)): reads desc.scores (any finite fp32),
 * writes the indices of the min(r, c+m) largest into desc.idx in ascending order;
 * equal scores are resolved towards the lower index (+0 and -0 are equal). */
finch_status finch_topk(finch_ctx* ctx, const finch_problem* host_desc,
                        const finch_problem* dev_desc, int32_t n_problems,
                        void* workspace, size_t workspace_bytes, void* stream);

/* Compaction (Method: Managing the Cache - the K,V pairs of the selected
 * positions are kept): k_out[t] = K[idx[t]], v_out[t] = V[idx[t]] for
 * t < min(r, c+m), where row j of K is k_cache[j] if j < c else k_chunk[j-c].
 * A bit-for-bit copy; rows of k_out/v_out beyond that are left untouched. */
finch_status finch_compact(finch_ctx* ctx, const finch_problem* host_desc,
                           const finch_problem* dev_desc, int32_t n_problems,
                           void* workspace, size_t workspace_bytes, void* stream);

/* Re-positioning (Method: Managing the Cache - the positional embedding of a kept
 * pair is adjusted to the place it moves to; for rotary embeddings by rotating the
 * key to the earlier or later position).  Once set on a context, the compaction of
 * finch_compact, finch_step and finch_loop becomes
 *   k_out[slot(t)] = Rot(K[idx[t]], slot(t) - idx[t]),  v_out[slot(t)] = V[idx[t]],
 * t < min(r, c+m): a candidate's old position is its index in [cache ; chunk], its
 * new one its slot.  Rot(x, s) turns channel pair u of x by the angle s * theta_u,
 * theta_u = base^(-2u/d): pairs are (u, u + d/2) for FINCH_ROPE_HALF (the layout of
 * Llama-style models) or (2u, 2u+1) for FINCH_ROPE_INTERLEAVED; FINCH_ROPE_OFF
 * leaves keys as they are.  slot(t) = t for FINCH_ORDER_ASCENDING; for
 * FINCH_ORDER_RANK the kept pairs are packed by relevance as in the paper's worked
 * example: slot = rank of the score among the kept ones, highest first, equal
 * scores by index (idx itself stays ascending; needs desc.scores in finch_compact
 * and at most 32768 kept rows per problem, else FINCH_ERR_CAPACITY).  Rotation is
 * computed in fp32 (angles reduced in fp64); bf16 results are rounded to nearest
 * even; a shift of 0 leaves the key bit-identical.  NULL, or {OFF, ASCENDING},
 * restores the plain copy.  With FINCH_ORDER_RANK the one-workgroup-per-problem kernels
 * take batches that keep at most 2048 rows per problem (the workgroup ranks its kept rows
 * in LDS); others run with one kernel per stage (FINCH_PATH_OWNER: FINCH_ERR_UNSUPPORTED). */
typedef enum { FINCH_ROPE_OFF = 0, FINCH_ROPE_HALF = 1, FINCH_ROPE_INTERLEAVED = 2 } finch_rope_pairing;
typedef enum { FINCH_ORDER_ASCENDING = 0, FINCH_ORDER_RANK = 1 } finch_order;
typedef struct {
  int32_t pairing; /* finch_rope_pairing */
  int32_t order;   /* finch_order        */
  double base;     /* rotary base (10000 for Llama 2); > 1 when pairing != OFF */
} finch_reposition;
finch_status finch_set_reposition(finch_ctx* ctx, const finch_reposition* how);

/* One prefill step (Method: Document Segmentation - the pairs kept at step i-1
 * compete with chunk i): score, then top-r, then compaction, stream-ordered with
 * no host synchronisation.  desc.scores may be NULL. */
finch_status finch_step(finch_ctx* ctx, const finch_problem* host_desc,
                        const finch_problem* dev_desc, int32_t n_problems,
                        void* workspace, size_t workspace_bytes, void* stream);

/* finch_step for callers that cannot allocate and have no workspace to pass: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same
 * step with the same results, but the scratch memory (row statistics, row
 * log-sum-exps, scores of descriptors whose `scores` is NULL, layer sums) is a
 * file-scope device array inside the library, finch_static_scratch_bytes() = 16 MiB on
 * every GPU the library is used on, held until the process ends.  A batch that needs
 * more (finch_workspace_size tells) is refused with FINCH_ERR_CAPACITY and a message on
 * stderr; nothing is launched then.  The call allocates nothing and frees nothing.
 * All calls on one GPU share that GPU's array, which keeps the last call's contents
 * (nothing in it has to start at zero): calls that overlap in time on one GPU - two
 * streams, two contexts, two threads - race; order them on one stream or with events. */
finch_status finch_step_static(finch_ctx* ctx, const finch_problem* host_desc,
                               const finch_problem* dev_desc, int32_t n_problems, void* stream);
size_t finch_static_scratch_bytes(void);

/* The whole chunk loop in one call (Method: Document Segmentation - chunk after
 * chunk, each step's kept pairs competing with the next chunk): the same results as
 * finch_step on the batch of step 0, then on that of step 1, and so on.  The
 * descriptors of step s are host_desc[step_first[s] .. step_first[s+1]) (dev_desc
 * holds the same bytes on the device); step_first has n_steps + 1 entries, starts at
 * 0, and the number of problems per step must not grow with s.  Slot j of every
 * step in which it is present describes the same problem (normally its k_cache /
 * v_cache at step s+1 are its k_out / v_out of step s), and no descriptor may read
 * memory that a descriptor in another slot writes: slots are processed
 * independently, each through all of its steps, possibly by one kernel launch for
 * the whole loop (one workgroup per slot; picked under FINCH_PATH_AUTO when the
 * slots fill the chip, forced by FINCH_PATH_OWNER), otherwise step by step.
 * host_step_first is host memory, dev_step_first a device copy of it.  The
 * workspace must hold finch_loop_workspace_size bytes (never more than
 * finch_workspace_size of all descriptors taken as one batch). */
finch_status finch_loop_workspace_size(const finch_ctx* ctx, const finch_problem* host_desc,
                                       const int32_t* host_step_first, int32_t n_steps,
                                       size_t* bytes);
finch_status finch_loop(finch_ctx* ctx, const finch_problem* host_desc,
                        const finch_problem* dev_desc, const int32_t* host_step_first,
                        const int32_t* dev_step_first, int32_t n_steps, void* workspace,
                        size_t workspace_bytes, void* stream);

/* The first word of a workspace is the status word of the launches that used it last.
 * Only one thing sets it: with FINCH_OPT_LAYER_GROUP > 1 the workgroups of a layer wait
 * for each other inside the one-workgroup-per-problem kernels, at most about 0.2 s each
 * time; a workgroup whose wait runs out sets the word and goes on with the scores it
 * finds, so the launch always ends, but its selection is then not the layer's.  This
 * call waits for `stream`, copies the word to *flags and returns FINCH_ERR_TIMEOUT if it
 * is not zero (which takes a chip on which other work keeps some of the batch's
 * workgroups from starting).  While FINCH_OPT_LAYER_GROUP > 1 every finch_step and
 * finch_loop call clears the word first; with the option at 1 the call reports 0. */
finch_status finch_workspace_status(finch_ctx* ctx, const void* workspace, void* stream, int32_t* flags);

/* Host-only: the argument checks of finch_loop on a descriptor set, without a context
 * and without touching a GPU (the pointers are only compared, never followed): step
 * table, pointers and alignment, outputs that overlap their own sources, and the rule
 * above that no slot may write memory another slot reads or writes
 * (FINCH_ERR_INVALID_ARG).  finch_loop makes the same checks itself; the one on
 * overlaps between slots it repeats only when the descriptors have changed since the
 * last call on the context. */
finch_status finch_loop_check(const finch_config* cfg, const finch_problem* host_desc,
                              const int32_t* host_step_first, int32_t n_steps);

/* Host-only: rows kept after each chunk step (Method: the update rule
 * r_{it+1} = m_{it+1}/sigma + c_it with sigma = n_cont/k, ending at r = k), in
 * integers: r_i = min(c_{i-1} + m_i, floor(min(k, n_cont) * seen_i / n_cont)).
 * Writes ceil(n_cont/m) values; `r_len` is the capacity of r_out. */
finch_status finch_schedule(int64_t n_cont, int32_t m, int64_t k, int32_t* r_out,
                            int32_t r_len);
/* The same with a choice of rule: FINCH_SCHEDULE_PROPORTIONAL is the rule above;
 * FINCH_SCHEDULE_CONSTANT keeps the whole budget from the start ("top-k under the
 * budget" read literally): r_i = min(c_{i-1} + m_i, min(k, n_cont)). */
typedef enum { FINCH_SCHEDULE_PROPORTIONAL = 0, FINCH_SCHEDULE_CONSTANT = 1 } finch_schedule_rule;
finch_status finch_schedule_mode(int64_t n_cont, int32_t m, int64_t k, int32_t mode,
                                 int32_t* r_out, int32_t r_len);

/* Options.  FINCH_OPT_STEP_PATH picks how the stages are launched.  SEPARATE uses
 * one kernel per stage: row statistics, merge, per-key sums, top-r, compaction.
 * OWNER gives every problem to one workgroup of 8 waves that runs all stages of the
 * step - or, in finch_loop, of all steps - back to back (bf16: matrix instructions;
 * fp32: the vector ALU, meant for small problems); batches it cannot run fail with
 * FINCH_ERR_UNSUPPORTED.  AUTO (default) takes OWNER for bf16 when the batch has enough
 * problems to fill the chip's compute units in whole rounds, for fp32 when no problem
 * has more than 4096 candidates or 64 prompt rows, else SEPARATE. */
typedef enum {
  FINCH_OPT_STEP_PATH = 1,
  /* tuning: target number of keys one workgroup of the two-pass bf16 scoring
   * kernels streams (default 2400); a problem is cut into round((c+m)/value) slices */
  FINCH_OPT_SLICE_KEYS = 3,
  /* Layer-wise selection as the paper words it (Method: "Sum over heads", then ONE
   * top-r per layer): value L > 1 makes every run of L consecutive problems of a
   * batch one layer (its KV heads; same c, m and r, batch size a multiple of L, else
   * FINCH_ERR_INVALID_ARG).  finch_topk, finch_step and finch_loop then add the
   * run's score vectors head by head, select once on the sum and write the same
   * indices to every problem of the run; each head compacts its own rows.  The
   * per-problem scores stay as they are.  1 (default): one selection per problem.
   * FINCH_ORDER_RANK is refused (FINCH_ERR_UNSUPPORTED) while L > 1.  The
   * one-workgroup-per-problem kernels take such batches when L <= 16 and the batch has
   * no more problems than the chip has compute units: the L workgroups of a run then
   * wait for each other's scores inside the launch (see finch_workspace_status);
   * other batches run with one kernel per stage. */
  FINCH_OPT_LAYER_GROUP = 4,
  /* how long a workgroup waits for the others of its layer before it gives up, in ticks
   * of the GPU's 100 MHz wall clock: 0 .. 10^9, default 2 * 10^7 (0.2 s).  A wait that
   * expires sets the workspace's status word (finch_workspace_status); the workgroup
   * leaves that step's indices and cache rows unwritten and the launch goes on to its
   * end: nothing is written outside its buffers, but indices and caches of that call are
   * not to be used.  0 makes the first workgroup of every layer give up at once: the way
   * to exercise the error path. */
  FINCH_OPT_LAYER_WAIT_TICKS = 5
} finch_option;
typedef enum { FINCH_PATH_AUTO = 0, FINCH_PATH_SEPARATE = 1, FINCH_PATH_OWNER = 3 } finch_path;
finch_status finch_set_option(finch_ctx* ctx, int32_t option, int64_t value);

/* Measurement helpers (not part of the method).  finch_profile(ctx, 1) creates a
 * pool of HIP events (this call allocates; make it outside any timed loop) and
 * from then on every kernel launch of this context is bracketed by two events on
 * the launch stream; finch_profile(ctx, 0) stops and frees them.
 * finch_profile_read waits for the recorded events, adds up the elapsed
 * milliseconds and launch counts per kernel class into ms[FINCH_KERNEL_COUNT] and
 * launches[FINCH_KERNEL_COUNT] (host arrays), and clears the pool.  At most 8192
 * launches are recorded between two reads; later ones are not timed. */
typedef enum {
  FINCH_KERNEL_ROWSTATS = 0, /* scoring pass 1: per-row softmax statistics   */
  FINCH_KERNEL_LSE = 1,      /* merge of the per-tile statistics             */
  FINCH_KERNEL_COLSUM = 2,   /* scoring pass 2: per-key sums of the weights  */
  FINCH_KERNEL_SELECT = 3,   /* top-r                                        */
  FINCH_KERNEL_GATHER = 4,   /* compaction                                   */
  FINCH_KERNEL_OWNER = 5,    /* all stages, one workgroup per problem        */
  FINCH_KERNEL_PROMPT_LSE = 6, /* finch_prompt_lse                             */
  FINCH_KERNEL_COUNT = 7
} finch_kernel;
finch_status finch_profile(finch_ctx* ctx, int32_t enable);
finch_status finch_profile_read(finch_ctx* ctx, float* ms, int32_t* launches);

/* The hipError_t (as int) of the last failed HIP call seen by this context. */
int32_t finch_last_hip_error(const finch_ctx* ctx);
const char* finch_status_string(finch_status s);
/* Library version, major*10000 + minor*100 + patch. */
int32_t finch_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FINCH_H */
