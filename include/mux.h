/*
 * mux.h - C ABI of the MI355X (gfx950) head-wise paged KV-cache library.
 *
 * The library implements the data path of MuxServe's unified KV cache
 * (arXiv 2404.02015, Section 3.4 "Resource Manager" and its closing
 * "Implementation" paragraph): the KV cache of every colocated LLM lives in ONE
 * pool of small blocks, each block holding the K and V of one KV head for a fixed
 * number of tokens; a memory manager hands blocks to the engines, the engines write
 * new K/V into the blocks they were given and run attention over them, and the
 * blocks go back to the pool when the request ends.
 *
 * Conventions for every call
 *   - plain C linkage, no exceptions; the return value is a status (MUX_OK or a negative
 *     mux_status_t) unless stated otherwise.  All state lives in the objects the calls
 *     take (pool, scheduler, runner).  The library itself keeps three things per process,
 *     none of which a caller can observe through results: a mutex-guarded table of
 *     "workgroups of kernel K resident on device D" (a hardware property, asked from the
 *     runtime on first use), the device addresses of mux_decode_attn_static's scratch
 *     array, and the tuning switches below.
 *   - tuning switches, read from the environment ONCE per process on first use (defaults
 *     are what the published measurements use; none changes a result beyond summation
 *     order): MUX_DECODE_SPAN_BLOCKS=n (blocks per span of a split context),
 *     MUX_DECODE_WG_PER_CU=n (overrides the occupancy query), MUX_DECODE_PLAN_KERNEL=1
 *     (always build the work list in a kernel of its own), MUX_DECODE_SPLIT_SHORT=1 (split
 *     contexts by the piece-count rule alone), MUX_PREFILL_BUNDLE=n (row tiles of one
 *     (sequence, head) dispatched back to back on one XCD), MUX_PREFILL_CB=1|2 (16-row
 *     column blocks per wave), MUX_RUNNER_STAGE_ALWAYS=1 (read by mux_runner_create: job
 *     arrays always travel through pinned staging memory, never as kernel arguments).
 *   - "HOST" pointers are ordinary process memory, "DEVICE" pointers are HIP device
 *     memory of the GPU that is current when the call is made.
 *   - the caller owns the pool memory, block tables, Q/O tensors and workspaces; the
 *     library owns only the ids and counters inside mux_pool_t.
 *   - pool management calls are synchronous host calls, do no GPU work and may be
 *     made from several host threads on the same pool.
 *   - the three kernel calls only ENQUEUE work on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and return; they never synchronise and never
 *     allocate device memory.  Calls for different models on different streams over
 *     the same pool are safe concurrently because their blocks are disjoint.
 *
 * Pool layout (part of the ABI): block `id` starts at
 *     kv_base + id * (2 * block_size * head_dim * elem_bytes)
 * and holds the K tile [block_size][head_dim] row-major, followed by the V tile
 * [block_size][head_dim] row-major, for one (model, layer, kv head, token span).
 *
 * Block tables: int32 [n_seqs][n_kv_heads][max_blocks]; entry [s][h][j] is the id of
 * the block holding tokens j*block_size .. (j+1)*block_size-1 of kv head h of
 * sequence s.  Entries past ceil(len/block_size) are never read.
 */
#ifndef MUX_H
#define MUX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MUX_API __attribute__((visibility("default")))

typedef struct mux_pool mux_pool_t; /* opaque, library-owned host object */

typedef enum { MUX_BF16 = 0, MUX_FP32 = 1 } mux_dtype_t;

typedef enum {
    MUX_OK = 0,
    MUX_ERR_INVALID = -1,     /* bad argument; unknown, foreign, repeated or already-free block id */
    MUX_ERR_NOMEM = -2,       /* not enough free blocks; ALL-OR-NOTHING: nothing changed */
    MUX_ERR_QUOTA = -3,       /* the request would take the model past its token-block quota; nothing changed */
    MUX_ERR_HIP = -4,         /* a HIP runtime call or kernel launch failed */
    MUX_ERR_UNSUPPORTED = -5, /* shape or dtype outside what the kernels are built for */
    MUX_ERR_TOO_LARGE = -6    /* the call needs more scratch than the library's fixed scratch array holds */
} mux_status_t;

#define MUX_MAX_MODELS 1024 /* model_id must lie in [0, MUX_MAX_MODELS) */

/* ---------------------------------------------------------------------------------
 * Unified KV space (Section 3.4: one space shared by all colocated LLMs, cut into
 * head-wise blocks).
 *
 * mux_pool_create carves the caller's device buffer into `num_blocks` blocks and
 * builds the free list.  kv_base: DEVICE, 16-byte aligned, at least
 * num_blocks * 2 * block_size * head_dim * elem_bytes long (kv_bytes is checked); it
 * stays owned by the caller and must outlive the pool.  init_free_order: HOST,
 * nullable; if given it must be a permutation of [0, num_blocks) and is the order in
 * which the fresh pool hands out ids (identity otherwise).  Supported: block_size
 * 1..256, head_dim 64 or 128, dtype bf16 or fp32; anything else MUX_ERR_UNSUPPORTED.
 * mux_pool_destroy frees host state only.
 * ------------------------------------------------------------------------------- */
MUX_API int mux_pool_create(mux_pool_t **out, void *kv_base, size_t kv_bytes, int64_t num_blocks,
                    int32_t block_size, int32_t head_dim, mux_dtype_t dtype,
                    const int32_t *init_free_order);
MUX_API int mux_pool_destroy(mux_pool_t *pool);

/* Counters: free blocks, blocks held by one model, bytes per block. Negative = error. */
MUX_API int64_t mux_pool_num_free(const mux_pool_t *pool);
MUX_API int64_t mux_pool_num_used(const mux_pool_t *pool, int32_t model_id);
MUX_API int64_t mux_pool_block_bytes(const mux_pool_t *pool);

/* ---------------------------------------------------------------------------------
 * Block manager (Section 3.4, Implementation: an engine requests new cache blocks,
 * keeps them from its prefill through its decoding steps, and they are released only
 * when the request finishes).  The free list is a LIFO stack: mux_alloc_blocks pops n
 * ids and returns them in pop order; mux_free_blocks pushes ids in the order given,
 * so the last id freed is the first one handed out again.
 *
 * out_ids / ids: HOST arrays of n int32.  n == 0 is a no-op.
 * mux_alloc_blocks: a model with a quota (below) that would hold more than it ->
 * MUX_ERR_QUOTA; else fewer than n free blocks -> MUX_ERR_NOMEM; in both cases pool and
 * out_ids are untouched.  mux_free_blocks: an id that is out of range, not currently held by
 * `model_id`, or named twice in the call -> MUX_ERR_INVALID, nothing changed.
 * ------------------------------------------------------------------------------- */
MUX_API int mux_alloc_blocks(mux_pool_t *pool, int32_t model_id, int64_t n, int32_t *out_ids);
MUX_API int mux_free_blocks(mux_pool_t *pool, int32_t model_id, int64_t n, const int32_t *ids);

/* ---------------------------------------------------------------------------------
 * Token-block quotas (Section 3.3 and Algorithm 3: every LLM of a unit gets a quota of
 * token blocks so that the shared cache is split fairly; the scheduler initialises the
 * quotas, checks them before it runs a job, and periodically moves blocks from LLMs that
 * use little of their quota to LLMs that use most of theirs).  Host calls; they never
 * touch device memory.  The paper gives no formulas; the rules are:
 *
 * mux_pool_set_quota: cap on the blocks `model_id` may hold, 0..num_blocks, or -1 for
 *   none (the state of a fresh pool).  A quota below the current holding takes nothing
 *   back: allocations fail with MUX_ERR_QUOTA until enough blocks were freed.
 * mux_pool_get_quota: *out = the quota or -1.   mux_pool_peak_used: *out = the largest
 *   number of blocks the model held since the last mux_pool_adapt_quotas (or creation).
 * mux_pool_init_quotas: models 0..n_models-1 share ALL num_blocks in proportion to
 *   weights[m] (host array of n_models finite doubles >= 0 with a positive sum; the
 *   paper normalises block usage by request rate, so pass rate x blocks per token):
 *   floor(num_blocks * w / sum) each, the blocks left over one each to the largest
 *   fractional parts, ties to the lower model id.
 * mux_pool_adapt_quotas: utilisation of a model = peak / quota.  A model with
 *   peak < low * quota gives away floor(step * (quota - peak)) blocks of quota; the blocks
 *   collected go to the models with peak > 0 and peak >= high * quota in proportion to
 *   their peaks (integer largest remainder, ties to the lower id).  Without givers or
 *   takers nothing moves.  The sum of quotas is unchanged, no quota drops below its
 *   model's peak, peaks restart from the current holdings.  *moved (may be NULL) = blocks
 *   of quota moved.  Needs 0 <= low <= high < inf, 0 <= step <= 1 and a quota on every
 *   model 0..n_models-1; else MUX_ERR_INVALID and nothing changes.
 * ------------------------------------------------------------------------------- */
MUX_API int mux_pool_set_quota(mux_pool_t *pool, int32_t model_id, int64_t max_blocks);
MUX_API int mux_pool_get_quota(const mux_pool_t *pool, int32_t model_id, int64_t *out);
MUX_API int mux_pool_peak_used(const mux_pool_t *pool, int32_t model_id, int64_t *out);
MUX_API int mux_pool_init_quotas(mux_pool_t *pool, int32_t n_models, const double *weights);
MUX_API int mux_pool_adapt_quotas(mux_pool_t *pool, int32_t n_models, double low, double high, double step,
                                  int64_t *moved);

/* ---------------------------------------------------------------------------------
 * KV append (Section 3.4, Implementation: the engine fills K/V into the blocks it
 * was assigned).  For every new token t, sequence s = tok_seq[t], position
 * p = tok_pos[t] and kv head h, the rows k_new[t][h][:] and v_new[t][h][:] are copied
 * bit for bit to row p % block_size of block block_tables[s][h][p / block_size].
 *
 * k_new, v_new: DEVICE [n_tokens][n_kv_heads][head_dim] in the pool dtype, 16-byte
 * aligned.  tok_seq, tok_pos: DEVICE int32 [n_tokens].  block_tables: DEVICE.
 * A token whose sequence, position or block id is out of range is skipped by the
 * kernel (nothing is written for it); no error can be reported for device-side data.
 * Two tokens of one call must not name the same (sequence, position).
 * ------------------------------------------------------------------------------- */
MUX_API int mux_kv_append(mux_pool_t *pool, const void *k_new, const void *v_new, const int32_t *tok_seq,
                  const int32_t *tok_pos, const int32_t *block_tables, int32_t n_tokens,
                  int32_t n_seqs, int32_t n_kv_heads, int32_t max_blocks, void *stream);

/* ---------------------------------------------------------------------------------
 * Decode attention (Section 2.1: one new token per step attends to the cached K/V of
 * all earlier tokens; Section 3.4: that cache is read through head-wise blocks).
 * For sequence s and query head i (kv head h = i / (n_q_heads / n_kv_heads)):
 *     out[s][i][:] = sum_j softmax_j(scale * <q[s][i], K_j>) V_j,  j < ctx_lens[s],
 * with K_j, V_j row j % block_size of block block_tables[s][h][j / block_size].
 * ctx_lens count the token appended in this step.  ctx_lens[s] == 0 gives zeros.
 * Storage is the pool dtype; all arithmetic and accumulation are fp32, with one
 * round-to-nearest-even to the storage type at the end.
 *
 * out, q: DEVICE [n_seqs][n_q_heads][head_dim], pool dtype, 16-byte aligned.
 * ctx_lens: DEVICE int32 [n_seqs].  max_ctx_len: HOST upper bound on ctx_lens, used
 * to size the grid and the split of long contexts without reading device memory
 * (tokens beyond it are ignored).  workspace: DEVICE scratch of at least
 * mux_decode_workspace_bytes(...) bytes (never 0: it holds the call's work list and, for
 * long contexts, the partial results of the spans), 16-byte aligned, private to this call
 * until it has finished on `stream`.
 * ------------------------------------------------------------------------------- */
MUX_API int mux_decode_attn(mux_pool_t *pool, void *out, const void *q, const int32_t *block_tables,
                    const int32_t *ctx_lens, int32_t n_seqs, int32_t n_q_heads, int32_t n_kv_heads,
                    int32_t max_blocks, int32_t max_ctx_len, float scale, void *workspace,
                    size_t workspace_bytes, void *stream);
MUX_API size_t mux_decode_workspace_bytes(const mux_pool_t *pool, int32_t n_seqs, int32_t n_q_heads,
                                  int32_t n_kv_heads, int32_t max_ctx_len);
/* For callers that allocate one workspace up front: the largest value mux_decode_workspace_bytes
 * returns for ANY call with 1 .. max_seqs sequences and 1 .. max_ctx_len as its max_ctx_len.  A
 * smaller call can need more than the largest one (few long rows are cut into many spans), so
 * sizing for the largest call alone is not enough.  Host arithmetic only; 0 for bad arguments. */
MUX_API size_t mux_decode_workspace_bound(const mux_pool_t *pool, int32_t max_seqs, int32_t n_q_heads,
                                  int32_t n_kv_heads, int32_t max_ctx_len);

/* ---------------------------------------------------------------------------------
 * Decode attention without a workspace argument, for callers that cannot allocate device
 * memory at all: code running under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels and bit-identical results as
 * mux_decode_attn; the call's scratch lives in a fixed array of MUX_STATIC_SCRATCH_BYTES that
 * is part of the library's device image (every GPU the library runs on holds it until the
 * process ends).  The call allocates and frees no device memory and calls no allocating
 * runtime routine; the only thing it may put on the host heap is one entry of a small table,
 * the first time a GPU runs one of the kernels (how many of its workgroups the GPU holds at once).
 * A call whose mux_decode_workspace_bytes(...) exceeds MUX_STATIC_SCRATCH_BYTES is refused with
 * MUX_ERR_TOO_LARGE and launches nothing.  Every call on one GPU uses that GPU's one array:
 * two such calls must not overlap on a GPU (same stream, or ordered by events) - overlapping
 * calls race on the scratch and give wrong outputs.  The array keeps the previous call's
 * contents; nothing in it needs to start at zero and no call reads what another one left.
 * ------------------------------------------------------------------------------- */
#define MUX_STATIC_SCRATCH_BYTES (32 * 1024 * 1024)
MUX_API int mux_decode_attn_static(mux_pool_t *pool, void *out, const void *q, const int32_t *block_tables,
                                   const int32_t *ctx_lens, int32_t n_seqs, int32_t n_q_heads, int32_t n_kv_heads,
                                   int32_t max_blocks, int32_t max_ctx_len, float scale, void *stream);

/* ---------------------------------------------------------------------------------
 * Fused decoding step (Section 3.4, Implementation: in one decoding step an engine fills the
 * new token's K/V into its blocks and runs attention over them; here both happen in one
 * launch, for all layers of the model at once).  Equivalent to, for every layer l:
 *     mux_kv_append(k_new[l], v_new[l], tok_seq = 0..n_seqs-1, tok_pos = ctx_lens - 1, block_tables[l])
 *     mux_decode_attn(out[l], q[l], block_tables[l], ctx_lens)
 * with the same results bit for bit in the pool and the same outputs.
 *
 * out, q: DEVICE [n_layers][n_seqs][n_q_heads][head_dim]; k_new, v_new: DEVICE
 * [n_layers][n_seqs][n_kv_heads][head_dim]; block_tables: DEVICE [n_layers][n_seqs][n_kv_heads]
 * [max_blocks] (every layer has its own blocks); ctx_lens: DEVICE [n_seqs], lengths AFTER the
 * append (the new token sits at position ctx_lens[s] - 1; sequences with ctx_lens[s] == 0
 * append nothing and return zeros).  The blocks of the new positions must already be in the
 * tables.  max_ctx_len must bound ctx_lens as in mux_decode_attn; a sequence whose ctx_lens[s]
 * exceeds it appends NOTHING (its new token lies beyond the part of the context this launch
 * was sized for) and attends to its first max_ctx_len cached tokens only.
 * workspace: at least mux_decode_step_workspace_bytes(...) bytes, 16-byte aligned.
 * ------------------------------------------------------------------------------- */
MUX_API int mux_decode_step(mux_pool_t *pool, void *out, const void *q, const void *k_new, const void *v_new,
                    const int32_t *block_tables, const int32_t *ctx_lens, int32_t n_layers, int32_t n_seqs,
                    int32_t n_q_heads, int32_t n_kv_heads, int32_t max_blocks, int32_t max_ctx_len,
                    float scale, void *workspace, size_t workspace_bytes, void *stream);
MUX_API size_t mux_decode_step_workspace_bytes(const mux_pool_t *pool, int32_t n_layers, int32_t n_seqs,
                                       int32_t n_q_heads, int32_t n_kv_heads, int32_t max_ctx_len);

/* ---------------------------------------------------------------------------------
 * Chunked causal prefill attention (Section 2.1: prefill processes the prompt tokens
 * in parallel).  Sequence s contributes the query rows cu_q_lens[s] .. cu_q_lens[s+1]-1
 * of the packed q; row r of that chunk sits at absolute position p = q_start[s] + r and
 * attends to keys 0 .. p.  The chunk's own K/V must already be in the pool
 * (mux_kv_append first).  Arithmetic as for decode; for bf16 the softmax weights are
 * rounded to bf16 before the P.V matrix product, accumulation stays fp32.
 *
 * out, q: DEVICE [total_q][n_q_heads][head_dim].  cu_q_lens: DEVICE int32 [n_seqs+1].
 * q_start: DEVICE int32 [n_seqs], tokens cached before this chunk.  max_q_len,
 * max_ctx_len: HOST upper bounds on the chunk lengths and on q_start + chunk length.
 * workspace: DEVICE scratch of at least mux_prefill_workspace_bytes(...) bytes, 16-byte
 * aligned; that function returns 0 (workspace may be NULL) for bf16 pools whose blocks hold
 * a power of two >= 8 tokens, which run on the matrix cores; other pools take a slow generic
 * path that may need scratch for long contexts.
 * ------------------------------------------------------------------------------- */
MUX_API int mux_prefill_attn(mux_pool_t *pool, void *out, const void *q, const int32_t *cu_q_lens,
                     const int32_t *q_start, const int32_t *block_tables, int32_t n_seqs,
                     int32_t total_q, int32_t max_q_len, int32_t max_ctx_len, int32_t n_q_heads,
                     int32_t n_kv_heads, int32_t max_blocks, float scale, void *workspace,
                     size_t workspace_bytes, void *stream);
MUX_API size_t mux_prefill_workspace_bytes(const mux_pool_t *pool, int32_t n_seqs, int32_t total_q,
                                   int32_t max_ctx_len, int32_t n_q_heads, int32_t n_kv_heads);
/* The largest value mux_prefill_workspace_bytes returns for any call with 1 .. max_total_q query
 * rows and 1 .. max_ctx_len as its max_ctx_len (0 for pools that run on the matrix cores). */
MUX_API size_t mux_prefill_workspace_bound(const mux_pool_t *pool, int32_t max_total_q, int32_t max_ctx_len,
                                   int32_t n_q_heads, int32_t n_kv_heads);

/* ---------------------------------------------------------------------------------
 * Batch scheduler (Section 3.3, Algorithm 3: adaptive batch scheduling).  Host code: it
 * owns the request queues and the block tables of the colocated models, takes blocks from
 * the pool (under the models' quotas) and tells the caller which jobs to launch; it
 * launches nothing itself and never touches device memory.
 *
 * One call of mux_sched_step is one iteration of the algorithm's loop:
 *  1. Prefill.  The first model, round-robin from the model after the one served last,
 *     that has a waiting request forms one prefill job: its waiting requests in arrival
 *     order, taken one by one while the job stays within max_prefill_tokens tokens (the
 *     first request is taken whatever its length), a sequence slot (lowest free) is left,
 *     and the request's ceil(len / block_size) x heads blocks fit the model's quota and the
 *     pool (one mux_alloc_blocks call per request; ids head-major in its table row).  The
 *     prefill yields the request's first output token.  A job with no request is no job.
 *     The algorithm's rule that a prefill without resources holds back decoding concerns
 *     compute capacity, which a synchronous caller always has; a prefill refused for lack
 *     of blocks is skipped for this iteration (decoding is what frees blocks).
 *  2. Decoding.  Every model with running requests, starting with a model that rotates by
 *     one per iteration, runs one step for all of them: each request appends the token it
 *     produced last (context + 1; a context that was a multiple of block_size opens a new
 *     block per head: one mux_alloc_blocks call of `heads` ids per such request, in
 *     admission order) and produces the next.  If the step's new blocks do not fit quota or
 *     pool, the model's most recently admitted request is preempted - blocks freed, back to
 *     the FRONT of the waiting queue, to be recomputed (its next prefill covers prompt +
 *     outputs so far - 1 tokens) - until the step fits.  A request preempted in the iteration
 *     that admitted it is taken out of that iteration's prefill job instead of being listed in
 *     a preempt job (its blocks may already belong to another model's decoding job of the same
 *     iteration, so its K/V must not be written); it counts as a preemption.
 *  3. A request ends when it has produced output_len tokens.  Its blocks and slot are
 *     released at the START of the next mux_sched_step (one mux_free_blocks call per
 *     request, ids in table order, requests in the order they ended): the caller launches
 *     the job that ends it after this call returns, and that job still reads them.  The
 *     caller must order the kernels of one step before those of the next (blocks freed at
 *     a step's start may be handed to another model in that same step).
 *     Every adapt_period iterations (0 = never)
 *     mux_pool_adapt_quotas(low_util, high_util, step_fraction) runs over all models.
 *
 * Jobs of the last step, in execution order: mux_sched_job gives kind / model / number of
 * sequences; mux_sched_job_seqs copies per sequence (any pointer may be NULL) the request
 * id, its slot (row of the model's table), its length (prefill: tokens to prefill, from
 * position 0; decode: context length including the appended token; preempt: tokens it had
 * cached) and flags.  mux_sched_table: the model's HOST table, int32
 * [max_seqs][heads][max_blocks], owned by the scheduler, valid until it is destroyed;
 * the caller mirrors rows flagged MUX_JOB_FLAG_TABLE to the device.  `heads` is the
 * number of blocks one block_size-token span of a sequence takes (KV heads x
 * layers).  mux_sched_counts: counts[0..4] = waiting, running, finished, preemptions of
 * the model, blocks of quota moved so far (all models).
 * mux_sched_submit: prompt_len, output_len >= 1, prompt_len + output_len <= max_blocks x
 * block_size, and the blocks of prompt_len + output_len - 1 cached tokens must fit the whole
 * pool (a request that could never fit would be preempted for ever); else MUX_ERR_INVALID.
 * A request larger than its model's quota is accepted (quotas move) and waits.
 * Not thread-safe: one caller at a time.
 * ------------------------------------------------------------------------------- */
typedef struct mux_sched mux_sched_t;
typedef struct mux_sched_config {
    int32_t n_models;
    const int32_t *heads;        /* HOST array of n_models; copied */
    int32_t max_seqs;            /* sequence slots (table rows) per model */
    int32_t max_blocks;          /* table columns: blocks per (sequence, head) */
    int32_t max_prefill_tokens;  /* token budget of one prefill job */
    int32_t adapt_period;        /* iterations between quota adaptations, 0 = never */
    double low_util, high_util, step_fraction;
} mux_sched_config;
enum { MUX_JOB_PREFILL = 1, MUX_JOB_DECODE = 2, MUX_JOB_PREEMPT = 3 };
enum { MUX_JOB_FLAG_TABLE = 1, MUX_JOB_FLAG_FINISHED = 2 };
MUX_API int mux_sched_create(mux_sched_t **out, mux_pool_t *pool, const mux_sched_config *cfg);
MUX_API int mux_sched_destroy(mux_sched_t *sched);
MUX_API int mux_sched_submit(mux_sched_t *sched, int32_t model, int64_t request_id, int32_t prompt_len,
                             int32_t output_len);
MUX_API int mux_sched_step(mux_sched_t *sched, int32_t *n_jobs);
MUX_API int mux_sched_job(const mux_sched_t *sched, int32_t job, int32_t *kind, int32_t *model, int32_t *n_seqs);
MUX_API int mux_sched_job_seqs(const mux_sched_t *sched, int32_t job, int64_t *request_ids, int32_t *slots,
                               int32_t *lens, int32_t *flags);
MUX_API const int32_t *mux_sched_table(const mux_sched_t *sched, int32_t model);
MUX_API int mux_sched_counts(const mux_sched_t *sched, int32_t model, int64_t *counts);

/* ---------------------------------------------------------------------------------
 * Job runner (Section 3.3, Algorithm 3 `execute`; Section 3.4: the engines fill K/V into the
 * blocks the manager assigned and run attention over them).  It launches the jobs of a
 * scheduler on the GPU: a decode job's integer arrays (context lengths, new block ids) ride
 * in the arguments of its one attention launch when they fit; any other job writes them into
 * pinned memory the runner owns, from where ONE small kernel installs the block ids the
 * scheduler just handed out into the runner's device copy of the model's table and copies the
 * per-token arrays to device memory (no host-to-device copy call), then the append and the
 * attention follow on the model's stream.  Unlike the calls above the runner OWNS device memory
 * (table copies, staging areas, kernel workspaces: allocated in mux_runner_create on the
 * current device, freed in mux_runner_destroy); launches allocate nothing.
 *
 * mux_runner_create: `sched` must have been created over `pool` and both must outlive the
 *   runner (destroy the runner first).  n_q_heads: HOST array per model, query heads of ONE
 *   layer.  n_layers: HOST array per model, or NULL for one layer each; the scheduler's
 *   `heads` of the model must be n_layers x (KV heads of a layer), its head index being
 *   layer x KV heads + head, and n_q_heads a multiple of the KV heads of a layer.  streams:
 *   HOST array of hipStream_t per model (NULL = all on the default stream); models may share
 *   a stream.
 * mux_runner_step: mux_sched_step, plus the ordering the scheduler asks for: for every model
 *   whose blocks went back to the pool in this iteration, what was launched so far on that
 *   model's stream (the last readers of those blocks) is ordered, by an event and without a
 *   host wait, before what is launched next on the other models' streams.
 * mux_runner_launch: enqueues job `job` of the last step, for ALL layers of its model; returns
 *   without waiting.  With L = the model's layers:
 *   Prefill job of n requests with T tokens in total: k_new, v_new DEVICE [L][T][kv heads][d],
 *   q, out DEVICE [L][T][q heads][d], rows packed request by request in the job's order
 *   (positions 0 .. len-1 of each); one append + one attention launch per layer.
 *   Decode job: k_new, v_new DEVICE [L][R][kv heads][d], q, out DEVICE [L][R][q heads][d], row =
 *   the sequence's SLOT (the row of the scheduler's table); R = max_seqs, or for a model of one
 *   layer any number of rows above the job's highest slot.  Rows of slots outside the job are
 *   neither read nor appended; their out rows (up to the job's highest slot, all of them for
 *   L > 1) are zeroed.  One launch for all layers (mux_decode_step).
 *   Preempt jobs launch nothing.  The buffers must stay untouched until the work has finished
 *   on the model's stream.  Jobs of one step are launched in job order, each at most once.
 * mux_runner_launch_layer: the same for ONE layer of the job's model, for engines that run
 *   attention layer by layer between their other kernels: k_new, v_new, q, out are that
 *   layer's slices ([T] or [R] rows, shapes as above without the layer dimension).  Layer 0
 *   of a job comes first (it stages the job's arrays and installs its block ids); the other
 *   layers of the same job follow in any order, before layer 0 of the model's next job.
 *   A layer launched twice appends its rows twice (same bytes) and is otherwise harmless.
 * mux_runner_set_buffers / mux_runner_run_step: for engines that keep their Q/K/V/output in
 *   fixed buffers (shapes as for mux_runner_launch: the decode set for max_seqs rows; the
 *   prefill set large enough for the largest prefill job, max(max_prefill_tokens, max_blocks x
 *   block_size) tokens - the layer stride of a prefill buffer is the job's own T rows).  mux_runner_run_step = mux_runner_step followed by mux_runner_launch
 *   of every job with its model's registered buffers and scale: one call per iteration.
 *   A job of a model without registered buffers -> MUX_ERR_INVALID (jobs before it were
 *   launched).
 * mux_runner_counts: counts[0..1] = prefill and decode jobs launched so far, and the sequences in
 *   them (every sequence of such a job yields one output token).
 * mux_runner_synchronize: waits for every model's stream.
 * mux_runner_read_table: waits for the model's stream and copies the runner's device copy of
 *   the model's table to host_out (HOST int32 [layers][max_seqs][KV heads of a layer]
 *   [max_blocks]; entries the scheduler never handed out are 0).  For checks; not part of the
 *   serving loop.
 * Errors: MUX_ERR_INVALID (arguments), MUX_ERR_HIP (runtime), MUX_ERR_NOMEM (host memory).
 * Not thread-safe: one caller at a time, the same as the scheduler it drives.
 * ------------------------------------------------------------------------------- */
typedef struct mux_runner mux_runner_t;
MUX_API int mux_runner_create(mux_runner_t **out, mux_pool_t *pool, mux_sched_t *sched, const int32_t *n_q_heads,
                              const int32_t *n_layers, void *const *streams);
MUX_API int mux_runner_destroy(mux_runner_t *runner);
MUX_API int mux_runner_step(mux_runner_t *runner, int32_t *n_jobs);
MUX_API int mux_runner_launch(mux_runner_t *runner, int32_t job, void *out, const void *q, const void *k_new,
                              const void *v_new, float scale);
MUX_API int mux_runner_launch_layer(mux_runner_t *runner, int32_t job, int32_t layer, void *out, const void *q,
                                    const void *k_new, const void *v_new, float scale);
MUX_API int mux_runner_set_buffers(mux_runner_t *runner, int32_t model, void *prefill_out, const void *prefill_q,
                                   const void *prefill_k, const void *prefill_v, void *decode_out, const void *decode_q,
                                   const void *decode_k, const void *decode_v, float scale);
MUX_API int mux_runner_run_step(mux_runner_t *runner, int32_t *n_jobs);
MUX_API int mux_runner_counts(const mux_runner_t *runner, int64_t *counts);
MUX_API int mux_runner_synchronize(mux_runner_t *runner);
MUX_API int mux_runner_read_table(mux_runner_t *runner, int32_t model, int32_t *host_out);

/* ---------------------------------------------------------------------------------
 * Compute partitioning (Section 3.4: the parallel runtime assigns compute to prefill and
 * decoding jobs at SM granularity, with MPS percentages on the paper's hardware).  Here a
 * job's share is a HIP stream restricted to a set of compute units: every kernel enqueued
 * on it - through the calls above or otherwise - runs only on those units.
 *
 * mux_device_cu_count: *out = compute units of the current device.
 * mux_stream_create_masked: cu_mask = HOST array of n_words (1..64) 32-bit words, bit b of
 *   word w set = compute unit 32 w + b may be used (the runtime's numbering; bits beyond the
 *   device's units are ignored); at least one bit must be set.  *out_stream = a new
 *   hipStream_t at default priority, owned by the caller until mux_stream_destroy.
 * Errors: MUX_ERR_INVALID for bad arguments, MUX_ERR_HIP if the runtime refuses.
 * ------------------------------------------------------------------------------- */
MUX_API int mux_device_cu_count(int32_t *out);
MUX_API int mux_stream_create_masked(void **out_stream, const uint32_t *cu_mask, int32_t n_words);
MUX_API int mux_stream_destroy(void *stream);

/* ---------------------------------------------------------------------------------
 * Throughput estimator (Section 3.3, Eq. 3; Appendix A.2).  In a stable serving state the
 * prefill phases of the colocated LLMs run one after another and the decoding phases
 * overlap, so a batch of b^m requests of LLM m takes the sum of all LLMs' prefill
 * latencies plus its own decoding latency times its average generation length:
 *     tpt(m) = min( b^m / ( sum_i t_p^i + t_d^m * l_o^m ), W_b ).
 * mux_estimate_tpt: HOST arrays of n_models doubles: batch sizes b^i, prefill latency of
 *   each LLM's batch t_p^i (seconds), decoding latency per step t_d^i (seconds), average
 *   generation lengths l_o^i; m = the LLM asked about; rate_cap = W_b, the request rate the
 *   workload offers (requests/s).  LLMs with batch 0 contribute no prefill.  Returns
 *   requests/s, or NaN for bad arguments (null, negative or NaN entries, m out of range).
 * mux_find_batch_size: the paper finds, by binary search, the batch size that satisfies the
 *   traffic.  With profiled latencies fitted as t_p(b) = p0 + p1 b and t_d(b) = d0 + d1 b
 *   (seconds), generation length gen_len and the other LLMs' prefill time other_prefill,
 *   b / (other_prefill + t_p(b) + t_d(b) gen_len) (evaluated in fp64, in this order) never
 *   decreases with b; returns the
 *   smallest b in [1, max_batch] whose value reaches `rate`, 0 if even max_batch does not,
 *   MUX_ERR_INVALID for negative or NaN arguments or max_batch < 1.
 * ------------------------------------------------------------------------------- */
MUX_API double mux_estimate_tpt(int32_t n_models, const double *batch, const double *t_prefill, const double *t_decode,
                                const double *gen_len, int32_t m, double rate_cap);
MUX_API int64_t mux_find_batch_size(double rate, int64_t max_batch, double p0, double p1, double d0, double d1,
                                    double gen_len, double other_prefill);

/* Human-readable name of a status code (static storage). */
MUX_API const char *mux_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* MUX_H */
