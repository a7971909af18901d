// Internal definitions shared by the translation units of the library (not part of the ABI).
#pragma once
#include <cstddef>
#include <cstdint>
#include <mutex>
#include <vector>

#include "mux.h"

struct mux_pool {
    // geometry of the unified KV space
    char *kv_base = nullptr;      // device memory, caller-owned
    int64_t num_blocks = 0;
    int32_t block_size = 0;       // tokens per block
    int32_t head_dim = 0;
    mux_dtype_t dtype = MUX_BF16;
    int32_t elem_bytes = 2;
    int64_t block_bytes = 0;      // 2 * block_size * head_dim * elem_bytes (K tile then V tile)

    // block manager state, guarded by `lock`
    mutable std::mutex lock;
    std::vector<int32_t> free_ids;          // LIFO: back() is handed out next
    std::vector<int32_t> holder;            // per block: model id, kFree, or kPending during a free call
    std::vector<int64_t> used_by_model;     // MUX_MAX_MODELS counters
    std::vector<int64_t> quota_of_model;    // cap on used_by_model, kNoQuota = none
    std::vector<int64_t> peak_of_model;     // high-water mark of used_by_model since the last quota adaptation

    static constexpr int32_t kFree = -1;
    static constexpr int32_t kPending = -2;
    static constexpr int64_t kNoQuota = -1;
};

// Kernel launchers (defined in the .hip files).  They validate nothing; the C entry
// points in mux_api.cpp check every host-visible argument first.
int mux_launch_kv_append(const mux_pool *pool, const void *k_new, const void *v_new, const int32_t *tok_seq,
                         const int32_t *tok_pos, const int32_t *tables, int32_t n_tokens, int32_t n_seqs,
                         int32_t n_kv_heads, int32_t max_blocks, void *stream);

struct mux_decode_plan {
    int32_t span_tokens;   // tokens of one sequence handled by one workgroup
    int32_t n_splits;      // ceil(max_ctx_len / span_tokens)
    int32_t heads_per_pass;  // query heads of one KV group handled together by a workgroup
    int32_t n_passes;        // ceil(group / heads_per_pass)
    size_t plan_bytes;       // work list at the start of the workspace (16-byte multiple)
    size_t workspace_bytes;  // plan_bytes + fp32 partial results of the spans (when n_splits > 1)
};
mux_decode_plan mux_plan_decode(const mux_pool *pool, int32_t n_seqs, int32_t n_q_heads, int32_t n_kv_heads,
                                int32_t max_ctx_len);
size_t mux_decode_workspace_upper_bound(const mux_pool *pool, int32_t max_rows, int32_t n_q_heads, int32_t n_kv_heads,
                                        int32_t max_ctx_len);
int mux_launch_decode_attn(const mux_pool *pool, const mux_decode_plan &plan, void *out, const void *q,
                           const int32_t *tables, const int32_t *ctx_lens, int32_t n_seqs, int32_t n_q_heads,
                           int32_t n_kv_heads, int32_t max_blocks, int32_t max_ctx_len, float scale,
                           void *workspace, void *stream);

// A decode step's small integer arrays handed over as kernel arguments instead of device memory
// (the job runner's usual decode job): v = HOST [rows] context length per table row (0 = not in
// this step), then [rows] index of the row's entry or -1, then per entry `heads` block ids - the
// block the row's new token has just opened, for every kv head of every layer of the model.
// head0: where the launch's first layer starts among them.  The attention kernel reads the
// lengths and those ids from its arguments and stores the ids in the device table for later steps.
// Precondition: no context length exceeds the launch's max_ctx_len.
#define MUX_INLINE_STEP_INTS 960   // 3 840 bytes: with the other arguments under the 4 KiB argument limit
struct mux_inline_step {
    const int32_t *v;
    int32_t rows, n_entries, heads, head0;
};
// ctx_lens may be null when inl is given (it is not read then).
int mux_launch_decode_step(const mux_pool *pool, const mux_decode_plan &plan, void *out, const void *q, const void *k_new,
                           const void *v_new, const int32_t *tables, const int32_t *ctx_lens, int32_t n_layers,
                           int32_t n_seqs, int32_t n_q_heads, int32_t n_kv_heads, int32_t max_blocks, int32_t max_ctx_len,
                           float scale, void *workspace, void *stream, const mux_inline_step *inl = nullptr);

int mux_launch_prefill_attn(const mux_pool *pool, void *out, const void *q, const int32_t *cu_q_lens,
                            const int32_t *q_start, const int32_t *tables, int32_t n_seqs, int32_t total_q,
                            int32_t max_q_len, int32_t max_ctx_len, int32_t n_q_heads, int32_t n_kv_heads,
                            int32_t max_blocks, float scale, void *workspace, void *stream);
bool mux_prefill_uses_mfma(const mux_pool *pool);

// Scheduler internals the job runner needs (defined in mux_sched.cpp).
struct mux_sched;
struct mux_runner;
mux_pool *mux_sched_pool(const mux_sched *s);
void mux_sched_geometry(const mux_sched *s, int32_t *n_models, int32_t *max_seqs, int32_t *max_blocks, int32_t *max_prefill_tokens);
int32_t mux_sched_heads(const mux_sched *s, int32_t model);
bool mux_sched_released_blocks(const mux_sched *s, int32_t model);   // the last mux_sched_step gave blocks of this model back to the pool
