// C entry points of the library: the unified KV space's block manager (host only) and
// argument checking in front of the three kernel launchers.
//
// MuxServe, Section 3.4 (Implementation): the memory manager is native code because block
// allocation sits on the serving path; engines request blocks, fill them, keep them across
// a request's prefill and decoding jobs and release them when the request finishes.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>

#include "mux_internal.h"

namespace {

bool shape_supported(int32_t block_size, int32_t head_dim, mux_dtype_t dtype)
{
    if (dtype != MUX_BF16 && dtype != MUX_FP32) return false;
    if (head_dim != 64 && head_dim != 128) return false;
    return block_size >= 1 && block_size <= 256;
}

bool heads_ok(int32_t n_q_heads, int32_t n_kv_heads)
{
    return n_q_heads > 0 && n_kv_heads > 0 && n_q_heads % n_kv_heads == 0;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

namespace {
bool model_in_range(int32_t m) { return m >= 0 && m < MUX_MAX_MODELS; }

// Deal `total` indivisible blocks out to `n` claimants: claimant i already has whole[i] and a
// remainder key[i] (larger = closer to one more block; negative = takes no part).  The blocks
// go one each to the largest keys, the lower index first among equals.
template <class Key>
void deal_leftovers(int64_t total, std::vector<int64_t> &whole, const std::vector<Key> &key)
{
    std::vector<int32_t> order;
    for (size_t i = 0; i < key.size(); ++i)
        if (!(key[i] < Key(0))) order.push_back(static_cast<int32_t>(i));
    if (order.empty()) return;
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return key[a] > key[b]; });
    for (size_t k = 0; total > 0; k = (k + 1) % order.size(), --total) whole[order[k]] += 1;
}
}  // namespace

extern "C" {

int mux_pool_create(mux_pool_t **out, void *kv_base, size_t kv_bytes, int64_t num_blocks, int32_t block_size,
                    int32_t head_dim, mux_dtype_t dtype, const int32_t *init_free_order)
{
    if (!out || !kv_base || num_blocks <= 0 || num_blocks > INT32_MAX || block_size <= 0 || head_dim <= 0)
        return MUX_ERR_INVALID;
    if (!shape_supported(block_size, head_dim, dtype)) return MUX_ERR_UNSUPPORTED;
    if (!aligned16(kv_base)) return MUX_ERR_INVALID;
    const int32_t elem = dtype == MUX_BF16 ? 2 : 4;
    const int64_t block_bytes = 2LL * block_size * head_dim * elem;
    if (static_cast<unsigned __int128>(block_bytes) * static_cast<unsigned __int128>(num_blocks) > kv_bytes)
        return MUX_ERR_INVALID;

    mux_pool *p = new (std::nothrow) mux_pool;
    if (!p) return MUX_ERR_INVALID;
    try {
        p->holder.assign(static_cast<size_t>(num_blocks), mux_pool::kFree);
        p->free_ids.resize(static_cast<size_t>(num_blocks));
        p->used_by_model.assign(MUX_MAX_MODELS, 0);
        p->quota_of_model.assign(MUX_MAX_MODELS, mux_pool::kNoQuota);
        p->peak_of_model.assign(MUX_MAX_MODELS, 0);
    } catch (const std::bad_alloc &) {
        delete p;
        return MUX_ERR_INVALID;
    }
    if (init_free_order) {
        // must name every id exactly once
        for (int64_t i = 0; i < num_blocks; ++i) {
            const int32_t id = init_free_order[i];
            if (id < 0 || id >= num_blocks || p->holder[id] == mux_pool::kPending) {
                delete p;
                return MUX_ERR_INVALID;
            }
            p->holder[id] = mux_pool::kPending;
        }
        std::fill(p->holder.begin(), p->holder.end(), mux_pool::kFree);
        // first id of the order must be popped first, so it goes to the back
        std::reverse_copy(init_free_order, init_free_order + num_blocks, p->free_ids.begin());
    } else {
        for (int64_t i = 0; i < num_blocks; ++i) p->free_ids[static_cast<size_t>(i)] = static_cast<int32_t>(num_blocks - 1 - i);
    }
    p->kv_base = static_cast<char *>(kv_base);
    p->num_blocks = num_blocks;
    p->block_size = block_size;
    p->head_dim = head_dim;
    p->dtype = dtype;
    p->elem_bytes = elem;
    p->block_bytes = block_bytes;
    *out = p;
    return MUX_OK;
}

int mux_pool_destroy(mux_pool_t *pool)
{
    if (!pool) return MUX_ERR_INVALID;
    delete pool;
    return MUX_OK;
}

int64_t mux_pool_num_free(const mux_pool_t *pool)
{
    if (!pool) return MUX_ERR_INVALID;
    std::lock_guard<std::mutex> g(pool->lock);
    return static_cast<int64_t>(pool->free_ids.size());
}

int64_t mux_pool_num_used(const mux_pool_t *pool, int32_t model_id)
{
    if (!pool || model_id < 0 || model_id >= MUX_MAX_MODELS) return MUX_ERR_INVALID;
    std::lock_guard<std::mutex> g(pool->lock);
    return pool->used_by_model[model_id];
}

int64_t mux_pool_block_bytes(const mux_pool_t *pool) { return pool ? pool->block_bytes : MUX_ERR_INVALID; }

int mux_alloc_blocks(mux_pool_t *pool, int32_t model_id, int64_t n, int32_t *out_ids)
{
    if (!pool || model_id < 0 || model_id >= MUX_MAX_MODELS || n < 0) return MUX_ERR_INVALID;
    if (n == 0) return MUX_OK;
    if (!out_ids) return MUX_ERR_INVALID;
    std::lock_guard<std::mutex> g(pool->lock);
    const int64_t cap = pool->quota_of_model[model_id];
    if (cap != mux_pool::kNoQuota && n > cap - pool->used_by_model[model_id]) return MUX_ERR_QUOTA;
    const size_t have = pool->free_ids.size();
    if (static_cast<uint64_t>(n) > have) return MUX_ERR_NOMEM;
    const int32_t *top = pool->free_ids.data() + have;  // one past the id popped first
    int32_t *holder = pool->holder.data();
    for (int64_t i = 0; i < n; ++i) {
        const int32_t id = *--top;
        holder[id] = model_id;
        out_ids[i] = id;
    }
    pool->free_ids.resize(have - static_cast<size_t>(n));
    const int64_t now = (pool->used_by_model[model_id] += n);
    pool->peak_of_model[model_id] = std::max(pool->peak_of_model[model_id], now);
    return MUX_OK;
}

int mux_free_blocks(mux_pool_t *pool, int32_t model_id, int64_t n, const int32_t *ids)
{
    if (!pool || model_id < 0 || model_id >= MUX_MAX_MODELS || n < 0) return MUX_ERR_INVALID;
    if (n == 0) return MUX_OK;
    if (!ids) return MUX_ERR_INVALID;
    std::lock_guard<std::mutex> g(pool->lock);
    int32_t *holder = pool->holder.data();
    // Pass 1 tags each id; a tag already present means the id was named twice.
    int64_t tagged = 0;
    for (; tagged < n; ++tagged) {
        const int32_t id = ids[tagged];
        if (id < 0 || id >= pool->num_blocks || holder[id] != model_id) break;
        holder[id] = mux_pool::kPending;
    }
    if (tagged != n) {
        for (int64_t i = 0; i < tagged; ++i) holder[ids[i]] = model_id;
        return MUX_ERR_INVALID;
    }
    for (int64_t i = 0; i < n; ++i) holder[ids[i]] = mux_pool::kFree;
    pool->free_ids.insert(pool->free_ids.end(), ids, ids + n);
    pool->used_by_model[model_id] -= n;
    return MUX_OK;
}

int mux_pool_set_quota(mux_pool_t *pool, int32_t model_id, int64_t max_blocks)
{
    if (!pool || !model_in_range(model_id)) return MUX_ERR_INVALID;
    if (max_blocks != mux_pool::kNoQuota && (max_blocks < 0 || max_blocks > pool->num_blocks)) return MUX_ERR_INVALID;
    std::lock_guard<std::mutex> g(pool->lock);
    pool->quota_of_model[model_id] = max_blocks;
    return MUX_OK;
}

int mux_pool_get_quota(const mux_pool_t *pool, int32_t model_id, int64_t *out)
{
    if (!pool || !model_in_range(model_id) || !out) return MUX_ERR_INVALID;
    std::lock_guard<std::mutex> g(pool->lock);
    *out = pool->quota_of_model[model_id];
    return MUX_OK;
}

int mux_pool_peak_used(const mux_pool_t *pool, int32_t model_id, int64_t *out)
{
    if (!pool || !model_in_range(model_id) || !out) return MUX_ERR_INVALID;
    std::lock_guard<std::mutex> g(pool->lock);
    *out = pool->peak_of_model[model_id];
    return MUX_OK;
}

int mux_pool_init_quotas(mux_pool_t *pool, int32_t n_models, const double *weights)
{
    if (!pool || n_models <= 0 || n_models > MUX_MAX_MODELS || !weights) return MUX_ERR_INVALID;
    double sum = 0.0;
    for (int32_t m = 0; m < n_models; ++m) {
        if (!std::isfinite(weights[m]) || weights[m] < 0.0) return MUX_ERR_INVALID;
        sum += weights[m];
    }
    if (!std::isfinite(sum) || !(sum > 0.0)) return MUX_ERR_INVALID;
    std::vector<int64_t> whole(static_cast<size_t>(n_models));
    std::vector<double> part(static_cast<size_t>(n_models));
    int64_t dealt = 0;
    for (int32_t m = 0; m < n_models; ++m) {
        const double share = static_cast<double>(pool->num_blocks) * weights[m] / sum;
        const double fl = std::floor(share);
        whole[m] = static_cast<int64_t>(fl);
        part[m] = share - fl;
        dealt += whole[m];
    }
    deal_leftovers(pool->num_blocks - dealt, whole, part);
    std::lock_guard<std::mutex> g(pool->lock);
    std::copy(whole.begin(), whole.end(), pool->quota_of_model.begin());
    return MUX_OK;
}

int mux_pool_adapt_quotas(mux_pool_t *pool, int32_t n_models, double low, double high, double step, int64_t *moved)
{
    if (!pool || n_models <= 0 || n_models > MUX_MAX_MODELS) return MUX_ERR_INVALID;
    if (!(low >= 0.0) || !(high >= low) || !std::isfinite(high) || !(step >= 0.0) || !(step <= 1.0))
        return MUX_ERR_INVALID;
    std::lock_guard<std::mutex> g(pool->lock);
    const size_t n = static_cast<size_t>(n_models);
    for (size_t m = 0; m < n; ++m)
        if (pool->quota_of_model[m] == mux_pool::kNoQuota) return MUX_ERR_INVALID;
    // who gives how much, and who takes with which weight
    std::vector<int64_t> gives(n, 0), gets(n, 0), rest(n, -1);
    int64_t collected = 0, demand = 0;
    for (size_t m = 0; m < n; ++m) {
        const double quota = static_cast<double>(pool->quota_of_model[m]);
        const double peak = static_cast<double>(pool->peak_of_model[m]);
        if (peak < low * quota) {
            gives[m] = static_cast<int64_t>(std::floor(step * (quota - peak)));
            collected += gives[m];
        } else if (pool->peak_of_model[m] > 0 && peak >= high * quota) {
            demand += pool->peak_of_model[m];
            rest[m] = 0;   // marks a taker until its remainder is known
        }
    }
    int64_t total = 0;
    if (collected > 0 && demand > 0) {
        int64_t dealt = 0;
        for (size_t m = 0; m < n; ++m) {
            if (rest[m] < 0) continue;
            const int64_t scaled = collected * pool->peak_of_model[m];   // < 2^62: both factors fit 31 bits
            gets[m] = scaled / demand;
            rest[m] = scaled % demand;
            dealt += gets[m];
        }
        deal_leftovers(collected - dealt, gets, rest);
        for (size_t m = 0; m < n; ++m) pool->quota_of_model[m] += gets[m] - gives[m];
        total = collected;
    }
    for (size_t m = 0; m < n; ++m) pool->peak_of_model[m] = pool->used_by_model[m];
    if (moved) *moved = total;
    return MUX_OK;
}

int mux_kv_append(mux_pool_t *pool, const void *k_new, const void *v_new, const int32_t *tok_seq,
                  const int32_t *tok_pos, const int32_t *block_tables, int32_t n_tokens, int32_t n_seqs,
                  int32_t n_kv_heads, int32_t max_blocks, void *stream)
{
    if (!pool || n_tokens < 0 || n_seqs < 0 || n_kv_heads <= 0 || max_blocks < 0) return MUX_ERR_INVALID;
    if (n_tokens == 0) return MUX_OK;
    if (!k_new || !v_new || !tok_seq || !tok_pos || !block_tables || n_seqs == 0 || max_blocks == 0)
        return MUX_ERR_INVALID;
    if (!aligned16(k_new) || !aligned16(v_new)) return MUX_ERR_INVALID;
    return mux_launch_kv_append(pool, k_new, v_new, tok_seq, tok_pos, block_tables, n_tokens, n_seqs, n_kv_heads,
                                max_blocks, stream);
}

size_t mux_decode_workspace_bytes(const mux_pool_t *pool, int32_t n_seqs, int32_t n_q_heads, int32_t n_kv_heads,
                                  int32_t max_ctx_len)
{
    if (!pool || n_seqs <= 0 || !heads_ok(n_q_heads, n_kv_heads) || max_ctx_len <= 0) return 0;
    return mux_plan_decode(pool, n_seqs, n_q_heads, n_kv_heads, max_ctx_len).workspace_bytes;
}

size_t mux_decode_workspace_bound(const mux_pool_t *pool, int32_t max_seqs, int32_t n_q_heads, int32_t n_kv_heads,
                                  int32_t max_ctx_len)
{
    if (!pool || max_seqs <= 0 || !heads_ok(n_q_heads, n_kv_heads) || max_ctx_len <= 0) return 0;
    return mux_decode_workspace_upper_bound(pool, max_seqs, n_q_heads, n_kv_heads, max_ctx_len);
}

int mux_decode_attn(mux_pool_t *pool, void *out, const void *q, const int32_t *block_tables,
                    const int32_t *ctx_lens, int32_t n_seqs, int32_t n_q_heads, int32_t n_kv_heads,
                    int32_t max_blocks, int32_t max_ctx_len, float scale, void *workspace, size_t workspace_bytes,
                    void *stream)
{
    if (!pool || n_seqs < 0 || !heads_ok(n_q_heads, n_kv_heads) || max_blocks < 0 || max_ctx_len < 0)
        return MUX_ERR_INVALID;
    if (n_seqs == 0) return MUX_OK;
    if (!out || !q || !block_tables || !ctx_lens || !aligned16(out) || !aligned16(q)) return MUX_ERR_INVALID;
    // the grid never looks past the table: clamp the hint to what the table can describe
    const int64_t table_tokens = static_cast<int64_t>(max_blocks) * pool->block_size;
    if (max_ctx_len > table_tokens) return MUX_ERR_INVALID;
    const mux_decode_plan plan = mux_plan_decode(pool, n_seqs, n_q_heads, n_kv_heads, std::max(max_ctx_len, 1));
    if (plan.workspace_bytes > 0) {
        if (!workspace || workspace_bytes < plan.workspace_bytes || !aligned16(workspace)) return MUX_ERR_INVALID;
    }
    return mux_launch_decode_attn(pool, plan, out, q, block_tables, ctx_lens, n_seqs, n_q_heads, n_kv_heads,
                                  max_blocks, max_ctx_len, scale, workspace, stream);
}

size_t mux_decode_step_workspace_bytes(const mux_pool_t *pool, int32_t n_layers, int32_t n_seqs, int32_t n_q_heads,
                                       int32_t n_kv_heads, int32_t max_ctx_len)
{
    if (!pool || n_layers <= 0 || n_seqs <= 0 || !heads_ok(n_q_heads, n_kv_heads) || max_ctx_len <= 0) return 0;
    if (static_cast<int64_t>(n_layers) * n_seqs > INT32_MAX) return 0;
    return mux_plan_decode(pool, n_layers * n_seqs, n_q_heads, n_kv_heads, max_ctx_len).workspace_bytes;
}

int mux_decode_step(mux_pool_t *pool, void *out, const void *q, const void *k_new, const void *v_new,
                    const int32_t *block_tables, const int32_t *ctx_lens, int32_t n_layers, int32_t n_seqs,
                    int32_t n_q_heads, int32_t n_kv_heads, int32_t max_blocks, int32_t max_ctx_len, float scale,
                    void *workspace, size_t workspace_bytes, void *stream)
{
    if (!pool || n_layers < 0 || n_seqs < 0 || !heads_ok(n_q_heads, n_kv_heads) || max_blocks < 0 || max_ctx_len < 0)
        return MUX_ERR_INVALID;
    if (n_layers == 0 || n_seqs == 0) return MUX_OK;
    if (static_cast<int64_t>(n_layers) * n_seqs > INT32_MAX) return MUX_ERR_UNSUPPORTED;
    if (!out || !q || !k_new || !v_new || !block_tables || !ctx_lens) return MUX_ERR_INVALID;
    if (!aligned16(out) || !aligned16(q) || !aligned16(k_new) || !aligned16(v_new)) return MUX_ERR_INVALID;
    if (max_ctx_len > static_cast<int64_t>(max_blocks) * pool->block_size) return MUX_ERR_INVALID;
    const mux_decode_plan plan = mux_plan_decode(pool, n_layers * n_seqs, n_q_heads, n_kv_heads, std::max(max_ctx_len, 1));
    if (plan.workspace_bytes > 0) {
        if (!workspace || workspace_bytes < plan.workspace_bytes || !aligned16(workspace)) return MUX_ERR_INVALID;
    }
    return mux_launch_decode_step(pool, plan, out, q, k_new, v_new, block_tables, ctx_lens, n_layers, n_seqs, n_q_heads,
                                  n_kv_heads, max_blocks, max_ctx_len, scale, workspace, stream);
}

size_t mux_prefill_workspace_bytes(const mux_pool_t *pool, int32_t n_seqs, int32_t total_q, int32_t max_ctx_len,
                                   int32_t n_q_heads, int32_t n_kv_heads)
{
    if (!pool || n_seqs <= 0 || total_q <= 0 || max_ctx_len <= 0 || !heads_ok(n_q_heads, n_kv_heads)) return 0;
    if (mux_prefill_uses_mfma(pool)) return 0;
    return mux_plan_decode(pool, total_q, n_q_heads, n_kv_heads, max_ctx_len).workspace_bytes;
}

size_t mux_prefill_workspace_bound(const mux_pool_t *pool, int32_t max_total_q, int32_t max_ctx_len, int32_t n_q_heads,
                                   int32_t n_kv_heads)
{
    if (!pool || max_total_q <= 0 || max_ctx_len <= 0 || !heads_ok(n_q_heads, n_kv_heads)) return 0;
    if (mux_prefill_uses_mfma(pool)) return 0;
    return mux_decode_workspace_upper_bound(pool, max_total_q, n_q_heads, n_kv_heads, max_ctx_len);
}

int mux_prefill_attn(mux_pool_t *pool, void *out, const void *q, const int32_t *cu_q_lens, const int32_t *q_start,
                     const int32_t *block_tables, int32_t n_seqs, int32_t total_q, int32_t max_q_len,
                     int32_t max_ctx_len, int32_t n_q_heads, int32_t n_kv_heads, int32_t max_blocks, float scale,
                     void *workspace, size_t workspace_bytes, void *stream)
{
    if (!pool || n_seqs < 0 || total_q < 0 || max_q_len < 0 || max_ctx_len < 0 || !heads_ok(n_q_heads, n_kv_heads) ||
        max_blocks < 0)
        return MUX_ERR_INVALID;
    if (n_seqs == 0 || total_q == 0 || max_q_len == 0) return MUX_OK;
    if (!out || !q || !cu_q_lens || !q_start || !block_tables || !aligned16(out) || !aligned16(q)) return MUX_ERR_INVALID;
    if (max_q_len > max_ctx_len || max_ctx_len > static_cast<int64_t>(max_blocks) * pool->block_size)
        return MUX_ERR_INVALID;
    const size_t need = mux_prefill_workspace_bytes(pool, n_seqs, total_q, max_ctx_len, n_q_heads, n_kv_heads);
    if (need > 0 && (!workspace || workspace_bytes < need || !aligned16(workspace))) return MUX_ERR_INVALID;
    return mux_launch_prefill_attn(pool, out, q, cu_q_lens, q_start, block_tables, n_seqs, total_q, max_q_len,
                                   max_ctx_len, n_q_heads, n_kv_heads, max_blocks, scale, workspace, stream);
}

const char *mux_status_string(int status)
{
    switch (status) {
        case MUX_OK: return "MUX_OK";
        case MUX_ERR_INVALID: return "MUX_ERR_INVALID";
        case MUX_ERR_NOMEM: return "MUX_ERR_NOMEM";
        case MUX_ERR_QUOTA: return "MUX_ERR_QUOTA";
        case MUX_ERR_HIP: return "MUX_ERR_HIP";
        case MUX_ERR_UNSUPPORTED: return "MUX_ERR_UNSUPPORTED";
        case MUX_ERR_TOO_LARGE: return "MUX_ERR_TOO_LARGE";
        default: return "MUX_ERR_UNKNOWN";
    }
}

}  // extern "C"
