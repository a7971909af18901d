/*
 * CPU oracle for the head-wise paged KV-cache path of MuxServe (arXiv 2404.02015).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU
 * library is checked against.  It shares no code with the GPU library and nothing
 * in the product path may call it; only the tests, the smoke check and the
 * benchmark's cpu_baseline leg do.
 *
 * What it follows:
 *   - Section 3.4 "Resource Manager": the KV cache is cut into small blocks, each
 *     block holds the K/V of ONE head for several tokens, and one space serves all
 *     colocated LLMs.
 *   - "Implementation" paragraph closing Section 3.4: an engine asks the memory manager
 *     for new blocks, fills K/V into the assigned blocks, the blocks stay with the
 *     request until it finishes and are released then.
 *   - Section 2.1: prefill handles all prompt tokens in parallel, decoding one
 *     token at a time on top of the cached K/V of every earlier token.  The
 *     attention itself is the Transformer's scaled dot-product attention, which
 *     the paper cites and does not restate; the head-wise paging is a memory
 *     layout, so the result it must reach is the textbook one.
 *
 * Where the paper is silent (block layout, free-list policy, scale, grouped-query mapping,
 * causal offset, ...) each function below states the reading it uses.
 *
 * Arithmetic: K/V/Q are widened to fp32 (bf16 -> fp32 is exact), scores, softmax
 * and the weighted sum are computed in fp32 in index order.  A second build of
 * the same attention row in fp64 (suffix _f64) exists so tests can bound the fp32
 * rounding of the oracle itself.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_INVALID (-1)
#define ORACLE_ERR_NOMEM (-2)
#define ORACLE_ERR_QUOTA (-3)
#define ORACLE_ERR_UNSUPPORTED (-5)

#define ORACLE_BF16 0
#define ORACLE_FP32 1
#define ORACLE_MAX_MODELS 1024

typedef struct oracle_pool {
    int64_t num_blocks;
    int32_t block_size; /* tokens per block */
    int32_t head_dim;
    int32_t dtype;
    size_t esize;        /* bytes per element */
    int32_t *free_stack; /* free_stack[n_free-1] is handed out next */
    int64_t n_free;
    int32_t *owner;      /* -1 = free, else the model that holds the block */
    int64_t used[ORACLE_MAX_MODELS];
    int64_t quota[ORACLE_MAX_MODELS]; /* cap on used[m]; -1 = none (Section 3.3: token block quota) */
    int64_t peak[ORACLE_MAX_MODELS];  /* largest used[m] since the last quota adaptation */
    uint8_t **tile;      /* tile[id] = K rows [block_size][head_dim], then V rows; NULL until written */
} oracle_pool;

/* ------------------------------------------------------------------------- */
/* Pool and block manager (the memory manager of Section 3.4, Implementation). */
/* Policy (the paper gives none): a LIFO stack.  A fresh pool hands out        */
/* order[0], order[1], ... (identity if order is NULL).  free() pushes ids in  */
/* the order given, so the last id freed is the first one handed out again.    */
/* ------------------------------------------------------------------------- */

int oracle_pool_create(oracle_pool **out, int64_t num_blocks, int32_t block_size, int32_t head_dim,
                       int32_t dtype, const int32_t *init_free_order)
{
    if (!out || num_blocks <= 0 || num_blocks > 0x7fffffffLL || block_size <= 0 || head_dim <= 0)
        return ORACLE_ERR_INVALID;
    if (dtype != ORACLE_BF16 && dtype != ORACLE_FP32) return ORACLE_ERR_UNSUPPORTED;
    oracle_pool *p = (oracle_pool *)calloc(1, sizeof(*p));
    if (!p) return ORACLE_ERR_INVALID;
    p->num_blocks = num_blocks;
    p->block_size = block_size;
    p->head_dim = head_dim;
    p->dtype = dtype;
    p->esize = dtype == ORACLE_BF16 ? 2 : 4;
    p->free_stack = (int32_t *)malloc(sizeof(int32_t) * (size_t)num_blocks);
    p->owner = (int32_t *)malloc(sizeof(int32_t) * (size_t)num_blocks);
    p->tile = (uint8_t **)calloc((size_t)num_blocks, sizeof(uint8_t *));
    if (!p->free_stack || !p->owner || !p->tile) return ORACLE_ERR_INVALID;
    for (int64_t i = 0; i < num_blocks; ++i) p->owner[i] = -1;
    for (int m = 0; m < ORACLE_MAX_MODELS; ++m) p->quota[m] = -1;
    if (init_free_order) {
        /* must be a permutation of [0, num_blocks) */
        for (int64_t i = 0; i < num_blocks; ++i) {
            int32_t id = init_free_order[i];
            if (id < 0 || id >= num_blocks || p->owner[id] != -1) {
                free(p->free_stack); free(p->owner); free(p->tile); free(p);
                return ORACLE_ERR_INVALID;
            }
            p->owner[id] = -2; /* seen */
        }
        for (int64_t i = 0; i < num_blocks; ++i) p->owner[i] = -1;
    }
    for (int64_t i = 0; i < num_blocks; ++i) {
        int32_t id = init_free_order ? init_free_order[i] : (int32_t)i;
        p->free_stack[num_blocks - 1 - i] = id; /* order[0] ends up on top */
    }
    p->n_free = num_blocks;
    *out = p;
    return ORACLE_OK;
}

void oracle_pool_destroy(oracle_pool *p)
{
    if (!p) return;
    for (int64_t i = 0; i < p->num_blocks; ++i) free(p->tile[i]);
    free(p->tile);
    free(p->owner);
    free(p->free_stack);
    free(p);
}

int64_t oracle_pool_num_free(const oracle_pool *p) { return p ? p->n_free : ORACLE_ERR_INVALID; }
int64_t oracle_pool_num_blocks(const oracle_pool *p) { return p ? p->num_blocks : ORACLE_ERR_INVALID; }

int64_t oracle_pool_num_used(const oracle_pool *p, int32_t model_id)
{
    if (!p || model_id < 0 || model_id >= ORACLE_MAX_MODELS) return ORACLE_ERR_INVALID;
    return p->used[model_id];
}

/* All-or-nothing: with fewer than n free blocks nothing changes and out_ids is untouched. */
int oracle_alloc_blocks(oracle_pool *p, int32_t model_id, int64_t n, int32_t *out_ids)
{
    if (!p || model_id < 0 || model_id >= ORACLE_MAX_MODELS || n < 0) return ORACLE_ERR_INVALID;
    if (n == 0) return ORACLE_OK;
    if (!out_ids) return ORACLE_ERR_INVALID;
    /* the model's own quota is looked at first: a request beyond it is refused whatever the pool holds */
    if (p->quota[model_id] >= 0 && p->used[model_id] + n > p->quota[model_id]) return ORACLE_ERR_QUOTA;
    if (n > p->n_free) return ORACLE_ERR_NOMEM;
    for (int64_t i = 0; i < n; ++i) {
        int32_t id = p->free_stack[--p->n_free];
        p->owner[id] = model_id;
        out_ids[i] = id;
    }
    p->used[model_id] += n;
    if (p->used[model_id] > p->peak[model_id]) p->peak[model_id] = p->used[model_id];
    return ORACLE_OK;
}

/* An id that is out of range, not held by model_id, or listed twice makes the whole
 * call fail with nothing changed. */
int oracle_free_blocks(oracle_pool *p, int32_t model_id, int64_t n, const int32_t *ids)
{
    if (!p || model_id < 0 || model_id >= ORACLE_MAX_MODELS || n < 0) return ORACLE_ERR_INVALID;
    if (n == 0) return ORACLE_OK;
    if (!ids) return ORACLE_ERR_INVALID;
    int64_t checked = 0;
    int bad = 0;
    for (; checked < n; ++checked) {
        int32_t id = ids[checked];
        if (id < 0 || id >= p->num_blocks || p->owner[id] != model_id) { bad = 1; break; }
        p->owner[id] = -3; /* marks "already named in this call" */
    }
    if (bad) {
        for (int64_t i = 0; i < checked; ++i) p->owner[ids[i]] = model_id;
        return ORACLE_ERR_INVALID;
    }
    for (int64_t i = 0; i < n; ++i) {
        p->owner[ids[i]] = -1;
        p->free_stack[p->n_free++] = ids[i];
    }
    p->used[model_id] -= n;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------- */
/* Token-block quotas (Section 3.3: every LLM of a unit gets a quota of token  */
/* blocks so that the shared cache is split fairly; Algorithm 3 initialises    */
/* the quotas, checks them before a job runs and adapts them periodically by   */
/* moving blocks from LLMs that use little of theirs to LLMs that use most).   */
/* The paper gives no formula; the rules below are this build's reading:       */
/*  - a quota caps the blocks a model holds; lowering it takes nothing back;   */
/*  - initial quotas split the pool in proportion to caller-given weights      */
/*    (request rate x blocks per token: usage normalised by rate is then equal)*/
/*    by the largest-remainder rule, ties to the lower model id;               */
/*  - utilisation of a model = peak blocks held since the last adaptation /    */
/*    quota; a model below `low` gives away floor(step x (quota - peak)); the  */
/*    blocks collected go to the models at or above `high` (and holding at     */
/*    least one block) in proportion to their peaks, largest remainder, ties   */
/*    to the lower id; without givers or takers nothing moves; peaks restart   */
/*    from the current usage.                                                  */
/* ------------------------------------------------------------------------- */

int oracle_set_quota(oracle_pool *p, int32_t model_id, int64_t max_blocks)
{
    if (!p || model_id < 0 || model_id >= ORACLE_MAX_MODELS) return ORACLE_ERR_INVALID;
    if (max_blocks < -1 || max_blocks > p->num_blocks) return ORACLE_ERR_INVALID;
    p->quota[model_id] = max_blocks;
    return ORACLE_OK;
}

int64_t oracle_get_quota(const oracle_pool *p, int32_t model_id)
{
    if (!p || model_id < 0 || model_id >= ORACLE_MAX_MODELS) return ORACLE_ERR_INVALID - 1; /* -2: not a quota value */
    return p->quota[model_id];
}

int64_t oracle_peak_used(const oracle_pool *p, int32_t model_id)
{
    if (!p || model_id < 0 || model_id >= ORACLE_MAX_MODELS) return ORACLE_ERR_INVALID;
    return p->peak[model_id];
}

int oracle_init_quotas(oracle_pool *p, int32_t n_models, const double *weights)
{
    if (!p || n_models <= 0 || n_models > ORACLE_MAX_MODELS || !weights) return ORACLE_ERR_INVALID;
    double total = 0.0;
    for (int m = 0; m < n_models; ++m) {
        if (!(weights[m] >= 0.0) || isinf(weights[m])) return ORACLE_ERR_INVALID;
        total += weights[m];
    }
    if (!(total > 0.0) || isinf(total)) return ORACLE_ERR_INVALID;
    double frac[ORACLE_MAX_MODELS];
    int64_t given = 0;
    for (int m = 0; m < n_models; ++m) {
        double share = (double)p->num_blocks * weights[m] / total;
        double whole = floor(share);
        p->quota[m] = (int64_t)whole;
        frac[m] = share - whole;
        given += p->quota[m];
    }
    /* the blocks left over go, one each, to the largest fractional parts (first one wins a tie) */
    for (int64_t left = p->num_blocks - given; left > 0; --left) {
        int best = -1;
        for (int m = 0; m < n_models; ++m)
            if (frac[m] >= 0.0 && (best < 0 || frac[m] > frac[best])) best = m;
        if (best < 0) { /* rounding left more blocks than models: start another round */
            for (int m = 0; m < n_models; ++m) frac[m] = 0.0;
            best = 0;
        }
        p->quota[best] += 1;
        frac[best] = -1.0;
    }
    return ORACLE_OK;
}

int oracle_adapt_quotas(oracle_pool *p, int32_t n_models, double low, double high, double step, int64_t *moved)
{
    if (!p || n_models <= 0 || n_models > ORACLE_MAX_MODELS) return ORACLE_ERR_INVALID;
    if (!(low >= 0.0) || !(high >= low) || isinf(high) || !(step >= 0.0) || !(step <= 1.0)) return ORACLE_ERR_INVALID;
    for (int m = 0; m < n_models; ++m)
        if (p->quota[m] < 0) return ORACLE_ERR_INVALID;
    int64_t give[ORACLE_MAX_MODELS], take_weight[ORACLE_MAX_MODELS];
    int64_t pot = 0, weight_sum = 0;
    for (int m = 0; m < n_models; ++m) {
        double q = (double)p->quota[m], pk = (double)p->peak[m];
        give[m] = 0;
        take_weight[m] = 0;
        if (pk < low * q) {
            give[m] = (int64_t)floor(step * (q - pk));
            pot += give[m];
        } else if (p->peak[m] > 0 && pk >= high * q) {
            take_weight[m] = p->peak[m];
            weight_sum += p->peak[m];
        }
    }
    int64_t total_moved = 0;
    if (pot > 0 && weight_sum > 0) {
        int64_t rest[ORACLE_MAX_MODELS];
        int64_t handed = 0;
        for (int m = 0; m < n_models; ++m) {
            p->quota[m] -= give[m];
            rest[m] = -1;
            if (take_weight[m] > 0) {
                int64_t part = pot * take_weight[m] / weight_sum;
                rest[m] = pot * take_weight[m] % weight_sum;
                p->quota[m] += part;
                handed += part;
            }
        }
        for (int64_t left = pot - handed; left > 0; --left) {
            int best = -1;
            for (int m = 0; m < n_models; ++m)
                if (rest[m] >= 0 && (best < 0 || rest[m] > rest[best])) best = m;
            p->quota[best] += 1;
            rest[best] = -1;
        }
        total_moved = pot;
    }
    for (int m = 0; m < n_models; ++m) p->peak[m] = p->used[m];
    if (moved) *moved = total_moved;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------- */
/* Logical append: the engine writes new K/V into the blocks it was given     */
/* (Section 3.4, Implementation).                                             */
/* token t of sequence s at position p, kv head h goes to row p % B of block   */
/* table[s][h][p / B]; bit patterns are copied unchanged.                      */
/* k_new, v_new: [n_tokens][n_kv_heads][head_dim] elements of the pool dtype.  */
/* ------------------------------------------------------------------------- */

static uint8_t *tile_of(oracle_pool *p, int32_t id, int create)
{
    if (!p->tile[id] && create) {
        size_t bytes = 2 * (size_t)p->block_size * (size_t)p->head_dim * p->esize;
        p->tile[id] = (uint8_t *)calloc(1, bytes);
    }
    return p->tile[id];
}

int oracle_kv_append(oracle_pool *p, const void *k_new, const void *v_new, const int32_t *tok_seq,
                     const int32_t *tok_pos, const int32_t *block_tables, int32_t n_tokens,
                     int32_t n_seqs, int32_t n_kv_heads, int32_t max_blocks)
{
    if (!p || n_tokens < 0 || n_seqs < 0 || n_kv_heads <= 0 || max_blocks < 0) return ORACLE_ERR_INVALID;
    const int B = p->block_size, d = p->head_dim;
    const size_t row = (size_t)d * p->esize;
    /* validate everything first so that a bad call changes nothing */
    for (int32_t t = 0; t < n_tokens; ++t) {
        int32_t s = tok_seq[t], pos = tok_pos[t];
        if (s < 0 || s >= n_seqs || pos < 0 || pos / B >= max_blocks) return ORACLE_ERR_INVALID;
        for (int32_t h = 0; h < n_kv_heads; ++h) {
            int32_t id = block_tables[((size_t)s * n_kv_heads + h) * max_blocks + pos / B];
            if (id < 0 || id >= p->num_blocks) return ORACLE_ERR_INVALID;
        }
    }
    for (int32_t t = 0; t < n_tokens; ++t) {
        int32_t s = tok_seq[t], pos = tok_pos[t];
        for (int32_t h = 0; h < n_kv_heads; ++h) {
            int32_t id = block_tables[((size_t)s * n_kv_heads + h) * max_blocks + pos / B];
            uint8_t *tile = tile_of(p, id, 1);
            if (!tile) return ORACLE_ERR_INVALID;
            const uint8_t *ksrc = (const uint8_t *)k_new + ((size_t)t * n_kv_heads + h) * row;
            const uint8_t *vsrc = (const uint8_t *)v_new + ((size_t)t * n_kv_heads + h) * row;
            memcpy(tile + (size_t)(pos % B) * row, ksrc, row);
            memcpy(tile + (size_t)B * row + (size_t)(pos % B) * row, vsrc, row);
        }
    }
    return ORACLE_OK;
}

/* Raw read-back of one logical row (for the scatter tests): which = 0 for K, 1 for V. */
int oracle_read_row(oracle_pool *p, int32_t block_id, int32_t slot, int32_t which, void *dst)
{
    if (!p || block_id < 0 || block_id >= p->num_blocks || slot < 0 || slot >= p->block_size) return ORACLE_ERR_INVALID;
    const size_t row = (size_t)p->head_dim * p->esize;
    uint8_t *tile = tile_of(p, block_id, 0);
    if (!tile) return ORACLE_ERR_INVALID; /* never written */
    memcpy(dst, tile + (which ? (size_t)p->block_size * row : 0) + (size_t)slot * row, row);
    return ORACLE_OK;
}

/* Drop the stored tiles of the listed blocks (streaming mode for very large pools). */
int oracle_drop_tiles(oracle_pool *p, int64_t n, const int32_t *ids)
{
    if (!p) return ORACLE_ERR_INVALID;
    for (int64_t i = 0; i < n; ++i) {
        if (ids[i] < 0 || ids[i] >= p->num_blocks) return ORACLE_ERR_INVALID;
        free(p->tile[ids[i]]);
        p->tile[ids[i]] = NULL;
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------- */
/* Gather: contiguous fp32 K and V [L][d] of one (sequence, kv head).          */
/* ------------------------------------------------------------------------- */

static float widen(const uint8_t *src, int dtype, size_t idx)
{
    if (dtype == ORACLE_BF16) {
        uint16_t b;
        memcpy(&b, src + 2 * idx, 2);
        uint32_t u = (uint32_t)b << 16; /* bf16 is the top half of an fp32 */
        float f;
        memcpy(&f, &u, 4);
        return f;
    }
    float f;
    memcpy(&f, src + 4 * idx, 4);
    return f;
}

/* table_row: the max_blocks ids of this (sequence, head).  Returns INVALID when a
 * needed block id is out of range or was never written. */
int oracle_gather(oracle_pool *p, const int32_t *table_row, int64_t L, float *K_out, float *V_out)
{
    if (!p || L < 0) return ORACLE_ERR_INVALID;
    const int B = p->block_size, d = p->head_dim;
    for (int64_t j = 0; j < L; ++j) {
        int32_t id = table_row[j / B];
        if (id < 0 || id >= p->num_blocks) return ORACLE_ERR_INVALID;
        const uint8_t *tile = tile_of(p, id, 0);
        if (!tile) return ORACLE_ERR_INVALID;
        const uint8_t *krow = tile + (size_t)(j % B) * d * p->esize;
        const uint8_t *vrow = krow + (size_t)B * d * p->esize;
        for (int c = 0; c < d; ++c) {
            K_out[j * d + c] = widen(krow, p->dtype, (size_t)c);
            V_out[j * d + c] = widen(vrow, p->dtype, (size_t)c);
        }
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------- */
/* One attention row over n keys: scaled dot-product attention as defined by   */
/* the Transformer.  x_j = scale * <q, K_j>, w_j = exp(x_j - max x),           */
/* o = sum_j w_j V_j / sum_j w_j.  n == 0 gives zeros.  weights (optional)      */
/* receives w_j / sum w.                                                        */
/* ------------------------------------------------------------------------- */

#define DEFINE_ATTN_ROW(NAME, REAL, EXPFN)                                                        \
    void NAME(const float *q, const float *K, const float *V, int64_t n, int32_t d, float scale, \
              float *out, REAL *weights, REAL *scratch)                                          \
    {                                                                                             \
        if (n <= 0) {                                                                             \
            for (int c = 0; c < d; ++c) out[c] = 0.0f;                                            \
            return;                                                                               \
        }                                                                                         \
        REAL *x = scratch; /* n entries */                                                        \
        REAL m = 0;                                                                               \
        for (int64_t j = 0; j < n; ++j) {                                                         \
            REAL dot = 0;                                                                         \
            for (int c = 0; c < d; ++c) dot += (REAL)q[c] * (REAL)K[j * d + c];                   \
            x[j] = (REAL)scale * dot;                                                             \
            if (j == 0 || x[j] > m) m = x[j];                                                     \
        }                                                                                         \
        REAL l = 0;                                                                               \
        for (int64_t j = 0; j < n; ++j) {                                                         \
            x[j] = EXPFN(x[j] - m);                                                               \
            l += x[j];                                                                            \
        }                                                                                         \
        for (int c = 0; c < d; ++c) {                                                             \
            REAL acc = 0;                                                                         \
            for (int64_t j = 0; j < n; ++j) acc += x[j] * (REAL)V[j * d + c];                     \
            out[c] = (float)(acc / l);                                                            \
        }                                                                                         \
        if (weights)                                                                              \
            for (int64_t j = 0; j < n; ++j) weights[j] = x[j] / l;                                \
    }

DEFINE_ATTN_ROW(oracle_attn_row_f32, float, expf)
DEFINE_ATTN_ROW(oracle_attn_row_f64, double, exp)

/* ------------------------------------------------------------------------- */
/* Batched decode: one query row per (sequence, q head), at position L_s - 1,  */
/* i.e. ctx_lens count the token appended this step.  kv head = q head / g,    */
/* g = n_q_heads / n_kv_heads.  q: [n_seqs][n_q_heads][d] in the pool dtype.   */
/* out: fp32 [n_seqs][n_q_heads][d].  use_f64 selects the fp64 row.            */
/* ------------------------------------------------------------------------- */

int oracle_decode_attn(oracle_pool *p, float *out, const void *q, const int32_t *block_tables,
                       const int32_t *ctx_lens, int32_t n_seqs, int32_t n_q_heads, int32_t n_kv_heads,
                       int32_t max_blocks, float scale, int32_t use_f64)
{
    if (!p || n_seqs < 0 || n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads) return ORACLE_ERR_INVALID;
    const int d = p->head_dim, g = n_q_heads / n_kv_heads, B = p->block_size;
    for (int32_t s = 0; s < n_seqs; ++s)
        if (ctx_lens[s] < 0 || (ctx_lens[s] + B - 1) / B > max_blocks) return ORACLE_ERR_INVALID;
    int status = ORACLE_OK;
    const int64_t n_work = (int64_t)n_seqs * n_kv_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t w = 0; w < n_work; ++w) {
        const int32_t s = (int32_t)(w / n_kv_heads), h = (int32_t)(w % n_kv_heads);
        const int64_t L = ctx_lens[s];
        float *K = (float *)malloc(sizeof(float) * (size_t)(L > 0 ? L : 1) * d);
        float *V = (float *)malloc(sizeof(float) * (size_t)(L > 0 ? L : 1) * d);
        double *scratch = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
        float *qf = (float *)malloc(sizeof(float) * d);
        int rc = oracle_gather(p, block_tables + ((size_t)s * n_kv_heads + h) * max_blocks, L, K, V);
        if (rc != ORACLE_OK) {
#pragma omp critical
            status = rc;
        } else {
            for (int i = h * g; i < (h + 1) * g; ++i) {
                const size_t row = ((size_t)s * n_q_heads + i) * d;
                for (int c = 0; c < d; ++c) qf[c] = widen((const uint8_t *)q, p->dtype, row + c);
                if (use_f64)
                    oracle_attn_row_f64(qf, K, V, L, d, scale, out + row, NULL, scratch);
                else
                    oracle_attn_row_f32(qf, K, V, L, d, scale, out + row, NULL, (float *)scratch);
            }
        }
        free(K); free(V); free(scratch); free(qf);
    }
    return status;
}

/* ------------------------------------------------------------------------- */
/* Chunked causal prefill: the chunk of sequence s has rows                    */
/* cu_q_lens[s] .. cu_q_lens[s+1]-1 of the packed q; row r of the chunk sits   */
/* at absolute position q_start[s] + r and attends to keys 0 .. that position. */
/* The chunk's own K/V are already in the pool.                                */
/* ------------------------------------------------------------------------- */

int oracle_prefill_attn(oracle_pool *p, float *out, const void *q, const int32_t *cu_q_lens,
                        const int32_t *q_start, const int32_t *block_tables, int32_t n_seqs,
                        int32_t n_q_heads, int32_t n_kv_heads, int32_t max_blocks, float scale,
                        int32_t use_f64)
{
    if (!p || n_seqs < 0 || n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads) return ORACLE_ERR_INVALID;
    const int d = p->head_dim, g = n_q_heads / n_kv_heads, B = p->block_size;
    for (int32_t s = 0; s < n_seqs; ++s) {
        int64_t ql = (int64_t)cu_q_lens[s + 1] - cu_q_lens[s];
        if (ql < 0 || q_start[s] < 0 || (q_start[s] + ql + B - 1) / B > max_blocks) return ORACLE_ERR_INVALID;
    }
    int status = ORACLE_OK;
    const int64_t n_work = (int64_t)n_seqs * n_kv_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t w = 0; w < n_work; ++w) {
        const int32_t s = (int32_t)(w / n_kv_heads), h = (int32_t)(w % n_kv_heads);
        const int64_t ql = (int64_t)cu_q_lens[s + 1] - cu_q_lens[s];
        const int64_t L = q_start[s] + ql;
        if (ql == 0) continue;
        float *K = (float *)malloc(sizeof(float) * (size_t)L * d);
        float *V = (float *)malloc(sizeof(float) * (size_t)L * d);
        double *scratch = (double *)malloc(sizeof(double) * (size_t)L);
        float *qf = (float *)malloc(sizeof(float) * d);
        int rc = oracle_gather(p, block_tables + ((size_t)s * n_kv_heads + h) * max_blocks, L, K, V);
        if (rc != ORACLE_OK) {
#pragma omp critical
            status = rc;
        } else {
            for (int64_t r = 0; r < ql; ++r) {
                const int64_t n_keys = q_start[s] + r + 1;
                for (int i = h * g; i < (h + 1) * g; ++i) {
                    const size_t row = ((size_t)(cu_q_lens[s] + r) * n_q_heads + i) * d;
                    for (int c = 0; c < d; ++c) qf[c] = widen((const uint8_t *)q, p->dtype, row + c);
                    if (use_f64)
                        oracle_attn_row_f64(qf, K, V, n_keys, d, scale, out + row, NULL, scratch);
                    else
                        oracle_attn_row_f32(qf, K, V, n_keys, d, scale, out + row, NULL, (float *)scratch);
                }
            }
        }
        free(K); free(V); free(scratch); free(qf);
    }
    return status;
}

/* Softmax weights of one decode row (sequence s, q head i): weights[0..L_s).  */
int oracle_decode_weights(oracle_pool *p, double *weights, const void *q, const int32_t *block_tables,
                          const int32_t *ctx_lens, int32_t s, int32_t i, int32_t n_q_heads,
                          int32_t n_kv_heads, int32_t max_blocks, float scale)
{
    if (!p || n_q_heads % n_kv_heads) return ORACLE_ERR_INVALID;
    const int d = p->head_dim, g = n_q_heads / n_kv_heads, h = i / g;
    const int64_t L = ctx_lens[s];
    if (L <= 0) return ORACLE_OK;
    float *K = (float *)malloc(sizeof(float) * (size_t)L * d);
    float *V = (float *)malloc(sizeof(float) * (size_t)L * d);
    float *x = (float *)malloc(sizeof(float) * (size_t)L);
    float *wf = (float *)malloc(sizeof(float) * (size_t)L);
    float *qf = (float *)malloc(sizeof(float) * d);
    float *o = (float *)malloc(sizeof(float) * d);
    int rc = oracle_gather(p, block_tables + ((size_t)s * n_kv_heads + h) * max_blocks, L, K, V);
    if (rc == ORACLE_OK) {
        const size_t row = ((size_t)s * n_q_heads + i) * d;
        for (int c = 0; c < d; ++c) qf[c] = widen((const uint8_t *)q, p->dtype, row + c);
        oracle_attn_row_f32(qf, K, V, L, d, scale, o, wf, x);
        for (int64_t j = 0; j < L; ++j) weights[j] = wf[j];
    }
    free(K); free(V); free(x); free(wf); free(qf); free(o);
    return rc;
}

/* Threads the parallel loops use from now on (n >= 1); for timing the oracle on one core. */
void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
