/*
 * CPU oracle for the batch scheduler of MuxServe (arXiv 2404.02015, Section 3.3, Algorithm 3:
 * adaptive batch scheduling, ADBS) as a host-side driver of the paged KV pool.
 *
 * TEST INFRASTRUCTURE ONLY, like the rest of this directory: it shares no code with the GPU
 * library; only the tests, the smoke check and the benchmark's CPU leg may use it.
 *
 * What Algorithm 3 fixes: a token-block quota per LLM, initialised once; in every iteration of
 * an endless loop, one prefill job picked round-robin over the LLMs and run if its resources are
 * there; then decoding jobs picked round-robin and run for as long as resources are there; then
 * a periodic adaptation of the quotas.  What it leaves open, and how this file reads it (the
 * GPU library is written to the same reading):
 *
 *  - An iteration is synchronous: its jobs run to completion inside it.  The rule that a
 *    prefill job which finds no resources holds back the decoding jobs is about compute
 *    capacity (the prefill waits for running jobs to drain); a synchronous driver always has the
 *    compute, and a prefill refused for lack of BLOCKS must not stop decoding, because only
 *    decoding ever finishes requests and frees blocks.  So: a prefill that does not fit is
 *    skipped for this iteration and the pointer moves on.
 *  - Prefill job of a model = its waiting requests in arrival order, taken one by one while the
 *    job stays within max_prefill_tokens tokens (the first request is taken whatever its length),
 *    a sequence slot is free, and the request's blocks fit both the model's quota and the pool.
 *    A request brings ceil(len / block_size) x heads blocks, one allocator call per request,
 *    ids laid out head-major in its table row.  Prefill produces the first output token.
 *  - Decoding job of a model = one step for all its running requests: each appends the token it
 *    produced last (a new block per head when its context length is a multiple of block_size,
 *    one allocator call of `heads` ids per such request, in admission order) and produces the
 *    next.  If the step's blocks do not fit the quota or the pool, the model's most recently
 *    admitted request is preempted (blocks freed, back to the FRONT of the waiting queue, to be
 *    recomputed: its next prefill covers prompt + outputs so far minus the last) until the step
 *    fits.  A request preempted in the very iteration that admitted it is struck from that
 *    iteration's prefill job instead of being listed as preempted: whoever launches the jobs
 *    must not write its K/V, because the blocks it gave back may already belong to another
 *    model's decoding job of the same iteration (it still counts as a preemption).  Every model with running requests gets one decoding step per iteration; the model
 *    served first rotates by one per iteration.
 *  - A request ends when it has produced output_len tokens.  Its blocks and its slot go back at
 *    the START of the next iteration (one call per request, ids in table order, head-major,
 *    requests in the order they ended): the job that ends a request still has to read them, and
 *    whoever launches the jobs does so after the iteration's decisions are taken.
 *  - Every adapt_period iterations the quotas are adapted (oracle_adapt_quotas).
 *  - A request is refused at submission if its prompt_len + output_len - 1 tokens of cache need
 *    more table columns than a row has or more blocks than the whole pool holds.  (One that
 *    exceeds its model's QUOTA is accepted: quotas move.)
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ADBS_OK 0
#define ADBS_ERR_INVALID (-1)
#define ADBS_PREFILL 1
#define ADBS_DECODE 2
#define ADBS_PREEMPT 3
#define ADBS_FLAG_TABLE 1    /* the sequence's table row changed in this job */
#define ADBS_FLAG_FINISHED 2 /* the request ended with this job */

/* the block manager of mux_oracle.c, used through its public functions only */
typedef struct oracle_pool oracle_pool;
int oracle_alloc_blocks(oracle_pool *p, int32_t model_id, int64_t n, int32_t *out_ids);
int oracle_free_blocks(oracle_pool *p, int32_t model_id, int64_t n, const int32_t *ids);
int64_t oracle_pool_num_free(const oracle_pool *p);
int64_t oracle_pool_num_blocks(const oracle_pool *p);
int64_t oracle_pool_num_used(const oracle_pool *p, int32_t model_id);
int64_t oracle_get_quota(const oracle_pool *p, int32_t model_id);
int oracle_adapt_quotas(oracle_pool *p, int32_t n_models, double low, double high, double step, int64_t *moved);

typedef struct {
    int64_t id;
    int32_t prompt_len, output_len;
    int32_t gen;   /* output tokens produced so far */
    int32_t ctx;   /* tokens whose K/V are cached (0 while waiting) */
    int32_t slot;  /* row of the model's table, -1 while waiting */
    int64_t order; /* admission stamp: larger = admitted later */
} req_t;

typedef struct {
    int32_t heads;
    req_t *wait; /* waiting[0] is next */
    int32_t n_wait, cap_wait;
    req_t *run;  /* in admission order */
    int32_t n_run;
    int32_t *table; /* [max_seqs][heads][max_blocks] */
    uint8_t *slot_used;
    int64_t finished, preempted;
} model_t;

typedef struct {
    int32_t kind, model, n;
    int64_t *ids;
    int32_t *slots, *lens, *flags;
} job_t;

typedef struct {
    int32_t model, slot, ctx;
} ended_t;

typedef struct adbs_oracle {
    ended_t *ended; /* requests that ended in the last iteration: blocks still held */
    int32_t n_ended, cap_ended;
    oracle_pool *pool;
    int32_t n_models, block_size, max_seqs, max_blocks, max_prefill_tokens, adapt_period;
    double low, high, step;
    model_t *m;
    int32_t prefill_ptr, decode_ptr;
    int64_t iteration, stamp, quota_moved;
    int64_t first_stamp; /* admission stamp at the start of the current iteration */
    job_t *jobs;
    int32_t n_jobs, cap_jobs;
} adbs_oracle;

static int32_t *row_of(adbs_oracle *s, model_t *md, int32_t slot)
{
    return md->table + (size_t)slot * md->heads * s->max_blocks;
}

static int32_t blocks_for(const adbs_oracle *s, int32_t tokens) { return (tokens + s->block_size - 1) / s->block_size; }

static job_t *new_job(adbs_oracle *s, int32_t kind, int32_t model)
{
    if (s->n_jobs == s->cap_jobs) {
        s->cap_jobs = s->cap_jobs ? 2 * s->cap_jobs : 8;
        s->jobs = (job_t *)realloc(s->jobs, sizeof(job_t) * (size_t)s->cap_jobs);
        memset(s->jobs + s->n_jobs, 0, sizeof(job_t) * (size_t)(s->cap_jobs - s->n_jobs));
    }
    job_t *j = &s->jobs[s->n_jobs++];
    j->kind = kind;
    j->model = model;
    j->n = 0;
    if (!j->ids) {
        j->ids = (int64_t *)malloc(sizeof(int64_t) * (size_t)s->max_seqs);
        j->slots = (int32_t *)malloc(sizeof(int32_t) * (size_t)s->max_seqs);
        j->lens = (int32_t *)malloc(sizeof(int32_t) * (size_t)s->max_seqs);
        j->flags = (int32_t *)malloc(sizeof(int32_t) * (size_t)s->max_seqs);
    }
    return j;
}

static void job_add(job_t *j, int64_t id, int32_t slot, int32_t len, int32_t flags)
{
    j->ids[j->n] = id;
    j->slots[j->n] = slot;
    j->lens[j->n] = len;
    j->flags[j->n] = flags;
    j->n++;
}

/* blocks the model may still take: bounded by its quota (if it has one) and by the pool */
static int64_t room(adbs_oracle *s, int32_t model)
{
    int64_t r = oracle_pool_num_free(s->pool);
    int64_t q = oracle_get_quota(s->pool, model);
    if (q >= 0) {
        int64_t slack = q - oracle_pool_num_used(s->pool, model);
        if (slack < r) r = slack;
    }
    return r < 0 ? 0 : r;
}

/* give back all blocks of a sequence (table order: head-major) and its slot */
static void release_slot(adbs_oracle *s, int32_t model, int32_t slot, int32_t ctx)
{
    model_t *md = &s->m[model];
    int32_t nb = blocks_for(s, ctx);
    int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * (size_t)(nb * md->heads + 1));
    int32_t *row = row_of(s, md, slot);
    int32_t k = 0;
    for (int32_t h = 0; h < md->heads; ++h)
        for (int32_t b = 0; b < nb; ++b) ids[k++] = row[h * s->max_blocks + b];
    oracle_free_blocks(s->pool, model, k, ids);
    free(ids);
    md->slot_used[slot] = 0;
}

/* a preempted request gives everything back at once: no job of this iteration reads its blocks */
static void release(adbs_oracle *s, int32_t model, req_t *r)
{
    release_slot(s, model, r->slot, r->ctx);
    r->slot = -1;
    r->ctx = 0;
}

/* a request that ended keeps blocks and slot until the next iteration starts */
static void retire(adbs_oracle *s, int32_t model, const req_t *r)
{
    if (s->n_ended == s->cap_ended) {
        s->cap_ended = s->cap_ended ? 2 * s->cap_ended : 16;
        s->ended = (ended_t *)realloc(s->ended, sizeof(ended_t) * (size_t)s->cap_ended);
    }
    ended_t e = {model, r->slot, r->ctx};
    s->ended[s->n_ended++] = e;
    s->m[model].finished++;
}

int adbs_oracle_create(adbs_oracle **out, oracle_pool *pool, int32_t n_models, const int32_t *heads,
                       int32_t block_size, int32_t max_seqs, int32_t max_blocks, int32_t max_prefill_tokens,
                       int32_t adapt_period, double low, double high, double step)
{
    if (!out || !pool || n_models <= 0 || n_models > 1024 || !heads || block_size <= 0 || max_seqs <= 0 ||
        max_blocks <= 0 || max_prefill_tokens <= 0 || adapt_period < 0)
        return ADBS_ERR_INVALID;
    for (int32_t i = 0; i < n_models; ++i)
        if (heads[i] <= 0 || heads[i] > 4096) return ADBS_ERR_INVALID;
    adbs_oracle *s = (adbs_oracle *)calloc(1, sizeof(*s));
    s->pool = pool;
    s->n_models = n_models;
    s->block_size = block_size;
    s->max_seqs = max_seqs;
    s->max_blocks = max_blocks;
    s->max_prefill_tokens = max_prefill_tokens;
    s->adapt_period = adapt_period;
    s->low = low;
    s->high = high;
    s->step = step;
    s->m = (model_t *)calloc((size_t)n_models, sizeof(model_t));
    for (int32_t i = 0; i < n_models; ++i) {
        model_t *md = &s->m[i];
        md->heads = heads[i];
        md->run = (req_t *)calloc((size_t)max_seqs, sizeof(req_t));
        md->table = (int32_t *)malloc(sizeof(int32_t) * (size_t)max_seqs * heads[i] * max_blocks);
        for (size_t k = 0; k < (size_t)max_seqs * heads[i] * max_blocks; ++k) md->table[k] = -1;
        md->slot_used = (uint8_t *)calloc((size_t)max_seqs, 1);
    }
    *out = s;
    return ADBS_OK;
}

void adbs_oracle_destroy(adbs_oracle *s)
{
    if (!s) return;
    for (int32_t i = 0; i < s->n_models; ++i) {
        free(s->m[i].wait);
        free(s->m[i].run);
        free(s->m[i].table);
        free(s->m[i].slot_used);
    }
    for (int32_t j = 0; j < s->cap_jobs; ++j) {
        free(s->jobs[j].ids);
        free(s->jobs[j].slots);
        free(s->jobs[j].lens);
        free(s->jobs[j].flags);
    }
    free(s->jobs);
    free(s->ended);
    free(s->m);
    free(s);
}

static void push_wait(model_t *md, req_t r, int front)
{
    if (md->n_wait == md->cap_wait) {
        md->cap_wait = md->cap_wait ? 2 * md->cap_wait : 16;
        md->wait = (req_t *)realloc(md->wait, sizeof(req_t) * (size_t)md->cap_wait);
    }
    if (front) {
        memmove(md->wait + 1, md->wait, sizeof(req_t) * (size_t)md->n_wait);
        md->wait[0] = r;
    } else {
        md->wait[md->n_wait] = r;
    }
    md->n_wait++;
}

int adbs_oracle_submit(adbs_oracle *s, int32_t model, int64_t id, int32_t prompt_len, int32_t output_len)
{
    if (!s || model < 0 || model >= s->n_models || prompt_len <= 0 || output_len <= 0) return ADBS_ERR_INVALID;
    if ((int64_t)prompt_len + output_len > (int64_t)s->max_blocks * s->block_size) return ADBS_ERR_INVALID;
    /* a request whose cache could not even fit an empty pool would be preempted for ever */
    if ((int64_t)blocks_for(s, prompt_len + output_len - 1) * s->m[model].heads > oracle_pool_num_blocks(s->pool))
        return ADBS_ERR_INVALID;
    req_t r = {id, prompt_len, output_len, 0, 0, -1, 0};
    push_wait(&s->m[model], r, 0);
    return ADBS_OK;
}

static void prefill_phase(adbs_oracle *s)
{
    /* round-robin: the first model, from the pointer on, that has a waiting request */
    int32_t model = -1;
    for (int32_t k = 0; k < s->n_models; ++k) {
        int32_t c = (s->prefill_ptr + k) % s->n_models;
        if (s->m[c].n_wait > 0) { model = c; break; }
    }
    if (model < 0) return;
    s->prefill_ptr = (model + 1) % s->n_models;
    model_t *md = &s->m[model];
    job_t *job = NULL;
    int32_t tokens = 0;
    while (md->n_wait > 0) {
        req_t r = md->wait[0];
        int32_t len = r.prompt_len + (r.gen > 0 ? r.gen - 1 : 0);
        if (job && tokens + len > s->max_prefill_tokens) break;
        int32_t slot = -1;
        for (int32_t i = 0; i < s->max_seqs; ++i)
            if (!md->slot_used[i]) { slot = i; break; }
        if (slot < 0) break;
        int32_t nb = blocks_for(s, len);
        int64_t need = (int64_t)nb * md->heads;
        if (need > room(s, model)) break;
        int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * (size_t)need);
        oracle_alloc_blocks(s->pool, model, need, ids);
        int32_t *row = row_of(s, md, slot);
        for (int32_t h = 0; h < md->heads; ++h)
            for (int32_t b = 0; b < nb; ++b) row[h * s->max_blocks + b] = ids[h * nb + b];
        free(ids);
        md->slot_used[slot] = 1;
        memmove(md->wait, md->wait + 1, sizeof(req_t) * (size_t)(md->n_wait - 1));
        md->n_wait--;
        r.slot = slot;
        r.ctx = len;
        if (r.gen == 0) r.gen = 1;
        r.order = s->stamp++;
        tokens += len;
        if (!job) job = new_job(s, ADBS_PREFILL, model);
        int32_t flags = ADBS_FLAG_TABLE;
        if (r.gen >= r.output_len) {
            flags |= ADBS_FLAG_FINISHED;
            job_add(job, r.id, slot, len, flags);
            retire(s, model, &r);
        } else {
            job_add(job, r.id, slot, len, flags);
            md->run[md->n_run++] = r;
        }
    }
}

/* the request was admitted in this iteration: take it out of the iteration's prefill job */
static void strike_from_prefill(adbs_oracle *s, int32_t model, const req_t *r)
{
    for (int32_t j = 0; j < s->n_jobs; ++j) {
        job_t *jb = &s->jobs[j];
        if (jb->kind != ADBS_PREFILL || jb->model != model) continue;
        for (int32_t i = 0; i < jb->n; ++i)
            if (jb->ids[i] == r->id && jb->slots[i] == r->slot) {
                for (int32_t k = i + 1; k < jb->n; ++k) {
                    jb->ids[k - 1] = jb->ids[k];
                    jb->slots[k - 1] = jb->slots[k];
                    jb->lens[k - 1] = jb->lens[k];
                    jb->flags[k - 1] = jb->flags[k];
                }
                jb->n--;
                return;
            }
    }
}

/* a job that lost all its requests is no job: close the gaps, keeping the order */
static void drop_empty_jobs(adbs_oracle *s)
{
    int32_t kept = 0;
    for (int32_t j = 0; j < s->n_jobs; ++j) {
        if (s->jobs[j].n == 0) continue;
        if (kept != j) {
            job_t t = s->jobs[kept];
            s->jobs[kept] = s->jobs[j];
            s->jobs[j] = t; /* the arrays of the empty one stay owned by the list */
        }
        kept++;
    }
    s->n_jobs = kept;
}

static void decode_phase(adbs_oracle *s)
{
    for (int32_t k = 0; k < s->n_models; ++k) {
        int32_t model = (s->decode_ptr + k) % s->n_models;
        model_t *md = &s->m[model];
        if (md->n_run == 0) continue;
        job_t *pre = NULL;
        for (;;) {
            int64_t need = 0;
            for (int32_t i = 0; i < md->n_run; ++i)
                if (md->run[i].ctx % s->block_size == 0) need += md->heads;
            if (need <= room(s, model)) break;
            /* preempt the request admitted last */
            int32_t y = 0;
            for (int32_t i = 1; i < md->n_run; ++i)
                if (md->run[i].order > md->run[y].order) y = i;
            req_t r = md->run[y];
            if (r.order >= s->first_stamp) {
                strike_from_prefill(s, model, &r);
            } else {
                if (!pre) pre = new_job(s, ADBS_PREEMPT, model);
                job_add(pre, r.id, r.slot, r.ctx, 0);
            }
            release(s, model, &r);
            memmove(md->run + y, md->run + y + 1, sizeof(req_t) * (size_t)(md->n_run - y - 1));
            md->n_run--;
            md->preempted++;
            push_wait(md, r, 1);
            if (md->n_run == 0) break;
        }
        if (md->n_run == 0) continue;
        job_t *job = new_job(s, ADBS_DECODE, model);
        int32_t kept = 0;
        for (int32_t i = 0; i < md->n_run; ++i) {
            req_t r = md->run[i];
            int32_t flags = 0;
            if (r.ctx % s->block_size == 0) {
                int32_t ids[4096];
                int32_t *row = row_of(s, md, r.slot);
                oracle_alloc_blocks(s->pool, model, md->heads, ids);
                for (int32_t h = 0; h < md->heads; ++h) row[h * s->max_blocks + r.ctx / s->block_size] = ids[h];
                flags |= ADBS_FLAG_TABLE;
            }
            r.ctx += 1;
            r.gen += 1;
            if (r.gen >= r.output_len) {
                job_add(job, r.id, r.slot, r.ctx, flags | ADBS_FLAG_FINISHED);
                retire(s, model, &r);
            } else {
                job_add(job, r.id, r.slot, r.ctx, flags);
                md->run[kept++] = r;
            }
        }
        md->n_run = kept;
    }
    s->decode_ptr = (s->decode_ptr + 1) % s->n_models;
}

int adbs_oracle_step(adbs_oracle *s, int32_t *n_jobs)
{
    if (!s || !n_jobs) return ADBS_ERR_INVALID;
    s->n_jobs = 0;
    for (int32_t i = 0; i < s->n_ended; ++i) release_slot(s, s->ended[i].model, s->ended[i].slot, s->ended[i].ctx);
    s->n_ended = 0;
    s->first_stamp = s->stamp;
    prefill_phase(s);
    decode_phase(s);
    drop_empty_jobs(s);
    s->iteration++;
    if (s->adapt_period > 0 && s->iteration % s->adapt_period == 0) {
        int64_t moved = 0;
        if (oracle_adapt_quotas(s->pool, s->n_models, s->low, s->high, s->step, &moved) == 0) s->quota_moved += moved;
    }
    *n_jobs = s->n_jobs;
    return ADBS_OK;
}

int adbs_oracle_job(const adbs_oracle *s, int32_t j, int32_t *kind, int32_t *model, int32_t *n_seqs)
{
    if (!s || j < 0 || j >= s->n_jobs || !kind || !model || !n_seqs) return ADBS_ERR_INVALID;
    *kind = s->jobs[j].kind;
    *model = s->jobs[j].model;
    *n_seqs = s->jobs[j].n;
    return ADBS_OK;
}

int adbs_oracle_job_seqs(const adbs_oracle *s, int32_t j, int64_t *ids, int32_t *slots, int32_t *lens, int32_t *flags)
{
    if (!s || j < 0 || j >= s->n_jobs) return ADBS_ERR_INVALID;
    const job_t *jb = &s->jobs[j];
    for (int32_t i = 0; i < jb->n; ++i) {
        if (ids) ids[i] = jb->ids[i];
        if (slots) slots[i] = jb->slots[i];
        if (lens) lens[i] = jb->lens[i];
        if (flags) flags[i] = jb->flags[i];
    }
    return ADBS_OK;
}

const int32_t *adbs_oracle_table(const adbs_oracle *s, int32_t model)
{
    if (!s || model < 0 || model >= s->n_models) return NULL;
    return s->m[model].table;
}

/* counts[0..4] = waiting, running, finished, preempted (of the model), quota blocks moved (all models) */
int adbs_oracle_counts(const adbs_oracle *s, int32_t model, int64_t *counts)
{
    if (!s || model < 0 || model >= s->n_models || !counts) return ADBS_ERR_INVALID;
    counts[0] = s->m[model].n_wait;
    counts[1] = s->m[model].n_run;
    counts[2] = s->m[model].finished;
    counts[3] = s->m[model].preempted;
    counts[4] = s->quota_moved;
    return ADBS_OK;
}

/* ------------------------------------------------------------------------- */
/* Throughput estimator (Section 3.3, Eq. 3; Appendix A.2): a stable batch of   */
/* b^m requests of LLM m takes the prefill latencies of ALL colocated LLMs (they */
/* run one after another) plus m's decoding latency times its average           */
/* generation length (decoding phases overlap); the estimate is the batch over   */
/* that time, capped by the offered rate W_b.  An LLM with an empty batch runs   */
/* no prefill.  Returns -1 for arguments outside the formula's domain.           */
/* ------------------------------------------------------------------------- */
double adbs_oracle_tpt(int32_t n_models, const double *batch, const double *t_prefill, const double *t_decode,
                       const double *gen_len, int32_t m, double rate_cap)
{
    if (n_models <= 0 || !batch || !t_prefill || !t_decode || !gen_len || m < 0 || m >= n_models) return -1.0;
    if (!(rate_cap >= 0.0)) return -1.0;
    double denom = 0.0;
    for (int32_t i = 0; i < n_models; ++i) {
        if (!(batch[i] >= 0.0) || !(t_prefill[i] >= 0.0) || !(t_decode[i] >= 0.0) || !(gen_len[i] >= 0.0)) return -1.0;
        if (batch[i] > 0.0) denom += t_prefill[i];
    }
    denom += t_decode[m] * gen_len[m];
    if (denom <= 0.0) return batch[m] > 0.0 ? rate_cap : 0.0;
    double tpt = batch[m] / denom;
    return tpt < rate_cap ? tpt : rate_cap;
}

/* "Binary search to find the batch size that can satisfy the traffic": by definition the      */
/* smallest batch size whose estimate reaches the rate.  Latencies are the caller's fitted     */
/* lines t_p(b) = p0 + p1 b, t_d(b) = d0 + d1 b.  Written as the plain scan over b = 1, 2, ... */
/* Returns 0 if no b <= max_batch does, -1 for bad arguments.                                   */
int64_t adbs_oracle_batch_size(double rate, int64_t max_batch, double p0, double p1, double d0, double d1,
                               double gen_len, double other_prefill)
{
    if (!(rate >= 0.0) || max_batch < 1 || !(p0 >= 0.0) || !(p1 >= 0.0) || !(d0 >= 0.0) || !(d1 >= 0.0) ||
        !(gen_len >= 0.0) || !(other_prefill >= 0.0))
        return -1;
    for (int64_t b = 1; b <= max_batch; ++b) {
        double t = other_prefill + (p0 + p1 * (double)b) + (d0 + d1 * (double)b) * gen_len;
        if (t <= 0.0 || (double)b / t >= rate) return b;
    }
    return 0;
}
