// Batch scheduler over the unified KV pool: MuxServe, Section 3.3, Algorithm 3 (adaptive batch
// scheduling).  Host code only: it decides which job runs next and keeps the block tables; the
// caller launches the kernels for the jobs it is handed.  The reading of what Algorithm 3 leaves
// open is stated with the entry points in mux.h.
#include <algorithm>
#include <deque>
#include <new>
#include <vector>

#include "mux_internal.h"

namespace {

struct Request {
    int64_t id = 0;
    int32_t prompt_len = 0, output_len = 0;
    int32_t produced = 0;   // output tokens so far
    int32_t cached = 0;     // tokens with K/V in the pool
    int32_t slot = -1;
    int64_t admitted = 0;   // stamp of the last admission
    int32_t recompute_len() const { return prompt_len + std::max(produced - 1, 0); }
};

struct Model {
    int32_t heads = 0;
    std::deque<Request> waiting;
    std::vector<Request> running;       // admission order
    std::vector<int32_t> table;         // [max_seqs][heads][max_blocks]
    std::vector<char> slot_taken;
    int64_t n_finished = 0, n_preempted = 0;
};

struct Job {
    int32_t kind = 0, model = 0;
    std::vector<int64_t> ids;
    std::vector<int32_t> slots, lens, flags;
    void add(int64_t id, int32_t slot, int32_t len, int32_t flag)
    {
        ids.push_back(id);
        slots.push_back(slot);
        lens.push_back(len);
        flags.push_back(flag);
    }
};

}  // namespace

struct mux_sched {
    mux_pool *pool = nullptr;
    mux_sched_config cfg{};
    std::vector<Model> models;
    int32_t next_prefill = 0, first_decode = 0;
    int64_t iterations = 0, stamp = 0, quota_moved = 0;
    int64_t first_stamp = 0;    // admission stamp at the start of the current iteration
    std::vector<Job> jobs;
    std::vector<int32_t> scratch_ids;
    struct Ended { int32_t model, slot, cached; };
    std::vector<Ended> ended;   // ended in the last iteration: blocks and slot held until the next one starts
    std::vector<char> released; // per model: the last iteration gave blocks of this model back to the pool

    int32_t *row(Model &m, int32_t slot) { return m.table.data() + static_cast<size_t>(slot) * m.heads * cfg.max_blocks; }
    int32_t blocks_of(int32_t tokens) const { return (tokens + pool->block_size - 1) / pool->block_size; }

    // blocks the model can still take right now (quota and pool)
    int64_t headroom(int32_t model) const
    {
        int64_t free_now = mux_pool_num_free(pool);
        int64_t quota = -1;
        mux_pool_get_quota(pool, model, &quota);
        if (quota >= 0) free_now = std::min(free_now, quota - mux_pool_num_used(pool, model));
        return std::max<int64_t>(free_now, 0);
    }

    void free_sequence(int32_t model, int32_t slot, int32_t cached)
    {
        Model &m = models[model];
        const int32_t nb = blocks_of(cached);
        scratch_ids.clear();
        const int32_t *t = row(m, slot);
        for (int32_t h = 0; h < m.heads; ++h)
            scratch_ids.insert(scratch_ids.end(), t + h * cfg.max_blocks, t + h * cfg.max_blocks + nb);
        mux_free_blocks(pool, model, static_cast<int64_t>(scratch_ids.size()), scratch_ids.data());
        m.slot_taken[slot] = 0;
        released[model] = 1;
    }

    // preemption: nothing launched for this iteration reads the request's blocks, they go back now
    void give_back(int32_t model, Request &r)
    {
        free_sequence(model, r.slot, r.cached);
        r.slot = -1;
        r.cached = 0;
    }

    // end of a request: its last job still reads the blocks, so they go back when the next iteration starts
    void retire(int32_t model, const Request &r)
    {
        ended.push_back(Ended{model, r.slot, r.cached});
        ++models[model].n_finished;
    }

    void run_prefill()
    {
        const int32_t n = static_cast<int32_t>(models.size());
        int32_t pick = -1;
        for (int32_t k = 0; k < n && pick < 0; ++k)
            if (!models[(next_prefill + k) % n].waiting.empty()) pick = (next_prefill + k) % n;
        if (pick < 0) return;
        next_prefill = (pick + 1) % n;
        Model &m = models[pick];
        Job job;
        job.kind = MUX_JOB_PREFILL;
        job.model = pick;
        int64_t tokens = 0;
        while (!m.waiting.empty()) {
            Request r = m.waiting.front();
            const int32_t len = r.recompute_len();
            if (!job.ids.empty() && tokens + len > cfg.max_prefill_tokens) break;
            const auto free_slot = std::find(m.slot_taken.begin(), m.slot_taken.end(), 0);
            if (free_slot == m.slot_taken.end()) break;
            const int32_t nb = blocks_of(len);
            const int64_t need = static_cast<int64_t>(nb) * m.heads;
            if (need > headroom(pick)) break;
            scratch_ids.resize(static_cast<size_t>(need));
            if (mux_alloc_blocks(pool, pick, need, scratch_ids.data()) != MUX_OK) break;
            r.slot = static_cast<int32_t>(free_slot - m.slot_taken.begin());
            *free_slot = 1;
            int32_t *t = row(m, r.slot);
            for (int32_t h = 0; h < m.heads; ++h)
                std::copy(scratch_ids.begin() + static_cast<size_t>(h) * nb, scratch_ids.begin() + static_cast<size_t>(h + 1) * nb,
                          t + h * cfg.max_blocks);
            m.waiting.pop_front();
            r.cached = len;
            r.produced = std::max(r.produced, 1);
            r.admitted = stamp++;
            tokens += len;
            if (r.produced >= r.output_len) {
                job.add(r.id, r.slot, len, MUX_JOB_FLAG_TABLE | MUX_JOB_FLAG_FINISHED);
                retire(pick, r);
            } else {
                job.add(r.id, r.slot, len, MUX_JOB_FLAG_TABLE);
                m.running.push_back(r);
            }
        }
        if (!job.ids.empty()) jobs.push_back(std::move(job));
    }

    // The blocks of a request preempted in the iteration that admitted it may be handed to another
    // model before the iteration's jobs are launched, so its entry leaves the prefill job.
    void cancel_prefill(int32_t model, const Request &r)
    {
        for (Job &job : jobs) {
            if (job.kind != MUX_JOB_PREFILL || job.model != model) continue;
            for (size_t i = 0; i < job.ids.size(); ++i)
                if (job.ids[i] == r.id && job.slots[i] == r.slot) {
                    job.ids.erase(job.ids.begin() + static_cast<std::ptrdiff_t>(i));
                    job.slots.erase(job.slots.begin() + static_cast<std::ptrdiff_t>(i));
                    job.lens.erase(job.lens.begin() + static_cast<std::ptrdiff_t>(i));
                    job.flags.erase(job.flags.begin() + static_cast<std::ptrdiff_t>(i));
                    return;
                }
        }
    }

    void run_decode(int32_t model)
    {
        Model &m = models[model];
        if (m.running.empty()) return;
        const int32_t B = pool->block_size;
        Job evicted;
        evicted.kind = MUX_JOB_PREEMPT;
        evicted.model = model;
        while (!m.running.empty()) {
            const int64_t opening = std::count_if(m.running.begin(), m.running.end(), [&](const Request &r) { return r.cached % B == 0; });
            if (opening * m.heads <= headroom(model)) break;
            auto youngest = std::max_element(m.running.begin(), m.running.end(),
                                             [](const Request &a, const Request &b) { return a.admitted < b.admitted; });
            Request r = *youngest;
            m.running.erase(youngest);
            if (r.admitted >= first_stamp)
                cancel_prefill(model, r);   // admitted in this very iteration: its prefill must not launch
            else
                evicted.add(r.id, r.slot, r.cached, 0);
            give_back(model, r);
            ++m.n_preempted;
            m.waiting.push_front(r);
        }
        if (!evicted.ids.empty()) jobs.push_back(std::move(evicted));
        if (m.running.empty()) return;
        Job job;
        job.kind = MUX_JOB_DECODE;
        job.model = model;
        std::vector<Request> still;
        still.reserve(m.running.size());
        scratch_ids.resize(static_cast<size_t>(m.heads));
        for (Request &r : m.running) {
            int32_t flag = 0;
            if (r.cached % B == 0) {
                mux_alloc_blocks(pool, model, m.heads, scratch_ids.data());
                int32_t *t = row(m, r.slot);
                for (int32_t h = 0; h < m.heads; ++h) t[h * cfg.max_blocks + r.cached / B] = scratch_ids[h];
                flag |= MUX_JOB_FLAG_TABLE;
            }
            ++r.cached;
            ++r.produced;
            if (r.produced >= r.output_len) {
                job.add(r.id, r.slot, r.cached, flag | MUX_JOB_FLAG_FINISHED);
                retire(model, r);
            } else {
                job.add(r.id, r.slot, r.cached, flag);
                still.push_back(r);
            }
        }
        m.running.swap(still);
        jobs.push_back(std::move(job));
    }
};

extern "C" {

int mux_sched_create(mux_sched_t **out, mux_pool_t *pool, const mux_sched_config *cfg)
{
    if (!out || !pool || !cfg || !cfg->heads || cfg->n_models <= 0 || cfg->n_models > MUX_MAX_MODELS || cfg->max_seqs <= 0 ||
        cfg->max_blocks <= 0 || cfg->max_prefill_tokens <= 0 || cfg->adapt_period < 0)
        return MUX_ERR_INVALID;
    for (int32_t i = 0; i < cfg->n_models; ++i)
        if (cfg->heads[i] <= 0 || cfg->heads[i] > 4096) return MUX_ERR_INVALID;
    mux_sched *s = new (std::nothrow) mux_sched();
    if (!s) return MUX_ERR_NOMEM;
    try {
        s->pool = pool;
        s->cfg = *cfg;
        s->cfg.heads = nullptr;   // copied into the models below; the caller's array is not kept
        s->models.resize(static_cast<size_t>(cfg->n_models));
        s->released.assign(static_cast<size_t>(cfg->n_models), 0);
        for (int32_t i = 0; i < cfg->n_models; ++i) {
            Model &m = s->models[i];
            m.heads = cfg->heads[i];
            m.table.assign(static_cast<size_t>(cfg->max_seqs) * m.heads * cfg->max_blocks, -1);
            m.slot_taken.assign(static_cast<size_t>(cfg->max_seqs), 0);
        }
    } catch (const std::bad_alloc &) {
        delete s;
        return MUX_ERR_NOMEM;
    }
    *out = s;
    return MUX_OK;
}

int mux_sched_destroy(mux_sched_t *sched)
{
    if (!sched) return MUX_ERR_INVALID;
    delete sched;
    return MUX_OK;
}

int mux_sched_submit(mux_sched_t *s, int32_t model, int64_t request_id, int32_t prompt_len, int32_t output_len)
{
    if (!s || model < 0 || model >= static_cast<int32_t>(s->models.size()) || prompt_len <= 0 || output_len <= 0)
        return MUX_ERR_INVALID;
    if (static_cast<int64_t>(prompt_len) + output_len > static_cast<int64_t>(s->cfg.max_blocks) * s->pool->block_size)
        return MUX_ERR_INVALID;
    // the most it will ever cache must fit an empty pool, or it would be preempted for ever
    if (static_cast<int64_t>(s->blocks_of(prompt_len + output_len - 1)) * s->models[model].heads > s->pool->num_blocks)
        return MUX_ERR_INVALID;
    Request r;
    r.id = request_id;
    r.prompt_len = prompt_len;
    r.output_len = output_len;
    s->models[model].waiting.push_back(r);
    return MUX_OK;
}

int mux_sched_step(mux_sched_t *s, int32_t *n_jobs)
{
    if (!s || !n_jobs) return MUX_ERR_INVALID;
    s->jobs.clear();
    std::fill(s->released.begin(), s->released.end(), 0);
    for (const mux_sched::Ended &e : s->ended) s->free_sequence(e.model, e.slot, e.cached);
    s->ended.clear();
    s->first_stamp = s->stamp;
    s->run_prefill();
    const int32_t n = static_cast<int32_t>(s->models.size());
    for (int32_t k = 0; k < n; ++k) s->run_decode((s->first_decode + k) % n);
    s->first_decode = (s->first_decode + 1) % n;
    s->jobs.erase(std::remove_if(s->jobs.begin(), s->jobs.end(), [](const Job &j) { return j.ids.empty(); }), s->jobs.end());
    ++s->iterations;
    if (s->cfg.adapt_period > 0 && s->iterations % s->cfg.adapt_period == 0) {
        int64_t moved = 0;
        if (mux_pool_adapt_quotas(s->pool, n, s->cfg.low_util, s->cfg.high_util, s->cfg.step_fraction, &moved) == MUX_OK)
            s->quota_moved += moved;
    }
    *n_jobs = static_cast<int32_t>(s->jobs.size());
    return MUX_OK;
}

int mux_sched_job(const mux_sched_t *s, int32_t j, int32_t *kind, int32_t *model, int32_t *n_seqs)
{
    if (!s || j < 0 || j >= static_cast<int32_t>(s->jobs.size()) || !kind || !model || !n_seqs) return MUX_ERR_INVALID;
    *kind = s->jobs[j].kind;
    *model = s->jobs[j].model;
    *n_seqs = static_cast<int32_t>(s->jobs[j].ids.size());
    return MUX_OK;
}

int mux_sched_job_seqs(const mux_sched_t *s, int32_t j, int64_t *request_ids, int32_t *slots, int32_t *lens, int32_t *flags)
{
    if (!s || j < 0 || j >= static_cast<int32_t>(s->jobs.size())) return MUX_ERR_INVALID;
    const Job &job = s->jobs[j];
    if (request_ids) std::copy(job.ids.begin(), job.ids.end(), request_ids);
    if (slots) std::copy(job.slots.begin(), job.slots.end(), slots);
    if (lens) std::copy(job.lens.begin(), job.lens.end(), lens);
    if (flags) std::copy(job.flags.begin(), job.flags.end(), flags);
    return MUX_OK;
}

const int32_t *mux_sched_table(const mux_sched_t *s, int32_t model)
{
    if (!s || model < 0 || model >= static_cast<int32_t>(s->models.size())) return nullptr;
    return s->models[model].table.data();
}

int mux_sched_counts(const mux_sched_t *s, int32_t model, int64_t *counts)
{
    if (!s || model < 0 || model >= static_cast<int32_t>(s->models.size()) || !counts) return MUX_ERR_INVALID;
    const Model &m = s->models[model];
    counts[0] = static_cast<int64_t>(m.waiting.size());
    counts[1] = static_cast<int64_t>(m.running.size());
    counts[2] = m.n_finished;
    counts[3] = m.n_preempted;
    counts[4] = s->quota_moved;
    return MUX_OK;
}

}  // extern "C"

// Accessors for the job runner (same library, not part of the ABI).
mux_pool *mux_sched_pool(const mux_sched *s) { return s->pool; }
void mux_sched_geometry(const mux_sched *s, int32_t *n_models, int32_t *max_seqs, int32_t *max_blocks, int32_t *max_prefill_tokens)
{
    *n_models = static_cast<int32_t>(s->models.size());
    *max_seqs = s->cfg.max_seqs;
    *max_blocks = s->cfg.max_blocks;
    *max_prefill_tokens = s->cfg.max_prefill_tokens;
}
int32_t mux_sched_heads(const mux_sched *s, int32_t model) { return s->models[model].heads; }
bool mux_sched_released_blocks(const mux_sched *s, int32_t model) { return s->released[model] != 0; }
