// Job runner: launches the jobs of the batch scheduler (MuxServe, Section 3.3, Algorithm 3) on
// the GPU - the part of the paper's serving loop between "the scheduler picked a job" and "the
// attention of that job ran over the unified KV cache" (Section 3.4).  For every job it stages
// the job's small integer arrays - as kernel arguments when they fit (the usual decode job),
// else in pinned memory that ONE kernel reads directly -, installs the block ids the
// scheduler just handed out into the device copy of the model's table, and enqueues append +
// attention on the model's stream.  Nothing here computes
// attention: the kernels are those behind mux_kv_append, mux_prefill_attn and mux_decode_step.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "mux_internal.h"

namespace {

constexpr int kRing = 4;          // staging areas per model: a job's area is rewritten 4 jobs later
constexpr int kEntryInts = 5;     // slot, job row (-1: none), first column, columns, offset of the ids

// Device tables are laid out [layer][max_seqs][kv heads of a layer][max_blocks]: the scheduler's
// head index hh = layer * hkv + head.  Cell of (row, hh):
__device__ __forceinline__ size_t table_cell(int row, int hh, int hkv, int max_seqs)
{
    return (static_cast<size_t>(hh / hkv) * max_seqs + row) * hkv + hh % hkv;
}

// A job's arrays arrive in a pinned host area and this one kernel takes them from there (a
// host-to-device copy, the event that says when the area is free again and a separate install
// kernel cost ~75 us of runtime calls per job; a kernel launch costs ~8):
//   - workgroups 0 .. n_entries-1 install one entry each: the ids of one sequence, head-major
//     [heads][n_cols], go to columns col0 .. col0+n_cols-1 of its row in the model's table and,
//     for a prefill, of the job's table (entries and ids are read from the host area: once each);
//   - the other workgroups copy the area's first copy_ints ints - the arrays that the append and
//     attention kernels read many times over - into the area's device twin;
//   - the workgroup that finishes last writes the area's stamp into pinned host memory.  Every
//     workgroup's reads of the host area have returned by then (their values were stored, or
//     used as addresses, before its barrier), so the host may refill the area as soon as it
//     sees the stamp: no event, no runtime call.
__global__ __launch_bounds__(256) void stage_install_kernel(const int32_t *__restrict__ host_area, int32_t *__restrict__ dev_area,
                                                            int copy_ints, int n_entries, int entries_at, int ids_at,
                                                            int32_t *__restrict__ slot_tables, int32_t *__restrict__ job_tables,
                                                            int heads, int hkv, int max_seqs, int max_blocks, int *arrivals,
                                                            int32_t *stamp_host, int32_t stamp)
{
    const int b = blockIdx.x;
    if (b < n_entries) {
        const int32_t *e = host_area + entries_at + static_cast<size_t>(b) * kEntryInts;
        const int slot = e[0], job_row = e[1], col0 = e[2], n_cols = e[3], at = e[4];
        const int32_t *ids = host_area + ids_at + at;
        for (int i = threadIdx.x; i < heads * n_cols; i += blockDim.x) {
            const int h = i / n_cols, j = i - h * n_cols;
            const int32_t id = ids[i];
            slot_tables[table_cell(slot, h, hkv, max_seqs) * max_blocks + col0 + j] = id;
            if (job_row >= 0) job_tables[table_cell(job_row, h, hkv, max_seqs) * max_blocks + col0 + j] = id;
        }
    } else {
        const int n_copy_wgs = static_cast<int>(gridDim.x) - n_entries;
        for (int i = (b - n_entries) * 256 + threadIdx.x; i < copy_ints; i += n_copy_wgs * 256) dev_area[i] = host_area[i];
    }
    __shared__ int last;
    __syncthreads();
    if (threadIdx.x == 0) {
        last = __hip_atomic_fetch_add(arrivals, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == static_cast<int>(gridDim.x) - 1;
        if (last) {
            __hip_atomic_store(arrivals, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // clean for the next job
            __hip_atomic_store(stamp_host, stamp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
}

struct ModelRun {
    int32_t hq = 0, hkv = 0;         // query and KV heads of ONE layer
    int32_t layers = 1, heads = 0;   // heads = layers * hkv = the scheduler's head count
    hipStream_t stream = nullptr;
    int32_t *tables = nullptr;       // DEVICE [layers][max_seqs][hkv][max_blocks], row = the scheduler's slot
    int32_t *job_tables = nullptr;   // DEVICE, same shape, row = position in the current prefill job
    void *decode_ws = nullptr, *prefill_ws = nullptr;
    size_t decode_ws_bytes = 0, prefill_ws_bytes = 0;
    int32_t *stage_dev = nullptr;    // DEVICE kRing areas
    int32_t *stage_host = nullptr;   // pinned HOST kRing areas, then one stamp per area (16 ints apart)
    int32_t *stage_host_dev = nullptr;   // the same memory as the GPU addresses it
    int *arrivals = nullptr;         // DEVICE: workgroups of the staging kernel that are done (zero between jobs)
    int32_t stamp_of[kRing] = {};    // what the staging kernel of the area's last job writes into its stamp; 0 = never used
    int32_t next_stamp = 1;
    int next_area = 0;
    hipEvent_t done = nullptr;       // everything launched for this model so far
    // buffers registered with mux_runner_set_buffers: [0] prefill, [1] decode
    void *reg_out[2] = {};
    const void *reg_q[2] = {}, *reg_k[2] = {}, *reg_v[2] = {};
    float reg_scale = 0.f;
    bool launched = false;           // since `done` was last recorded
    // the job whose arrays were staged and whose block ids were installed last (mux_runner_launch[_layer])
    struct Prepared {
        int64_t step = -1;               // scheduler iteration the job belongs to
        int32_t job = -1, kind = 0, n = 0, total = 0, longest = 0, rows = 0;
        const int32_t *seq = nullptr, *pos = nullptr, *cu = nullptr, *start = nullptr, *ctx = nullptr;   // DEVICE
        // decode job whose arrays are small enough to travel as kernel arguments of the attention
        // launch itself (no copy, no staging, no kernel ahead of it): see mux_inline_step
        bool as_arguments = false;
        int32_t n_entries = 0;
        int32_t inl[MUX_INLINE_STEP_INTS];
    } prep;
};

}  // namespace

struct mux_runner {
    mux_pool *pool = nullptr;
    mux_sched *sched = nullptr;
    int32_t max_seqs = 0, max_blocks = 0, max_tokens = 0;
    size_t area_ints = 0;
    std::vector<ModelRun> models;
    bool one_stream = true;
    int64_t jobs_launched = 0, seqs_launched = 0, steps = 0;
    bool stage_always = false;   // MUX_RUNNER_STAGE_ALWAYS=1 when the runner was created: never pass arrays as arguments
    std::vector<int64_t> ids64;
    std::vector<int32_t> slots, lens, flags;
};

namespace {

bool ok(hipError_t e)
{
    if (e == hipSuccess) return true;
    (void)hipGetLastError();
    return false;
}

void release(mux_runner *r)
{
    for (ModelRun &m : r->models) {
        (void)hipStreamSynchronize(m.stream);
        if (m.tables) (void)hipFree(m.tables);
        if (m.job_tables) (void)hipFree(m.job_tables);
        if (m.decode_ws) (void)hipFree(m.decode_ws);
        if (m.prefill_ws) (void)hipFree(m.prefill_ws);
        if (m.stage_dev) (void)hipFree(m.stage_dev);
        if (m.stage_host) (void)hipHostFree(m.stage_host);
        if (m.arrivals) (void)hipFree(m.arrivals);
        if (m.done) (void)hipEventDestroy(m.done);
    }
    delete r;
}

// Blocks a model gave back may be handed to any other model from now on: what that model has
// launched so far (the last readers of those blocks) comes before whatever is launched next on
// the other models' streams.  Its own stream is ordered anyway.
int order_after(mux_runner *r, ModelRun &m)
{
    if (r->one_stream || !m.launched) return MUX_OK;
    if (!ok(hipEventRecord(m.done, m.stream))) return MUX_ERR_HIP;
    for (ModelRun &other : r->models)
        if (other.stream != m.stream && !ok(hipStreamWaitEvent(other.stream, m.done, 0))) return MUX_ERR_HIP;
    m.launched = false;
    return MUX_OK;
}

constexpr int kStampStride = 16;   // ints between the stamps of two areas (a cache line of their own)

int32_t *stamp_word(const ModelRun &m, size_t area_ints, int area)
{
    return m.stage_host + static_cast<size_t>(kRing) * area_ints + static_cast<size_t>(area) * kStampStride;
}

// Claims the model's next staging area; waits (rarely: kRing jobs later) until the staging kernel
// of the area's last job has read it (that kernel's stamp in pinned memory says so).
int claim_area(ModelRun &m, size_t area_ints, int32_t **host, int32_t **dev, int *area)
{
    const int a = m.next_area;
    m.next_area = (a + 1) % kRing;
    if (m.stamp_of[a] != 0) {
        const int32_t *word = stamp_word(m, area_ints, a);
        long spins = 0;
        while (__atomic_load_n(word, __ATOMIC_ACQUIRE) != m.stamp_of[a]) {
            // the kernel is at most kRing jobs behind: this wait ends as soon as the stream gets there; the
            // runtime is asked now and then so that a failed stream ends the wait with an error
            if (++spins % 4096 == 0 && hipStreamQuery(m.stream) != hipErrorNotReady) {
                if (__atomic_load_n(word, __ATOMIC_ACQUIRE) == m.stamp_of[a]) break;
                (void)hipGetLastError();
                return MUX_ERR_HIP;
            }
        }
    }
    *host = m.stage_host + static_cast<size_t>(a) * area_ints;
    *dev = m.stage_dev + static_cast<size_t>(a) * area_ints;
    *area = a;
    return MUX_OK;
}

// Hands the filled area to the GPU: its first copy_ints ints go to the device twin, its entries
// (n_entries of them from entries_at, their ids from ids_at) into the tables.
int stage_and_install(mux_runner *r, ModelRun &m, int area, const int32_t *host, int32_t *dev, size_t copy_ints, int n_entries,
                      size_t entries_at, size_t ids_at, bool prefill)
{
    const int32_t stamp = m.next_stamp;
    m.next_stamp = stamp == 0x7fffffff ? 1 : stamp + 1;
    m.stamp_of[area] = stamp;
    const unsigned copy_wgs = static_cast<unsigned>(std::min<size_t>((copy_ints + 1023) / 1024, 64));
    const unsigned grid = static_cast<unsigned>(n_entries) + std::max(copy_wgs, n_entries == 0 ? 1u : 0u);
    const int32_t *host_as_gpu = m.stage_host_dev + (host - m.stage_host);
    int32_t *stamp_as_gpu = m.stage_host_dev + (stamp_word(m, r->area_ints, area) - m.stage_host);
    hipLaunchKernelGGL(stage_install_kernel, dim3(grid), dim3(256), 0, m.stream, host_as_gpu, dev, static_cast<int>(copy_ints), n_entries,
                       static_cast<int>(entries_at), static_cast<int>(ids_at), m.tables, prefill ? m.job_tables : nullptr, m.heads,
                       m.hkv, r->max_seqs, r->max_blocks, m.arrivals, stamp_as_gpu, stamp);
    return ok(hipGetLastError()) ? MUX_OK : MUX_ERR_HIP;
}

}  // namespace

extern "C" {

int mux_runner_create(mux_runner_t **out, mux_pool_t *pool, mux_sched_t *sched, const int32_t *n_q_heads, const int32_t *n_layers,
                      void *const *streams)
{
    if (!out || !pool || !sched || !n_q_heads || mux_sched_pool(sched) != pool) return MUX_ERR_INVALID;
    int32_t n_models = 0, max_seqs = 0, max_blocks = 0, budget = 0;
    mux_sched_geometry(sched, &n_models, &max_seqs, &max_blocks, &budget);
    for (int32_t i = 0; i < n_models; ++i) {
        const int32_t heads = mux_sched_heads(sched, i), layers = n_layers ? n_layers[i] : 1;
        if (layers <= 0 || heads % layers != 0) return MUX_ERR_INVALID;
        if (n_q_heads[i] <= 0 || n_q_heads[i] % (heads / layers) != 0) return MUX_ERR_INVALID;
    }
    const int64_t max_ctx = static_cast<int64_t>(max_blocks) * pool->block_size;
    if (max_ctx > 0x7fffffff) return MUX_ERR_UNSUPPORTED;
    mux_runner *r = new (std::nothrow) mux_runner();
    if (!r) return MUX_ERR_NOMEM;
    r->pool = pool;
    r->sched = sched;
    const char *stage = std::getenv("MUX_RUNNER_STAGE_ALWAYS");
    r->stage_always = stage && stage[0] == '1';
    r->max_seqs = max_seqs;
    r->max_blocks = max_blocks;
    // a prefill job holds at most `budget` tokens, or one request of any admissible length
    r->max_tokens = static_cast<int32_t>(std::max<int64_t>(budget, max_ctx));
    int32_t max_heads = 0;
    for (int32_t i = 0; i < n_models; ++i) max_heads = std::max(max_heads, mux_sched_heads(sched, i));
    const size_t prefill_ints = 2 * static_cast<size_t>(r->max_tokens) + (2 + kEntryInts) * static_cast<size_t>(max_seqs) + 1 +
                                (static_cast<size_t>(r->max_tokens) / pool->block_size + max_seqs) * max_heads;
    const size_t decode_ints = static_cast<size_t>(max_seqs) * (1 + kEntryInts + max_heads);
    r->area_ints = (std::max(prefill_ints, decode_ints) + 3) / 4 * 4;   // areas stay 16-byte aligned
    try {
        r->models.resize(static_cast<size_t>(n_models));
        r->ids64.resize(static_cast<size_t>(max_seqs));
        r->slots.resize(static_cast<size_t>(max_seqs));
        r->lens.resize(static_cast<size_t>(max_seqs));
        r->flags.resize(static_cast<size_t>(max_seqs));
    } catch (const std::bad_alloc &) {
        delete r;
        return MUX_ERR_NOMEM;
    }
    for (int32_t i = 0; i < n_models; ++i) {
        r->models[i].stream = streams ? static_cast<hipStream_t>(streams[i]) : nullptr;
        if (r->models[i].stream != r->models[0].stream) r->one_stream = false;
    }
    for (int32_t i = 0; i < n_models; ++i) {
        ModelRun &m = r->models[i];
        m.hq = n_q_heads[i];
        m.heads = mux_sched_heads(sched, i);
        m.layers = n_layers ? n_layers[i] : 1;
        m.hkv = m.heads / m.layers;
        const size_t table_bytes = static_cast<size_t>(max_seqs) * m.heads * max_blocks * sizeof(int32_t);
        // The split of long contexts depends on both the number of rows and the longest context, and
        // a small job can need more scratch than the largest one: size both workspaces for the worst
        // launch this scheduler can produce (all layers in one launch, or one layer at a time; a
        // prefill job holds 1 .. max_tokens rows behind contexts of up to max_ctx tokens).
        for (int32_t layers : {1, m.layers})
            m.decode_ws_bytes = std::max(m.decode_ws_bytes, mux_decode_workspace_upper_bound(pool, layers * max_seqs, m.hq, m.hkv,
                                                                                             static_cast<int32_t>(max_ctx)));
        m.prefill_ws_bytes = mux_prefill_workspace_bound(pool, r->max_tokens, static_cast<int32_t>(max_ctx), m.hq, m.hkv);
        bool good = m.decode_ws_bytes != 0;
        good = good && ok(hipMalloc(&m.tables, table_bytes)) && ok(hipMalloc(&m.job_tables, table_bytes));
        good = good && ok(hipMemset(m.tables, 0, table_bytes)) && ok(hipMemset(m.job_tables, 0, table_bytes));
        good = good && ok(hipMalloc(&m.decode_ws, m.decode_ws_bytes));
        good = good && (m.prefill_ws_bytes == 0 || ok(hipMalloc(&m.prefill_ws, m.prefill_ws_bytes)));
        good = good && ok(hipMalloc(&m.stage_dev, kRing * r->area_ints * sizeof(int32_t)));
        // pinned and mapped: the staging kernel reads the areas, and writes their stamps, in place
        const size_t stage_ints = kRing * r->area_ints + static_cast<size_t>(kRing) * kStampStride;
        good = good && ok(hipHostMalloc(&m.stage_host, stage_ints * sizeof(int32_t), hipHostMallocMapped | hipHostMallocPortable));
        if (good) std::memset(m.stage_host, 0, stage_ints * sizeof(int32_t));
        good = good && ok(hipHostGetDevicePointer(reinterpret_cast<void **>(&m.stage_host_dev), m.stage_host, 0));
        good = good && ok(hipMalloc(&m.arrivals, sizeof(int))) && ok(hipMemset(m.arrivals, 0, sizeof(int)));
        good = good && ok(hipEventCreateWithFlags(&m.done, hipEventDisableTiming));
        if (!good) {
            release(r);
            return MUX_ERR_HIP;
        }
    }
    if (!ok(hipDeviceSynchronize())) {   // the tables are cleared before any stream uses them
        release(r);
        return MUX_ERR_HIP;
    }
    *out = r;
    return MUX_OK;
}

int mux_runner_destroy(mux_runner_t *r)
{
    if (!r) return MUX_ERR_INVALID;
    release(r);
    return MUX_OK;
}

int mux_runner_step(mux_runner_t *r, int32_t *n_jobs)
{
    if (!r || !n_jobs) return MUX_ERR_INVALID;
    const int rc = mux_sched_step(r->sched, n_jobs);
    if (rc != MUX_OK) return rc;
    ++r->steps;
    for (size_t i = 0; i < r->models.size(); ++i)
        if (mux_sched_released_blocks(r->sched, static_cast<int32_t>(i))) {
            const int rc2 = order_after(r, r->models[i]);
            if (rc2 != MUX_OK) return rc2;
        }
    return MUX_OK;
}

// Stages the job's arrays, installs the block ids it brought and remembers where the arrays are:
// everything a launch needs apart from the K/V/Q values.  *model_out = the job's model, or -1 for
// a job that launches nothing (a preemption).
static int prepare_job(mux_runner_t *r, int32_t job, int32_t *model_out)
{
    int32_t kind = 0, model = 0, n = 0;
    int rc = mux_sched_job(r->sched, job, &kind, &model, &n);
    if (rc != MUX_OK) return rc;
    *model_out = -1;
    if (kind == MUX_JOB_PREEMPT || n == 0) return MUX_OK;
    if (n > r->max_seqs || (kind != MUX_JOB_PREFILL && kind != MUX_JOB_DECODE)) return MUX_ERR_INVALID;
    rc = mux_sched_job_seqs(r->sched, job, nullptr, r->slots.data(), r->lens.data(), r->flags.data());
    if (rc != MUX_OK) return rc;
    ModelRun &m = r->models[model];
    const int32_t *table = mux_sched_table(r->sched, model);
    const int32_t B = r->pool->block_size, heads = m.heads, cols = r->max_blocks;
    ModelRun::Prepared p;
    p.step = r->steps, p.job = job, p.kind = kind, p.n = n;

    if (kind == MUX_JOB_PREFILL) {
        int32_t *host = nullptr, *dev = nullptr;
        int area = 0;
        rc = claim_area(m, r->area_ints, &host, &dev, &area);
        if (rc != MUX_OK) return rc;
        int64_t total = 0, id_ints = 0;
        int32_t longest = 0;
        for (int32_t i = 0; i < n; ++i) {
            total += r->lens[i];
            id_ints += static_cast<int64_t>((r->lens[i] + B - 1) / B) * heads;
            longest = std::max(longest, r->lens[i]);
        }
        const size_t need = 2 * static_cast<size_t>(total) + 2 * static_cast<size_t>(n) + 1 + static_cast<size_t>(kEntryInts) * n +
                            static_cast<size_t>(id_ints);
        if (total > r->max_tokens || need > r->area_ints) return MUX_ERR_INVALID;
        // area: token -> job row | token -> position | chunk starts (n + 1) | tokens cached before (n zeros) | entries | ids
        int32_t *tok_seq = host, *tok_pos = host + total, *cu = host + 2 * total, *q_start = cu + n + 1;
        int32_t *entries = q_start + n, *ids = entries + kEntryInts * n;
        int32_t t = 0, at = 0;
        for (int32_t i = 0; i < n; ++i) {
            const int32_t len = r->lens[i], nb = (len + B - 1) / B, slot = r->slots[i];
            if (slot < 0 || slot >= r->max_seqs || nb > cols) return MUX_ERR_INVALID;
            cu[i] = t;
            q_start[i] = 0;
            for (int32_t pos = 0; pos < len; ++pos, ++t) {
                tok_seq[t] = i;
                tok_pos[t] = pos;
            }
            int32_t *e = entries + kEntryInts * i;
            e[0] = slot, e[1] = i, e[2] = 0, e[3] = nb, e[4] = at;
            const int32_t *row = table + static_cast<size_t>(slot) * heads * cols;
            for (int32_t h = 0; h < heads; ++h, at += nb) std::memcpy(ids + at, row + static_cast<size_t>(h) * cols, sizeof(int32_t) * nb);
        }
        cu[n] = t;
        // the per-token arrays and the chunk starts go to device memory, the entries and ids straight into the tables
        const size_t entries_at = 2 * static_cast<size_t>(total) + 2 * static_cast<size_t>(n) + 1;
        rc = stage_and_install(r, m, area, host, dev, entries_at, n, entries_at, entries_at + static_cast<size_t>(kEntryInts) * n, true);
        if (rc != MUX_OK) return rc;
        p.seq = dev, p.pos = dev + total, p.cu = dev + 2 * total, p.start = p.cu + n + 1;
        p.total = static_cast<int32_t>(total), p.longest = longest;
    } else {
        // arrays: context length per slot (0 = not in this step), up to the highest slot | entries | ids
        int32_t rows = 0, longest = 0, n_entries = 0;
        for (int32_t i = 0; i < n; ++i) {
            if (r->slots[i] < 0 || r->slots[i] >= r->max_seqs) return MUX_ERR_INVALID;
            rows = std::max(rows, r->slots[i] + 1);
            longest = std::max(longest, r->lens[i]);
            n_entries += (r->flags[i] & MUX_JOB_FLAG_TABLE) ? 1 : 0;
        }
        if (m.layers > 1) rows = r->max_seqs;   // the layers of the device table are max_seqs rows apart
        const size_t need = static_cast<size_t>(rows) + static_cast<size_t>(n_entries) * (kEntryInts + heads);
        if (need > r->area_ints) return MUX_ERR_INVALID;
        const size_t need_inline = 2 * static_cast<size_t>(rows) + static_cast<size_t>(n_entries) * heads;
        p.as_arguments = !r->stage_always && need_inline <= static_cast<size_t>(MUX_INLINE_STEP_INTS);
        if (p.as_arguments) {
            // context length per slot | index of the slot's entry or -1 | ids of the entries
            int32_t *ctx = p.inl, *entry_of = ctx + rows, *ids = entry_of + rows;
            std::fill(ctx, ctx + rows, 0);
            std::fill(entry_of, entry_of + rows, -1);
            int32_t e_at = 0;
            for (int32_t i = 0; i < n; ++i) {
                const int32_t slot = r->slots[i], len = r->lens[i];
                ctx[slot] = len;
                if (!(r->flags[i] & MUX_JOB_FLAG_TABLE)) continue;
                const int32_t col = (len - 1) / B;   // the block the appended token opened
                if (len <= 0 || col >= cols) return MUX_ERR_INVALID;
                entry_of[slot] = e_at;
                const int32_t *row = table + static_cast<size_t>(slot) * heads * cols;
                for (int32_t h = 0; h < heads; ++h) ids[e_at * heads + h] = row[static_cast<size_t>(h) * cols + col];
                ++e_at;
            }
            p.n_entries = n_entries;
            p.ctx = nullptr;
        } else {
            int32_t *host = nullptr, *dev = nullptr;
            int area = 0;
            rc = claim_area(m, r->area_ints, &host, &dev, &area);
            if (rc != MUX_OK) return rc;
            int32_t *ctx = host, *entries = host + rows, *ids = entries + kEntryInts * n_entries;
            std::fill(ctx, ctx + rows, 0);
            int32_t e_at = 0;
            for (int32_t i = 0; i < n; ++i) {
                const int32_t slot = r->slots[i], len = r->lens[i];
                ctx[slot] = len;
                if (!(r->flags[i] & MUX_JOB_FLAG_TABLE)) continue;
                const int32_t col = (len - 1) / B;   // the block the appended token opened
                if (len <= 0 || col >= cols) return MUX_ERR_INVALID;
                int32_t *e = entries + kEntryInts * e_at;
                e[0] = slot, e[1] = -1, e[2] = col, e[3] = 1, e[4] = e_at * heads;
                const int32_t *row = table + static_cast<size_t>(slot) * heads * cols;
                for (int32_t h = 0; h < heads; ++h) ids[e_at * heads + h] = row[static_cast<size_t>(h) * cols + col];
                ++e_at;
            }
            rc = stage_and_install(r, m, area, host, dev, rows, n_entries, rows, static_cast<size_t>(rows) + static_cast<size_t>(kEntryInts) * n_entries,
                                   false);
            if (rc != MUX_OK) return rc;
            p.ctx = dev;
        }
        p.rows = rows, p.longest = longest;
    }
    m.launched = true;
    m.prep = p;
    ++r->jobs_launched;
    r->seqs_launched += n;
    *model_out = model;
    return MUX_OK;
}

// Append + attention of the prepared job for layers l0 .. l1-1.  The buffers start at layer l0.
static int run_layers(mux_runner_t *r, ModelRun &m, int32_t l0, int32_t l1, void *out, const void *q, const void *k_new,
                      const void *v_new, float scale)
{
    const ModelRun::Prepared &p = m.prep;
    const int32_t cols = r->max_blocks;
    const size_t layer_cells = static_cast<size_t>(r->max_seqs) * m.hkv * cols;   // table entries of one layer
    if (p.kind == MUX_JOB_PREFILL) {
        // layer by layer: buffers are [layer][token][heads][d], the job's tables [layer][max_seqs rows][hkv][max_blocks]
        const size_t eb = static_cast<size_t>(r->pool->elem_bytes) * r->pool->head_dim * static_cast<size_t>(p.total);
        for (int32_t l = l0; l < l1; ++l) {
            const int32_t *tab = m.job_tables + l * layer_cells;
            const size_t at = static_cast<size_t>(l - l0) * eb;
            const char *kl = static_cast<const char *>(k_new) + at * m.hkv, *vl = static_cast<const char *>(v_new) + at * m.hkv;
            const char *ql = static_cast<const char *>(q) + at * m.hq;
            char *ol = static_cast<char *>(out) + at * m.hq;
            int rc = mux_kv_append(r->pool, kl, vl, p.seq, p.pos, tab, p.total, p.n, m.hkv, cols, m.stream);
            if (rc != MUX_OK) return rc;
            rc = mux_prefill_attn(r->pool, ol, ql, p.cu, p.start, tab, p.n, p.total, p.longest, p.longest, m.hq, m.hkv, cols, scale,
                                  m.prefill_ws, m.prefill_ws_bytes, m.stream);
            if (rc != MUX_OK) return rc;
        }
        return MUX_OK;
    }
    // one launch for the layers asked for (their tables follow one another)
    if (!p.as_arguments)
        return mux_decode_step(r->pool, out, q, k_new, v_new, m.tables + l0 * layer_cells, p.ctx, l1 - l0, p.rows, m.hq, m.hkv, cols,
                               p.longest, scale, m.decode_ws, m.decode_ws_bytes, m.stream);
    // the same launch with the job's arrays in its arguments: the attention kernel installs the new ids itself
    if (!out || !q || !k_new || !v_new || p.rows <= 0 || l1 <= l0) return MUX_ERR_INVALID;
    if (((reinterpret_cast<uintptr_t>(out) | reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k_new) |
          reinterpret_cast<uintptr_t>(v_new)) & 15u) != 0)
        return MUX_ERR_INVALID;
    if (p.longest > static_cast<int64_t>(cols) * r->pool->block_size) return MUX_ERR_INVALID;
    const mux_decode_plan plan = mux_plan_decode(r->pool, (l1 - l0) * p.rows, m.hq, m.hkv, std::max(p.longest, 1));
    if (plan.workspace_bytes > m.decode_ws_bytes) return MUX_ERR_INVALID;
    const mux_inline_step inl{p.inl, p.rows, p.n_entries, m.heads, l0 * m.hkv};
    return mux_launch_decode_step(r->pool, plan, out, q, k_new, v_new, m.tables + l0 * layer_cells, nullptr, l1 - l0, p.rows, m.hq,
                                  m.hkv, cols, p.longest, scale, m.decode_ws, m.stream, &inl);
}

int mux_runner_launch(mux_runner_t *r, int32_t job, void *out, const void *q, const void *k_new, const void *v_new, float scale)
{
    if (!r) return MUX_ERR_INVALID;
    int32_t kind = 0, model = 0, n = 0;
    int rc = mux_sched_job(r->sched, job, &kind, &model, &n);
    if (rc != MUX_OK) return rc;
    if (kind == MUX_JOB_PREEMPT || n == 0) return MUX_OK;
    if (!out || !q || !k_new || !v_new) return MUX_ERR_INVALID;
    rc = prepare_job(r, job, &model);
    if (rc != MUX_OK || model < 0) return rc;
    ModelRun &m = r->models[model];
    return run_layers(r, m, 0, m.layers, out, q, k_new, v_new, scale);
}

int mux_runner_launch_layer(mux_runner_t *r, int32_t job, int32_t layer, void *out, const void *q, const void *k_new,
                            const void *v_new, float scale)
{
    if (!r) return MUX_ERR_INVALID;
    int32_t kind = 0, model = 0, n = 0;
    int rc = mux_sched_job(r->sched, job, &kind, &model, &n);
    if (rc != MUX_OK) return rc;
    if (layer < 0 || layer >= r->models[model].layers) return MUX_ERR_INVALID;
    if (kind == MUX_JOB_PREEMPT || n == 0) return MUX_OK;
    if (!out || !q || !k_new || !v_new) return MUX_ERR_INVALID;
    ModelRun &m = r->models[model];
    if (layer == 0) {
        rc = prepare_job(r, job, &model);
        if (rc != MUX_OK) return rc;
    } else if (m.prep.step != r->steps || m.prep.job != job) {
        return MUX_ERR_INVALID;   // layer 0 of this job comes first
    }
    return run_layers(r, m, layer, layer + 1, out, q, k_new, v_new, scale);
}

int mux_runner_set_buffers(mux_runner_t *r, int32_t model, void *prefill_out, const void *prefill_q, const void *prefill_k,
                           const void *prefill_v, void *decode_out, const void *decode_q, const void *decode_k,
                           const void *decode_v, float scale)
{
    if (!r || model < 0 || model >= static_cast<int32_t>(r->models.size())) return MUX_ERR_INVALID;
    if (!prefill_out || !prefill_q || !prefill_k || !prefill_v || !decode_out || !decode_q || !decode_k || !decode_v)
        return MUX_ERR_INVALID;
    ModelRun &m = r->models[model];
    m.reg_out[0] = prefill_out, m.reg_q[0] = prefill_q, m.reg_k[0] = prefill_k, m.reg_v[0] = prefill_v;
    m.reg_out[1] = decode_out, m.reg_q[1] = decode_q, m.reg_k[1] = decode_k, m.reg_v[1] = decode_v;
    m.reg_scale = scale;
    return MUX_OK;
}

int mux_runner_run_step(mux_runner_t *r, int32_t *n_jobs)
{
    int rc = mux_runner_step(r, n_jobs);
    if (rc != MUX_OK) return rc;
    for (int32_t j = 0; j < *n_jobs; ++j) {
        int32_t kind = 0, model = 0, n = 0;
        rc = mux_sched_job(r->sched, j, &kind, &model, &n);
        if (rc != MUX_OK) return rc;
        if (kind == MUX_JOB_PREEMPT) continue;
        const ModelRun &m = r->models[model];
        const int which = kind == MUX_JOB_DECODE ? 1 : 0;
        if (!m.reg_out[which]) return MUX_ERR_INVALID;   // no buffers registered for this model
        rc = mux_runner_launch(r, j, m.reg_out[which], m.reg_q[which], m.reg_k[which], m.reg_v[which], m.reg_scale);
        if (rc != MUX_OK) return rc;
    }
    return MUX_OK;
}

int mux_runner_counts(const mux_runner_t *r, int64_t *counts)
{
    if (!r || !counts) return MUX_ERR_INVALID;
    counts[0] = r->jobs_launched;
    counts[1] = r->seqs_launched;
    return MUX_OK;
}

int mux_runner_synchronize(mux_runner_t *r)
{
    if (!r) return MUX_ERR_INVALID;
    for (ModelRun &m : r->models)
        if (!ok(hipStreamSynchronize(m.stream))) return MUX_ERR_HIP;
    return MUX_OK;
}

int mux_runner_read_table(mux_runner_t *r, int32_t model, int32_t *host_out)
{
    if (!r || model < 0 || model >= static_cast<int32_t>(r->models.size()) || !host_out) return MUX_ERR_INVALID;
    ModelRun &m = r->models[model];
    const size_t bytes = static_cast<size_t>(r->max_seqs) * m.heads * r->max_blocks * sizeof(int32_t);
    if (!ok(hipStreamSynchronize(m.stream)) || !ok(hipMemcpy(host_out, m.tables, bytes, hipMemcpyDeviceToHost))) return MUX_ERR_HIP;
    return MUX_OK;
}

}  // extern "C"
