// The library used through its C ABI alone (include/mux.h + the HIP runtime for device memory):
// no Python, no torch.  Two checks, both with exact expected results:
//   1. one sequence, one cached token: decode attention must return that token's V row bit for
//      bit (a softmax over a single key has weight 1), through alloc -> append -> decode;
//   2. the batch scheduler and the job runner serve a small stream of requests for two models
//      until it is drained; every request must finish and every block must be back in the pool.
// Prints "c_abi_demo OK" and exits 0, or says what failed and exits 1.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "mux.h"

#define CHECK(cond)                                                              \
    do {                                                                         \
        if (!(cond)) {                                                           \
            std::fprintf(stderr, "c_abi_demo: %s failed (line %d)\n", #cond, __LINE__); \
            return 1;                                                            \
        }                                                                        \
    } while (0)

int main()
{
    const int32_t B = 16, d = 128;
    const int64_t n_blocks = 4096;
    const size_t block_bytes = 2 * B * d * 2;
    void *kv = nullptr;
    CHECK(hipMalloc(&kv, n_blocks * block_bytes) == hipSuccess);
    CHECK(hipMemset(kv, 0, n_blocks * block_bytes) == hipSuccess);
    mux_pool_t *pool = nullptr;
    CHECK(mux_pool_create(&pool, kv, n_blocks * block_bytes, n_blocks, B, d, MUX_BF16, nullptr) == MUX_OK);

    // ---- 1. a single cached token comes back exactly -------------------------------------
    const int32_t hq = 4, hkv = 2, max_blocks = 4;
    int32_t ids[2];
    CHECK(mux_alloc_blocks(pool, 7, hkv, ids) == MUX_OK);
    CHECK(ids[0] == 0 && ids[1] == 1);                       // a fresh pool hands out 0, 1, ...
    std::vector<int32_t> table(hkv * max_blocks, -1);
    for (int h = 0; h < hkv; ++h) table[h * max_blocks] = ids[h];
    std::vector<uint16_t> k(hkv * d), v(hkv * d), q(hq * d, 0x3F80 /* 1.0 */), out(hq * d, 0);
    for (int i = 0; i < hkv * d; ++i) {
        k[i] = static_cast<uint16_t>(0x3C00 + i);            // small positive bf16 values
        v[i] = static_cast<uint16_t>(0xBE00 + 3 * i);        // negative ones, all different
    }
    const int32_t zero = 0, one = 1;
    void *d_k, *d_v, *d_q, *d_out, *d_table, *d_seq, *d_pos, *d_ctx, *d_ws;
    const size_t ws_bytes = mux_decode_workspace_bytes(pool, 1, hq, hkv, 1);
    CHECK(ws_bytes > 0);
    CHECK(hipMalloc(&d_k, k.size() * 2) == hipSuccess && hipMalloc(&d_v, v.size() * 2) == hipSuccess);
    CHECK(hipMalloc(&d_q, q.size() * 2) == hipSuccess && hipMalloc(&d_out, out.size() * 2) == hipSuccess);
    CHECK(hipMalloc(&d_table, table.size() * 4) == hipSuccess && hipMalloc(&d_seq, 4) == hipSuccess);
    CHECK(hipMalloc(&d_pos, 4) == hipSuccess && hipMalloc(&d_ctx, 4) == hipSuccess && hipMalloc(&d_ws, ws_bytes) == hipSuccess);
    CHECK(hipMemcpy(d_k, k.data(), k.size() * 2, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(hipMemcpy(d_v, v.data(), v.size() * 2, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(hipMemcpy(d_q, q.data(), q.size() * 2, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(hipMemcpy(d_table, table.data(), table.size() * 4, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(hipMemcpy(d_seq, &zero, 4, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(hipMemcpy(d_pos, &zero, 4, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(hipMemcpy(d_ctx, &one, 4, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(mux_kv_append(pool, d_k, d_v, static_cast<int32_t *>(d_seq), static_cast<int32_t *>(d_pos),
                        static_cast<int32_t *>(d_table), 1, 1, hkv, max_blocks, nullptr) == MUX_OK);
    CHECK(mux_decode_attn(pool, d_out, d_q, static_cast<int32_t *>(d_table), static_cast<int32_t *>(d_ctx), 1, hq, hkv, max_blocks,
                          1, 0.0884f, d_ws, ws_bytes, nullptr) == MUX_OK);
    CHECK(hipDeviceSynchronize() == hipSuccess);
    CHECK(hipMemcpy(out.data(), d_out, out.size() * 2, hipMemcpyDeviceToHost) == hipSuccess);
    for (int i = 0; i < hq; ++i)
        CHECK(std::memcmp(&out[i * d], &v[(i / (hq / hkv)) * d], d * 2) == 0);
    // the row also sits where the layout says: block ids[h], K tile then V tile, slot 0
    std::vector<uint16_t> blk(2 * B * d);
    CHECK(hipMemcpy(blk.data(), static_cast<char *>(kv) + ids[1] * block_bytes, block_bytes, hipMemcpyDeviceToHost) == hipSuccess);
    CHECK(std::memcmp(&blk[0], &k[d], d * 2) == 0 && std::memcmp(&blk[B * d], &v[d], d * 2) == 0);

    // ---- 2. scheduler + runner drain a request stream ----------------------------------------
    const int32_t heads[2] = {2, 4}, q_heads[2] = {4, 8};
    mux_sched_config cfg{};
    cfg.n_models = 2, cfg.heads = heads, cfg.max_seqs = 8, cfg.max_blocks = 16, cfg.max_prefill_tokens = 128;
    cfg.adapt_period = 8, cfg.low_util = 0.5, cfg.high_util = 0.9, cfg.step_fraction = 0.5;
    const double weights[2] = {1.0, 2.0};
    CHECK(mux_pool_set_quota(pool, 7, 2) == MUX_OK);         // model 7 keeps its two blocks and takes no more
    CHECK(mux_pool_init_quotas(pool, 2, weights) == MUX_OK);
    mux_sched_t *sched = nullptr;
    CHECK(mux_sched_create(&sched, pool, &cfg) == MUX_OK);
    mux_runner_t *runner = nullptr;
    CHECK(mux_runner_create(&runner, pool, sched, q_heads, nullptr, nullptr) == MUX_OK);
    const size_t max_tokens = 16 * 16;                       // max(max_prefill_tokens, max_blocks x block_size)
    void *buf[2][8];
    for (int m = 0; m < 2; ++m) {
        const size_t rows[2] = {max_tokens, 8};
        for (int set = 0; set < 2; ++set) {
            const size_t qb = rows[set] * q_heads[m] * d * 2, kb = rows[set] * heads[m] * d * 2;
            CHECK(hipMalloc(&buf[m][4 * set + 0], qb) == hipSuccess && hipMalloc(&buf[m][4 * set + 1], qb) == hipSuccess);
            CHECK(hipMalloc(&buf[m][4 * set + 2], kb) == hipSuccess && hipMalloc(&buf[m][4 * set + 3], kb) == hipSuccess);
            CHECK(hipMemset(buf[m][4 * set + 1], 0, qb) == hipSuccess && hipMemset(buf[m][4 * set + 2], 0, kb) == hipSuccess);
            CHECK(hipMemset(buf[m][4 * set + 3], 0, kb) == hipSuccess);
        }
        CHECK(mux_runner_set_buffers(runner, m, buf[m][0], buf[m][1], buf[m][2], buf[m][3], buf[m][4], buf[m][5], buf[m][6],
                                     buf[m][7], 0.0884f) == MUX_OK);
    }
    const int n_requests = 20;
    for (int r = 0; r < n_requests; ++r)
        CHECK(mux_sched_submit(sched, r % 2, 1000 + r, 5 + 11 * r % 90, 1 + 7 * r % 40) == MUX_OK);
    CHECK(mux_sched_submit(sched, 0, 1, 250, 10) == MUX_ERR_INVALID);   // 259 cached tokens do not fit 16 columns
    int64_t c0[5], c1[5];
    int passes = 0;
    for (; passes < 5000; ++passes) {
        int32_t n_jobs = 0;
        CHECK(mux_runner_run_step(runner, &n_jobs) == MUX_OK);
        CHECK(mux_sched_counts(sched, 0, c0) == MUX_OK && mux_sched_counts(sched, 1, c1) == MUX_OK);
        if (c0[0] + c0[1] + c1[0] + c1[1] == 0 && n_jobs == 0) break;
    }
    CHECK(mux_runner_synchronize(runner) == MUX_OK);
    CHECK(c0[2] + c1[2] == n_requests);
    CHECK(mux_pool_num_free(pool) == n_blocks - 2 && mux_pool_num_used(pool, 0) == 0 && mux_pool_num_used(pool, 1) == 0);
    int64_t launched[2];
    CHECK(mux_runner_counts(runner, launched) == MUX_OK && launched[1] >= n_requests);
    CHECK(mux_runner_destroy(runner) == MUX_OK && mux_sched_destroy(sched) == MUX_OK);
    CHECK(mux_free_blocks(pool, 7, 2, ids) == MUX_OK && mux_pool_num_free(pool) == n_blocks);
    CHECK(mux_pool_destroy(pool) == MUX_OK);
    std::printf("c_abi_demo OK: single-token decode exact; %d requests served in %d scheduler passes, %lld sequences launched\n",
                n_requests, passes, static_cast<long long>(launched[1]));
    return 0;
}
