// Decode attention for callers that cannot allocate: the same kernels as mux_decode_attn, with
// the call's scratch (work list and, for split contexts, the fp32 partial results of the
// spans) in a fixed array that is part of the library's device image instead of a buffer
// the caller brings.
//
// The array exists once per GPU (the runtime places a copy on every device that loads the
// library) and lives until the process ends.  Its name is only a handle on the host side:
// the device address is asked from the runtime once per device and kept, and that address -
// never the name - is what the kernels receive.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <mutex>

#include "mux_internal.h"

namespace {

static __device__ __align__(256) __attribute__((used)) unsigned char scratch[MUX_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void *g_scratch_of_device[kMaxDevices] = {};   // device address of `scratch` on each GPU, once known

// Address of the current device's copy of `scratch` (asked on first use per device).
int scratch_of_current_device(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return MUX_ERR_HIP;
    }
    std::lock_guard<std::mutex> guard(g_lock);
    if (g_scratch_of_device[dev] == nullptr) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
            (void)hipGetLastError();
            return MUX_ERR_HIP;
        }
        g_scratch_of_device[dev] = ptr;
    }
    *out = g_scratch_of_device[dev];
    return MUX_OK;
}

}  // namespace

extern "C" int mux_decode_attn_static(mux_pool_t *pool, void *out, const void *q, const int32_t *block_tables,
                                      const int32_t *ctx_lens, int32_t n_seqs, int32_t n_q_heads, int32_t n_kv_heads,
                                      int32_t max_blocks, int32_t max_ctx_len, float scale, void *stream)
{
    if (!pool || n_seqs < 0 || n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads != 0 || max_blocks < 0 ||
        max_ctx_len < 0)
        return MUX_ERR_INVALID;
    if (n_seqs == 0) return MUX_OK;
    if (!out || !q || !block_tables || !ctx_lens) return MUX_ERR_INVALID;
    if ((reinterpret_cast<uintptr_t>(out) & 15u) != 0 || (reinterpret_cast<uintptr_t>(q) & 15u) != 0) return MUX_ERR_INVALID;
    if (max_ctx_len > static_cast<int64_t>(max_blocks) * pool->block_size) return MUX_ERR_INVALID;
    const mux_decode_plan plan = mux_plan_decode(pool, n_seqs, n_q_heads, n_kv_heads, std::max(max_ctx_len, 1));
    if (plan.workspace_bytes > static_cast<size_t>(MUX_STATIC_SCRATCH_BYTES)) return MUX_ERR_TOO_LARGE;
    void *ws = nullptr;
    const int rc = scratch_of_current_device(&ws);
    if (rc != MUX_OK) return rc;
    // Nothing in the scratch has to start at zero: the work list is written in full by the
    // kernel that builds it, and every partial result that the merge reads was written by
    // this call's attention kernel.  What the previous call left there is never read.
    return mux_launch_decode_attn(pool, plan, out, q, block_tables, ctx_lens, n_seqs, n_q_heads, n_kv_heads, max_blocks,
                                  max_ctx_len, scale, ws, stream);
}
