// Streams restricted to a subset of the compute units: the analogue, on this hardware, of the
// per-job SM shares the paper's parallel runtime sets with MPS (Section 3.4: computation
// resources of an LLM unit are managed at SM granularity and assigned to prefill and decoding
// jobs).  A kernel launched on such a stream only runs on the compute units whose bit is set.
#include <hip/hip_runtime.h>

#include "mux_internal.h"

extern "C" {

int mux_device_cu_count(int32_t *out)
{
    if (!out) return MUX_ERR_INVALID;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
        (void)hipGetLastError();
        return MUX_ERR_HIP;
    }
    *out = cus;
    return MUX_OK;
}

int mux_stream_create_masked(void **out_stream, const uint32_t *cu_mask, int32_t n_words)
{
    if (!out_stream || !cu_mask || n_words <= 0 || n_words > 64) return MUX_ERR_INVALID;
    bool any = false;
    for (int32_t i = 0; i < n_words; ++i) any = any || cu_mask[i] != 0;
    if (!any) return MUX_ERR_INVALID;   // a stream without compute units could never run anything
    hipStream_t s = nullptr;
    if (hipExtStreamCreateWithCUMask(&s, static_cast<uint32_t>(n_words), cu_mask) != hipSuccess) {
        (void)hipGetLastError();
        return MUX_ERR_HIP;
    }
    *out_stream = s;
    return MUX_OK;
}

int mux_stream_destroy(void *stream)
{
    if (!stream) return MUX_ERR_INVALID;
    if (hipStreamDestroy(static_cast<hipStream_t>(stream)) != hipSuccess) {
        (void)hipGetLastError();
        return MUX_ERR_HIP;
    }
    return MUX_OK;
}

}  // extern "C"
