// placeholder until the MFMA kernel lands
#include <hip/hip_runtime.h>
#include "mux_internal.h"
int mux_launch_prefill_attn(const mux_pool *, void *, const void *, const int32_t *, const int32_t *, const int32_t *,
                            int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, float, void *)
{
    return MUX_ERR_UNSUPPORTED;
}
