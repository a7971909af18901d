// Ceiling probes: what the memory system and the matrix cores of the GPU at hand sustain with
// nothing else in the way.  They put the attention kernels' figures in context (fraction of the
// nominal peak is what is reported as the roofline; fraction of these is what a kernel could at
// best reach).  Not part of the attention path.
#include <hip/hip_runtime.h>

#include "mux_internal.h"
#include "mux_probes.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Plain streaming read: every wave takes whole contiguous 8 KiB chunks, 16 bytes per lane per
// load, non-temporal, 8 loads (one chunk) issued back to back.
__global__ __launch_bounds__(256) void probe_read_kernel(const char *src, long long n_chunks, unsigned *sink)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    u32x4 acc = {0, 0, 0, 0};
    for (long long c = static_cast<long long>(blockIdx.x) * 4 + wave; c < n_chunks; c += static_cast<long long>(gridDim.x) * 4) {
        const char *p = src + c * 8192 + lane * 16;
#pragma unroll
        for (int k = 0; k < 8; ++k) acc ^= __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p + k * 1024));
    }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) *sink = 1;   // keeps the loads alive
}

// Independent accumulating matrix instructions, 8 chains per wave.
__global__ __launch_bounds__(256) void probe_mfma_kernel(float *sink, int iters)
{
    const unsigned lane = threadIdx.x;
    f32x4 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    const bf16x8 a = __builtin_bit_cast(bf16x8, u32x4{0x3F803F80u + (lane << 16), 0x3F803F80u, 0x3F803F80u, 0x3F803F80u});
    const bf16x8 b = __builtin_bit_cast(bf16x8, u32x4{0x3F003F00u, 0x3F003F00u + (lane << 16), 0x3F003F00u, 0x3F003F00u});
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    if (s == 12345.678f) *sink = s;
}

}  // namespace

extern "C" {

int mux_probe_stream_read(const void *buf, size_t bytes, void *sink, int32_t workgroups, void *stream)
{
    if (!buf || !sink || bytes < 8192 || workgroups <= 0 || (reinterpret_cast<size_t>(buf) & 15) != 0) return MUX_ERR_INVALID;
    hipLaunchKernelGGL(probe_read_kernel, dim3(static_cast<unsigned>(workgroups)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const char *>(buf), static_cast<long long>(bytes / 8192), static_cast<unsigned *>(sink));
    return hipGetLastError() == hipSuccess ? MUX_OK : MUX_ERR_HIP;
}

int mux_probe_mfma(void *sink, int32_t workgroups, int32_t iters, double *flops, void *stream)
{
    if (!sink || workgroups <= 0 || iters <= 0) return MUX_ERR_INVALID;
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(static_cast<unsigned>(workgroups)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<float *>(sink), iters);
    if (flops) *flops = static_cast<double>(workgroups) * 4.0 * iters * 16.0 * (2.0 * 16 * 16 * 32);
    return hipGetLastError() == hipSuccess ? MUX_OK : MUX_ERR_HIP;
}

}  // extern "C"
