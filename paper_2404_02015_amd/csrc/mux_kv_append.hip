// KV append: scatter the new tokens' K/V rows into their head-wise blocks.
//
// MuxServe, Section 3.4 (Implementation): an engine writes the K/V of new tokens into the
// cache blocks the memory manager assigned to it.  Here one thread moves one 16-byte piece
// of a K row and the matching piece of the V row; the pieces of a row are handled by
// neighbouring lanes, so both the dense source rows and the destination rows inside a
// block are read and written with coalesced 16-byte accesses.  Pure bit copy, bounded by
// HBM bandwidth (2 * n_tokens * n_kv_heads * head_dim * elem_bytes read and written).
#include <hip/hip_runtime.h>

#include "mux_internal.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void kv_append_kernel(
    char *__restrict__ kv_base, const long long block_bytes, const long long num_blocks, const int block_size,
    const int pieces_per_row,  // head_dim * elem_bytes / 16
    const u32x4 *__restrict__ k_new, const u32x4 *__restrict__ v_new, const int *__restrict__ tok_seq,
    const int *__restrict__ tok_pos, const int *__restrict__ tables, const long long n_pieces, const int n_seqs,
    const int n_kv_heads, const int max_blocks)
{
    const long long idx = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (idx >= n_pieces) return;
    const int piece = static_cast<int>(idx % pieces_per_row);
    const long long row = idx / pieces_per_row;  // = t * n_kv_heads + h
    const int h = static_cast<int>(row % n_kv_heads);
    const int t = static_cast<int>(row / n_kv_heads);
    const int s = tok_seq[t];
    const int pos = tok_pos[t];
    if (s < 0 || s >= n_seqs || pos < 0) return;
    const int j = pos / block_size;
    if (j >= max_blocks) return;
    const int id = tables[(static_cast<long long>(s) * n_kv_heads + h) * max_blocks + j];
    if (id < 0 || id >= num_blocks) return;
    const int slot = pos - j * block_size;
    const long long row_bytes = 16LL * pieces_per_row;
    char *k_dst = kv_base + id * block_bytes + slot * row_bytes + 16LL * piece;
    char *v_dst = k_dst + block_size * row_bytes;
    *reinterpret_cast<u32x4 *>(k_dst) = k_new[idx];
    *reinterpret_cast<u32x4 *>(v_dst) = v_new[idx];
}

}  // namespace

int mux_launch_kv_append(const mux_pool *pool, const void *k_new, const void *v_new, const int32_t *tok_seq,
                         const int32_t *tok_pos, const int32_t *tables, int32_t n_tokens, int32_t n_seqs,
                         int32_t n_kv_heads, int32_t max_blocks, void *stream)
{
    const int pieces_per_row = pool->head_dim * pool->elem_bytes / 16;
    const long long n_pieces = static_cast<long long>(n_tokens) * n_kv_heads * pieces_per_row;
    const long long n_groups = (n_pieces + 255) / 256;
    if (n_groups > 0x7fffffffLL) return MUX_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(kv_append_kernel, dim3(static_cast<unsigned>(n_groups)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), pool->kv_base, static_cast<long long>(pool->block_bytes),
                       static_cast<long long>(pool->num_blocks), pool->block_size, pieces_per_row,
                       static_cast<const u32x4 *>(k_new), static_cast<const u32x4 *>(v_new), tok_seq, tok_pos, tables,
                       n_pieces, n_seqs, n_kv_heads, max_blocks);
    return hipGetLastError() == hipSuccess ? MUX_OK : MUX_ERR_HIP;
}
