// Chunked causal prefill attention over the unified head-wise paged KV pool (gfx950).
//
// MuxServe, Section 2.1: the prefill phase processes all prompt tokens in parallel and is the
// compute-heavy phase; Section 3.4: its K/V live in the same head-wise blocks as everyone
// else's.  Row r of a chunk sits at absolute position q_start + r and attends to keys 0..that
// position; the chunk's own K/V were appended before the call.
//
// The work is two dense contractions per (query tile, KV tile), so it runs on the matrix cores
// (v_mfma_f32_16x16x32_bf16), arranged so that no register shuffling sits between them:
//   S^T = K . Q^T   A = K tile  [16 tokens x 32 dims per instruction, from LDS]
//                   B = Q^T     [held in registers for the whole kernel]
//                   C = S^T     lane (g, c) holds tokens 4g..4g+3 of query row c
//   O^T = V^T . P^T A = V^T     [16 dims x 32 tokens, from an LDS copy transposed on store]
//                   B = P^T     = the S^T registers after softmax, rounded to bf16 in place
//                   C = O^T     lane (g, c) holds dims 4g..4g+3 of query row c
// Both results keep the query row in the lane's low 4 bits, so the running max / sum of a row
// and the rescaling of its accumulator never leave the lane group.
//
// A workgroup of 4 waves owns one (sequence, kv head) and a tile of 16-row slices: 4 row slices
// of one head for multi-head attention, or fewer row slices times several query heads of the
// group for grouped-query attention; all waves share the K/V tiles, which are fetched once per
// workgroup with coalesced 16-byte loads, double-buffered in LDS, 32 tokens per step.
//
// Pools in fp32 or with a block size other than 16 take a slow generic path (each query row
// handled like a decode step); see mux_launch_prefill_attn.
#include <hip/hip_runtime.h>

#include "mux_internal.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr int kBS = 16;            // tokens per block on this path
constexpr int kKT = 32;            // tokens per pipeline step (two blocks)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -3.0e38f;

struct PrefillArgs {
    const char *kv_base;
    long long block_bytes;
    int num_blocks;
    void *out;
    const void *q;
    const int *cu_q_lens;
    const int *q_start;
    const int *tables;
    int n_seqs, total_q, n_q_heads, n_kv_heads, max_blocks;
    int n_row_tiles;   // ceil(max_q_len / rows per workgroup)
    int n_passes;      // head passes per kv head
    float scale_log2e;
};

__device__ __forceinline__ unsigned pack_bf16(float a, float b)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 v = {static_cast<__bf16>(a), static_cast<__bf16>(b)};  // round to nearest even
    return __builtin_bit_cast(unsigned, v);
}

// D: head size.  HT: query heads per workgroup (1, 2 or 4); the other kWaves / HT waves take
// further 16-row slices.
template <int D, int HT>
__global__ __launch_bounds__(kThreads) void prefill_attn_kernel(const PrefillArgs a)
{
    constexpr int RT = kWaves / HT;              // 16-row slices per workgroup
    constexpr int QT = 16 * RT;                  // query rows per workgroup
    constexpr int KC = D / 32;                   // 32-dim slabs of the head
    constexpr int NT = D / 16;                   // 16-dim slabs of the output
    constexpr int KROW = D * 2 + 16;             // bytes per K row in LDS (padded: conflict-free 16-byte reads)
    constexpr int VROW = kKT * 2 + 16;           // bytes per V^T row in LDS
    constexpr int KBUF = kKT * KROW;
    constexpr int VBUF = D * VROW;
    constexpr int PIECES = kKT * D * 2 / 16;     // 16-byte pieces per K (or V) step
    constexpr int PPT = PIECES / kThreads;       // pieces per thread
    static_assert(PIECES % kThreads == 0, "tile must split evenly over the workgroup");
    constexpr int PPR = D * 2 / 16;              // pieces per token row

    __shared__ __attribute__((aligned(16))) char smem[2 * (KBUF + VBUF)];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;

    // blockIdx -> (row tile, sequence, kv head, pass); later row tiles (more keys) first
    int w = blockIdx.x;
    const int pass = w % a.n_passes;      w /= a.n_passes;
    const int kvh = w % a.n_kv_heads;     w /= a.n_kv_heads;
    const int s = w % a.n_seqs;           w /= a.n_seqs;
    const int tile = a.n_row_tiles - 1 - w;

    const int q_lo = a.cu_q_lens[s];
    const int q_len = min(a.cu_q_lens[s + 1], a.total_q) - q_lo;   // never past the packed q / out
    const int start = a.q_start[s];
    const int row0 = tile * QT;                  // first chunk row of this workgroup
    if (q_lo < 0 || row0 >= q_len || start < 0) return;
    const int rows_here = min(QT, q_len - row0);
    int kv_end = start + row0 + rows_here;       // keys 0 .. kv_end-1 are visible to the last row
    kv_end = min(kv_end, a.max_blocks * kBS);
    const int n_steps = (kv_end + kKT - 1) / kKT;
    const int total_len = start + q_len;         // tokens of this sequence that hold real K/V

    const int group = a.n_q_heads / a.n_kv_heads;
    const int slice = wave / HT;                 // which 16-row slice
    const int head_in_group = pass * HT + wave % HT;
    const bool head_ok = head_in_group < group;
    const int head = kvh * group + min(head_in_group, group - 1);
    const int my_row0 = row0 + slice * 16;       // first chunk row of this wave
    const bool wave_active = head_ok && my_row0 < q_len;
    const int my_row = min(my_row0 + c, q_len - 1);   // clamp: surplus rows repeat the last one
    const int my_pos = start + my_row;                // absolute position of this lane's row
    const int wave_last_pos = start + min(my_row0 + 15, q_len - 1);

    // Q^T operand: lane (g, c) holds dims 32k + 8g .. +8 of row c, for every slab k
    bf16x8 qreg[KC];
    {
        const char *qrow = static_cast<const char *>(a.q) + (static_cast<long long>(q_lo + my_row) * a.n_q_heads + head) * (D * 2);
#pragma unroll
        for (int k = 0; k < KC; ++k)
            qreg[k] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(qrow + (32 * k + 8 * g) * 2));
    }

    f32x4 acc[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) acc[n] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = kNegBig, l_run = 0.f;          // l_run: this lane's share of the row sum

    const int *trow = a.tables + (static_cast<long long>(s) * a.n_kv_heads + kvh) * a.max_blocks;

    // global -> registers for one step (K and V pieces of two blocks)
    u32x4 kreg[PPT], vreg[PPT];
    auto fetch = [&](int step) {
#pragma unroll
        for (int p = 0; p < PPT; ++p) {
            const int i = tid + kThreads * p;            // piece index inside the 32-token step
            const int tok = i / PPR;                     // 0..31
            const int blk = step * 2 + tok / kBS;
            int id = blk < a.max_blocks ? trow[blk] : 0;
            id = min(max(id, 0), a.num_blocks - 1);      // a stale or corrupt entry must not leave the pool
            const char *src = a.kv_base + static_cast<long long>(id) * a.block_bytes + (tok % kBS) * (D * 2) + (i % PPR) * 16;
            kreg[p] = *reinterpret_cast<const u32x4 *>(src);
            vreg[p] = *reinterpret_cast<const u32x4 *>(src + kBS * D * 2);
        }
    };
    // registers -> LDS: K rows as they are, V transposed ([dim][token]); slots past the
    // sequence's tokens hold stale bytes (possibly NaN) and are zeroed so that 0 * x stays 0
    auto stage = [&](int step, int buf) {
        char *kb = smem + buf * (KBUF + VBUF);
        char *vb = kb + KBUF;
#pragma unroll
        for (int p = 0; p < PPT; ++p) {
            const int i = tid + kThreads * p;
            const int tok = i / PPR, piece = i % PPR;
            const bool real = step * kKT + tok < total_len;
            const u32x4 kk = real ? kreg[p] : u32x4{0, 0, 0, 0};
            const u32x4 vv = real ? vreg[p] : u32x4{0, 0, 0, 0};
            *reinterpret_cast<u32x4 *>(kb + tok * KROW + piece * 16) = kk;
            unsigned short *vt = reinterpret_cast<unsigned short *>(vb + (piece * 8) * VROW + tok * 2);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                vt[(2 * e) * (VROW / 2)] = static_cast<unsigned short>(vv[e] & 0xffffu);
                vt[(2 * e + 1) * (VROW / 2)] = static_cast<unsigned short>(vv[e] >> 16);
            }
        }
    };

    if (n_steps > 0) fetch(0);
    for (int step = 0; step < n_steps; ++step) {
        const int buf = step & 1;
        stage(step, buf);
        if (step + 1 < n_steps) fetch(step + 1);
        __syncthreads();
        const int kv0 = step * kKT;
        if (wave_active && kv0 <= wave_last_pos) {
            const char *kb = smem + buf * (KBUF + VBUF);
            const char *vb = kb + KBUF;
            // S^T for the two 16-token halves
            f32x4 st[2];
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                st[hf] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int k = 0; k < KC; ++k) {
                    const bf16x8 kop = __builtin_bit_cast(
                        bf16x8, *reinterpret_cast<const u32x4 *>(kb + (hf * 16 + c) * KROW + (32 * k + 8 * g) * 2));
                    st[hf] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop, qreg[k], st[hf], 0, 0, 0);
                }
            }
            // scale, causal mask (only steps that touch the diagonal), online softmax
            const bool diag = kv0 + kKT - 1 > start + my_row0;   // wave-uniform
            float sc[8];
            float mx = kNegBig;
#pragma unroll
            for (int hf = 0; hf < 2; ++hf)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float x = st[hf][i] * a.scale_log2e;
                    if (diag && kv0 + hf * 16 + 4 * g + i > my_pos) x = kNegBig;
                    sc[hf * 4 + i] = x;
                    mx = fmaxf(mx, x);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run, mx);
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            float psum = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                float e = __builtin_amdgcn_exp2f(sc[j] - m_new);
                if (diag && sc[j] == kNegBig) e = 0.f;
                sc[j] = e;
                psum += e;
            }
            l_run = l_run * alpha + psum;
            m_run = m_new;
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
                for (int n = 0; n < NT; ++n) acc[n] *= alpha;
            }
            // P^T operand: k-slot j of lane group g is token 4g+j of half 0 (j < 4) or half 1
            u32x4 pw;
            pw[0] = pack_bf16(sc[0], sc[1]);
            pw[1] = pack_bf16(sc[2], sc[3]);
            pw[2] = pack_bf16(sc[4], sc[5]);
            pw[3] = pack_bf16(sc[6], sc[7]);
            const bf16x8 pop = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
            for (int n = 0; n < NT; ++n) {
                const char *vrow = vb + (16 * n + c) * VROW + (4 * g) * 2;
                const u32x2 lo = *reinterpret_cast<const u32x2 *>(vrow);        // tokens 4g..4g+3 of half 0
                const u32x2 hi = *reinterpret_cast<const u32x2 *>(vrow + 32);   // same of half 1
                const bf16x8 vop = __builtin_bit_cast(bf16x8, u32x4{lo[0], lo[1], hi[0], hi[1]});
                acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, pop, acc[n], 0, 0, 0);
            }
        }
    }

    if (!wave_active) return;
    float l_tot = l_run + __shfl_xor(l_run, 16);
    l_tot += __shfl_xor(l_tot, 32);
    if (my_row0 + c >= q_len) return;            // surplus row of a ragged tile
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    char *orow = static_cast<char *>(a.out) + (static_cast<long long>(q_lo + my_row) * a.n_q_heads + head) * (D * 2);
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        u32x2 o;
        o[0] = pack_bf16(acc[n][0] * inv, acc[n][1] * inv);
        o[1] = pack_bf16(acc[n][2] * inv, acc[n][3] * inv);
        *reinterpret_cast<u32x2 *>(orow + (16 * n + 4 * g) * 2) = o;   // dims 16n+4g .. +3 of this row
    }
}

template <int D, int HT>
void launch_mfma(const PrefillArgs &a, int max_q_len, hipStream_t st, PrefillArgs &scratch)
{
    constexpr int QT = 16 * (kWaves / HT);
    scratch = a;
    scratch.n_row_tiles = (max_q_len + QT - 1) / QT;
    const int group = a.n_q_heads / a.n_kv_heads;
    scratch.n_passes = (group + HT - 1) / HT;
    const long long grid = static_cast<long long>(scratch.n_row_tiles) * a.n_seqs * a.n_kv_heads * scratch.n_passes;
    hipLaunchKernelGGL((prefill_attn_kernel<D, HT>), dim3(static_cast<unsigned>(grid)), dim3(kThreads), 0, st, scratch);
}

}  // namespace

// Generic path (any supported dtype / block size): defined next to the decode kernel, which it reuses.
int mux_launch_prefill_rows_as_decode(const mux_pool *pool, void *out, const void *q, const int32_t *cu_q_lens,
                                      const int32_t *q_start, const int32_t *tables, int32_t n_seqs, int32_t total_q,
                                      int32_t max_ctx_len, int32_t n_q_heads, int32_t n_kv_heads, int32_t max_blocks,
                                      float scale, void *workspace, void *stream);

bool mux_prefill_uses_mfma(const mux_pool *pool) { return pool->dtype == MUX_BF16 && pool->block_size == kBS; }

int mux_launch_prefill_attn(const mux_pool *pool, void *out, const void *q, const int32_t *cu_q_lens,
                            const int32_t *q_start, const int32_t *tables, int32_t n_seqs, int32_t total_q,
                            int32_t max_q_len, int32_t max_ctx_len, int32_t n_q_heads, int32_t n_kv_heads,
                            int32_t max_blocks, float scale, void *workspace, void *stream)
{
    if (!mux_prefill_uses_mfma(pool))
        return mux_launch_prefill_rows_as_decode(pool, out, q, cu_q_lens, q_start, tables, n_seqs, total_q, max_ctx_len,
                                                 n_q_heads, n_kv_heads, max_blocks, scale, workspace, stream);
    PrefillArgs a{};
    a.kv_base = pool->kv_base;
    a.block_bytes = pool->block_bytes;
    a.num_blocks = static_cast<int>(pool->num_blocks);
    a.out = out;
    a.q = q;
    a.cu_q_lens = cu_q_lens;
    a.q_start = q_start;
    a.tables = tables;
    a.n_seqs = n_seqs;
    a.total_q = total_q;
    a.n_q_heads = n_q_heads;
    a.n_kv_heads = n_kv_heads;
    a.max_blocks = max_blocks;
    a.scale_log2e = scale * kLog2e;
    const int group = n_q_heads / n_kv_heads;
    const int ht = group >= 4 ? 4 : (group >= 2 ? 2 : 1);
    const long long rows_per_wg = 16 * (kWaves / ht);
    const long long grid = ((max_q_len + rows_per_wg - 1) / rows_per_wg) * n_seqs * n_kv_heads * ((group + ht - 1) / ht);
    if (grid > 0x7fffffffLL) return MUX_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    PrefillArgs launched;
    if (pool->head_dim == 128) {
        if (ht == 4) launch_mfma<128, 4>(a, max_q_len, st, launched);
        else if (ht == 2) launch_mfma<128, 2>(a, max_q_len, st, launched);
        else launch_mfma<128, 1>(a, max_q_len, st, launched);
    } else if (pool->head_dim == 64) {
        if (ht == 4) launch_mfma<64, 4>(a, max_q_len, st, launched);
        else if (ht == 2) launch_mfma<64, 2>(a, max_q_len, st, launched);
        else launch_mfma<64, 1>(a, max_q_len, st, launched);
    } else {
        return MUX_ERR_UNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? MUX_OK : MUX_ERR_HIP;
}
