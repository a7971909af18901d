// Decode attention over the unified head-wise paged KV pool (gfx950, wave64).
//
// MuxServe, Section 2.1 (each decoding step attends to the cached K/V of every earlier
// token) and Section 3.4 (that cache is a pool of blocks, each holding one KV head for a
// few tokens).  The result is plain softmax(scale * q K^T) V per (sequence, query head).
//
// Shape of the work: for multi-head models every K/V byte is used once, about one flop per
// byte, so the kernel is a gather at HBM speed.  Design:
//   - a workgroup of 4 waves works on one (sequence, kv head, span of the context) at a time;
//     long contexts are split into spans; the launch holds as many workgroups as fit on the
//     GPU and each walks its share of a longest-first list of spans that a small kernel
//     prepares (see decode_plan_kernel and take_work);
//   - a wave reads whole blocks: each load instruction is 64 lanes x 16 bytes = 1 KiB of
//     contiguous tile, i.e. RPL = 1024 / row_bytes full rows; a 16-token block of 128 bf16
//     is 4 loads of K and 4 of V, all issued before any of them is used, and the next
//     block's 8 loads are issued before the current block is consumed;
//   - the lanes that share a row reduce their partial dot products with DPP row
//     operations; each group of lanes that owns a row slot keeps its own running
//     max / sum / accumulator (online softmax), so nothing crosses rows inside the loop;
//   - the block ids of a wave are fetched with one coalesced load up front and broadcast
//     with readlane, so block addresses are scalar;
//   - the row slots of a wave are merged with shuffles, the 4 waves through LDS, and spans
//     through a small fp32 workspace and a combine kernel.
// All arithmetic is fp32; the output is rounded once to the storage type.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <map>
#include <mutex>
#include <type_traits>
#include <utility>

#include "mux_internal.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

#ifndef MUX_GROUP_MIN_WAVES
#define MUX_GROUP_MIN_WAVES 2
#endif
#ifndef MUX_DECODE_MIN_WAVES
#define MUX_DECODE_MIN_WAVES 1
#endif
constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr int kMaxWaveBlocks = 64;              // block ids a wave keeps in one register
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -3.0e38f;             // "no score seen yet"; finite so that differences stay finite

template <int CTRL>
__device__ __forceinline__ float dpp_move(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}

// Sum over each group of LPR consecutive lanes; every lane of the group gets the sum.
template <int LPR>
__device__ __forceinline__ float row_sum(float x)
{
    x += dpp_move<0xB1>(x);                      // quad_perm [1,0,3,2]
    x += dpp_move<0x4E>(x);                      // quad_perm [2,3,0,1]
    if (LPR >= 8) x += dpp_move<0x141>(x);       // row_half_mirror
    if (LPR >= 16) x += dpp_move<0x140>(x);      // row_mirror
    if (LPR >= 32) x += __shfl_xor(x, 16);
    return x;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <bool BF16>
struct Piece {  // the 16 bytes one lane loads
    static constexpr int N = BF16 ? 8 : 4;
    static __device__ __forceinline__ void widen(const u32x4 v, float (&x)[N])
    {
        if constexpr (BF16) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x[2 * i] = __uint_as_float(v[i] << 16);
                x[2 * i + 1] = __uint_as_float(v[i] & 0xffff0000u);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) x[i] = __uint_as_float(v[i]);
        }
    }
};

__device__ __forceinline__ unsigned short to_bf16_rne(float f)
{
    unsigned u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<unsigned short>(u >> 16);
}

template <bool BF16>
__device__ __forceinline__ void store_out(void *out, long long idx, float v)
{
    if constexpr (BF16)
        static_cast<unsigned short *>(out)[idx] = to_bf16_rne(v);
    else
        static_cast<float *>(out)[idx] = v;
}

struct DecodeArgs {
    const char *kv_base;
    long long block_bytes;
    int num_blocks;
    int block_size;
    void *out;
    const void *q;
    const int *tables;
    const int *ctx_lens;    // decode: context length of every row
    // generic prefill: every query row of every chunk is one "decode" row; its table row and
    // context length follow from cu_q_lens / q_start (both null for decode)
    const int *cu_q_lens;
    const int *q_start;
    int n_table_seqs;       // sequences in the block table (== n_seqs for decode)
    int n_seqs;             // sequences (entries of ctx_lens); rows of q / out = n_seqs * n_layers
    // fused step: rows are laid out [layer][sequence]; every row's new K/V (k_new / v_new,
    // [rows][n_kv_heads][D]) is written to position len - 1 of its blocks by the workgroup that
    // reads that block, and used from registers.  Plain decode: n_layers = 1, k_new = null.
    int n_layers;
    const void *k_new;
    const void *v_new;
    int n_q_heads, n_kv_heads, max_blocks, max_ctx_len;
    float scale_log2e;
    int span_blocks;  // blocks per workgroup span
    int n_splits;
    int n_passes;
    float *ws_acc;  // [rows][n_q_heads][n_splits][D]
    float *ws_ml;   // [rows][n_q_heads][n_splits][2]
    // work list written by decode_plan_kernel: plan[1] = number of units, then from plan + 4 the
    // units as (row, split) pairs, longest first
    int *plan;
    int grid_wgs;   // workgroups of the attention launch
};

// Arguments of a fused step whose small integer arrays ride in the kernel arguments, so that no
// kernel has to run ahead of this one to put them into device memory (ctx_lens is not read
// then).  inl holds, for the n_seqs rows of a layer: the context length; then the index of the
// row's entry or -1; then, per entry, inl_heads block ids: the block that the row's new token
// has just opened, for every kv head of every layer of the model (this launch's first layer
// starts at inl_head0).  The id of such a block is taken from here instead of the table (where
// head pass 0 stores it for the steps to come).  Only the INL instantiations of the kernels take
// this (4 KiB of arguments cost ~2 us per launch, which the ordinary launches should not pay).
struct DecodeArgsInl : DecodeArgs {
    int inl_heads, inl_head0;
    int inl[MUX_INLINE_STEP_INTS];
};
static_assert(sizeof(DecodeArgsInl) <= 4096, "kernel arguments are limited to 4 KiB");
template <bool INL>
using Args = std::conditional_t<INL, DecodeArgsInl, DecodeArgs>;

// The id of the block that column `col` of row s (kv head kvh) refers to, when the step's arrays
// ride in the arguments and the row's new token has just opened that block; `id` otherwise.  Head
// pass 0 leaves the id in the table.  L: the row's context length (0 for a row that is not part of
// the step, or whose context was cut at the launch's bound: its new token lies beyond the cut).
__device__ __forceinline__ int inline_block_id(const DecodeArgsInl &a, int s, int kvh, int pass, int L, int col, int id,
                                               const int *table_row)
{
    if (L <= 0) return id;
    const int e = a.inl[a.n_seqs + s % a.n_seqs];
    if (e < 0 || col != (L - 1) / a.block_size) return id;
    id = a.inl[2 * a.n_seqs + e * a.inl_heads + a.inl_head0 + (s / a.n_seqs) * a.n_kv_heads + kvh];
    if (pass == 0) const_cast<int *>(table_row)[col] = id;
    return id;
}

// Row r of q/out -> (block-table row, context length).  The length is cut at max_ctx_len (the
// host's bound, which sized the launch); *cut, when asked for, tells whether that happened.
template <bool INL>
__device__ __forceinline__ void resolve_row(const Args<INL> &a, int r, int &table_row, int &len, bool *cut = nullptr)
{
    if (a.cu_q_lens == nullptr) {
        table_row = r;
        if constexpr (INL)
            len = a.inl[r % a.n_seqs];
        else
            len = a.ctx_lens[r % a.n_seqs];
    } else {
        int lo = 0, hi = a.n_table_seqs - 1;  // last sequence whose first row is <= r
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (a.cu_q_lens[mid] <= r) lo = mid; else hi = mid - 1;
        }
        table_row = lo;
        len = a.q_start[lo] + (r - a.cu_q_lens[lo]) + 1;  // causal: keys up to and including its own
    }
    if (cut) *cut = len > a.max_ctx_len;
    len = min(max(len, 0), a.max_ctx_len);
}

// Scheduling.  A unit of work is one span of one row (sequence): all its kv heads and head
// passes.  Spans differ in length by orders of magnitude inside one batch, so the order in
// which they are started decides how long the GPU idles at the end of a launch.  A one-workgroup
// kernel lists the units longest first (all full spans, then the last span of every row by
// falling length; rows with an empty context get a unit too, so that their zeros are written),
// and the attention kernel is launched with exactly as many workgroups as are resident at once,
// each of which walks a fixed share of that list (see take_work).  No workgroup is ever started
// for an empty span, and the longest units are never started last.
template <bool INL>
__global__ __launch_bounds__(256) void decode_plan_kernel(const Args<INL> a)
{
    __shared__ int sm_scan[256];
    __shared__ int sm_bin[kWaves * kMaxWaveBlocks + 1];   // by length of the last span, 0 .. span_blocks
    __shared__ int sm_base;
    const int tid = threadIdx.x;
    const int B = a.block_size, span = a.span_blocks;
    const int n_rows = a.n_seqs * a.n_layers;
    int2 *units = reinterpret_cast<int2 *>(a.plan + 4);
    auto shape_of = [&](int r, int &full, int &rem) {   // full spans before the last one, blocks in the last one
        int table_row, len;
        resolve_row<INL>(a, r, table_row, len);
        const int blocks = (len + B - 1) / B;
        full = blocks > 0 ? (blocks - 1) / span : 0;
        rem = blocks - full * span;
    };
    for (int i = tid; i <= span; i += 256) sm_bin[i] = 0;
    if (tid == 0) sm_base = 0;
    __syncthreads();
    // full spans, in row order (256 rows at a time, workgroup-wide inclusive scan of their counts)
    for (int r0 = 0; r0 < n_rows; r0 += 256) {
        const int r = r0 + tid;
        int full = 0, rem = 0;
        if (r < n_rows) {
            shape_of(r, full, rem);
            atomicAdd(&sm_bin[rem], 1);
        }
        if (a.n_splits == 1) continue;   // a single span per row: there are no full spans to list
        sm_scan[tid] = full;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {
            const int below = tid >= off ? sm_scan[tid - off] : 0;
            __syncthreads();
            sm_scan[tid] += below;
            __syncthreads();
        }
        const int first = sm_base + sm_scan[tid] - full;
        for (int p = 0; p < full; ++p) units[first + p] = int2{r, p};
        __syncthreads();
        if (tid == 255) sm_base += sm_scan[255];
        __syncthreads();
    }
    __syncthreads();
    const int n_full = sm_base;
    // last spans: counting sort by falling length
    if (tid == 0) {
        int run = n_full;
        for (int b = span; b >= 0; --b) {
            const int c = sm_bin[b];
            sm_bin[b] = run;
            run += c;
        }
    }
    __syncthreads();
    for (int r = tid; r < n_rows; r += 256) {
        int full, rem;
        shape_of(r, full, rem);
        units[atomicAdd(&sm_bin[rem], 1)] = int2{r, full};
    }
    if (tid == 0) a.plan[1] = n_full + n_rows;
}

// Work distribution inside the attention kernels.  Piece w of the work is unit w / (kv heads x
// head passes) of the list, for one kv head and one pass.  With G workgroups, workgroup i takes
// pieces i, 2G-1-i, 2G+i, 4G-1-i, ...: the list is dealt out in rounds whose direction
// alternates, so the workgroup that got the longest piece of one round gets the shortest of the
// next and the shares come out nearly equal.  The assignment is fixed: a shared counter that
// workgroups claim pieces from was measured to cost ~25 % on short launches, since a thousand
// device-wide atomics on one address take tens of microseconds to drain and every load issued
// behind one waits for it.
struct WorkCursor {
    int round;        // pieces this workgroup has taken so far
    // LDS, when the workgroup orders the work itself: the row of every rank (rank_rows), or the
    // units as row | span << 16 with their number behind them (list_units)
    const int *rows;
};

// Short launches (one span per row, at most kMaxRankedRows rows) skip the plan kernel: every
// workgroup ranks the rows by context length itself - one row per thread, its rank is the
// number of rows that are longer (or as long and earlier) - and leaves "row of rank r" in LDS.
// That costs a few hundred cycles per workgroup and saves a dependent kernel launch per call.
constexpr int kMaxRankedRows = kThreads;

template <bool INL>
__device__ __forceinline__ void rank_rows(const Args<INL> &a, int tid, int *sm_len, int *sm_row)
{
    if (a.plan != nullptr) return;
    const int n_rows = a.n_seqs * a.n_layers;
    if (tid < n_rows) {
        int table_row, len;
        resolve_row<INL>(a, tid, table_row, len);
        sm_len[tid] = len;
    }
    __syncthreads();
    if (tid < n_rows) {
        const int mine = sm_len[tid];
        int rank = 0;
        for (int j = 0; j < n_rows; ++j) {
            const int other = sm_len[j];
            rank += (other > mine || (other == mine && j < tid)) ? 1 : 0;
        }
        sm_row[rank] = tid;
    }
    // the barrier at the top of take_work makes sm_row visible
}

// Launches of few rows whose contexts ARE cut into spans skip the plan kernel too: every workgroup
// builds the same list as decode_plan_kernel in LDS - the full spans in row order, then every
// row's last span by falling length - with one row per thread: a thread's place among the full
// spans is the number of full spans of the rows before it, its place among the last spans the
// number of rows whose last span is longer (or as long and earlier).  Everything is a pure
// function of the context lengths, so all workgroups arrive at the same list.
constexpr int kMaxInlineUnits = 1024;

template <bool INL>
__device__ __forceinline__ void list_units(const Args<INL> &a, int tid, int *sm_shape, int *sm_units)
{
    const int n_rows = a.n_seqs * a.n_layers;
    const int span = a.span_blocks;
    int full = 0, rem = 0;
    if (tid < n_rows) {
        int table_row, len;
        resolve_row<INL>(a, tid, table_row, len);
        const int blocks = (len + a.block_size - 1) / a.block_size;
        full = blocks > 0 ? (blocks - 1) / span : 0;   // full spans before the last one
        rem = blocks - full * span;                    // blocks in the last one
        sm_shape[tid] = full << 16 | rem;
    }
    __syncthreads();
    int before = 0, all_full = 0, rank = 0;
    for (int j = 0; j < n_rows; ++j) {
        const int shape = sm_shape[j];
        const int f = shape >> 16, r = shape & 0xffff;
        all_full += f;
        before += j < tid ? f : 0;
        rank += (r > rem || (r == rem && j < tid)) ? 1 : 0;
    }
    if (tid < n_rows) {
        for (int p = 0; p < full; ++p) sm_units[before + p] = tid | p << 16;
        sm_units[all_full + rank] = tid | full << 16;
    }
    if (tid == 0) sm_units[kMaxInlineUnits] = all_full + n_rows;
    // the barrier at the top of take_work makes the list visible
}

__device__ __forceinline__ bool take_work(const DecodeArgs &a, int tid, WorkCursor &cur, bool first, int &row, int &split,
                                          int &kvh, int &pass)
{
    __syncthreads();   // the previous piece's LDS is no longer in use
    const int G = a.grid_wgs;
    const int k = first ? 0 : cur.round;
    int w = k * G + ((k & 1) ? G - 1 - static_cast<int>(blockIdx.x) : static_cast<int>(blockIdx.x));
    cur.round = k + 1;
    const int per_unit = a.n_kv_heads * a.n_passes;
    if (a.plan == nullptr && a.n_splits == 1) {
        if (w / per_unit >= a.n_seqs * a.n_layers) return false;
        row = __builtin_amdgcn_readfirstlane(cur.rows[w / per_unit]);
        split = 0;
    } else if (a.plan == nullptr) {
        if (w / per_unit >= __builtin_amdgcn_readfirstlane(cur.rows[kMaxInlineUnits])) return false;
        const int u = __builtin_amdgcn_readfirstlane(cur.rows[w / per_unit]);
        row = u & 0xffff;
        split = u >> 16;
    } else {
        const int n_units = __builtin_amdgcn_readfirstlane(a.plan[1]);
        if (w / per_unit >= n_units) return false;
        const int2 u = reinterpret_cast<const int2 *>(a.plan + 4)[w / per_unit];
        row = __builtin_amdgcn_readfirstlane(u.x);
        split = __builtin_amdgcn_readfirstlane(u.y);
    }
    w %= per_unit;
    pass = w % a.n_passes;
    kvh = w / a.n_passes;
    return true;
}

// Last stage of a workgroup: every wave has left, per query head h, its running max, sum and
// un-normalised accumulator in LDS; merge the waves and write either the final output row
// (single span) or this span's partial result.
template <bool BF16, int D, int GT>
__device__ __forceinline__ void merge_waves_and_store(const DecodeArgs &a, const float (*sm_acc)[GT][D],
                                                      const float (*sm_m)[GT], const float (*sm_l)[GT], int tid,
                                                      int s, int head0, int heads_left, int split)
{
    for (int idx = tid; idx < GT * D; idx += kThreads) {
        const int h = idx / D, c = idx % D;
        if (h >= heads_left) continue;
        float mm = sm_m[0][h];
#pragma unroll
        for (int k = 1; k < kWaves; ++k) mm = fmaxf(mm, sm_m[k][h]);
        float o = 0.f, ll = 0.f;
#pragma unroll
        for (int k = 0; k < kWaves; ++k) {
            const float wk = fast_exp2(sm_m[k][h] - mm);
            o += sm_acc[k][h][c] * wk;
            ll += sm_l[k][h] * wk;
        }
        const long long qrow = static_cast<long long>(s) * a.n_q_heads + head0 + h;
        if (a.n_splits == 1) {
            store_out<BF16>(a.out, qrow * D + c, ll > 0.f ? o / ll : 0.f);
        } else {
            const long long part = qrow * a.n_splits + split;
            a.ws_acc[part * D + c] = o;
            if (c == 0) {
                a.ws_ml[part * 2] = mm;
                a.ws_ml[part * 2 + 1] = ll;
            }
        }
    }
}

// BF16: storage type; D: head size; BS: tokens per block at compile time (0 = run time);
// GT: query heads of one KV group handled together.
template <bool BF16, int D, int BS, int GT, bool INL>
__global__ __launch_bounds__(kThreads, MUX_DECODE_MIN_WAVES) void decode_attn_kernel(const Args<INL> a)
{
    constexpr int EB = BF16 ? 2 : 4;
    constexpr int EPL = 16 / EB;          // elements per lane per load
    constexpr int LPR = D / EPL;          // lanes per row
    constexpr int RPL = 64 / LPR;         // rows per load instruction
    static_assert(LPR >= 4 && LPR <= 32, "unsupported head size");
    constexpr bool kFixed = BS > 0;
    // A block of a compile-time size is consumed in sub-tiles of 16 tokens (one sub-tile for
    // the 16-token blocks of the paper's workloads): the registers of a wave hold two of them.
    constexpr int TB = 16;                     // tokens per sub-tile
    constexpr int SUBS = kFixed ? BS / TB : 1;   // sub-tiles per block
    static_assert(!kFixed || (BS % TB == 0 && TB % RPL == 0), "fixed block size must hold whole sub-tiles of whole load groups");
    constexpr int NG = kFixed ? TB / RPL : 1;  // loads per sub-tile, handled at once

    const int B = kFixed ? BS : a.block_size;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: keeps the block loop scalar
    const int rg = lane / LPR;            // row slot of this lane inside a load
    const int c0 = (lane % LPR) * EPL;    // first head dimension of this lane

    int s, split, kvh, pass;   // s: row of q / out / the table
    __shared__ int sm_rank_len[kMaxRankedRows], sm_rank_row[kMaxInlineUnits + 1];
    if (a.plan == nullptr && a.n_splits > 1)
        list_units<INL>(a, tid, sm_rank_len, sm_rank_row);
    else
        rank_rows<INL>(a, tid, sm_rank_len, sm_rank_row);
    WorkCursor cursor{0, sm_rank_row};
    for (bool first = true; take_work(a, tid, cursor, first, s, split, kvh, pass); first = false) {
    // Block ids of this wave: block blk_lo + wave + kWaves * j sits in lane j.  The load does
    // not wait for the context length (any entry inside the table row may be read; entries
    // past the sequence's blocks are never used), so the two latencies overlap.
    const int blk_lo = split * a.span_blocks;
    int table_row, L;
    bool cut;
    resolve_row<INL>(a, s, table_row, L, &cut);
    table_row = __builtin_amdgcn_readfirstlane(table_row);   // same for every lane: keep the block loop scalar
    L = __builtin_amdgcn_readfirstlane(L);
    // A fused step appends the row's new token at position L - 1.  A row whose context was cut at
    // max_ctx_len has its new token beyond the cut: nothing is appended for it (position L - 1 of
    // the cut context holds an older token, which must stay as it is).
    const bool appends = a.k_new != nullptr && __builtin_amdgcn_readfirstlane(static_cast<int>(cut)) == 0;
    const int *row = a.tables + (static_cast<long long>(table_row) * a.n_kv_heads + kvh) * a.max_blocks;
    int my_ids = 0;
    {
        const int col = blk_lo + wave + kWaves * lane;
        if (col < a.max_blocks) {
            my_ids = row[col];
            if constexpr (INL) my_ids = inline_block_id(a, s, kvh, pass, cut ? 0 : L, col, my_ids, row);
        }
    }
    const int n_blk_seq = (L + B - 1) / B;
    const int blk_hi = min(blk_lo + a.span_blocks, n_blk_seq);   // blk_lo < n_blk_seq unless the context is empty

    const int group = a.n_q_heads / a.n_kv_heads;
    const int head0 = kvh * group + pass * GT;  // first query head of this pass

    // q rows, pre-multiplied by scale * log2(e): scores live in the exp2 domain
    float qf[GT][EPL];
#pragma unroll
    for (int h = 0; h < GT; ++h) {
        const int qh = min(head0 + h, kvh * group + group - 1);
        const u32x4 raw = *reinterpret_cast<const u32x4 *>(static_cast<const char *>(a.q) +
                                                           ((static_cast<long long>(s) * a.n_q_heads + qh) * D + c0) * EB);
        Piece<BF16>::widen(raw, qf[h]);
#pragma unroll
        for (int e = 0; e < EPL; ++e) qf[h][e] *= a.scale_log2e;
    }

    float m[GT], l[GT], acc[GT][EPL];
#pragma unroll
    for (int h = 0; h < GT; ++h) {
        m[h] = kNegBig;
        l[h] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[h][e] = 0.f;
    }

    const int n_mine = blk_hi - blk_lo > wave ? (blk_hi - blk_lo - wave + kWaves - 1) / kWaves : 0;

    auto tile_ptr = [&](int j) -> const char * {
        int id = __builtin_amdgcn_readlane(my_ids, j);
        id = min(max(id, 0), a.num_blocks - 1);  // a corrupt table must not leave the pool
        return a.kv_base + static_cast<long long>(id) * a.block_bytes;
    };

    // Fold NG row groups (K pieces k[], V pieces v[]) into the running softmax state.
    // Rows whose index (g * RPL + rg) is >= n_valid are ignored when MASKED.
    auto fold = [&](const u32x4 (&k)[NG], const u32x4 (&v)[NG], auto masked_tag, int n_valid) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        float p[GT][NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            float kf[EPL];
            Piece<BF16>::widen(k[g], kf);
            const bool ok = !MASKED || (g * RPL + rg < n_valid);
#pragma unroll
            for (int h = 0; h < GT; ++h) {
                float dot = 0.f;
#pragma unroll
                for (int e = 0; e < EPL; ++e) dot = __builtin_fmaf(qf[h][e], kf[e], dot);
                dot = row_sum<LPR>(dot);
                p[h][g] = ok ? dot : kNegBig;
            }
        }
#pragma unroll
        for (int h = 0; h < GT; ++h) {
            float mx = p[h][0];
#pragma unroll
            for (int g = 1; g < NG; ++g) mx = fmaxf(mx, p[h][g]);
            const float m_new = fmaxf(m[h], mx);
            const float alpha = fast_exp2(m[h] - m_new);
            float sum = 0.f;
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                float e = fast_exp2(p[h][g] - m_new);
                if (MASKED && !(g * RPL + rg < n_valid)) e = 0.f;
                p[h][g] = e;
                sum += e;
            }
            l[h] = l[h] * alpha + sum;
            m[h] = m_new;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[h][e] *= alpha;
        }
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            float vf[EPL];
            Piece<BF16>::widen(v[g], vf);
            if (MASKED && !(g * RPL + rg < n_valid)) {
#pragma unroll
                for (int e = 0; e < EPL; ++e) vf[e] = 0.f;  // stale bytes may be NaN
            }
#pragma unroll
            for (int h = 0; h < GT; ++h)
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[h][e] = __builtin_fmaf(p[h][g], vf[e], acc[h][e]);
        }
    };

    if constexpr (kFixed && SUBS == 1) {
        // blocks of 16 tokens: one sub-tile per block (kept apart from the general case below so that its code,
        // the one every measured configuration runs, does not depend on it)
        constexpr int kTileBytes = BS * D * EB;
        auto load_tile = [&](int j, u32x4 (&k)[NG], u32x4 (&v)[NG]) {
            const char *t = tile_ptr(j) + static_cast<unsigned>(lane * 16);
#pragma unroll
            for (int g = 0; g < NG; ++g) k[g] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(t + g * 1024));
#pragma unroll
            for (int g = 0; g < NG; ++g)
                v[g] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(t + kTileBytes + g * 1024));
        };
        // Every block but the wave's last one is full, so only the last may need masking; it is
        // also the only one that can hold the token a fused step appends.
        auto consume_full = [&](const u32x4 (&k)[NG], const u32x4 (&v)[NG]) { fold(k, v, std::false_type{}, BS); };
        auto consume_last = [&](int j, u32x4 (&k)[NG], u32x4 (&v)[NG]) {
            const int blk = blk_lo + wave + kWaves * j;
            const int n_valid = L - blk * BS;  // wave-uniform, >= 1
            if (appends && blk == n_blk_seq - 1) {
                // the new token's row: take it from k_new / v_new, and let pass 0 store it in the pool
                const int r = n_valid - 1;
                char *tile = const_cast<char *>(tile_ptr(j));
#pragma unroll
                for (int g = 0; g < NG; ++g)
                    if (g * RPL + rg == r) {
                        const long long src = ((static_cast<long long>(s) * a.n_kv_heads + kvh) * D + c0) * EB;
                        k[g] = *reinterpret_cast<const u32x4 *>(static_cast<const char *>(a.k_new) + src);
                        v[g] = *reinterpret_cast<const u32x4 *>(static_cast<const char *>(a.v_new) + src);
                        if (pass == 0) {
                            char *dst = tile + static_cast<long long>(r) * (D * EB) + c0 * EB;
                            *reinterpret_cast<u32x4 *>(dst) = k[g];
                            *reinterpret_cast<u32x4 *>(dst + kTileBytes) = v[g];
                        }
                    }
            }
            if (n_valid >= BS)
                fold(k, v, std::false_type{}, BS);
            else
                fold(k, v, std::true_type{}, n_valid);
        };
        // Two register sets alternate; the loads of the next block are always issued before
        // the current block is consumed, and unconditionally inside the loop so that the wait
        // counters only cover the block being consumed.
        if (n_mine > 0) {
            u32x4 ka[NG], va[NG], kb[NG], vb[NG];
            load_tile(0, ka, va);
            int j = 0;
            for (; j + 2 < n_mine; j += 2) {
                load_tile(j + 1, kb, vb);
                consume_full(ka, va);
                load_tile(j + 2, ka, va);
                consume_full(kb, vb);
            }
            if (j + 1 < n_mine) {
                load_tile(j + 1, kb, vb);
                consume_full(ka, va);
                consume_last(j + 1, kb, vb);
            } else {
                consume_last(j, ka, va);
            }
        }
    } else if constexpr (kFixed) {
        constexpr int kTileBytes = BS * D * EB;      // K tile of a block; its V tile follows
        constexpr int kSubBytes = TB * D * EB;
        // sub-tile jj of the wave: sub-tile jj % SUBS of its block jj / SUBS
        auto sub_ptr = [&](int jj) { return tile_ptr(jj / SUBS) + (jj % SUBS) * kSubBytes; };
        auto load_tile = [&](int jj, u32x4 (&k)[NG], u32x4 (&v)[NG]) {
            const char *t = sub_ptr(jj) + static_cast<unsigned>(lane * 16);
#pragma unroll
            for (int g = 0; g < NG; ++g) k[g] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(t + g * 1024));
#pragma unroll
            for (int g = 0; g < NG; ++g)
                v[g] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(t + kTileBytes + g * 1024));
        };
        // Every sub-tile but the wave's last one is full, so only the last may need masking; it is
        // also the only one that can hold the token a fused step appends.
        auto consume_full = [&](const u32x4 (&k)[NG], const u32x4 (&v)[NG]) { fold(k, v, std::false_type{}, TB); };
        auto consume_last = [&](int jj, u32x4 (&k)[NG], u32x4 (&v)[NG]) {
            const int blk = blk_lo + wave + kWaves * (jj / SUBS);
            const int n_valid = L - blk * BS - (jj % SUBS) * TB;  // wave-uniform, >= 1
            if (appends && blk == n_blk_seq - 1) {
                // the new token's row: take it from k_new / v_new, and let pass 0 store it in the pool
                const int r = n_valid - 1;
                char *tile = const_cast<char *>(sub_ptr(jj));
#pragma unroll
                for (int g = 0; g < NG; ++g)
                    if (g * RPL + rg == r) {
                        const long long src = ((static_cast<long long>(s) * a.n_kv_heads + kvh) * D + c0) * EB;
                        k[g] = *reinterpret_cast<const u32x4 *>(static_cast<const char *>(a.k_new) + src);
                        v[g] = *reinterpret_cast<const u32x4 *>(static_cast<const char *>(a.v_new) + src);
                        if (pass == 0) {
                            char *dst = tile + static_cast<long long>(r) * (D * EB) + c0 * EB;
                            *reinterpret_cast<u32x4 *>(dst) = k[g];
                            *reinterpret_cast<u32x4 *>(dst + kTileBytes) = v[g];
                        }
                    }
            }
            if (n_valid >= TB)
                fold(k, v, std::false_type{}, TB);
            else
                fold(k, v, std::true_type{}, n_valid);
        };
        // sub-tiles of this wave: all of its blocks but the last, and of that one those that hold tokens
        const int n_sub = n_mine > 0
                              ? (n_mine - 1) * SUBS + (min(BS, L - (blk_lo + wave + kWaves * (n_mine - 1)) * BS) + TB - 1) / TB
                              : 0;
        // Two register sets alternate; the loads of the next sub-tile are always issued before
        // the current one is consumed, and unconditionally inside the loop so that the wait
        // counters only cover the sub-tile being consumed.
        if (n_sub > 0) {
            u32x4 ka[NG], va[NG], kb[NG], vb[NG];
            load_tile(0, ka, va);
            int j = 0;
            for (; j + 2 < n_sub; j += 2) {
                load_tile(j + 1, kb, vb);
                consume_full(ka, va);
                load_tile(j + 2, ka, va);
                consume_full(kb, vb);
            }
            if (j + 1 < n_sub) {
                load_tile(j + 1, kb, vb);
                consume_full(ka, va);
                consume_last(j + 1, kb, vb);
            } else {
                consume_last(j, ka, va);
            }
        }
    } else {
        const long long tile_bytes = static_cast<long long>(B) * D * EB;
        // The wave's blocks, RPL rows at a time.  The loads of the next group are issued before
        // the current one is folded in; lanes past a block's rows load its last row again (the
        // fold ignores them), so the loads are unconditional and the waits cover one group only.
        auto rows_of = [&](int j) { return min(B, L - (blk_lo + wave + kWaves * j) * B); };
        auto load_group = [&](int j, int r0, int rows_here, u32x4 &k, u32x4 &v) {
            const int r = min(r0 + rg, rows_here - 1);
            char *src = const_cast<char *>(tile_ptr(j)) + static_cast<long long>(r) * (D * EB) + (lane % LPR) * 16;
            k = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src));
            v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + tile_bytes));
            const int tok0 = (blk_lo + wave + kWaves * j) * B + r0;   // first token of the group (same in all lanes)
            if (appends && tok0 <= L - 1 && L - 1 < tok0 + min(RPL, rows_here - r0)) {
                if (tok0 + rg == L - 1) {   // the token a fused step appends (a row of this block: see the check above)
                    const long long nsrc = ((static_cast<long long>(s) * a.n_kv_heads + kvh) * D + c0) * EB;
                    k = *reinterpret_cast<const u32x4 *>(static_cast<const char *>(a.k_new) + nsrc);
                    v = *reinterpret_cast<const u32x4 *>(static_cast<const char *>(a.v_new) + nsrc);
                    if (pass == 0) {
                        *reinterpret_cast<u32x4 *>(src) = k;
                        *reinterpret_cast<u32x4 *>(src + tile_bytes) = v;
                    }
                }
            }
        };
        if (n_mine > 0) {
            int j = 0, r0 = 0, rows_here = rows_of(0);
            u32x4 kc[1], vc[1], kn[1], vn[1];
            load_group(0, 0, rows_here, kc[0], vc[0]);
            for (;;) {
                int nj = j, nr0 = r0 + RPL, nrows = rows_here;
                if (nr0 >= rows_here) {
                    nj = j + 1;
                    nr0 = 0;
                    nrows = nj < n_mine ? rows_of(nj) : 0;
                }
                const bool more = nj < n_mine;
                if (more) load_group(nj, nr0, nrows, kn[0], vn[0]);
                fold(kc, vc, std::true_type{}, rows_here - r0);
                if (!more) break;
                kc[0] = kn[0], vc[0] = vn[0];
                j = nj, r0 = nr0, rows_here = nrows;
            }
        }
    }

    // Merge the RPL row slots of the wave: afterwards every lane holds the wave's state.
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
        for (int h = 0; h < GT; ++h) {
            const float mo = __shfl_xor(m[h], off);
            const float lo = __shfl_xor(l[h], off);
            const float mn = fmaxf(m[h], mo);
            const float wa = fast_exp2(m[h] - mn), wb = fast_exp2(mo - mn);
            l[h] = l[h] * wa + lo * wb;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[h][e] = acc[h][e] * wa + __shfl_xor(acc[h][e], off) * wb;
            m[h] = mn;
        }
    }

    __shared__ float sm_acc[kWaves][GT][D];
    __shared__ float sm_m[kWaves][GT], sm_l[kWaves][GT];
    if (lane < LPR) {
#pragma unroll
        for (int h = 0; h < GT; ++h) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) sm_acc[wave][h][c0 + e] = acc[h][e];
            if (lane == 0) {
                sm_m[wave][h] = m[h];
                sm_l[wave][h] = l[h];
            }
        }
    }
    __syncthreads();

    merge_waves_and_store<BF16, D, GT>(a, sm_acc, sm_m, sm_l, tid, s, head0, group - pass * GT, split);
    }   // next piece of work
}

// Grouped-query decode on the matrix cores (bf16 pools, 16-token blocks, groups of >= 4
// query heads).  With g heads per KV head the vector kernel above would spend g times the
// arithmetic per byte and go ALU-bound; here the g heads of a group (padded to 16) are the
// columns of two MFMA contractions per 16-token block, exactly as in the prefill kernel:
//   S^T = K . Q^T   (v_mfma_f32_16x16x32_bf16, K rows from LDS, Q^T in registers)
//   O^T = V^T . P^T (v_mfma_f32_16x16x16_bf16; the V^T operand - four tokens of one dim per
//                    lane - comes out of the row-major LDS tile through the transposing read
//                    ds_read_b64_tr_b16; P^T = the S^T registers after softmax)
// Each wave streams its own blocks (same interleaving, id broadcast and register prefetch as
// the vector kernel) through a private LDS tile; no barrier is needed inside the loop.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// Maximum over the four lanes l, l^16, l^32, l^48 without a trip through LDS: with both
// operands holding x, v_permlane32_swap / v_permlane16_swap leave "x of my half / row" in one
// result and "x of the other half / row" in the other.
__device__ __forceinline__ float row_max_across_groups(float x)
{
    typedef unsigned u32pair __attribute__((ext_vector_type(2)));
    const unsigned u = __float_as_uint(x);
    const u32pair h = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const float y = fmaxf(__uint_as_float(h[0]), __uint_as_float(h[1]));
    const unsigned v = __float_as_uint(y);
    const u32pair r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Transposing LDS read: within each group of 16 lanes, lane i receives element (i % 4) of the
// four 8-byte chunks addressed by lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12 of the group.
__device__ __forceinline__ s16x4 lds_read_tr16(const char *p)
{
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p));
}

__device__ __forceinline__ unsigned pack2_bf16(float x, float y)
{
    return static_cast<unsigned>(to_bf16_rne(x)) | (static_cast<unsigned>(to_bf16_rne(y)) << 16);
}

template <int D, bool INL>
__global__ __launch_bounds__(kThreads, MUX_GROUP_MIN_WAVES) void decode_attn_group_kernel(const Args<INL> a)
{
    constexpr int BS = 16, GT = 16;
    constexpr int KC = D / 32, NT = D / 16;
    constexpr int KROW = D * 2 + 16;           // padded K row in LDS (bytes)
    constexpr int VROW = D * 2 + 32;           // padded V row in LDS: keeps the transposing reads conflict-free
    constexpr int TILE = BS * KROW + BS * VROW;  // one wave's K tile + V tile
    constexpr int PPR = D * 2 / 16;            // 16-byte pieces per token row
    constexpr int NP = BS * PPR / 64;          // pieces per lane per tile (K; same for V)
    constexpr int MERGE = kWaves * GT * D * 4 + 2 * kWaves * GT * 4;
    constexpr int SMEM = kWaves * TILE > MERGE ? kWaves * TILE : MERGE;
    __shared__ __attribute__((aligned(16))) char smem[SMEM];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;

    int s, split, kvh, pass;   // s: row of q / out / the table
    __shared__ int sm_rank_len[kMaxRankedRows], sm_rank_row[kMaxInlineUnits + 1];
    if (a.plan == nullptr && a.n_splits > 1)
        list_units<INL>(a, tid, sm_rank_len, sm_rank_row);
    else
        rank_rows<INL>(a, tid, sm_rank_len, sm_rank_row);
    WorkCursor cursor{0, sm_rank_row};
    for (bool first = true; take_work(a, tid, cursor, first, s, split, kvh, pass); first = false) {
    const int blk_lo = split * a.span_blocks;
    int table_row, L;
    bool cut;
    resolve_row<INL>(a, s, table_row, L, &cut);
    table_row = __builtin_amdgcn_readfirstlane(table_row);   // same for every lane: keep the block loop scalar
    L = __builtin_amdgcn_readfirstlane(L);
    const bool appends = a.k_new != nullptr && __builtin_amdgcn_readfirstlane(static_cast<int>(cut)) == 0;   // a row cut at max_ctx_len appends nothing (see the vector kernel)
    const int *row = a.tables + (static_cast<long long>(table_row) * a.n_kv_heads + kvh) * a.max_blocks;
    int my_ids = 0;
    {
        const int col = blk_lo + wave + kWaves * lane;
        if (col < a.max_blocks) {
            my_ids = row[col];
            if constexpr (INL) my_ids = inline_block_id(a, s, kvh, pass, cut ? 0 : L, col, my_ids, row);
        }
    }
    const int n_blk_seq = (L + BS - 1) / BS;
    const int blk_hi = min(blk_lo + a.span_blocks, n_blk_seq);
    const int n_mine = blk_hi - blk_lo > wave ? (blk_hi - blk_lo - wave + kWaves - 1) / kWaves : 0;

    const int group = a.n_q_heads / a.n_kv_heads;
    const int head0 = kvh * group + pass * GT;
    const int heads_left = group - pass * GT;

    // Q^T operand: lane (g, c) holds dims 32k + 8g .. +8 of head c (surplus columns repeat the last head)
    bf16x8 qreg[KC];
    {
        const int qh = head0 + min(c, heads_left - 1);
        const char *qrow = static_cast<const char *>(a.q) + (static_cast<long long>(s) * a.n_q_heads + qh) * (D * 2);
#pragma unroll
        for (int k = 0; k < KC; ++k)
            qreg[k] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(qrow + (32 * k + 8 * g) * 2));
    }

    f32x4 acc[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) acc[n] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = kNegBig, l_run = 0.f;   // of head c; l_run is this lane's share of the sum

    char *ktile = smem + wave * TILE;
    char *vtile = ktile + BS * KROW;

    auto load_tile = [&](int j, u32x4 (&k)[NP], u32x4 (&v)[NP]) {
        int id = __builtin_amdgcn_readlane(my_ids, j);
        id = min(max(id, 0), a.num_blocks - 1);
        const char *t = a.kv_base + static_cast<long long>(id) * a.block_bytes + static_cast<unsigned>(lane * 16);
#pragma unroll
        for (int i = 0; i < NP; ++i) k[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(t + i * 1024));
#pragma unroll
        for (int i = 0; i < NP; ++i)
            v[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(t + BS * D * 2 + i * 1024));
    };

    // A fused step appends one token: the wave that reads the sequence's last block takes that
    // row from k_new / v_new (and, in pass 0, stores it in the pool).
    auto patch_new_row = [&](int j, u32x4 (&k)[NP], u32x4 (&v)[NP]) {
        const int blk = blk_lo + wave + kWaves * j;
        if (!appends || blk != n_blk_seq - 1) return;
        const int r = L - 1 - blk * BS;
        int id = __builtin_amdgcn_readlane(my_ids, j);
        id = min(max(id, 0), a.num_blocks - 1);
        char *tile = const_cast<char *>(a.kv_base) + static_cast<long long>(id) * a.block_bytes;
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int piece = lane + 64 * i;
            if (piece / PPR != r) continue;
            const long long src = ((static_cast<long long>(s) * a.n_kv_heads + kvh) * D) * 2 + (piece % PPR) * 16;
            k[i] = *reinterpret_cast<const u32x4 *>(static_cast<const char *>(a.k_new) + src);
            v[i] = *reinterpret_cast<const u32x4 *>(static_cast<const char *>(a.v_new) + src);
            if (pass == 0) {
                char *dst = tile + piece * 16;
                *reinterpret_cast<u32x4 *>(dst) = k[i];
                *reinterpret_cast<u32x4 *>(dst + BS * D * 2) = v[i];
            }
        }
    };
    // n_valid: tokens of this block that belong to the sequence (BS except possibly in the last block)
    auto consume = [&](const u32x4 (&k)[NP], const u32x4 (&v)[NP], int n_valid) {
        // registers -> this wave's LDS tile, rows padded so that both access patterns below
        // are free of bank conflicts
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int piece = lane + 64 * i;
            const int tok = piece / PPR, pc = piece % PPR;
            *reinterpret_cast<u32x4 *>(ktile + tok * KROW + pc * 16) = k[i];
            const u32x4 vv = tok < n_valid ? v[i] : u32x4{0, 0, 0, 0};   // stale slots may hold NaN
            *reinterpret_cast<u32x4 *>(vtile + tok * VROW + pc * 16) = vv;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        f32x4 st = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KC; ++kk) {
            const bf16x8 kop =
                __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(ktile + c * KROW + (32 * kk + 8 * g) * 2));
            st = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop, qreg[kk], st, 0, 0, 0);
        }
        float sc[4];
        float mx = kNegBig;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float x = st[i] * a.scale_log2e;
            if (4 * g + i >= n_valid) x = kNegBig;
            sc[i] = x;
            mx = fmaxf(mx, x);
        }
        mx = row_max_across_groups(mx);
        const float m_new = fmaxf(m_run, mx);
        const float alpha = fast_exp2(m_run - m_new);
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float e = fast_exp2(sc[i] - m_new);
            if (4 * g + i >= n_valid) e = 0.f;
            sc[i] = e;
            psum += e;
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
            for (int n = 0; n < NT; ++n) acc[n] *= alpha;
        }
        const u32x2 pw = {pack2_bf16(sc[0], sc[1]), pack2_bf16(sc[2], sc[3])};
        const s16x4 pop = __builtin_bit_cast(s16x4, pw);
#pragma unroll
        for (int n = 0; n < NT; ++n) {
            // V^T operand: lane (g, j) points at dims 16n + 4(j%4) .. +3 of token 4g + j/4; the
            // transposing read hands dim 16n + c of tokens 4g .. 4g+3 to lane (g, c)
            const s16x4 vop = lds_read_tr16(vtile + (4 * g + (c >> 2)) * VROW + (16 * n + 4 * (c & 3)) * 2);
            acc[n] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vop, pop, acc[n], 0, 0, 0);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };
    auto valid_in = [&](int j) { return min(BS, L - (blk_lo + wave + kWaves * j) * BS); };

    if (n_mine > 0) {
        u32x4 ka[NP], va[NP], kb[NP], vb[NP];
        load_tile(0, ka, va);
        int j = 0;
        for (; j + 2 < n_mine; j += 2) {
            load_tile(j + 1, kb, vb);
            consume(ka, va, BS);
            load_tile(j + 2, ka, va);
            consume(kb, vb, BS);
        }
        if (j + 1 < n_mine) {
            load_tile(j + 1, kb, vb);
            consume(ka, va, BS);
            patch_new_row(j + 1, kb, vb);
            consume(kb, vb, valid_in(j + 1));
        } else {
            patch_new_row(j, ka, va);
            consume(ka, va, valid_in(j));
        }
    }

    float l_tot = l_run + __shfl_xor(l_run, 16);
    l_tot += __shfl_xor(l_tot, 32);
    __syncthreads();   // every wave is done with its tile: the same LDS now carries the merge
    float (*sm_acc)[GT][D] = reinterpret_cast<float (*)[GT][D]>(smem);
    float (*sm_m)[GT] = reinterpret_cast<float (*)[GT]>(smem + kWaves * GT * D * 4);
    float (*sm_l)[GT] = reinterpret_cast<float (*)[GT]>(smem + kWaves * GT * D * 4 + kWaves * GT * 4);
#pragma unroll
    for (int n = 0; n < NT; ++n)
#pragma unroll
        for (int i = 0; i < 4; ++i) sm_acc[wave][c][16 * n + 4 * g + i] = acc[n][i];
    if (g == 0) {
        sm_m[wave][c] = m_run;
        sm_l[wave][c] = l_tot;
    }
    __syncthreads();
    merge_waves_and_store<true, D, GT>(a, sm_acc, sm_m, sm_l, tid, s, head0, heads_left, split);
    }   // next piece of work
}

// Merge the spans of one (sequence, query head): thread c owns head dimension c.
template <bool BF16, int D, bool INL>
__global__ __launch_bounds__(D) void decode_combine_kernel(const Args<INL> a)
{
    const int qrow = blockIdx.x;  // s * n_q_heads + head
    const int s = qrow / a.n_q_heads;
    const int c = threadIdx.x;
    const int B = a.block_size;
    int table_row, L;
    resolve_row<INL>(a, s, table_row, L);
    const int n_blk_seq = (L + B - 1) / B;
    const int n_parts = min((n_blk_seq + a.span_blocks - 1) / a.span_blocks, a.n_splits);
    const float *ml = a.ws_ml + static_cast<long long>(qrow) * a.n_splits * 2;
    const float *pa = a.ws_acc + static_cast<long long>(qrow) * a.n_splits * D;
    float mm = kNegBig;
    for (int i = 0; i < n_parts; ++i) mm = fmaxf(mm, ml[2 * i]);
    float o = 0.f, ll = 0.f;
    for (int i = 0; i < n_parts; ++i) {
        const float wi = fast_exp2(ml[2 * i] - mm);
        o += pa[static_cast<long long>(i) * D + c] * wi;
        ll += ml[2 * i + 1] * wi;
    }
    store_out<BF16>(a.out, static_cast<long long>(qrow) * D + c, ll > 0.f ? o / ll : 0.f);
}

template <bool INL>
using AttnKernel = void (*)(Args<INL>);

template <bool BF16, int D, int BS, bool INL>
AttnKernel<INL> kernel_by_heads(int gt)
{
    switch (gt) {
        case 1: return decode_attn_kernel<BF16, D, BS, 1, INL>;
        case 2: return decode_attn_kernel<BF16, D, BS, 2, INL>;
        case 4: return decode_attn_kernel<BF16, D, BS, 4, INL>;
        default: return decode_attn_kernel<BF16, D, BS, 8, INL>;
    }
}

template <bool BF16, int D, bool INL>
AttnKernel<INL> kernel_by_block(int block_size, int gt)
{
    // the block sizes serving systems use get the unrolled, prefetching tile loop; the rest the run-time one
    if (block_size == 16) return kernel_by_heads<BF16, D, 16, INL>(gt);
    if (BF16 && block_size == 32) return kernel_by_heads<BF16, D, 32, INL>(gt);
    if (BF16 && block_size == 64) return kernel_by_heads<BF16, D, 64, INL>(gt);
    return kernel_by_heads<BF16, D, 0, INL>(gt);
}

// The kernels of one launch: attention, and the work-list and merge kernels it may need.  INL: the
// instantiations that take the step's context lengths and new block ids from the kernel
// arguments (see DecodeArgsInl).
template <bool INL>
struct LaunchKernels {
    AttnKernel<INL> attn = nullptr, plan = nullptr, combine = nullptr;
};
template <bool INL>
LaunchKernels<INL> kernels_for(const mux_pool *pool, int gt)
{
    const bool bf16 = pool->dtype == MUX_BF16;
    LaunchKernels<INL> k;
    k.plan = decode_plan_kernel<INL>;
    if (pool->head_dim == 128) {
        k.combine = bf16 ? decode_combine_kernel<true, 128, INL> : decode_combine_kernel<false, 128, INL>;
        k.attn = gt == 16 ? decode_attn_group_kernel<128, INL>
                          : (bf16 ? kernel_by_block<true, 128, INL>(pool->block_size, gt) : kernel_by_block<false, 128, INL>(pool->block_size, gt));
    } else if (pool->head_dim == 64) {
        k.combine = bf16 ? decode_combine_kernel<true, 64, INL> : decode_combine_kernel<false, 64, INL>;
        k.attn = gt == 16 ? decode_attn_group_kernel<64, INL>
                          : (bf16 ? kernel_by_block<true, 64, INL>(pool->block_size, gt) : kernel_by_block<false, 64, INL>(pool->block_size, gt));
    }
    return k;
}

// The matrix-core kernel covers bf16 pools with 16-token blocks and groups of >= 4 query heads.
bool uses_group_kernel(const mux_pool *pool, int group)
{
    return pool->dtype == MUX_BF16 && pool->block_size == 16 && group >= 4;
}

int env_int(const char *name, int fallback)
{
    const char *v = std::getenv(name);
    return v && *v ? std::atoi(v) : fallback;
}

// Workgroups of `fn` the current GPU holds at once: compute units x the occupancy the runtime
// reports for the kernel (asked once per (device, kernel); MUX_DECODE_WG_PER_CU overrides it).
// The attention launch has exactly this many workgroups, so all of them start together and each
// walks its own share of the work list.  The cache is the library's only process-wide state:
// a read-mostly table of numbers that are properties of the hardware, guarded by a mutex.
long long resident_workgroups(const void *fn)
{
    static std::mutex mu;
    static std::map<std::pair<int, const void *>, long long> known;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        dev = 0;
    }
    std::lock_guard<std::mutex> lock(mu);
    const auto key = std::make_pair(dev, fn);
    auto it = known.find(key);
    if (it != known.end()) return it->second;
    int cus = 0, per_cu = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    static const int forced = env_int("MUX_DECODE_WG_PER_CU", 0);
    if (forced > 0)
        per_cu = forced;
    else if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kThreads, 0) !=
                 hipSuccess ||
             per_cu <= 0)
        per_cu = 2;
    (void)hipGetLastError();
    const long long n = static_cast<long long>(cus) * per_cu;
    known[key] = n;
    return n;
}

}  // namespace

// A launch is cut into at least this many pieces (row x kv head x head pass x span) when its rows
// are long enough to be cut at all.
constexpr long long kWantedPieces = 2048;

mux_decode_plan mux_plan_decode(const mux_pool *pool, int32_t n_seqs, int32_t n_q_heads, int32_t n_kv_heads,
                                int32_t max_ctx_len)
{
    mux_decode_plan plan{};
    const int group = n_q_heads / n_kv_heads;
    int gt = 1;
    while (gt < group && gt < 8) gt *= 2;
    if (uses_group_kernel(pool, group)) gt = 16;
    plan.heads_per_pass = gt;
    plan.n_passes = (group + gt - 1) / gt;

    const int B = pool->block_size;
    const long long ctx_blocks = (static_cast<long long>(max_ctx_len) + B - 1) / B;
    // Span: as long as possible (a workgroup pays its start-up latency and the merge of its
    // waves once, and a lone long workgroup still streams fast), but short enough that the
    // grid has at least ~2 workgroups per resident slot; whole blocks, a multiple of the wave
    // count, at most what a wave can index from one register.
    static const int forced = env_int("MUX_DECODE_SPAN_BLOCKS", 0);
    const long long max_span = kWaves * kMaxWaveBlocks;
    long long span;
    if (forced > 0) {
        span = forced;
    } else {
        const long long items = static_cast<long long>(n_seqs) * n_kv_heads * plan.n_passes;
        long long want_splits = (kWantedPieces + items - 1) / items;
        // Splitting adds the work-list and merge kernels to the chain (~20 us end to end) and only pays
        // when whole rows cannot keep the GPU busy: a lone workgroup streams ~50 GB/s, so a
        // few hundred of them already saturate the memory system, and the longest-first
        // assignment balances whole rows well.  Estimate both ways from what the host knows
        // (every row at max_ctx_len; a typical batch holds ~0.56 of that) and keep the rows
        // whole unless the split wins.  MUX_DECODE_SPLIT_SHORT=1 switches the estimate off.
        static const bool always_split = env_int("MUX_DECODE_SPLIT_SHORT", 0) != 0;
        if (want_splits > 1 && ctx_blocks <= max_span && !always_split) {
            const double row_us = static_cast<double>(ctx_blocks) * pool->block_bytes / 50e3;
            const double total_us = 0.56 * static_cast<double>(items) * ctx_blocks * pool->block_bytes / 6.5e6;
            const long long slots = uses_group_kernel(pool, group) ? 512 : 1024;
            const long long whole = (items + slots - 1) / slots;
            const double uneven = items >= slots ? static_cast<double>(whole) * slots / items : 1.0;   // equal rows, worst case
            if (std::max(row_us * whole, total_us * uneven) <= total_us + 20.0) want_splits = 1;
        }
        if (want_splits > ctx_blocks) want_splits = ctx_blocks;
        if (want_splits < 1) want_splits = 1;
        span = (ctx_blocks + want_splits - 1) / want_splits;
    }
    span = (span + kWaves - 1) / kWaves * kWaves;
    if (span > max_span) span = max_span;
    plan.span_tokens = static_cast<int32_t>(span * B);
    plan.n_splits = static_cast<int32_t>((ctx_blocks + span - 1) / span);
    if (plan.n_splits < 1) plan.n_splits = 1;
    // work list: header (4 ints) + one (row, span) pair per possible unit
    plan.plan_bytes = (16 + static_cast<size_t>(n_seqs) * plan.n_splits * 8 + 15) / 16 * 16;
    const size_t partials =
        plan.n_splits > 1 ? static_cast<size_t>(n_seqs) * n_q_heads * plan.n_splits * (pool->head_dim + 2) * sizeof(float) : 0;
    plan.workspace_bytes = plan.plan_bytes + partials;
    return plan;
}

// The largest workspace any launch of 1 .. max_rows rows with max_ctx_len of at most
// max_ctx_len tokens can ask for.  Fewer rows or shorter contexts can need MORE than the largest
// launch (few rows are cut into many spans, each with its partial results), so the bound is a scan:
// the number of spans depends on the row count only while rows x kv heads x passes is below
// kWantedPieces; beyond that it depends on the context alone and the workspace grows with the rows.
size_t mux_decode_workspace_upper_bound(const mux_pool *pool, int32_t max_rows, int32_t n_q_heads, int32_t n_kv_heads,
                                        int32_t max_ctx_len)
{
    const int B = pool->block_size;
    const int32_t max_blocks = static_cast<int32_t>((static_cast<long long>(max_ctx_len) + B - 1) / B);
    const int32_t knee = static_cast<int32_t>(std::min<long long>(max_rows, kWantedPieces));
    size_t worst = 0;
    for (int32_t nb = 1; nb <= max_blocks; ++nb) {
        const int32_t ctx = static_cast<int32_t>(std::min<long long>(static_cast<long long>(nb) * B, max_ctx_len));
        for (int32_t rows = 1; rows <= knee; ++rows)
            worst = std::max(worst, mux_plan_decode(pool, rows, n_q_heads, n_kv_heads, ctx).workspace_bytes);
        worst = std::max(worst, mux_plan_decode(pool, max_rows, n_q_heads, n_kv_heads, ctx).workspace_bytes);
    }
    return worst;
}

namespace {
// Work list (if the attention kernel cannot build it itself), attention, merge of the spans.
template <bool INL>
int launch_kernels(const mux_pool *pool, const mux_decode_plan &plan, Args<INL> &a, long long n_rows, int32_t n_q_heads,
                   int32_t n_kv_heads, hipStream_t st)
{
    const int gt = plan.heads_per_pass;
    const LaunchKernels<INL> k = kernels_for<INL>(pool, gt);
    if (k.attn == nullptr) return MUX_ERR_UNSUPPORTED;
    // as many workgroups as are resident at once (they walk the work list); never more than there is work
    const long long most = n_rows * plan.n_splits * n_kv_heads * plan.n_passes;
    const unsigned g = static_cast<unsigned>(std::min<long long>(most, resident_workgroups(reinterpret_cast<const void *>(k.attn))));
    a.grid_wgs = static_cast<int>(g);
    static const int force_plan_kernel = env_int("MUX_DECODE_PLAN_KERNEL", 0);
    if (n_rows <= kMaxRankedRows && n_rows * plan.n_splits <= kMaxInlineUnits && !force_plan_kernel) {
        a.plan = nullptr;   // the workgroups order the work themselves (see rank_rows and list_units)
    } else {
        hipLaunchKernelGGL(k.plan, dim3(1), dim3(256), 0, st, a);
        if (hipGetLastError() != hipSuccess) return MUX_ERR_HIP;
    }
    hipLaunchKernelGGL(k.attn, dim3(g), dim3(kThreads), 0, st, a);
    if (hipGetLastError() != hipSuccess) return MUX_ERR_HIP;
    if (plan.n_splits > 1) {
        if (n_rows * n_q_heads > 0x7fffffffLL) return MUX_ERR_UNSUPPORTED;
        const unsigned rows = static_cast<unsigned>(n_rows * n_q_heads);
        hipLaunchKernelGGL(k.combine, dim3(rows), dim3(static_cast<unsigned>(pool->head_dim)), 0, st, a);
        if (hipGetLastError() != hipSuccess) return MUX_ERR_HIP;
    }
    return MUX_OK;
}

int launch_rows(const mux_pool *pool, const mux_decode_plan &plan, void *out, const void *q, const int32_t *tables,
                const int32_t *ctx_lens, const int32_t *cu_q_lens, const int32_t *q_start, int32_t n_table_seqs,
                int32_t n_seqs, int32_t n_q_heads, int32_t n_kv_heads, int32_t max_blocks, int32_t max_ctx_len,
                float scale, void *workspace, void *stream, int32_t n_layers = 1, const void *k_new = nullptr,
                const void *v_new = nullptr, const mux_inline_step *inl = nullptr)
{
    DecodeArgsInl a{};   // the ordinary launches pass only its base part
    if (inl != nullptr) {
        const long long ints = 2LL * inl->rows + static_cast<long long>(inl->n_entries) * inl->heads;
        if (inl->rows != n_seqs || inl->rows <= 0 || inl->n_entries < 0 || ints > MUX_INLINE_STEP_INTS || k_new == nullptr ||
            inl->head0 < 0 || inl->head0 + n_layers * n_kv_heads > inl->heads)
            return MUX_ERR_INVALID;
        a.inl_heads = inl->heads;
        a.inl_head0 = inl->head0;
        std::copy(inl->v, inl->v + ints, a.inl);
    }
    a.n_layers = n_layers;
    a.k_new = k_new;
    a.v_new = v_new;
    const long long n_rows = static_cast<long long>(n_seqs) * n_layers;
    a.cu_q_lens = cu_q_lens;
    a.q_start = q_start;
    a.n_table_seqs = n_table_seqs;
    a.kv_base = pool->kv_base;
    a.block_bytes = pool->block_bytes;
    a.num_blocks = static_cast<int>(pool->num_blocks);
    a.block_size = pool->block_size;
    a.out = out;
    a.q = q;
    a.tables = tables;
    a.ctx_lens = ctx_lens;
    a.n_seqs = n_seqs;
    a.n_q_heads = n_q_heads;
    a.n_kv_heads = n_kv_heads;
    a.max_blocks = max_blocks;
    a.max_ctx_len = max_ctx_len;
    a.scale_log2e = scale * kLog2e;
    a.span_blocks = plan.span_tokens / pool->block_size;
    a.n_splits = plan.n_splits;
    a.n_passes = plan.n_passes;
    a.plan = static_cast<int *>(workspace);
    if (plan.n_splits > 1) {
        a.ws_acc = reinterpret_cast<float *>(static_cast<char *>(workspace) + plan.plan_bytes);
        a.ws_ml = a.ws_acc + static_cast<size_t>(n_rows) * n_q_heads * plan.n_splits * pool->head_dim;
    }
    if (n_rows * plan.n_splits * n_kv_heads * plan.n_passes > 0x7fffffffLL) return MUX_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (inl != nullptr) return launch_kernels<true>(pool, plan, a, n_rows, n_q_heads, n_kv_heads, st);
    return launch_kernels<false>(pool, plan, static_cast<DecodeArgs &>(a), n_rows, n_q_heads, n_kv_heads, st);
}
}  // namespace

int mux_launch_decode_attn(const mux_pool *pool, const mux_decode_plan &plan, void *out, const void *q,
                           const int32_t *tables, const int32_t *ctx_lens, int32_t n_seqs, int32_t n_q_heads,
                           int32_t n_kv_heads, int32_t max_blocks, int32_t max_ctx_len, float scale, void *workspace,
                           void *stream)
{
    return launch_rows(pool, plan, out, q, tables, ctx_lens, nullptr, nullptr, n_seqs, n_seqs, n_q_heads, n_kv_heads,
                       max_blocks, max_ctx_len, scale, workspace, stream);
}

// Generic prefill (fp32 pools, block sizes that are not a power of two >= 8): every query row is handled as a
// decode row whose context ends at its own position.  Correct for any supported pool, but it
// re-reads the keys for every row; the matrix-core kernel covers the hot configuration.
int mux_launch_prefill_rows_as_decode(const mux_pool *pool, void *out, const void *q, const int32_t *cu_q_lens,
                                      const int32_t *q_start, const int32_t *tables, int32_t n_seqs, int32_t total_q,
                                      int32_t max_ctx_len, int32_t n_q_heads, int32_t n_kv_heads, int32_t max_blocks,
                                      float scale, void *workspace, void *stream)
{
    const mux_decode_plan plan = mux_plan_decode(pool, total_q, n_q_heads, n_kv_heads, max_ctx_len);
    return launch_rows(pool, plan, out, q, tables, nullptr, cu_q_lens, q_start, n_seqs, total_q, n_q_heads, n_kv_heads,
                       max_blocks, max_ctx_len, scale, workspace, stream);
}

// Fused decoding step over n_layers layers: rows are [layer][sequence]; the plan is made for
// n_layers * n_seqs rows.
int mux_launch_decode_step(const mux_pool *pool, const mux_decode_plan &plan, void *out, const void *q, const void *k_new,
                           const void *v_new, const int32_t *tables, const int32_t *ctx_lens, int32_t n_layers,
                           int32_t n_seqs, int32_t n_q_heads, int32_t n_kv_heads, int32_t max_blocks, int32_t max_ctx_len,
                           float scale, void *workspace, void *stream, const mux_inline_step *inl)
{
    return launch_rows(pool, plan, out, q, tables, ctx_lens, nullptr, nullptr, n_seqs, n_seqs, n_q_heads, n_kv_heads,
                       max_blocks, max_ctx_len, scale, workspace, stream, n_layers, k_new, v_new, inl);
}
