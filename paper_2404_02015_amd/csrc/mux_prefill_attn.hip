// Chunked causal prefill attention over the unified head-wise paged KV pool (gfx950).
//
// MuxServe, Section 2.1: the prefill phase processes all prompt tokens in parallel and is the
// compute-heavy phase; Section 3.4: its K/V live in the same head-wise blocks as everyone
// else's.  Row r of a chunk sits at absolute position q_start + r and attends to keys 0..that
// position; the chunk's own K/V were appended before the call.
//
// The work is two dense contractions per (query tile, KV tile), so it runs on the matrix cores
// (v_mfma_f32_16x16x32_bf16), arranged so that no register shuffling sits between them:
//   S^T = K . Q^T   A = K tile  [16 tokens x 32 dims per instruction, 16-byte reads from LDS]
//                   B = Q^T     [held in registers for the whole kernel]
//                   C = S^T     lane (g, c) holds tokens 4g..4g+3 of query row c
//   O^T = V^T . P^T A = V^T     [16 dims x 32 tokens; ds_read_b64_tr_b16 hands each lane four
//                                tokens of one dim straight out of the row-major LDS tile]
//                   B = P^T     = the S^T registers after softmax, rounded to bf16 in place
//                   C = O^T     lane (g, c) holds dims 4g..4g+3 of query row c
// Both results keep the query row in the lane's low 4 bits, so the running max / sum of a row
// and the rescaling of its accumulator never leave the lane group.
//
// A workgroup of 4 waves owns one (sequence, kv head) and a tile of query-row slices; a wave
// holds CB column blocks of 16 rows (CB = 2: each K / V^T operand read from LDS feeds two
// MFMAs).  Multi-head attention: 4 slices of one head; grouped-query attention: several query
// heads of the group share the K/V tiles.  K/V tiles are fetched once per workgroup, 32 tokens
// per step, with global_load_lds_dwordx4: 16 bytes per lane go from HBM/L2 straight into LDS,
// no registers in between, so several steps can be in flight (kBufs LDS buffers) while the
// matrix cores work on the current one.  Such a load writes the lanes' data contiguously, so
// rows cannot be padded; bank conflicts are avoided by an XOR swizzle of the 16-byte pieces
// inside each row, applied on the global side of the copy.  Block ids are cached in LDS up
// front.  The accumulator is rescaled lazily: the reference maximum of a row only moves
// when a score exceeds it by more than 2^kLazyBits, so most steps skip the rescale.
//
// Blocks of 16 tokens have the block arithmetic folded at compile time; blocks of 8, 32, 64,
// 128 or 256 tokens run the same kernel with it done at run time.  Pools in fp32 or with any
// other block size take a slow generic path (each query row handled like a decode step); see
// mux_launch_prefill_attn.
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <type_traits>

#include "mux_internal.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr int kBS = 16;              // tokens per block of the instantiations with the block size built in
constexpr int kKT = 32;              // tokens per pipeline step (two blocks of 16)
constexpr int kMaxCachedIds = 1024;  // block ids kept in LDS (16 384 tokens of context)
#ifndef MUX_PREFILL_BUFS
#define MUX_PREFILL_BUFS 3
#endif
constexpr int kWgsPerCu = 3;          // 3 x (3 x 16 KiB + ids) of LDS and 3 x 4 x 170 vector registers fit a compute unit
constexpr int kBufs = MUX_PREFILL_BUFS;  // LDS buffers: kBufs - 1 steps are in flight while one is consumed
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -3.0e38f;
constexpr float kLazyBits = 8.0f;    // softmax weights may reach 2^8 before the row is rescaled

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
    int tile_bundle;   // row tiles of one unit dispatched back to back (see the kernel's blockIdx mapping)
    int log2_block;    // log2(tokens per block), for the instantiations that take the block size at run time
    float scale_log2e;
};

__device__ __forceinline__ unsigned pack_bf16(float a, float b)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 v = {static_cast<__bf16>(a), static_cast<__bf16>(b)};  // round to nearest even
    return __builtin_bit_cast(unsigned, v);
}

// Maximum over the four lanes l, l^16, l^32, l^48 (the lane groups that share a query row),
// without a trip through LDS: v_permlane32_swap exchanges the upper half of one register with
// the lower half of another, v_permlane16_swap the odd 16-lane rows with the even ones; with
// both registers holding x, the two results hold "x of my half/row" and "x of the other".
__device__ __forceinline__ float row_max_across_groups(float x)
{
    typedef unsigned u32pair __attribute__((ext_vector_type(2)));
    // plain v_max_f32: fmaxf on values that come out of a bit cast is preceded by one canonicalising
    // max per operand (the inputs are never NaN here); the trailing wait states cover the hazard
    // between a vector write and the lane swap that reads it, which the compiler cannot see
    auto vmax = [](unsigned p, unsigned q) {
        unsigned r;
        asm("v_max_f32 %0, %1, %2\n\ts_nop 1" : "=v"(r) : "v"(p), "v"(q));
        return r;
    };
    const unsigned u = __float_as_uint(x);
    const u32pair h = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const unsigned v = vmax(h[0], h[1]);
    const u32pair r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    return __uint_as_float(vmax(r[0], r[1]));
}

// Transposing LDS read: within each group of 16 lanes, lane i receives element (i % 4) of the
// four 8-byte chunks addressed by lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12 of the group.  The LDS
// byte address is held as a number (see the pinned offsets in the kernel).
__device__ __forceinline__ u32x2 lds_read_tr16_at(unsigned addr)
{
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<lds_s16x4 *>(static_cast<size_t>(addr)));
    return __builtin_bit_cast(u32x2, r);
}
__device__ __forceinline__ u32x4 lds_read16_at(unsigned addr)
{
    typedef __attribute__((address_space(3))) const u32x4 lds_u32x4;
    return *reinterpret_cast<lds_u32x4 *>(static_cast<size_t>(addr));
}

// The K/V tiles travel global -> LDS asynchronously and several of them are meant to stay in
// flight across workgroup barriers.  The compiler cannot know which LDS buffer an in-flight copy
// targets and would wait for all of them before every LDS read and every barrier, so the copy,
// the barrier and the waits of the pipeline are issued by hand; the compiler still orders the
// ordinary LDS reads and writes it generates itself ("memory" clobbers keep them in place).
// A lane's source is base (wave-uniform, scalar registers) + offset (per lane); its 16 bytes
// land at LDS address lds_addr + 16 * lane (lds_addr is wave-uniform).
__device__ __forceinline__ void lds_dma16(const char *base, unsigned offset, unsigned lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 ::"v"(offset), "s"(base), "s"(lds_addr) : "memory", "m0");
}
__device__ __forceinline__ void raw_barrier() { asm volatile("s_barrier" ::: "memory"); }
// s_waitcnt with one counter set and the others left at "do not wait"
template <int N>
__device__ __forceinline__ void wait_vmem()   // at most N vector-memory operations (incl. LDS copies) in flight
{
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}
__device__ __forceinline__ void wait_lds() { __builtin_amdgcn_s_waitcnt(0xF | (0x3 << 14) | (0x7 << 4) | (0x0 << 8)); }

// D: head size.  HT: query heads per workgroup (1, 2 or 4); the other kWaves / HT waves take
// further row slices.  CB: 16-row column blocks per wave.  B16: blocks of 16 tokens (every
// configuration of the paper's workloads), block arithmetic folded at compile time; otherwise the
// block size is a run-time power of two >= 8 (a wave's 8-token run of a tile copy must lie in one block).
#ifndef MUX_PREFILL_MIN_WGS
#define MUX_PREFILL_MIN_WGS 2
#endif
template <int D, int HT, int CB, bool B16>
__global__ __launch_bounds__(kThreads, MUX_PREFILL_MIN_WGS) void prefill_attn_kernel(const PrefillArgs a)
{
    const int lb = B16 ? 4 : a.log2_block;       // log2(tokens per block)
    const int BS = 1 << lb;
    constexpr int RS = 16 * CB;                  // query rows per wave
    constexpr int RT = kWaves / HT;              // row slices per workgroup
    constexpr int QT = RS * RT;                  // query rows per workgroup
    constexpr int KC = D / 32;                   // 32-dim slabs of the head
    constexpr int NT = D / 16;                   // 16-dim slabs of the output
    constexpr int ROWB = D * 2;                  // bytes per token row (unpadded: see the swizzles below)
    constexpr int KBUF = kKT * ROWB;
    constexpr int VBUF = kKT * ROWB;
    constexpr int PIECES = kKT * D * 2 / 16;     // 16-byte pieces per K (or V) step
    constexpr int PPT = PIECES / kThreads;       // pieces per thread
    static_assert(PIECES % kThreads == 0, "tile must split evenly over the workgroup");
    constexpr int PPR = D * 2 / 16;              // pieces per token row
    constexpr int RPC = 256 / ROWB;              // rows per 256-byte sweep over the 64 LDS banks
    static_assert(PPT == 2 || PPT == 1, "a wave copies whole 1 KiB runs");
    // Piece p of row r is stored at piece position p ^ swz(r).  For K the 16 lanes of an operand
    // read take the same piece of 16 different rows: XOR with the row number spreads them over
    // all banks.  For V a transposing read takes two adjacent pieces of 4 (or 8) consecutive rows:
    // XOR with twice the row number keeps the pair adjacent and the rows apart.
    auto kswz = [](int r) { return (r / RPC) % PPR; };
    auto vswz = [](int r) { return 2 * ((r / RPC) % (PPR / 2)); };

    // dynamic LDS (the launcher sizes it): kBufs tile buffers, then the block-id cache
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int *sm_ids = reinterpret_cast<int *>(smem + kBufs * (KBUF + VBUF));
    // the LDS byte address of smem, as a number
    const unsigned smem_lds = static_cast<unsigned>(reinterpret_cast<size_t>((__attribute__((address_space(3))) char *)smem));

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;

    // blockIdx -> (sequence, kv head, pass, row tile).  Two concerns shape the order.  Balance:
    // later row tiles see more keys, so they must be dispatched first.  L2 reuse: workgroups go
    // to the 8 XCDs round-robin and every XCD has its own L2, so row tiles that read the same
    // K/V (same sequence, kv head, pass) should sit on ONE XCD and run at the same time.  Hence:
    // row tiles are taken in bundles of a.tile_bundle, heaviest bundle first; within a bundle all
    // (sequence, head, pass) units are listed, each unit's tiles in consecutive slots of the XCD
    // that owns the unit.  Small launches use bundles of 1 (pure heaviest-first: the tail of the
    // launch matters most), large ones bundle all tiles of a unit (L2 reuse matters most).
    constexpr int kXcds = 8;
    const int kPair = a.tile_bundle;
    const int n_units = a.n_seqs * a.n_kv_heads * a.n_passes;
    const int units_per_xcd = (n_units + kXcds - 1) / kXcds;
    const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
    const int pair = slot / (units_per_xcd * kPair), rem = slot % (units_per_xcd * kPair);
    const int tile = a.n_row_tiles - 1 - (pair * kPair + rem % kPair);
    int w = (rem / kPair) * kXcds + xcd;   // which (sequence, kv head, pass)
    if (tile < 0 || w >= n_units) return;
    const int pass = w % a.n_passes;      w /= a.n_passes;
    const int kvh = w % a.n_kv_heads;     w /= a.n_kv_heads;
    const int s = w;

    const int q_lo = a.cu_q_lens[s];
    const int q_len = min(a.cu_q_lens[s + 1], a.total_q) - q_lo;   // never past the packed q / out
    const int start = a.q_start[s];
    const int row0 = tile * QT;                  // first chunk row of this workgroup
    if (q_lo < 0 || row0 >= q_len || start < 0) return;
    const int rows_here = min(QT, q_len - row0);
    int kv_end = start + row0 + rows_here;       // keys 0 .. kv_end-1 are visible to the last row
    kv_end = min(kv_end, a.max_blocks * BS);
    const int n_steps = (kv_end + kKT - 1) / kKT;
    if (n_steps <= 0) return;
    const int total_len = start + q_len;         // tokens of this sequence that hold real K/V

    const int group = a.n_q_heads / a.n_kv_heads;
    const int slice = wave / HT;                 // which row slice
    const int head_in_group = pass * HT + wave % HT;
    const bool head_ok = head_in_group < group;
    const int head = kvh * group + min(head_in_group, group - 1);
    const int my_row0 = row0 + slice * RS;       // first chunk row of this wave
    const bool wave_active = head_ok && my_row0 < q_len;
    const int wave_first_pos = start + my_row0;
    const int wave_last_pos = start + min(my_row0 + RS - 1, q_len - 1);

    // Q^T operands: for column block b, lane (g, c) holds dims 32k + 8g .. +8 of row 16b + c
    bf16x8 qreg[CB][KC];
    int my_pos[CB];                              // absolute position of this lane's row in block b
#pragma unroll
    for (int b = 0; b < CB; ++b) {
        const int r = min(my_row0 + 16 * b + c, q_len - 1);   // clamp: surplus rows repeat the last one
        my_pos[b] = start + r;
        const char *qrow = static_cast<const char *>(a.q) + (static_cast<long long>(q_lo + r) * a.n_q_heads + head) * (D * 2);
#pragma unroll
        for (int k = 0; k < KC; ++k)
            qreg[b][k] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(qrow + (32 * k + 8 * g) * 2));
    }

    // O^T accumulators, and the row sums of P as one more output slab: with an all-ones A
    // operand the matrix core adds up the (bf16-rounded, as in the numerator) weights of a row
    // over all 32 tokens of a step, so the sum costs no vector instructions and needs no
    // exchange between lane groups (every element of l_acc[b] of lane (g, c) is the sum of row c)
    f32x4 acc[CB][NT], l_acc[CB];
    float m_ref[CB];                             // reference max (log2 domain)
#pragma unroll
    for (int b = 0; b < CB; ++b) {
        m_ref[b] = kNegBig;
        l_acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int n = 0; n < NT; ++n) acc[b][n] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const bf16x8 ones = __builtin_bit_cast(bf16x8, u32x4{0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u});

    // Block ids of the whole key range go to LDS once, so that the K/V loads inside the loop
    // do not wait for a table load first (contexts past kMaxCachedIds blocks read the table).
    const int *trow = a.tables + (static_cast<long long>(s) * a.n_kv_heads + kvh) * a.max_blocks;
    const int n_ids = min(min((n_steps * kKT + BS - 1) >> lb, a.max_blocks), kMaxCachedIds);
    for (int i = tid; i < n_ids; i += kThreads) sm_ids[i] = min(max(trow[i], 0), a.num_blocks - 1);
    __syncthreads();

    // One step's K and V tiles, global -> LDS.  A wave-level load deposits lane l's 16 bytes at
    // (uniform base) + 16 l, i.e. a contiguous 1 KiB run of the tile; the swizzle decides which
    // piece of the row the lane fetches.  The runs of one wave lie inside ONE block, so the block
    // address is wave-uniform (scalar registers) and the lane's part of the address - its row
    // inside the block and its swizzled piece - is the same in every step (two registers per run).
    // The step index is clamped so that every iteration issues the same number of loads and the
    // wait counts below stay exact.
    constexpr int TPR = 64 / PPR;                        // tokens per 1 KiB run
    constexpr int WT = PPT * TPR;                        // tokens of a tile that one wave copies
    static_assert(kBS % WT == 0 && WT == 8, "the runs of a wave must not straddle blocks");
    const int wave_tok0 = wave * WT;                     // first token of the tile this wave copies
    unsigned koff[PPT], voff[PPT];
#pragma unroll
    for (int p = 0; p < PPT; ++p) {
        const int slot = (wave * PPT + p) * 64 + lane;   // 16-byte slot inside the tile
        const int tok = slot / PPR, pos = slot % PPR;
        // with 16-token blocks the row inside the block is the same in every step and part of the
        // lane's offset; otherwise it goes into the wave-uniform base (see issue)
        const int row = B16 ? tok % kBS : tok - wave_tok0;
        koff[p] = row * ROWB + (pos ^ kswz(tok)) * 16;
        voff[p] = (B16 ? kBS * ROWB : 0) + row * ROWB + (pos ^ vswz(tok)) * 16;
    }
    auto block_id = [&](int step_raw) {                  // id of this wave's block in a step (same in all lanes)
        const int blk = (min(step_raw, n_steps - 1) * kKT + wave_tok0) >> lb;
        if (blk < n_ids) return sm_ids[blk];
        return blk < a.max_blocks ? min(max(trow[blk], 0), a.num_blocks - 1) : 0;   // a stale or corrupt entry must not leave the pool
    };
    auto issue = [&](int id, int step_raw, int buf) {
        const char *base = a.kv_base + static_cast<long long>(__builtin_amdgcn_readfirstlane(id)) * a.block_bytes;
        const char *vbase = base;
        if constexpr (!B16) {
            const int row0 = (min(step_raw, n_steps - 1) * kKT + wave_tok0) & (BS - 1);   // first row of the wave's run in its block
            base += row0 * ROWB;
            vbase = base + BS * ROWB;
        }
        const unsigned kb = smem_lds + buf * (KBUF + VBUF);
        const unsigned vb = kb + KBUF;
#pragma unroll
        for (int p = 0; p < PPT; ++p) {
            const int run = wave * PPT + p;              // which 1 KiB run of the tile
            lds_dma16(base, koff[p], kb + run * 1024);
            lds_dma16(vbase, voff[p], vb + run * 1024);
        }
    };
    constexpr int LPS = 2 * PPT;                         // copies per step per lane

    wait_vmem<0>();   // q rows and table entries have arrived: from here on only tile copies are in flight
    for (int t = 0; t < kBufs - 1; ++t) issue(block_id(t), t, t);
    int next_id = block_id(kBufs - 1);   // fetched one iteration ahead of its use
    // Per-lane LDS addresses of the operand reads inside tile 0 (they never change): K piece of
    // slab k in row c (the second 16-token half sits 16 rows further), V piece pair of slab n in
    // row 4g + c/4.  Each is pinned to a register of its own; left alone the compiler keeps a few
    // partial sums instead and re-adds them before every read.
    unsigned k_off[KC], v_off[NT];
#pragma unroll
    for (int k = 0; k < KC; ++k) {
        k_off[k] = smem_lds + c * ROWB + (((4 * k + g) ^ kswz(c)) * 16);
        asm volatile("" : "+v"(k_off[k]));
    }
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int vr = 4 * g + (c >> 2);                        // row inside a half; halves are 16 rows apart,
        const int vpiece = (2 * n + ((c & 3) >> 1)) ^ vswz(vr);  // which leaves the swizzle unchanged
        v_off[n] = smem_lds + vr * ROWB + vpiece * 16 + (c & 1) * 8;
        asm volatile("" : "+v"(v_off[n]));
    }
    // The loop is unrolled over the kBufs buffers so that every LDS address of a step is a
    // loop-invariant per-lane register plus a compile-time offset.
    auto run_step = [&](int step, auto buf_tag) {
        constexpr int buf = decltype(buf_tag)::value;
        // this wave's copies for `step` have landed once only the younger steps' copies are in flight
        wait_vmem<(kBufs - 2) * LPS>();
        raw_barrier();     // everyone's copies for `step` are in LDS, and everyone is done with step - 1 ...
        issue(next_id, step + kBufs - 1, (buf + kBufs - 1) % kBufs);   // ... so its buffer can be refilled
        next_id = block_id(step + kBufs);
        const int kv0 = step * kKT;
        if (kv0 + kKT > total_len) {
            // slots past the sequence's tokens hold stale bytes (possibly NaN): zero those V rows
            // so that 0 * x stays 0 (their scores are masked: they lie beyond every row's position)
            char *vz = smem + buf * (KBUF + VBUF) + KBUF;
            const int first = max(total_len - kv0, 0) * PPR;
            for (int i = first + tid; i < kKT * PPR; i += kThreads) *reinterpret_cast<u32x4 *>(vz + i * 16) = u32x4{0, 0, 0, 0};
            wait_lds();
            raw_barrier();
        }
        if (wave_active && kv0 <= wave_last_pos) {
            // S^T for the two 16-token halves and the CB column blocks
            f32x4 st[CB][2];
#pragma unroll
            for (int b = 0; b < CB; ++b) st[b][0] = st[b][1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int hf = 0; hf < 2; ++hf)
#pragma unroll
                for (int k = 0; k < KC; ++k) {
                    const bf16x8 kop = __builtin_bit_cast(bf16x8, lds_read16_at(k_off[k] + buf * (KBUF + VBUF) + hf * 16 * ROWB));
#pragma unroll
                    for (int b = 0; b < CB; ++b)
                        st[b][hf] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop, qreg[b][k], st[b][hf], 0, 0, 0);
                }
            // Causal mask, only on steps that touch the diagonal (wave-uniform test): masked scores
            // become a huge negative number, whose weight below is exactly 0.  This is the only
            // code that differs between the two kinds of step and it touches nothing but the
            // scores: keeping the accumulators out of duplicated code paths lets them stay in
            // place in their registers (with the softmax written out once per kind of step they
            // were copied to fresh registers in every step).
            if (kv0 + kKT - 1 > wave_first_pos) {
#pragma unroll
                for (int b = 0; b < CB; ++b)
#pragma unroll
                    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (kv0 + hf * 16 + 4 * g + i > my_pos[b]) st[b][hf][i] = kNegBig;
            }
            // lazy online softmax
            bf16x8 pop[CB];
#pragma unroll
            for (int b = 0; b < CB; ++b) {
                float mx = kNegBig;
#pragma unroll
                for (int hf = 0; hf < 2; ++hf)
#pragma unroll
                    for (int i = 0; i < 4; ++i) mx = fmaxf(mx, st[b][hf][i]);
                mx = row_max_across_groups(mx) * a.scale_log2e;   // scale > 0: the max commutes with it
                if (__builtin_amdgcn_ballot_w64(mx > m_ref[b] + kLazyBits) != 0) {
                    const float m_new = fmaxf(m_ref[b], mx);
                    const float alpha = __builtin_amdgcn_exp2f(m_ref[b] - m_new);
                    l_acc[b] *= alpha;
#pragma unroll
                    for (int n = 0; n < NT; ++n) acc[b][n] *= alpha;
                    m_ref[b] = m_new;
                }
                float e[8];
#pragma unroll
                for (int hf = 0; hf < 2; ++hf)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        e[hf * 4 + i] = __builtin_amdgcn_exp2f(__builtin_fmaf(st[b][hf][i], a.scale_log2e, -m_ref[b]));
                // P^T operand: k-slot j of lane group g is token 4g+j of half 0 (j < 4) or half 1
                const u32x4 pw = {pack_bf16(e[0], e[1]), pack_bf16(e[2], e[3]), pack_bf16(e[4], e[5]),
                                  pack_bf16(e[6], e[7])};
                pop[b] = __builtin_bit_cast(bf16x8, pw);
                l_acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pop[b], l_acc[b], 0, 0, 0);
            }
#pragma unroll
            for (int n = 0; n < NT; ++n) {
                // V^T operand: lane (g, j) points at dims 16n + 4(j%4) .. +3 of token 4g + j/4; the
                // transposing read returns dim 16n + c of tokens 4g .. 4g+3 to lane (g, c)
                const unsigned vsrc = v_off[n] + buf * (KBUF + VBUF) + KBUF;
                const u32x2 lo = lds_read_tr16_at(vsrc);                 // half 0
                const u32x2 hi = lds_read_tr16_at(vsrc + 16 * ROWB);     // half 1
                const bf16x8 vop = __builtin_bit_cast(bf16x8, u32x4{lo[0], lo[1], hi[0], hi[1]});
#pragma unroll
                for (int b = 0; b < CB; ++b)
                    acc[b][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, pop[b], acc[b][n], 0, 0, 0);
            }
        }
    };
    static_assert(kBufs == 3, "the unrolling below names the buffers one by one");
    for (int step = 0; step < n_steps; step += kBufs) {
        run_step(step, std::integral_constant<int, 0>{});
        if (step + 1 < n_steps) run_step(step + 1, std::integral_constant<int, 1>{});
        if (step + 2 < n_steps) run_step(step + 2, std::integral_constant<int, 2>{});
    }

    wait_vmem<0>();   // the clamped copies issued past the last step must land before the LDS is reused
    raw_barrier();    // every wave is done with the tile buffers: from here on they carry the outputs
    if (!wave_active) return;
    // The accumulators hold O^T: a lane owns 4 dims of one row per slab, i.e. 8-byte pieces spread
    // over 16 rows per instruction.  Written to memory like that, the stores reach only ~3 TB/s
    // (measured: they cost more than the kernel's whole K/V traffic on short prompts).  Each wave
    // therefore turns its RS x D block around in LDS (row stride padded by 16 bytes: conflict-free
    // both ways) and stores whole rows, 16 bytes per lane, 1 KiB of consecutive rows per instruction.
    constexpr int OSTR = ROWB + 16;
    static_assert(kWaves * RS * OSTR <= kBufs * (KBUF + VBUF), "the output blocks must fit the tile buffers");
    char *oblk = smem + wave * (RS * OSTR);
#pragma unroll
    for (int b = 0; b < CB; ++b) {
        const float l_tot = l_acc[b][0];
        const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
        char *orow = oblk + (16 * b + c) * OSTR + 8 * g;
#pragma unroll
        for (int n = 0; n < NT; ++n) {
            u32x2 o;
            o[0] = pack_bf16(acc[b][n][0] * inv, acc[b][n][1] * inv);
            o[1] = pack_bf16(acc[b][n][2] * inv, acc[b][n][3] * inv);
            *reinterpret_cast<u32x2 *>(orow + 32 * n) = o;   // dims 16n+4g .. +3 of this row
        }
    }
    // LDS operations of one wave complete in order: the reads below see all lanes' writes above
    constexpr int RPI = 1024 / ROWB;             // rows per store instruction
#pragma unroll
    for (int i = 0; i < RS / RPI; ++i) {
        const int row = i * RPI + lane / PPR, piece = lane % PPR;
        const int r = my_row0 + row;
        const u32x4 val = *reinterpret_cast<const u32x4 *>(oblk + row * OSTR + piece * 16);
        if (r < q_len)                           // surplus rows of a ragged tile are dropped
            *reinterpret_cast<u32x4 *>(static_cast<char *>(a.out) + (static_cast<long long>(q_lo + r) * a.n_q_heads + head) * ROWB +
                                       piece * 16) = val;
    }
}

template <int D, int HT, int CB, bool B16>
hipError_t launch_mfma(PrefillArgs a, int max_q_len, hipStream_t st)
{
    constexpr int QT = 16 * CB * (kWaves / HT);
    a.n_row_tiles = (max_q_len + QT - 1) / QT;
    const int group = a.n_q_heads / a.n_kv_heads;
    a.n_passes = (group + HT - 1) / HT;
    const long long units = static_cast<long long>(a.n_seqs) * a.n_kv_heads * a.n_passes;
    // with fewer than ~4 rounds of workgroups balance beats L2 reuse
    a.tile_bundle = units * a.n_row_tiles <= 4 * kWgsPerCu * 256 ? 1 : a.n_row_tiles;
    static const int forced_bundle = std::getenv("MUX_PREFILL_BUNDLE") ? std::atoi(std::getenv("MUX_PREFILL_BUNDLE")) : 0;
    if (forced_bundle > 0) a.tile_bundle = std::min(forced_bundle, a.n_row_tiles);
    const long long bundles = (a.n_row_tiles + a.tile_bundle - 1) / a.tile_bundle;
    const long long grid = (units + 7) / 8 * 8 * bundles * a.tile_bundle;   // see the blockIdx mapping in the kernel
    constexpr int kLds = kBufs * 2 * kKT * D * 2 + kMaxCachedIds * 4;
    // more than 64 KiB of LDS per workgroup has to be granted once per kernel (asked on first use; a
    // refusal is reported by every launch)
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&prefill_attn_kernel<D, HT, CB, B16>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL((prefill_attn_kernel<D, HT, CB, B16>), dim3(static_cast<unsigned>(grid)), dim3(kThreads), kLds, st, a);
    return hipGetLastError();
}

template <int D, int CB, bool B16>
hipError_t launch_by_heads2(int ht, const PrefillArgs &a, int max_q_len, hipStream_t st)
{
    if (ht == 4) return launch_mfma<D, 4, CB, B16>(a, max_q_len, st);
    if (ht == 2) return launch_mfma<D, 2, CB, B16>(a, max_q_len, st);
    return launch_mfma<D, 1, CB, B16>(a, max_q_len, st);
}

template <int D, int CB>
hipError_t launch_by_heads(int ht, const PrefillArgs &a, int max_q_len, hipStream_t st)
{
    if (a.log2_block == 4) return launch_by_heads2<D, CB, true>(ht, a, max_q_len, st);
    return launch_by_heads2<D, CB, false>(ht, a, max_q_len, st);
}

}  // namespace

// Generic path (any supported dtype / block size): defined next to the decode kernel, which it reuses.
int mux_launch_prefill_rows_as_decode(const mux_pool *pool, void *out, const void *q, const int32_t *cu_q_lens,
                                      const int32_t *q_start, const int32_t *tables, int32_t n_seqs, int32_t total_q,
                                      int32_t max_ctx_len, int32_t n_q_heads, int32_t n_kv_heads, int32_t max_blocks,
                                      float scale, void *workspace, void *stream);

// bf16 pools whose blocks hold a power of two >= 8 tokens run on the matrix cores
bool mux_prefill_uses_mfma(const mux_pool *pool)
{
    const int b = pool->block_size;
    return pool->dtype == MUX_BF16 && b >= 8 && (b & (b - 1)) == 0;
}

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
    for (a.log2_block = 0; (1 << a.log2_block) < pool->block_size; ++a.log2_block) {
    }
    const int group = n_q_heads / n_kv_heads;
    const int ht = group >= 4 ? 4 : (group >= 2 ? 2 : 1);
    // Two column blocks per wave (each K / V operand read feeds two matrix instructions) once the
    // chunks are long enough to fill them AND the launch would still fill the GPU: a launch of
    // few rows over long contexts (the last stage of a chunked batch) is a few long-running
    // workgroups, and halving their rows doubles the workgroups that share the work.
    static const int forced_cb = std::getenv("MUX_PREFILL_CB") ? std::atoi(std::getenv("MUX_PREFILL_CB")) : 0;
    int cb = max_q_len >= 32 * (kWaves / ht) ? 2 : 1;
    if (cb == 2) {
        const long long rows2 = 32 * (kWaves / ht);
        const long long est_wgs = static_cast<long long>(n_kv_heads) * ((group + ht - 1) / ht) * (total_q / rows2 + (n_seqs + 1) / 2);
        if (est_wgs < kWgsPerCu * 256) cb = 1;
    }
    if (forced_cb) cb = forced_cb;
    const long long rows_per_wg = 16 * cb * (kWaves / ht);
    const long long grid = ((max_q_len + rows_per_wg - 1) / rows_per_wg + 1) * (static_cast<long long>(n_seqs) * n_kv_heads * ((group + ht - 1) / ht) + 7);
    if (grid > 0x7fffffffLL) return MUX_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t rc;
    if (pool->head_dim == 128)
        rc = cb == 2 ? launch_by_heads<128, 2>(ht, a, max_q_len, st) : launch_by_heads<128, 1>(ht, a, max_q_len, st);
    else if (pool->head_dim == 64)
        rc = cb == 2 ? launch_by_heads<64, 2>(ht, a, max_q_len, st) : launch_by_heads<64, 1>(ht, a, max_q_len, st);
    else
        return MUX_ERR_UNSUPPORTED;
    if (rc != hipSuccess) {
        (void)hipGetLastError();
        return MUX_ERR_HIP;
    }
    return MUX_OK;
}
