"""GPU parity: the HIP path against the CPU oracle, element by element, through the C ABI.

Block tables and appended bytes must be bit-exact; attention outputs must agree within
max-abs 2e-2 (bf16 K/V) or 1e-4 (fp32 K/V).  Inputs are seeded and synthetic.
"""
import numpy as np
import pytest
import torch

import mux_harness as H
from paper_2404_02015_amd import binding as mx
from paper_2404_02015_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[case] " + msg, flush=True)


# ---------------------------------------------------------------------------------
# KV append: bit-exact scatter, nothing else touched
# ---------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,head_dim,block_size,n_kv", [
    ("bf16", 128, 16, 4), ("bf16", 64, 16, 8), ("fp32", 128, 16, 2), ("fp32", 64, 8, 3), ("bf16", 128, 1, 2),
    ("bf16", 64, 32, 5),
])
def test_append_is_bit_exact_and_touches_nothing_else(dtype, head_dim, block_size, n_kv):
    _say("append %s d=%d B=%d Hkv=%d" % (dtype, head_dim, block_size, n_kv))
    rng = np.random.Generator(np.random.PCG64(101))
    n_blocks = 700
    ls = H.Lockstep(n_blocks, block_size, head_dim, dtype, wl.placement_order(rng, n_blocks))
    shape = wl.ModelShape("t", n_kv, n_kv, head_dim)
    lens = np.array([0, 1, block_size, block_size + 1, 3 * block_size + 2, 5], dtype=np.int32)
    job = H.open_job(ls, 0, shape, lens.size, int(lens.max()) + 2 * block_size + 3)
    H.extend(ls, job, lens, seed=5)                       # many tokens per sequence (prefill-like)
    H.extend(ls, job, lens + 1, seed=6)                   # one token per sequence (decode-like)
    H.extend(ls, job, lens + np.array([0, 2, 0, block_size, 1, 0], np.int32) + 1, seed=7)
    torch.cuda.synchronize()
    got = ls.pool_image()
    want = np.full_like(got, H.SENTINEL16)
    for s in range(job.n_seqs):
        for pos in range(int(job.lens[s])):
            for h in range(n_kv):
                bid = job.tables[s, h, pos // block_size]
                for which in (0, 1):
                    want[bid, which, pos % block_size] = ls.orc.read_row(bid, pos % block_size, which).view(np.uint16)
    assert np.array_equal(got, want)
    ls.check_counters()


def test_append_skips_out_of_range_tokens():
    ls = H.Lockstep(64, 16, 128, "bf16")
    shape = wl.ModelShape("t", 2, 2, 128)
    job = H.open_job(ls, 0, shape, 2, 64, poison=True)
    ids = ls.alloc(0, 2)
    job.tables[0, :, 0] = ids
    job.tables_dev.copy_(torch.from_numpy(job.tables))
    k = wl.randn_values(1, (5, 2, 128)).cuda()
    v = wl.randn_values(2, (5, 2, 128)).cuda()
    # token 0 is fine; the others name a bad sequence, a negative position, a position past
    # the table and an entry holding an out-of-range id
    tok_seq = torch.tensor([0, 7, 0, 0, 0], dtype=torch.int32, device="cuda")
    tok_pos = torch.tensor([3, 0, -1, 4000, 16], dtype=torch.int32, device="cuda")
    mx.mux_kv_append(ls.lib, k, v, tok_seq, tok_pos, job.tables_dev)
    torch.cuda.synchronize()
    img = ls.pool_image()
    want = np.full_like(img, H.SENTINEL16)
    for h in range(2):
        want[ids[h], 0, 3] = wl.as_bits(k.cpu())[0, h]
        want[ids[h], 1, 3] = wl.as_bits(v.cpu())[0, h]
    assert np.array_equal(img, want)


# ---------------------------------------------------------------------------------
# decode attention
# ---------------------------------------------------------------------------------
def _decode_case(dtype, head_dim, block_size, n_q, n_kv, lens, seed, scale=None, n_blocks=None):
    lens = np.asarray(lens, dtype=np.int32)
    need = int(((lens + block_size - 1) // block_size).sum()) * n_kv
    n_blocks = n_blocks or need + 64
    rng = np.random.Generator(np.random.PCG64(seed))
    ls = H.Lockstep(n_blocks, block_size, head_dim, dtype, wl.placement_order(rng, n_blocks))
    shape = wl.ModelShape("t", n_q, n_kv, head_dim)
    job = H.open_job(ls, 0, shape, lens.size, int(lens.max()) + block_size)
    H.extend(ls, job, np.maximum(lens - 1, 0), seed=seed * 10 + 1)   # history
    H.extend(ls, job, lens, seed=seed * 10 + 3)                       # this step's token
    q = H.make_q(ls, job, seed * 10 + 5)
    scale = H.default_scale(head_dim) if scale is None else scale
    got = H.decode_gpu(ls, job, q, scale)
    want = H.decode_oracle(ls, job, q, scale)
    torch.cuda.synchronize()
    return ls, job, q, got, want


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_config1_two_models_share_one_pool(dtype):
    """Configuration 1: models A (8 heads) and B (4 heads), head size 64, 4 sequences each,
    contexts uniform in [1,128], one pool of 1024 blocks in seeded random order; each sequence
    appends one token (alloc -> append -> decode)."""
    w = wl.config(1)
    _say("config 1 %s lens=%s" % (dtype, [j.lens.tolist() for j in w.jobs]))
    ls = H.Lockstep(w.num_blocks, w.block_size, w.head_dim, dtype, wl.placement_order(w.rng(), w.num_blocks))
    jobs = [H.open_job(ls, j.model_id, j.shape, j.n_seqs, 128 + 16) for j in w.jobs]
    for j, st in zip(w.jobs, jobs):
        H.extend(ls, st, j.lens - 1, seed=w.seed * 100 + j.model_id)
    streams = [torch.cuda.Stream() for _ in jobs]
    outs = []
    for j, st, stream in zip(w.jobs, jobs, streams):
        stream.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(stream):
            H.extend(ls, st, j.lens, seed=w.seed * 100 + 10 + j.model_id, stream=stream)
            q = H.make_q(ls, st, w.seed * 100 + 20 + j.model_id)
            outs.append((q, H.decode_gpu(ls, st, q, H.default_scale(w.head_dim), stream=stream)))
    torch.cuda.synchronize()
    for st, (q, got) in zip(jobs, outs):
        H.assert_close(got, H.decode_oracle(ls, st, q, H.default_scale(w.head_dim)), dtype, "model %d" % st.model_id)
    all_ids = np.concatenate([st.tables[s, :, :(int(st.lens[s]) + w.block_size - 1) // w.block_size].ravel()
                              for st in jobs for s in range(st.n_seqs)])
    assert len(set(all_ids.tolist())) == all_ids.size       # no block belongs to two (sequence, head) pairs
    ls.check_counters()


@pytest.mark.parametrize("dtype,head_dim,block_size,n_q,n_kv", [
    ("bf16", 128, 16, 4, 4), ("bf16", 128, 16, 8, 2), ("bf16", 128, 16, 16, 2), ("bf16", 128, 16, 6, 2),
    ("bf16", 128, 16, 32, 2), ("bf16", 64, 16, 4, 4), ("bf16", 64, 16, 8, 1),
    ("fp32", 128, 16, 4, 2), ("fp32", 64, 16, 3, 3),
    ("bf16", 128, 1, 2, 2), ("bf16", 128, 8, 4, 2), ("bf16", 128, 32, 2, 2), ("bf16", 64, 8, 2, 1),
    ("bf16", 128, 64, 4, 4), ("bf16", 128, 32, 8, 1), ("bf16", 64, 64, 4, 2), ("bf16", 64, 32, 16, 2), ("bf16", 128, 128, 2, 2),
    ("fp32", 128, 8, 2, 2), ("fp32", 64, 1, 2, 2), ("bf16", 128, 24, 2, 2),
])
def test_decode_matches_oracle_across_shapes(dtype, head_dim, block_size, n_q, n_kv):
    # lengths: empty, single token, block boundaries, several spans with ragged tails
    lens = [0, 1, 2, block_size, block_size + 1, 63, 64, 65, 200, 513, 1000, 1500]
    _say("decode %s d=%d B=%d Hq=%d Hkv=%d" % (dtype, head_dim, block_size, n_q, n_kv))
    ls, job, q, got, want = _decode_case(dtype, head_dim, block_size, n_q, n_kv, lens, seed=block_size + n_q)
    err = H.assert_close(got, want, dtype)
    g = got.float().cpu().numpy()
    assert np.array_equal(g[0], np.zeros_like(g[0]))                          # empty context -> zeros
    # a single cached token returns its V row exactly, for every query head of the group
    v_row = np.stack([ls.orc.read_row(job.tables[1, h, 0], 0, 1) for h in range(n_kv)])
    v_row = torch.from_numpy(v_row.view(np.int16) if dtype == "bf16" else v_row)
    v_row = (v_row.view(torch.bfloat16) if dtype == "bf16" else v_row).float().numpy()
    assert np.array_equal(g[1], np.repeat(v_row, n_q // n_kv, axis=0))
    print("max abs err %.2e" % err)


@pytest.mark.parametrize("n_q,n_kv", [(4, 4), (8, 1)])
def test_decode_batches_too_large_to_rank_in_the_kernel(n_q, n_kv):
    """More than 256 sequences of one span each: the work list comes from the plan kernel rather
    than from the attention kernel's own ranking.  Includes empty and one-token contexts."""
    _say("decode with 700 sequences, Hq=%d Hkv=%d" % (n_q, n_kv))
    rng = np.random.default_rng(n_q)
    lens = rng.integers(0, 260, 700)
    lens[:4] = [0, 1, 16, 17]
    ls, job, q, got, want = _decode_case("bf16", 128, 16, n_q, n_kv, [int(x) for x in lens], seed=40 + n_q)
    err = H.assert_close(got, want, "bf16")
    assert not got[0].float().abs().max().item()
    print("max abs err %.2e" % err)


@pytest.mark.parametrize("n_q,n_kv", [(2, 2), (8, 1), (4, 1)])
def test_decode_few_long_rows_are_split_into_spans(n_q, n_kv):
    """A handful of long rows cannot fill the GPU as whole rows: the host plan splits them into spans
    (partial results in the workspace, merged by the combine kernel).  Short and empty rows ride along."""
    _say("decode, few long rows, Hq=%d Hkv=%d" % (n_q, n_kv))
    lens = [4000, 3000, 17, 0, 2500]
    ls, job, q, got, want = _decode_case("bf16", 128, 16, n_q, n_kv, lens, seed=60 + n_q)
    plan_only = 16 + len(lens) * 8 + 16
    assert mx.mux_decode_workspace_bytes(ls.lib, len(lens), n_q, n_kv, 4000) > plan_only    # the plan did split
    err = H.assert_close(got, want, "bf16")
    assert not got[3].float().abs().max().item()
    print("max abs err %.2e" % err)


@pytest.mark.parametrize("n_rows,longest", [(230, 16000), (250, 21000)])
@pytest.mark.parametrize("n_q,n_kv", [(2, 2), (8, 1)])
def test_decode_one_long_row_among_hundreds_of_short_ones(n_q, n_kv, n_rows, longest):
    """The span count follows the longest context, so one long row makes every row a split row.
    230 rows x 4 spans = 920 units: the attention kernel lists them itself; 250 rows x 6 spans =
    1 500 units: more than it holds, the plan kernel lists them.  Every other row has a short (or
    empty) context and only a last span."""
    _say("decode, %d rows, one of %d tokens, Hq=%d Hkv=%d" % (n_rows, longest, n_q, n_kv))
    rng = np.random.default_rng(n_rows + n_q)
    lens = rng.integers(0, 70, n_rows)
    lens[n_rows // 3] = longest
    lens[5] = 4097                                   # one more row with a full span and a one-token last span
    ls, job, q, got, want = _decode_case("bf16", 128, 16, n_q, n_kv, [int(x) for x in lens], seed=90 + n_q)
    spans = -(-longest // 4096)
    assert (n_rows * spans <= 1024) == (n_rows == 230)
    err = H.assert_close(got, want, "bf16")
    print("max abs err %.2e" % err)


def test_decode_rows_sum_to_one_on_gpu():
    """V == 1 everywhere => O == 1 (softmax weights sum to one), checked on the GPU path."""
    rng = np.random.Generator(np.random.PCG64(3))
    ls = H.Lockstep(4096, 16, 128, "bf16", wl.placement_order(rng, 4096))
    shape = wl.ModelShape("t", 8, 4, 128)
    lens = np.array([5, 77, 640, 1999], dtype=np.int32)
    job = H.open_job(ls, 0, shape, 4, 2048)
    k, v, ts, tp = H.extend(ls, job, lens, seed=9)
    mx.mux_kv_append(ls.lib, k, torch.ones_like(v), ts, tp, job.tables_dev)
    q = H.make_q(ls, job, 10)
    got = H.decode_gpu(ls, job, q, 0.3).float().cpu().numpy()
    assert np.abs(got - 1.0).max() <= 2.0 ** -8


def test_decode_dominant_key_and_large_scores():
    ls = H.Lockstep(512, 16, 128, "fp32")
    shape = wl.ModelShape("t", 1, 1, 128)
    job = H.open_job(ls, 0, shape, 1, 320)
    k, v, ts, tp = H.extend(ls, job, np.array([300], np.int32), seed=21)
    q = (30.0 * k[123]).reshape(1, 1, 128).contiguous()     # scores of a few thousand
    got = H.decode_gpu(ls, job, q, 1.0)
    want = H.decode_oracle(ls, job, q, 1.0)
    H.assert_close(got, want, "fp32")
    assert np.abs(got.cpu().numpy()[0, 0] - v[123, 0].cpu().numpy()).max() < 1e-4


def test_physical_placement_is_invisible_bit_for_bit():
    outs = []
    for scramble_seed in (1, 2):
        rng = np.random.Generator(np.random.PCG64(scramble_seed))
        ls = H.Lockstep(3000, 16, 128, "bf16", wl.placement_order(rng, 3000))
        shape = wl.ModelShape("t", 8, 2, 128)
        job = H.open_job(ls, 0, shape, 3, 1200)
        H.extend(ls, job, np.array([17, 600, 1111], np.int32), seed=33)
        q = H.make_q(ls, job, 34)
        outs.append((job.tables.copy(), H.decode_gpu(ls, job, q, 0.09).cpu()))
    assert not np.array_equal(outs[0][0], outs[1][0])
    assert torch.equal(outs[0][1].view(torch.int16), outs[1][1].view(torch.int16))


def test_max_ctx_hint_larger_than_needed_changes_nothing():
    ls, job, q, got, want = _decode_case("bf16", 128, 16, 4, 4, [40, 300], seed=77)
    loose = H.decode_gpu(ls, job, q, H.default_scale(128), max_ctx_len=job.tables.shape[2] * 16)
    H.assert_close(loose, want, "bf16")


@pytest.mark.parametrize("hint", [1, 64, 100, 1000])
def test_max_ctx_hint_smaller_than_a_context_cuts_it_there(hint):
    """Tokens beyond max_ctx_len are ignored (the header says so): the result is the attention over the
    first max_ctx_len tokens of the longer sequences, and nothing is read past the hint."""
    _say("decode with max_ctx_len %d below some contexts" % hint)
    lens = [300, 40, 100, 0, 1500]
    ls, job, q, _, _ = _decode_case("bf16", 128, 16, 8, 2, lens, seed=78)
    got = H.decode_gpu(ls, job, q, H.default_scale(128), max_ctx_len=hint)
    want = H.decode_oracle(ls, job, q, H.default_scale(128), ctx_lens=np.minimum(job.lens, hint))
    H.assert_close(got, want, "bf16")


@pytest.mark.parametrize("idx", [2, 3, 5])
def test_small_decode_configs_every_output(idx):
    """Shrunk versions of configurations 2, 3 and 5 (same models, fewer and shorter sequences)
    where the oracle checks every output element."""
    w = wl.config(idx, small=True)
    _say("small config %d: %s" % (idx, [(j.shape.name, j.n_seqs, int(j.lens.max())) for j in w.jobs]))
    rng = w.rng()
    if w.placement == "churn":
        ls = H.Lockstep(w.num_blocks, w.block_size, w.head_dim, "bf16", None)
        wl.run_churn(rng, w.churn_ops, 512, ls.alloc_or_none, ls.free, n_models=len(w.jobs))
        ls.check_counters()
    else:
        ls = H.Lockstep(w.num_blocks, w.block_size, w.head_dim, "bf16", wl.placement_order(rng, w.num_blocks))
    states, outs = [], []
    for j in w.jobs:
        st = H.open_job(ls, j.model_id, j.shape, j.n_seqs, int(j.lens.max()) + 16)
        H.extend(ls, st, j.lens - 1, seed=w.seed * 100 + j.model_id)
        states.append(st)
    streams = [torch.cuda.Stream() for _ in states]
    torch.cuda.synchronize()
    for j, st, stream in zip(w.jobs, states, streams):
        with torch.cuda.stream(stream):
            H.extend(ls, st, j.lens, seed=w.seed * 100 + 50 + j.model_id, stream=stream)
            q = H.make_q(ls, st, w.seed * 100 + 70 + j.model_id)
            outs.append((q, H.decode_gpu(ls, st, q, H.default_scale(w.head_dim), stream=stream)))
    torch.cuda.synchronize()
    for st, (q, got) in zip(states, outs):
        err = H.assert_close(got, H.decode_oracle(ls, st, q, H.default_scale(w.head_dim)), "bf16", st.shape.name)
        print("model %s max abs err %.2e" % (st.shape.name, err))
    ls.check_counters()


# ---------------------------------------------------------------------------------
# chunked causal prefill attention
# ---------------------------------------------------------------------------------
def _prefill_case(dtype, head_dim, block_size, n_q, n_kv, lens, q_starts, seed, scale=None):
    """Sequences of `lens` tokens, all K/V appended; the chunk of sequence s is its rows
    q_starts[s] .. lens[s]-1."""
    lens, q_starts = np.asarray(lens, np.int32), np.asarray(q_starts, np.int32)
    need = int(((lens + block_size - 1) // block_size).sum()) * n_kv
    rng = np.random.Generator(np.random.PCG64(seed))
    ls = H.Lockstep(need + 64, block_size, head_dim, dtype, wl.placement_order(rng, need + 64))
    shape = wl.ModelShape("t", n_q, n_kv, head_dim)
    job = H.open_job(ls, 0, shape, lens.size, int(lens.max()) + block_size)
    H.extend(ls, job, q_starts, seed=seed * 10 + 1)        # earlier chunks
    H.extend(ls, job, lens, seed=seed * 10 + 3)            # this chunk's K/V (append before attention)
    q_lens = lens - q_starts
    q = H.make_q(ls, job, seed * 10 + 5, n_rows=int(q_lens.sum()))
    scale = H.default_scale(head_dim) if scale is None else scale
    got = H.prefill_gpu(ls, job, q, q_lens, q_starts, scale)
    want = H.prefill_oracle(ls, job, q, q_lens, q_starts, scale)
    torch.cuda.synchronize()
    return ls, job, q, got, want


@pytest.mark.parametrize("dtype,head_dim,block_size,n_q,n_kv", [
    ("bf16", 128, 16, 2, 2), ("bf16", 128, 16, 4, 2), ("bf16", 128, 16, 8, 2), ("bf16", 128, 16, 16, 2),
    ("bf16", 128, 16, 6, 2), ("bf16", 128, 16, 5, 1), ("bf16", 64, 16, 4, 4), ("bf16", 64, 16, 8, 1),
    ("fp32", 128, 16, 2, 2), ("fp32", 64, 8, 4, 2), ("bf16", 128, 8, 2, 2), ("bf16", 64, 32, 2, 1),
    # other block sizes on the matrix-core path (powers of two from 8 on) and off it (4, 24)
    ("bf16", 128, 32, 4, 2), ("bf16", 128, 64, 8, 1), ("bf16", 128, 128, 2, 2), ("bf16", 64, 8, 4, 4), ("bf16", 64, 64, 2, 2),
    ("bf16", 128, 4, 2, 2), ("bf16", 128, 24, 2, 1),
])
def test_prefill_matches_oracle_across_shapes(dtype, head_dim, block_size, n_q, n_kv):
    # fresh prompts and later chunks; lengths around tile (16/32/64) and block boundaries; a 1-row chunk
    lens =     [1, 15, 16, 17, 31, 33, 64, 65, 130, 200, 257, 300]
    q_starts = [0,  0,  0,  3,  0, 32,  0, 64,   7, 128, 256, 299]
    _say("prefill %s d=%d B=%d Hq=%d Hkv=%d" % (dtype, head_dim, block_size, n_q, n_kv))
    ls, job, q, got, want = _prefill_case(dtype, head_dim, block_size, n_q, n_kv, lens, q_starts, seed=block_size + n_q)
    err = H.assert_close(got, want, dtype)
    # first row of a fresh prompt sees one key: it returns V[0] (exactly, even in bf16)
    g = got.float().cpu().numpy()
    v0 = np.stack([ls.orc.read_row(job.tables[0, h, 0], 0, 1) for h in range(n_kv)])
    v0 = torch.from_numpy(v0.view(np.int16) if dtype == "bf16" else v0)
    v0 = (v0.view(torch.bfloat16) if dtype == "bf16" else v0).float().numpy()
    assert np.array_equal(g[0], np.repeat(v0, n_q // n_kv, axis=0))
    print("max abs err %.2e" % err)


@pytest.mark.parametrize("chunk,block_size", [(1, 16), (7, 16), (16, 16), (33, 16), (64, 16), (100, 16), (33, 8), (50, 32), (40, 64)])
def test_chunked_prefill_equals_oracle_and_unchunked(chunk, block_size):
    """Prompts processed in chunks of any size (alloc -> append -> attend per chunk) give the
    rows an unchunked pass gives."""
    lens = np.array([19, 150, 77], dtype=np.int32)
    n_q, n_kv, d = 4, 2, 128
    rng = np.random.Generator(np.random.PCG64(5))
    ls = H.Lockstep(512, block_size, d, "bf16", wl.placement_order(rng, 512))
    job = H.open_job(ls, 0, wl.ModelShape("t", n_q, n_kv, d), 3, 160)
    q_all = wl.randn_values(55, (int(lens.sum()), n_q, d)).cuda()
    cu_all = np.concatenate([[0], np.cumsum(lens)])
    got = torch.zeros_like(q_all)
    done = np.zeros(3, dtype=np.int32)
    step = 0
    while (done < lens).any():
        q_lens = np.minimum(chunk, lens - done).astype(np.int32)
        H.extend(ls, job, done + q_lens, seed=1000 + step)
        rows = np.concatenate([np.arange(cu_all[s] + done[s], cu_all[s] + done[s] + q_lens[s]) for s in range(3)])
        rows_dev = torch.from_numpy(rows).cuda()
        part = H.prefill_gpu(ls, job, q_all.index_select(0, rows_dev).contiguous(), q_lens, done, 0.09)
        got.index_copy_(0, rows_dev, part)
        done = done + q_lens
        step += 1
    want = H.prefill_oracle(ls, job, q_all, lens, np.zeros(3, np.int32), 0.09)
    H.assert_close(got, want, "bf16")


def test_prefill_chunk_behind_a_context_longer_than_the_id_cache():
    """The MFMA prefill kernel keeps the block ids of the first 1 024 blocks (16 384 tokens) of a
    sequence in LDS and reads the table for the rest; a late chunk of a 17 000-token prompt next to a
    short prompt exercises both paths in one launch."""
    print("[case] prefill chunk at context 17 000", flush=True)
    lens = np.array([17000, 300], dtype=np.int32)
    q_lens = np.array([150, 100], dtype=np.int32)
    n_q, n_kv, d, B = 4, 2, 128, 16
    need = int(((lens + B - 1) // B).sum()) * n_kv
    rng = np.random.Generator(np.random.PCG64(8))
    ls = H.Lockstep(need + 32, B, d, "bf16", wl.placement_order(rng, need + 32))
    job = H.open_job(ls, 0, wl.ModelShape("t", n_q, n_kv, d), 2, int(lens.max()) + B)
    H.extend(ls, job, lens, seed=77)
    q = wl.randn_values(78, (int(q_lens.sum()), n_q, d)).cuda()
    q_start = lens - q_lens
    got = H.prefill_gpu(ls, job, q, q_lens, q_start, H.default_scale(d))
    want = H.prefill_oracle(ls, job, q, q_lens, q_start, H.default_scale(d))
    err = H.assert_close(got, want, "bf16")
    print("max abs err %.2e" % err, flush=True)


def test_prefill_rows_equal_decode_rows_on_gpu():
    """A prefill row at position p and a decode step with context p+1 and the same query see the
    same keys; the two kernels agree within the bf16 tolerance of each against the oracle."""
    ls, job, q, got, want = _prefill_case("bf16", 128, 16, 4, 4, [90], [40], seed=9)
    for r in (0, 17, 49):
        dec = H.decode_gpu(ls, job, q[r:r + 1].contiguous(), H.default_scale(128), ctx_lens=np.array([40 + r + 1], np.int32))
        assert (dec.float() - got[r:r + 1].float()).abs().max().item() <= 2e-2


def test_small_config4_prefill_and_decode_share_the_pool():
    """Shrunk configuration 4: one model runs chunked causal prefill while two others decode,
    each on its own stream, all in one pool."""
    w = wl.config(4, small=True)
    _say("small config 4: %s" % [(j.kind, j.shape.name, j.lens.tolist()) for j in w.jobs])
    ls = H.Lockstep(w.num_blocks, w.block_size, w.head_dim, "bf16", wl.placement_order(w.rng(), w.num_blocks))
    pj, dj = w.jobs[0], w.jobs[1:]
    scale = H.default_scale(w.head_dim)
    dec_states = []
    for j in dj:
        st = H.open_job(ls, j.model_id, j.shape, j.n_seqs, int(j.lens.max()) + 16)
        H.extend(ls, st, j.lens - 1, seed=w.seed * 100 + j.model_id)
        dec_states.append(st)
    pst = H.open_job(ls, pj.model_id, pj.shape, pj.n_seqs, int(pj.lens.max()) + 16)
    streams = [torch.cuda.Stream() for _ in range(3)]
    torch.cuda.synchronize()
    # decode steps on two streams
    dec_out = []
    for j, st, stream in zip(dj, dec_states, streams[1:]):
        with torch.cuda.stream(stream):
            H.extend(ls, st, j.lens, seed=w.seed * 100 + 50 + j.model_id, stream=stream)
            q = H.make_q(ls, st, w.seed * 100 + 70 + j.model_id)
            dec_out.append((q, H.decode_gpu(ls, st, q, scale, stream=stream)))
    # chunked prefill on the third
    q_all = wl.randn_values(w.seed * 100 + 90, (int(pj.lens.sum()), pj.shape.n_q_heads, w.head_dim)).cuda()
    cu_all = np.concatenate([[0], np.cumsum(pj.lens)])
    got = torch.zeros_like(q_all)
    done = np.zeros(pj.n_seqs, dtype=np.int32)
    step = 0
    with torch.cuda.stream(streams[0]):
        while (done < pj.lens).any():
            q_lens = np.minimum(pj.chunk, pj.lens - done).astype(np.int32)
            H.extend(ls, pst, done + q_lens, seed=w.seed * 100 + 200 + step, stream=streams[0])
            rows = np.concatenate([np.arange(cu_all[s] + done[s], cu_all[s] + done[s] + q_lens[s]) for s in range(pj.n_seqs)])
            rows_dev = torch.from_numpy(rows).cuda()
            part = H.prefill_gpu(ls, pst, q_all.index_select(0, rows_dev).contiguous(), q_lens, done, scale, stream=streams[0])
            got.index_copy_(0, rows_dev, part)
            done = done + q_lens
            step += 1
    torch.cuda.synchronize()
    H.assert_close(got, H.prefill_oracle(ls, pst, q_all, pj.lens, np.zeros(pj.n_seqs, np.int32), scale), "bf16", "prefill")
    for st, (q, o) in zip(dec_states, dec_out):
        H.assert_close(o, H.decode_oracle(ls, st, q, scale), "bf16", st.shape.name)
    ls.check_counters()


# ---------------------------------------------------------------------------------
# fused decoding step: append + attention for all layers in one launch
# ---------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,head_dim,block_size,n_q,n_kv,n_layers", [
    ("bf16", 128, 16, 4, 4, 1), ("bf16", 128, 16, 4, 4, 3), ("bf16", 128, 16, 16, 2, 2), ("bf16", 128, 16, 40, 1, 2),
    ("bf16", 128, 16, 6, 2, 2), ("bf16", 64, 16, 8, 2, 2), ("fp32", 128, 16, 2, 2, 2), ("bf16", 128, 8, 4, 2, 2),
    ("fp32", 64, 1, 2, 1, 2), ("bf16", 128, 16, 36, 2, 1),
    ("bf16", 128, 32, 4, 2, 2), ("bf16", 128, 64, 4, 4, 2), ("bf16", 64, 32, 8, 1, 1), ("bf16", 128, 24, 2, 2, 2),
])
def test_fused_step_equals_append_then_decode(dtype, head_dim, block_size, n_q, n_kv, n_layers):
    """mux_decode_step must leave the pool bit-identical to mux_kv_append (checked against the
    oracle's pool) and return what the oracle's append-then-attend returns, layer by layer."""
    _say("fused step %s d=%d B=%d Hq=%d Hkv=%d layers=%d" % (dtype, head_dim, block_size, n_q, n_kv, n_layers))
    # lengths AFTER the step: an idle sequence (0), a first token (1), block boundaries, long ones with several spans
    new_lens = np.array([0, 1, 2, block_size, block_size + 1, 2 * block_size + 1, 64, 65, 257, 1000, 1489], dtype=np.int32)
    old_lens = np.maximum(new_lens - 1, 0)
    n = new_lens.size
    need = int(((new_lens + block_size - 1) // block_size).sum()) * n_kv * n_layers
    rng = np.random.Generator(np.random.PCG64(n_q + n_layers))
    ls = H.Lockstep(need + 64, block_size, head_dim, dtype, wl.placement_order(rng, need + 64))
    shape = wl.ModelShape("t", n_q, n_kv, head_dim)
    layers = [H.open_job(ls, 0, shape, n, int(new_lens.max()) + block_size) for _ in range(n_layers)]
    for l, st in enumerate(layers):
        H.extend(ls, st, old_lens, seed=100 + 7 * l)              # history (per layer its own values and blocks)
    for st in layers:                                             # blocks for the new positions, no data yet
        wl.grow_tables(ls.alloc, 0, st.tables, old_lens, new_lens, block_size, want_changed=False)
        st.tables_dev.copy_(torch.from_numpy(st.tables))
    tables_dev = torch.stack([st.tables_dev for st in layers]).contiguous()
    k_new = wl.randn_values(901, (n_layers, n, n_kv, head_dim), dtype).cuda()
    v_new = wl.randn_values(902, (n_layers, n, n_kv, head_dim), dtype).cuda()
    q = wl.randn_values(903, (n_layers, n, n_q, head_dim), dtype).cuda()
    out = torch.full_like(q, float("nan"))
    lens_dev = torch.from_numpy(new_lens).cuda()
    scale = H.default_scale(head_dim)
    ws = mx.mux_decode_step_workspace_bytes(ls.lib, n_layers, n, n_q, n_kv, int(new_lens.max()))
    wsb = torch.empty(max(ws, 16), dtype=torch.uint8, device="cuda")
    mx.mux_decode_step(ls.lib, out, q, k_new, v_new, tables_dev, lens_dev, int(new_lens.max()), scale, wsb)
    torch.cuda.synchronize()
    # oracle: append the new token of every active sequence, then attend
    active = np.nonzero(new_lens > 0)[0].astype(np.int32)
    for l, st in enumerate(layers):
        ls.orc.kv_append(H.to_oracle(k_new[l])[active], H.to_oracle(v_new[l])[active], active, new_lens[active] - 1, st.tables)
        want = ls.orc.decode_attn(H.to_oracle(q[l]), st.tables, new_lens, n_q, scale)
        H.assert_close(out[l], want, dtype, "layer %d" % l)
    # pool bytes: everything the oracle holds must be in the device pool, bit for bit, and nothing else changed
    got = ls.pool_image()
    want_img = np.full_like(got, H.SENTINEL16)
    for st in layers:
        for s in range(n):
            for pos in range(int(new_lens[s])):
                for h in range(n_kv):
                    bid = st.tables[s, h, pos // block_size]
                    for which in (0, 1):
                        want_img[bid, which, pos % block_size] = ls.orc.read_row(bid, pos % block_size, which).view(np.uint16)
    assert np.array_equal(got, want_img)


@pytest.mark.parametrize("dtype,block_size,n_q,n_kv", [("bf16", 16, 4, 4), ("bf16", 16, 16, 2), ("fp32", 8, 2, 2), ("bf16", 32, 4, 2)])
def test_fused_step_leaves_rows_beyond_the_length_bound_alone(dtype, block_size, n_q, n_kv):
    """mux_decode_step with a max_ctx_len below some rows' lengths: those rows append nothing (not
    one pool byte changes for them) and attend to their first max_ctx_len tokens, exactly as
    mux_decode_attn does with the same bound; the other rows append and attend as usual."""
    print("[case] fused step with rows beyond max_ctx_len, %s B=%d Hq=%d Hkv=%d" % (dtype, block_size, n_q, n_kv), flush=True)
    d = 128
    lens = np.array([40, 100, 33, 64, 7, 65], np.int32)       # lengths after this step's append
    bound = 64                                                 # rows 1 and 5 lie beyond it
    rng = np.random.Generator(np.random.PCG64(91))
    ls = H.Lockstep(800, block_size, d, dtype, wl.placement_order(rng, 800))
    st = H.open_job(ls, 0, wl.ModelShape("t", n_q, n_kv, d), lens.size, 160)
    H.extend(ls, st, lens - 1, seed=41)                                      # history
    wl.grow_tables(ls.alloc, 0, st.tables, lens - 1, lens, block_size, want_changed=False)
    st.tables_dev.copy_(torch.from_numpy(st.tables))
    before = ls.pool_image().copy()
    k_new = wl.randn_values(42, (1, lens.size, n_kv, d), dtype).cuda()
    v_new = wl.randn_values(43, (1, lens.size, n_kv, d), dtype).cuda()
    q = wl.randn_values(44, (1, lens.size, n_q, d), dtype).cuda()
    out = torch.full_like(q, float("nan"))
    scale = H.default_scale(d)
    ws = torch.empty(max(mx.mux_decode_step_workspace_bytes(ls.lib, 1, lens.size, n_q, n_kv, bound), 16), dtype=torch.uint8, device="cuda")
    mx.mux_decode_step(ls.lib, out, q, k_new, v_new, st.tables_dev[None].contiguous(), torch.from_numpy(lens).cuda(), bound, scale, ws)
    torch.cuda.synchronize()
    inside = np.nonzero(lens <= bound)[0].astype(np.int32)
    # pool: exactly the new rows of the sequences inside the bound were written
    want_img = before.copy()
    kb, vb = H.to_oracle(k_new[0]), H.to_oracle(v_new[0])
    row16 = d * ls.elem // 2
    for s in inside:
        p = int(lens[s]) - 1
        for h in range(n_kv):
            bid = st.tables[s, h, p // block_size]
            want_img[bid, 0, p % block_size] = kb[s, h].view(np.uint16).reshape(row16)
            want_img[bid, 1, p % block_size] = vb[s, h].view(np.uint16).reshape(row16)
    assert np.array_equal(ls.pool_image(), want_img)
    # outputs: the oracle with the appended tokens for rows inside the bound, the first `bound` tokens for the others
    ls.orc.kv_append(kb[inside], vb[inside], inside, lens[inside] - 1, st.tables)
    want = ls.orc.decode_attn(H.to_oracle(q[0]), st.tables, np.minimum(lens, bound), n_q, scale)
    H.assert_close(out[0], want, dtype)


def test_decode_on_a_cu_masked_stream_is_bit_identical():
    """A stream restricted to a quarter of the compute units (spread over all XCDs) runs the same
    kernels: outputs equal those of an ordinary stream bit for bit, and the oracle's within tolerance."""
    print("[case] decode on a CU-masked stream", flush=True)
    n_cu = mx.mux_device_cu_count()
    assert n_cu >= 64
    rng = np.random.default_rng(5)
    ls = H.Lockstep(6000, 16, 128, "bf16", wl.placement_order(rng, 6000))
    lens = rng.integers(1, 900, 24).astype(np.int32)
    st = H.open_job(ls, 0, wl.ModelShape("m", 8, 4, 128), lens.size, int(lens.max()) + 16)
    H.extend(ls, st, lens, seed=3)
    q = H.make_q(ls, st, 4)
    scale = H.default_scale(128)
    plain = H.decode_gpu(ls, st, q, scale)
    torch.cuda.synchronize()
    ms = mx.MaskedStream(range(n_cu // 4))
    try:
        with torch.cuda.stream(ms.stream):
            masked = H.decode_gpu(ls, st, q, scale, stream=ms.stream)
        ms.stream.synchronize()
        assert torch.equal(masked.view(torch.int16), plain.view(torch.int16))
        H.assert_close(masked, H.decode_oracle(ls, st, q, scale), "bf16")
    finally:
        torch.cuda.synchronize()
        ms.close()


@pytest.mark.parametrize("n_q,n_kv,share", [(8, 8, 4), (16, 2, 4), (8, 8, 2)])
def test_prefill_on_a_cu_masked_stream_is_bit_identical(n_q, n_kv, share):
    """The prefill kernel maps workgroup index to XCD to keep the row tiles of a (sequence, head)
    on one L2; on a stream restricted to 1/share of the compute units (spread over all XCDs) that
    only changes where a workgroup runs, never what it computes: outputs equal those of an
    ordinary stream bit for bit (many row tiles per head, chunks behind cached prefixes, enough
    workgroups for several rounds on the masked share), and the oracle's within tolerance."""
    print("[case] prefill on a CU-masked stream Hq=%d Hkv=%d share 1/%d" % (n_q, n_kv, share), flush=True)
    n_cu = mx.mux_device_cu_count()
    assert n_cu >= 64
    lens = np.array([700, 1300, 129, 512, 64, 1000, 333, 2048], np.int32)
    q_starts = np.array([0, 788, 0, 256, 63, 0, 300, 1536], np.int32)
    ls, job, q, plain, want = _prefill_case("bf16", 128, 16, n_q, n_kv, lens, q_starts, seed=70 + n_q)
    q_lens = lens - q_starts
    ms = mx.MaskedStream(range(n_cu // share))
    try:
        with torch.cuda.stream(ms.stream):
            masked = H.prefill_gpu(ls, job, q, q_lens, q_starts, H.default_scale(128), stream=ms.stream)
        ms.stream.synchronize()
        assert torch.equal(masked.view(torch.int16), plain.view(torch.int16))
        err = H.assert_close(masked, want, "bf16")
        print("max abs err %.2e" % err, flush=True)
    finally:
        torch.cuda.synchronize()
        ms.close()


def test_decode_step_captured_in_a_graph_replays_correctly():
    """One model's step (mux_kv_append + mux_decode_attn) captured once into a HIP graph and
    replayed for several consecutive steps, with eager work (table growth, input copies, syncs)
    between the replays; every replay must match the oracle.  The entry points allocate nothing
    and enqueue kernels only, so they can be captured."""
    print("[case] decode step in a HIP graph", flush=True)
    rng = np.random.default_rng(12)
    B, d = 16, 128
    shape = wl.ModelShape("g", 16, 4, d)                      # grouped-query: the matrix-core decode kernel
    lens = rng.integers(1, 700, 20).astype(np.int32)
    lens[:3] = [15, 16, 17]                                   # block boundaries are crossed during the replays
    n = lens.size
    ls = H.Lockstep(8000, B, d, "bf16", wl.placement_order(rng, 8000))
    st = H.open_job(ls, 0, shape, n, int(lens.max()) + 64)
    H.extend(ls, st, lens, seed=5)
    scale = H.default_scale(d)
    max_ctx = int(lens.max()) + 16
    k_new = torch.zeros(n, shape.n_kv_heads, d, dtype=torch.bfloat16, device="cuda")
    v_new = torch.zeros_like(k_new)
    q = torch.zeros(n, shape.n_q_heads, d, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros_like(q)
    tok_seq = torch.arange(n, dtype=torch.int32, device="cuda")
    tok_pos = torch.zeros(n, dtype=torch.int32, device="cuda")
    ctx = torch.zeros(n, dtype=torch.int32, device="cuda")
    ws = torch.empty(mx.mux_decode_workspace_bytes(ls.lib, n, shape.n_q_heads, shape.n_kv_heads, max_ctx), dtype=torch.uint8,
                     device="cuda")

    def enqueue():
        mx.mux_kv_append(ls.lib, k_new, v_new, tok_seq, tok_pos, st.tables_dev)
        mx.mux_decode_attn(ls.lib, out, q, st.tables_dev, ctx, max_ctx, scale, ws)

    def next_inputs(step):
        new_lens = st.lens + 1
        wl.grow_tables(ls.alloc, 0, st.tables, st.lens, new_lens, B, want_changed=False)
        st.tables_dev.copy_(torch.from_numpy(st.tables))
        kk, vv = wl.randn_values(700 + step, tuple(k_new.shape)), wl.randn_values(800 + step, tuple(k_new.shape))
        qq = wl.randn_values(900 + step, tuple(q.shape))
        k_new.copy_(kk)
        v_new.copy_(vv)
        q.copy_(qq)
        tok_pos.copy_(torch.from_numpy(new_lens - 1))
        ctx.copy_(torch.from_numpy(new_lens))
        ls.orc.kv_append(H.to_oracle(kk), H.to_oracle(vv), np.arange(n, dtype=np.int32), new_lens - 1, st.tables)
        st.lens = new_lens
        return ls.orc.decode_attn(H.to_oracle(qq), st.tables, new_lens, shape.n_q_heads, scale)

    side = torch.cuda.Stream()
    want = next_inputs(0)                                     # step 0 runs eagerly (also warms every kernel up)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        enqueue()
    side.synchronize()
    H.assert_close(out, want, "bf16", "eager step")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        enqueue()
    worst = 0.0
    for step in range(1, 6):
        want = next_inputs(step)
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        worst = max(worst, H.assert_close(out, want, "bf16", "replay %d" % step))
    ls.check_counters()
    print("graph replays: max abs err %.2e" % worst, flush=True)


@pytest.mark.parametrize("dtype,block_size", [("bf16", 16), ("bf16", 32), ("fp32", 8)])
def test_degenerate_launches(dtype, block_size):
    """Launches with nothing (or next to nothing) to do: a batch whose contexts are all empty, a
    chunked prefill in which some sequences contribute no rows, an append of zero tokens.  No
    output row may be left unwritten or hold anything but what the definition gives."""
    _say("degenerate launches %s B=%d" % (dtype, block_size))
    # decode: every context empty -> all zeros (also through the fused step)
    ls, job, q, got, _ = _decode_case(dtype, 128, block_size, 4, 2, [0, 0, 0], seed=90)
    assert not got.float().abs().max().item()
    # prefill: sequences 0 and 2 have no rows in this chunk, sequence 1 has 37 behind 20 cached tokens, sequence 3 one row
    lens, starts = [33, 57, 0, 1], [33, 20, 0, 0]
    ls, job, q, got, want = _prefill_case(dtype, 128, block_size, 4, 2, lens, starts, seed=91)
    assert got.shape[0] == 38
    H.assert_close(got, want, dtype)
    # append of zero tokens: accepted, nothing written
    before = ls.kv.clone()
    z = torch.zeros(0, 2, 128, dtype=H.torch_dtype(dtype), device="cuda")
    zi = torch.zeros(0, dtype=torch.int32, device="cuda")
    mx.mux_kv_append(ls.lib, z, z, zi, zi, job.tables_dev)
    torch.cuda.synchronize()
    assert torch.equal(before, ls.kv)


@pytest.mark.parametrize("n_q,n_kv", [(2, 1), (8, 1)])
def test_decode_one_very_long_context(n_q, n_kv):
    """A 40 000-token context (2 500 blocks, ten spans of the longest span a workgroup handles) beside
    short ones: many partial results per row, merged by the combine kernel."""
    _say("decode with a 40 000-token context, Hq=%d Hkv=%d" % (n_q, n_kv))
    ls, job, q, got, want = _decode_case("bf16", 128, 16, n_q, n_kv, [40000, 5, 0, 4097], seed=95 + n_q)
    err = H.assert_close(got, want, "bf16")
    print("max abs err %.2e" % err)
