"""Pins for the CPU oracle: closed forms, invariants, brute force and library routines.

The paper prints no worked numeric example for this path, so the oracle is pinned to
what the mathematics fixes: dense softmax attention computed independently in float64
without paging, closed-form special cases, invariants of the paged layout (Section 3.4:
one head per block, several tokens per block, one space for all models), and torch's
own scaled-dot-product attention as a third implementation.  Every test here runs on
the CPU.
"""
import numpy as np
import pytest
import torch

from paper_2404_02015_amd import workloads as wl


# ---------------------------------------------------------------------------------
# helpers that DO NOT use the oracle's arithmetic
# ---------------------------------------------------------------------------------
def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def to_f64(a: np.ndarray) -> np.ndarray:
    return bf16_to_f64(a) if a.dtype == np.uint16 else a.astype(np.float64)


def dense_attention_f64(q, K, V, scale):
    """Textbook softmax(q K^T * scale) V in float64, naive softmax (no max shift)."""
    x = (K @ q) * scale
    w = np.exp(x)
    return (w / w.sum()) @ V, w / w.sum()


def make_case(oracle, seed, n_seqs, n_q, n_kv, d, B, lens, dtype="bf16", num_blocks=None, scramble=True):
    """Random logical K/V per sequence, appended into an oracle pool through random tables."""
    rng = np.random.Generator(np.random.PCG64(seed))
    lens = np.asarray(lens, dtype=np.int32)
    max_blocks = wl.max_blocks_for(lens, B) + 1
    need = int(((lens + B - 1) // B).sum()) * n_kv
    num_blocks = num_blocks or need + 7
    order = wl.placement_order(rng, num_blocks) if scramble else None
    pool = oracle.OraclePool(num_blocks, B, d, oracle.BF16 if dtype == "bf16" else oracle.FP32, order)
    tables = wl.build_tables(lambda m, n: pool.alloc(m, n), 0, lens, n_kv, B, max_blocks)
    total = int(lens.sum())
    k = wl.as_bits(wl.randn_values(seed * 3 + 1, (total, n_kv, d), dtype))
    v = wl.as_bits(wl.randn_values(seed * 3 + 2, (total, n_kv, d), dtype))
    q = wl.as_bits(wl.randn_values(seed * 3 + 3, (n_seqs, n_q, d), dtype))
    tok_seq = np.repeat(np.arange(n_seqs, dtype=np.int32), lens)
    tok_pos = np.concatenate([np.arange(L, dtype=np.int32) for L in lens]) if total else np.zeros(0, np.int32)
    if total:
        pool.kv_append(k, v, tok_seq, tok_pos, tables)
    return pool, tables, lens, q, k, v, tok_seq, tok_pos


# ---------------------------------------------------------------------------------
# attention: brute force, closed forms, invariants
# ---------------------------------------------------------------------------------
@pytest.mark.parametrize("B", [1, 4, 16])
@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("n_q,n_kv", [(2, 2), (4, 2), (6, 1)])
def test_decode_matches_dense_float64(oracle, B, dtype, n_q, n_kv):
    d, lens = 8, [1, 17, 40]
    pool, tables, lens, q, k, v, tok_seq, _ = make_case(oracle, 11 + B, 3, n_q, n_kv, d, B, lens, dtype)
    scale = 0.37
    out = pool.decode_attn(q, tables, lens, n_q, scale)
    g = n_q // n_kv
    kf, vf, qf = to_f64(k), to_f64(v), to_f64(q)
    for s in range(3):
        sel = tok_seq == s
        for i in range(n_q):
            ref, _ = dense_attention_f64(qf[s, i], kf[sel][:, i // g], vf[sel][:, i // g], scale)
            np.testing.assert_allclose(out[s, i], ref, rtol=0, atol=2e-6)


def test_f32_and_f64_rows_agree(oracle):
    pool, tables, lens, q, *_ = make_case(oracle, 5, 2, 4, 4, 64, 16, [333, 1500])
    a = pool.decode_attn(q, tables, lens, 4, 0.125)
    b = pool.decode_attn(q, tables, lens, 4, 0.125, use_f64=True)
    assert np.abs(a - b).max() < 5e-6


def test_weights_sum_to_one_and_ones_value(oracle):
    pool, tables, lens, q, k, v, tok_seq, tok_pos = make_case(oracle, 7, 2, 4, 2, 16, 4, [9, 30])
    for s in range(2):
        for i in range(4):
            w = pool.decode_weights(q, tables, lens, s, i, 4, 0.25)
            assert w.shape == (lens[s],) and (w >= 0).all()
            assert abs(w.sum() - 1.0) < 1e-6
    # V == 1 everywhere  =>  O == 1
    ones = np.full_like(v, 0x3F80)  # bf16 bit pattern of 1.0
    pool.kv_append(k, ones, tok_seq, tok_pos, tables)
    out = pool.decode_attn(q, tables, lens, 4, 0.25)
    np.testing.assert_allclose(out, 1.0, rtol=0, atol=1e-6)


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_single_token_returns_v_exactly(oracle, dtype):
    pool, tables, lens, q, k, v, *_ = make_case(oracle, 13, 3, 4, 2, 32, 16, [1, 1, 1], dtype)
    out = pool.decode_attn(q, tables, lens, 4, 0.5)
    vf = to_f64(v).astype(np.float32)  # [3 tokens][2 kv heads][d]
    for s in range(3):
        for i in range(4):
            assert np.array_equal(out[s, i], vf[s, i // 2])


def test_identical_keys_give_mean_of_values(oracle):
    n, d = 23, 16
    rng = np.random.default_rng(3)
    K = np.tile(rng.standard_normal(d).astype(np.float32), (n, 1))
    V = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal(d).astype(np.float32)
    out = oracle.attn_row(q, K, V, 0.3)
    np.testing.assert_allclose(out, V.astype(np.float64).mean(0), atol=1e-6)


def test_dominant_key_selects_its_value_without_overflow(oracle):
    n, d = 50, 16
    rng = np.random.default_rng(4)
    K = rng.standard_normal((n, d)).astype(np.float32)
    V = rng.standard_normal((n, d)).astype(np.float32)
    q = (30.0 * K[17]).astype(np.float32)  # scores of several hundred: exp overflows without the max shift
    out = oracle.attn_row(q, K, V, 1.0)
    assert np.isfinite(out).all()
    np.testing.assert_allclose(out, V[17], atol=1e-5)


def test_empty_context_gives_zeros(oracle):
    pool, tables, lens, q, *_ = make_case(oracle, 17, 2, 2, 2, 8, 4, [0, 5])
    out = pool.decode_attn(q, tables, lens, 2, 1.0)
    assert np.array_equal(out[0], np.zeros_like(out[0])) and np.isfinite(out).all()


def test_physical_block_permutation_is_invisible(oracle):
    lens, n_kv, d, B = [5, 33, 64], 2, 16, 8
    a = make_case(oracle, 19, 3, 4, n_kv, d, B, lens, scramble=False)
    b = make_case(oracle, 19, 3, 4, n_kv, d, B, lens, scramble=True, num_blocks=257)
    assert not np.array_equal(a[1], b[1])            # tables differ ...
    out_a = a[0].decode_attn(a[3], a[1], a[2], 4, 0.25)
    out_b = b[0].decode_attn(b[3], b[1], b[2], 4, 0.25)
    assert np.array_equal(out_a, out_b)              # ... outputs are bit-identical


def test_gqa_equals_mha_with_repeated_kv_heads(oracle):
    lens, d, B, n_q, n_kv = [12, 31], 16, 4, 6, 2
    pool, tables, lens, q, k, v, tok_seq, tok_pos = make_case(oracle, 23, 2, n_q, n_kv, d, B, lens)
    out_gqa = pool.decode_attn(q, tables, lens, n_q, 0.25)
    g = n_q // n_kv
    k_rep, v_rep = np.repeat(k, g, axis=1), np.repeat(v, g, axis=1)
    mha = oracle.OraclePool(512, B, d, oracle.BF16)
    t2 = wl.build_tables(lambda m, n: mha.alloc(m, n), 0, lens, n_q, B, tables.shape[2])
    mha.kv_append(k_rep, v_rep, tok_seq, tok_pos, t2)
    out_mha = mha.decode_attn(q, t2, lens, n_q, 0.25)
    assert np.array_equal(out_gqa, out_mha)


def test_torch_sdpa_agrees(oracle):
    lens, d, B, n_q, n_kv = [77, 200], 64, 16, 4, 4
    pool, tables, lens, q, k, v, tok_seq, _ = make_case(oracle, 29, 2, n_q, n_kv, d, B, lens, "fp32")
    scale = 1.0 / np.sqrt(d)
    out = pool.decode_attn(q, tables, lens, n_q, scale)
    for s in range(2):
        sel = tok_seq == s
        Kt = torch.from_numpy(k[sel]).permute(1, 0, 2)  # [heads][L][d]
        Vt = torch.from_numpy(v[sel]).permute(1, 0, 2)
        Qt = torch.from_numpy(q[s]).unsqueeze(1)        # [heads][1][d]
        ref = torch.nn.functional.scaled_dot_product_attention(Qt, Kt, Vt, scale=float(scale)).squeeze(1).numpy()
        np.testing.assert_allclose(out[s], ref, atol=2e-6, rtol=0)


# ---------------------------------------------------------------------------------
# prefill: causal offset and chunk bookkeeping
# ---------------------------------------------------------------------------------
def _prefill_inputs(seed, q_lens, n_q, d, dtype="bf16"):
    cu = np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int32)
    qp = wl.as_bits(wl.randn_values(seed, (int(cu[-1]), n_q, d), dtype))
    return cu, qp


def test_prefill_rows_equal_decode_at_that_length(oracle):
    lens, d, B, n_q, n_kv = [21, 40], 16, 8, 4, 2
    pool, tables, lens, _, k, v, *_ = make_case(oracle, 31, 2, n_q, n_kv, d, B, lens)
    q_start = np.array([5, 0], dtype=np.int32)
    q_lens = lens - q_start
    cu, qp = _prefill_inputs(77, q_lens, n_q, d)
    out = pool.prefill_attn(qp, cu, q_start, tables, n_q, 0.25)
    for s in range(2):
        for r in range(int(q_lens[s])):
            L = np.array([0, 0], dtype=np.int32)
            L[s] = q_start[s] + r + 1
            qd = np.zeros((2, n_q, d), dtype=qp.dtype)
            qd[s] = qp[cu[s] + r]
            dec = pool.decode_attn(qd, tables, L, n_q, 0.25)
            assert np.array_equal(out[cu[s] + r], dec[s])


def test_prefill_full_prompt_matches_torch_causal(oracle):
    L, d, B, n_q = 45, 32, 16, 2
    pool, tables, lens, _, k, v, *_ = make_case(oracle, 37, 1, n_q, n_q, d, B, [L], "fp32")
    cu, qp = _prefill_inputs(78, [L], n_q, d, "fp32")
    out = pool.prefill_attn(qp, cu, np.zeros(1, np.int32), tables, n_q, 0.2)
    Qt = torch.from_numpy(qp).permute(1, 0, 2)
    Kt = torch.from_numpy(k).permute(1, 0, 2)
    Vt = torch.from_numpy(v).permute(1, 0, 2)
    ref = torch.nn.functional.scaled_dot_product_attention(Qt, Kt, Vt, is_causal=True, scale=0.2).permute(1, 0, 2).numpy()
    np.testing.assert_allclose(out, ref, atol=2e-6, rtol=0)
    # first row of a fresh prompt sees one key: it returns V[0] exactly
    assert np.array_equal(out[0], v[0])


@pytest.mark.parametrize("chunk", [1, 7, 16, 100])
def test_chunked_prefill_equals_unchunked(oracle, chunk):
    lens, d, B, n_q, n_kv = [19, 50], 16, 8, 4, 2
    pool, tables, lens, *_ = make_case(oracle, 41, 2, n_q, n_kv, d, B, lens)
    cu_full, qp = _prefill_inputs(79, lens, n_q, d)
    full = pool.prefill_attn(qp, cu_full, np.zeros(2, np.int32), tables, n_q, 0.25)
    done = np.zeros(2, dtype=np.int32)
    got = np.zeros_like(full)
    while (done < lens).any():
        q_lens = np.minimum(chunk, lens - done)
        cu = np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int32)
        rows = np.concatenate([np.arange(cu_full[s] + done[s], cu_full[s] + done[s] + q_lens[s]) for s in range(2)])
        part = pool.prefill_attn(qp[rows], cu, done, tables, n_q, 0.25)
        got[rows] = part
        done = done + q_lens
    assert np.array_equal(got, full)


# ---------------------------------------------------------------------------------
# block manager (Section 3.4, Implementation: request blocks, keep them, release at
# request end) with the LIFO policy this build fixes
# ---------------------------------------------------------------------------------
def test_allocator_hand_example(oracle):
    p = oracle.OraclePool(8, 16, 8)
    assert list(p.alloc(0, 3)) == [0, 1, 2]
    p.free(0, [1])
    assert list(p.alloc(0, 2)) == [1, 3]
    p.free(0, [0, 3])
    assert list(p.alloc(0, 1)) == [3]
    assert p.num_free() == 8 - 3 and p.num_used(0) == 3


def test_allocator_initial_order_and_errors(oracle):
    order = [3, 0, 2, 1]
    p = oracle.OraclePool(4, 16, 8, init_free_order=order)
    assert list(p.alloc(1, 2)) == [3, 0]
    rc, ids = p.alloc_status(1, 3)
    assert rc == oracle.ERR_NOMEM and ids is None and p.num_free() == 2
    assert p.free_status(1, [3, 3]) == oracle.ERR_INVALID      # named twice
    assert p.free_status(1, [2]) == oracle.ERR_INVALID         # not allocated
    assert p.free_status(0, [3]) == oracle.ERR_INVALID         # held by another model
    assert p.free_status(1, [7]) == oracle.ERR_INVALID         # out of range
    assert p.free_status(1, [0, 9]) == oracle.ERR_INVALID
    assert p.num_used(1) == 2 and p.num_free() == 2            # nothing changed
    p.free(1, [0, 3])
    assert list(p.alloc(2, 4)) == [3, 0, 2, 1]
    with pytest.raises(oracle.OracleError):
        oracle.OraclePool(4, 16, 8, init_free_order=[0, 1, 1, 2])


def test_allocator_invariants_under_churn(oracle):
    n_blocks = 5000
    p = oracle.OraclePool(n_blocks, 16, 8)
    live = {}
    state = {"nomem": 0}

    def check():
        used = sum(p.num_used(m) for m in range(4))
        assert used + p.num_free() == n_blocks
        assert used == len(live)

    def alloc(m, n):
        before = p.num_free()
        rc, ids = p.alloc_status(m, n)
        if rc != oracle.OK:
            assert rc == oracle.ERR_NOMEM and n > before and p.num_free() == before
            state["nomem"] += 1
            return None
        for i in ids:
            assert 0 <= i < n_blocks and int(i) not in live
            live[int(i)] = m
        check()
        return ids

    def free(m, ids):
        p.free(m, ids)
        for i in ids:
            assert live.pop(int(i)) == m
        assert p.free_status(m, ids[:1]) == oracle.ERR_INVALID   # double free
        check()

    rng = np.random.Generator(np.random.PCG64(99))
    wl.run_churn(rng, 2000, 400, alloc, free)
    assert state["nomem"] > 0 and p.num_free() == n_blocks and not live


# ---------------------------------------------------------------------------------
# append scatter
# ---------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_append_reads_back_exact_bits(oracle, dtype):
    lens, n_kv, d, B = [3, 20], 3, 8, 8
    pool, tables, lens, q, k, v, tok_seq, tok_pos = make_case(oracle, 43, 2, 3, n_kv, d, B, lens, dtype)
    for t in range(len(tok_seq)):
        s, pos = tok_seq[t], tok_pos[t]
        for h in range(n_kv):
            bid = tables[s, h, pos // B]
            assert np.array_equal(pool.read_row(bid, pos % B, 0), k[t, h])
            assert np.array_equal(pool.read_row(bid, pos % B, 1), v[t, h])
    # every (sequence, head, block) owns a distinct id
    ids = tables[tables >= 0]
    assert len(set(ids.tolist())) == ids.size
    # bad calls change nothing and say so
    bad = tables.copy()
    bad[1, 0, 0] = pool.num_blocks
    with pytest.raises(oracle.OracleError):
        pool.kv_append(k, v, tok_seq, tok_pos, bad)
    with pytest.raises(oracle.OracleError):
        pool.kv_append(k, v, tok_seq, tok_pos + 1000, tables)


def test_gather_is_logical_order(oracle):
    lens, n_kv, d, B = [37], 2, 8, 4
    pool, tables, lens, q, k, v, *_ = make_case(oracle, 47, 1, 2, n_kv, d, B, lens, "fp32")
    for h in range(n_kv):
        K, V = pool.gather(tables[0, h], 37)
        assert np.array_equal(K, k[:, h]) and np.array_equal(V, v[:, h])


def test_bf16_widening_matches_torch(oracle):
    t = wl.randn_values(5, (64, 1, 8), "bf16")
    bits = wl.as_bits(t)
    pool = oracle.OraclePool(8, 64, 8)
    table = np.arange(1, dtype=np.int32).reshape(1, 1, 1)
    pool.alloc(0, 1)
    pool.kv_append(bits, bits, np.zeros(64, np.int32), np.arange(64, dtype=np.int32), table)
    K, _ = pool.gather(table[0, 0], 64)
    assert np.array_equal(K, t.float().numpy()[:, 0])


# ---------------------------------------------------------------------------------
# streaming mode: dropping tiles, and checking a batch a slice of sequences at a time
# ---------------------------------------------------------------------------------
def test_drop_tiles_forgets_exactly_the_listed_blocks(oracle):
    pool, tables, lens, q, k, v, tok_seq, tok_pos = make_case(oracle, 31, 3, 2, 2, 16, 4, [9, 4, 6])
    before = pool.decode_attn(q, tables, lens, 2, 0.3)
    ids_seq0 = tables[0, :, :3].ravel()
    keep = {int(b): (pool.read_row(int(b), 0, 0).copy(), pool.read_row(int(b), 0, 1).copy())
            for b in np.concatenate([tables[1, :, :1].ravel(), tables[2, :, :2].ravel()])}
    n_free = pool.num_free()
    pool.drop_tiles(ids_seq0)
    for b in ids_seq0:                                   # the listed tiles are gone ...
        with pytest.raises(oracle.OracleError) as e:
            pool.read_row(int(b), 0, 0)
        assert e.value.status == oracle.ERR_INVALID
    with pytest.raises(oracle.OracleError):
        pool.gather(tables[0, 0], 9)
    for b, (kr, vr) in keep.items():                     # ... every other tile is untouched
        assert np.array_equal(pool.read_row(b, 0, 0), kr) and np.array_equal(pool.read_row(b, 0, 1), vr)
    assert pool.num_free() == n_free                     # dropping data is not freeing blocks
    assert np.array_equal(pool.decode_attn(q[1:], tables[1:], lens[1:], 2, 0.3), before[1:])
    with pytest.raises(oracle.OracleError) as e:         # bad id: INVALID
        pool.drop_tiles(np.array([pool.num_blocks], np.int32))
    assert e.value.status == oracle.ERR_INVALID
    pool.drop_tiles(ids_seq0)                            # dropping twice is harmless
    # appending the same rows again restores the outputs bit for bit
    sel = tok_seq == 0
    pool.kv_append(k[sel], v[sel], tok_seq[sel], tok_pos[sel], tables)
    assert np.array_equal(pool.decode_attn(q, tables, lens, 2, 0.3), before)


def test_sliced_check_equals_the_whole_batch_and_catches_a_planted_error(oracle):
    """The full-size GPU tests feed the oracle a slice of sequences at a time; on a batch small
    enough to hold at once, the sliced walk must reproduce the all-at-once oracle bit for bit,
    leave no tile behind, and name the sequence of a planted wrong output."""
    import types

    import mux_harness as H

    B, d, n_kv, n_q = 4, 16, 2, 4
    lens = np.array([13, 1, 8, 0, 21, 5, 16], np.int32)
    whole, tables, _, q, k, v, tok_seq, tok_pos = make_case(oracle, 47, lens.size, n_q, n_kv, d, B, lens, scramble=False)
    want = whole.decode_attn(q, tables, lens, n_q, 0.25)
    # the same appends as two recorded calls (history, then each sequence's last token), as CPU tensors
    last = np.zeros(tok_seq.size, bool)
    last[np.cumsum(lens[lens > 0]) - 1] = True
    as_t = lambda a: torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16)
    recs = [H.AppendRecord(tok_seq[~last], tok_pos[~last], as_t(k[~last]), as_t(v[~last])),
            H.AppendRecord(tok_seq[last], tok_pos[last], as_t(k[last]), as_t(v[last]))]
    streamed = oracle.OraclePool(whole.num_blocks, B, d, oracle.BF16, None)
    assert np.array_equal(streamed.alloc(0, int(tables.max()) + 1), np.arange(int(tables.max()) + 1))
    ls = types.SimpleNamespace(orc=streamed, block_size=B, head_dim=d, elem=2, dtype="bf16")
    job = H.JobState(0, wl.ModelShape("t", n_q, n_kv, d), lens, tables, None, np.zeros(lens.size, bool))
    per_seq_bytes = 2 * n_kv * d * 2
    slices = list(H.seq_slices(lens, per_seq_bytes, 20 * per_seq_bytes))
    assert len(slices) >= 4 and slices[0][0] == 0 and slices[-1][1] == lens.size
    assert all(a[1] == b[0] for a, b in zip(slices, slices[1:]))
    errs = H.decode_check_streaming(ls, job, recs, as_t(q), torch.from_numpy(want), 0.25, slice_bytes=20 * per_seq_bytes)
    assert errs.shape == (lens.size,) and not errs.any()          # bit-identical to the all-at-once oracle
    for b in range(int(tables.max()) + 1):                         # nothing is left in the streamed pool
        with pytest.raises(oracle.OracleError):
            streamed.read_row(b, 0, 0)
    wrong = want.copy()
    wrong[4, 1, 3] += 0.05
    with pytest.raises(AssertionError, match="sequence 4"):
        H.decode_check_streaming(ls, job, recs, as_t(q), torch.from_numpy(wrong), 0.25, slice_bytes=20 * per_seq_bytes)
