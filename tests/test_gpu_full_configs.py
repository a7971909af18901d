"""The five configurations at FULL size on the GPU, EVERY output compared with the oracle.

The oracle cannot hold tens of gigabytes of K/V at once, so it is fed a slice of sequences at
a time: the inputs of every append call are kept (on the device; configuration 5 re-uses
slices of a 1 GiB bank of N(0,1) values, since 70 GB of fresh normals would take minutes),
and after the GPU step each slice's K/V goes into the oracle's own pool - at the ids of the
oracle's own block manager - is attended to, compared element by element, and dropped again.
Block ids are compared for EVERY allocator call (both block managers run in lockstep), so
tables are bit-exact at full size.
"""
import time

import numpy as np
import pytest
import torch

import mux_harness as H
from paper_2404_02015_amd import binding as mx
from paper_2404_02015_amd import workloads as wl

pytestmark = pytest.mark.gpu

SLICE = 256 << 20      # K/V bytes the oracle holds at a time


def _say(msg):
    print("[case] " + msg, flush=True)


def _progress_to(capsys):
    """Progress lines that reach the terminal while the test runs (a long check must not look hung)."""
    def say(msg):
        with capsys.disabled():
            print("\n[progress] " + msg, flush=True)
    return say


def _nobody_sampled(n):
    return np.zeros(n, dtype=bool)


def _fill_in_slices(ls, st, target, seed, records, bytes_per_call=SLICE, bank=None):
    """Append history up to `target` tokens per sequence, a slice of sequences at a time so the
    dense K/V staging tensors stay around `bytes_per_call`; the inputs are kept in `records`."""
    per_tok = 2 * st.shape.n_kv_heads * ls.head_dim * 2
    for call, (s0, s1) in enumerate(H.seq_slices(target, per_tok, bytes_per_call)):
        nl = st.lens.copy()
        nl[s0:s1] = target[s0:s1]
        H.extend(ls, st, nl, seed=seed + call, on_device_values=True, bank=bank, record=records)


def _decode_step_all_models(ls, w, jobs, states, records, seed, progress=None):
    streams = [torch.cuda.Stream() for _ in states]
    torch.cuda.synchronize()
    outs = []
    scale = H.default_scale(w.head_dim)
    for j, st, stream in zip(jobs, states, streams):
        with torch.cuda.stream(stream):
            H.extend(ls, st, j.lens, seed=seed + 50 + j.model_id, stream=stream, record=records[j.model_id])   # alloc -> append one token
            q = H.make_q(ls, st, seed + 70 + j.model_id)
            outs.append((q, H.decode_gpu(ls, st, q, scale, stream=stream)))            # -> attend
    torch.cuda.synchronize()
    for st, (q, got) in zip(states, outs):
        t0 = time.time()
        errs = H.decode_check_streaming(ls, st, records[st.model_id], q, got, scale, SLICE, progress)
        msg = ("model %d %s: all %d sequences (%d tokens) checked by the oracle in %.1f s, max abs err %.2e (median %.2e)"
               % (st.model_id, st.shape.name, st.n_seqs, int(st.lens.sum()), time.time() - t0, errs.max(), np.median(errs)))
        print(msg, flush=True)
        if progress is not None:
            progress(msg)
    ls.check_counters()


@pytest.mark.parametrize("idx", [2, 3])
def test_full_decode_configs_every_sequence(idx, capsys):
    w = wl.config(idx)
    _say("full config %d: %s, pool %d blocks" % (idx, [(j.shape.name, j.n_seqs) for j in w.jobs], w.num_blocks))
    rng = w.rng()
    ls = H.Lockstep(w.num_blocks, w.block_size, w.head_dim, "bf16", wl.placement_order(rng, w.num_blocks))
    states, records = [], {}
    for j in w.jobs:
        st = H.open_job(ls, j.model_id, j.shape, j.n_seqs, int(j.lens.max()) + 16, sampled=_nobody_sampled(j.n_seqs))
        records[j.model_id] = []
        _fill_in_slices(ls, st, j.lens - 1, w.seed * 100 + 1000 * j.model_id, records[j.model_id])
        states.append(st)
    _decode_step_all_models(ls, w, w.jobs, states, records, w.seed * 100, _progress_to(capsys))


def test_full_config4_prefill_and_decode_every_output():
    """Configuration 4: the 13B-shaped model prefills its 8 prompts in chunks of 512 on one stream
    while the 7B- and 65B-GQA-shaped models decode 128 sequences each on two more.  Every prompt
    row (chunked on the GPU, unchunked in the oracle) and every decode sequence is compared."""
    w = wl.config(4)
    _say("full config 4: %s, pool %d blocks" % ([(j.kind, j.shape.name, j.n_seqs) for j in w.jobs], w.num_blocks))
    rng = w.rng()
    ls = H.Lockstep(w.num_blocks, w.block_size, w.head_dim, "bf16", wl.placement_order(rng, w.num_blocks))
    pj, dj = w.jobs[0], w.jobs[1:]
    scale = H.default_scale(w.head_dim)
    dstates, records = [], {}
    for j in dj:
        st = H.open_job(ls, j.model_id, j.shape, j.n_seqs, int(j.lens.max()) + 16, sampled=_nobody_sampled(j.n_seqs))
        records[j.model_id] = []
        _fill_in_slices(ls, st, j.lens - 1, w.seed * 100 + 1000 * j.model_id, records[j.model_id])
        dstates.append(st)
    pst = H.open_job(ls, pj.model_id, pj.shape, pj.n_seqs, int(pj.lens.max()) + 16, sampled=_nobody_sampled(pj.n_seqs))
    precords = []
    g = torch.Generator(device="cuda")
    g.manual_seed(w.seed)
    q_all = torch.randn(int(pj.lens.sum()), pj.shape.n_q_heads, w.head_dim, generator=g, device="cuda").to(torch.bfloat16)
    cu_all = np.concatenate([[0], np.cumsum(pj.lens)])
    got = torch.zeros_like(q_all)
    pstream = torch.cuda.Stream()
    done = np.zeros(pj.n_seqs, dtype=np.int32)
    torch.cuda.synchronize()
    # the decode models run their step on their own streams while the prefill chunks run on a third
    streams = [torch.cuda.Stream() for _ in dstates]
    outs = []
    for j, st, stream in zip(dj, dstates, streams):
        with torch.cuda.stream(stream):
            H.extend(ls, st, j.lens, seed=w.seed * 100 + 50 + j.model_id, stream=stream, record=records[j.model_id])
            q = H.make_q(ls, st, w.seed * 100 + 70 + j.model_id)
            outs.append((q, H.decode_gpu(ls, st, q, scale, stream=stream)))
    step = 0
    with torch.cuda.stream(pstream):
        while (done < pj.lens).any():
            q_lens = np.minimum(pj.chunk, pj.lens - done).astype(np.int32)
            H.extend(ls, pst, done + q_lens, seed=w.seed * 100 + 200 + step, on_device_values=True, stream=pstream,
                     record=precords)
            rows = np.concatenate([np.arange(cu_all[s] + done[s], cu_all[s] + done[s] + q_lens[s]) for s in range(pj.n_seqs)])
            rows_dev = torch.from_numpy(rows).cuda()
            part = H.prefill_gpu(ls, pst, q_all.index_select(0, rows_dev).contiguous(), q_lens, done, scale, stream=pstream)
            got.index_copy_(0, rows_dev, part)
            done = done + q_lens
            step += 1
        # the same prompts once more in one unchunked launch (their K/V are all cached by now)
        whole = H.prefill_gpu(ls, pst, q_all, pj.lens, np.zeros(pj.n_seqs, np.int32), scale, stream=pstream)
    torch.cuda.synchronize()
    assert step <= 4 and torch.isfinite(got.float()).all() and torch.isfinite(whole.float()).all()
    # oracle: every prompt, all its rows, unchunked; one prompt's K/V in the oracle's pool at a time
    for s in range(pj.n_seqs):
        H.feed_oracle_slice(ls, pst, precords, s, s + 1)
        lo, hi = int(cu_all[s]), int(cu_all[s + 1])
        want = ls.orc.prefill_attn(H.to_oracle(q_all[lo:hi]), np.array([0, hi - lo], np.int32), np.zeros(1, np.int32),
                                   pst.tables[s:s + 1], pj.shape.n_q_heads, scale)
        H.drop_oracle_slice(ls, pst, s, s + 1)
        err = H.assert_close(got[lo:hi], want, "bf16", "prompt %d, chunked" % s)
        err_whole = H.assert_close(whole[lo:hi], want, "bf16", "prompt %d, unchunked" % s)
        print("prefill prompt %d (%d tokens): max abs err %.2e in chunks of %d, %.2e in one launch"
              % (s, hi - lo, err, pj.chunk, err_whole), flush=True)
    for st, (q, o) in zip(dstates, outs):
        errs = H.decode_check_streaming(ls, st, records[st.model_id], q, o, scale, SLICE)
        print("decode %s: all %d sequences checked by the oracle, max abs err %.2e" % (st.shape.name, st.n_seqs, errs.max()),
              flush=True)
    ls.check_counters()


@pytest.mark.timeout(900)
def test_full_config5_pool_stress(capsys):
    """Pool of ~80 % of free HBM, fragmented by a seeded 10 000-op alloc/free churn, 512 sequences
    over 4 models with contexts in [1024, 16384] (about 70 GB of K/V); offsets are 64-bit.  All 512
    sequences are compared with the oracle (its host pool holds one slice of them at a time)."""
    w = wl.config(5)
    free_bytes, _ = torch.cuda.mem_get_info()
    block_bytes = 2 * w.block_size * w.head_dim * 2
    num_blocks = int(w.hbm_fraction * free_bytes) // block_bytes
    demand = w.demand_blocks()
    _say("full config 5: free %.1f GB -> pool of %d blocks (%.1f GB), demand %d blocks (%.1f GB)"
         % (free_bytes / 1e9, num_blocks, num_blocks * block_bytes / 1e9, demand, demand * block_bytes / 1e9))
    assert num_blocks > demand and num_blocks * block_bytes > (1 << 32)
    rng = w.rng()
    t0 = time.time()
    ls = H.Lockstep(num_blocks, w.block_size, w.head_dim, "bf16", None)
    n_ops = wl.run_churn(rng, w.churn_ops, 4096, ls.alloc_or_none, ls.free, n_models=len(w.jobs))
    ls.check_counters()
    print("churn: %d ops took effect, %.1f s" % (n_ops, time.time() - t0), flush=True)
    g = torch.Generator(device="cuda")
    g.manual_seed(w.seed)
    bank = {"k": torch.randn(1 << 28, generator=g, device="cuda").to(torch.bfloat16),
            "v": torch.randn(1 << 28, generator=g, device="cuda").to(torch.bfloat16)}
    states, records = [], {}
    for j in w.jobs:
        st = H.open_job(ls, j.model_id, j.shape, j.n_seqs, int(j.lens.max()) + 16, sampled=_nobody_sampled(j.n_seqs))
        records[j.model_id] = []
        _fill_in_slices(ls, st, j.lens - 1, w.seed * 100 + 1000 * j.model_id, records[j.model_id], bank=bank)
        states.append(st)
        _progress_to(capsys)("filled model %d (%s): %d sequences, %.1f s" % (j.model_id, j.shape.name, j.n_seqs, time.time() - t0))
    # fragmentation really happened: the ids of one head's consecutive blocks are not consecutive
    t = states[0].tables[0, 0, :64].astype(np.int64)
    assert (np.abs(np.diff(t)) != 1).mean() > 0.5
    top_id = max(int(st.tables[st.tables < num_blocks].max()) for st in states)
    assert top_id * block_bytes > (1 << 32)                                          # offsets beyond 4 GiB are in use
    _decode_step_all_models(ls, w, w.jobs, states, records, w.seed * 100, _progress_to(capsys))
    print("total %.1f s" % (time.time() - t0), flush=True)
