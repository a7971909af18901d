#!/usr/bin/env python3
"""Benchmark of the head-wise paged KV-cache hot path on one MI355X.

Workload (N=1): the second configuration - two colocated LLaMA-7B-shaped models (32 heads x
128, bf16) sharing one pool of 16-token head-blocks in seeded random placement, 64 decoding
sequences per model with contexts uniform in [128, 2048].  One *step* is one decoding step of
one layer for every model, each model on its own HIP stream:

    mux_alloc_blocks (for sequences whose new token opens a block) -> table patch ->
    mux_kv_append (one token per sequence) -> mux_decode_attn (all cached tokens)

Everything is resident in HBM before the timed region.  `value` is the K/V bytes the decode
attention has to read (valid tokens only) per second of wall time over the whole step loop.
The `roofline` object prices the dominant kernel (decode attention) against the 8 TB/s HBM
peak from HIP-event durations of its launches inside the timed loop; `cpu_baseline` times the
CPU oracle on a bounded sample of the same sequences on this machine's host cores.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import math
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2404_02015_amd import binding as mx  # noqa: E402
from paper_2404_02015_amd import workloads as wl  # noqa: E402

HBM_PEAK_GBS = 8000.0
# HBM bytes per decode_attn launch on configuration 2, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# (each scaled by a plain 1 GiB copy in the same run): 567 486 KiB x 2.000 fetched + 512 KiB written.
MEASURED_TRAFFIC_CFG2 = {"bytes": 567567.7 * 1024 * 2.0 + 512.0 * 1024, "source": "profiles/decode_attn_config2_pmc.md",
                         "note": "stored figure from the profile named in traffic_source (two rocprofv3 --pmc runs of this "
                                 "script, 7 steps each), not counters of this run"}


class DecodeModel:
    """Device state of one colocated model: tables, lengths, per-step inputs, its stream."""

    def __init__(self, pool, job: wl.ModelJob, block_size: int, total_steps: int, seed: int, device: str, bank=None):
        self.pool, self.job, self.B = pool, job, block_size
        self.shape = job.shape
        self.n = job.n_seqs
        n_kv, n_q, d = self.shape.n_kv_heads, self.shape.n_q_heads, self.shape.head_dim
        self.lens = (job.lens.astype(np.int64) - 1).astype(np.int32)   # cached before the first step
        self.max_blocks = wl.max_blocks_for(job.lens, block_size, extra_tokens=total_steps + 1)
        self.stream = torch.cuda.Stream()
        self.device = device
        g = torch.Generator(device=device)
        g.manual_seed(seed)
        # block tables for the history, ids from the library's block manager
        self.tables = wl.build_tables(lambda m, k: mx.mux_alloc_blocks(pool, m, k), job.model_id, self.lens, n_kv,
                                      block_size, self.max_blocks)
        self.tables_dev = torch.from_numpy(self.tables).to(device)
        # history K/V ~ N(0,1), drawn on the device sequence by sequence and appended
        per_call = 8 if bank is None else 2
        for s0 in range(0, self.n, per_call):
            s1 = min(self.n, s0 + per_call)
            cnt = self.lens[s0:s1].astype(np.int64)
            nt = int(cnt.sum())
            if nt == 0:
                continue
            if bank is None:
                k = torch.randn(nt, n_kv, d, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
                v = torch.randn(nt, n_kv, d, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
            else:  # slices of a pre-drawn bank of N(0,1) values (tens of GB of fresh normals would take minutes)
                need = nt * n_kv * d
                off = ((seed + s0) * 7919) % (bank[0].numel() - need)
                off -= off % 8
                k, v = bank[0][off:off + need].view(nt, n_kv, d), bank[1][off:off + need].view(nt, n_kv, d)
            seq = np.repeat(np.arange(s0, s1, dtype=np.int32), cnt)
            pos = (np.arange(nt, dtype=np.int64) - np.repeat(np.cumsum(cnt) - cnt, cnt)).astype(np.int32)
            mx.mux_kv_append(pool, k, v, torch.from_numpy(seq).to(device), torch.from_numpy(pos).to(device),
                             self.tables_dev)
        torch.cuda.synchronize()
        # per-step inputs: one new K/V row and one query row per sequence
        self.k_steps = torch.randn(total_steps, self.n, n_kv, d, generator=g, device=device).to(torch.bfloat16)
        self.v_steps = torch.randn(total_steps, self.n, n_kv, d, generator=g, device=device).to(torch.bfloat16)
        self.q_steps = torch.randn(total_steps, self.n, n_q, d, generator=g, device=device).to(torch.bfloat16)
        self.out = torch.empty(self.n, n_q, d, device=device, dtype=torch.bfloat16)
        self.tok_seq = torch.arange(self.n, dtype=torch.int32, device=device)
        # row 0: position of the token appended this step, row 1: context length after the append
        # per step: positions of the appended tokens and context lengths after the append (known
        # in advance: every sequence grows by one token per step), so no kernel has to bump them
        steps = np.arange(1, total_steps + 1, dtype=np.int32)[:, None]
        self.pos_steps = torch.from_numpy(self.lens[None, :] + steps - 1).to(device)
        self.len_steps = torch.from_numpy(self.lens[None, :] + steps).to(device)
        self.pos_len = torch.stack([self.pos_steps[0] - 1, self.len_steps[0] - 1]).contiguous()   # state before step 0
        max_final = int(job.lens.max()) + total_steps + 1
        ws = mx.mux_decode_workspace_bound(pool, self.n, n_q, n_kv, max_final)   # the hint grows step by step: cover every plan
        self.workspace = torch.empty(max(ws, 16), dtype=torch.uint8, device=device)
        # pinned staging ring for table patches: flat table indices and the ids, which
        # mux_alloc_blocks writes there itself
        cap = self.n * n_kv
        self.pin_idx = torch.empty(total_steps, cap, dtype=torch.int64, pin_memory=True)
        self.pin_ids = torch.empty(total_steps, cap, dtype=torch.int32, pin_memory=True)
        self.pin_idx_np, self.pin_ids_np = self.pin_idx.numpy(), self.pin_ids.numpy()
        self.flat_tables = self.tables_dev.view(-1)
        self.head_base = (np.arange(n_kv, dtype=np.int64) * self.max_blocks)
        self.scale = 1.0 / math.sqrt(d)
        self.step_no = 0
        self.fused = False
        self.kv_bytes_per_token = 2 * n_kv * d * 2
        self.decode_events = []

    def step(self, record: bool, after=None):
        """Enqueue one decoding step on this model's stream.  `after`: an event the decode
        attention (not the small kernels before it) waits for.  Returns the K/V bytes the
        decode attention has to read and the event that marks its end."""
        i = self.step_no
        self.step_no += 1
        n_kv = self.shape.n_kv_heads
        new_lens = self.lens + 1
        crossing = np.nonzero((new_lens - 1) % self.B == 0)[0]
        with torch.cuda.stream(self.stream):
            if crossing.size:
                # new blocks: ids from the block manager (written straight into pinned memory), then
                # two small host-to-device copies and a scatter into the device table
                cnt = 0
                for s in crossing:
                    mx.mux_alloc_blocks(self.pool, self.job.model_id, n_kv, self.pin_ids_np[i, cnt:cnt + n_kv])
                    col = int(new_lens[s] - 1) // self.B
                    self.pin_idx_np[i, cnt:cnt + n_kv] = (int(s) * n_kv * self.max_blocks + col) + self.head_base
                    cnt += n_kv
                idx_dev = self.pin_idx[i, :cnt].to(self.device, non_blocking=True)
                ids_dev = self.pin_ids[i, :cnt].to(self.device, non_blocking=True)
                self.flat_tables.index_copy_(0, idx_dev, ids_dev)
            if not self.fused:
                mx.mux_kv_append(self.pool, self.k_steps[i], self.v_steps[i], self.tok_seq, self.pos_steps[i], self.tables_dev,
                                 stream=self.stream)
            max_ctx = int(new_lens.max())
            if after is not None:
                self.stream.wait_event(after)
            e0, e1 = torch.cuda.Event(enable_timing=record), torch.cuda.Event(enable_timing=record)
            if record:
                e0.record(self.stream)
            if self.fused:   # append and attention in one launch
                mx.mux_decode_step(self.pool, self.out[None], self.q_steps[i][None], self.k_steps[i][None], self.v_steps[i][None],
                                   self.tables_dev[None], self.len_steps[i], max_ctx, self.scale, self.workspace, stream=self.stream)
            else:
                mx.mux_decode_attn(self.pool, self.out, self.q_steps[i], self.tables_dev, self.len_steps[i], max_ctx, self.scale,
                                   self.workspace, stream=self.stream)
            e1.record(self.stream)
            if record:
                self.decode_events.append((e0, e1, int(new_lens.astype(np.int64).sum()) * self.kv_bytes_per_token))
        self.lens = new_lens
        return int(new_lens.astype(np.int64).sum()) * self.kv_bytes_per_token, e1


class PrefillModel:
    """A model running chunked causal prefill on its own stream.  All prompts are processed chunk
    by chunk; benchmark step i runs chunk stage i mod n_stages (append the chunk's K/V, then
    attend), so the cycle of stages repeats over the step loop."""

    def __init__(self, pool, job: wl.ModelJob, block_size: int, seed: int, device: str):
        self.pool, self.job, self.B, self.shape = pool, job, block_size, job.shape
        n_kv, n_q, d = self.shape.n_kv_heads, self.shape.n_q_heads, self.shape.head_dim
        lens = job.lens.astype(np.int32)
        self.stream = torch.cuda.Stream()
        self.scale = 1.0 / math.sqrt(d)
        max_blocks = wl.max_blocks_for(lens, block_size)
        tables = wl.build_tables(lambda m, k: mx.mux_alloc_blocks(pool, m, k), job.model_id, lens, n_kv, block_size, max_blocks)
        self.tables_dev = torch.from_numpy(tables).to(device)
        g = torch.Generator(device=device)
        g.manual_seed(seed)
        self.stages = []
        done = np.zeros(lens.size, dtype=np.int32)
        while (done < lens).any():
            ql = np.minimum(job.chunk, lens - done).astype(np.int32)
            cu = np.concatenate([[0], np.cumsum(ql)]).astype(np.int32)
            nt = int(cu[-1])
            seq = np.repeat(np.arange(lens.size, dtype=np.int32), ql)
            pos = (np.repeat(done, ql) + np.arange(nt) - np.repeat(cu[:-1], ql)).astype(np.int32)
            flops = sum(n_q * 4 * d * (int(ql[i]) * int(done[i]) + int(ql[i]) * (int(ql[i]) + 1) // 2) for i in range(lens.size))
            st = {
                "k": torch.randn(nt, n_kv, d, generator=g, device=device).to(torch.bfloat16),
                "v": torch.randn(nt, n_kv, d, generator=g, device=device).to(torch.bfloat16),
                "q": torch.randn(nt, n_q, d, generator=g, device=device).to(torch.bfloat16),
                "seq": torch.from_numpy(seq).to(device), "pos": torch.from_numpy(pos).to(device),
                "cu": torch.from_numpy(cu).to(device), "start": torch.from_numpy(done.copy()).to(device),
                "max_q": int(ql.max()), "max_ctx": int((done + ql).max()), "flops": flops,
                "kv_bytes": int((done + ql)[ql > 0].astype(np.int64).sum()) * 2 * n_kv * d * 2,
                # everything the stage moves: K/V prefix reads, Q read + O written, the chunk's K/V rows read and written
                "all_bytes": int((done + ql)[ql > 0].astype(np.int64).sum()) * 2 * n_kv * d * 2 + 2 * nt * n_q * d * 2
                             + 2 * 2 * nt * n_kv * d * 2,
            }
            st["out"] = torch.empty_like(st["q"])
            self.stages.append(st)
            done = done + ql
        # the first pass over the stages fills the cache (later stages read earlier chunks)
        for st in self.stages:
            mx.mux_kv_append(pool, st["k"], st["v"], st["seq"], st["pos"], self.tables_dev)
        torch.cuda.synchronize()
        self.step_no = 0
        self.events = []
        self.bytes_moved = 0      # algorithmic bytes of the recorded stages, appends included

    def step(self, record: bool):
        st = self.stages[self.step_no % len(self.stages)]
        self.step_no += 1
        if record:
            self.bytes_moved += st["all_bytes"]
        with torch.cuda.stream(self.stream):
            mx.mux_kv_append(self.pool, st["k"], st["v"], st["seq"], st["pos"], self.tables_dev, stream=self.stream)
            e0, e1 = torch.cuda.Event(enable_timing=record), torch.cuda.Event(enable_timing=record)
            if record:
                e0.record(self.stream)
            mx.mux_prefill_attn(self.pool, st["out"], st["q"], st["cu"], st["start"], self.tables_dev, st["max_q"],
                                st["max_ctx"], self.scale, None, stream=self.stream)
            if record:
                e1.record(self.stream)
                self.events.append((e0, e1, st["flops"], st["kv_bytes"]))


def build_workload(cfg_index: int, total_steps: int, device: str = "cuda", prefill_override=None, with_decode: bool = True):
    """Pool, decode models and (configuration 4) the prefill model of one configuration.
    prefill_override = (prompts, tokens per prompt, chunk) replaces the prefill model's prompts."""
    w = wl.config(cfg_index)
    if prefill_override is not None:
        n, length, chunk = prefill_override
        for j in w.jobs:
            if j.kind == "prefill":
                j.lens = np.full(n, length, dtype=np.int32)
                j.chunk = chunk
        w.num_blocks = max(w.num_blocks, int(w.demand_blocks() * 1.25) // 8192 * 8192 + 8192)
    decode_jobs = [j for j in w.jobs if j.kind == "decode"] if with_decode else []
    prefill_jobs = [j for j in w.jobs if j.kind == "prefill"]
    if not with_decode:
        w.jobs = prefill_jobs
    growth = sum(j.n_seqs * j.shape.n_kv_heads * (total_steps // w.block_size + 2) for j in decode_jobs)
    block_bytes = 2 * w.block_size * w.head_dim * 2
    bank = None
    if w.num_blocks > 0:
        num_blocks = max(w.num_blocks, w.demand_blocks() + growth)
    else:  # a fraction of the free device memory, read at run time
        free_bytes, _ = torch.cuda.mem_get_info()
        num_blocks = int(w.hbm_fraction * free_bytes) // block_bytes
    kv = torch.empty(num_blocks * block_bytes, dtype=torch.uint8, device=device)
    rng = w.rng()
    if w.placement == "churn":
        pool = mx.mux_pool_create(kv, num_blocks, w.block_size, w.head_dim, mx.MUX_BF16, None)

        def try_alloc(m, n):
            rc, ids = mx.mux_alloc_blocks_status(pool, m, n)
            return ids if rc == mx.MUX_OK else None

        wl.run_churn(rng, w.churn_ops, 4096, try_alloc, lambda m, ids: mx.mux_free_blocks(pool, m, ids), n_models=len(w.jobs))
        g = torch.Generator(device=device)
        g.manual_seed(w.seed)
        bank = (torch.randn(1 << 28, generator=g, device=device).to(torch.bfloat16),
                torch.randn(1 << 28, generator=g, device=device).to(torch.bfloat16))
    else:
        pool = mx.mux_pool_create(kv, num_blocks, w.block_size, w.head_dim, mx.MUX_BF16, wl.placement_order(rng, num_blocks))
    models = [DecodeModel(pool, j, w.block_size, total_steps, w.seed * 1000 + j.model_id, device, bank) for j in decode_jobs]
    prefills = [PrefillModel(pool, j, w.block_size, w.seed * 1000 + j.model_id, device) for j in prefill_jobs]
    del bank
    return w, pool, models, prefills


def cpu_baseline(models, budget_s: float = 12.0, single_core: bool = True):
    """Time the CPU oracle (as it stands) on a bounded sample of the workload's sequences: from
    every decode model of the configuration, its longest sequences up to ~1/8 of its tokens and
    at most 192 MB of K/V (the oracle's pool holds the sample; the loop repeats passes over it
    until the time budget is spent)."""
    from oracle import mux_oracle as orc

    orc.build()
    rng = np.random.default_rng(1)
    samples, per_model = [], []
    for m in models:
        B, d, n_kv, n_q = m.B, m.shape.head_dim, m.shape.n_kv_heads, m.shape.n_q_heads
        order = np.argsort(-m.lens, kind="stable")
        target = min(int(m.lens.astype(np.int64).sum() // 8), (192 << 20) // m.kv_bytes_per_token)
        pick, tok = [], 0
        for s in order:
            if pick and tok + int(m.lens[s]) > target:
                break
            pick.append(int(s))
            tok += int(m.lens[s])
        lens = m.lens[np.array(sorted(pick))]
        nb = int(((lens + B - 1) // B).sum()) * n_kv
        pool = orc.OraclePool(nb + 8, B, d, orc.BF16)
        tables = wl.build_tables(lambda mid, k: pool.alloc(mid, k), 0, lens, n_kv, B, int((lens.max() + B - 1) // B))
        for i, L in enumerate(lens):  # values do not matter for the timing; N(0,1) in bf16
            k = (rng.standard_normal((int(L), n_kv, d), dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)
            v = (rng.standard_normal((int(L), n_kv, d), dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)
            pool.kv_append(k, v, np.full(int(L), i, np.int32), np.arange(int(L), dtype=np.int32), tables)
        q = (rng.standard_normal((len(lens), n_q, d), dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)
        samples.append((pool, q, tables, lens, n_q, m.scale, int(lens.astype(np.int64).sum()) * m.kv_bytes_per_token, m.shape.name))
    cores = orc.num_threads()

    def run(budget):
        """Passes over all models' samples until the budget is spent; returns bytes/s overall and per model."""
        spent = [0.0] * len(samples)
        reps = 0
        t0 = time.perf_counter()
        while True:
            for i, (pool, q, tables, lens, n_q, scale, _, _) in enumerate(samples):
                t1 = time.perf_counter()
                pool.decode_attn(q, tables, lens, n_q, scale)
                spent[i] += time.perf_counter() - t1
            reps += 1
            if time.perf_counter() - t0 > budget:
                break
        dt = time.perf_counter() - t0
        total = sum(smp[6] for smp in samples)
        return total * reps / dt / 1e9, [smp[6] * reps / max(t, 1e-9) / 1e9 for smp, t in zip(samples, spent)], reps, dt

    all_gbs, per_gbs, reps, dt = run(budget_s)
    out = {
        "value": all_gbs, "unit": "GB/s", "cores": cores, "kind": "oracle",
        "sample": "longest sequences of every decode model up to 1/8 of its tokens and 192 MB: %s; %d passes in %.1f s"
                  % ("; ".join("%s %d seqs, %d tokens, %.1f MB" % (smp[7], len(smp[3]), int(smp[3].sum()), smp[6] / 1e6) for smp in samples),
                     reps, dt),
        "per_model_GBps": [round(x, 2) for x in per_gbs],
    }
    if single_core:
        orc.set_num_threads(1)
        out["single_core_value"] = run(budget_s / 4)[0]
        orc.set_num_threads(cores)
    return out


def measure_ceilings(device: str = "cuda"):
    """What this GPU sustains with nothing in the way: a plain streaming read of 4 GiB and
    back-to-back bf16 matrix instructions (the library's probe kernels)."""
    buf = torch.empty(1 << 32, dtype=torch.uint8, device=device)
    buf.view(torch.int32).fill_(1)
    sink = torch.zeros(1, dtype=torch.float32, device=device)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n_cu = mx.mux_device_cu_count()
    mx.mux_probe_stream_read(buf, sink, 16 * n_cu)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(3):
        mx.mux_probe_stream_read(buf, sink, 16 * n_cu)
    e1.record()
    torch.cuda.synchronize()
    read_gbs = 3 * buf.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del buf
    n_wg = 4 * n_cu                              # four waves per SIMD: one alone cannot issue at full rate
    mx.mux_probe_mfma(sink, n_wg, 1000)
    torch.cuda.synchronize()
    e0.record()
    flops = mx.mux_probe_mfma(sink, n_wg, 10000)
    e1.record()
    torch.cuda.synchronize()
    return {"stream_read_GBps": read_gbs, "mfma_bf16_TFLOPps": flops / (e0.elapsed_time(e1) * 1e-3) / 1e12,
            "note": "measured on this GPU by the library's probe kernels: 4 GiB streaming read (16-byte non-temporal loads) "
                    "in whole 8 KiB chunks per wave and independent v_mfma_f32_16x16x32_bf16 with four waves per SIMD"}


def measure_append(device: str = "cuda"):
    """mux_kv_append alone (it is excluded from the decode figure): a prefill-shaped call large
    enough to miss the last-level cache (16 sequences x 2048 tokens, 32 KV heads: 0.54 GB read,
    0.54 GB written) and a decode-shaped one (64 sequences x 1 token: a launch-bound 2 MB)."""
    B, d, hkv, n_seqs, chunk = 16, 128, 32, 16, 2048
    per_seq = chunk // B
    n_blocks = n_seqs * hkv * per_seq + 64 * hkv
    kv = torch.empty(n_blocks * 2 * B * d * 2, dtype=torch.uint8, device=device)
    pool = mx.mux_pool_create(kv, n_blocks, B, d, mx.MUX_BF16, None)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    out = {}
    for name, seqs, toks, first in (("prefill_16x2048", n_seqs, chunk, 0), ("decode_64x1", 64, 1, n_seqs * hkv * per_seq)):
        nb = (toks + B - 1) // B
        tables = (first + torch.arange(seqs * hkv * nb, dtype=torch.int32, device=device)).view(seqs, hkv, nb).contiguous()
        n = seqs * toks
        k = torch.randn(n, hkv, d, device=device).to(torch.bfloat16)
        v = torch.randn(n, hkv, d, device=device).to(torch.bfloat16)
        tok_seq = torch.arange(seqs, dtype=torch.int32, device=device).repeat_interleave(toks).contiguous()
        tok_pos = torch.arange(toks, dtype=torch.int32, device=device).repeat(seqs).contiguous()
        reps = 20
        mx.mux_kv_append(pool, k, v, tok_seq, tok_pos, tables)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            mx.mux_kv_append(pool, k, v, tok_seq, tok_pos, tables)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / reps * 1e3
        moved = 2 * 2 * n * hkv * d * 2                       # K and V rows, read once and written once
        out[name] = {"us": us, "GBps_read_plus_write": moved / (us * 1e-6) / 1e9, "bytes": moved}
    out["note"] = ("back-to-back launches on one stream, HIP events; bytes = new K/V rows read + the same written; the "
                   "decode-shaped call is bound by the launch rate of the Python binding, not by the kernel (~5 us)")
    mx.mux_pool_destroy(pool)
    return out


def allocator_ns_per_block():
    """Host cost of the block manager (the one cost the paper flags on this path, Section 3.4,
    Implementation): nanoseconds per block id, for decode-sized and prefill-sized calls."""
    n_blocks = 1 << 20
    kv = torch.empty(64, dtype=torch.uint8)
    h = ctypes.c_void_p()
    lib = mx.load()
    rc = lib.mux_pool_create(ctypes.byref(h), kv.data_ptr(), n_blocks * 8192, n_blocks, 16, 128, mx.MUX_BF16, None)
    assert rc == 0
    out = {}
    for name, n in (("alloc32_free32", 32), ("alloc1280_free1280", 1280)):
        ids = np.zeros(n, dtype=np.int32)
        reps = 20000 if n == 32 else 2000
        t0 = time.perf_counter()
        for _ in range(reps):
            lib.mux_alloc_blocks(h, 0, n, ids.ctypes.data)
            lib.mux_free_blocks(h, 0, n, ids.ctypes.data)
        out[name] = (time.perf_counter() - t0) / (2 * reps * n) * 1e9
    lib.mux_pool_destroy(h)
    out["note"] = "ns per block id, one alloc + one free call through ctypes (call overhead included)"
    return out


def run_adbs(args) -> int:
    """Second workload: the batch scheduler (Algorithm 3) serving a Poisson stream of requests for
    three colocated models, rates 2:8:8 and request lengths 2:1:1 as in the paper's cache-usage
    ablation (Section 4.4), on a pool that cannot hold everybody's demand.  Every job is launched
    on the GPU.  Run twice: with quotas in proportion to rate x blocks per token (adapted
    periodically) and without quotas; reports output tokens/s and how the block usage is shared."""
    from paper_2404_02015_amd import adbs_engine as eng

    shapes = [wl.LLAMA_13B, wl.LLAMA_7B, wl.LLAMA_7B]
    rates = np.array([2.0, 8.0, 8.0])
    length_scale = [2, 1, 1]
    S = max(int(args.adbs_scale), 1)                   # pool, slots, arrivals and prefill budget grow together
    layers = [40, 32, 32] if args.adbs_layers else [1, 1, 1]   # LLaMA-13B / 7B depths: the whole model's K/V
    if args.adbs_layers and args.adbs_driver == "python":
        raise SystemExit("--adbs-layers needs the runner (the Python driver handles one layer)")
    B, d, n_blocks, max_seqs, max_blocks = 16, 128, 40000 * S * (32 if args.adbs_layers else 1), min(64 * S, 1024), 96
    budget = 2048 * S
    iters = max(args.steps, 1) * 8
    warm = max(args.warmup, 1) * 8 * (2 if S > 1 else 1)
    per_iter = S * rates / rates.sum()                 # requests per iteration and model
    out = {}
    for mode in ("adbs", "no-quota"):
        kv = torch.empty(n_blocks * 2 * B * d * 2, dtype=torch.uint8, device="cuda")
        rng = np.random.Generator(np.random.PCG64(20240402))
        pool = mx.mux_pool_create(kv, n_blocks, B, d, mx.MUX_BF16, wl.placement_order(rng, n_blocks))
        kw = {}
        if mode == "adbs":
            weights = rates * np.array([s.n_kv_heads * n for s, n in zip(shapes, layers)])
            assert mx.mux_pool_init_quotas(pool, weights) == 0
            kw = dict(adapt_period=16, low=0.5, high=0.9, step=0.25)
        if args.adbs_driver == "python":
            engine = eng.Engine(pool, shapes, max_seqs, max_blocks, budget, eng.DeviceRandomSource(shapes, d, seed=1),
                                keep_outputs=False, **kw)
        else:
            engine = eng.NativeEngine(pool, shapes, max_seqs, max_blocks, budget, None,
                                      shared_stream=args.adbs_driver == "runner-one-stream", layers=layers, **kw)
        use = np.zeros(len(shapes))
        rid, t0, tok0, host_s = 0, None, 0, 0.0
        for it in range(warm + iters):
            if it == warm:
                torch.cuda.synchronize()
                t0, tok0 = time.perf_counter(), engine.tokens()
            for m in range(len(shapes)):
                for _ in range(int(rng.poisson(per_iter[m]))):
                    engine.submit(m, rid, int(rng.integers(64, 385)) * length_scale[m], int(rng.integers(32, 129)) * length_scale[m])
                    rid += 1
            h0 = time.perf_counter()
            engine.step()
            if it >= warm:
                host_s += time.perf_counter() - h0
                use += [mx.mux_pool_num_used(pool, m) for m in range(len(shapes))]
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        counts = [engine.sched.counts(m) for m in range(len(shapes))]
        out[mode] = {
            "tokens_per_s": (engine.tokens() - tok0) / dt,
            "ms_per_iteration": dt / iters * 1e3,
            "host_ms_per_iteration": host_s / iters * 1e3,     # scheduler pass + enqueueing its jobs, without waiting for the GPU
            "block_usage_share": [round(float(x), 4) for x in use / max(use.sum(), 1)],
            "mean_blocks_in_use": float(use.sum() / iters),
            "kv_GBps_decode_reads": float(use.sum() / iters) * 2 * B * d * 2 / (dt / iters) / 1e9,
            "finished": [c[2] for c in counts], "preemptions": [c[3] for c in counts], "waiting_at_end": [c[0] for c in counts],
            "quota_blocks_moved": counts[0][4],
        }
        del engine, pool, kv
        torch.cuda.empty_cache()
    a = out["adbs"]
    line = {
        "metric": "ADBS-scheduled serving: output tokens/s, attention path only", "value": a["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": iters, "warmup": warm, "ms_per_step": a["ms_per_iteration"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "storage_dtype": "bf16", "data": "synthetic",
        "config": {"workload": "batch scheduler (Algorithm 3) over 13B/7B/7B-shaped models, Poisson arrivals 2:8:8, request "
                               "lengths 2:1:1, %d requests per pass, %d head-blocks, %d slots per model, prefill budget %d tokens; every job "
                               "launched on the GPU, driver: %s; layers per model: %s" % (S, n_blocks, max_seqs, budget, args.adbs_driver, layers)},
        "rate_share": [round(float(x), 4) for x in rates / rates.sum()],
        "adbs": a, "no_quota": out["no-quota"],
    }
    print(json.dumps(line))
    return 0


def run_estimate(args) -> int:
    """The throughput estimator (Section 3.3, Eq. 3; Appendix A.2) fed by latencies measured on this
    GPU.  For the shapes of configuration 4 - a 13B-shaped LLM prefilling next to 7B- and
    65B-GQA-shaped LLMs that decode - the attention path of ONE layer is timed at four batch
    sizes per phase (prefill: prompts of 1 280 tokens, the mean of U[512, 2048]; decoding: contexts
    U[256, 4096]) and fitted as lines in the batch size, t_p(b) = p0 + p1 b and t_d(b) = d0 + d1 b.
    With a generation length of 338 tokens (the paper's ShareGPT mean) mux_find_batch_size then gives,
    per decoding LLM, the batch that meets a request rate; the rates tried are fractions of the rate
    the LLM can sustain at all, 1 / (d1 l_o) requests/s.  Beside each prediction: the measured
    throughput at that batch size (its own t_d measured, not the fit)."""
    dev, B, d = "cuda", 16, 128
    gen_len = 338.0
    rng = np.random.default_rng(4)

    def make_pool(n_blocks):
        kv = torch.empty(n_blocks * 2 * B * d * 2, dtype=torch.uint8, device=dev)
        return kv, mx.mux_pool_create(kv, n_blocks, B, d, mx.MUX_BF16, wl.placement_order(rng, n_blocks))

    def time_it(fn, reps=20):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e-3

    def decode_latency(shape, b):
        lens = rng.integers(256, 4097, b).astype(np.int32)
        nb = int(((lens + B - 1) // B).sum()) * shape.n_kv_heads + 64
        kv, pool = make_pool(nb)
        mb = int((lens.max() + B - 1) // B)
        tables = torch.from_numpy(wl.build_tables(lambda m, k: mx.mux_alloc_blocks(pool, m, k), 0, lens, shape.n_kv_heads, B, mb)).to(dev)
        q = torch.randn(b, shape.n_q_heads, d, device=dev).to(torch.bfloat16)
        k = torch.randn(b, shape.n_kv_heads, d, device=dev).to(torch.bfloat16)
        out = torch.empty_like(q)
        lens_dev = torch.from_numpy(lens).to(dev)
        ws = torch.empty(max(mx.mux_decode_step_workspace_bytes(pool, 1, b, shape.n_q_heads, shape.n_kv_heads, int(lens.max())), 16),
                         dtype=torch.uint8, device=dev)
        kv.zero_()      # values do not matter for the timing, but the pool must not hold NaN patterns
        t = time_it(lambda: mx.mux_decode_step(pool, out[None], q[None], k[None], k[None], tables[None], lens_dev, int(lens.max()),
                                               1.0 / math.sqrt(d), ws))
        mx.mux_pool_destroy(pool)
        return t

    def prefill_latency(shape, b, plen=1280):
        nb = b * (plen // B) * shape.n_kv_heads + 64
        kv, pool = make_pool(nb)
        lens = np.full(b, plen, np.int32)
        tables = torch.from_numpy(wl.build_tables(lambda m, k: mx.mux_alloc_blocks(pool, m, k), 0, lens, shape.n_kv_heads, B, plen // B)).to(dev)
        n = b * plen
        q = torch.randn(n, shape.n_q_heads, d, device=dev).to(torch.bfloat16)
        k = torch.randn(n, shape.n_kv_heads, d, device=dev).to(torch.bfloat16)
        out = torch.empty_like(q)
        seq = torch.arange(b, dtype=torch.int32, device=dev).repeat_interleave(plen).contiguous()
        pos = torch.arange(plen, dtype=torch.int32, device=dev).repeat(b).contiguous()
        cu = torch.arange(0, n + 1, plen, dtype=torch.int32, device=dev)
        start = torch.zeros(b, dtype=torch.int32, device=dev)

        def step():
            mx.mux_kv_append(pool, k, k, seq, pos, tables)
            mx.mux_prefill_attn(pool, out, q, cu, start, tables, plen, plen, 1.0 / math.sqrt(d), None)

        t = time_it(step, reps=10)
        mx.mux_pool_destroy(pool)
        return t

    def fit(bs, ts):
        c1, c0 = np.polyfit(np.asarray(bs, float), np.asarray(ts, float), 1)
        return max(float(c0), 0.0), max(float(c1), 0.0)

    p_bs = [1, 2, 4, 8]
    p_ts = [prefill_latency(wl.LLAMA_13B, b) for b in p_bs]
    p0, p1 = fit(p_bs, p_ts)
    other_prefill = p0 + p1 * 4          # the colocated prefilling LLM's batch of four prompts
    report = {"prefill_13B": {"batch": p_bs, "seconds": p_ts, "fit": [p0, p1]}, "decoders": []}
    d_bs = [16, 32, 64, 128]
    for shape in (wl.LLAMA_7B, wl.GQA_65B):
        d_ts = [decode_latency(shape, b) for b in d_bs]
        d0, d1 = fit(d_bs, d_ts)
        own_p = [prefill_latency(shape, b) for b in (1, 4)]
        q1 = (own_p[1] - own_p[0]) / 3.0
        q0 = max(own_p[0] - q1, 0.0)
        ceiling = 1.0 / (d1 * gen_len) if d1 > 0 else float("inf")      # requests/s as b grows without bound
        rows = []
        for frac in (0.25, 0.5, 0.75, 0.9):
            rate = frac * ceiling
            b = int(mx.mux_find_batch_size(rate, 4096, q0, q1, d0, d1, gen_len, other_prefill))
            row = {"rate_req_s": rate, "fraction_of_ceiling": frac, "batch_from_eq3": b}
            if 0 < b <= 512:
                td = decode_latency(shape, b)
                tp = q0 + q1 * b
                tput = b / (other_prefill + tp + td * gen_len)
                row.update({"measured_t_d_s": td, "measured_req_s_at_that_batch": tput, "meets_rate": bool(tput >= 0.97 * rate)})
            rows.append(row)
        report["decoders"].append({"model": shape.name, "batch": d_bs, "seconds": d_ts, "fit": [d0, d1], "own_prefill_fit": [q0, q1],
                                   "ceiling_req_s": ceiling, "rates": rows})
    line = {"metric": "Eq. 3 estimator fed by measured attention latencies (one layer)", "value": report["decoders"][0]["ceiling_req_s"],
            "unit": "requests/s", "n_gpus": 1, "higher_is_better": True, "dtype": "f32", "storage_dtype": "bf16", "data": "synthetic",
            "config": {"workload": "configuration 4's shapes: 13B-shaped prefill (prompts of 1 280 tokens) next to 7B- and 65B-GQA-shaped decoding "
                                   "(contexts U[256, 4096]); generation length 338; latencies of the attention path of one layer"},
            "estimate": report}
    print(json.dumps(line))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", choices=["all", "decode", "prefill"], default="all",
                    help="run only the decode models or only the prefill model of the configuration")
    ap.add_argument("--fused", action="store_true", help="use mux_decode_step (append + attention in one launch)")
    ap.add_argument("--chain-decode", action="store_true",
                    help="make each decode kernel wait for the previous model's (adds cross-stream event latency)")
    ap.add_argument("--cu-fraction", type=float, default=0.0,
                    help="run every model's stream on the first F x (compute units) only (CU-masked streams)")
    ap.add_argument("--cu-split", type=float, default=0.0,
                    help="decode streams get the first F x (compute units), prefill streams the rest")
    ap.add_argument("--adbs", action="store_true",
                    help="second workload: the batch scheduler serving a request stream (prints its own JSON line)")
    ap.add_argument("--adbs-driver", choices=["runner", "runner-one-stream", "python"], default="runner",
                    help="who launches the scheduler's jobs: the library's runner (one stream per model, or one for all) "
                         "or the Python driver")
    ap.add_argument("--adbs-layers", action="store_true",
                    help="--adbs: models with all their layers (40 / 32 / 32) and a pool 32x as large: whole-model K/V traffic")
    ap.add_argument("--adbs-scale", type=int, default=1,
                    help="--adbs: multiply pool size, sequence slots, arrivals per pass and prefill token budget")
    ap.add_argument("--prefill-prompts", type=int, default=0,
                    help="--config 4 --only prefill: N prompts of --prefill-len tokens in chunks of --prefill-chunk instead of the configuration's 8")
    ap.add_argument("--prefill-len", type=int, default=0)
    ap.add_argument("--prefill-chunk", type=int, default=0)
    ap.add_argument("--estimate", action="store_true",
                    help="measure prefill / decode latencies against the batch size and feed the Eq. 3 estimator (prints its own JSON line)")
    ap.add_argument("--no-solo", action="store_true", help="skip the per-model solo passes after the timed loop")
    ap.add_argument("--models", type=int, default=0, help="run only the first N decode models of the configuration (0 = all)")
    ap.add_argument("--sustain-ms", type=float, default=150.0,
                    help="after the timed steps, keep stepping for about this long and report the rate of that longer window too")
    ap.add_argument("--pmc-calibration", action="store_true", help="also run three 1 GiB device copies after the timed loop")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        return 2
    if int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: launched with WORLD_SIZE > 1; this build runs on one GPU only", file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    mx.load()
    if args.adbs:
        return run_adbs(args)
    if args.estimate:
        return run_estimate(args)
    SOLO_STEPS = 20
    SUSTAIN_STEPS = 0 if args.sustain_ms <= 0 else {2: 400, 3: 300, 4: 150, 5: 15}.get(args.config, 100)
    total = args.steps + args.warmup + SOLO_STEPS + SUSTAIN_STEPS
    override = None
    if args.prefill_prompts > 0:
        if args.config != 4 or args.only != "prefill" or args.prefill_len <= 0:
            print("bench.py: --prefill-prompts needs --config 4 --only prefill --prefill-len L", file=sys.stderr)
            return 2
        override = (args.prefill_prompts, args.prefill_len, args.prefill_chunk if args.prefill_chunk > 0 else args.prefill_len)
    w, pool, models, prefills = build_workload(args.config, total, prefill_override=override, with_decode=args.only != "prefill")
    if args.models > 0:
        models = models[:args.models]
    step_models = [] if args.only == "prefill" else models
    for m in models:
        m.fused = args.fused
    if args.only == "decode":
        prefills = []
    if not step_models and not prefills:
        print("bench.py: configuration %d has nothing to run with --only %s" % (args.config, args.only), file=sys.stderr)
        return 2

    # Optional compute partitioning (the analogue of the paper's MPS shares): CU-masked streams.
    # Unit i of the mask belongs to XCD i % 8, so "the first n" units are spread evenly over the
    # XCDs when n is a multiple of 8 (a mask that leaves an XCD without units is refused).
    partition = None
    if args.cu_fraction > 0 or args.cu_split > 0:
        n_cu = mx.mux_device_cu_count()
        frac = args.cu_fraction if args.cu_fraction > 0 else args.cu_split
        n_first = min(n_cu, max(8, int(round(frac * n_cu / 8)) * 8))
        torch.cuda.synchronize()
        masked = []
        for m in step_models:
            masked.append(mx.MaskedStream(range(n_first)))
            m.stream = masked[-1].stream
        for pm in prefills:
            cus = range(n_first) if args.cu_fraction > 0 else range(n_first, n_cu)
            masked.append(mx.MaskedStream(cus))
            pm.stream = masked[-1].stream
        partition = {"compute_units": n_cu, "decode_units": n_first if step_models else 0,
                     "prefill_units": (n_first if args.cu_fraction > 0 else n_cu - n_first) if prefills else 0}

    # Every model has its own stream and nothing orders the streams against each other: the
    # small kernels of one model overlap with the other's decode attention, and the decode
    # kernels, each of which fills the GPU on its own, end up back to back.  (--chain-decode
    # orders them explicitly through events; the cross-stream waits cost 15-50 us per launch.)
    last = None
    for _ in range(args.warmup):
        for pm in prefills:
            pm.step(record=False)
        for m in step_models:
            _, ev = m.step(record=False, after=last)
            last = ev if args.chain_decode else None
    torch.cuda.synchronize()
    ref = torch.cuda.Event(enable_timing=True)
    ref.record()
    t0 = time.perf_counter()
    kv_bytes = 0
    for _ in range(args.steps):
        for pm in prefills:   # prefill jobs are scheduled first (Section 3.3: prefill is prioritised)
            pm.step(record=True)
        for m in step_models:
            b, ev = m.step(record=True, after=last)
            last = ev if args.chain_decode else None
            kv_bytes += b
    t_enqueued = time.perf_counter() - t0
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # the same loop over a longer window (the timed region above is only steps x ms_per_step long)
    sustained = None
    if SUSTAIN_STEPS > 0 and (step_models or prefills):
        n_timed = [len(m.decode_events) for m in step_models]
        t1 = time.perf_counter()
        b1 = 0
        n1 = 0
        while n1 < SUSTAIN_STEPS and (time.perf_counter() - t1) * 1e3 < args.sustain_ms:
            for pm in prefills:
                pm.step(record=False)
            for m in step_models:
                b, ev = m.step(record=False, after=last)
                last = ev if args.chain_decode else None
                b1 += b
            n1 += 1
        torch.cuda.synchronize()
        dt1 = time.perf_counter() - t1
        sustained = {"steps": n1, "window_ms": dt1 * 1e3, "GBps": b1 / dt1 / 1e9, "ms_per_step": dt1 / n1 * 1e3}
    # each decode model alone: nothing else runs on the GPU, so a launch's start-to-end duration is its own
    solo = []
    solo_durs, solo_algo = [], []
    if step_models and not args.no_solo:
        for m in step_models:
            torch.cuda.synchronize()
            n_before = len(m.decode_events)
            t1 = time.perf_counter()
            b1 = 0
            for _ in range(SOLO_STEPS):
                b, _ = m.step(record=True)
                b1 += b
            torch.cuda.synchronize()
            wall = time.perf_counter() - t1
            mine = m.decode_events[n_before:]
            del m.decode_events[n_before:]
            d = [e0.elapsed_time(e1) * 1e-3 for e0, e1, _ in mine]
            solo_durs += d
            solo_algo += [bb for _, _, bb in mine]
            solo.append({"model": m.shape.name, "seqs": m.n, "GBps": b1 / max(wall, 1e-9) / 1e9,
                         "launch_ms": float(np.mean(d) * 1e3), "launch_GBps": float(np.sum([bb for _, _, bb in mine]) / np.sum(d) / 1e9)})
    if args.pmc_calibration:
        # a plain copy of known size in the same process, for scaling rocprofv3 --pmc byte counters
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    # dominant kernel: decode attention (main kernel + span combine), HIP-event durations
    roofline = None
    if step_models:
        durs, algo = [], []
        for m in step_models:
            for e0, e1, b in m.decode_events:
                durs.append(e0.elapsed_time(e1) * 1e-3)
                algo.append(b)
        # The decode launches of different models sit on different streams and may run at the same
        # time, sharing HBM; a launch's own start-to-end duration then counts the shared time twice.
        # The time during which at least one decode kernel was running counts it once: with no overlap
        # it equals the sum of the launch durations.
        spans = sorted((ref.elapsed_time(e0), ref.elapsed_time(e1)) for m in step_models for e0, e1, _ in m.decode_events)
        busy, cur_lo, cur_hi = 0.0, None, None
        for lo, hi in spans:
            if cur_hi is None or lo > cur_hi:
                busy += 0.0 if cur_hi is None else cur_hi - cur_lo
                cur_lo, cur_hi = lo, hi
            else:
                cur_hi = max(cur_hi, hi)
        busy = (busy + cur_hi - cur_lo) * 1e-3
        union = float(np.sum(algo) / busy / 1e9)             # bytes / time with at least one decode launch running
        overlapped = float(np.sum(algo) / np.sum(durs) / 1e9)  # bytes / start-to-end durations, shared time counted per launch
        if solo_durs:
            # launches of the same models with nothing else on the GPU: the kernel's own duration
            achieved, avg_ms, per_launch = float(np.sum(solo_algo) / np.sum(solo_durs) / 1e9), float(np.mean(solo_durs) * 1e3), float(np.mean(solo_algo))
            basis = ("solo: %d launches per model after the timed region, one model at a time, HIP events on the model's stream "
                     "around the decode launch (no other kernel runs meanwhile)" % SOLO_STEPS)
        else:
            achieved, avg_ms, per_launch = overlapped, float(np.mean(durs) * 1e3), float(np.mean(algo))
            basis = "timed region: mean start-to-end duration of a decode launch (launches of different models may overlap)"
        roofline = {
            "kernel": "decode_attn_kernel (alone for launches of whole rows; followed by decode_combine_kernel when contexts are split, preceded by decode_plan_kernel beyond 256 rows), one launch per model per step",
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "frac_basis": basis,
            "traffic": MEASURED_TRAFFIC_CFG2["bytes"] if args.config == 2 else None,
            "traffic_source": MEASURED_TRAFFIC_CFG2["source"] if args.config == 2 else None,
            "traffic_note": MEASURED_TRAFFIC_CFG2["note"] if args.config == 2 else None,
            "avg_launch_ms": avg_ms, "algorithmic_bytes_per_launch": per_launch, "launches": len(solo_durs) or len(durs),
            "frac_solo": achieved / HBM_PEAK_GBS if solo_durs else None,
            "timed_region": {
                "launches": len(durs), "algorithmic_bytes_per_launch": float(np.mean(algo)),
                "frac_union": union / HBM_PEAK_GBS, "union_GBps": union, "union_ms_per_launch": busy / len(durs) * 1e3,
                "frac_overlapped": overlapped / HBM_PEAK_GBS, "overlapped_avg_launch_ms": float(np.mean(durs) * 1e3),
                "overlapped_median_launch_ms": float(np.median(durs) * 1e3), "overlapped_min_launch_ms": float(np.min(durs) * 1e3),
                "overlap": float(np.sum(durs) / busy),
                "note": "launches of different models run on different streams and overlap: union = bytes / time with at least "
                        "one decode launch running; overlapped = bytes / mean start-to-end duration of a launch, which counts "
                        "the time two launches share once per launch; overlap = their ratio",
            },
        }
    n_seqs = sum(m.n for m in step_models)
    result = {
        "metric": "decode-attn KV GB/s (% of HBM peak) + tokens/s, multi-LLM mixed batch",
        "value": kv_bytes / dt / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "storage_dtype": "bf16", "data": "synthetic",
        "config": {
            "workload": "config %d: %s; block_size %d; %d head-blocks, seeded random placement; per step and model: "
                        "alloc -> table patch -> %s, one stream per model, decode kernels %s"
                        % (args.config, ", ".join(["%s x%d decoding seqs" % (m.shape.name, m.n) for m in models] +
                                                  ["%s x%d prompts%s in chunks of %d" % (pm.shape.name, pm.job.n_seqs, " of %d tokens" % args.prefill_len
                                                                                       if override else "", pm.job.chunk)
                                                   for pm in prefills]), w.block_size, pool.num_blocks,
                           "decode_step (fused append + attention)" if args.fused else "kv_append(1 token/seq) -> decode_attn",
                           "chained by events" if args.chain_decode else "unordered across streams"),
            "layers": 1,
        },
        "pct_hbm_peak": 100.0 * kv_bytes / dt / 1e9 / HBM_PEAK_GBS,
        "tokens_per_s": n_seqs * args.steps / dt,
        "host_enqueue_ms_per_step": t_enqueued / args.steps * 1e3,
        "roofline": roofline,
    }
    if prefills:
        ev = [e for pm in prefills for e in pm.events]
        t = sum(e0.elapsed_time(e1) for e0, e1, _, _ in ev) * 1e-3
        fl = sum(f for _, _, f, _ in ev)
        result["prefill"] = {
            "kernel": "prefill_attn_kernel, one launch per chunk stage", "launches": len(ev), "tflops": fl / t / 1e12,
            "bound": "mfma", "peak_tflops": 2500.0, "frac": fl / t / 2.5e15, "avg_launch_ms": t / len(ev) * 1e3,
            "flops_per_launch": fl / len(ev), "kv_bytes_per_launch": sum(b for _, _, _, b in ev) / len(ev),
        }
        if roofline is not None:
            # what the memory system carried in the timed loop: the decode models' K/V plus what the prefill stages move
            result["all_streams_GBps"] = (kv_bytes + sum(pm.bytes_moved for pm in prefills)) / dt / 1e9
        if roofline is None:   # prefill only: the MFMA-bound kernel is the dominant one
            result["metric"], result["unit"], result["value"] = "prefill-attn causal TFLOP/s (% of MFMA peak)", "TFLOP/s", fl / t / 1e12
            result["dtype"] = "bf16"   # matrix products in bf16, accumulation in f32
            result["roofline"] = {"kernel": "prefill_attn_kernel", "bound": "mfma", "achieved": fl / t / 1e12, "peak": 2500.0,
                                  "unit": "TFLOP/s", "frac": fl / t / 2.5e15, "traffic": None}
    if sustained:
        result["sustained"] = sustained
    if solo:
        result["solo_decode"] = solo
    result["ceilings"] = measure_ceilings()
    result["allocator_ns_per_block"] = allocator_ns_per_block()
    result["kv_append"] = measure_append()
    if partition:
        result["config"]["cu_partition"] = partition
    if not args.no_cpu_baseline and models:
        result["cpu_baseline"] = cpu_baseline(models, single_core=args.config <= 2)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
