"""Drivers that run the jobs of the batch scheduler (MuxServe, Section 3.3, Algorithm 3) on the
GPU, one HIP stream per model.  The K/V rows and queries come from a caller-given source (a real
engine would compute them with its QKV projections); everything that decides or computes is in
the library.

Engine       mirrors the scheduler's block tables to the device itself and calls mux_kv_append,
             mux_prefill_attn and mux_decode_attn for every job (a handful of small copies and
             launches per job from Python).
NativeEngine hands every job to the library's runner (mux_runner_launch): the job's arrays, the
             table update and the kernels are issued from C++.

Used by the tests (with a seeded CPU source mirrored into the oracle) and by bench.py.
"""
from __future__ import annotations

import math
from typing import List, Sequence

import numpy as np
import torch

from . import binding as mx


class DeviceRandomSource:
    """Synthetic K/V/Q: fresh N(0,1) values drawn on the device (their values do not matter for
    timing; a recomputed request simply gets new ones)."""

    def __init__(self, shapes, head_dim: int, device="cuda", seed: int = 0):
        self.shapes, self.d, self.device = shapes, head_dim, device
        self.gen = torch.Generator(device=device)
        self.gen.manual_seed(seed)

    def _draw(self, n, heads):
        return torch.randn(n, heads, self.d, generator=self.gen, device=self.device).to(torch.bfloat16)

    def kv(self, model, request_id, pos0, pos1):
        h = self.shapes[model].n_kv_heads
        return self._draw(pos1 - pos0, h), self._draw(pos1 - pos0, h)

    def q(self, model, request_id, pos0, pos1):
        return self._draw(pos1 - pos0, self.shapes[model].n_q_heads)

    def job_values(self, model, request_ids, pos0, pos1):
        """K, V and Q of a whole job in three draws (rows in request order)."""
        n = int(np.sum(np.asarray(pos1) - np.asarray(pos0)))
        s = self.shapes[model]
        return self._draw(n, s.n_kv_heads), self._draw(n, s.n_kv_heads), self._draw(n, s.n_q_heads)


def _job_values(values, model, ids, pos0, pos1):
    """K/V rows and queries of positions pos0[i] .. pos1[i]-1 of every request of a job,
    concatenated in request order."""
    if hasattr(values, "job_values"):
        return values.job_values(model, ids, pos0, pos1)
    ks, vs, qs = [], [], []
    for rid, p0, p1 in zip(ids.tolist(), pos0.tolist(), pos1.tolist()):
        k, v = values.kv(model, rid, p0, p1)
        ks.append(k)
        vs.append(v)
        qs.append(values.q(model, rid, p0, p1))
    return torch.cat(ks), torch.cat(vs), torch.cat(qs)


class _ModelState:
    def __init__(self, pool, shape, max_seqs, max_blocks, device):
        self.shape = shape
        self.tables = torch.zeros(max_seqs, shape.n_kv_heads, max_blocks, dtype=torch.int32, device=device)
        self.ctx = torch.zeros(max_seqs, dtype=torch.int32, device=device)
        self.q_all = torch.zeros(max_seqs, shape.n_q_heads, pool.head_dim, dtype=torch.bfloat16, device=device)
        self.out_all = torch.zeros_like(self.q_all)
        self.stream = torch.cuda.Stream(device=device)
        # the split of long contexts depends on the rows and the longest context of the launch: size for the worst one
        ws = mx.mux_decode_workspace_bound(pool, max_seqs, shape.n_q_heads, shape.n_kv_heads, max_blocks * pool.block_size)
        self.workspace = torch.empty(ws, dtype=torch.uint8, device=device)
        self.done = torch.cuda.Event()
        self.tokens = 0          # output tokens produced
        self.kv_bytes_read = 0   # K/V bytes the decode steps had to read


class Engine:
    """submit() requests, then step(): one iteration of the scheduler, its jobs launched on the
    GPU.  step() returns [(job, out)], out = attention output rows of the job's sequences
    ([total prefill rows | n decode sequences][Hq][d]) or None for a preemption."""

    def __init__(self, pool: mx.Pool, shapes: Sequence, max_seqs: int, max_blocks: int, max_prefill_tokens: int, values,
                 device="cuda", keep_outputs: bool = True, **sched_kw):
        self.pool, self.shapes, self.values, self.device = pool, list(shapes), values, device
        self.max_seqs, self.max_blocks, self.keep_outputs = max_seqs, max_blocks, keep_outputs
        self.sched = mx.Scheduler(pool, [s.n_kv_heads for s in shapes], max_seqs, max_blocks, max_prefill_tokens, **sched_kw)
        self.models: List[_ModelState] = [_ModelState(pool, s, max_seqs, max_blocks, device) for s in shapes]
        self.scale = 1.0 / math.sqrt(pool.head_dim)
        self.iterations = 0

    def submit(self, model: int, request_id: int, prompt_len: int, output_len: int) -> None:
        rc = self.sched.submit(model, request_id, prompt_len, output_len)
        if rc != mx.MUX_OK:
            raise mx.MuxError(rc, "mux_sched_submit")

    # -- helpers -----------------------------------------------------------------
    def _dev(self, a, dtype):
        return torch.from_numpy(np.ascontiguousarray(a)).to(self.device, dtype=dtype, non_blocking=False)

    def _mirror_rows(self, st: _ModelState, model: int, slots: np.ndarray) -> None:
        if slots.size == 0:
            return
        rows = self.sched.table(model)[slots]
        # entries never written stay -1 on the host; the device copy only needs valid ids where they are used
        st.tables.index_copy_(0, self._dev(slots, torch.int64), self._dev(np.maximum(rows, 0), torch.int32))

    def _prefill(self, model: int, job) -> torch.Tensor:
        st = self.models[model]
        slots, lens, ids = job["slots"], job["lens"], job["ids"]
        self._mirror_rows(st, model, slots)
        k, v, q = _job_values(self.values, model, ids, np.zeros_like(lens), lens)
        n, total = len(lens), int(lens.sum())
        # one host-to-device copy for all the small integer arrays of the job
        packed = self._dev(np.concatenate([np.repeat(slots, lens), np.concatenate([np.arange(x) for x in lens]),
                                           [0], np.cumsum(lens), np.zeros(n, np.int64), slots]), torch.int32)
        tok_seq, tok_pos = packed[:total], packed[total:2 * total]
        cu, q_start, slots_dev = packed[2 * total:2 * total + n + 1], packed[2 * total + n + 1:2 * total + 2 * n + 1], packed[2 * total + 2 * n + 1:]
        mx.mux_kv_append(self.pool, k, v, tok_seq, tok_pos, st.tables, stream=st.stream)
        tables_job = st.tables.index_select(0, slots_dev)
        out = torch.empty_like(q)
        mx.mux_prefill_attn(self.pool, out, q, cu, q_start, tables_job, int(lens.max()), int(lens.max()), self.scale,
                            stream=st.stream)
        st.tokens += len(lens)
        return out

    def _decode(self, model: int, job) -> torch.Tensor:
        st = self.models[model]
        slots, lens, ids, flags = job["slots"], job["lens"], job["ids"], job["flags"]
        self._mirror_rows(st, model, slots[(flags & mx.MUX_JOB_FLAG_TABLE) != 0])
        k, v, q = _job_values(self.values, model, ids, lens - 1, lens)
        n = len(lens)
        ctx = np.zeros(self.max_seqs, dtype=np.int32)     # slots outside the job attend to nothing
        ctx[slots] = lens
        packed = self._dev(np.concatenate([slots, lens - 1, ctx]), torch.int32)   # one copy for the job's integer arrays
        slots32, pos = packed[:n], packed[n:2 * n]
        slots_dev = slots32.long()
        mx.mux_kv_append(self.pool, k, v, slots32, pos, st.tables, stream=st.stream)
        st.ctx.copy_(packed[2 * n:])
        st.q_all.index_copy_(0, slots_dev, q)
        mx.mux_decode_attn(self.pool, st.out_all, st.q_all, st.tables, st.ctx, int(lens.max()), self.scale, st.workspace,
                           stream=st.stream)
        st.tokens += len(lens)
        st.kv_bytes_read += int(lens.astype(np.int64).sum()) * 2 * st.shape.n_kv_heads * self.pool.head_dim * 2
        return st.out_all.index_select(0, slots_dev) if self.keep_outputs else None

    def step(self):
        # kernels of the previous iteration come first on every stream: blocks released at the
        # start of this iteration may change hands
        for st in self.models:
            for other in self.models:
                if other is not st:
                    st.stream.wait_event(other.done)
        jobs = self.sched.step()
        results = []
        for job in jobs:
            st = self.models[job["model"]]
            with torch.cuda.stream(st.stream):
                if job["kind"] == mx.MUX_JOB_PREFILL:
                    results.append((job, self._prefill(job["model"], job)))
                elif job["kind"] == mx.MUX_JOB_DECODE:
                    results.append((job, self._decode(job["model"], job)))
                else:
                    results.append((job, None))
        for st in self.models:
            st.done.record(st.stream)
            if self.keep_outputs:
                st.stream.synchronize()   # the caller reads the outputs from another stream
        self.iterations += 1
        return results

    def idle(self) -> bool:
        return all(self.sched.counts(m)[:2] == (0, 0) for m in range(len(self.models)))

    def tokens(self) -> int:
        """Output tokens produced so far."""
        return sum(st.tokens for st in self.models)


class _NativeModel:
    def __init__(self, pool, shape, layers, max_seqs, max_tokens, device, stream):
        d = pool.head_dim
        kw = dict(dtype=torch.bfloat16, device=device)
        self.shape, self.layers, self.stream = shape, layers, stream
        # decode buffers: [layer][slot][heads][d]; prefill buffers: room for [layer][the job's tokens, packed][heads][d]
        self.k_dec, self.v_dec = (torch.randn(layers, max_seqs, shape.n_kv_heads, d, **kw) for _ in range(2))
        self.q_dec, self.out_dec = (torch.randn(layers, max_seqs, shape.n_q_heads, d, **kw) for _ in range(2))
        self.k_pre, self.v_pre = (torch.randn(layers * max_tokens, shape.n_kv_heads, d, **kw) for _ in range(2))
        self.q_pre, self.out_pre = (torch.randn(layers * max_tokens, shape.n_q_heads, d, **kw) for _ in range(2))

    def layered(self, wide: torch.Tensor) -> torch.Tensor:
        """[rows][layers * heads][d] (the layout of a value source: one wide layer) -> [layers][rows][heads][d]."""
        rows, wide_heads, d = wide.shape
        return wide.view(rows, self.layers, wide_heads // self.layers, d).permute(1, 0, 2, 3)

    def wide(self, layered: torch.Tensor) -> torch.Tensor:
        layers, rows, heads, d = layered.shape
        return layered.permute(1, 0, 2, 3).reshape(rows, layers * heads, d)


class NativeEngine:
    """Engine's interface on top of mux_runner_*.  shapes = the shape of ONE layer of every model,
    layers = layers per model (default 1 each); the scheduler sees layers x KV heads blocks per
    token span.  values = a source as for Engine, which sees a model as one wide layer of
    layers x heads heads, or None: the buffers keep the random values they were created with
    (timing runs; step() then returns the number of jobs and reads nothing back)."""

    def __init__(self, pool: mx.Pool, shapes: Sequence, max_seqs: int, max_blocks: int, max_prefill_tokens: int, values=None,
                 device="cuda", keep_outputs: bool = True, shared_stream: bool = False, layers=None, **sched_kw):
        self.pool, self.shapes, self.values, self.device = pool, list(shapes), values, device
        self.layers = [1] * len(self.shapes) if layers is None else [int(x) for x in layers]
        self.keep_outputs = keep_outputs and values is not None
        self.sched = mx.Scheduler(pool, [s.n_kv_heads * n for s, n in zip(shapes, self.layers)], max_seqs, max_blocks,
                                  max_prefill_tokens, **sched_kw)
        one = torch.cuda.Stream(device=device) if shared_stream else None
        streams = [one or torch.cuda.Stream(device=device) for _ in shapes]
        self.runner = mx.Runner(self.sched, [s.n_q_heads for s in shapes], streams, n_layers=self.layers)
        max_tokens = max(max_prefill_tokens, max_blocks * pool.block_size)
        self.models = [_NativeModel(pool, s, n, max_seqs, max_tokens, device, st) for s, n, st in zip(shapes, self.layers, streams)]
        torch.cuda.synchronize()
        self.scale = 1.0 / math.sqrt(pool.head_dim)
        self.iterations = 0
        if values is None:
            for i, st in enumerate(self.models):
                self.runner.set_buffers(i, (st.out_pre, st.q_pre, st.k_pre, st.v_pre), (st.out_dec, st.q_dec, st.k_dec, st.v_dec),
                                        self.scale)

    def tokens(self) -> int:
        """Output tokens produced so far: every request of a prefill or decode job yields one."""
        return self.runner.counts()[1]

    def submit(self, model: int, request_id: int, prompt_len: int, output_len: int) -> None:
        rc = self.sched.submit(model, request_id, prompt_len, output_len)
        if rc != mx.MUX_OK:
            raise mx.MuxError(rc, "mux_sched_submit")

    def _fill(self, st, job):
        """Copies the job's K/V/Q rows from the source into the buffers the runner reads."""
        model, lens, ids = job["model"], job["lens"], job["ids"]
        if job["kind"] == mx.MUX_JOB_PREFILL:
            k, v, q = _job_values(self.values, model, ids, np.zeros_like(lens), lens)
            n = int(lens.sum())
            for buf, val in ((st.k_pre, k), (st.v_pre, v), (st.q_pre, q)):
                buf[:st.layers * n].view(st.layers, n, buf.shape[1], buf.shape[2]).copy_(st.layered(val))
        else:
            k, v, q = _job_values(self.values, model, ids, lens - 1, lens)
            slots = torch.from_numpy(job["slots"].astype(np.int64)).to(self.device)
            for buf, val in ((st.k_dec, k), (st.v_dec, v), (st.q_dec, q)):
                buf.index_copy_(1, slots, st.layered(val))

    def step(self):
        if self.values is None:
            n = self.runner.run_step()
            self.iterations += 1
            return n
        n = self.runner.step()
        results = []
        for j, job in enumerate(self.sched.jobs(n)):
            st = self.models[job["model"]]
            if job["kind"] == mx.MUX_JOB_PREEMPT:
                results.append((job, None))
                continue
            prefill = job["kind"] == mx.MUX_JOB_PREFILL
            with torch.cuda.stream(st.stream):
                self._fill(st, job)
                if prefill:
                    self.runner.launch(j, st.out_pre, st.q_pre, st.k_pre, st.v_pre, self.scale)
                else:
                    self.runner.launch(j, st.out_dec, st.q_dec, st.k_dec, st.v_dec, self.scale)
                out = None
                if self.keep_outputs:
                    if prefill:
                        t = int(job["lens"].sum())
                        out = st.wide(st.out_pre[:st.layers * t].view(st.layers, t, st.shape.n_q_heads, self.pool.head_dim))
                    else:
                        out = st.wide(st.out_dec.index_select(1, torch.from_numpy(job["slots"].astype(np.int64)).to(self.device)))
            results.append((job, out))
        if self.keep_outputs:
            self.runner.synchronize()
        self.iterations += 1
        return results

    def idle(self) -> bool:
        return all(self.sched.counts(m)[:2] == (0, 0) for m in range(len(self.models)))
