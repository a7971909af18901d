"""Driver that runs the jobs of the batch scheduler (MuxServe, Section 3.3, Algorithm 3) on the
GPU: it mirrors the scheduler's block tables to the device and launches mux_kv_append,
mux_prefill_attn and mux_decode_attn for every job, one HIP stream per model.  The K/V rows and
queries come from a caller-given source (a real engine would compute them with its QKV
projections); everything that decides or computes is in the library.

Used by the tests (with a seeded CPU source mirrored into the oracle) and by bench.py (with a
device random source).
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


class _ModelState:
    def __init__(self, pool, shape, max_seqs, max_blocks, device):
        self.shape = shape
        self.tables = torch.zeros(max_seqs, shape.n_kv_heads, max_blocks, dtype=torch.int32, device=device)
        self.ctx = torch.zeros(max_seqs, dtype=torch.int32, device=device)
        self.q_all = torch.zeros(max_seqs, shape.n_q_heads, pool.head_dim, dtype=torch.bfloat16, device=device)
        self.out_all = torch.zeros_like(self.q_all)
        self.stream = torch.cuda.Stream(device=device)
        ws = mx.mux_decode_workspace_bytes(pool, max_seqs, shape.n_q_heads, shape.n_kv_heads, max_blocks * pool.block_size)
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

    def _job_values(self, model, ids, pos0, pos1):
        """K/V rows and queries of positions pos0[i] .. pos1[i]-1 of every request of a job,
        concatenated in request order."""
        if hasattr(self.values, "job_values"):
            return self.values.job_values(model, ids, pos0, pos1)
        ks, vs, qs = [], [], []
        for rid, p0, p1 in zip(ids.tolist(), pos0.tolist(), pos1.tolist()):
            k, v = self.values.kv(model, rid, p0, p1)
            ks.append(k)
            vs.append(v)
            qs.append(self.values.q(model, rid, p0, p1))
        return torch.cat(ks), torch.cat(vs), torch.cat(qs)

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
        k, v, q = self._job_values(model, ids, np.zeros_like(lens), lens)
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
        k, v, q = self._job_values(model, ids, lens - 1, lens)
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
        self.iterations += 1
        return results

    def idle(self) -> bool:
        return all(self.sched.counts(m)[:2] == (0, 0) for m in range(len(self.models)))
