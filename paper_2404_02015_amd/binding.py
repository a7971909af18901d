"""Thin ctypes binding of libmux.so: same names as include/mux.h, argument marshalling only.

Tensors are torch tensors used purely as handles to device memory (`data_ptr()`); streams
are torch.cuda.Stream objects (or None for the current stream).  Every step of the path runs
inside the library's HIP kernels; there is no fallback: if libmux.so is missing or fails to
load, importing a function from here raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np
import torch  # must be imported before libmux.so so both share one HIP runtime

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmux.so")

MUX_OK, MUX_ERR_INVALID, MUX_ERR_NOMEM, MUX_ERR_QUOTA, MUX_ERR_HIP, MUX_ERR_UNSUPPORTED, MUX_ERR_TOO_LARGE = 0, -1, -2, -3, -4, -5, -6
MUX_STATIC_SCRATCH_BYTES = 32 * 1024 * 1024
MUX_BF16, MUX_FP32 = 0, 1

EXPORTS = [
    "mux_pool_create", "mux_pool_destroy", "mux_pool_num_free", "mux_pool_num_used", "mux_pool_block_bytes",
    "mux_alloc_blocks", "mux_free_blocks", "mux_kv_append", "mux_decode_attn", "mux_decode_workspace_bytes",
    "mux_prefill_attn", "mux_prefill_workspace_bytes", "mux_status_string", "mux_decode_step",
    "mux_decode_step_workspace_bytes", "mux_pool_set_quota", "mux_pool_get_quota", "mux_pool_peak_used",
    "mux_pool_init_quotas", "mux_pool_adapt_quotas", "mux_sched_create", "mux_sched_destroy", "mux_sched_submit",
    "mux_sched_step", "mux_sched_job", "mux_sched_job_seqs", "mux_sched_table", "mux_sched_counts",
    "mux_device_cu_count", "mux_stream_create_masked", "mux_stream_destroy", "mux_probe_stream_read", "mux_probe_mfma",
    "mux_estimate_tpt", "mux_find_batch_size", "mux_runner_create", "mux_runner_destroy", "mux_runner_step",
    "mux_runner_launch", "mux_runner_launch_layer", "mux_runner_set_buffers", "mux_runner_run_step", "mux_runner_counts", "mux_runner_synchronize", "mux_runner_read_table",
    "mux_decode_attn_static", "mux_decode_workspace_bound", "mux_prefill_workspace_bound",
]

MUX_JOB_PREFILL, MUX_JOB_DECODE, MUX_JOB_PREEMPT = 1, 2, 3
MUX_JOB_FLAG_TABLE, MUX_JOB_FLAG_FINISHED = 1, 2


class SchedConfig(C.Structure):
    _fields_ = [("n_models", C.c_int32), ("heads", C.POINTER(C.c_int32)), ("max_seqs", C.c_int32),
                ("max_blocks", C.c_int32), ("max_prefill_tokens", C.c_int32), ("adapt_period", C.c_int32),
                ("low_util", C.c_double), ("high_util", C.c_double), ("step_fraction", C.c_double)]


class MuxError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__("%s: %s (%d)" % (what, status_string(status), status))
        self.status = status


_lib = None


def load() -> C.CDLL:
    """Load libmux.so (built by paper_2404_02015_amd.build); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("%s not found: run `python -m paper_2404_02015_amd.build` first" % LIB_PATH)
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t
    L.mux_pool_create.argtypes = [C.POINTER(vp), vp, sz, i64, i32, i32, C.c_int, vp]
    L.mux_pool_create.restype = C.c_int
    L.mux_pool_destroy.argtypes = [vp]
    L.mux_pool_num_free.argtypes = [vp]
    L.mux_pool_num_free.restype = i64
    L.mux_pool_set_quota.argtypes = [vp, i32, i64]
    L.mux_pool_get_quota.argtypes = [vp, i32, C.POINTER(i64)]
    L.mux_pool_peak_used.argtypes = [vp, i32, C.POINTER(i64)]
    L.mux_pool_init_quotas.argtypes = [vp, i32, vp]
    L.mux_pool_adapt_quotas.argtypes = [vp, i32, C.c_double, C.c_double, C.c_double, C.POINTER(i64)]
    L.mux_estimate_tpt.argtypes = [i32, vp, vp, vp, vp, i32, C.c_double]
    L.mux_estimate_tpt.restype = C.c_double
    L.mux_find_batch_size.argtypes = [C.c_double, i64] + [C.c_double] * 6
    L.mux_find_batch_size.restype = i64
    L.mux_probe_stream_read.argtypes = [vp, C.c_size_t, vp, i32, vp]
    L.mux_probe_mfma.argtypes = [vp, i32, i32, C.POINTER(C.c_double), vp]
    L.mux_device_cu_count.argtypes = [C.POINTER(i32)]
    L.mux_stream_create_masked.argtypes = [C.POINTER(vp), vp, i32]
    L.mux_stream_destroy.argtypes = [vp]
    L.mux_sched_create.argtypes = [C.POINTER(vp), vp, C.POINTER(SchedConfig)]
    L.mux_sched_destroy.argtypes = [vp]
    L.mux_sched_submit.argtypes = [vp, i32, i64, i32, i32]
    L.mux_sched_step.argtypes = [vp, C.POINTER(i32)]
    L.mux_sched_job.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
    L.mux_sched_job_seqs.argtypes = [vp, i32, vp, vp, vp, vp]
    L.mux_sched_table.argtypes = [vp, i32]
    L.mux_sched_table.restype = C.POINTER(i32)
    L.mux_sched_counts.argtypes = [vp, i32, vp]
    L.mux_runner_create.argtypes = [C.POINTER(vp), vp, vp, vp, vp, vp]
    L.mux_runner_destroy.argtypes = [vp]
    L.mux_runner_step.argtypes = [vp, C.POINTER(i32)]
    L.mux_runner_launch.argtypes = [vp, i32, vp, vp, vp, vp, f32]
    L.mux_runner_launch_layer.argtypes = [vp, i32, i32, vp, vp, vp, vp, f32]
    L.mux_runner_set_buffers.argtypes = [vp, i32] + [vp] * 8 + [f32]
    L.mux_runner_run_step.argtypes = [vp, C.POINTER(i32)]
    L.mux_runner_counts.argtypes = [vp, vp]
    L.mux_runner_synchronize.argtypes = [vp]
    L.mux_runner_read_table.argtypes = [vp, i32, vp]
    L.mux_pool_num_used.argtypes = [vp, i32]
    L.mux_pool_num_used.restype = i64
    L.mux_pool_block_bytes.argtypes = [vp]
    L.mux_pool_block_bytes.restype = i64
    L.mux_alloc_blocks.argtypes = [vp, i32, i64, vp]
    L.mux_free_blocks.argtypes = [vp, i32, i64, vp]
    L.mux_kv_append.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp]
    L.mux_decode_attn.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, vp, sz, vp]
    L.mux_decode_attn_static.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, vp]
    L.mux_decode_workspace_bytes.argtypes = [vp, i32, i32, i32, i32]
    L.mux_decode_workspace_bytes.restype = sz
    L.mux_decode_workspace_bound.argtypes = [vp, i32, i32, i32, i32]
    L.mux_decode_workspace_bound.restype = sz
    L.mux_prefill_workspace_bound.argtypes = [vp, i32, i32, i32, i32]
    L.mux_prefill_workspace_bound.restype = sz
    L.mux_decode_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, f32, vp, sz, vp]
    L.mux_decode_step_workspace_bytes.argtypes = [vp, i32, i32, i32, i32, i32]
    L.mux_decode_step_workspace_bytes.restype = sz
    L.mux_prefill_attn.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, f32, vp, sz, vp]
    L.mux_prefill_workspace_bytes.argtypes = [vp, i32, i32, i32, i32, i32]
    L.mux_prefill_workspace_bytes.restype = sz
    L.mux_status_string.argtypes = [C.c_int]
    L.mux_status_string.restype = C.c_char_p
    _lib = L
    return L


def status_string(status: int) -> str:
    return load().mux_status_string(int(status)).decode()


def _check(status: int, what: str) -> None:
    if status != MUX_OK:
        raise MuxError(status, what)


def _dev(t: Optional[torch.Tensor], dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError("expected %s, got %s" % (dtype, t.dtype))
    return t.data_ptr()


def _device_pool(pool: "Pool") -> int:
    if not pool.kv.is_cuda:
        raise ValueError("this pool lives in host memory: kernels need a device pool")
    return pool.handle


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def _host_ids(ids) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(ids), dtype=np.int32)


class Pool:
    """Handle of a mux_pool_t plus the torch tensor that backs it (kept alive here)."""

    def __init__(self, handle: int, kv: torch.Tensor, num_blocks: int, block_size: int, head_dim: int, dtype: int):
        self.handle, self.kv = handle, kv
        self.num_blocks, self.block_size, self.head_dim, self.dtype = num_blocks, block_size, head_dim, dtype
        self.torch_dtype = torch.bfloat16 if dtype == MUX_BF16 else torch.float32
        self.elem_bytes = 2 if dtype == MUX_BF16 else 4
        self.block_bytes = 2 * block_size * head_dim * self.elem_bytes

    def __del__(self):
        try:
            mux_pool_destroy(self)
        except Exception:
            pass


def mux_pool_create(kv: torch.Tensor, num_blocks: int, block_size: int, head_dim: int, dtype: int = MUX_BF16,
                    init_free_order=None) -> Pool:
    """kv: a contiguous device tensor (any dtype) whose storage becomes the unified KV space.
    (A host tensor is accepted too: the block manager never touches the memory, only the
    kernel calls do, and those insist on device memory.)"""
    if not kv.is_contiguous():
        raise ValueError("expected a contiguous tensor")
    h = C.c_void_p()
    order = None if init_free_order is None else _host_ids(init_free_order)
    if order is not None and order.size != num_blocks:
        raise MuxError(MUX_ERR_INVALID, "mux_pool_create")
    rc = load().mux_pool_create(C.byref(h), kv.data_ptr(), kv.numel() * kv.element_size(), num_blocks, block_size, head_dim,
                                dtype, None if order is None else order.ctypes.data)
    _check(rc, "mux_pool_create")
    return Pool(h.value, kv, num_blocks, block_size, head_dim, dtype)


def mux_pool_destroy(pool: Pool) -> None:
    if pool.handle:
        load().mux_pool_destroy(pool.handle)
        pool.handle = None


def mux_pool_num_free(pool: Pool) -> int:
    return load().mux_pool_num_free(pool.handle)


def mux_pool_num_used(pool: Pool, model_id: int) -> int:
    return load().mux_pool_num_used(pool.handle, model_id)


def mux_pool_set_quota(pool: Pool, model_id: int, max_blocks: int) -> int:
    """max_blocks = -1 removes the quota.  Returns the status."""
    return load().mux_pool_set_quota(pool.handle, model_id, max_blocks)


def _read_i64(fn, pool: Pool, model_id: int, what: str) -> int:
    out = C.c_int64()
    rc = fn(pool.handle, model_id, C.byref(out))
    if rc != MUX_OK:
        raise MuxError(rc, what)
    return out.value


def mux_pool_get_quota(pool: Pool, model_id: int) -> int:
    return _read_i64(load().mux_pool_get_quota, pool, model_id, "mux_pool_get_quota")


def mux_pool_peak_used(pool: Pool, model_id: int) -> int:
    return _read_i64(load().mux_pool_peak_used, pool, model_id, "mux_pool_peak_used")


def mux_pool_init_quotas(pool: Pool, weights) -> int:
    w = np.ascontiguousarray(weights, dtype=np.float64)
    return load().mux_pool_init_quotas(pool.handle, w.size, w.ctypes.data)


def mux_pool_adapt_quotas(pool: Pool, n_models: int, low: float, high: float, step: float):
    """Returns (status, blocks of quota moved)."""
    moved = C.c_int64(-1)
    rc = load().mux_pool_adapt_quotas(pool.handle, n_models, low, high, step, C.byref(moved))
    return rc, moved.value


def mux_alloc_blocks_status(pool: Pool, model_id: int, n: int, out: Optional[np.ndarray] = None):
    """Returns (status, ids); ids is the filled array when status == MUX_OK, else None."""
    if out is None:
        out = np.full(max(n, 0), -7, dtype=np.int32)
    assert out.dtype == np.int32 and out.size >= n and out.flags.c_contiguous
    rc = load().mux_alloc_blocks(pool.handle, model_id, n, out.ctypes.data)
    return rc, (out if rc == MUX_OK else None)


def mux_alloc_blocks(pool: Pool, model_id: int, n: int, out: Optional[np.ndarray] = None) -> np.ndarray:
    rc, ids = mux_alloc_blocks_status(pool, model_id, n, out)
    _check(rc, "mux_alloc_blocks")
    return ids


def mux_free_blocks_status(pool: Pool, model_id: int, ids) -> int:
    ids = _host_ids(ids)
    return load().mux_free_blocks(pool.handle, model_id, ids.size, ids.ctypes.data)


def mux_free_blocks(pool: Pool, model_id: int, ids) -> None:
    _check(mux_free_blocks_status(pool, model_id, ids), "mux_free_blocks")


def mux_kv_append(pool: Pool, k_new: torch.Tensor, v_new: torch.Tensor, tok_seq: torch.Tensor, tok_pos: torch.Tensor,
                  block_tables: torch.Tensor, stream=None) -> None:
    n_tokens, n_kv, d = k_new.shape
    n_seqs, n_kv2, max_blocks = block_tables.shape
    if d != pool.head_dim or n_kv != n_kv2 or v_new.shape != k_new.shape or tok_seq.numel() != n_tokens or tok_pos.numel() != n_tokens:
        raise MuxError(MUX_ERR_INVALID, "mux_kv_append")
    rc = load().mux_kv_append(_device_pool(pool), _dev(k_new, pool.torch_dtype), _dev(v_new, pool.torch_dtype),
                              _dev(tok_seq, torch.int32), _dev(tok_pos, torch.int32), _dev(block_tables, torch.int32),
                              n_tokens, n_seqs, n_kv, max_blocks, _stream(stream))
    _check(rc, "mux_kv_append")


def mux_decode_workspace_bytes(pool: Pool, n_seqs: int, n_q_heads: int, n_kv_heads: int, max_ctx_len: int) -> int:
    return load().mux_decode_workspace_bytes(pool.handle, n_seqs, n_q_heads, n_kv_heads, max_ctx_len)


def mux_decode_workspace_bound(pool: Pool, max_seqs: int, n_q_heads: int, n_kv_heads: int, max_ctx_len: int) -> int:
    return load().mux_decode_workspace_bound(pool.handle, max_seqs, n_q_heads, n_kv_heads, max_ctx_len)


def mux_prefill_workspace_bound(pool: Pool, max_total_q: int, max_ctx_len: int, n_q_heads: int, n_kv_heads: int) -> int:
    return load().mux_prefill_workspace_bound(pool.handle, max_total_q, max_ctx_len, n_q_heads, n_kv_heads)


def mux_decode_attn(pool: Pool, out: torch.Tensor, q: torch.Tensor, block_tables: torch.Tensor, ctx_lens: torch.Tensor,
                    max_ctx_len: int, scale: float, workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    n_seqs, n_q, d = q.shape
    n_seqs2, n_kv, max_blocks = block_tables.shape
    if d != pool.head_dim or n_seqs2 != n_seqs or out.shape != q.shape or ctx_lens.numel() != n_seqs:
        raise MuxError(MUX_ERR_INVALID, "mux_decode_attn")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().mux_decode_attn(_device_pool(pool), _dev(out, pool.torch_dtype), _dev(q, pool.torch_dtype),
                                _dev(block_tables, torch.int32), _dev(ctx_lens, torch.int32), n_seqs, n_q, n_kv,
                                max_blocks, max_ctx_len, scale, _dev(workspace), ws_bytes, _stream(stream))
    _check(rc, "mux_decode_attn")


def mux_decode_attn_static(pool: Pool, out: torch.Tensor, q: torch.Tensor, block_tables: torch.Tensor,
                           ctx_lens: torch.Tensor, max_ctx_len: int, scale: float, stream=None) -> None:
    n_seqs, n_q, d = q.shape
    n_seqs2, n_kv, max_blocks = block_tables.shape
    if d != pool.head_dim or n_seqs2 != n_seqs or out.shape != q.shape or ctx_lens.numel() != n_seqs:
        raise MuxError(MUX_ERR_INVALID, "mux_decode_attn_static")
    rc = load().mux_decode_attn_static(_device_pool(pool), _dev(out, pool.torch_dtype), _dev(q, pool.torch_dtype),
                                       _dev(block_tables, torch.int32), _dev(ctx_lens, torch.int32), n_seqs, n_q, n_kv,
                                       max_blocks, max_ctx_len, scale, _stream(stream))
    _check(rc, "mux_decode_attn_static")


def mux_decode_step_workspace_bytes(pool: Pool, n_layers: int, n_seqs: int, n_q_heads: int, n_kv_heads: int,
                                    max_ctx_len: int) -> int:
    return load().mux_decode_step_workspace_bytes(pool.handle, n_layers, n_seqs, n_q_heads, n_kv_heads, max_ctx_len)


def mux_decode_step(pool: Pool, out: torch.Tensor, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                    block_tables: torch.Tensor, ctx_lens: torch.Tensor, max_ctx_len: int, scale: float,
                    workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    """All tensors carry a leading layer dimension: q/out [layers][seqs][Hq][d], k_new/v_new
    [layers][seqs][Hkv][d], block_tables [layers][seqs][Hkv][max_blocks]; ctx_lens [seqs]."""
    n_layers, n_seqs, n_q, d = q.shape
    n_layers2, n_seqs2, n_kv, max_blocks = block_tables.shape
    if (d != pool.head_dim or (n_layers2, n_seqs2) != (n_layers, n_seqs) or out.shape != q.shape
            or k_new.shape != (n_layers, n_seqs, n_kv, d) or v_new.shape != k_new.shape or ctx_lens.numel() != n_seqs):
        raise MuxError(MUX_ERR_INVALID, "mux_decode_step")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().mux_decode_step(_device_pool(pool), _dev(out, pool.torch_dtype), _dev(q, pool.torch_dtype),
                                _dev(k_new, pool.torch_dtype), _dev(v_new, pool.torch_dtype),
                                _dev(block_tables, torch.int32), _dev(ctx_lens, torch.int32), n_layers, n_seqs, n_q, n_kv,
                                max_blocks, max_ctx_len, scale, _dev(workspace), ws_bytes, _stream(stream))
    _check(rc, "mux_decode_step")


def mux_prefill_workspace_bytes(pool: Pool, n_seqs: int, total_q: int, max_ctx_len: int, n_q_heads: int,
                                n_kv_heads: int) -> int:
    return load().mux_prefill_workspace_bytes(pool.handle, n_seqs, total_q, max_ctx_len, n_q_heads, n_kv_heads)


def mux_prefill_attn(pool: Pool, out: torch.Tensor, q: torch.Tensor, cu_q_lens: torch.Tensor, q_start: torch.Tensor,
                     block_tables: torch.Tensor, max_q_len: int, max_ctx_len: int, scale: float,
                     workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    total_q, n_q, d = q.shape
    n_seqs, n_kv, max_blocks = block_tables.shape
    if d != pool.head_dim or out.shape != q.shape or cu_q_lens.numel() != n_seqs + 1 or q_start.numel() != n_seqs:
        raise MuxError(MUX_ERR_INVALID, "mux_prefill_attn")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().mux_prefill_attn(_device_pool(pool), _dev(out, pool.torch_dtype), _dev(q, pool.torch_dtype),
                                 _dev(cu_q_lens, torch.int32), _dev(q_start, torch.int32),
                                 _dev(block_tables, torch.int32), n_seqs, total_q, max_q_len, max_ctx_len, n_q, n_kv,
                                 max_blocks, scale, _dev(workspace), ws_bytes, _stream(stream))
    _check(rc, "mux_prefill_attn")


class Scheduler:
    """mux_sched_* with the same semantics: step() runs one iteration of the scheduling loop and
    returns its jobs as dicts (kind, model, ids, slots, lens, flags as numpy arrays)."""

    def __init__(self, pool: Pool, heads, max_seqs: int, max_blocks: int, max_prefill_tokens: int,
                 adapt_period: int = 0, low: float = 0.5, high: float = 0.9, step: float = 0.5):
        self.pool = pool
        self.heads = np.ascontiguousarray(heads, dtype=np.int32)
        self.max_seqs, self.max_blocks = max_seqs, max_blocks
        cfg = SchedConfig(self.heads.size, self.heads.ctypes.data_as(C.POINTER(C.c_int32)), max_seqs, max_blocks,
                          max_prefill_tokens, adapt_period, low, high, step)
        h = C.c_void_p()
        rc = load().mux_sched_create(C.byref(h), pool.handle, C.byref(cfg))
        if rc != MUX_OK:
            raise MuxError(rc, "mux_sched_create")
        self.handle = h.value

    def close(self):
        if getattr(self, "handle", None):
            load().mux_sched_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:       # interpreter shutdown: the module's globals may already be gone
            pass

    def submit(self, model: int, request_id: int, prompt_len: int, output_len: int) -> int:
        return load().mux_sched_submit(self.handle, model, request_id, prompt_len, output_len)

    def step(self):
        n = C.c_int32()
        _check(load().mux_sched_step(self.handle, C.byref(n)), "mux_sched_step")
        return self.jobs(n.value)

    def job(self, j: int):
        """(kind, model, number of sequences) of job j of the last step."""
        kind, model, cnt = C.c_int32(), C.c_int32(), C.c_int32()
        _check(load().mux_sched_job(self.handle, j, C.byref(kind), C.byref(model), C.byref(cnt)), "mux_sched_job")
        return kind.value, model.value, cnt.value

    def jobs(self, n: int):
        """The first n jobs of the last step as dicts."""
        lib, jobs = load(), []
        for j in range(n):
            kind, model, cnt = C.c_int32(), C.c_int32(), C.c_int32()
            lib.mux_sched_job(self.handle, j, C.byref(kind), C.byref(model), C.byref(cnt))
            ids = np.zeros(cnt.value, np.int64)
            slots, lens, flags = (np.zeros(cnt.value, np.int32) for _ in range(3))
            lib.mux_sched_job_seqs(self.handle, j, ids.ctypes.data, slots.ctypes.data, lens.ctypes.data, flags.ctypes.data)
            jobs.append({"kind": kind.value, "model": model.value, "ids": ids, "slots": slots, "lens": lens, "flags": flags})
        return jobs

    def table(self, model: int) -> np.ndarray:
        """View of the scheduler's host table [max_seqs][heads][max_blocks] (not a copy)."""
        n = self.max_seqs * int(self.heads[model]) * self.max_blocks
        p = load().mux_sched_table(self.handle, model)
        return np.ctypeslib.as_array(p, shape=(n,)).reshape(self.max_seqs, int(self.heads[model]), self.max_blocks)

    def counts(self, model: int):
        c = np.zeros(5, np.int64)
        load().mux_sched_counts(self.handle, model, c.ctypes.data)
        return tuple(int(x) for x in c)


class Runner:
    """mux_runner_*: launches the scheduler's jobs on the GPU (one stream per model, or None for
    the current stream for all).  The tensors passed to launch() must stay alive and untouched
    until the work has finished on the model's stream."""

    def __init__(self, sched: Scheduler, n_q_heads, streams=None, n_layers=None):
        self.sched = sched
        self.n_q_heads = np.ascontiguousarray(n_q_heads, dtype=np.int32)
        self.n_layers = np.ascontiguousarray(n_layers if n_layers is not None else np.ones(sched.heads.size), dtype=np.int32)
        if self.n_q_heads.size != sched.heads.size or self.n_layers.size != sched.heads.size:
            raise ValueError("one query-head count and one layer count per model")
        self.streams = list(streams) if streams is not None else [torch.cuda.current_stream()] * sched.heads.size
        handles = (C.c_void_p * len(self.streams))(*[s.cuda_stream or None for s in self.streams])
        h = C.c_void_p()
        _check(load().mux_runner_create(C.byref(h), sched.pool.handle, sched.handle, self.n_q_heads.ctypes.data,
                                        self.n_layers.ctypes.data, handles), "mux_runner_create")
        self.handle = h.value

    def close(self):
        if getattr(self, "handle", None):
            load().mux_runner_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:       # interpreter shutdown: the module's globals may already be gone
            pass

    def step(self) -> int:
        """One scheduler iteration (plus stream ordering when blocks changed hands); number of jobs."""
        n = C.c_int32()
        _check(load().mux_runner_step(self.handle, C.byref(n)), "mux_runner_step")
        return n.value

    def launch(self, job: int, out: torch.Tensor, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor, scale: float) -> None:
        _check(load().mux_runner_launch(self.handle, job, _dev(out), _dev(q), _dev(k_new), _dev(v_new), scale), "mux_runner_launch")

    def launch_layer(self, job: int, layer: int, out: torch.Tensor, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                     scale: float) -> None:
        _check(load().mux_runner_launch_layer(self.handle, job, layer, _dev(out), _dev(q), _dev(k_new), _dev(v_new), scale),
               "mux_runner_launch_layer")

    def set_buffers(self, model: int, prefill, decode, scale: float) -> None:
        """prefill, decode = (out, q, k_new, v_new) tensors the model's jobs use from now on (kept alive here)."""
        self._buffers = getattr(self, "_buffers", {})
        self._buffers[model] = (tuple(prefill), tuple(decode))
        _check(load().mux_runner_set_buffers(self.handle, model, *[_dev(t) for t in prefill], *[_dev(t) for t in decode], scale),
               "mux_runner_set_buffers")

    def run_step(self) -> int:
        """step() and launch() of every job with the registered buffers; number of jobs."""
        n = C.c_int32()
        _check(load().mux_runner_run_step(self.handle, C.byref(n)), "mux_runner_run_step")
        return n.value

    def counts(self):
        """(jobs launched, sequences in them = output tokens produced)."""
        c = np.zeros(2, np.int64)
        _check(load().mux_runner_counts(self.handle, c.ctypes.data), "mux_runner_counts")
        return int(c[0]), int(c[1])

    def synchronize(self) -> None:
        _check(load().mux_runner_synchronize(self.handle), "mux_runner_synchronize")

    def read_table(self, model: int) -> np.ndarray:
        """Host copy of the runner's device table of a model, [layers][max_seqs][KV heads of a layer][max_blocks]."""
        layers = int(self.n_layers[model])
        host = np.empty((layers, self.sched.max_seqs, int(self.sched.heads[model]) // layers, self.sched.max_blocks), np.int32)
        _check(load().mux_runner_read_table(self.handle, model, host.ctypes.data), "mux_runner_read_table")
        return host


def mux_device_cu_count() -> int:
    n = C.c_int32()
    _check(load().mux_device_cu_count(C.byref(n)), "mux_device_cu_count")
    return n.value


class MaskedStream:
    """A HIP stream restricted to the compute units in `cus` (mux_stream_create_masked), wrapped
    as a torch stream (`.stream`) so that it can be passed wherever the binding takes one."""

    def __init__(self, cus, device="cuda"):
        cus = sorted(set(int(c) for c in cus))
        words = np.zeros(max(cus) // 32 + 1 if cus else 1, dtype=np.uint32)
        for c in cus:
            words[c // 32] |= np.uint32(1 << (c % 32))
        h = C.c_void_p()
        _check(load().mux_stream_create_masked(C.byref(h), words.ctypes.data, words.size), "mux_stream_create_masked")
        self.handle, self.cus = h.value, cus
        self.stream = torch.cuda.ExternalStream(self.handle, device=device)

    def close(self):
        if getattr(self, "handle", None):
            load().mux_stream_destroy(self.handle)
            self.handle = None


def mux_probe_stream_read(buf: torch.Tensor, sink: torch.Tensor, workgroups: int, stream=None) -> None:
    _check(load().mux_probe_stream_read(_dev(buf), buf.numel() * buf.element_size(), _dev(sink), workgroups, _stream(stream)),
           "mux_probe_stream_read")


def mux_probe_mfma(sink: torch.Tensor, workgroups: int, iters: int, stream=None) -> float:
    """Enqueues the probe; returns the floating-point operations of the launch."""
    flops = C.c_double()
    _check(load().mux_probe_mfma(_dev(sink), workgroups, iters, C.byref(flops), _stream(stream)), "mux_probe_mfma")
    return flops.value


def mux_estimate_tpt(batch, t_prefill, t_decode, gen_len, m: int, rate_cap: float) -> float:
    arrs = [np.ascontiguousarray(a, dtype=np.float64) for a in (batch, t_prefill, t_decode, gen_len)]
    n = arrs[0].size
    if any(a.size != n for a in arrs):
        raise MuxError(MUX_ERR_INVALID, "mux_estimate_tpt")
    return load().mux_estimate_tpt(n, *[a.ctypes.data for a in arrs], m, rate_cap)


def mux_find_batch_size(rate: float, max_batch: int, p0: float, p1: float, d0: float, d1: float, gen_len: float,
                        other_prefill: float) -> int:
    return load().mux_find_batch_size(rate, max_batch, p0, p1, d0, d1, gen_len, other_prefill)
