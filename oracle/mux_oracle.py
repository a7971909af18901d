"""ctypes wrapper around the CPU oracle (oracle/mux_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  It never imports the GPU package and the GPU package
never imports it.

Arrays are numpy: bf16 data travels as uint16 bit patterns, fp32 as float32, ids and
lengths as int32.  Outputs of the attention calls are float32.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mux_oracle.c")
_SRCS = [_SRC, os.path.join(_HERE, "adbs_oracle.c")]
_LIB = os.path.join(_HERE, "libmux_oracle.so")

OK, ERR_INVALID, ERR_NOMEM, ERR_QUOTA, ERR_UNSUPPORTED = 0, -1, -2, -3, -5
BF16, FP32 = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 and OpenMP; returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(os.path.getmtime(f) for f in _SRCS)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC", "-o", tmp] + _SRCS + ["-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        i32p, vp, i64, i32, f32 = C.POINTER(C.c_int32), C.c_void_p, C.c_int64, C.c_int32, C.c_float
        L.oracle_pool_create.argtypes = [C.POINTER(vp), i64, i32, i32, i32, vp]
        L.oracle_pool_destroy.argtypes = [vp]
        L.oracle_pool_destroy.restype = None
        L.oracle_pool_num_free.argtypes = [vp]
        L.oracle_pool_num_free.restype = i64
        L.oracle_pool_num_used.argtypes = [vp, i32]
        L.oracle_pool_num_used.restype = i64
        L.oracle_alloc_blocks.argtypes = [vp, i32, i64, vp]
        L.oracle_free_blocks.argtypes = [vp, i32, i64, vp]
        L.oracle_set_quota.argtypes = [vp, i32, i64]
        L.oracle_get_quota.argtypes = [vp, i32]
        L.oracle_get_quota.restype = i64
        L.oracle_peak_used.argtypes = [vp, i32]
        L.oracle_peak_used.restype = i64
        L.oracle_init_quotas.argtypes = [vp, i32, vp]
        L.oracle_adapt_quotas.argtypes = [vp, i32, C.c_double, C.c_double, C.c_double, C.POINTER(i64)]
        L.oracle_kv_append.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32]
        L.oracle_read_row.argtypes = [vp, i32, i32, i32, vp]
        L.oracle_drop_tiles.argtypes = [vp, i64, vp]
        L.oracle_gather.argtypes = [vp, vp, i64, vp, vp]
        L.oracle_attn_row_f32.argtypes = [vp, vp, vp, i64, i32, f32, vp, vp, vp]
        L.oracle_attn_row_f32.restype = None
        L.oracle_attn_row_f64.argtypes = [vp, vp, vp, i64, i32, f32, vp, vp, vp]
        L.oracle_attn_row_f64.restype = None
        L.oracle_decode_attn.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, f32, i32]
        L.oracle_prefill_attn.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, f32, i32]
        L.oracle_decode_weights.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, f32]
        L.oracle_num_threads.restype = i32
        L.oracle_set_num_threads.argtypes = [i32]
        L.oracle_set_num_threads.restype = None
        f64 = C.c_double
        L.adbs_oracle_create.argtypes = [C.POINTER(vp), vp, i32, vp, i32, i32, i32, i32, i32, f64, f64, f64]
        L.adbs_oracle_destroy.argtypes = [vp]
        L.adbs_oracle_destroy.restype = None
        L.adbs_oracle_submit.argtypes = [vp, i32, i64, i32, i32]
        L.adbs_oracle_step.argtypes = [vp, C.POINTER(i32)]
        L.adbs_oracle_job.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
        L.adbs_oracle_job_seqs.argtypes = [vp, i32, vp, vp, vp, vp]
        L.adbs_oracle_table.argtypes = [vp, i32]
        L.adbs_oracle_table.restype = C.POINTER(i32)
        L.adbs_oracle_counts.argtypes = [vp, i32, vp]
        L.adbs_oracle_tpt.argtypes = [i32, vp, vp, vp, vp, i32, f64]
        L.adbs_oracle_tpt.restype = f64
        L.adbs_oracle_batch_size.argtypes = [f64, i64] + [f64] * 6
        L.adbs_oracle_batch_size.restype = i64
        _lib = L
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.int32)


class OracleError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__("%s failed with status %d" % (what, status))
        self.status = status


class OraclePool:
    """The oracle's own pool: block manager + sparse host copy of the K/V tiles."""

    def __init__(self, num_blocks: int, block_size: int, head_dim: int, dtype: int = BF16, init_free_order=None):
        self.num_blocks, self.block_size, self.head_dim, self.dtype = num_blocks, block_size, head_dim, dtype
        self.np_dtype = np.uint16 if dtype == BF16 else np.float32
        self._h = C.c_void_p()
        order = None if init_free_order is None else _i32(init_free_order)
        if order is not None and order.size != num_blocks:
            raise OracleError(ERR_INVALID, "oracle_pool_create")
        rc = lib().oracle_pool_create(
            C.byref(self._h), num_blocks, block_size, head_dim, dtype, None if order is None else _ptr(order)
        )
        if rc != OK:
            self._h = None
            raise OracleError(rc, "oracle_pool_create")

    def close(self):
        if getattr(self, "_h", None):
            lib().oracle_pool_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    # -- block manager -----------------------------------------------------
    def num_free(self) -> int:
        return lib().oracle_pool_num_free(self._h)

    def num_used(self, model_id: int) -> int:
        return lib().oracle_pool_num_used(self._h, model_id)

    def alloc_status(self, model_id: int, n: int):
        """Returns (status, ids); ids is None unless status == OK."""
        out = np.full(max(n, 0), -7, dtype=np.int32)
        rc = lib().oracle_alloc_blocks(self._h, model_id, n, _ptr(out))
        return rc, (out if rc == OK else None)

    def alloc(self, model_id: int, n: int) -> np.ndarray:
        rc, ids = self.alloc_status(model_id, n)
        if rc != OK:
            raise OracleError(rc, "oracle_alloc_blocks")
        return ids

    def free_status(self, model_id: int, ids) -> int:
        ids = _i32(ids)
        return lib().oracle_free_blocks(self._h, model_id, ids.size, _ptr(ids))

    def free(self, model_id: int, ids) -> None:
        rc = self.free_status(model_id, ids)
        if rc != OK:
            raise OracleError(rc, "oracle_free_blocks")

    # -- token-block quotas --------------------------------------------------
    def set_quota(self, model_id: int, max_blocks: int) -> int:
        """max_blocks = -1 removes the quota.  Returns the status."""
        return lib().oracle_set_quota(self._h, model_id, max_blocks)

    def get_quota(self, model_id: int) -> int:
        return lib().oracle_get_quota(self._h, model_id)

    def peak_used(self, model_id: int) -> int:
        return lib().oracle_peak_used(self._h, model_id)

    def init_quotas(self, weights) -> int:
        w = np.ascontiguousarray(weights, dtype=np.float64)
        return lib().oracle_init_quotas(self._h, w.size, _ptr(w))

    def adapt_quotas(self, n_models: int, low: float, high: float, step: float):
        """Returns (status, blocks moved)."""
        moved = C.c_int64(-1)
        rc = lib().oracle_adapt_quotas(self._h, n_models, low, high, step, C.byref(moved))
        return rc, moved.value

    # -- data path ---------------------------------------------------------
    def _elems(self, a) -> np.ndarray:
        a = np.ascontiguousarray(a)
        if a.dtype != self.np_dtype:
            raise TypeError("expected %s, got %s" % (self.np_dtype, a.dtype))
        return a

    def kv_append(self, k_new, v_new, tok_seq, tok_pos, block_tables) -> None:
        k_new, v_new = self._elems(k_new), self._elems(v_new)
        tok_seq, tok_pos, bt = _i32(tok_seq), _i32(tok_pos), _i32(block_tables)
        n_tokens, n_kv, d = k_new.shape
        assert d == self.head_dim and v_new.shape == k_new.shape and tok_seq.size == n_tokens == tok_pos.size
        n_seqs, n_kv2, max_blocks = bt.shape
        assert n_kv2 == n_kv
        rc = lib().oracle_kv_append(
            self._h, _ptr(k_new), _ptr(v_new), _ptr(tok_seq), _ptr(tok_pos), _ptr(bt), n_tokens, n_seqs, n_kv, max_blocks
        )
        if rc != OK:
            raise OracleError(rc, "oracle_kv_append")

    def read_row(self, block_id: int, slot: int, which: int) -> np.ndarray:
        out = np.empty(self.head_dim, dtype=self.np_dtype)
        rc = lib().oracle_read_row(self._h, block_id, slot, which, _ptr(out))
        if rc != OK:
            raise OracleError(rc, "oracle_read_row")
        return out

    def drop_tiles(self, ids) -> None:
        ids = _i32(ids)
        rc = lib().oracle_drop_tiles(self._h, ids.size, _ptr(ids))
        if rc != OK:
            raise OracleError(rc, "oracle_drop_tiles")

    def gather(self, table_row, L: int):
        """Contiguous fp32 K, V of shape [L][head_dim] for one (sequence, kv head)."""
        row = _i32(table_row)
        K = np.empty((L, self.head_dim), dtype=np.float32)
        V = np.empty((L, self.head_dim), dtype=np.float32)
        rc = lib().oracle_gather(self._h, _ptr(row), L, _ptr(K), _ptr(V))
        if rc != OK:
            raise OracleError(rc, "oracle_gather")
        return K, V

    def decode_attn(self, q, block_tables, ctx_lens, n_q_heads: int, scale: float, use_f64: bool = False) -> np.ndarray:
        q, bt, cl = self._elems(q), _i32(block_tables), _i32(ctx_lens)
        n_seqs, n_kv, max_blocks = bt.shape
        assert q.shape == (n_seqs, n_q_heads, self.head_dim) and cl.size == n_seqs
        out = np.zeros(q.shape, dtype=np.float32)
        rc = lib().oracle_decode_attn(
            self._h, _ptr(out), _ptr(q), _ptr(bt), _ptr(cl), n_seqs, n_q_heads, n_kv, max_blocks, scale, int(use_f64)
        )
        if rc != OK:
            raise OracleError(rc, "oracle_decode_attn")
        return out

    def prefill_attn(self, q, cu_q_lens, q_start, block_tables, n_q_heads: int, scale: float, use_f64: bool = False) -> np.ndarray:
        q, bt = self._elems(q), _i32(block_tables)
        cu, qs = _i32(cu_q_lens), _i32(q_start)
        n_seqs, n_kv, max_blocks = bt.shape
        assert cu.size == n_seqs + 1 and qs.size == n_seqs
        assert q.shape == (int(cu[-1]), n_q_heads, self.head_dim)
        out = np.zeros(q.shape, dtype=np.float32)
        rc = lib().oracle_prefill_attn(
            self._h, _ptr(out), _ptr(q), _ptr(cu), _ptr(qs), _ptr(bt), n_seqs, n_q_heads, n_kv, max_blocks, scale, int(use_f64)
        )
        if rc != OK:
            raise OracleError(rc, "oracle_prefill_attn")
        return out

    def decode_weights(self, q, block_tables, ctx_lens, s: int, i: int, n_q_heads: int, scale: float) -> np.ndarray:
        q, bt, cl = self._elems(q), _i32(block_tables), _i32(ctx_lens)
        n_seqs, n_kv, max_blocks = bt.shape
        w = np.zeros(int(cl[s]), dtype=np.float64)
        rc = lib().oracle_decode_weights(self._h, _ptr(w), _ptr(q), _ptr(bt), _ptr(cl), s, i, n_q_heads, n_kv, max_blocks, scale)
        if rc != OK:
            raise OracleError(rc, "oracle_decode_weights")
        return w


def attn_row(q, K, V, scale: float, use_f64: bool = False) -> np.ndarray:
    """One attention row over contiguous fp32 K, V [n][d] (no paging)."""
    q = np.ascontiguousarray(q, dtype=np.float32)
    K = np.ascontiguousarray(K, dtype=np.float32)
    V = np.ascontiguousarray(V, dtype=np.float32)
    n, d = K.shape
    out = np.zeros(d, dtype=np.float32)
    scratch = np.zeros(max(n, 1), dtype=np.float64)
    fn = lib().oracle_attn_row_f64 if use_f64 else lib().oracle_attn_row_f32
    fn(_ptr(q), _ptr(K), _ptr(V), n, d, scale, _ptr(out), None, _ptr(scratch))
    return out


def num_threads() -> int:
    return lib().oracle_num_threads()


def set_num_threads(n: int) -> None:
    lib().oracle_set_num_threads(int(n))


PREFILL, DECODE, PREEMPT = 1, 2, 3
FLAG_TABLE, FLAG_FINISHED = 1, 2


class OracleScheduler:
    """The oracle's batch scheduler (Algorithm 3) over an OraclePool.  step() runs one iteration
    and returns its jobs as dicts: kind, model, ids, slots, lens, flags (numpy arrays)."""

    def __init__(self, pool: OraclePool, heads, max_seqs: int, max_blocks: int, max_prefill_tokens: int,
                 adapt_period: int = 0, low: float = 0.5, high: float = 0.9, step: float = 0.5):
        self.pool, self.heads = pool, _i32(heads)
        self.max_seqs, self.max_blocks = max_seqs, max_blocks
        self._h = C.c_void_p()
        rc = lib().adbs_oracle_create(C.byref(self._h), pool._h, self.heads.size, _ptr(self.heads), pool.block_size,
                                      max_seqs, max_blocks, max_prefill_tokens, adapt_period, low, high, step)
        if rc != OK:
            self._h = None
            raise OracleError(rc, "adbs_oracle_create")

    def close(self):
        if getattr(self, "_h", None):
            lib().adbs_oracle_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def submit(self, model: int, req_id: int, prompt_len: int, output_len: int) -> int:
        return lib().adbs_oracle_submit(self._h, model, req_id, prompt_len, output_len)

    def step(self):
        n = C.c_int32()
        rc = lib().adbs_oracle_step(self._h, C.byref(n))
        if rc != OK:
            raise OracleError(rc, "adbs_oracle_step")
        jobs = []
        for j in range(n.value):
            kind, model, cnt = C.c_int32(), C.c_int32(), C.c_int32()
            lib().adbs_oracle_job(self._h, j, C.byref(kind), C.byref(model), C.byref(cnt))
            ids = np.zeros(cnt.value, np.int64)
            slots, lens, flags = (np.zeros(cnt.value, np.int32) for _ in range(3))
            lib().adbs_oracle_job_seqs(self._h, j, _ptr(ids), _ptr(slots), _ptr(lens), _ptr(flags))
            jobs.append({"kind": kind.value, "model": model.value, "ids": ids, "slots": slots, "lens": lens, "flags": flags})
        return jobs

    def table(self, model: int) -> np.ndarray:
        """The model's host block table [max_seqs][heads][max_blocks] (a copy)."""
        n = self.max_seqs * int(self.heads[model]) * self.max_blocks
        p = lib().adbs_oracle_table(self._h, model)
        return np.ctypeslib.as_array(p, shape=(n,)).reshape(self.max_seqs, int(self.heads[model]), self.max_blocks).copy()

    def counts(self, model: int):
        """(waiting, running, finished, preempted, quota blocks moved so far)."""
        c = np.zeros(5, np.int64)
        lib().adbs_oracle_counts(self._h, model, _ptr(c))
        return tuple(int(x) for x in c)


def estimate_tpt(batch, t_prefill, t_decode, gen_len, m: int, rate_cap: float) -> float:
    """Eq. 3 (oracle); -1 for arguments outside its domain."""
    arrs = [np.ascontiguousarray(a, dtype=np.float64) for a in (batch, t_prefill, t_decode, gen_len)]
    return lib().adbs_oracle_tpt(arrs[0].size, *[_ptr(a) for a in arrs], m, rate_cap)


def find_batch_size(rate, max_batch, p0, p1, d0, d1, gen_len, other_prefill) -> int:
    return lib().adbs_oracle_batch_size(rate, max_batch, p0, p1, d0, d1, gen_len, other_prefill)
