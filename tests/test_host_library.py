"""CPU-only checks of the library: every symbol the header declares is exported, the block
manager (Section 3.4, Implementation: request blocks, keep them, release at request end)
agrees call by call with the oracle's, and argument errors are reported without touching a
GPU.  No kernel is launched here.
"""
import ctypes as C
import os
import re

import numpy as np
import pytest
import torch

from oracle import mux_oracle as orc
from paper_2404_02015_amd import binding as mx
from paper_2404_02015_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def host_pool(num_blocks, block_size=16, head_dim=128, dtype=mx.MUX_BF16, order=None):
    elem = 2 if dtype == mx.MUX_BF16 else 4
    # the block manager never touches the memory: a small host buffer stands in for it and
    # the byte count is given as if it were the full pool
    kv = torch.empty(64, dtype=torch.uint8)
    h = C.c_void_p()
    o = None if order is None else np.ascontiguousarray(order, dtype=np.int32)
    rc = mx.load().mux_pool_create(C.byref(h), kv.data_ptr(), num_blocks * 2 * block_size * head_dim * elem, num_blocks,
                                   block_size, head_dim, dtype, None if o is None else o.ctypes.data)
    if rc != 0:
        raise mx.MuxError(rc, "mux_pool_create")
    return mx.Pool(h.value, kv, num_blocks, block_size, head_dim, dtype)


def test_every_declared_symbol_is_exported():
    import glob

    headers = sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))
    assert [os.path.basename(h) for h in headers] == ["mux.h", "mux_probes.h"]
    declared = []
    for h in headers:
        declared += re.findall(r"MUX_API\s+[\w\s\*]+?\b(mux_\w+)\s*\(", open(h).read())
    assert len(declared) >= 13 and set(declared) == set(mx.EXPORTS) and len(declared) == len(set(declared))
    # the measurement probes live in a header of their own: the product boundary is mux.h
    product = re.findall(r"MUX_API\s+[\w\s\*]+?\b(mux_\w+)\s*\(", open(headers[0]).read())
    assert not [n for n in product if n.startswith("mux_probe")]
    lib = mx.load()
    for name in declared:
        assert getattr(lib, name) is not None
    for name in ("mux_pool_create", "mux_alloc_blocks", "mux_free_blocks", "mux_kv_append", "mux_decode_attn",
                 "mux_prefill_attn"):
        assert name in declared


def test_status_strings():
    assert mx.status_string(0) == "MUX_OK" and mx.status_string(-2) == "MUX_ERR_NOMEM"
    assert mx.status_string(-5) == "MUX_ERR_UNSUPPORTED" and "UNKNOWN" in mx.status_string(-99)


def test_allocator_hand_example_and_errors():
    p = host_pool(8)
    assert list(mx.mux_alloc_blocks(p, 0, 3)) == [0, 1, 2]
    mx.mux_free_blocks(p, 0, [1])
    assert list(mx.mux_alloc_blocks(p, 0, 2)) == [1, 3]
    mx.mux_free_blocks(p, 0, [0, 3])
    assert list(mx.mux_alloc_blocks(p, 0, 1)) == [3]
    assert mx.mux_pool_num_free(p) == 5 and mx.mux_pool_num_used(p, 0) == 3
    out = np.full(8, -7, dtype=np.int32)
    rc, ids = mx.mux_alloc_blocks_status(p, 1, 6, out)
    assert rc == mx.MUX_ERR_NOMEM and ids is None and (out == -7).all() and mx.mux_pool_num_free(p) == 5
    assert mx.mux_free_blocks_status(p, 0, [1, 1]) == mx.MUX_ERR_INVALID
    assert mx.mux_free_blocks_status(p, 0, [0]) == mx.MUX_ERR_INVALID       # already free
    assert mx.mux_free_blocks_status(p, 1, [1]) == mx.MUX_ERR_INVALID       # other model's
    assert mx.mux_free_blocks_status(p, 0, [1, 8]) == mx.MUX_ERR_INVALID    # out of range
    assert mx.mux_free_blocks_status(p, 0, [-1]) == mx.MUX_ERR_INVALID
    assert mx.mux_free_blocks_status(p, 4000, [1]) == mx.MUX_ERR_INVALID    # model id out of range
    assert mx.mux_pool_num_used(p, 0) == 3 and mx.mux_pool_num_free(p) == 5
    assert mx.mux_alloc_blocks_status(p, 0, -1)[0] == mx.MUX_ERR_INVALID
    assert mx.mux_alloc_blocks_status(p, 0, 0)[0] == mx.MUX_OK


def test_pool_create_argument_checks():
    with pytest.raises(mx.MuxError) as e:
        host_pool(4, order=[0, 1, 1, 2])
    assert e.value.status == mx.MUX_ERR_INVALID
    for kw in (dict(head_dim=96), dict(block_size=512), dict(dtype=7)):
        with pytest.raises(mx.MuxError) as e:
            host_pool(4, **kw)
        assert e.value.status == mx.MUX_ERR_UNSUPPORTED
    # a buffer smaller than the pool is refused
    kv = torch.empty(1024, dtype=torch.uint8)
    with pytest.raises(mx.MuxError):
        mx.mux_pool_create(kv, 8, 16, 128)
    p = host_pool(4, order=[3, 0, 2, 1])
    assert list(mx.mux_alloc_blocks(p, 0, 4)) == [3, 0, 2, 1]


def test_library_and_oracle_allocators_agree_under_churn():
    n_blocks = 6000
    rng = np.random.Generator(np.random.PCG64(7))
    order = wl.placement_order(rng, n_blocks)
    lib, ora = host_pool(n_blocks, order=order), orc.OraclePool(n_blocks, 16, 128, init_free_order=order)
    stats = {"nomem": 0}

    def alloc(m, n):
        rc_l, ids_l = mx.mux_alloc_blocks_status(lib, m, n)
        rc_o, ids_o = ora.alloc_status(m, n)
        assert rc_l == rc_o
        if rc_l != 0:
            stats["nomem"] += 1
            return None
        assert np.array_equal(ids_l, ids_o)
        return ids_l

    def free(m, ids):
        assert mx.mux_free_blocks_status(lib, m, ids) == ora.free_status(m, ids) == 0
        assert mx.mux_pool_num_free(lib) == ora.num_free()

    wl.run_churn(rng, 3000, 500, alloc, free)
    assert stats["nomem"] > 0
    assert mx.mux_pool_num_free(lib) == ora.num_free() == n_blocks
    # after the churn the free lists are in the same (scrambled) order
    assert np.array_equal(mx.mux_alloc_blocks(lib, 0, n_blocks), ora.alloc(0, n_blocks))


def test_config2_named_pool_runs_out_identically():
    """The second configuration names a 200 000-block pool, less than its sequences need: both
    block managers must fail at the same call and stay unchanged."""
    w = wl.config(2)
    n_blocks = 200000
    order = wl.placement_order(w.rng(), n_blocks)
    lib, ora = host_pool(n_blocks, order=order), orc.OraclePool(n_blocks, 16, 128, init_free_order=order)
    failed_at = None
    for job in w.jobs:
        for s, L in enumerate(job.lens):
            n = int((L + 15) // 16) * job.shape.n_kv_heads
            rc_l, ids_l = mx.mux_alloc_blocks_status(lib, job.model_id, n)
            rc_o, ids_o = ora.alloc_status(job.model_id, n)
            assert rc_l == rc_o
            if rc_l != 0:
                assert rc_l == mx.MUX_ERR_NOMEM
                failed_at = (job.model_id, s, mx.mux_pool_num_free(lib))
                break
            assert np.array_equal(ids_l, ids_o)
        if failed_at:
            break
    assert failed_at is not None and failed_at[2] == ora.num_free() and failed_at[2] < n
    assert w.demand_blocks() > n_blocks


def test_kernel_calls_reject_bad_host_arguments_before_launching():
    p = host_pool(64)
    lib = mx.load()
    h = p.handle
    fake = 4096  # never dereferenced: every call below fails its host-side checks first
    big = 1 << 30
    assert lib.mux_decode_attn(h, fake, fake, fake, fake, 2, 6, 4, 4, 64, 1.0, fake, big, None) == mx.MUX_ERR_INVALID  # 6 % 4
    assert lib.mux_decode_attn(h, fake, fake, fake, fake, 2, 4, 4, 4, 65, 1.0, fake, big, None) == mx.MUX_ERR_INVALID  # hint > table
    assert lib.mux_decode_attn(h, fake + 2, fake, fake, fake, 2, 4, 4, 4, 64, 1.0, fake, big, None) == mx.MUX_ERR_INVALID  # alignment
    assert lib.mux_decode_attn(h, None, fake, fake, fake, 2, 4, 4, 4, 64, 1.0, fake, big, None) == mx.MUX_ERR_INVALID
    assert lib.mux_decode_attn(h, fake, fake, fake, fake, 0, 4, 4, 4, 64, 1.0, None, 0, None) == mx.MUX_OK           # empty batch
    # every decode call needs its workspace (work list, and partial results for long contexts)
    need = lib.mux_decode_workspace_bytes(h, 2, 4, 4, 4096)
    assert need > 0
    assert lib.mux_decode_attn(h, fake, fake, fake, fake, 2, 4, 4, 256, 4096, 1.0, None, 0, None) == mx.MUX_ERR_INVALID
    assert lib.mux_decode_attn(h, fake, fake, fake, fake, 2, 4, 4, 256, 4096, 1.0, fake, need - 1, None) == mx.MUX_ERR_INVALID
    assert lib.mux_decode_attn(h, fake, fake, fake, fake, 2, 4, 4, 256, 4096, 1.0, fake + 4, need, None) == mx.MUX_ERR_INVALID
    assert lib.mux_decode_step(h, fake, fake, fake, fake, fake, fake, 2, 2, 6, 4, 4, 64, 1.0, fake, big, None) == mx.MUX_ERR_INVALID
    assert lib.mux_decode_step(h, fake, fake, None, fake, fake, fake, 2, 2, 4, 4, 4, 64, 1.0, fake, big, None) == mx.MUX_ERR_INVALID
    assert lib.mux_decode_step(h, fake, fake, fake, fake, fake, fake, 0, 2, 4, 4, 4, 64, 1.0, None, 0, None) == mx.MUX_OK
    assert lib.mux_kv_append(h, fake, fake, fake, fake, fake, -1, 1, 4, 4, None) == mx.MUX_ERR_INVALID
    assert lib.mux_kv_append(h, fake, fake, fake, fake, fake, 0, 1, 4, 4, None) == mx.MUX_OK
    assert lib.mux_kv_append(h, fake + 8, fake, fake, fake, fake, 3, 1, 4, 4, None) == mx.MUX_ERR_INVALID
    assert lib.mux_prefill_attn(h, fake, fake, fake, fake, fake, 1, 8, 8, 4, 4, 4, 4, 1.0, None, 0, None) == mx.MUX_ERR_INVALID  # q longer than ctx
    assert lib.mux_prefill_attn(h, fake, fake, fake, fake, fake, 1, 8, 8, 8, 5, 4, 4, 1.0, None, 0, None) == mx.MUX_ERR_INVALID  # 5 % 4
    assert lib.mux_prefill_attn(h, fake, fake, fake, fake, fake, 0, 0, 0, 0, 4, 4, 4, 1.0, None, 0, None) == mx.MUX_OK
    # the Python layer refuses to launch kernels on a host pool
    with pytest.raises(ValueError):
        mx.mux_kv_append(p, torch.zeros(1, 4, 128, dtype=torch.bfloat16), torch.zeros(1, 4, 128, dtype=torch.bfloat16),
                         torch.zeros(1, dtype=torch.int32), torch.zeros(1, dtype=torch.int32),
                         torch.zeros(1, 4, 4, dtype=torch.int32))


def test_decode_plan_workspace_is_monotone_and_bounded():
    p = host_pool(64)
    lib = mx.load()
    assert 0 < lib.mux_decode_workspace_bytes(p.handle, 4096, 32, 32, 16) <= 16 + 4096 * 8   # one span: only the work list
    prev = 0
    for ctx in (1024, 4096, 16384):
        b = lib.mux_decode_workspace_bytes(p.handle, 64, 32, 32, ctx)
        assert b >= prev and b < 64 * 32 * (ctx // 16 + 4) * 130 * 4
        prev = b


def test_masked_stream_argument_checks_need_no_gpu():
    lib = mx.load()
    import ctypes as C
    h = C.c_void_p()
    words = np.zeros(2, dtype=np.uint32)
    assert lib.mux_stream_create_masked(C.byref(h), words.ctypes.data, 2) == mx.MUX_ERR_INVALID     # no unit enabled
    words[0] = 0xFF
    assert lib.mux_stream_create_masked(None, words.ctypes.data, 2) == mx.MUX_ERR_INVALID
    assert lib.mux_stream_create_masked(C.byref(h), None, 2) == mx.MUX_ERR_INVALID
    assert lib.mux_stream_create_masked(C.byref(h), words.ctypes.data, 0) == mx.MUX_ERR_INVALID
    assert lib.mux_stream_create_masked(C.byref(h), words.ctypes.data, 65) == mx.MUX_ERR_INVALID
    assert lib.mux_stream_destroy(None) == mx.MUX_ERR_INVALID
    assert lib.mux_device_cu_count(None) == mx.MUX_ERR_INVALID
    assert h.value is None


def test_probe_argument_checks_need_no_gpu():
    lib = mx.load()
    fake = 4096
    assert lib.mux_probe_stream_read(None, 1 << 20, fake, 64, None) == mx.MUX_ERR_INVALID
    assert lib.mux_probe_stream_read(fake, 1 << 20, None, 64, None) == mx.MUX_ERR_INVALID
    assert lib.mux_probe_stream_read(fake, 100, fake, 64, None) == mx.MUX_ERR_INVALID          # less than one chunk
    assert lib.mux_probe_stream_read(fake + 4, 1 << 20, fake, 64, None) == mx.MUX_ERR_INVALID  # alignment
    assert lib.mux_probe_stream_read(fake, 1 << 20, fake, 0, None) == mx.MUX_ERR_INVALID
    assert lib.mux_probe_mfma(None, 4, 4, None, None) == mx.MUX_ERR_INVALID
    assert lib.mux_probe_mfma(fake, 0, 4, None, None) == mx.MUX_ERR_INVALID
    assert lib.mux_probe_mfma(fake, 4, 0, None, None) == mx.MUX_ERR_INVALID


def test_block_manager_is_safe_from_several_host_threads():
    """The header allows pool calls from several host threads (one per colocated model): eight
    threads allocate and free concurrently on one pool (ctypes drops the interpreter lock during
    the calls).  No id may ever be held twice, counters must add up, foreign frees must fail."""
    import threading

    n_blocks, n_threads, ops = 4096, 8, 3000
    p = host_pool(n_blocks)
    lib = mx.load()
    held = [[] for _ in range(n_threads)]          # per thread: arrays of ids it holds
    errors = []
    start = threading.Barrier(n_threads)

    def worker(t):
        rng = np.random.default_rng(1000 + t)
        ids = np.zeros(64, np.int32)
        start.wait()
        for _ in range(ops):
            if held[t] and rng.random() < 0.5:
                mine = held[t].pop(int(rng.integers(len(held[t]))))
                if lib.mux_free_blocks(p.handle, t, mine.size, mine.ctypes.data) != 0:
                    errors.append("thread %d: freeing its own ids failed" % t)
            else:
                n = int(rng.integers(1, 65))
                rc = lib.mux_alloc_blocks(p.handle, t, n, ids.ctypes.data)
                if rc == 0:
                    held[t].append(ids[:n].copy())
                elif rc != mx.MUX_ERR_NOMEM:
                    errors.append("thread %d: alloc returned %d" % (t, rc))

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(n_threads)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors, errors[:3]
    all_ids = np.concatenate([a for h in held for a in h]) if any(held) else np.zeros(0, np.int32)
    assert all_ids.size == np.unique(all_ids).size and (all_ids >= 0).all() and (all_ids < n_blocks).all()
    for t in range(n_threads):
        assert mx.mux_pool_num_used(p, t) == sum(a.size for a in held[t])
    assert mx.mux_pool_num_free(p) == n_blocks - all_ids.size
    # an id held by thread 0's model cannot be freed on behalf of model 1
    if held[0]:
        assert lib.mux_free_blocks(p.handle, 1, 1, held[0][0][:1].ctypes.data) == mx.MUX_ERR_INVALID
    for t in range(n_threads):
        for a in held[t]:
            assert lib.mux_free_blocks(p.handle, t, a.size, a.ctypes.data) == 0
    assert mx.mux_pool_num_free(p) == n_blocks


def test_decode_plan_splits_only_where_whole_rows_cannot_fill_the_gpu():
    """Host-side span planning, seen through the workspace size (a plan without a split needs only
    the work list): a few very long rows are split into spans, batches that already hold enough
    whole rows are not, and contexts longer than one span (4 096 tokens) always are."""
    p = host_pool(64)
    lib = mx.load()

    def is_split(n_seqs, hq, hkv, ctx):
        return lib.mux_decode_workspace_bytes(p.handle, n_seqs, hq, hkv, ctx) > 16 + n_seqs * 8 + 16

    assert is_split(2, 32, 32, 4000) and is_split(1, 8, 1, 4096) and is_split(2, 2, 2, 4000)
    assert not is_split(8, 32, 32, 2048) and not is_split(64, 32, 32, 2048) and not is_split(16, 32, 32, 512)
    assert not is_split(128, 64, 8, 2048) and not is_split(50, 64, 8, 512)
    assert is_split(8, 32, 32, 8192) and is_split(128, 64, 8, 4097)
    assert not is_split(4096, 32, 32, 16)


def test_workspace_bounds_cover_every_smaller_call():
    """A runner or engine that allocates its scratch once must size it for the worst call, which
    is not the largest one: few long rows are cut into many spans.  The bound functions must cover
    every (rows, context) below their arguments - checked by a full sweep on a small range and at
    sampled points on a large one - and be attained by some call."""
    for dtype, B, hq, hkv in ((mx.MUX_FP32, 16, 8, 1), (mx.MUX_BF16, 12, 4, 4), (mx.MUX_BF16, 16, 32, 32), (mx.MUX_BF16, 16, 64, 8)):
        pool = host_pool(64, B, 128, dtype)
        max_rows, max_ctx = 40, 40 * B
        bound = mx.mux_decode_workspace_bound(pool, max_rows, hq, hkv, max_ctx)
        every = [mx.mux_decode_workspace_bytes(pool, r, hq, hkv, c) for r in range(1, max_rows + 1) for c in range(1, max_ctx + 1, 3)]
        assert max(every) == bound
        assert bound >= mx.mux_decode_workspace_bytes(pool, max_rows, hq, hkv, max_ctx)
    # a prefill job of the generic path (fp32 pool): 1 031 rows behind a 1 024-token context need far more
    # scratch than the largest job a scheduler with a 4 096-token budget and 256-block tables can form
    pool = host_pool(64, 16, 128, mx.MUX_FP32)
    largest = mx.mux_prefill_workspace_bytes(pool, 8, 4096, 4096, 8, 1)
    small = mx.mux_prefill_workspace_bytes(pool, 2, 1031, 1024, 8, 1)
    bound = mx.mux_prefill_workspace_bound(pool, 4096, 4096, 8, 1)
    assert small > largest and bound >= small
    rng = np.random.default_rng(3)
    for _ in range(3000):
        rows, ctx = int(rng.integers(1, 4097)), int(rng.integers(1, 4097))
        assert mx.mux_prefill_workspace_bytes(pool, 1, rows, ctx, 8, 1) <= bound
    # pools that run prefill on the matrix cores need no scratch at all
    assert mx.mux_prefill_workspace_bound(host_pool(64, 16, 128, mx.MUX_BF16), 4096, 4096, 8, 1) == 0
    assert mx.mux_decode_workspace_bound(pool, 0, 8, 1, 16) == 0 and mx.mux_decode_workspace_bound(pool, 4, 8, 3, 16) == 0


def test_static_scratch_call_refuses_oversized_launches_on_the_host():
    """mux_decode_attn_static checks the launch against its fixed scratch before it touches the GPU."""
    pool = host_pool(64, 16, 128, mx.MUX_BF16)
    n_seqs, n_q, n_kv, max_blocks = 4096, 32, 32, 1024
    assert mx.mux_decode_workspace_bytes(pool, n_seqs, n_q, n_kv, max_blocks * 16) > mx.MUX_STATIC_SCRATCH_BYTES
    buf = torch.zeros(64, dtype=torch.uint8)
    rc = mx.load().mux_decode_attn_static(pool.handle, buf.data_ptr(), buf.data_ptr(), buf.data_ptr(), buf.data_ptr(),
                                          n_seqs, n_q, n_kv, max_blocks, max_blocks * 16, 1.0, None)
    assert rc == mx.MUX_ERR_TOO_LARGE and mx.status_string(rc) == "MUX_ERR_TOO_LARGE"
    assert mx.load().mux_decode_attn_static(pool.handle, buf.data_ptr(), buf.data_ptr(), buf.data_ptr(), buf.data_ptr(),
                                            4, 6, 4, 8, 64, 1.0, None) == mx.MUX_ERR_INVALID
    header = open(os.path.join(ROOT, "include", "mux.h")).read()
    assert "#define MUX_STATIC_SCRATCH_BYTES (32 * 1024 * 1024)" in header and mx.MUX_STATIC_SCRATCH_BYTES == 32 * 1024 * 1024
