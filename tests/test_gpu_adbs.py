"""The batch scheduler driving the kernels on the GPU (Section 3.3, Algorithm 3 on top of the
unified KV pool of Section 3.4): every job the library's scheduler hands out is launched through
the C ABI by the engine, and mirrored - same seeded K/V/Q - into the oracle's own pool through the
oracle's own scheduler.  Jobs, tables and pool counters must be identical, every attention output
within the bf16 tolerance of the oracle's.
"""
import numpy as np
import pytest
import torch

import mux_harness as H
from oracle import mux_oracle as orc
from paper_2404_02015_amd import adbs_engine as eng
from paper_2404_02015_amd import binding as mx
from paper_2404_02015_amd import workloads as wl

pytestmark = pytest.mark.gpu


class SeededSource:
    """K/V/Q of request r of model m are N(0,1) values rounded to bf16, drawn from a generator
    seeded with (seed, m, r): a recomputed request gets the same values again."""

    def __init__(self, shapes, d, max_len, seed):
        self.shapes, self.d, self.max_len, self.seed, self.cache = shapes, d, max_len, seed, {}

    def _get(self, m, r):
        if (m, r) not in self.cache:
            s = self.shapes[m]
            base = (self.seed * 1000 + m) * 100000 + 3 * r
            self.cache[(m, r)] = tuple(wl.as_bits(wl.randn_values(base + i, (self.max_len, h, self.d))).copy()
                                       for i, h in enumerate((s.n_kv_heads, s.n_kv_heads, s.n_q_heads)))
        return self.cache[(m, r)]

    def bits(self, m, r, which, p0, p1):
        return self._get(m, r)[which][p0:p1]

    def _t(self, a):
        return torch.from_numpy(a.view(np.int16).copy()).cuda().view(torch.bfloat16)

    def kv(self, m, r, p0, p1):
        return self._t(self.bits(m, r, 0, p0, p1)), self._t(self.bits(m, r, 1, p0, p1))

    def q(self, m, r, p0, p1):
        return self._t(self.bits(m, r, 2, p0, p1))


def oracle_job_outputs(op, os_, src, shapes, job, scale):
    m, slots, lens, ids = job["model"], job["slots"], job["lens"], job["ids"]
    table = os_.table(m)
    hq = shapes[m].n_q_heads
    if job["kind"] == orc.PREFILL:
        k = np.concatenate([src.bits(m, r, 0, 0, n) for r, n in zip(ids, lens)])
        v = np.concatenate([src.bits(m, r, 1, 0, n) for r, n in zip(ids, lens)])
        q = np.concatenate([src.bits(m, r, 2, 0, n) for r, n in zip(ids, lens)])
        op.kv_append(k, v, np.repeat(slots, lens), np.concatenate([np.arange(n) for n in lens]), np.maximum(table, 0))
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        return op.prefill_attn(q, cu, np.zeros(len(lens), np.int32), np.maximum(table[slots], 0), hq, scale)
    k = np.concatenate([src.bits(m, r, 0, n - 1, n) for r, n in zip(ids, lens)])
    v = np.concatenate([src.bits(m, r, 1, n - 1, n) for r, n in zip(ids, lens)])
    q = np.concatenate([src.bits(m, r, 2, n - 1, n) for r, n in zip(ids, lens)])
    op.kv_append(k, v, slots, lens - 1, np.maximum(table, 0))
    return op.decode_attn(q, np.maximum(table[slots], 0), lens, hq, scale)


CASES = [(c, d) for c in ("roomy", "tight-quota", "preempting")
         for d in ("python", "runner", "runner-one-stream", "runner-staged", "runner-layers")]
# hundreds of short requests at once: decode jobs of more than 256 rows (the work list then comes from
# the plan kernel) whose arrays still fit the attention launch's arguments, and some that do not
CASES += [("many-slots", "runner"), ("many-slots", "runner-layers")]


@pytest.mark.parametrize("case,driver", CASES)
def test_scheduler_drives_kernels_like_the_oracle(case, driver, monkeypatch):
    print("[case] adbs %s, driver %s" % (case, driver), flush=True)
    shapes = [wl.ModelShape("a", 8, 8, 128), wl.ModelShape("b", 16, 4, 128), wl.ModelShape("c", 4, 4, 128)]
    d, B = 128, 16
    n_blocks = {"roomy": 4000, "tight-quota": 600, "preempting": 300, "many-slots": 9000}[case]
    max_seqs, max_blocks, budget = 6, 24, 256
    many = case == "many-slots"
    if many:
        shapes = [wl.ModelShape("a", 4, 2, 128), wl.ModelShape("b", 8, 2, 128), wl.ModelShape("c", 2, 2, 128)]
        max_seqs, max_blocks, budget = 300, 5, 2048
    rng = np.random.default_rng({"roomy": 1, "tight-quota": 2, "preempting": 3, "many-slots": 4}[case])
    order = wl.placement_order(rng, n_blocks)
    kv = torch.empty(n_blocks * 2 * B * d * 2, dtype=torch.uint8, device="cuda")
    kv.view(torch.int16).fill_(0x7FC1)                      # NaN pattern: a read of a never-written slot shows
    pool = mx.mux_pool_create(kv, n_blocks, B, d, mx.MUX_BF16, order)
    op = orc.OraclePool(n_blocks, B, d, init_free_order=order)
    kw = dict(adapt_period=4, low=0.5, high=0.85, step=0.5) if case == "tight-quota" else {}
    if case == "tight-quota":
        w = np.array([1.0, 3.0, 1.0]) * np.array([s.n_kv_heads for s in shapes])
        assert mx.mux_pool_init_quotas(pool, w) == 0 == op.init_quotas(w)
    src = SeededSource(shapes, d, max_blocks * B, seed=77)
    if driver == "python":
        engine = eng.Engine(pool, shapes, max_seqs, max_blocks, budget, src, **kw)
    else:
        # decode jobs send their arrays as kernel arguments when they fit; "staged" forces the pinned-memory copy instead
        monkeypatch.setenv("MUX_RUNNER_STAGE_ALWAYS", "1" if driver == "runner-staged" else "0")
        # "layers": models a and b run as 2 layers of half the heads each; the scheduler, the value source and the
        # oracle still see one wide layer (head index = layer x heads of a layer + head)
        layers = [2, 2, 1] if driver == "runner-layers" else [1, 1, 1]
        per_layer = [wl.ModelShape(s.name, s.n_q_heads // n, s.n_kv_heads // n, d) for s, n in zip(shapes, layers)]
        engine = eng.NativeEngine(pool, per_layer, max_seqs, max_blocks, budget, src, shared_stream=driver == "runner-one-stream",
                                  layers=layers, **kw)
    os_ = orc.OracleScheduler(op, [s.n_kv_heads for s in shapes], max_seqs, max_blocks, budget, **kw)
    scale = H.default_scale(d)
    rid, worst, kinds, most_rows = 0, 0.0, set(), 0
    for it in range(400):
        if it < (12 if many else 60):
            for _ in range(int(rng.poisson(90 if many else 0.7))):
                m = int(rng.integers(3))
                plen, olen = (int(rng.integers(1, 24)), int(rng.integers(20, 50))) if many else (int(rng.integers(1, 200)), int(rng.integers(1, 60)))
                engine.submit(m, rid, plen, olen)
                assert os_.submit(m, rid, plen, olen) == 0
                rid += 1
        results = engine.step()
        want_jobs = os_.step()
        assert len(results) == len(want_jobs)
        for (job, out), wj in zip(results, want_jobs):
            assert job["kind"] == wj["kind"] and job["model"] == wj["model"]
            for k in ("ids", "slots", "lens", "flags"):
                assert np.array_equal(job[k], wj[k])
            kinds.add(job["kind"])
            if job["kind"] == mx.MUX_JOB_PREEMPT:
                continue
            if job["kind"] == mx.MUX_JOB_DECODE:
                most_rows = max(most_rows, int(job["slots"].max()) + 1)
            want = oracle_job_outputs(op, os_, src, shapes, wj, scale)
            worst = max(worst, H.assert_close(out, want, "bf16", "%s job of model %d, iteration %d" % (
                "prefill" if job["kind"] == mx.MUX_JOB_PREFILL else "decode", job["model"], it)))
        for m in range(3):
            assert np.array_equal(engine.sched.table(m), os_.table(m))
            assert mx.mux_pool_num_used(pool, m) == op.num_used(m)
        if driver != "python":
            # the runner's device tables hold the blocks of every sequence that just decoded
            for wj in want_jobs:
                if wj["kind"] != orc.DECODE:
                    continue
                got_t, want_t = engine.runner.read_table(wj["model"]), os_.table(wj["model"])
                got_t = got_t.transpose(1, 0, 2, 3).reshape(want_t.shape)       # [layer][slot][head] -> [slot][layer x head]
                for slot, n in zip(wj["slots"], wj["lens"]):
                    nb = (n + B - 1) // B
                    assert np.array_equal(got_t[slot, :, :nb], want_t[slot, :, :nb])
        if it >= 60 and engine.idle():
            break
    torch.cuda.synchronize()
    assert engine.idle() and rid > 20
    engine.step(), os_.step()
    assert mx.mux_pool_num_free(pool) == n_blocks == op.num_free()
    assert {mx.MUX_JOB_PREFILL, mx.MUX_JOB_DECODE} <= kinds
    if case == "preempting":
        assert mx.MUX_JOB_PREEMPT in kinds
    if many:
        assert most_rows > 256
    print("adbs %s: %d requests, %d iterations, max abs err %.2e" % (case, rid, engine.iterations, worst), flush=True)


def test_runner_on_a_pool_outside_the_matrix_core_path():
    """Blocks of 12 tokens: prefill takes the generic path, whose scratch depends on the job (few
    rows behind a long context are cut into many spans and need far more than the largest job).
    The runner sizes its scratch once, for the worst job the scheduler can form; every job must
    launch and match the oracle.  Long prompts against a small token budget make such jobs."""
    print("[case] adbs runner, 12-token blocks (generic prefill path)", flush=True)
    shapes = [wl.ModelShape("a", 8, 2, 128), wl.ModelShape("b", 4, 4, 128)]
    d, B, n_blocks, max_seqs, max_blocks, budget = 128, 12, 3000, 5, 64, 64
    rng = np.random.default_rng(12)
    order = wl.placement_order(rng, n_blocks)
    kv = torch.empty(n_blocks * 2 * B * d * 2, dtype=torch.uint8, device="cuda")
    kv.view(torch.int16).fill_(0x7FC1)
    pool = mx.mux_pool_create(kv, n_blocks, B, d, mx.MUX_BF16, order)
    op = orc.OraclePool(n_blocks, B, d, init_free_order=order)
    # the premise: some job shape needs more scratch than the largest job
    largest = mx.mux_prefill_workspace_bytes(pool, max_seqs, max_blocks * B, max_blocks * B, 8, 2)
    assert mx.mux_prefill_workspace_bytes(pool, 1, 600, 600, 8, 2) > largest       # one 600-token prompt of model a
    assert mx.mux_prefill_workspace_bound(pool, max_blocks * B, max_blocks * B, 8, 2) > largest
    src = SeededSource(shapes, d, max_blocks * B, seed=78)
    engine = eng.NativeEngine(pool, shapes, max_seqs, max_blocks, budget, src)
    os_ = orc.OracleScheduler(op, [s.n_kv_heads for s in shapes], max_seqs, max_blocks, budget)
    scale = H.default_scale(d)
    rid, worst, longest_prefill = 0, 0.0, 0
    for it in range(200):
        if it < 16:
            arrivals = [(int(rng.integers(2)), int(rng.integers(1, 700)), int(rng.integers(1, 12))) for _ in range(int(rng.poisson(0.8)))]
            if it in (0, 9):
                arrivals.append((0, 600 + it, 3))      # the job shape that needs the most scratch
            for m, plen, olen in arrivals:
                engine.submit(m, rid, plen, olen)
                assert os_.submit(m, rid, plen, olen) == 0
                rid += 1
        results = engine.step()
        want_jobs = os_.step()
        assert len(results) == len(want_jobs)
        for (job, out), wj in zip(results, want_jobs):
            assert job["kind"] == wj["kind"] and job["model"] == wj["model"]
            for k in ("ids", "slots", "lens", "flags"):
                assert np.array_equal(job[k], wj[k])
            if job["kind"] == mx.MUX_JOB_PREEMPT:
                continue
            if job["kind"] == mx.MUX_JOB_PREFILL:
                longest_prefill = max(longest_prefill, int(job["lens"].max()))
            want = oracle_job_outputs(op, os_, src, shapes, wj, scale)
            worst = max(worst, H.assert_close(out, want, "bf16", "job of model %d, iteration %d" % (job["model"], it)))
        if it >= 16 and engine.idle():
            break
    torch.cuda.synchronize()
    assert engine.idle() and rid > 6 and longest_prefill > 300
    print("adbs, 12-token blocks: %d requests, longest prefill %d tokens, max abs err %.2e" % (rid, longest_prefill, worst), flush=True)


def test_run_step_with_registered_buffers_equals_step_plus_launch():
    """mux_runner_run_step (one call per iteration, buffers registered once) does what mux_runner_step +
    mux_runner_launch per job do: same jobs, same bytes in the pool, same outputs, bit for bit."""
    print("[case] runner run_step against step + launch", flush=True)
    shapes = [wl.ModelShape("a", 8, 8, 128), wl.ModelShape("b", 16, 4, 128)]
    d, B, n_blocks, max_seqs, max_blocks, budget = 128, 16, 500, 6, 24, 256
    order = wl.placement_order(np.random.default_rng(5), n_blocks)
    sides = []
    for _ in range(2):
        kv = torch.zeros(n_blocks * 2 * B * d * 2, dtype=torch.uint8, device="cuda")
        pool = mx.mux_pool_create(kv, n_blocks, B, d, mx.MUX_BF16, order)
        torch.manual_seed(11)                                           # both sides get the same buffer contents
        engine = eng.NativeEngine(pool, shapes, max_seqs, max_blocks, budget, None)
        sides.append((kv, pool, engine))
    (kv_a, _, a), (kv_b, _, b) = sides
    for st_a, st_b in zip(a.models, b.models):
        for name in ("k_dec", "v_dec", "q_dec", "k_pre", "v_pre", "q_pre"):
            assert torch.equal(getattr(st_a, name), getattr(st_b, name))
    rng = np.random.default_rng(6)
    rid = 0
    for it in range(400):
        if it < 40:
            for _ in range(int(rng.poisson(0.7))):
                m, plen, olen = int(rng.integers(2)), int(rng.integers(1, 200)), int(rng.integers(1, 60))
                a.submit(m, rid, plen, olen)
                b.submit(m, rid, plen, olen)
                rid += 1
        n_a = a.step()                                                  # registered buffers, one call
        n_b = b.runner.step()
        assert n_a == n_b
        for j in range(n_b):
            kind, model, _ = b.sched.job(j)
            st = b.models[model]
            if kind == mx.MUX_JOB_PREFILL:
                b.runner.launch(j, st.out_pre, st.q_pre, st.k_pre, st.v_pre, b.scale)
            elif kind == mx.MUX_JOB_DECODE:
                b.runner.launch(j, st.out_dec, st.q_dec, st.k_dec, st.v_dec, b.scale)
        a.runner.synchronize()
        b.runner.synchronize()
        for st_a, st_b in zip(a.models, b.models):
            assert torch.equal(st_a.out_dec.view(torch.int16), st_b.out_dec.view(torch.int16))
            assert torch.equal(st_a.out_pre.view(torch.int16), st_b.out_pre.view(torch.int16))
        if it >= 40 and a.idle():
            break
    assert a.idle() and b.idle() and rid > 10
    assert torch.equal(kv_a, kv_b)
    assert a.runner.counts() == b.runner.counts() and a.tokens() > rid


def test_layer_by_layer_launches_equal_the_all_layers_launch():
    """mux_runner_launch_layer, one layer at a time (as an engine with other kernels between the
    attention layers would call it), leaves the same bytes in the pool and the same outputs as
    mux_runner_launch for all layers at once."""
    print("[case] runner layer by layer against all layers at once", flush=True)
    per_layer = [wl.ModelShape("a", 4, 4, 128), wl.ModelShape("b", 8, 2, 128)]
    layers = [3, 2]
    d, B, n_blocks, max_seqs, max_blocks, budget = 128, 16, 900, 5, 12, 128
    order = wl.placement_order(np.random.default_rng(15), n_blocks)
    sides = []
    for _ in range(2):
        kv = torch.zeros(n_blocks * 2 * B * d * 2, dtype=torch.uint8, device="cuda")
        pool = mx.mux_pool_create(kv, n_blocks, B, d, mx.MUX_BF16, order)
        torch.manual_seed(21)
        sides.append((kv, pool, eng.NativeEngine(pool, per_layer, max_seqs, max_blocks, budget, None, layers=layers)))
    (kv_a, _, a), (kv_b, _, b) = sides
    rng = np.random.default_rng(16)
    rid = 0
    for it in range(300):
        if it < 30:
            for _ in range(int(rng.poisson(0.6))):
                m, plen, olen = int(rng.integers(2)), int(rng.integers(1, 120)), int(rng.integers(1, 50))
                a.submit(m, rid, plen, olen)
                b.submit(m, rid, plen, olen)
                rid += 1
        n_a = a.step()                                                  # all layers of a job in one call
        assert n_a == b.runner.step()
        for j, job in enumerate(b.sched.jobs(n_a)):
            st = b.models[job["model"]]
            if job["kind"] == mx.MUX_JOB_PREEMPT:
                continue
            for layer in range(st.layers):
                if job["kind"] == mx.MUX_JOB_PREFILL:
                    t = int(job["lens"].sum())
                    sl = slice(layer * t, (layer + 1) * t)
                    b.runner.launch_layer(j, layer, st.out_pre[sl], st.q_pre[sl], st.k_pre[sl], st.v_pre[sl], b.scale)
                else:
                    b.runner.launch_layer(j, layer, st.out_dec[layer], st.q_dec[layer], st.k_dec[layer], st.v_dec[layer], b.scale)
        a.runner.synchronize()
        b.runner.synchronize()
        for st_a, st_b in zip(a.models, b.models):
            assert torch.equal(st_a.out_dec.view(torch.int16), st_b.out_dec.view(torch.int16))
            assert torch.equal(st_a.out_pre.view(torch.int16), st_b.out_pre.view(torch.int16))
        if it >= 30 and a.idle():
            break
    assert a.idle() and b.idle() and rid > 8
    assert torch.equal(kv_a, kv_b) and a.runner.counts() == b.runner.counts()
    # a later layer of a job whose layer 0 was not launched in this iteration is refused
    b.submit(0, 10_000, 20, 3)
    assert b.runner.step() >= 1
    st = b.models[0]
    with pytest.raises(mx.MuxError):
        b.runner.launch_layer(0, 1, st.out_pre[:20], st.q_pre[:20], st.k_pre[:20], st.v_pre[:20], b.scale)
