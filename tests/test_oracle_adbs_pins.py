"""Pins of the oracle's batch scheduler (Section 3.3, Algorithm 3) against hand-worked traces
and invariants that any correct reading must keep.  CPU only.
"""
import numpy as np
import pytest

from oracle import mux_oracle as orc

P, D, X = orc.PREFILL, orc.DECODE, orc.PREEMPT
T, F = orc.FLAG_TABLE, orc.FLAG_FINISHED


def brief(jobs):
    return [(j["kind"], j["model"], j["ids"].tolist(), j["slots"].tolist(), j["lens"].tolist(), j["flags"].tolist())
            for j in jobs]


def test_single_request_hand_trace():
    # 2 heads, 16-token blocks, prompt 20, 5 outputs: prefill caches 20 tokens (2 blocks per head)
    # and yields output 1; four decoding steps append tokens 21..24 and yield outputs 2..5
    p = orc.OraclePool(64, 16, 128)
    s = orc.OracleScheduler(p, [2], max_seqs=4, max_blocks=8, max_prefill_tokens=64)
    assert s.submit(0, 100, 20, 5) == 0
    assert brief(s.step()) == [(P, 0, [100], [0], [20], [T]), (D, 0, [100], [0], [21], [0])]
    assert p.num_free() == 60 and p.num_used(0) == 4
    t = s.table(0)
    assert t[0, 0, :2].tolist() == [0, 1] and t[0, 1, :2].tolist() == [2, 3]      # head-major ids
    assert brief(s.step()) == [(D, 0, [100], [0], [22], [0])]
    assert brief(s.step()) == [(D, 0, [100], [0], [23], [0])]
    assert brief(s.step()) == [(D, 0, [100], [0], [24], [F])]
    # the ended request keeps its blocks until the next iteration starts (its last job reads them)
    assert p.num_free() == 60 and s.counts(0) == (0, 0, 1, 0, 0)
    assert s.step() == [] and p.num_free() == 64
    # the blocks came back in table order: the next request gets them in reverse (LIFO)
    assert s.submit(0, 101, 16, 3) == 0
    assert brief(s.step()) == [(P, 0, [101], [0], [16], [T]), (D, 0, [101], [0], [17], [T])]   # 16 % 16 == 0: new block
    t = s.table(0)
    # frees pushed 0,1,2,3: the prefill pops 3 (head 0), 2 (head 1); the new block pops 1, 0
    assert t[0, :, 0].tolist() == [3, 2] and t[0, :, 1].tolist() == [1, 0]
    assert brief(s.step()) == [(D, 0, [101], [0], [18], [F])]
    assert s.step() == [] and p.num_free() == 64


def test_single_output_request_ends_with_its_prefill():
    p = orc.OraclePool(16, 16, 128)
    s = orc.OracleScheduler(p, [1], 2, 4, 64)
    s.submit(0, 7, 10, 1)
    assert brief(s.step()) == [(P, 0, [7], [0], [10], [T | F])]
    assert p.num_free() == 15 and s.counts(0)[:3] == (0, 0, 1)
    assert s.step() == [] and p.num_free() == 16


def test_round_robin_prefill_and_rotating_decode_start():
    # 3 models, one request per prefill job (token budget 8 < any two prompts)
    p = orc.OraclePool(400, 16, 128)
    s = orc.OracleScheduler(p, [1, 2, 1], max_seqs=4, max_blocks=8, max_prefill_tokens=8)
    for m in range(3):
        for k in range(2):
            s.submit(m, 10 * m + k, 6, 50)
    order = []
    for it in range(6):
        jobs = s.step()
        pre = [j for j in jobs if j["kind"] == P]
        assert len(pre) == 1 and pre[0]["ids"].size == 1
        order.append((pre[0]["model"], int(pre[0]["ids"][0])))
        dec = [j["model"] for j in jobs if j["kind"] == D]
        first = it % 3                                         # the model served first rotates by one
        running = {m for m, _ in order}
        want = [m for m in [(first + k) % 3 for k in range(3)] if m in running]
        assert dec == want
    assert order == [(0, 0), (1, 10), (2, 20), (0, 1), (1, 11), (2, 21)]
    assert not [j for j in s.step() if j["kind"] == P]        # nothing left to prefill


def test_prefill_batches_up_to_the_token_budget_and_slots():
    p = orc.OraclePool(400, 16, 128)
    s = orc.OracleScheduler(p, [1], max_seqs=3, max_blocks=8, max_prefill_tokens=40)
    for k, plen in enumerate([30, 8, 5, 4, 4]):
        s.submit(0, k, plen, 20)
    j = s.step()[0]
    assert j["kind"] == P and j["ids"].tolist() == [0, 1] and j["lens"].tolist() == [30, 8]     # 30+8 <= 40 < 30+8+5
    j = s.step()[0]
    assert j["kind"] == P and j["ids"].tolist() == [2]                                          # one slot left
    assert s.step()[0]["kind"] == D and s.counts(0)[:2] == (2, 3)                               # no slot: no prefill
    # a first request longer than the budget is still taken, alone
    s2 = orc.OracleScheduler(orc.OraclePool(400, 16, 128), [1], 3, 8, 16)
    s2.submit(0, 0, 100, 2)
    s2.submit(0, 1, 4, 2)
    assert s2.step()[0]["ids"].tolist() == [0]


def test_quota_holds_back_admission_but_not_decoding():
    p = orc.OraclePool(100, 16, 128)
    s = orc.OracleScheduler(p, [2, 2], max_seqs=4, max_blocks=8, max_prefill_tokens=256)
    assert p.set_quota(0, 6) == 0 and p.set_quota(1, 94) == 0
    s.submit(0, 0, 40, 4)      # 3 blocks x 2 heads = 6: fills the quota of model 0
    s.submit(0, 1, 10, 4)      # 2 more: must wait until request 0 is gone
    s.submit(1, 2, 10, 4)
    trace = []
    for _ in range(6):
        trace.append(brief(s.step()))
        for m in (0, 1):
            assert p.num_used(m) <= p.get_quota(m)
    # iteration 0: the prefill of model 0 takes request 0 only; model 1 is prefilled in iteration 1
    assert trace[0] == [(P, 0, [0], [0], [40], [T]), (D, 0, [0], [0], [41], [0])]
    assert trace[1][0] == (P, 1, [2], [0], [10], [T])
    assert trace[2][0][0] == D                                  # model 0 cannot admit request 1 yet: 6 + 2 > 6
    # request 0 ends in iteration 2 (outputs 2, 3, 4 in iterations 0, 1, 2); request 1 enters in iteration 3
    assert (D, 0, [0], [0], [43], [F]) in trace[2]
    assert (P, 0, [1], [0], [10], [T]) in trace[3]


def test_preemption_of_the_youngest_and_recompute_length():
    # pool of 6 blocks, 1 head: two requests of 31 tokens hold 2 blocks each; both reach a block
    # boundary in the same step (context 32) and need 2 new blocks -> fits (2 free); at context 48
    # they need 2 more and none is free -> the younger one is preempted and recomputed later
    p = orc.OraclePool(6, 16, 128)
    s = orc.OracleScheduler(p, [1], max_seqs=2, max_blocks=8, max_prefill_tokens=256)
    s.submit(0, 0, 31, 40)
    s.submit(0, 1, 31, 40)
    events = []
    for it in range(200):
        jobs = s.step()
        events += [(it, j["kind"], j["ids"].tolist(), j["lens"].tolist(), j["flags"].tolist()) for j in jobs]
        if s.counts(0)[2] == 2:
            break
    pre = [e for e in events if e[1] == X]
    assert pre and pre[0][2] == [1] and pre[0][3] == [48]          # request 1 (the younger) at context 48
    it_pre = pre[0][0]
    # outputs so far: 1 from prefill + one per decoding step taken = 48 - 31 + 1 = 18
    redo = [e for e in events if e[1] == P and e[0] > it_pre and 1 in e[2]]
    assert redo and redo[0][3] == [31 + 18 - 1]                    # prompt + outputs so far - the last one
    # each request took exactly output_len - 1 decoding steps in total, preempted or not
    for rid in (0, 1):
        steps = sum(e[2].count(rid) for e in events if e[1] == D)
        assert steps == 39
    assert s.step() == []                                          # flushes the blocks of the request that ended last
    assert p.num_free() == 6 and s.counts(0)[2:4] == (2, len(pre))


def test_request_preempted_in_the_iteration_that_admitted_it_never_launches():
    # 3 blocks of 4 tokens, 1 head.  Request 0 (prompt 4) holds 2 blocks after its first iteration.
    # Request 1 (prompt 4) is admitted into the last free block, and in the same iteration its
    # decoding step needs a block that is not there: it is the youngest, goes back to the queue,
    # and - its block being free again for anybody - must not appear in any job of that iteration.
    p = orc.OraclePool(3, 4, 128)
    s = orc.OracleScheduler(p, [1], max_seqs=2, max_blocks=8, max_prefill_tokens=64)
    assert s.submit(0, 0, 4, 9) == 0
    assert brief(s.step()) == [(P, 0, [0], [0], [4], [T]), (D, 0, [0], [0], [5], [T])]
    assert s.submit(0, 1, 4, 9) == 0
    assert brief(s.step()) == [(D, 0, [0], [0], [6], [0])]
    assert s.counts(0)[:4] == (1, 1, 0, 1) and p.num_used(0) == 2 and p.num_free() == 1
    assert brief(s.step()) == [(D, 0, [0], [0], [7], [0])]
    assert s.counts(0)[:4] == (1, 1, 0, 2)
    assert brief(s.step()) == [(D, 0, [0], [0], [8], [0])]
    # context 8 opens a block for request 0: request 1 is admitted first, struck again, and the block goes to request 0
    assert brief(s.step()) == [(D, 0, [0], [0], [9], [T])]
    assert p.num_free() == 0 and s.counts(0)[:4] == (1, 1, 0, 4)
    events = []
    for _ in range(40):
        events += brief(s.step())
        if s.counts(0)[2] == 2:
            break
    assert s.step() == [] and p.num_free() == 3
    # request 1 was prefilled exactly once (after request 0 ended) and no preempt job was ever listed
    assert [e for e in events if e[0] == P] == [(P, 0, [1], [0], [4], [T])]
    assert not [e for e in events if e[0] == X]
    assert sum(e[2].count(1) for e in events if e[0] == D) == 8


def _check_state(p, s, n_models, heads, B, live, ended):
    """Block conservation and table sanity: what the pool says a model holds is what its running
    requests (and those that ended in this iteration) need; all ids in use are distinct."""
    seen = set()
    for m in range(n_models):
        t = s.table(m)
        need = 0
        for (mm, rid), (slot, ctx) in list(live.items()) + ended:
            if mm != m:
                continue
            nb = (ctx + B - 1) // B
            need += nb * heads[m]
            ids = t[slot, :, :nb].reshape(-1).tolist()
            assert all(0 <= i < p.num_blocks for i in ids)
            assert not (seen & set(ids)) and len(set(ids)) == len(ids)
            seen |= set(ids)
        assert p.num_used(m) == need
    assert p.num_free() == p.num_blocks - len(seen)


@pytest.mark.parametrize("seed,with_quota", [(0, False), (1, True), (2, True), (3, False)])
def test_invariants_under_random_traffic(seed, with_quota):
    rng = np.random.default_rng(seed)
    n_models = int(rng.integers(2, 5))
    heads = [int(h) for h in rng.choice([1, 2, 4, 8], n_models)]
    B, n_blocks, max_seqs, max_blocks = 16, 3000, 12, 24
    p = orc.OraclePool(n_blocks, B, 128)
    if with_quota:
        assert p.init_quotas(rng.random(n_models) + 0.2) == 0
    s = orc.OracleScheduler(p, heads, max_seqs, max_blocks, 300, adapt_period=7 if with_quota else 0,
                            low=0.5, high=0.9, step=0.3)
    want_out, dec_steps, first_admit, live = {}, {}, {m: [] for m in range(n_models)}, {}
    submitted = {m: [] for m in range(n_models)}
    rid = 0
    for it in range(1500):
        if it < 900:
            for _ in range(int(rng.poisson(0.6))):
                m = int(rng.integers(n_models))
                plen, olen = int(rng.integers(1, 200)), int(rng.integers(1, 150))
                assert s.submit(m, rid, plen, olen) == 0
                want_out[(m, rid)] = olen
                dec_steps[(m, rid)] = 0
                submitted[m].append(rid)
                rid += 1
        jobs = s.step()
        ended = []
        kinds = [j["kind"] for j in jobs]
        assert kinds.count(P) <= 1 and (P not in kinds or kinds[0] == P)       # at most one prefill job, first
        dec_models = [j["model"] for j in jobs if j["kind"] == D]
        assert len(dec_models) == len(set(dec_models))                           # one decoding step per model
        for j in jobs:
            m = j["model"]
            for r, slot, ln, fl in zip(j["ids"].tolist(), j["slots"].tolist(), j["lens"].tolist(), j["flags"].tolist()):
                key = (m, r)
                if j["kind"] == P:
                    assert key not in live
                    if r not in first_admit[m]:
                        first_admit[m].append(r)
                    live[key] = (slot, ln)
                elif j["kind"] == D:
                    assert key in live and live[key] == (slot, ln - 1)
                    live[key] = (slot, ln)
                    dec_steps[key] += 1
                else:
                    assert live.pop(key) == (slot, ln)
                if fl & F:
                    assert j["kind"] != X
                    ended.append((key, live.pop(key)))
                    assert dec_steps[key] == want_out[key] - 1                   # exactly output_len tokens
                    del want_out[key]
        if with_quota:
            for m in range(n_models):
                assert p.num_used(m) <= max(p.get_quota(m), p.peak_used(m))
        if it % 50 == 0:
            _check_state(p, s, n_models, heads, B, live, ended)
        if it >= 900 and not want_out:
            break
    assert not want_out and not live, "every request must finish once arrivals stop"
    assert s.step() == [] and p.num_free() == n_blocks
    for m in range(n_models):
        assert first_admit[m] == submitted[m]                                    # first admission is first come first served
        assert s.counts(m)[:2] == (0, 0)
    if with_quota:
        assert sum(p.get_quota(m) for m in range(n_models)) == n_blocks


def test_usage_shares_follow_quotas_under_contention():
    """The paper's ablation (Section 4.4, cache usage figure): without quotas a model with long
    requests crowds the shared cache whatever the arrival rates are; with quotas in proportion to
    the rates the block usage is aligned with them.  Shape only: rates 1:4, request lengths 4:1."""
    def run(quota):
        rng = np.random.default_rng(4)
        p = orc.OraclePool(2400, 16, 128)
        heads = [8, 8]
        if quota:
            assert p.init_quotas([1.0, 4.0]) == 0
        s = orc.OracleScheduler(p, heads, 64, 64, 2048)
        use = np.zeros(2)
        rid = 0
        for it in range(3000):
            for m, rate, scale in ((0, 0.15, 4), (1, 0.6, 1)):
                for _ in range(int(rng.poisson(rate))):
                    s.submit(m, rid, int(rng.integers(40, 120)) * scale, int(rng.integers(20, 60)) * scale)
                    rid += 1
            s.step()
            if it >= 500:
                use += [p.num_used(0), p.num_used(1)]
        return use / use.sum()
    free_for_all, with_quota = run(False), run(True)
    rate_share = np.array([0.2, 0.8])
    assert abs(with_quota - rate_share).max() < abs(free_for_all - rate_share).max()
    assert abs(with_quota - rate_share).max() < 0.08 and free_for_all[0] > with_quota[0] + 0.15
