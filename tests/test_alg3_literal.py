"""Algorithm 3 (Section 3.3, adaptive batch scheduling) written out literally, as a check of the
scheduler oracle that is not built like it.

`LiteralADBS.one_pass` below is the body of the algorithm's endless loop, statement by statement:
the prefill_waiting flag, one round-robin prefill job that runs only if its resources are there,
and - unless a prefill is waiting - round-robin decoding jobs for as long as resources are there.
It counts blocks; it hands out no ids and keeps no tables.  What the algorithm leaves open is
taken as the oracle's header states it, and only where a literal loop needs it at all:
  - a pass is synchronous, so "no prefill jobs in execution" holds at the start of every pass;
    "round-robin a job" finds nothing when no LLM has one (then nothing is waiting either);
  - a prefill job = the LLM's waiting requests in arrival order while token budget, slots and
    blocks allow (the first whatever its length); a decoding job = one step of all running
    requests of an LLM; an LLM decodes at most once per pass (a second step needs the first's
    output); a finished request gives its blocks back at the start of the next pass.

Three readings of the oracle are NOT in the literal loop, and the tests pin exactly where the
two part ways: a prefill that cannot run (no blocks, or no free sequence slot) holds decoding
back (literal) or is skipped (oracle); a decoding step that finds no block ends the pass's
decoding (literal) or preempts the LLM's newest request (oracle); the decode pointer simply
carries on (literal) or the first LLM served rotates by one per pass (oracle).  On traffic where no request for blocks or slots is ever
refused the first two never arise and the two must agree job for job, up to the order of a pass's
decoding jobs.
"""
from collections import deque

import numpy as np

from oracle import mux_oracle as orc

P, D, X = orc.PREFILL, orc.DECODE, orc.PREEMPT


class LiteralADBS:
    def __init__(self, n_blocks, heads, block_size, max_seqs, max_prefill_tokens, quota=None):
        self.free, self.heads, self.B = n_blocks, list(heads), block_size
        self.max_seqs, self.budget = max_seqs, max_prefill_tokens
        n = len(self.heads)
        self.quota = list(quota) if quota is not None else [None] * n      # init_token_block_quota(M)
        self.used = [0] * n
        self.waiting = [deque() for _ in range(n)]
        self.running = [[] for _ in range(n)]            # [id, ctx, gen, output_len], admission order
        self.ended = []                                  # (model, blocks) released at the next pass
        self.prefill_ptr = self.decode_ptr = 0
        self.prefill_waiting = False

    def submit(self, m, rid, prompt_len, output_len):
        self.waiting[m].append([rid, prompt_len, output_len])

    def blocks(self, tokens):
        return -(-tokens // self.B)

    def room(self, m):
        return self.free if self.quota[m] is None else min(self.free, self.quota[m] - self.used[m])

    def take(self, m, n):
        self.free -= n
        self.used[m] += n

    def round_robin(self, ptr, has_job):
        n = len(self.heads)
        return next(((ptr + k) % n for k in range(n) if has_job((ptr + k) % n)), None)

    def one_pass(self):
        jobs = []
        for m, nb in self.ended:                         # requests that ended in the pass before
            self.free += nb
            self.used[m] -= nb
        self.ended = []
        # "if no prefill jobs in execution" - always, in a synchronous pass
        m = self.round_robin(self.prefill_ptr, lambda c: len(self.waiting[c]) > 0)
        self.prefill_waiting = m is not None             # prefill_waiting <- True (there is one to wait for)
        if m is not None:
            self.prefill_ptr = (m + 1) % len(self.heads)
            ids, lens, fin, tokens = [], [], [], 0
            while self.waiting[m]:                       # the job: requests while budget, slots and blocks allow
                rid, plen, olen = self.waiting[m][0]
                need = self.blocks(plen) * self.heads[m]
                if (ids and tokens + plen > self.budget) or len(self.running[m]) >= self.max_seqs or need > self.room(m):
                    break
                self.waiting[m].popleft()
                self.take(m, need)
                tokens += plen
                ids.append(rid), lens.append(plen), fin.append(olen == 1)
                if olen == 1:
                    self.ended.append((m, need))
                else:
                    self.running[m].append([rid, plen, 1, olen])
            if ids:                                      # resource_enough(m, quota): execute_and_update
                jobs.append((P, m, ids, lens, fin))
                self.prefill_waiting = False
        if not self.prefill_waiting:
            served = set()
            while True:
                m = self.round_robin(self.decode_ptr, lambda c: self.running[c] and c not in served)
                if m is None:
                    break
                need = sum(self.heads[m] for r in self.running[m] if r[1] % self.B == 0)
                if need > self.room(m):                  # not resource_enough: the inner loop ends
                    break
                self.decode_ptr = (m + 1) % len(self.heads)
                served.add(m)
                self.take(m, need)
                ids, lens, fin, keep = [], [], [], []
                for r in self.running[m]:
                    r[1] += 1
                    r[2] += 1
                    ids.append(r[0]), lens.append(r[1]), fin.append(r[2] >= r[3])
                    if r[2] >= r[3]:
                        self.ended.append((m, self.blocks(r[1]) * self.heads[m]))
                    else:
                        keep.append(r)
                self.running[m] = keep
                jobs.append((D, m, ids, lens, fin))
        return jobs                                      # (quota adaptation: not exercised here)


def oracle_jobs(sched):
    return [(j["kind"], j["model"], j["ids"].tolist(), j["lens"].tolist(), [bool(f & orc.FLAG_FINISHED) for f in j["flags"]])
            for j in sched.step()]


def test_oracle_equals_the_literal_loop_when_no_request_for_blocks_is_refused():
    """Poisson traffic for three LLMs on a pool that always has room and slots: per pass the same
    prefill job and the same decoding jobs (as a set: their order is the third reading above)."""
    heads, B, max_seqs, budget = [2, 4, 1], 16, 64, 96
    n_blocks = 20000
    pool = orc.OraclePool(n_blocks, B, 128)
    sched = orc.OracleScheduler(pool, heads, max_seqs, max_blocks=64, max_prefill_tokens=budget)
    lit = LiteralADBS(n_blocks, heads, B, max_seqs, budget)
    rng = np.random.default_rng(2404)
    rid, n_prefill, n_decode, multi = 0, 0, 0, 0
    for it in range(600):
        if it < 200:
            for _ in range(int(rng.poisson(0.9))):
                m, plen, olen = int(rng.integers(3)), int(rng.integers(1, 120)), int(rng.integers(1, 40))
                assert sched.submit(m, rid, plen, olen) == 0
                lit.submit(m, rid, plen, olen)
                rid += 1
        got, want = oracle_jobs(sched), lit.one_pass()
        assert not [j for j in got if j[0] == X], "the pool was meant to be roomy"
        assert all(len(r) < max_seqs for r in lit.running), "and so were the slots"
        assert [j for j in got if j[0] == P] == [j for j in want if j[0] == P], "pass %d: prefill job" % it
        assert got[:1] == want[:1] or (got and want and got[0][0] == D and want[0][0] == D)   # the prefill job comes first
        key = lambda j: j[1]
        assert sorted((j for j in got if j[0] == D), key=key) == sorted((j for j in want if j[0] == D), key=key), "pass %d" % it
        n_prefill += sum(j[0] == P for j in got)
        n_decode += sum(j[0] == D for j in got)
        multi += sum(j[0] == P and len(j[2]) > 1 for j in got)
        assert pool.num_free() == lit.free and [pool.num_used(m) for m in range(3)] == lit.used
    assert rid > 100 and n_prefill > 80 and n_decode > 500 and multi > 5
    assert all(sched.counts(m)[:2] == (0, 0) for m in range(3)) and lit.free == n_blocks


def test_where_they_part_1_decode_order():
    """Three LLMs, all decoding in every pass.  Literal: the pointer carries on from the last LLM
    served, which after a full round is where it started - the same order in every pass.
    Oracle: the LLM served first rotates by one per pass."""
    pool = orc.OraclePool(400, 16, 128)
    sched = orc.OracleScheduler(pool, [1, 1, 1], max_seqs=2, max_blocks=8, max_prefill_tokens=64)
    lit = LiteralADBS(400, [1, 1, 1], 16, 2, 64)
    for m in range(3):
        sched.submit(m, m, 8, 30)
        lit.submit(m, m, 8, 30)
    orders_o, orders_l = [], []
    for _ in range(6):
        orders_o.append([j[1] for j in oracle_jobs(sched) if j[0] == D])
        orders_l.append([j[1] for j in lit.one_pass() if j[0] == D])
    # passes 0-2 admit one LLM each (prefill round-robin); from pass 2 on all three decode.  Literal:
    # the pointer stands behind LLM 0 after pass 0, and a full round brings it back there every time.
    assert orders_l == [[0], [1, 0], [1, 2, 0], [1, 2, 0], [1, 2, 0], [1, 2, 0]]
    assert orders_o == [[0], [1, 0], [2, 0, 1], [0, 1, 2], [1, 2, 0], [2, 0, 1]]


def test_where_they_part_2_prefill_refused_for_blocks():
    """8 blocks.  LLM 0 runs a request that holds 5 and will finish; LLM 1's prompt needs 4.
    Literal: the refused prefill leaves prefill_waiting set, decoding stops, and since only
    decoding frees blocks nothing ever runs again.  Oracle: the prefill is skipped, LLM 0
    decodes to its end, its blocks come back and LLM 1 is admitted."""
    pool = orc.OraclePool(8, 16, 128)
    sched = orc.OracleScheduler(pool, [1, 1], max_seqs=2, max_blocks=8, max_prefill_tokens=128)
    lit = LiteralADBS(8, [1, 1], 16, 2, 128)
    for s in (sched, lit):
        s.submit(0, 0, 70, 6)                 # 5 blocks, ends with 75 cached tokens
    assert [j[:2] for j in oracle_jobs(sched)] == [(P, 0), (D, 0)] == [j[:2] for j in lit.one_pass()]
    for s in (sched, lit):
        s.submit(1, 1, 64, 2)                 # 4 blocks > 3 free
    lit_passes = [lit.one_pass() for _ in range(12)]
    assert lit_passes == [[]] * 12 and lit.prefill_waiting and lit.free == 3          # stuck for good
    trace = [[j[:2] for j in oracle_jobs(sched)] for _ in range(8)]
    assert trace[:4] == [[(D, 0)]] * 4                     # outputs 3..6 of request 0; it ends in the 4th pass
    assert trace[4] == [(P, 1), (D, 1)] and trace[5] == [] and pool.num_free() == 8


def test_where_they_part_3_decoding_step_finds_no_block():
    """6 blocks, one LLM, two requests of 32 tokens (2 blocks each) + one free pair.  After both are
    admitted the first decoding step needs a block for each (context 32 = a block boundary): 2 <= 2,
    fine.  At context 48 both need a block again and none is free.  Literal: not resource_enough,
    the decoding loop ends, nothing frees a block, nothing runs again.  Oracle: the newest request is
    preempted (its 3 blocks come back, it waits at the front to be recomputed), the other goes on."""
    pool = orc.OraclePool(6, 16, 128)
    sched = orc.OracleScheduler(pool, [1], max_seqs=2, max_blocks=8, max_prefill_tokens=64)
    lit = LiteralADBS(6, [1], 16, 2, 64)
    for s in (sched, lit):
        s.submit(0, 0, 32, 40)
        s.submit(0, 1, 32, 40)
    for it in range(16):                                    # contexts 33 .. 48: identical
        got, want = oracle_jobs(sched), lit.one_pass()
        assert got == want and got[-1][:2] == (D, 0) and got[-1][3] == [33 + it, 33 + it]
    assert pool.num_free() == 0 == lit.free
    assert [lit.one_pass() for _ in range(5)] == [[]] * 5   # literal: stuck
    got = oracle_jobs(sched)
    assert [(j[0], j[2]) for j in got] == [(X, [1]), (D, [0])] and sched.counts(0)[3] == 1
    assert got[1][3] == [49] and pool.num_free() == 2       # request 1 gave back 3 blocks, request 0 took 1
