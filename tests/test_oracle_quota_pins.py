"""Pins of the oracle's token-block quotas (Section 3.3; Algorithm 3: initial quota, the check
before a job runs, periodic adaptation) against hand-worked examples, closed forms and
invariants.  The paper prints no numbers for quotas; the rules pinned here are the readings the
oracle's header states.  CPU only.
"""
import numpy as np
import pytest

from oracle import mux_oracle as orc


def quotas(p, n):
    return [p.get_quota(m) for m in range(n)]


def test_quota_is_checked_before_the_pool_and_changes_nothing():
    p = orc.OraclePool(10, 16, 128)
    assert p.get_quota(0) == -1                                # none by default
    assert p.set_quota(0, 4) == orc.OK and p.get_quota(0) == 4
    assert list(p.alloc(0, 3)) == [0, 1, 2]
    rc, ids = p.alloc_status(0, 2)                             # 3 + 2 > 4
    assert rc == orc.ERR_QUOTA and ids is None and p.num_used(0) == 3 and p.num_free() == 7
    assert list(p.alloc(0, 1)) == [3]                          # exactly up to the quota
    assert p.alloc_status(0, 1)[0] == orc.ERR_QUOTA
    # a request that breaks the quota AND exceeds the pool reports the quota
    assert p.alloc_status(0, 100)[0] == orc.ERR_QUOTA
    # a model without a quota is bounded by the pool only
    assert p.alloc_status(1, 7)[0] == orc.ERR_NOMEM and p.alloc_status(1, 6)[0] == orc.OK
    # lowering a quota below the usage takes nothing back; frees make room again
    assert p.set_quota(0, 2) == orc.OK and p.num_used(0) == 4
    assert p.alloc_status(0, 1)[0] == orc.ERR_QUOTA
    p.free(0, [0, 1, 2])
    assert list(p.alloc(0, 1)) == [2] and p.alloc_status(0, 1)[0] == orc.ERR_QUOTA
    # removing the quota
    assert p.set_quota(0, -1) == orc.OK and p.alloc_status(0, 2)[0] == orc.OK
    # argument errors
    assert p.set_quota(0, 11) == orc.ERR_INVALID and p.set_quota(0, -2) == orc.ERR_INVALID
    assert p.set_quota(-1, 1) == orc.ERR_INVALID and p.set_quota(1024, 1) == orc.ERR_INVALID


def test_peak_follows_the_high_water_mark():
    p = orc.OraclePool(32, 16, 128)
    a = p.alloc(0, 10)
    p.free(0, a[:6])
    p.alloc(0, 3)
    assert p.num_used(0) == 7 and p.peak_used(0) == 10
    p.alloc(0, 5)
    assert p.peak_used(0) == 12
    assert p.alloc_status(0, 100)[0] == orc.ERR_NOMEM and p.peak_used(0) == 12   # failed calls leave it alone


@pytest.mark.parametrize("n_blocks, weights, want", [
    (100, [0.5, 0.3, 0.2], [50, 30, 20]),           # exact shares
    (7, [3, 2, 2], [3, 2, 2]),                      # weights need not sum to one
    (10, [1, 1, 1], [4, 3, 3]),                     # 3.33 each: the spare block goes to the first of the tie
    (10, [0.45, 0.35, 0.2], [5, 3, 2]),             # 4.5 / 3.5 / 2.0: fractions tie, lower id wins
    (10, [0.2, 0.35, 0.45], [2, 4, 4]),             # 2.0 / 3.5 / 4.5: spare to model 1 (first of the tie)
    (11, [1, 2, 4], [2, 3, 6]),                     # 1.571 / 3.143 / 6.286 -> 1, 3, 6 + spare to the .571
    (5, [0, 1, 0], [0, 5, 0]),                      # zero weight, zero quota
    (3, [1, 1, 1, 1, 1], [1, 1, 1, 0, 0]),          # more models than blocks
])
def test_initial_quotas_largest_remainder(n_blocks, weights, want):
    p = orc.OraclePool(n_blocks, 16, 128)
    assert p.init_quotas(weights) == orc.OK
    assert quotas(p, len(weights)) == want and sum(want) == n_blocks


def test_initial_quotas_properties_and_errors():
    rng = np.random.default_rng(5)
    for _ in range(200):
        n_models = int(rng.integers(1, 20))
        n_blocks = int(rng.integers(1, 100000))
        w = rng.random(n_models) ** 3 + 1e-9
        p = orc.OraclePool(n_blocks, 16, 128)
        assert p.init_quotas(w) == orc.OK
        q = np.array(quotas(p, n_models))
        assert q.sum() == n_blocks                                           # the whole pool is shared out
        assert (np.abs(q - n_blocks * w / w.sum()) < 1.0).all()              # each within one block of its share
        order = np.argsort(-w, kind="stable")
        assert (np.diff(q[order]) <= 0).all()                                # a larger weight never gets less
        p2 = orc.OraclePool(n_blocks, 16, 128)
        assert p2.init_quotas(w * 7.5) == orc.OK and quotas(p2, n_models) == list(q)   # scale-free
    p = orc.OraclePool(10, 16, 128)
    for bad in ([0, 0], [1, -1], [1, float("nan")], [1, float("inf")], []):
        assert p.init_quotas(bad) == orc.ERR_INVALID
    assert quotas(p, 2) == [-1, -1]


def _pool_with(n_blocks, q, peaks, used=None):
    p = orc.OraclePool(n_blocks, 16, 128)
    used = peaks if used is None else used
    for m, (pk, u) in enumerate(zip(peaks, used)):
        ids = p.alloc(m, pk) if pk else np.zeros(0, np.int32)
        if u < pk:
            p.free(m, ids[u:])
    for m, qm in enumerate(q):
        assert p.set_quota(m, qm) == orc.OK
    return p


def test_adaptation_hand_example():
    # quotas 50/30/20, peaks 10/30/19: utilisation 0.2 / 1.0 / 0.95; low 0.5, high 0.9, step 0.5
    # model 0 gives floor(0.5 * 40) = 20; takers weigh 30 and 19 (sum 49):
    #   20*30/49 = 12 rest 12, 20*19/49 = 7 rest 37 -> the spare block goes to model 2: +12, +8
    p = _pool_with(100, [50, 30, 20], [10, 30, 19])
    assert p.adapt_quotas(3, 0.5, 0.9, 0.5) == (orc.OK, 20)
    assert quotas(p, 3) == [30, 42, 28]
    # second period, nothing new allocated: peaks restarted at the usage (10/30/19): utilisation
    # 0.33 / 0.71 / 0.68 -> a giver but no taker: nothing moves
    assert p.adapt_quotas(3, 0.5, 0.9, 0.5) == (orc.OK, 0) and quotas(p, 3) == [30, 42, 28]
    # model 1 fills its quota, model 0 keeps giving half of its slack: 20 -> 10 -> 5 -> 3 -> 2 ...
    p.alloc(1, 12)
    assert p.adapt_quotas(3, 0.5, 0.9, 0.5) == (orc.OK, 10) and quotas(p, 3) == [20, 52, 28]


def test_adaptation_uses_the_peak_not_the_current_usage():
    p = _pool_with(100, [50, 50], [40, 50], used=[5, 50])
    # model 0 peaked at 40 of 50 (0.8 >= low): it gives nothing although it holds 5 blocks now
    assert p.adapt_quotas(2, 0.5, 0.9, 1.0) == (orc.OK, 0) and quotas(p, 2) == [50, 50]
    # the next period starts from the usage: 5 of 50 -> gives all of its slack with step 1
    assert p.adapt_quotas(2, 0.5, 0.9, 1.0) == (orc.OK, 45) and quotas(p, 2) == [5, 95]


def test_adaptation_geometric_decay_of_the_slack():
    # a lone giver with constant usage u and a taker, low = high = 1 (anything short of full use
    # gives): its slack s_k = q_k - u obeys s_{k+1} = s_k - floor(step * s_k)
    u, q0, step = 100, 1100, 0.25
    p = _pool_with(5000, [q0, 2000], [u, 2000])
    s = q0 - u
    for _ in range(30):
        give = int(np.floor(step * s))
        assert p.adapt_quotas(2, 1.0, 1.0, step) == (orc.OK, give)
        s -= give
        assert p.get_quota(0) == u + s and p.get_quota(1) == 2000 + (q0 - u - s)
        p.alloc(1, give)                      # the taker fills what it got, so it stays a taker
    assert s == 3                             # floor(0.25 * 3) = 0: the slack stops shrinking at 3


def test_adaptation_invariants_under_random_traffic():
    rng = np.random.default_rng(11)
    n_models, n_blocks = 6, 20000
    p = orc.OraclePool(n_blocks, 16, 128)
    assert p.init_quotas(rng.random(n_models) + 0.1) == orc.OK
    held = [[] for _ in range(n_models)]
    moved_total = 0
    for it in range(400):
        for _ in range(20):
            m = int(rng.integers(n_models))
            if rng.random() < 0.55 + 0.3 * (m % 2):           # odd models are hungrier
                rc, ids = p.alloc_status(m, int(rng.integers(1, 300)))
                assert rc in (orc.OK, orc.ERR_QUOTA, orc.ERR_NOMEM)
                if rc == orc.OK:
                    held[m].append(ids)
            elif held[m]:
                p.free(m, held[m].pop(int(rng.integers(len(held[m])))))
        before = quotas(p, n_models)
        peaks = [p.peak_used(m) for m in range(n_models)]
        used = [p.num_used(m) for m in range(n_models)]
        rc, moved = p.adapt_quotas(n_models, 0.6, 0.9, 0.3)
        after = quotas(p, n_models)
        assert rc == orc.OK and sum(after) == sum(before) == n_blocks          # conservation
        for m in range(n_models):
            assert used[m] <= peaks[m]
            if after[m] < before[m]:                                            # a giver
                assert peaks[m] < 0.6 * before[m] and after[m] >= peaks[m]      # keeps what it used
            if after[m] > before[m]:                                            # a taker
                assert peaks[m] >= 0.9 * before[m]
            assert p.peak_used(m) == used[m]                                    # peaks restart
        assert moved == sum(max(0, b - a) for a, b in zip(after, before))
        moved_total += moved
    assert moved_total > 0


def test_adaptation_degenerate_cases_and_errors():
    p = _pool_with(100, [50, 50], [10, 50])
    assert p.adapt_quotas(2, 0.5, 0.9, 0.0) == (orc.OK, 0) and quotas(p, 2) == [50, 50]     # step 0
    p = _pool_with(100, [50, 50], [10, 10])
    assert p.adapt_quotas(2, 0.5, 0.9, 0.5) == (orc.OK, 0) and quotas(p, 2) == [50, 50]     # givers only
    p = _pool_with(100, [50, 50], [50, 50])
    assert p.adapt_quotas(2, 0.5, 0.9, 0.5) == (orc.OK, 0) and quotas(p, 2) == [50, 50]     # takers only
    p = _pool_with(100, [60, 0, 40], [10, 0, 40])
    # a model with quota 0 and nothing held is no taker (0 >= 0.9 * 0 holds, but it uses nothing)
    assert p.adapt_quotas(3, 0.5, 0.9, 0.5) == (orc.OK, 25) and quotas(p, 3) == [35, 0, 65]
    p = _pool_with(100, [50, 50], [10, 50])
    for low, high, step in ((-0.1, 0.9, 0.5), (0.9, 0.5, 0.5), (0.5, 0.9, 1.5), (0.5, 0.9, -0.1),
                            (float("nan"), 0.9, 0.5), (0.5, float("inf"), 0.5)):
        assert p.adapt_quotas(2, low, high, step)[0] == orc.ERR_INVALID
    assert p.adapt_quotas(3, 0.5, 0.9, 0.5)[0] == orc.ERR_INVALID            # model 2 has no quota
    assert p.adapt_quotas(0, 0.5, 0.9, 0.5)[0] == orc.ERR_INVALID
    assert quotas(p, 2) == [50, 50] and p.peak_used(0) == 10                 # failed calls change nothing
