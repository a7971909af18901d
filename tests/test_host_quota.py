"""Token-block quotas of the library (Section 3.3, Algorithm 3) against the oracle's, call by
call: statuses, ids, quotas, peaks and the blocks moved by every adaptation must be identical.
CPU only; no kernel is launched.
"""
import numpy as np
import pytest

from oracle import mux_oracle as orc
from paper_2404_02015_amd import binding as mx
from paper_2404_02015_amd import workloads as wl
from test_host_library import host_pool


class Both:
    """The two block managers driven in lockstep."""

    def __init__(self, n_blocks, order=None):
        self.lib = host_pool(n_blocks, order=order)
        self.ora = orc.OraclePool(n_blocks, 16, 128, init_free_order=order)

    def alloc(self, m, n):
        rc_l, ids_l = mx.mux_alloc_blocks_status(self.lib, m, n)
        rc_o, ids_o = self.ora.alloc_status(m, n)
        assert rc_l == rc_o, (rc_l, rc_o)
        if rc_l == 0:
            assert np.array_equal(ids_l, ids_o)
        return rc_l, ids_l

    def free(self, m, ids):
        assert mx.mux_free_blocks_status(self.lib, m, ids) == self.ora.free_status(m, ids) == 0

    def set_quota(self, m, q):
        rc = mx.mux_pool_set_quota(self.lib, m, q)
        assert rc == self.ora.set_quota(m, q)
        return rc

    def init(self, w):
        rc = mx.mux_pool_init_quotas(self.lib, w)
        assert rc == self.ora.init_quotas(w)
        return rc

    def adapt(self, n, low, high, step):
        got, want = mx.mux_pool_adapt_quotas(self.lib, n, low, high, step), self.ora.adapt_quotas(n, low, high, step)
        if want[0] != 0:
            assert got[0] == want[0]
        else:
            assert got == want
        return got

    def check(self, n_models):
        for m in range(n_models):
            assert mx.mux_pool_get_quota(self.lib, m) == self.ora.get_quota(m)
            assert mx.mux_pool_peak_used(self.lib, m) == self.ora.peak_used(m)
            assert mx.mux_pool_num_used(self.lib, m) == self.ora.num_used(m)
        assert mx.mux_pool_num_free(self.lib) == self.ora.num_free()


def test_quota_status_codes_and_strings():
    assert mx.status_string(mx.MUX_ERR_QUOTA) == "MUX_ERR_QUOTA" and mx.MUX_ERR_QUOTA == orc.ERR_QUOTA == -3
    b = Both(10)
    assert mx.mux_pool_get_quota(b.lib, 0) == -1
    assert b.set_quota(0, 4) == 0
    assert b.alloc(0, 3)[0] == 0
    out = np.full(4, -7, dtype=np.int32)
    rc, ids = mx.mux_alloc_blocks_status(b.lib, 0, 2, out)
    assert rc == mx.MUX_ERR_QUOTA and ids is None and (out == -7).all()       # nothing written
    assert b.alloc(0, 2)[0] == mx.MUX_ERR_QUOTA and b.alloc(0, 100)[0] == mx.MUX_ERR_QUOTA
    assert b.alloc(1, 8)[0] == mx.MUX_ERR_NOMEM
    assert b.set_quota(0, 11) == mx.MUX_ERR_INVALID and b.set_quota(0, -2) == mx.MUX_ERR_INVALID
    assert b.set_quota(2000, 1) == mx.MUX_ERR_INVALID
    assert b.set_quota(0, 2) == 0 and b.alloc(0, 1)[0] == mx.MUX_ERR_QUOTA     # below the holding
    assert b.set_quota(0, -1) == 0 and b.alloc(0, 2)[0] == 0
    b.check(3)
    with pytest.raises(mx.MuxError):
        mx.mux_pool_get_quota(b.lib, -1)


@pytest.mark.parametrize("seed", range(6))
def test_initial_quotas_agree(seed):
    rng = np.random.default_rng(100 + seed)
    for _ in range(60):
        n_models = int(rng.integers(1, 40))
        n_blocks = int(rng.integers(1, 500000))
        b = Both(n_blocks)
        kind = rng.integers(3)
        if kind == 0:
            w = rng.random(n_models) + 1e-6
        elif kind == 1:
            w = rng.integers(0, 4, n_models).astype(np.float64)                 # many exact ties and zeros
            w[int(rng.integers(n_models))] += 1.0
        else:
            w = wl.zipf_shares(n_models, float(rng.choice([0.7, 0.9, 1.3, 1.7, 2.1])))
        assert b.init(w) == 0
        b.check(n_models)
    b = Both(10)
    for bad in ([0.0, 0.0], [1.0, -1.0], [1.0, float("nan")], [float("inf"), 1.0]):
        assert b.init(bad) == mx.MUX_ERR_INVALID
    b.check(2)


@pytest.mark.parametrize("seed", range(4))
def test_quota_traffic_and_adaptation_in_lockstep(seed):
    """Zipf-popular models allocate and free under quotas; every few hundred calls the quotas are
    adapted.  Both managers must agree on every status, id, quota and peak throughout."""
    rng = np.random.default_rng(200 + seed)
    n_models, n_blocks = int(rng.integers(2, 9)), 40000
    order = wl.placement_order(rng, n_blocks)
    b = Both(n_blocks, order)
    rate = wl.zipf_shares(n_models, 1.3)
    blocks_per_token = rng.choice([32, 40, 8], n_models)
    assert b.init(rate * blocks_per_token) == 0
    held = [[] for _ in range(n_models)]
    seen = {0: 0, mx.MUX_ERR_QUOTA: 0, mx.MUX_ERR_NOMEM: 0}
    moved_total = 0
    for it in range(40):
        demand = rng.permutation(n_models)                       # popularity drifts: who is hungry changes
        for _ in range(150):
            m = int(rng.integers(n_models))
            hungry = demand[m] < max(1, n_models // 2)
            if rng.random() < (0.75 if hungry else 0.35):
                rc, ids = b.alloc(m, int(rng.integers(1, 600)))
                seen[rc] += 1
                if rc == 0:
                    held[m].append(ids)
            elif held[m]:
                b.free(m, held[m].pop(int(rng.integers(len(held[m])))))
        low, high, step = [(0.5, 0.9, 0.5), (0.6, 0.8, 0.25), (1.0, 1.0, 1.0), (0.3, 0.3, 0.1)][it % 4]
        rc, moved = b.adapt(n_models, low, high, step)
        assert rc == 0
        moved_total += moved
        b.check(n_models)
        assert sum(mx.mux_pool_get_quota(b.lib, m) for m in range(n_models)) == n_blocks
    assert seen[0] > 0 and seen[mx.MUX_ERR_QUOTA] > 0 and moved_total > 0
    for m in range(n_models):
        for ids in held[m]:
            b.free(m, ids)
    b.check(n_models)
    assert mx.mux_pool_num_free(b.lib) == n_blocks


def test_adaptation_argument_errors_agree():
    b = Both(100)
    assert b.init([1, 1]) == 0
    b.alloc(0, 10)
    for low, high, step in ((-0.1, 0.9, 0.5), (0.9, 0.5, 0.5), (0.5, 0.9, 1.5), (0.5, 0.9, -0.1),
                            (float("nan"), 0.9, 0.5), (0.5, float("inf"), 0.5), (0.5, float("nan"), 0.5)):
        assert b.adapt(2, low, high, step)[0] == mx.MUX_ERR_INVALID
    assert b.adapt(3, 0.5, 0.9, 0.5)[0] == mx.MUX_ERR_INVALID        # model 2 has no quota
    assert b.adapt(0, 0.5, 0.9, 0.5)[0] == mx.MUX_ERR_INVALID
    b.check(3)
    assert mx.mux_pool_peak_used(b.lib, 0) == 10                     # failed calls do not restart the peaks
    # moved may be NULL
    assert mx.load().mux_pool_adapt_quotas(b.lib.handle, 2, 0.5, 0.9, 0.5, None) == 0
