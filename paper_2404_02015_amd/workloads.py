"""Seeded synthetic workloads shaped like MuxServe's colocations.

This module only draws inputs: model shapes, popularity shares, context lengths,
block placement, the order of allocator calls, and random K/V/Q values.  It holds
none of the method's arithmetic and imports neither the GPU library nor the CPU
oracle; tests and the benchmark hand the same bits it produces to both.

Where the numbers come from:
  - model shapes follow the LLaMA size buckets of Table 1 (7B: 32 heads, 13B: 40
    heads, 65B-shaped GQA: 64 query / 8 KV heads; head size 128, Section 3.4);
  - request popularity follows a power law with exponent alpha (Section 4.2,
    "Workloads"): rate_i proportional to i^-alpha for the i-th listed model.  With
    19 models this reproduces the paper's statement that alpha = 0.9 / 2.1 gives the
    top 20 % of models about 50 % / 90 % of the traffic;
  - the paper draws request lengths from ShareGPT and a ChatLMSYS trace, which are
    not available here; uniform / log-normal context lengths stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence

import numpy as np

BASE_SEED = 20240402


# ----------------------------------------------------------------------------------
# shapes and shares
# ----------------------------------------------------------------------------------
@dataclass(frozen=True)
class ModelShape:
    name: str
    n_q_heads: int
    n_kv_heads: int
    head_dim: int

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


LLAMA_7B = ModelShape("7B", 32, 32, 128)
LLAMA_13B = ModelShape("13B", 40, 40, 128)
GQA_65B = ModelShape("65B-GQA", 64, 8, 128)


def zipf_shares(n: int, alpha: float) -> np.ndarray:
    """Popularity shares rate_i ~ i^-alpha, i = 1..n, normalised to 1."""
    r = np.arange(1, n + 1, dtype=np.float64) ** (-alpha)
    return r / r.sum()


def largest_remainder(total: int, shares: Sequence[float]) -> List[int]:
    """Split `total` items by `shares`; leftovers go to the largest fractional parts."""
    raw = np.asarray(shares, dtype=np.float64) * total
    base = np.floor(raw).astype(np.int64)
    left = int(total - base.sum())
    order = np.argsort(-(raw - base), kind="stable")
    for k in range(left):
        base[order[k]] += 1
    return [int(x) for x in base]


def uniform_lengths(rng: np.random.Generator, n: int, lo: int, hi: int) -> np.ndarray:
    """n integers uniform in the inclusive range [lo, hi]."""
    return rng.integers(lo, hi + 1, size=n).astype(np.int32)


def lognormal_lengths(rng: np.random.Generator, n: int, mu: float, sigma: float, lo: int, hi: int) -> np.ndarray:
    z = rng.standard_normal(n)
    return np.clip(np.rint(np.exp(mu + sigma * z)), lo, hi).astype(np.int32)


# ----------------------------------------------------------------------------------
# workload description
# ----------------------------------------------------------------------------------
@dataclass
class ModelJob:
    model_id: int
    shape: ModelShape
    kind: str                       # "decode" or "prefill"
    lens: np.ndarray                # decode: post-append context lengths; prefill: prompt lengths
    chunk: int = 0                  # prefill chunk size

    @property
    def n_seqs(self) -> int:
        return int(self.lens.size)


@dataclass
class Workload:
    name: str
    seed: int
    block_size: int
    head_dim: int
    num_blocks: int                 # <= 0: sized at run time from free device memory
    placement: str                  # "permutation" or "churn"
    jobs: List[ModelJob] = field(default_factory=list)
    hbm_fraction: float = 0.0       # used when num_blocks <= 0
    churn_ops: int = 0

    def rng(self) -> np.random.Generator:
        return np.random.Generator(np.random.PCG64(self.seed))

    def demand_blocks(self) -> int:
        b = self.block_size
        return int(sum(int(((j.lens.astype(np.int64) + b - 1) // b).sum()) * j.shape.n_kv_heads for j in self.jobs))


def _blocks_with_headroom(demand: int, headroom: float = 1.25) -> int:
    return int(-(-int(demand * headroom) // 8192) * 8192)


def config(index: int, *, small: bool = False) -> Workload:
    """The five benchmark configurations (1-based).  `small=True` shrinks sequence
    counts and lengths (same structure) so the CPU oracle can check every output."""
    seed = BASE_SEED + index
    rng = np.random.Generator(np.random.PCG64(seed))
    if index == 1:
        a = ModelShape("A", 8, 8, 64)
        b = ModelShape("B", 4, 4, 64)
        jobs = [ModelJob(0, a, "decode", uniform_lengths(rng, 4, 1, 128)),
                ModelJob(1, b, "decode", uniform_lengths(rng, 4, 1, 128))]
        return Workload("cfg1", seed, 16, 64, 1024, "permutation", jobs)
    if index == 2:
        n, lo, hi = (6, 128, 512) if small else (64, 128, 2048)
        jobs = [ModelJob(0, LLAMA_7B, "decode", uniform_lengths(rng, n, lo, hi)),
                ModelJob(1, LLAMA_7B, "decode", uniform_lengths(rng, n, lo, hi))]
        # The configuration names 200 000 head-blocks, which is less than the ~280 000
        # the sequences need; the timed run uses 327 680 and a separate test drives the
        # 200 000-block pool into its out-of-memory path.
        w = Workload("cfg2", seed, 16, 128, 327680, "permutation", jobs)
        if small:
            w.num_blocks = _blocks_with_headroom(w.demand_blocks())
        return w
    if index == 3:
        total = 24 if small else 256
        counts = largest_remainder(total, zipf_shares(3, 0.9))
        hi = 600 if small else 4096
        mu = 5.0 if small else 6.5
        jobs = [ModelJob(m, shp, "decode", lognormal_lengths(rng, counts[m], mu, 0.8, 16, hi))
                for m, shp in enumerate((LLAMA_7B, LLAMA_13B, GQA_65B))]
        w = Workload("cfg3", seed, 16, 128, 0, "permutation", jobs)
        w.num_blocks = _blocks_with_headroom(w.demand_blocks())
        return w
    if index == 4:
        n_p, p_lo, p_hi, chunk = (3, 40, 200, 64) if small else (8, 512, 2048, 512)
        n_d, d_lo, d_hi = (5, 64, 400) if small else (128, 256, 4096)
        jobs = [ModelJob(0, LLAMA_13B, "prefill", uniform_lengths(rng, n_p, p_lo, p_hi), chunk),
                ModelJob(1, LLAMA_7B, "decode", uniform_lengths(rng, n_d, d_lo, d_hi)),
                ModelJob(2, GQA_65B, "decode", uniform_lengths(rng, n_d, d_lo, d_hi))]
        w = Workload("cfg4", seed, 16, 128, 0, "permutation", jobs)
        w.num_blocks = _blocks_with_headroom(w.demand_blocks())
        return w
    if index == 5:
        total = 16 if small else 512
        counts = largest_remainder(total, zipf_shares(4, 1.2))
        lo, hi = (64, 1024) if small else (1024, 16384)
        jobs = [ModelJob(m, shp, "decode", uniform_lengths(rng, counts[m], lo, hi))
                for m, shp in enumerate((LLAMA_7B, LLAMA_7B, LLAMA_13B, GQA_65B))]
        w = Workload("cfg5", seed, 16, 128, 0, "churn", jobs, hbm_fraction=0.8, churn_ops=10000)
        if small:
            w.num_blocks = _blocks_with_headroom(w.demand_blocks(), 1.5)
            w.churn_ops = 300
        return w
    raise ValueError("config index must be 1..5")


# ----------------------------------------------------------------------------------
# placement: the order of block-manager calls (run identically on any allocator)
# ----------------------------------------------------------------------------------
def placement_order(rng: np.random.Generator, num_blocks: int) -> np.ndarray:
    """A seeded permutation of the block ids: the order a fresh pool hands them out."""
    return rng.permutation(num_blocks).astype(np.int32)


def run_churn(rng: np.random.Generator, n_ops: int, max_n: int,
              alloc: Callable[[int, int], Optional[np.ndarray]],
              free: Callable[[int, np.ndarray], None], n_models: int = 4) -> int:
    """Seeded alloc/free churn that fragments the free list before a measurement.

    Operation k is, with probability 1/2, an allocation of a size uniform in
    [1, max_n] for a random model (skipped when `alloc` returns None, i.e. the pool is
    short), else a release of one live allocation, its ids in shuffled order.  At the
    end everything still live is released, again shuffled.  Returns the number of
    operations that took effect."""
    live: List[tuple] = []
    done = 0
    for _ in range(n_ops):
        do_alloc = rng.random() < 0.5
        if do_alloc or not live:
            n = int(rng.integers(1, max_n + 1))
            m = int(rng.integers(0, n_models))
            ids = alloc(m, n)
            if ids is not None:
                live.append((m, np.array(ids, dtype=np.int32, copy=True)))
                done += 1
        else:
            k = int(rng.integers(0, len(live)))
            m, ids = live.pop(k)
            free(m, rng.permutation(ids))
            done += 1
    while live:
        k = int(rng.integers(0, len(live)))
        m, ids = live.pop(k)
        free(m, rng.permutation(ids))
    return done


def max_blocks_for(lens: np.ndarray, block_size: int, extra_tokens: int = 0) -> int:
    return int((int(lens.max()) + extra_tokens + block_size - 1) // block_size) if lens.size else 1


def build_tables(alloc: Callable[[int, int], np.ndarray], model_id: int, lens: np.ndarray,
                 n_kv_heads: int, block_size: int, max_blocks: int) -> np.ndarray:
    """Block tables [n_seqs][n_kv_heads][max_blocks] (int32, unused entries -1) for
    sequences that hold `lens` tokens.  One allocator call per sequence; the ids come
    back head-major: ids[h * n_blocks + j] is block j of kv head h."""
    n_seqs = int(lens.size)
    tables = np.full((n_seqs, n_kv_heads, max_blocks), -1, dtype=np.int32)
    for s in range(n_seqs):
        nb = int((int(lens[s]) + block_size - 1) // block_size)
        if nb == 0:
            continue
        ids = np.asarray(alloc(model_id, nb * n_kv_heads), dtype=np.int32)
        tables[s, :, :nb] = ids.reshape(n_kv_heads, nb)
    return tables


def grow_tables(alloc: Callable[[int, int], np.ndarray], model_id: int, tables: np.ndarray,
                old_lens: np.ndarray, new_lens: np.ndarray, block_size: int, want_changed: bool = True) -> np.ndarray:
    """Extend `tables` in place for sequences growing from old_lens to new_lens tokens.
    One allocator call per sequence that needs blocks, ids head-major as in build_tables.
    Returns the flat indices of the entries that changed."""
    n_seqs, n_kv, max_blocks = tables.shape
    changed = []
    for s in range(n_seqs):
        nb0 = int((int(old_lens[s]) + block_size - 1) // block_size)
        nb1 = int((int(new_lens[s]) + block_size - 1) // block_size)
        if nb1 <= nb0:
            continue
        ids = np.asarray(alloc(model_id, (nb1 - nb0) * n_kv), dtype=np.int32)
        tables[s, :, nb0:nb1] = ids.reshape(n_kv, nb1 - nb0)
        for h in range(n_kv if want_changed else 0):
            base = (s * n_kv + h) * max_blocks
            changed.extend(range(base + nb0, base + nb1))
    return np.asarray(changed, dtype=np.int64)


# ----------------------------------------------------------------------------------
# values
# ----------------------------------------------------------------------------------
def randn_values(seed: int, shape, dtype: str = "bf16"):
    """N(0,1) values drawn in fp32 on the CPU and rounded once (nearest-even) to the
    storage type.  Returns a torch CPU tensor (bfloat16 or float32)."""
    import torch

    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    x = torch.randn(*shape, generator=g, dtype=torch.float32)
    return x.to(torch.bfloat16) if dtype == "bf16" else x


def as_bits(t):
    """numpy view of a torch CPU tensor as the oracle takes it: uint16 for bf16."""
    import torch

    t = t.contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()
