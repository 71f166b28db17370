"""Seeded synthetic inputs shared by the device library's tests/benchmark and the CPU oracle.

This module holds none of the table's arithmetic: it only draws sparse-feature ID batches with the
shapes of the paper's workloads (multi-hot categorical slots per sample, long-tail distributed IDs:
section 2.1, "IDs are long-tail distributed"; 26 slots stand in for the categorical fields of the
public display-ads dataset of section 3.1) and pooled upstream gradients.  No record of any dataset
is reproduced; everything is drawn from numpy's PCG64 with a SeedSequence of (seed, workload, step).
"""
from dataclasses import dataclass, replace

import numpy as np

_M1 = np.uint64(0xD6E8FEB86659FD93)  # odd multipliers of the ID scramble (not the table's mixer)
_M2 = np.uint64(0xA5A5A5A5A5A5A5A5 | 1)


@dataclass(frozen=True)
class Workload:
    name: str
    wid: int                # enters the seed sequence
    capacity: int           # table slots = rows (power of two)
    dim: int
    bf16: bool
    freq_threshold: int
    expire_steps: int
    samples: int
    slots: int
    poisson_lam: float      # bag length = Poisson(lam) + 1; 0 -> exactly one ID per bag
    dist: str               # "uniform" | "zipf"
    alpha: float            # Zipf exponent (unused for uniform)
    universe_bits: int      # IDs live in [0, 2^universe_bits)
    grad_sigma: float = 0.1  # pooled upstream gradients ~ N(0, sigma^2); "N(0,1e-2)" read as variance
    lr: float = 0.05
    eps: float = 1e-8
    drift_frac: float = 0.0  # fraction of the tracked hot ranks whose IDs are permuted each step
    drift_ranks: int = 0     # number of hottest ranks whose rank -> ID map is kept explicitly

    @property
    def n_bags(self):
        return self.samples * self.slots


# The five configurations of the build's problem statement.  cfg1 draws uniform IDs from [0, 2^20).
CONFIGS = {
    "cfg1": Workload("cfg1", 1, 1 << 16, 16, False, 1, 0, 4096, 1, 0.0, "uniform", 0.0, 20),
    "cfg2": Workload("cfg2", 2, 1 << 24, 32, False, 3, 0, 65536, 26, 3.0, "zipf", 1.05, 32),
    "cfg3": Workload("cfg3", 3, 1 << 26, 64, False, 1, 0, 131072, 40, 4.0, "zipf", 1.1, 40),
    "cfg4": Workload("cfg4", 4, 1 << 25, 32, False, 5, 20, 65536, 26, 3.0, "zipf", 1.1, 40,
                     drift_frac=0.05, drift_ranks=1 << 26),
    "cfg5": Workload("cfg5", 5, 1 << 28, 64, True, 2, 50, 262144, 4, 0.0, "zipf", 1.2, 63),
}

# The batch shape of cfg2 over the 2^48 ID space of the paper's production model (section 3.1), for the
# quotient-remainder embedding (two dense tables of 2^24 rows; no table object, so capacity etc. are unused).
QR_WORKLOAD = Workload("qr", 6, 1 << 25, 32, False, 0, 0, 65536, 26, 3.0, "zipf", 1.05, 48)


def scaled(wl, samples, capacity, drift_ranks=None):
    """Same distributions, smaller batch and table: parity-test sized variants of a configuration."""
    return replace(wl, name="%s@%dx%d" % (wl.name, samples, capacity), samples=samples, capacity=capacity,
                   drift_ranks=wl.drift_ranks if drift_ranks is None else drift_ranks)


def _rng(seed, wl, step, stream=0):
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, wl.wid, step, stream])))


def scramble(x, bits):
    """Bijection of [0, 2^bits): hot ranks must not be neighbouring integers."""
    mask = np.uint64((1 << bits) - 1) if bits < 64 else np.uint64(0xFFFFFFFFFFFFFFFF)
    s = np.uint64(bits // 2 + 1)
    x = np.asarray(x, dtype=np.uint64)
    x = (x * _M1) & mask
    x = x ^ (x >> s)
    x = (x * _M2) & mask
    x = x ^ (x >> s)
    return x


def zipf_ranks(rng, alpha, universe, size):
    """Ranks r in [1, universe] with P(r) ~ r^-alpha (numpy's Zipf sampler, truncated by rejection)."""
    out = np.empty(size, dtype=np.int64)
    universe = min(int(universe), int(np.iinfo(np.int64).max))
    filled = 0
    while filled < size:
        need = size - filled
        draw = rng.zipf(alpha, int(need * 1.6) + 16)
        draw = draw[(draw >= 1) & (draw <= universe)][:need]
        out[filled:filled + draw.shape[0]] = draw
        filled += draw.shape[0]
    return out


class DriftMap:
    """Explicit rank -> ID map of the `drift_ranks` hottest ranks; each step a seeded sample of
    `drift_frac` of those ranks has its IDs permuted among themselves, so the hot set rotates."""

    def __init__(self, wl, seed):
        self.wl, self.seed = wl, seed
        self.ids = scramble(np.arange(wl.drift_ranks, dtype=np.uint64), wl.universe_bits)
        self.step_done = -1

    def advance_to(self, step):
        while self.step_done < step:
            self.step_done += 1
            if self.step_done == 0:
                continue
            rng = _rng(self.seed, self.wl, self.step_done, stream=1)
            k = int(self.wl.drift_ranks * self.wl.drift_frac)
            pick = rng.choice(self.wl.drift_ranks, size=k, replace=False)
            self.ids[pick] = self.ids[rng.permutation(pick)]

    def map(self, ranks):
        r0 = ranks - 1
        ids = scramble(r0.astype(np.uint64), self.wl.universe_bits)
        hot = r0 < self.wl.drift_ranks
        ids[hot] = self.ids[r0[hot]]
        return ids


def make_batch(wl, seed, step, with_grad=False, drift=None):
    """One batch: keys int64[N], offsets int64[n_bags + 1] and, if asked, grad float32[n_bags, dim].

    `drift` (a DriftMap) must be passed for workloads with drift_frac > 0 and is advanced to `step`.
    """
    rng = _rng(seed, wl, step)
    n_bags = wl.n_bags
    if wl.poisson_lam > 0:
        lengths = rng.poisson(wl.poisson_lam, n_bags).astype(np.int64) + 1
    else:
        lengths = np.ones(n_bags, dtype=np.int64)
    offsets = np.zeros(n_bags + 1, dtype=np.int64)
    np.cumsum(lengths, out=offsets[1:])
    n = int(offsets[-1])
    if wl.dist == "uniform":
        keys = rng.integers(0, 1 << wl.universe_bits, size=n, dtype=np.int64)
    else:
        ranks = zipf_ranks(rng, wl.alpha, 1 << wl.universe_bits, n)
        if wl.drift_frac > 0:
            drift.advance_to(step)
            keys = drift.map(ranks).astype(np.int64)
        else:
            keys = scramble((ranks - 1).astype(np.uint64), wl.universe_bits).astype(np.int64)
    batch = {"keys": keys, "offsets": offsets, "step": step}
    if with_grad:
        g = _rng(seed, wl, step, stream=2).standard_normal((n_bags, wl.dim), dtype=np.float32)
        g *= np.float32(wl.grad_sigma)
        batch["grad"] = g
    return batch


def hottest_ids(wl, count, drift=None):
    """IDs of ranks 1..count (used to pre-fill a table to a target load factor)."""
    ranks = np.arange(1, count + 1, dtype=np.int64)
    if wl.drift_frac > 0:
        return drift.map(ranks).astype(np.int64)
    return scramble((ranks - 1).astype(np.uint64), wl.universe_bits).astype(np.int64)
