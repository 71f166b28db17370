"""The seeded workload generator (CPU only): it feeds the oracle and the device alike, so what matters
is that it is reproducible, has the stated shapes and distributions, and that its ID maps are bijections."""
from dataclasses import replace

import numpy as np

from paper_2209_07663_amd import synth


def test_batches_are_reproducible_and_differ_by_seed_and_step():
    wl = synth.scaled(synth.CONFIGS["cfg2"], samples=512, capacity=1 << 16)
    a, b = synth.make_batch(wl, 3, 5, with_grad=True), synth.make_batch(wl, 3, 5, with_grad=True)
    for k in ("keys", "offsets", "grad"):
        assert (a[k] == b[k]).all()
    c, d = synth.make_batch(wl, 3, 6, with_grad=True), synth.make_batch(wl, 4, 5, with_grad=True)
    assert not np.array_equal(a["keys"], c["keys"]) and not np.array_equal(a["keys"], d["keys"])
    assert not np.array_equal(a["grad"], c["grad"])


def test_shapes_lengths_and_ranges_of_the_named_configurations():
    for name, lam, bits in [("cfg1", 0.0, 20), ("cfg2", 3.0, 32), ("cfg3", 4.0, 40), ("cfg5", 0.0, 63)]:
        wl = synth.scaled(synth.CONFIGS[name], samples=2048, capacity=1 << 16)
        b = synth.make_batch(wl, 1, 0, with_grad=True)
        lens = np.diff(b["offsets"])
        assert b["offsets"][0] == 0 and b["offsets"][-1] == b["keys"].shape[0] and (lens >= 1).all()
        assert lens.shape[0] == wl.n_bags == 2048 * wl.slots and b["grad"].shape == (wl.n_bags, wl.dim)
        assert abs(lens.mean() - (lam + 1)) < 0.05 * (lam + 1)              # Poisson(lam) + 1, or exactly 1
        if lam == 0:
            assert (lens == 1).all()
        assert (b["keys"] >= 0).all() and int(b["keys"].max()).bit_length() <= bits
        assert abs(float(b["grad"].std()) - wl.grad_sigma) < 0.02 * wl.grad_sigma and b["grad"].dtype == np.float32


def test_zipf_ranks_follow_the_power_law_and_the_truncation():
    rng = np.random.default_rng(0)
    r = synth.zipf_ranks(rng, 1.05, 1 << 32, 400000)
    assert r.min() >= 1 and r.max() <= 1 << 32
    c1, c2, c4 = (r == 1).sum(), (r == 2).sum(), (r == 4).sum()
    assert abs(c1 / c2 - 2 ** 1.05) < 0.08 and abs(c2 / c4 - 2 ** 1.05) < 0.12    # P(r) ~ r^-alpha
    small = synth.zipf_ranks(rng, 1.2, 1000, 50000)
    assert small.max() <= 1000


def test_scramble_is_a_bijection_that_separates_neighbours():
    for bits in (8, 12, 16):
        x = np.arange(1 << bits, dtype=np.uint64)
        y = synth.scramble(x, bits)
        assert np.unique(y).shape[0] == 1 << bits and int(y.max()) < 1 << bits
    y = synth.scramble(np.arange(1000, dtype=np.uint64), 32).astype(np.int64)
    assert np.abs(np.diff(y)).min() > 1000                                    # hot ranks are not neighbouring IDs


def test_drift_map_permutes_a_fraction_of_the_hot_ranks_per_step_and_stays_a_bijection():
    wl = replace(synth.scaled(synth.CONFIGS["cfg4"], samples=64, capacity=1 << 12, drift_ranks=1 << 12), drift_frac=0.05)
    m = synth.DriftMap(wl, 9)
    ranks = np.arange(1, (1 << 12) + 1, dtype=np.int64)
    before = m.map(ranks).copy()
    m.advance_to(1)
    after = m.map(ranks)
    moved = (before != after).sum()
    assert 0 < moved <= int(0.05 * (1 << 12))                                 # at most the sampled 5 % moved
    assert sorted(before.tolist()) == sorted(after.tolist())                  # among themselves: still a bijection
    m2 = synth.DriftMap(wl, 9)
    m2.advance_to(1)
    assert (m2.map(ranks) == after).all()                                     # reproducible
    cold = np.array([(1 << 12) + 5, 1 << 20], dtype=np.int64)
    assert (m.map(cold) == synth.scramble((cold - 1).astype(np.uint64), wl.universe_bits)).all()


def test_hottest_ids_are_the_ids_of_the_lowest_ranks():
    wl = synth.scaled(synth.CONFIGS["cfg2"], samples=64, capacity=1 << 12)
    hot = synth.hottest_ids(wl, 100)
    assert (hot == synth.scramble(np.arange(100, dtype=np.uint64), wl.universe_bits).astype(np.int64)).all()
    b = synth.make_batch(wl, 1, 0)
    top = np.bincount(np.searchsorted(np.sort(hot), b["keys"][np.isin(b["keys"], hot)])).max()
    assert np.isin(b["keys"], hot).mean() > 0.2 and top > 10                   # the lowest ranks carry the mass
