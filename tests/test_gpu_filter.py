"""The occurrence filter with several hashes per key on the device against the oracle (needs an MI355X).
Small counter arrays on purpose: keys share counters, so over-counting, the minimum over a key's
counters and two hashes of a key falling on one counter all occur."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import Oracle
from paper_2209_07663_amd import synth
from tests.test_gpu_parity import compare_step

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "gpu tests need a GPU"
    return torch.device("cuda:0")


def _workload(name):
    if name == "forward":       # configs[1] shapes: threshold 3, nothing ages (counters double as a negative lookup)
        return synth.scaled(synth.CONFIGS["cfg2"], samples=2048, capacity=1 << 20)   # room even if all is admitted
    return replace(synth.scaled(synth.CONFIGS["cfg4"], samples=1024, capacity=1 << 18, drift_ranks=1 << 14),
                   expire_steps=3, freq_threshold=3, drift_frac=0.3)  # ageing counters, expiry, drifting hot set


@pytest.mark.parametrize("name", ["forward", "drift"])
@pytest.mark.parametrize("hashes,filter_log2", [(2, 0), (3, 13), (4, 16), (2, 6)])
def test_multi_hash_filter_matches_the_oracle(dev, name, hashes, filter_log2):
    from paper_2209_07663_amd.binding import Table
    wl, seed = _workload(name), 101 + hashes
    tab = Table(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, max_ids=1 << 18,
                max_bags=wl.n_bags, device=dev, filter_hashes=hashes, filter_log2=filter_log2)
    orc = Oracle(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, kind="cuckoo",
                 n_filter=tab.n_filter, filter_hashes=hashes)
    drift = synth.DriftMap(wl, seed) if wl.drift_frac > 0 else None
    admitted = []
    for step in range(6):
        b = synth.make_batch(wl, seed, step, with_grad=True, drift=drift)
        compare_step(tab, orc, b, dev, 1e-5, exact_rows=False, train=True, lr=wl.lr, eps=wl.eps,
                     sweep_at=step if wl.expire_steps else None)
        assert (tab.mono_filter_export() == orc.filter_words()).all(), "counter words differ at step %d" % step
        admitted.append(tab.mono_table_stats()["n_admitted"])
    assert admitted[-1] > 0
    tab.close()


def test_growing_a_table_with_a_multi_hash_filter(dev):
    from paper_2209_07663_amd.binding import Table
    wl, seed, hashes = _workload("drift"), 111, 2
    tab = Table(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, max_ids=1 << 18,
                max_bags=wl.n_bags, device=dev, filter_hashes=hashes, filter_log2=12)
    orc = Oracle(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, kind="cuckoo",
                 n_filter=1 << 12, filter_hashes=hashes)
    drift = synth.DriftMap(wl, seed)
    batches = [synth.make_batch(wl, seed, s, with_grad=True, drift=drift) for s in range(6)]
    for b in batches[:3]:
        compare_step(tab, orc, b, dev, 1e-5, exact_rows=False, train=True, sweep_at=b["step"])
    big = tab.rehashed(wl.capacity * 2, 0)                  # same hash functions, twice the room
    orc.rehash(wl.capacity * 2, 0)
    tab.close()
    assert big.n_filter == 1 << 13 and (big.mono_filter_export() == orc.filter_words()).all()
    for b in batches[3:]:
        compare_step(big, orc, b, dev, 1e-5, exact_rows=False, train=True, sweep_at=b["step"])
        assert (big.mono_filter_export() == orc.filter_words()).all()
    big.close()
