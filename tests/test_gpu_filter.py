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


@pytest.mark.parametrize("expire_steps", [0, 3])
@pytest.mark.parametrize("thr,hashes", [(255, 1), (200, 2), (1, 1)])
def test_counters_saturate_at_255_on_shared_words(dev, expire_steps, thr, hashes):
    """Sixteen counters for forty keys, hundreds of occurrences per key and batch: every word runs far
    past 255 (the device keeps counts unsaturated and reads them as min(count, 255)), keys below the
    threshold keep missing on saturated words, later batches touch them again, and with expiry the
    words age in between.  Words, presence and the expired sets must equal the oracle's every step."""
    from paper_2209_07663_amd.binding import Table
    seed, cap, dim = 131, 1 << 10, 4
    tab = Table(cap, dim, seed, freq_threshold=thr, expire_steps=expire_steps, max_ids=1 << 15, max_bags=1 << 15,
                device=dev, filter_hashes=hashes, filter_log2=4)
    orc = Oracle(cap, dim, seed, thr, expire_steps, False, kind="cuckoo", n_filter=16, filter_hashes=hashes)
    rng = np.random.default_rng(7)
    universe = (np.arange(40, dtype=np.int64) + 11) * 104729
    for step in (0, 1, 2, 3, 7, 8, 20):                          # gaps let words and keys age
        reps = rng.integers(1, 400, size=universe.shape[0])      # some keys below any threshold, some far above
        reps[rng.integers(0, 40, size=10)] = 0
        keys_h = np.repeat(universe, reps)
        keys_h = keys_h[rng.permutation(keys_h.shape[0])]
        offs_h = np.arange(keys_h.shape[0] + 1, dtype=np.int64)
        compare_step(tab, orc, {"keys": keys_h, "offsets": offs_h, "step": step}, dev, 1e-5, exact_rows=True,
                     train=False, sweep_at=step if expire_steps else None)
        words = tab.mono_filter_export()
        assert (words == orc.filter_words()).all(), "counter words differ at step %d" % step
    assert ((words & 255) == 255).any()
    tab.close()
