"""Full-size configurations on the device, in the launch configuration bench.py times.

Every configuration runs whole against the oracle on the same seeded batches: presence of every
occurrence, every pooled row, refused counts, expired sets, and at the end the whole table (keys,
last-seen steps, rows, accumulators, placement) and every counter word.
"""
import numpy as np
import pytest
import torch

from oracle import Oracle
from paper_2209_07663_amd import synth
from tests import table_checks as tc

pytestmark = pytest.mark.gpu


def _table(wl, seed, max_ids, dev):
    from paper_2209_07663_amd.binding import Table
    return Table(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, max_ids=max_ids,
                 max_bags=wl.n_bags, device=dev)


@pytest.mark.timeout(900)
def test_config2_full_size_against_oracle(say):
    dev = torch.device("cuda:0")
    wl, seed = synth.CONFIGS["cfg2"], 1
    batches = [synth.make_batch(wl, seed, s, with_grad=True) for s in range(3)]
    tab = _table(wl, seed, max(b["keys"].shape[0] for b in batches), dev)
    orc = Oracle(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, kind="cuckoo")
    for b in batches:
        say("config2 full size, step", b["step"])
        keys, offs = torch.from_numpy(b["keys"]).to(dev), torch.from_numpy(b["offsets"]).to(dev)
        rows = tab.mono_lookup_or_insert(keys, b["step"])
        present = orc.lookup_or_insert(b["keys"], b["step"])
        assert ((rows.cpu().numpy() >= 0) == present).all()
        pooled = tab.mono_gather_pool(rows, offs).cpu().numpy()
        tc.rows_close(pooled, orc.pool(b["keys"], b["offsets"]), 1e-5)
        tab.mono_apply_grad_adagrad(rows, offs, torch.from_numpy(b["grad"]).to(dev), wl.lr, wl.eps)
        orc.apply_grad_adagrad(b["keys"], b["offsets"], b["grad"], wl.lr, wl.eps)
        tab.mono_expire_sweep(b["step"])
        assert orc.expire_sweep(b["step"]).shape[0] == 0
        d = tab.mono_table_export()
        tc.assert_same_table(d, orc.dump(), exact_rows=False, rtol=1e-5)
        tc.check_placement(d, wl.capacity, 8, seed)
    assert (tab.mono_filter_export() == orc.filter_words()).all()
    st = tab.mono_table_stats()
    assert st["n_insert_failed"] == 0 and st["n_lost"] == 0 and st["n_full"] == 0 and orc.insert_failures == 0
    tab.close()


def _full_step_against_oracle(tab, orc, b, dev, wl, rtol, sweep, out_buf):
    """One whole step on both sides at full size: presence of every occurrence, every pooled row, the update,
    and (if asked) the sweep with its set of expired keys."""
    step = b["step"]
    keys, offs = torch.from_numpy(b["keys"]).to(dev), torch.from_numpy(b["offsets"]).to(dev)
    rows = tab.mono_lookup_or_insert(keys, step)
    present = orc.lookup_or_insert(b["keys"], step)
    assert ((rows.cpu().numpy() >= 0) == present).all(), "presence differs at step %d" % step
    pooled = tab.mono_gather_pool(rows, offs).cpu().numpy()
    tc.rows_close(pooled, orc.pool(b["keys"], b["offsets"]), rtol)
    del pooled
    tab.mono_apply_grad_adagrad(rows, offs, torch.from_numpy(b["grad"]).to(dev), wl.lr, wl.eps)
    orc.apply_grad_adagrad(b["keys"], b["offsets"], b["grad"], wl.lr, wl.eps)
    n = 0
    if sweep:
        n_exp = torch.zeros(1, dtype=torch.int64, device=dev)
        tab.mono_expire_sweep(step, n_exp, out_buf)
        want = orc.expire_sweep(step)
        n = int(n_exp.item())
        assert n == want.shape[0], "expired counts differ at step %d: %d vs %d" % (step, n, want.shape[0])
        if n:
            got = np.sort(out_buf[:n].cpu().numpy().view(np.uint64)).view(np.int64)
            assert (got == want).all(), "expired sets differ at step %d" % step
    st = tab.mono_table_stats()
    assert st["n_insert_failed"] == 0 and st["n_lost"] == 0 and orc.insert_failures == 0
    assert st["n_full"] == orc.refused_full
    return n, st


def _whole_tables_equal(tab, orc, wl, seed, rtol):
    d = tab.mono_table_export()
    tc.check_placement(d, wl.capacity, 8, seed)
    tc.assert_same_table(d, orc.dump(), exact_rows=False, rtol=rtol)
    del d
    assert (tab.mono_filter_export() == orc.filter_words()).all(), "counter words differ"


@pytest.mark.timeout(900)
def test_config3_full_size_against_oracle(say):
    """configs[2] whole against the oracle: 131072 samples x 40 slots (26 M IDs per step), dim 64, Adagrad,
    two steps from the empty table (about 4 M keys admitted per step); whole table, every pooled row and
    every counter word compared."""
    dev = torch.device("cuda:0")
    wl, seed = synth.CONFIGS["cfg3"], 3
    tab, orc = None, Oracle(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, kind="cuckoo")
    for step in range(2):
        say("config3 full size, step", step)
        b = synth.make_batch(wl, seed, step, with_grad=True)
        if tab is None:
            tab = _table(wl, seed, int(b["keys"].shape[0] * 1.05) + 1024, dev)
        _full_step_against_oracle(tab, orc, b, dev, wl, 1e-5, sweep=False, out_buf=None)
    say("config3 full size, comparing the tables")
    _whole_tables_equal(tab, orc, wl, seed, 1e-5)
    assert tab.mono_table_stats()["size"] > 5_000_000
    tab.close()


@pytest.mark.timeout(900)
def test_config5_full_size_against_oracle(say):
    """configs[4] whole against the oracle: capacity 2^28, bf16 rows of dim 64, threshold 2, one ID per bag,
    1 M IDs per step; three steps with a sweep each (nothing is 50 steps old yet: the scaled run in
    test_gpu_parity.py crosses the expiry), whole table (rows within the bf16 tolerance), all 2^30 counter
    words and every pooled row compared."""
    dev = torch.device("cuda:0")
    wl, seed = synth.CONFIGS["cfg5"], 5
    orc = Oracle(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, kind="cuckoo")
    tab = _table(wl, seed, wl.n_bags, dev)
    out = torch.zeros(1 << 20, dtype=torch.int64, device=dev)
    for step in range(3):
        say("config5 full size, step", step)
        b = synth.make_batch(wl, seed, step, with_grad=True)
        n, st = _full_step_against_oracle(tab, orc, b, dev, wl, 1e-2, sweep=True, out_buf=out)
        assert n == 0
    say("config5 full size, comparing the tables")
    _whole_tables_equal(tab, orc, wl, seed, 1e-2)
    assert tab.mono_table_stats()["size"] > 50_000
    tab.close()


@pytest.mark.timeout(1100)
def test_config4_full_size_as_specified_through_the_fill_limit_and_the_first_expiry(say):
    """configs[3] exactly as the benchmark spec states it, at full size, against the oracle: capacity 2^25, the
    0.9 * capacity hottest IDs admitted first (threshold 5: each is looked up five times, on both sides),
    then 21 drifting batches (5 % of the hot ranks permuted per step) with a sweep after every step and an
    expiry time of 20 steps.  The load climbs to the fill limit (0.9645 < 31/32 at step 12); from step 13
    on every batch's new keys are refused whole, on both sides alike; the sweep of step 20 removes the 23 M
    keys of the fill that were never seen again, and step 21 admits again.  Presence, pooled rows, refused
    counts and expired sets at every step; whole table and counter words at the end."""
    dev = torch.device("cuda:0")
    wl, seed = synth.CONFIGS["cfg4"], 4
    assert wl.freq_threshold == 5 and wl.expire_steps == 20 and wl.drift_frac == 0.05
    drift = synth.DriftMap(wl, seed)
    hot = synth.hottest_ids(wl, int(0.9 * wl.capacity), drift)
    max_ids = 1 << 23
    tab = _table(wl, seed, max_ids, dev)
    orc = Oracle(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, kind="cuckoo")
    rows = torch.empty(max_ids, dtype=torch.int32, device=dev)
    for lo in range(0, hot.shape[0], max_ids):
        chunk = hot[lo:lo + max_ids]
        dchunk = torch.from_numpy(chunk).to(dev)
        for rep in range(wl.freq_threshold):
            tab.mono_lookup_or_insert(dchunk, 0, rows[: chunk.shape[0]])
            present = orc.lookup_or_insert(chunk, 0)
        assert ((rows[: chunk.shape[0]].cpu().numpy() >= 0) == present).all() and present.all()
        say("config4 full size: filled chunk at", lo)
    assert tab.mono_table_stats()["size"] == hot.shape[0]
    out = torch.zeros(wl.capacity, dtype=torch.int64, device=dev)
    expired, refused, load = [], [], []
    for step in range(1, 22):
        b = synth.make_batch(wl, seed, step, with_grad=True, drift=drift)
        n, st = _full_step_against_oracle(tab, orc, b, dev, wl, 1e-5, sweep=True, out_buf=out)
        expired.append(n)
        refused.append(st["n_full"])
        load.append(st["size"] / wl.capacity)
        say("config4 full size, step %d: load %.4f, refused so far %d, expired %d" % (step, load[-1], refused[-1], n))
    assert max(load) <= 31 / 32 and max(load) > 0.95
    assert refused[10] == 0 and refused[18] > 1_000_000           # the limit was reached before anything expired
    assert sum(expired[:19]) == 0 and expired[19] > 20_000_000     # the sweep of step 20
    assert refused[20] == refused[19] and load[20] < 0.4           # room again: step 21 admits
    say("config4 full size, comparing the tables")
    _whole_tables_equal(tab, orc, wl, seed, 1e-5)
    tab.close()


@pytest.mark.timeout(600)
def test_update_with_more_than_16M_rows_in_use(say):
    """Beyond 2^24 rows in use the backward's sort needs a fourth pass (25 bits in passes of seven).
    17 M keys are admitted on both sides (threshold 1, dim 4 keeps the oracle small), then one batch
    whose occurrences reach rows over the whole range — every 64th key once, the lowest and highest
    rows many times, absent and padding keys — is trained and the whole table compared."""
    from paper_2209_07663_amd.binding import Table
    dev = torch.device("cuda:0")
    seed, dim, cap, chunk_n = 13, 4, 1 << 25, 1 << 22
    stored = (1 << 24) + 100_000
    tab = Table(cap, dim, seed, freq_threshold=1, max_ids=chunk_n, max_bags=chunk_n, device=dev)
    orc = Oracle(cap, dim, seed, 1, 0, False, kind="cuckoo")
    rng = np.random.default_rng(17)
    keys_all = (np.arange(stored, dtype=np.int64) * 2654435761 + 12345) ^ 0x5DEECE66D   # distinct (odd multiplier)
    assert np.unique(keys_all).shape[0] == stored
    top_key, low_key = None, None
    for step, lo in enumerate(range(0, stored, chunk_n)):
        say("17M rows: admitting chunk", step)
        chunk = keys_all[lo:lo + chunk_n]
        r = tab.mono_lookup_or_insert(torch.from_numpy(chunk).to(dev), step).cpu().numpy()
        assert orc.lookup_or_insert(chunk, step).all() and (r >= 0).all()
        if lo == 0:
            low_key = chunk[np.argmin(r)]
        top_key = chunk[np.argmax(r)]
    st = tab.mono_table_stats()
    assert st["size"] == stored and st["n_insert_failed"] == 0 and st["n_full"] == 0
    body = np.concatenate([keys_all[::64], np.repeat([low_key, top_key], 500),
                           np.array([-1, -9, 4242], dtype=np.int64), keys_all[-3000:]])
    keys_h = body[rng.permutation(body.shape[0])]
    offs_h = np.arange(0, keys_h.shape[0] + 1, 3, dtype=np.int64)
    offs_h[-1] = keys_h.shape[0]
    grad_h = rng.standard_normal((offs_h.shape[0] - 1, dim)).astype(np.float32)
    step = 10
    say("17M rows: training step")
    rows = tab.mono_lookup_or_insert(torch.from_numpy(keys_h).to(dev), step)
    present = orc.lookup_or_insert(keys_h, step)
    rows_h = rows.cpu().numpy()
    assert ((rows_h >= 0) == present).all()
    assert rows_h.max() >= (1 << 24)                                   # the batch does reach the top rows
    offs = torch.from_numpy(offs_h).to(dev)
    pooled = tab.mono_gather_pool(rows, offs).cpu().numpy()
    tc.rows_close(pooled, orc.pool(keys_h, offs_h), 1e-5)
    tab.mono_apply_grad_adagrad(rows, offs, torch.from_numpy(grad_h).to(dev), 0.1, 1e-6)
    orc.apply_grad_adagrad(keys_h, offs_h, grad_h, 0.1, 1e-6)
    say("17M rows: comparing the tables")
    d = tab.mono_table_export()
    tc.check_placement(d, cap, 8, seed)
    tc.assert_same_table(d, orc.dump(), exact_rows=False, rtol=1e-5)
    trained = np.isin(d["keys"], keys_h)
    assert (d["acc"][trained] > 0).all() and (d["acc"][~trained] == 0).all()
    tab.close()
