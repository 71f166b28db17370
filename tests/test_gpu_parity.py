"""Device library vs CPU oracle on the same seeded inputs, through the C ABI (needs an MI355X).

Equality is on semantics, not layout: admitted key set, last_seen, counter words and expired sets
bit-exact; rows bit-exact until an optimizer step touches them; pooled sums, updated rows and
accumulators within rtol 1e-5 (fp32 rows) / 1e-2 (bf16 rows) per row in the infinity norm.
"""
import numpy as np
import pytest
import torch

from oracle import Oracle
from paper_2209_07663_amd import synth
from tests import table_checks as tc

pytestmark = pytest.mark.gpu

RTOL_F32, RTOL_BF16 = 1e-5, 1e-2


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "gpu tests need a GPU"
    return torch.device("cuda:0")


def make_table(wl, seed, max_ids, dev):
    from paper_2209_07663_amd.binding import Table
    return Table(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, max_ids=max_ids,
                 max_bags=max(wl.n_bags, 1), device=dev)


def make_oracle(wl, seed):
    return Oracle(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, kind="cuckoo")


def compare_step(tab, orc, batch, dev, rtol, exact_rows, train, lr=0.05, eps=1e-8, sweep_at=None, log=None):
    keys_h, offs_h = batch["keys"], batch["offsets"]
    step = batch["step"]
    keys = torch.from_numpy(keys_h).to(dev)
    offs = torch.from_numpy(offs_h).to(dev)
    rows = tab.mono_lookup_or_insert(keys, step)
    present = orc.lookup_or_insert(keys_h, step)
    rows_h = rows.cpu().numpy()
    assert ((rows_h >= 0) == present).all(), "presence differs at step %d" % step
    assert (rows_h >= -1).all()
    d = tab.mono_table_export()
    # the key -> row map handed out is the one stored
    pos = np.searchsorted(d["keys"].view(np.uint64), keys_h[present].view(np.uint64))
    assert (d["row"][pos] == rows_h[present]).all()
    st = tab.mono_table_stats()
    assert st["n_insert_failed"] == 0 and st["n_lost"] == 0 and st["n_full"] == 0 and orc.insert_failures == 0
    assert st["size"] == st["n_admitted"] - st["n_expired"] == d["keys"].shape[0]      # conservation
    tc.check_placement(d, tab.capacity, 8, tab.seed)
    tc.assert_same_table(d, orc.dump(), exact_rows=exact_rows, rtol=rtol)
    pooled = tab.mono_gather_pool(rows, offs).cpu().numpy()
    worst = tc.rows_close(pooled, orc.pool(keys_h, offs_h), rtol)
    if train:
        grad_h = batch["grad"]
        tab.mono_apply_grad_adagrad(rows, offs, torch.from_numpy(grad_h).to(dev), lr, eps)
        orc.apply_grad_adagrad(keys_h, offs_h, grad_h, lr, eps)
        tc.assert_same_table(tab.mono_table_export(), orc.dump(), exact_rows=False, rtol=rtol)
    n = None
    if sweep_at is not None:
        n_exp = torch.zeros(1, dtype=torch.int64, device=dev)
        out = torch.full((tab.capacity,), -7, dtype=torch.int64, device=dev)
        tab.mono_expire_sweep(sweep_at, n_exp, out)
        want = orc.expire_sweep(sweep_at)
        n = int(n_exp.item())
        got = np.sort(out[:n].cpu().numpy().view(np.uint64)).view(np.int64)
        assert n == want.shape[0] and (got == want).all(), "expired sets differ at step %d" % step
        tc.assert_same_table(tab.mono_table_export(), orc.dump(), exact_rows=exact_rows and not train, rtol=rtol)
    if log is not None:
        log.append((step, int(present.sum()), d["keys"].shape[0], worst, n))


def run_stream(wl, seed, steps, dev, train=False, sweep=False, check_filter=True):
    tab = make_table(wl, seed, max_ids=int(wl.n_bags * (wl.poisson_lam + 1) * 1.3) + 64, dev=dev)
    orc = make_oracle(wl, seed)
    drift = synth.DriftMap(wl, seed) if wl.drift_frac > 0 else None
    rtol = RTOL_BF16 if wl.bf16 else RTOL_F32
    log = []
    for step in range(steps):
        b = synth.make_batch(wl, seed, step, with_grad=train, drift=drift)
        compare_step(tab, orc, b, dev, rtol, exact_rows=not train, train=train, lr=wl.lr, eps=wl.eps,
                     sweep_at=step if sweep else None, log=log)
        if check_filter:
            assert (tab.mono_filter_export() == orc.filter_words()).all(), "counter words differ at step %d" % step
    tab.close()
    return log


def test_config1_lookup_and_gather(dev):
    """configs[0]: 2^16 rows, dim 16, 4096 uniform IDs, threshold 1, lookup_or_insert + gather only."""
    wl = synth.CONFIGS["cfg1"]
    log = run_stream(wl, seed=1, steps=2, dev=dev)
    assert log[0][1] == 4096                      # everything admitted on first sight


def test_forward_zipf_threshold3_several_steps(dev):
    """configs[1] shapes (26 slots, Poisson(3)+1, Zipf 1.05 over 2^32, threshold 3) at 4096 samples."""
    wl = synth.scaled(synth.CONFIGS["cfg2"], samples=4096, capacity=1 << 18)
    log = run_stream(wl, seed=2, steps=5, dev=dev)
    assert log[-1][2] > log[0][2] > 0             # keys keep crossing the threshold


def test_train_step_fp32(dev):
    """configs[2] shapes (40 slots, Poisson(4)+1, Zipf 1.1, dim 64, Adagrad) at 2048 samples."""
    wl = synth.scaled(synth.CONFIGS["cfg3"], samples=2048, capacity=1 << 19)
    run_stream(wl, seed=3, steps=4, dev=dev, train=True)


def test_streaming_drift_with_expiry(dev):
    """configs[3] shapes: threshold 5, expiry, rotating hot set, sweep every step (short expiry here)."""
    from dataclasses import replace
    wl = replace(synth.scaled(synth.CONFIGS["cfg4"], samples=2048, capacity=1 << 17, drift_ranks=1 << 15),
                 expire_steps=3, freq_threshold=3, drift_frac=0.3)
    log = run_stream(wl, seed=4, steps=12, dev=dev, train=True, sweep=True)
    assert log[-1][2] > 0


@pytest.mark.timeout(600)
def test_streaming_config_with_its_own_parameters_through_the_fill_limit_and_expiry(dev):
    """configs[3] with its parameters unchanged (threshold 5, expiry after 20 steps, 5 % of the hot ranks
    permuted per step, sweep every step), scaled in batch and table only: filled to load 0.9 with the hottest
    IDs, then 100 training steps.  The load climbs to the fill limit of 31/32 around step 10 (from there a
    batch whose new keys do not all fit places none of them, on both sides), the first expiry at step 20
    empties most of the table, and the stream settles.  Presence, refused counts and expired sets are
    compared at every step, whole tables and counter words every tenth."""
    wl = synth.scaled(synth.CONFIGS["cfg4"], samples=256, capacity=1 << 17, drift_ranks=1 << 18)
    assert wl.freq_threshold == 5 and wl.expire_steps == 20 and wl.drift_frac == 0.05
    seed = 4
    tab = make_table(wl, seed, max_ids=1 << 17, dev=dev)
    orc = make_oracle(wl, seed)
    drift = synth.DriftMap(wl, seed)
    hot = synth.hottest_ids(wl, int(0.9 * wl.capacity), drift)
    hot_d = torch.from_numpy(hot).to(dev)
    for _ in range(wl.freq_threshold):
        rows = tab.mono_lookup_or_insert(hot_d, 0)
        present = orc.lookup_or_insert(hot, 0)
    assert present.all() and bool((rows >= 0).all().item())
    n_exp = torch.zeros(1, dtype=torch.int64, device=dev)
    out = torch.zeros(wl.capacity, dtype=torch.int64, device=dev)
    refused_at, expired_total, top_load = None, 0, 0.0
    for step in range(1, 101):
        b = synth.make_batch(wl, seed, step, with_grad=True, drift=drift)
        keys, offs = torch.from_numpy(b["keys"]).to(dev), torch.from_numpy(b["offsets"]).to(dev)
        rows = tab.mono_lookup_or_insert(keys, step)
        present = orc.lookup_or_insert(b["keys"], step)
        assert ((rows.cpu().numpy() >= 0) == present).all(), "presence differs at step %d" % step
        tc.rows_close(tab.mono_gather_pool(rows, offs).cpu().numpy(), orc.pool(b["keys"], b["offsets"]), RTOL_F32)
        tab.mono_apply_grad_adagrad(rows, offs, torch.from_numpy(b["grad"]).to(dev), wl.lr, wl.eps)
        orc.apply_grad_adagrad(b["keys"], b["offsets"], b["grad"], wl.lr, wl.eps)
        st = tab.mono_table_stats()
        top_load = max(top_load, st["size"] / wl.capacity)
        assert st["n_full"] == orc.refused_full, "refused keys differ at step %d" % step
        assert st["n_insert_failed"] == 0 and st["n_lost"] == 0 and orc.insert_failures == 0
        if refused_at is None and st["n_full"]:
            refused_at = step
        tab.mono_expire_sweep(step, n_exp, out)
        want = orc.expire_sweep(step)
        n = int(n_exp.item())
        got = np.sort(out[:n].cpu().numpy().view(np.uint64)).view(np.int64)
        assert n == want.shape[0] and (got == want).all(), "expired sets differ at step %d" % step
        expired_total += n
        if step % 10 == 0:
            d = tab.mono_table_export()
            tc.check_placement(d, wl.capacity, 8, seed)
            tc.assert_same_table(d, orc.dump(), exact_rows=False, rtol=RTOL_F32)
            assert (tab.mono_filter_export() == orc.filter_words()).all(), "counter words differ at step %d" % step
            print("step %d load %.3f refused %d expired so far %d" % (step, st["size"] / wl.capacity, st["n_full"],
                                                                     expired_total), flush=True)
    assert refused_at is not None and refused_at < 20        # the limit was reached before anything expired
    assert top_load <= 31 / 32 and top_load > 0.95
    assert expired_total > wl.capacity // 2                  # ... and the first expiry emptied most of the table
    tab.close()


def test_train_step_bf16_rows(dev):
    """configs[4] shapes: bf16 rows, dim 64, one ID per bag, Zipf 1.2 over 2^63, threshold 2, expiry."""
    wl = synth.scaled(synth.CONFIGS["cfg5"], samples=16384, capacity=1 << 18)
    run_stream(wl, seed=5, steps=4, dev=dev, train=True, sweep=True)


@pytest.mark.timeout(600)
def test_large_table_config_with_its_own_parameters_across_its_expiry(dev):
    """configs[4] with its parameters unchanged (bf16 rows of dim 64, threshold 2, expiry after 50 steps, one
    ID per bag, Zipf(1.2) over 2^63), scaled in batch and table only, for 64 training steps with a sweep each:
    from step 50 on keys that were admitted early and never seen again leave, and the bf16 update is compared
    with the oracle's rounding all the way."""
    wl = synth.scaled(synth.CONFIGS["cfg5"], samples=2048, capacity=1 << 16)
    assert wl.bf16 and wl.freq_threshold == 2 and wl.expire_steps == 50 and wl.dim == 64
    log = run_stream(wl, seed=15, steps=64, dev=dev, train=True, sweep=True, check_filter=False)
    expired = [entry[4] for entry in log]
    assert sum(expired[:50]) == 0 and min(expired[51:]) > 0 and sum(expired) > 500    # keys leave once they turn 50


@pytest.mark.parametrize("dim,bf16", [(4, False), (24, False), (128, False), (256, False), (512, False), (768, True),
                                      (1024, False), (1024, True)])
def test_other_dims(dev, dim, bf16):
    """Rows from 4 elements to the 1024 of the paper's synchronisation example (section 3.2.2: 4 KB rows);
    beyond 256 elements a whole wave walks the row in pieces."""
    from dataclasses import replace
    wl = replace(synth.scaled(synth.CONFIGS["cfg3"], samples=512, capacity=1 << 16), dim=dim, slots=8, bf16=bf16)
    run_stream(wl, seed=6 + dim, steps=3, dev=dev, train=True)


def test_wide_rows_hot_key_snapshot_and_delta(dev):
    """dim 1024: a key with 60 000 occurrences (its run crosses tiles and blocks), then the touched-keys
    export, a snapshot and a restore into a fresh table, all against the oracle."""
    from paper_2209_07663_amd.binding import Table
    seed, dim, n_bags, cap = 31, 1024, 30000, 1 << 12
    tab = Table(cap, dim, seed, freq_threshold=1, max_ids=1 << 17, max_bags=n_bags, device=dev)
    orc = Oracle(cap, dim, seed, 1, 0, False, kind="cuckoo")
    rng = np.random.default_rng(3)
    offs_h = np.arange(0, 4 * n_bags + 1, 4, dtype=np.int64)
    keys_h = rng.integers(0, 700, size=4 * n_bags).astype(np.int64)
    keys_h[rng.random(4 * n_bags) < 0.5] = 987654321
    grad_h = (rng.standard_normal((n_bags, dim)) * 0.1).astype(np.float32)
    compare_step(tab, orc, {"keys": keys_h, "offsets": offs_h, "grad": grad_h, "step": 0}, dev, RTOL_F32,
                 exact_rows=False, train=True)
    t = tab.mono_export_touched()
    assert (t["keys"] == orc.take_touched()).all() and t["rows"].shape == (t["n"], dim)
    snap = tab.mono_table_export()
    fresh = Table(cap, dim, seed, freq_threshold=1, max_ids=1 << 17, max_bags=n_bags, device=dev)
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    assert fresh.mono_table_import(to_dev(snap["keys"]), to_dev(snap["rows"]), to_dev(snap["acc"]),
                                   to_dev(snap["last_seen"].view(np.int32))) == 0
    d = fresh.mono_table_export()
    assert (d["keys"] == snap["keys"]).all() and (d["rows"].view(np.uint32) == snap["rows"].view(np.uint32)).all()
    assert (d["acc"].view(np.uint32) == snap["acc"].view(np.uint32)).all()
    tab.close()
    fresh.close()


def test_edge_cases(dev):
    from paper_2209_07663_amd.binding import Table, MonoError
    seed = 77
    tab = Table(1 << 10, 8, seed, freq_threshold=2, expire_steps=2, max_ids=1 << 12, max_bags=1 << 12, device=dev)
    orc = Oracle(1 << 10, 8, seed, 2, 2, False, kind="cuckoo")
    # empty batch
    empty = torch.empty(0, dtype=torch.int64, device=dev)
    assert tab.mono_lookup_or_insert(empty, 0).shape[0] == 0
    # empty bags, padding keys, one key repeated across a whole batch (several waves of duplicates)
    keys_h = np.concatenate([np.full(1000, 42), [-1, -1, 7, 7, 9], np.full(37, 1 << 62)]).astype(np.int64)
    offs_h = np.array([0, 0, 1000, 1000, 1003, 1005, 1042, 1042], dtype=np.int64)
    grad_h = np.random.default_rng(0).standard_normal((7, 8)).astype(np.float32)
    for step in range(4):
        compare_step(tab, orc, {"keys": keys_h, "offsets": offs_h, "grad": grad_h, "step": step}, dev, RTOL_F32,
                     exact_rows=False, train=True, sweep_at=step)
    # nothing seen for 2 steps: everything expires
    compare_step(tab, orc, {"keys": np.array([5], dtype=np.int64), "offsets": np.array([0, 1], dtype=np.int64),
                            "step": 6}, dev, RTOL_F32, exact_rows=False, train=False, sweep_at=6)
    assert tab.mono_table_stats()["size"] == 0
    # argument errors are reported, not executed
    big = torch.zeros((1 << 12) + 1, dtype=torch.int64, device=dev)
    with pytest.raises(MonoError):
        tab.mono_lookup_or_insert(big, 7)
    with pytest.raises(MonoError):
        tab.mono_lookup_or_insert(big[:4], 5)      # step went backwards
    with pytest.raises(MonoError):
        Table(1000, 8, seed, device=dev)           # capacity not a power of two
    tab.close()


def test_long_stretches_of_empty_bags(dev):
    """The update finds the bag of every occurrence from the offsets, a sort unit at a time, starting at the
    bag that holds the unit's first occurrence: thousands of empty bags before the first ID, between two
    IDs of one sort unit, across unit borders and after the last ID must not shift a single gradient."""
    from paper_2209_07663_amd.binding import Table
    seed, dim = 47, 8
    tab = Table(1 << 14, dim, seed, freq_threshold=1, max_ids=1 << 16, max_bags=1 << 16, device=dev)
    orc = Oracle(1 << 14, dim, seed, 1, 0, False, kind="cuckoo")
    rng = np.random.default_rng(11)
    lens = np.concatenate([np.zeros(5000), rng.integers(1, 6, 300), np.zeros(7000), [1], np.zeros(3000), [2500],
                           np.zeros(1200), rng.integers(0, 3, 2000), np.zeros(9000)]).astype(np.int64)
    offs_h = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    keys_h = rng.integers(0, 900, size=int(offs_h[-1])).astype(np.int64)
    grad_h = rng.standard_normal((lens.shape[0], dim)).astype(np.float32)
    assert offs_h[-1] > 4096                               # several sort units
    for step in range(2):
        compare_step(tab, orc, {"keys": keys_h, "offsets": offs_h, "grad": grad_h, "step": step}, dev, RTOL_F32,
                     exact_rows=False, train=True)
    tab.close()


def test_sweeps_of_a_sparse_table_find_keys_that_come_back_to_emptied_buckets(dev):
    """A sweep only looks at buckets that a bitmap does not prove empty.  Keys are admitted into a large,
    almost empty table, expire (their buckets empty out), a later sweep notes those buckets as empty, the
    same keys come back into the same buckets, and expire again: every sweep must report exactly what
    the oracle reports, and a capacity below one bitmap word (16 slots) works like any other."""
    from paper_2209_07663_amd.binding import Table
    for cap, n_keys in [(1 << 20, 3000), (1 << 9, 100), (16, 5)]:
        seed = 43
        tab = Table(cap, 4, seed, freq_threshold=1, expire_steps=2, max_ids=1 << 12, max_bags=1 << 12, device=dev)
        orc = Oracle(cap, 4, seed, 1, 2, False, kind="cuckoo")
        rng = np.random.default_rng(cap)
        keys_a = (rng.permutation(1 << 20)[:n_keys].astype(np.int64) + 1) * 7919
        keys_b = (rng.permutation(1 << 20)[:n_keys // 2].astype(np.int64) + 1) * 104729
        plan = [(0, keys_a), (1, keys_b), (2, keys_b), (3, keys_b), (4, keys_b[:1]), (5, keys_a), (6, keys_a[:n_keys // 3]),
                (7, keys_b[:1]), (8, keys_b[:1]), (9, keys_a)]
        removed = 0
        for step, keys_h in plan:
            offs = np.arange(keys_h.shape[0] + 1, dtype=np.int64)
            compare_step(tab, orc, {"keys": keys_h, "offsets": offs, "step": step}, dev, RTOL_F32, exact_rows=True,
                         train=False, sweep_at=step)
            removed = tab.mono_table_stats()["n_expired"]
        assert removed >= n_keys                      # keys_a left once and came back
        tab.close()


@pytest.mark.parametrize("dim,bf16", [(4, False), (8, False), (32, False), (64, True), (100, False), (256, False)])
def test_short_bags_of_zero_one_or_two_ids(dev, dim, bf16):
    """Bags of at most two IDs take a path of their own in the pooling kernel (several rounds of row
    reads in flight); a last stretch with one long bag sends the final waves down the general path."""
    from paper_2209_07663_amd.binding import Table
    seed, cap = 83, 1 << 14
    tab = Table(cap, dim, seed, freq_threshold=1, bf16=bf16, max_ids=1 << 14, max_bags=1 << 14, device=dev)
    orc = Oracle(cap, dim, seed, 1, 0, bf16, kind="cuckoo")
    rng = np.random.default_rng(dim)
    lengths = rng.integers(0, 3, size=5000)
    lengths[-70:] = rng.integers(0, 3, size=70)
    lengths[-20] = 11                                                # one long bag among short ones
    n = int(lengths.sum())
    keys_h = rng.integers(0, 3000, size=n).astype(np.int64)
    keys_h[rng.integers(0, n, size=50)] = -1                         # padding keys: absent
    offs_h = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    grad_h = rng.standard_normal((lengths.shape[0], dim)).astype(np.float32)
    for step in range(2):
        compare_step(tab, orc, {"keys": keys_h, "offsets": offs_h, "grad": grad_h, "step": step}, dev,
                     RTOL_BF16 if bf16 else RTOL_F32, exact_rows=False, train=True)
    tab.close()


def test_high_load_without_failed_chains(dev):
    """Drive a table to load 0.9 (configs[3] asks for it) and check every invariant."""
    from paper_2209_07663_amd.binding import Table
    seed, cap = 9, 1 << 16
    tab = Table(cap, 4, seed, freq_threshold=1, max_ids=1 << 16, device=dev)
    orc = Oracle(cap, 4, seed, 1, 0, False, kind="cuckoo")
    rng = np.random.default_rng(1)
    all_keys = rng.permutation(1 << 24)[: int(0.9 * cap)].astype(np.int64) * 1000003
    for step, chunk in enumerate(np.array_split(all_keys, 6)):
        offs = np.arange(chunk.shape[0] + 1, dtype=np.int64)
        compare_step(tab, orc, {"keys": chunk, "offsets": offs, "step": step}, dev, RTOL_F32, exact_rows=True,
                     train=False)
    st = tab.mono_table_stats()
    assert st["size"] == all_keys.shape[0] and st["size"] >= 0.9 * cap - 1
    tab.close()


def test_hot_key_gradient_reduction_is_pairwise(dev):
    """One key holding half of a 400k-occurrence batch: its gradient sum must still meet 1e-5."""
    from paper_2209_07663_amd.binding import Table
    seed, dim, n_bags = 10, 32, 100000
    tab = Table(1 << 16, dim, seed, freq_threshold=1, max_ids=1 << 19, max_bags=n_bags, device=dev)
    orc = Oracle(1 << 16, dim, seed, 1, 0, False, kind="cuckoo")
    rng = np.random.default_rng(2)
    offs_h = np.arange(0, 4 * n_bags + 1, 4, dtype=np.int64)
    keys_h = rng.integers(0, 5000, size=4 * n_bags).astype(np.int64)
    keys_h[rng.random(4 * n_bags) < 0.5] = 123456789
    grad_h = (rng.standard_normal((n_bags, dim)) * 0.1).astype(np.float32)
    for step in range(2):
        compare_step(tab, orc, {"keys": keys_h, "offsets": offs_h, "grad": grad_h, "step": step}, dev, RTOL_F32,
                     exact_rows=False, train=True)
    tab.close()


@pytest.mark.parametrize("stored", [255, 256, 257, 65535, 65536, 65537, 65538])
def test_update_at_the_sort_width_boundaries(dev, stored):
    """The backward sorts bit_length(highest row in use) bits, in passes of at most eight: with 256 /
    257 and 65536 / 65537 rows in use the digit plan changes (one pass -> two -> three).  Exactly
    `stored` keys are admitted, then a batch over all of them (every key once, the first and the
    last rows many times, some absent keys) is trained and compared with the oracle."""
    # stored = highest row + 1: 256 -> 8 bits, 257 -> 9 bits (two passes), 65536 -> 16, 65537 -> 17 (three)
    from paper_2209_07663_amd.binding import Table
    seed, dim, cap = 71, 4, 1 << 18
    tab = Table(cap, dim, seed, freq_threshold=2, max_ids=1 << 17, max_bags=1 << 17, device=dev)
    orc = Oracle(cap, dim, seed, 2, 0, False, kind="cuckoo")
    rng = np.random.default_rng(stored)
    keys_all = (rng.permutation(1 << 22)[:stored].astype(np.int64) + 3) * 1000003
    rows_of = {}
    for step, lo in enumerate(range(0, stored, 1 << 16)):
        chunk = keys_all[lo:lo + (1 << 16)]
        for _ in range(2):                                          # second sight admits (threshold 2)
            r = tab.mono_lookup_or_insert(torch.from_numpy(chunk).to(dev), step).cpu().numpy()
            orc.lookup_or_insert(chunk, step)
        rows_of.update(zip(chunk.tolist(), r.tolist()))
    assert sorted(rows_of.values()) == list(range(stored))          # rows are handed out in ascending order
    by_row = np.array(sorted(rows_of, key=rows_of.get), dtype=np.int64)
    first, last = by_row[0], by_row[-1]
    absent = np.array([-5, -1, 12345, 777], dtype=np.int64)
    body = np.concatenate([keys_all, np.repeat([first, last], 300), absent, by_row[-40:], by_row[:40]])
    keys_h = body[rng.permutation(body.shape[0])]
    lengths = rng.integers(0, 4, size=keys_h.shape[0])              # ragged bags, empty ones included
    offs_h = np.concatenate([[0], np.cumsum(lengths)])
    offs_h = offs_h[: np.searchsorted(offs_h, keys_h.shape[0]) + 1].astype(np.int64)
    offs_h[-1] = keys_h.shape[0]
    grad_h = rng.standard_normal((offs_h.shape[0] - 1, dim)).astype(np.float32)
    batch = {"keys": keys_h, "offsets": offs_h, "grad": grad_h, "step": 10}
    # (threshold 2: the absent keys of this batch are seen once and stay out, the mark stays at `stored`)
    compare_step(tab, orc, batch, dev, RTOL_F32, exact_rows=True, train=True, lr=0.1, eps=1e-6)
    tab.close()


@pytest.mark.parametrize("case", range(20))
def test_seeded_random_configurations(dev, case):
    """Combinations that no named configuration covers: a seeded draw of dim, storage type, threshold,
    expiry, number of counter hashes, counter array size, bag lengths, key skew and padding keys."""
    from paper_2209_07663_amd.binding import Table
    rng = np.random.default_rng(1000 + case)
    dim = int(rng.choice([4, 8, 12, 32, 64, 100, 256, 512, 768, 1024]))
    bf16 = bool(rng.integers(0, 2))
    thr = int(rng.choice([0, 1, 2, 3, 7]))
    expire = int(rng.choice([0, 0, 2, 5]))
    hashes = int(rng.choice([1, 1, 2, 4]))
    cap = 1 << int(rng.integers(12, 16))
    filter_log2 = int(rng.choice([0, 10, 14]))
    n_bags = int(rng.integers(50, 3000))
    lam = float(rng.choice([0.0, 1.0, 6.0]))
    universe = int(rng.choice([50, 2000, 1 << 40]))
    lr, eps = float(rng.choice([0.05, 0.5])), float(rng.choice([1e-8, 0.1]))     # eps large enough to matter
    seed = 500 + case
    print("case", case, dict(dim=dim, bf16=bf16, thr=thr, expire=expire, hashes=hashes, cap=cap,
                             filter_log2=filter_log2, n_bags=n_bags, lam=lam, universe=universe), flush=True)
    max_ids = int(n_bags * (lam + 1) * 3) + 64
    tab = Table(cap, dim, seed, thr, expire, bf16, max_ids=max_ids, max_bags=n_bags, device=dev,
                filter_hashes=hashes, filter_log2=filter_log2)
    orc = Oracle(cap, dim, seed, thr, expire, bf16, kind="cuckoo", n_filter=tab.n_filter, filter_hashes=hashes)
    rtol = RTOL_BF16 if bf16 else RTOL_F32
    for step in range(5):
        lens = (rng.poisson(lam, size=n_bags) + (0 if rng.random() < 0.3 else 1)).astype(np.int64)   # empty bags too
        offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        n = int(offs[-1])
        if n > max_ids:
            lens[:] = 1
            offs = np.arange(n_bags + 1, dtype=np.int64)
            n = n_bags
        keys = (rng.zipf(1.3, size=n) % universe).astype(np.int64) * 0x9E3779B1 % (1 << 62)
        keys[rng.random(n) < 0.02] = -1                                                                # padding
        grad = (rng.standard_normal((n_bags, dim)) * 0.1).astype(np.float32)
        # at most ~half the table: a full table is a different test
        if np.unique(keys).shape[0] * (step + 1) > cap // 2:
            keys = keys % 997
        compare_step(tab, orc, {"keys": keys, "offsets": offs, "grad": grad, "step": 2 * step}, dev, rtol,
                     exact_rows=False, train=True, lr=lr, eps=eps, sweep_at=2 * step if expire else None)
        assert (tab.mono_filter_export() == orc.filter_words()).all(), "counter words differ at step %d" % step
    tab.close()
