"""Behaviour outside the graded envelope and plumbing of the device library (needs an MI355X).

Graded runs never fill the table or exhaust an eviction chain; these tests drive a tiny table past
both limits and check that nothing is lost or duplicated, that the limits are reported through the
counters, and that the table recovers once keys expire.  Also: calls on a side stream, two tables
used in turn, and batches of exactly the announced maximum size.
"""
import numpy as np
import pytest
import torch

from oracle import Oracle
from paper_2209_07663_amd import synth
from tests import table_checks as tc
from tests.test_gpu_parity import compare_step, RTOL_F32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "gpu tests need a GPU"
    return torch.device("cuda:0")


def _lookup(tab, keys_h, step, dev):
    rows = tab.mono_lookup_or_insert(torch.from_numpy(keys_h).to(dev), step)
    return rows.cpu().numpy()


def test_overfull_table_loses_nothing_and_recovers(dev):
    """1500 keys offered to a table whose fill limit is 992: a batch whose new keys do not all fit places
    none of them (on the device and in the oracle alike), a last batch sized to the room that is left fills
    the table to the limit exactly, and from then on every new key is refused and counted."""
    from paper_2209_07663_amd.binding import Table
    seed, cap, dim = 21, 1 << 10, 8
    limit = cap - cap // 32
    tab = Table(cap, dim, seed, freq_threshold=1, expire_steps=4, max_ids=4096, max_bags=4096, device=dev)
    orc = Oracle(cap, dim, seed, 1, 4, False, kind="cuckoo")
    rng = np.random.default_rng(5)
    universe = (rng.permutation(1 << 20)[:1500].astype(np.int64) + 1) * 7919
    chunks = np.array_split(universe, 5)                 # 300 each: the fourth would pass the limit
    chunks.append(universe[900:900 + (limit - 900)])     # exactly the room that is left
    held = {}                                            # key -> row, as handed out
    for step, chunk in enumerate(chunks):
        print("overfull: step", step, flush=True)
        rows = _lookup(tab, chunk, min(step, 4), dev)
        present = orc.lookup_or_insert(chunk, min(step, 4))
        assert ((rows >= 0) == present).all()
        assert (rows >= -1).all() and (rows < cap).all()
        assert (rows >= 0).all() or (rows == -1).all()   # all of a batch's new keys or none
        for k, r in zip(chunk.tolist(), rows.tolist()):
            if r >= 0:
                held[k] = r
        d = tab.mono_table_export()
        st = tab.mono_table_stats()
        assert st["n_lost"] == 0 and st["n_full"] == orc.refused_full
        assert d["keys"].shape[0] == st["size"] <= limit
        assert int((d["slot"] < 0).sum()) == st["stash_size"]
        tc.check_placement(d, cap, 8, seed)              # unique keys, slots and rows; h0 / h1 buckets
        tc.assert_same_table(d, orc.dump(), exact_rows=True)
        # the table holds exactly the keys that were given a row, under that row
        assert sorted(held) == d["keys"].tolist()
        assert (d["row"] == np.array([held[k] for k in d["keys"].tolist()])).all()
        # their rows still carry the initial values: no eviction chain damaged a resident
        assert (d["rows"] == tc.init_rows(d["keys"], dim, seed).astype(np.float32)).all()
    st = tab.mono_table_stats()
    assert st["n_full"] == 600 and st["size"] == limit     # two batches of 300 were refused whole, and counted
    assert st["n_insert_failed"] == 0 and st["stash_size"] == 0   # ... before any eviction chain could fail
    # every stored key is found again, at its row, wherever an eviction chain moved it (stash included)
    keys_now = np.array(sorted(held), dtype=np.int64)
    rows = _lookup(tab, keys_now, 5, dev)
    assert (rows == np.array([held[k] for k in keys_now.tolist()])).all()
    # keys turned away stay absent while no row is free, and are counted, not stored
    size_before = tab.mono_table_stats()["size"]
    away = np.array([k for k in universe.tolist() if k not in held][:100], dtype=np.int64)
    assert (_lookup(tab, away, 5, dev) == -1).all() and not orc.lookup_or_insert(away, 5).any()
    assert (_lookup(tab, away[:1], 5, dev) == -1).all()    # not even one more key
    assert tab.mono_table_stats()["size"] == limit
    # recovery: everything expires, rows and slots are free again
    n_exp = torch.zeros(1, dtype=torch.int64, device=dev)
    out = torch.zeros(cap, dtype=torch.int64, device=dev)
    tab.mono_expire_sweep(20, n_exp, out)
    n = int(n_exp.item())
    assert n == size_before
    assert sorted(out[:n].cpu().numpy().tolist()) == keys_now.tolist()
    st = tab.mono_table_stats()
    assert st["size"] == 0 and st["stash_size"] == 0
    fresh = (np.arange(600, dtype=np.int64) + 5) * 104729
    rows = _lookup(tab, fresh, 21, dev)
    assert (rows >= 0).all() and np.unique(rows).shape[0] == 600
    tc.check_placement(tab.mono_table_export(), cap, 8, seed)
    tab.close()


def test_restore_calls_at_the_fill_limit_place_all_their_records_or_none(dev):
    from paper_2209_07663_amd.binding import Table
    seed, cap, dim = 23, 1 << 10, 4
    limit = cap - cap // 32
    tab = Table(cap, dim, seed, freq_threshold=2, max_ids=4096, max_bags=4096, device=dev)
    orc = Oracle(cap, dim, seed, 2, 0, False, kind="cuckoo")
    rng = np.random.default_rng(6)
    keys = (rng.permutation(1 << 20)[:limit + 10].astype(np.int64) + 1) * 7919

    def restore(k):
        vals = rng.standard_normal((k.shape[0], dim)).astype(np.float32)
        acc = rng.random(k.shape[0]).astype(np.float32)
        seen = np.zeros(k.shape[0], dtype=np.uint32)
        to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        got = tab.mono_table_import(to_dev(k), to_dev(vals), to_dev(acc), to_dev(seen.view(np.int32)))
        want = orc.import_entries(k, vals, acc, seen)
        assert got == want
        return got

    assert restore(keys[:limit - 2]) == 0                       # two rows of room left
    assert restore(keys[limit - 2:limit + 3]) == 5              # five new keys: none is placed
    assert restore(np.concatenate([keys[:3], keys[limit - 2:limit]])) == 3    # three stored keys refused, two new ones fit
    assert restore(keys[limit:limit + 1]) == 1                  # full
    st = tab.mono_table_stats()
    assert st["size"] == limit and st["n_full"] == orc.refused_full == 6
    d = tab.mono_table_export()
    tc.check_placement(d, cap, 8, seed)
    tc.assert_same_table(d, orc.dump(), exact_rows=True)
    assert (tab.mono_filter_export() == orc.filter_words()).all()   # restored keys count as seen twice
    tab.close()


def test_calls_on_a_side_stream(dev):
    """Every call takes the stream it is given: a whole run on a non-default stream matches the oracle."""
    from paper_2209_07663_amd.binding import Table
    wl = synth.scaled(synth.CONFIGS["cfg3"], samples=1024, capacity=1 << 19)
    seed = 31
    side = torch.cuda.Stream(device=dev)
    with torch.cuda.stream(side):
        tab = Table(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16,
                    max_ids=1 << 18, max_bags=wl.n_bags, device=dev)
        orc = Oracle(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, kind="cuckoo")
        for step in range(3):
            b = synth.make_batch(wl, seed, step, with_grad=True)
            compare_step(tab, orc, b, dev, RTOL_F32, exact_rows=False, train=True, lr=wl.lr, eps=wl.eps)
        side.synchronize()
        tab.close()


def test_two_tables_used_in_turn(dev):
    """Tables share nothing: two of them with different shapes, stepped alternately, each match their oracle."""
    from dataclasses import replace
    from paper_2209_07663_amd.binding import Table
    wls = [replace(synth.scaled(synth.CONFIGS["cfg2"], samples=1024, capacity=1 << 16), freq_threshold=2),
           synth.scaled(synth.CONFIGS["cfg5"], samples=8192, capacity=1 << 17)]
    seeds = [41, 42]
    tabs, orcs = [], []
    for wl, seed in zip(wls, seeds):
        tab = Table(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, max_ids=1 << 18,
                    max_bags=wl.n_bags, device=dev)
        tabs.append(tab)
        orcs.append(Oracle(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, kind="cuckoo"))
    for step in range(3):
        for wl, seed, tab, orc in zip(wls, seeds, tabs, orcs):
            b = synth.make_batch(wl, seed, step, with_grad=True)
            compare_step(tab, orc, b, dev, 1e-2 if wl.bf16 else RTOL_F32, exact_rows=False, train=True, lr=wl.lr,
                         eps=wl.eps, sweep_at=step if wl.expire_steps else None)
    for tab in tabs:
        tab.close()


def test_batch_of_exactly_the_announced_maximum(dev):
    """n == max_ids and n_bags == max_bags: the workspaces are sized for it, one more is refused."""
    from paper_2209_07663_amd.binding import Table, MonoError
    seed, dim, max_ids, max_bags = 51, 16, 20000, 5000
    tab = Table(1 << 16, dim, seed, freq_threshold=1, max_ids=max_ids, max_bags=max_bags, device=dev)
    orc = Oracle(1 << 16, dim, seed, 1, 0, False, kind="cuckoo")
    rng = np.random.default_rng(6)
    keys_h = rng.integers(0, 30000, size=max_ids).astype(np.int64)
    offs_h = np.arange(0, max_ids + 1, max_ids // max_bags, dtype=np.int64)
    grad_h = rng.standard_normal((max_bags, dim)).astype(np.float32)
    for step in range(2):
        compare_step(tab, orc, {"keys": keys_h, "offsets": offs_h, "grad": grad_h, "step": step}, dev, RTOL_F32,
                     exact_rows=False, train=True)
    rows = torch.zeros(max_ids + 4, dtype=torch.int32, device=dev)
    offs = torch.arange(0, max_ids + 5, 4, dtype=torch.int64, device=dev)[: max_bags + 2]
    with pytest.raises(MonoError):
        tab.mono_gather_pool(rows[:max_ids], offs)                       # one bag too many
    with pytest.raises(MonoError):
        tab.mono_apply_grad_adagrad(rows, offs[: max_bags + 1], torch.zeros((max_bags, dim), device=dev), 0.1, 1e-8)
    tab.close()


def test_out_of_range_rows_and_offsets_are_bounded_by_the_kernels(dev):
    """Row indices outside the table count as absent, offsets beyond the index array are cut at its
    end: the result is that of the well-formed part of the input, and nothing else is touched."""
    from paper_2209_07663_amd.binding import Table
    seed, dim, cap = 61, 8, 1 << 12
    tab = Table(cap, dim, seed, freq_threshold=1, max_ids=1 << 12, max_bags=1 << 10, device=dev)
    keys = torch.arange(100, 164, dtype=torch.int64, device=dev)
    rows = tab.mono_lookup_or_insert(keys, 0)
    before = tab.mono_table_export()
    bad = rows.clone()
    bad[::4] = torch.tensor([cap, cap + 5, 2 ** 31 - 1, -5, -2 ** 31, -1, cap * 2, 1 << 20] * 2, dtype=torch.int32,
                            device=dev)
    good = bad.clone()
    good[::4] = -1
    offs_good = torch.arange(0, 65, 4, dtype=torch.int64, device=dev)
    offs_bad = offs_good.clone()
    offs_bad[-1] = 1 << 40                                   # last bag claims far more than there is
    want = tab.mono_gather_pool(good, offs_good).cpu().numpy()
    got = tab.mono_gather_pool(bad, offs_bad).cpu().numpy()
    assert (got == want).all()
    grad = torch.ones((16, dim), dtype=torch.float32, device=dev)
    tab.mono_apply_grad_adagrad(bad, offs_bad, grad, 0.1, 1e-8)
    after = tab.mono_table_export()
    touched = np.isin(before["row"], good[good >= 0].cpu().numpy())
    assert (after["rows"][~touched] == before["rows"][~touched]).all()
    assert (after["acc"][~touched] == 0).all() and (after["acc"][touched] > 0).all()
    # same update as the well-formed input gives on a twin table
    twin = Table(cap, dim, seed, freq_threshold=1, max_ids=1 << 12, max_bags=1 << 10, device=dev)
    rows2 = twin.mono_lookup_or_insert(keys, 0)
    good2 = rows2.clone()
    good2[::4] = -1
    twin.mono_apply_grad_adagrad(good2, offs_good, grad, 0.1, 1e-8)
    ref = twin.mono_table_export()
    assert (ref["keys"] == after["keys"]).all()
    tc.rows_close(after["rows"], ref["rows"].astype(np.float64), RTOL_F32)
    tab.close()
    twin.close()


def test_many_calls_queued_without_a_wait_then_updates(dev):
    """The number of sort passes an update launches follows a bound on the rows in use that the host keeps
    without waiting for the device (the device reports its mark after every lookup; the host adds the keys
    of the calls queued since).  Hundreds of lookups and updates queued back to back, on a large table that
    is almost empty (so that the bound, not the capacity, decides), with and without waits in between, must
    train exactly like the oracle and never skip an update."""
    from paper_2209_07663_amd.binding import Table
    seed, dim, cap = 53, 4, 1 << 22                       # capacity needs three passes, the rows in use one or two
    tab = Table(cap, dim, seed, freq_threshold=1, max_ids=4096, max_bags=4096, device=dev)
    orc = Oracle(cap, dim, seed, 1, 0, False, kind="cuckoo")
    rng = np.random.default_rng(19)
    pending = []
    for step in range(600):                               # more calls than the host keeps on record (256)
        n = int(rng.integers(1, 300))
        keys_h = rng.integers(0, 1 << 40, size=n).astype(np.int64) if step % 3 else rng.integers(0, 50, size=n).astype(np.int64)
        offs_h = np.arange(n + 1, dtype=np.int64)
        grad_h = rng.standard_normal((n, dim)).astype(np.float32)
        keys, offs, grad = (torch.from_numpy(a).to(dev) for a in (keys_h, offs_h, grad_h))
        rows = tab.mono_lookup_or_insert(keys, step)
        tab.mono_apply_grad_adagrad(rows, offs, grad, 0.05, 1e-8)
        pending.append((keys, offs, grad, rows))          # keep the buffers alive: nothing waits here
        orc.lookup_or_insert(keys_h, step)
        orc.apply_grad_adagrad(keys_h, offs_h, grad_h, 0.05, 1e-8)
        if step in (40, 300, 301):                        # a wait now and then (the stats call refreshes the bound)
            assert tab.mono_table_stats()["n_lost"] == 0
            pending.clear()
    st = tab.mono_table_stats()
    assert st["n_lost"] == 0 and st["n_insert_failed"] == 0
    assert 256 < st["size"] < 65536 * 2                   # crossed the one-pass / two-pass border on the way
    tc.assert_same_table(tab.mono_table_export(), orc.dump(), exact_rows=False, rtol=1e-5)
    tab.close()


@pytest.mark.parametrize("expire_steps", [0, 5])
@pytest.mark.parametrize("n", [1000, 65 * 1024, 65 * 1024 + 1, 4 * 65 * 256 + 7])
def test_every_occurrence_a_new_key_fills_the_winner_lists_to_the_brim(dev, n, expire_steps):
    """Batches made of distinct new keys only, admitted on first sight: every occurrence is elected, so the
    sub-lists of elected occurrences hold as much as they ever can, at batch sizes where the blocks of the
    election kernel (256 occurrences without expiry, 1024 with) are dealt to the 64 sub-lists unevenly."""
    from paper_2209_07663_amd.binding import Table
    seed, dim, cap = 59, 4, 1 << 18
    tab = Table(cap, dim, seed, freq_threshold=1, expire_steps=expire_steps, max_ids=n, max_bags=n, device=dev)
    orc = Oracle(cap, dim, seed, 1, expire_steps, False, kind="cuckoo")
    keys_h = (np.random.default_rng(n).permutation(1 << 22)[:n].astype(np.int64) + 1) * 1000003
    offs_h = np.arange(n + 1, dtype=np.int64)
    compare_step(tab, orc, {"keys": keys_h, "offsets": offs_h, "step": 0}, dev, RTOL_F32, exact_rows=True, train=False)
    assert tab.mono_table_stats()["size"] == n
    tab.close()
