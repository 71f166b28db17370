"""Maintenance operations of the device library against the oracle (needs an MI355X): touched keys
and their delta export (paper section 2.2.3)."""
import numpy as np
import pytest
import torch

from oracle import Oracle
from paper_2209_07663_amd import synth
from tests import table_checks as tc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "gpu tests need a GPU"
    return torch.device("cuda:0")


def _step(tab, orc, b, dev, wl, train=True, sweep=True):
    keys, offs = torch.from_numpy(b["keys"]).to(dev), torch.from_numpy(b["offsets"]).to(dev)
    rows = tab.mono_lookup_or_insert(keys, b["step"])
    present = orc.lookup_or_insert(b["keys"], b["step"])
    assert ((rows.cpu().numpy() >= 0) == present).all()
    if train:
        tab.mono_apply_grad_adagrad(rows, offs, torch.from_numpy(b["grad"]).to(dev), wl.lr, wl.eps)
        orc.apply_grad_adagrad(b["keys"], b["offsets"], b["grad"], wl.lr, wl.eps)
    if sweep and wl.expire_steps:
        tab.mono_expire_sweep(b["step"])
        orc.expire_sweep(b["step"])


def _check_delta(delta, orc, rtol):
    want = orc.take_touched()
    assert delta["n"] == want.shape[0] and (delta["keys"] == want).all(), "touched sets differ"
    ref = orc.dump()
    pos = np.searchsorted(ref["keys"].view(np.uint64), want.view(np.uint64))
    assert (ref["keys"][pos] == want).all()
    tc.rows_close(delta["rows"], ref["rows"][pos].astype(np.float64), rtol)
    a, b = delta["acc"].astype(np.float64), ref["acc"][pos].astype(np.float64)
    assert (np.abs(a - b) <= rtol * np.maximum(np.abs(b), 1e-30)).all()


@pytest.mark.parametrize("name,samples,cap", [("cfg3", 1024, 1 << 20), ("cfg5", 16384, 1 << 18)])
def test_touched_keys_and_delta_export(dev, name, samples, cap):
    """Windows of several steps; steps that only look up; expiry between training and synchronisation
    (the bf16 configuration expires keys); a buffer that is too small leaves the window open."""
    from dataclasses import replace
    from paper_2209_07663_amd.binding import Table
    wl = synth.scaled(synth.CONFIGS[name], samples=samples, capacity=cap)
    if wl.expire_steps:
        wl = replace(wl, expire_steps=2)
    seed = 71
    rtol = 1e-2 if wl.bf16 else 1e-5
    tab = Table(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, max_ids=1 << 18,
                max_bags=wl.n_bags, device=dev)
    orc = Oracle(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, kind="cuckoo")
    assert tab.mono_export_touched()["n"] == 0                       # nothing trained yet
    for step in range(9):
        b = synth.make_batch(wl, seed, step, with_grad=True)
        _step(tab, orc, b, dev, wl, train=step % 4 != 1)
        if step == 3:                                                # too small a buffer: nothing is taken
            n = tab.mono_export_touched(max_n=8)["n"]
            assert n > 8
        if step % 3 == 2 or step == 3:
            delta = tab.mono_export_touched()
            assert delta["n"] > 0
            _check_delta(delta, orc, rtol)
            d = tab.mono_table_export()                              # handed-out row indices are the table's
            pos = np.searchsorted(d["keys"].view(np.uint64), delta["keys"].view(np.uint64))
            assert (d["row"][pos] == delta["row"]).all()
            assert tab.mono_export_touched()["n"] == 0               # the window was closed
    tab.close()


# ---- snapshot / restore (paper section 2.3) and rehash / grow (section 2.1) ---------------------------

def _full_step(tab, orc, b, dev, wl, rtol, generation=0, seed=None):
    """One whole step on both sides with every comparison of the parity tests."""
    keys, offs = torch.from_numpy(b["keys"]).to(dev), torch.from_numpy(b["offsets"]).to(dev)
    rows = tab.mono_lookup_or_insert(keys, b["step"])
    present = orc.lookup_or_insert(b["keys"], b["step"])
    assert ((rows.cpu().numpy() >= 0) == present).all(), "presence differs at step %d" % b["step"]
    tc.rows_close(tab.mono_gather_pool(rows, offs).cpu().numpy(), orc.pool(b["keys"], b["offsets"]), rtol)
    tab.mono_apply_grad_adagrad(rows, offs, torch.from_numpy(b["grad"]).to(dev), wl.lr, wl.eps)
    orc.apply_grad_adagrad(b["keys"], b["offsets"], b["grad"], wl.lr, wl.eps)
    if wl.expire_steps:
        n_exp = torch.zeros(1, dtype=torch.int64, device=dev)
        out = torch.zeros(tab.capacity, dtype=torch.int64, device=dev)
        tab.mono_expire_sweep(b["step"], n_exp, out)
        want = orc.expire_sweep(b["step"])
        got = np.sort(out[: int(n_exp.item())].cpu().numpy().view(np.uint64)).view(np.int64)
        assert got.shape == want.shape and (got == want).all(), "expired sets differ"
    d = tab.mono_table_export()
    tc.assert_same_table(d, orc.dump(), exact_rows=False, rtol=rtol)
    tc.check_placement(d, tab.capacity, 8, seed, generation)
    assert (tab.mono_filter_export() == orc.filter_words()).all(), "counter words differ"
    st = tab.mono_table_stats()
    assert st["n_lost"] == 0 and st["n_full"] == 0 and st["stash_size"] == 0
    assert st["size"] == st["n_admitted"] - st["n_expired"] == d["keys"].shape[0]      # conservation, also across
    return d                                                                          # restore and rehash


def _small_cfg(name):
    from dataclasses import replace
    if name == "cfg4":
        return replace(synth.scaled(synth.CONFIGS["cfg4"], samples=1024, capacity=1 << 16, drift_ranks=1 << 14),
                       expire_steps=3, freq_threshold=2, drift_frac=0.3)
    return replace(synth.scaled(synth.CONFIGS["cfg5"], samples=16384, capacity=1 << 17), expire_steps=3)


@pytest.mark.parametrize("name", ["cfg4", "cfg5"])
def test_restore_from_snapshot_then_train_on(dev, name):
    from paper_2209_07663_amd.binding import Table
    wl, seed = _small_cfg(name), 81
    rtol = 1e-2 if wl.bf16 else 1e-5
    mk_tab = lambda max_ids: Table(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16,
                                   max_ids=max_ids, max_bags=wl.n_bags, device=dev)
    mk_orc = lambda: Oracle(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, kind="cuckoo")
    drift = synth.DriftMap(wl, seed) if wl.drift_frac > 0 else None
    batches = [synth.make_batch(wl, seed, s, with_grad=True, drift=drift) for s in range(8)]
    tab_a, orc_a = mk_tab(1 << 17), mk_orc()
    for b in batches[:4]:
        _full_step(tab_a, orc_a, b, dev, wl, rtol, seed=seed)
    # each side is restored from its OWN snapshot: table dump + counter words
    snap, words = tab_a.mono_table_export(), tab_a.mono_filter_export()
    osnap, owords = orc_a.dump(), orc_a.filter_words()
    n = snap["keys"].shape[0]
    assert n > 500
    tab_b, orc_b = mk_tab(1 << 17), mk_orc()
    perm = np.random.default_rng(1).permutation(n)
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    k_d, v_d, a_d = to_dev(snap["keys"][perm]), to_dev(snap["rows"][perm]), to_dev(snap["acc"][perm])
    s_d = to_dev(snap["last_seen"][perm].view(np.int32))
    third = n // 3
    refused = 0
    for lo, hi in [(0, third), (third, 2 * third), (2 * third, n)]:
        refused += tab_b.mono_table_import(k_d[lo:hi], v_d[lo:hi], a_d[lo:hi], s_d[lo:hi])
    assert refused == 0
    tab_b.mono_filter_import(torch.from_numpy(words.view(np.int32)).to(dev))
    assert orc_b.import_entries(osnap["keys"], osnap["rows"], osnap["acc"], osnap["last_seen"]) == 0
    orc_b.write_filter_words(owords)
    # the restored table is the snapshot, bit for bit, placed by the table's own hash functions
    d = tab_b.mono_table_export()
    assert (d["keys"] == snap["keys"]).all() and (d["last_seen"] == snap["last_seen"]).all()
    assert (d["rows"].view(np.uint32) == snap["rows"].view(np.uint32)).all()
    assert (d["acc"].view(np.uint32) == snap["acc"].view(np.uint32)).all()
    tc.check_placement(d, wl.capacity, 8, seed)
    assert (tab_b.mono_filter_export() == words).all()
    assert tab_b.mono_table_stats()["size"] == n and tab_b.mono_export_touched()["n"] == 0
    # records that must be refused: a stored key, the reserved key, the second record of a key
    bad = torch.tensor([int(snap["keys"][0]), -1, 123456789123, 123456789123], dtype=torch.int64, device=dev)
    vals = torch.full((4, wl.dim), 1.00390625 + 2.0 ** -12, dtype=torch.float32, device=dev)
    assert tab_b.mono_table_import(bad, vals, torch.ones(4, device=dev), torch.full((4,), 3, dtype=torch.int32,
                                                                                  device=dev)) == 3
    orc_b.import_entries(np.array([123456789123], dtype=np.int64), vals[:1].cpu().numpy(), np.ones(1, np.float32),
                         np.array([3], dtype=np.uint32))
    d = tab_b.mono_table_export()
    i = int(np.searchsorted(d["keys"].view(np.uint64), np.uint64(123456789123)))
    want = vals[0].to(torch.bfloat16).to(torch.float32) if wl.bf16 else vals[0]
    assert d["keys"][i] == 123456789123 and (d["rows"][i] == want.cpu().numpy()).all() and d["acc"][i] == 1.0
    # continue-training equivalence: the restored pair goes through the same further batches as the original pair
    for b in batches[4:]:
        da = _full_step(tab_a, orc_a, b, dev, wl, rtol, seed=seed)
        db = _full_step(tab_b, orc_b, b, dev, wl, rtol, seed=seed)
        common = np.isin(db["keys"], da["keys"])
        assert common.sum() == da["keys"].shape[0]            # b additionally holds the extra record until it expires
        assert (db["last_seen"][common] == da["last_seen"]).all()
        tc.rows_close(db["rows"][common], da["rows"].astype(np.float64), rtol)
    tab_a.close()
    tab_b.close()


def test_rehash_in_place_size_then_grow(dev):
    from paper_2209_07663_amd.binding import Table
    wl, seed = _small_cfg("cfg4"), 91
    rtol = 1e-5
    tab = Table(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, max_ids=1 << 17,
                max_bags=wl.n_bags, device=dev)
    orc = Oracle(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, kind="cuckoo")
    drift = synth.DriftMap(wl, seed)
    batches = [synth.make_batch(wl, seed, s, with_grad=True, drift=drift) for s in range(9)]
    for b in batches[:3]:
        before = _full_step(tab, orc, b, dev, wl, rtol, seed=seed)
    stats0 = tab.mono_table_stats()
    for (cap, generation), chunk in zip([(wl.capacity, 1), (wl.capacity * 4, 2)], [batches[3:6], batches[6:]]):
        new = tab.rehashed(cap, generation)
        orc.rehash(cap, generation)
        tab.close()
        tab = new
        after = tab.mono_table_export()
        # same keys under the same row indices with the same contents; only the positions moved
        assert (after["keys"] == before["keys"]).all() and (after["row"] == before["row"]).all()
        assert (after["last_seen"] == before["last_seen"]).all()
        assert (after["rows"].view(np.uint32) == before["rows"].view(np.uint32)).all()
        assert (after["acc"].view(np.uint32) == before["acc"].view(np.uint32)).all()
        tc.check_placement(after, cap, 8, seed, generation)
        assert (tab.mono_filter_export() == orc.filter_words()).all()
        st = tab.mono_table_stats()
        assert st["capacity"] == cap and st["size"] == stats0["size"] and st["n_admitted"] == stats0["n_admitted"]
        assert st["n_expired"] == stats0["n_expired"] and st["stash_size"] == 0
        # the touched set survives the move (it is trained state, not placement)
        delta = tab.mono_export_touched()
        want = orc.take_touched()
        assert delta["n"] == want.shape[0] and (delta["keys"] == want).all()
        for b in chunk:
            before = _full_step(tab, orc, b, dev, wl, rtol, generation=generation, seed=seed)
        stats0 = tab.mono_table_stats()
    tab.close()


def test_growing_an_overfull_table_empties_its_stash_and_makes_room(dev):
    from paper_2209_07663_amd.binding import Table
    seed, cap, dim = 95, 1 << 10, 8
    tab = Table(cap, dim, seed, freq_threshold=1, max_ids=4096, max_bags=4096, device=dev)
    rng = np.random.default_rng(8)
    universe = (rng.permutation(1 << 20)[:1400].astype(np.int64) + 1) * 7919
    limit = cap - cap // 32
    held = {}
    # up to the limit in two batches, then the rest: a batch that does not fit is refused whole
    for step, chunk in enumerate([universe[:500], universe[500:limit], universe[limit:]]):
        rows = tab.mono_lookup_or_insert(torch.from_numpy(chunk).to(dev), step).cpu().numpy()
        held.update({k: r for k, r in zip(chunk.tolist(), rows.tolist()) if r >= 0})
    st = tab.mono_table_stats()
    assert st["size"] == len(held) == limit and st["n_full"] == 1400 - limit and st["n_lost"] == 0
    big = tab.rehashed(cap * 2, 1)
    tab.close()
    st = big.mono_table_stats()
    assert st["size"] == len(held) and st["stash_size"] == 0 and st["capacity"] == 2 * cap
    d = big.mono_table_export()
    tc.check_placement(d, 2 * cap, 8, seed, generation=1)
    assert d["keys"].tolist() == sorted(held) and (d["row"] == np.array([held[k] for k in sorted(held)])).all()
    assert (d["slot"] >= 0).all()
    assert (d["rows"] == tc.init_rows(d["keys"], dim, seed).astype(np.float32)).all()
    # the keys turned away before now fit, and get rows beyond the old capacity or freed ones, all distinct
    away = np.array([k for k in universe.tolist() if k not in held], dtype=np.int64)
    rows = big.mono_lookup_or_insert(torch.from_numpy(away).to(dev), 4).cpu().numpy()
    assert (rows >= 0).all()
    d = big.mono_table_export()
    assert d["keys"].shape[0] == universe.shape[0] and np.unique(d["row"]).shape[0] == universe.shape[0]
    tc.check_placement(d, 2 * cap, 8, seed, generation=1)
    big.close()


@pytest.mark.parametrize("cap", [1 << 12, 1 << 20])
def test_rehash_at_the_fill_limit_loses_nothing(dev, cap):
    """A table filled to its limit (31/32 of the rows) moves to new hash functions at the SAME size:
    every element is re-inserted at once into an empty table, the hardest case for the eviction chains.
    Nothing may be lost; an element whose chain hits the bound is kept in the stash and still found."""
    from paper_2209_07663_amd.binding import Table
    seed, dim, max_ids = 97, 4, 1 << 18
    tab = Table(cap, dim, seed, freq_threshold=1, max_ids=max_ids, max_bags=1, device=dev)
    universe = (np.random.default_rng(9).permutation(4 * cap)[: cap + cap // 8].astype(np.int64) + 1) * 7919
    limit = cap - cap // 32
    held = {}
    # exactly `limit` keys in batches that fit, then the rest of the universe in one batch that does not
    bounds = list(range(0, limit, max_ids)) + [limit, universe.shape[0]]
    for step, (lo, hi) in enumerate(zip(bounds[:-1], bounds[1:])):
        chunk = universe[lo:hi]
        rows = tab.mono_lookup_or_insert(torch.from_numpy(chunk).to(dev), step).cpu().numpy()
        held.update({k: r for k, r in zip(chunk.tolist(), rows.tolist()) if r >= 0})
    st = tab.mono_table_stats()
    assert st["size"] == len(held) == limit and st["n_lost"] == 0 and st["n_full"] == universe.shape[0] - limit
    keys_now = np.array(sorted(held), dtype=np.int64)
    rows_now = np.array([held[k] for k in keys_now.tolist()])
    for generation in (1, 2, 3):
        print("rehash at the fill limit: capacity", cap, "generation", generation, flush=True)
        new = tab.rehashed(cap, generation)
        tab.close()
        tab = new
        st = tab.mono_table_stats()
        assert st["n_lost"] == 0 and st["size"] == limit, st
        d = tab.mono_table_export()
        tc.check_placement(d, cap, 8, seed, generation)
        assert d["keys"].tolist() == keys_now.tolist() and (d["row"] == rows_now).all()
        assert int((d["slot"] < 0).sum()) == st["stash_size"] <= 16    # the stash is a last resort, not a shelf
        assert (d["rows"] == tc.init_rows(d["keys"], dim, seed).astype(np.float32)).all()
        for lo in range(0, limit, max_ids):                              # every key is found, at its row
            got = tab.mono_lookup_or_insert(torch.from_numpy(keys_now[lo:lo + max_ids]).to(dev), 100 + generation)
            assert (got.cpu().numpy() == rows_now[lo:lo + max_ids]).all()
    tab.close()


def test_long_stream_with_every_operation(dev):
    """Forty steps of a drifting stream with expiry: lookup, pool, update and sweep every step, a
    synchronisation every seventh, a grow under new hash functions at step 15, a snapshot + restore
    into a fresh table at step 25 - device and oracle side by side throughout."""
    from paper_2209_07663_amd.binding import Table
    wl, seed, rtol = _small_cfg("cfg4"), 131, 1e-5
    tab = Table(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, max_ids=1 << 17,
                max_bags=wl.n_bags, device=dev, filter_hashes=2)
    orc = Oracle(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, kind="cuckoo",
                 n_filter=tab.n_filter, filter_hashes=2)
    drift = synth.DriftMap(wl, seed)
    generation = 0
    for step in range(40):
        b = synth.make_batch(wl, seed, step, with_grad=True, drift=drift)
        _full_step(tab, orc, b, dev, wl, rtol, generation=generation, seed=seed)
        if step % 7 == 6:
            delta, want = tab.mono_export_touched(), orc.take_touched()
            assert delta["n"] == want.shape[0] and (delta["keys"] == want).all(), "touched sets differ at step %d" % step
        if step == 15:
            generation = 5
            new = tab.rehashed(wl.capacity * 2, generation)
            orc.rehash(wl.capacity * 2, generation)
            tab.close()
            tab = new
        if step == 25:
            snap, words = tab.mono_table_export(), tab.mono_filter_export()
            osnap, owords = orc.dump(), orc.filter_words()
            fresh = Table(tab.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, max_ids=1 << 17,
                          max_bags=wl.n_bags, device=dev, filter_hashes=2, filter_log2=tab.n_filter.bit_length() - 1)
            to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
            assert fresh.mono_table_import(to_dev(snap["keys"]), to_dev(snap["rows"]), to_dev(snap["acc"]),
                                           to_dev(snap["last_seen"].view(np.int32))) == 0
            fresh.mono_filter_import(to_dev(words.view(np.int32)))
            tab.close()
            tab, generation = fresh, 0               # a restored table starts with the hash functions of a new one
            orc2 = Oracle(orc.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, kind="cuckoo",
                          n_filter=orc.n_filter, filter_hashes=2)
            assert orc2.import_entries(osnap["keys"], osnap["rows"], osnap["acc"], osnap["last_seen"]) == 0
            orc2.write_filter_words(owords)
            orc.take_touched()                       # the restored pair starts a new synchronisation window
            orc = orc2
    assert tab.mono_table_stats()["n_insert_failed"] == 0
    tab.close()


@pytest.mark.parametrize("hashes", [1, 3])
def test_restore_without_counters_on_a_table_that_never_expires(dev, hashes):
    """With expire_steps == 0 a lookup trusts a counter below the threshold as proof of absence; records
    restored WITHOUT their counters must still be found, and the counters they raise match the oracle."""
    from paper_2209_07663_amd.binding import Table
    wl, seed = synth.scaled(synth.CONFIGS["cfg2"], samples=1024, capacity=1 << 17), 141
    mk = lambda: (Table(wl.capacity, wl.dim, seed, wl.freq_threshold, 0, False, max_ids=1 << 18, max_bags=wl.n_bags,
                        device=dev, filter_hashes=hashes),
                  Oracle(wl.capacity, wl.dim, seed, wl.freq_threshold, 0, False, kind="cuckoo", filter_hashes=hashes))
    tab_a, orc_a = mk()
    batches = [synth.make_batch(wl, seed, s, with_grad=True) for s in range(6)]
    for b in batches[:3]:
        _full_step(tab_a, orc_a, b, dev, wl, 1e-5, seed=seed)
    snap, osnap = tab_a.mono_table_export(), orc_a.dump()
    assert snap["keys"].shape[0] > 1000
    tab_b, orc_b = mk()                                   # records only: the counters start from zero
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    assert tab_b.mono_table_import(to_dev(snap["keys"]), to_dev(snap["rows"]), to_dev(snap["acc"]),
                                   to_dev(snap["last_seen"].view(np.int32))) == 0
    assert orc_b.import_entries(osnap["keys"], osnap["rows"], osnap["acc"], osnap["last_seen"]) == 0
    assert (tab_b.mono_filter_export() == orc_b.filter_words()).all()
    rows = tab_b.mono_lookup_or_insert(to_dev(snap["keys"]), 3)
    assert bool((rows >= 0).all().item())                  # every restored key is found
    assert orc_b.lookup_or_insert(snap["keys"], 3).all()
    for b in batches[3:]:
        _full_step(tab_b, orc_b, b, dev, wl, 1e-5, seed=seed)
    tab_a.close()
    tab_b.close()


@pytest.mark.parametrize("hashes", [1, 2])
def test_counter_words_imported_over_a_populated_table_hide_no_key(dev, hashes):
    """All-zero counter words (and then random ones over a window) written into a populated table that never
    expires keys: a lookup there trusts a counter below the threshold as proof of absence, so the import
    must leave every stored key counted.  Counter words = oracle's, every key still found on both sides."""
    from paper_2209_07663_amd.binding import Table
    wl, seed = synth.scaled(synth.CONFIGS["cfg2"], samples=1024, capacity=1 << 16), 151
    tab = Table(wl.capacity, wl.dim, seed, wl.freq_threshold, 0, False, max_ids=1 << 18, max_bags=wl.n_bags,
                device=dev, filter_hashes=hashes)
    orc = Oracle(wl.capacity, wl.dim, seed, wl.freq_threshold, 0, False, kind="cuckoo", filter_hashes=hashes)
    batches = [synth.make_batch(wl, seed, s, with_grad=True) for s in range(5)]
    for b in batches[:3]:
        _full_step(tab, orc, b, dev, wl, 1e-5, seed=seed)
    stored = tab.mono_table_export(with_values=False)["keys"]
    assert stored.shape[0] > 1000
    zeros = np.zeros(tab.n_filter, dtype=np.uint32)
    tab.mono_filter_import(torch.from_numpy(zeros.view(np.int32)).to(dev))
    orc.write_filter_words(zeros)
    got = tab.mono_filter_export()
    assert (got == orc.filter_words()).all() and np.count_nonzero(got) >= stored.shape[0] // 2
    k_d = torch.from_numpy(stored).to(dev)
    assert bool((tab.mono_lookup_or_insert(k_d, 3) >= 0).all().item()) and orc.lookup_or_insert(stored, 3).all()
    rng = np.random.default_rng(2)
    first, count = tab.n_filter // 4, tab.n_filter // 2
    words = ((rng.integers(0, 4, size=count) << 8) | rng.integers(0, 3, size=count)).astype(np.uint32)
    tab.mono_filter_import(torch.from_numpy(words.view(np.int32)).to(dev), first)
    orc.write_filter_words(words, first)
    assert (tab.mono_filter_export() == orc.filter_words()).all()
    assert bool((tab.mono_lookup_or_insert(k_d, 3) >= 0).all().item()) and orc.lookup_or_insert(stored, 3).all()
    for b in batches[3:]:
        _full_step(tab, orc, b, dev, wl, 1e-5, seed=seed)
    tab.close()
