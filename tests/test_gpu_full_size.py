"""Full-size configurations on the device, in the launch configuration bench.py times.

configs[1] runs whole against the oracle (it finishes a step in a few seconds).  configs[2],
configs[3] (filled to load 0.9 first) and configs[4] are too large for that, so they are checked on
sampled outputs recomputed one by one in numpy from the device's own table dumps, plus the invariants
that hold at any size.
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
def test_config2_full_size_against_oracle():
    dev = torch.device("cuda:0")
    wl, seed = synth.CONFIGS["cfg2"], 1
    batches = [synth.make_batch(wl, seed, s, with_grad=True) for s in range(3)]
    tab = _table(wl, seed, max(b["keys"].shape[0] for b in batches), dev)
    orc = Oracle(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, kind="cuckoo")
    for b in batches:
        print("config2 full size, step", b["step"], flush=True)
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


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name,samples", [("cfg3", None), ("cfg5", None)])
def test_large_configs_sampled(name, samples):
    dev = torch.device("cuda:0")
    wl, seed = synth.CONFIGS[name], 3
    rtol = 1e-2 if wl.bf16 else 1e-5
    rng = np.random.default_rng(0)
    tab = None
    seen_before = set()
    for step in range(2):
        print(name, "full size, step", step, flush=True)
        b = synth.make_batch(wl, seed, step, with_grad=True)
        keys_h, offs_h, grad_h = b["keys"], b["offsets"], b["grad"]
        if tab is None:
            tab = _table(wl, seed, int(keys_h.shape[0] * 1.05) + 1024, dev)
        keys, offs = torch.from_numpy(keys_h).to(dev), torch.from_numpy(offs_h).to(dev)
        rows = tab.mono_lookup_or_insert(keys, step)
        rows_h = rows.cpu().numpy()
        before = tab.mono_table_export()
        tc.check_placement(before, wl.capacity, 8, seed)
        # the key -> row map handed out is the one stored, and absent keys are exactly the non-admitted ones
        present = rows_h >= 0
        pos = np.searchsorted(before["keys"].view(np.uint64), keys_h[present].view(np.uint64))
        assert (before["keys"][pos] == keys_h[present]).all() and (before["row"][pos] == rows_h[present]).all()
        assert not np.isin(keys_h[~present], before["keys"]).any()
        # admission rule on a sample of distinct keys: present <=> counter word reached the threshold
        uniq = np.unique(keys_h)
        some = rng.choice(uniq, size=min(20000, uniq.shape[0]), replace=False)
        widx = tc.filter_index(some, 4 * wl.capacity, seed).astype(np.int64)
        words = np.array([tab.mono_filter_export(int(i), 1)[0] for i in widx[:300]])
        is_in = np.isin(some[:300], before["keys"])
        was_in = np.array([k in seen_before for k in some[:300].tolist()])
        assert ((words & 255) >= max(wl.freq_threshold, 1))[is_in & ~was_in].all()
        assert (is_in | ((words & 255) < max(wl.freq_threshold, 1)))[~was_in].all()
        # freshly admitted rows carry the initial values
        new = ~np.isin(before["keys"], np.fromiter(seen_before, dtype=np.int64, count=len(seen_before)))
        pick = np.flatnonzero(new)[:2000]
        want = tc.init_rows(before["keys"][pick], wl.dim, seed).astype(np.float32)
        if wl.bf16:
            want = torch.from_numpy(want).to(torch.bfloat16).to(torch.float32).numpy()
        assert (before["rows"][pick] == want).all() and (before["acc"][pick] == 0).all()
        assert (before["last_seen"][np.isin(before["keys"], uniq)] == step).all()
        # pooled sums of sampled bags from the dumped rows
        pooled = tab.mono_gather_pool(rows, offs)
        bags = rng.choice(wl.n_bags, size=3000, replace=False)
        rowmap = np.full(int(before["row"].max()) + 1, -1, dtype=np.int64)
        rowmap[before["row"]] = np.arange(before["row"].shape[0])
        ref = np.zeros((bags.shape[0], wl.dim), dtype=np.float64)
        for j, bg in enumerate(bags.tolist()):
            r = rows_h[offs_h[bg]:offs_h[bg + 1]]
            ref[j] = before["rows"][rowmap[r[r >= 0]]].astype(np.float64).sum(axis=0)
        tc.rows_close(pooled[torch.from_numpy(bags).to(dev)].cpu().numpy(), ref, 1e-5 if not wl.bf16 else 1e-5)
        # update: the hottest keys and a random sample, recomputed from their occurrences
        tab.mono_apply_grad_adagrad(rows, offs, torch.from_numpy(grad_h).to(dev), wl.lr, wl.eps)
        after = tab.mono_table_export()
        assert (after["keys"] == before["keys"]).all() and (after["last_seen"] == before["last_seen"]).all()
        vals, counts = np.unique(keys_h[present], return_counts=True)
        hot = vals[np.argsort(counts)[-8:]]
        chosen = np.unique(np.concatenate([hot, rng.choice(vals, size=400, replace=False)]))
        bag_of = np.repeat(np.arange(wl.n_bags), np.diff(offs_h))
        sel = np.isin(keys_h, chosen)
        k_sel, b_sel = keys_h[sel], bag_of[sel]
        order = np.argsort(k_sel, kind="stable")
        k_sel, b_sel = k_sel[order], b_sel[order]
        starts = np.flatnonzero(np.r_[True, k_sel[1:] != k_sel[:-1]])
        gsum = np.add.reduceat(grad_h[b_sel].astype(np.float64), starts, axis=0)
        kk = k_sel[starts]
        p = np.searchsorted(before["keys"].view(np.uint64), kk.view(np.uint64))
        acc = before["acc"][p].astype(np.float64) + (gsum ** 2).sum(axis=1) / wl.dim
        w = before["rows"][p].astype(np.float64) - wl.lr * gsum / (np.sqrt(acc)[:, None] + wl.eps)
        tc.rows_close(after["rows"][p], w, rtol)
        assert (np.abs(after["acc"][p] - acc) <= 1e-5 * acc).all()
        # rows of keys outside the batch are untouched
        idle = ~np.isin(before["keys"], uniq)
        assert (after["rows"][idle] == before["rows"][idle]).all() and (after["acc"][idle] == before["acc"][idle]).all()
        tab.mono_expire_sweep(step)
        seen_before = set(tab.mono_table_export(with_values=False)["keys"].tolist())
        st = tab.mono_table_stats()
        assert st["n_insert_failed"] == 0 and st["n_lost"] == 0 and st["n_full"] == 0
    tab.close()


@pytest.mark.timeout(900)
def test_config4_filled_to_load_09_then_streaming_steps():
    """configs[3] at full size: the 0.9 * capacity hottest IDs are admitted first (threshold 5: each
    is looked up five times), then drifting batches with a sweep every step.  30 M keys are too many
    for the oracle, so: placement, uniqueness and conservation on the whole dump, the admission rule
    and initial rows on samples, no failed eviction chain, and the same sampled checks per step."""
    dev = torch.device("cuda:0")
    wl, seed = synth.CONFIGS["cfg4"], 4
    drift = synth.DriftMap(wl, seed)
    hot = synth.hottest_ids(wl, int(0.9 * wl.capacity), drift)
    assert np.unique(hot).shape[0] == hot.shape[0]
    batches = [synth.make_batch(wl, seed, s, with_grad=True, drift=drift) for s in range(1, 4)]
    max_ids = max(1 << 23, max(b["keys"].shape[0] for b in batches))
    tab = _table(wl, seed, max_ids, dev)
    rows = torch.empty(max_ids, dtype=torch.int32, device=dev)
    for lo in range(0, hot.shape[0], max_ids):
        chunk = torch.from_numpy(hot[lo:lo + max_ids]).to(dev)
        for rep in range(wl.freq_threshold):
            tab.mono_lookup_or_insert(chunk, 0, rows[: chunk.shape[0]])
        # on the fifth sighting at the latest (keys that share a counter with others get there earlier)
        assert int((rows[: chunk.shape[0]] >= 0).sum().item()) == chunk.shape[0]
    print("config4: filled", flush=True)
    st = tab.mono_table_stats()
    assert st["size"] == hot.shape[0] and st["n_insert_failed"] == 0 and st["n_lost"] == 0 and st["n_full"] == 0
    d = tab.mono_table_export(with_values=False)
    assert (d["keys"].view(np.uint64) == np.sort(hot.view(np.uint64))).all()
    tc.check_placement(d, wl.capacity, 8, seed)
    rng = np.random.default_rng(0)
    stored = d["keys"]
    for b in batches:
        step = b["step"]
        print("config4 full size, step", step, flush=True)
        keys_h, offs_h = b["keys"], b["offsets"]
        keys, offs = torch.from_numpy(keys_h).to(dev), torch.from_numpy(offs_h).to(dev)
        r = tab.mono_lookup_or_insert(keys, step)
        r_h = r.cpu().numpy()
        present = r_h >= 0
        was_stored = np.isin(keys_h, stored)
        assert present[was_stored].all()                      # a stored key is always found
        # the others: present exactly if their counter word reached the threshold (sampled)
        cand = np.unique(keys_h[~was_stored])
        some = rng.choice(cand, size=min(300, cand.shape[0]), replace=False)
        widx = tc.filter_index(some, 4 * wl.capacity, seed).astype(np.int64)
        words = np.array([tab.mono_filter_export(int(i), 1)[0] for i in widx])
        got_in = np.isin(some, keys_h[present])
        assert (got_in == ((words & 255) >= wl.freq_threshold)).all()
        pooled = tab.mono_gather_pool(r, offs)
        tab.mono_apply_grad_adagrad(r, offs, torch.from_numpy(b["grad"]).to(dev), wl.lr, wl.eps)
        assert bool(torch.isfinite(pooled).all().item())
        n_exp = torch.zeros(1, dtype=torch.int64, device=dev)
        tab.mono_expire_sweep(step, n_exp, None)
        assert int(n_exp.item()) == 0                          # nothing is 20 steps old yet
        d = tab.mono_table_export(with_values=False)
        tc.check_placement(d, wl.capacity, 8, seed)
        assert np.isin(stored, d["keys"]).all()
        assert (d["last_seen"][np.isin(d["keys"], np.unique(keys_h[present]))] == step).all()
        stored = d["keys"]
        st = tab.mono_table_stats()
        assert st["size"] == stored.shape[0] and st["n_insert_failed"] == 0 and st["n_lost"] == 0 and st["n_full"] == 0
    assert stored.shape[0] > hot.shape[0]                      # keys keep being admitted at load 0.9
    tab.close()


@pytest.mark.timeout(600)
def test_update_with_more_than_16M_rows_in_use():
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
        print("17M rows: admitting chunk", step, flush=True)
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
    print("17M rows: training step", flush=True)
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
    print("17M rows: comparing the tables", flush=True)
    d = tab.mono_table_export()
    tc.check_placement(d, cap, 8, seed)
    tc.assert_same_table(d, orc.dump(), exact_rows=False, rtol=1e-5)
    trained = np.isin(d["keys"], keys_h)
    assert (d["acc"][trained] > 0).all() and (d["acc"][~trained] == 0).all()
    tab.close()
