"""Pins for the oracle's maintenance operations: touched keys (the paper's incremental parameter
synchronisation), snapshot / restore (its fault tolerance) and rehash / grow (section 2.1).

Each is pinned to something other than the oracle's own code: a Python set kept beside the run, the
payload size the paper prints for its synchronisation example, equality of a restored table with
the one it was taken from (also across the two independent models, and through further training),
and the index relation that top-bit addressing fixes between a counter and its children.
"""
import numpy as np
import pytest
import torch

from oracle import Oracle
from tests import table_checks as tc

KINDS = ["map", "cuckoo"]


def _batch(rng, n_bags, universe, dim, lam=2.0):
    lens = rng.poisson(lam, size=n_bags) + 1
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    keys = rng.zipf(1.3, size=int(offs[-1])).astype(np.int64) % universe
    grad = rng.standard_normal((n_bags, dim)).astype(np.float32)
    return keys, offs, grad


def _same_dump(a, b, slots=False):
    assert (a["keys"] == b["keys"]).all() and (a["last_seen"] == b["last_seen"]).all()
    assert (a["rows"].view(np.uint32) == b["rows"].view(np.uint32)).all()
    assert (a["acc"].view(np.uint32) == b["acc"].view(np.uint32)).all()
    if slots:
        assert (a["slot"] == b["slot"]).all()


# ---- touched keys ---------------------------------------------------------------------------------

@pytest.mark.parametrize("kind", KINDS)
def test_touched_keys_follow_a_python_set(kind):
    rng = np.random.default_rng(11)
    dim = 4
    o = Oracle(1 << 12, dim, 7, freq_threshold=2, expire_steps=3, kind=kind, n_filter=1 << 20)
    mine = set()
    for step in range(14):
        keys, offs, grad = _batch(rng, 60, 400, dim)
        present = o.lookup_or_insert(keys, step)
        if step % 3 != 2:                                # some steps only look up: nothing is trained
            o.apply_grad_adagrad(keys, offs, grad, 0.05, 1e-8)
            mine |= set(keys[present].tolist())          # trained = stored keys that received a gradient
        if step % 2 == 1:
            mine -= set(o.expire_sweep(step).tolist())   # an erased key has no parameters to push
        if step % 4 == 3:
            got = o.take_touched()
            assert got.tolist() == sorted(mine)
            assert set(got.tolist()) <= set(o.dump()["keys"].tolist())
            mine.clear()
            assert o.take_touched().shape[0] == 0        # taking the set clears it


@pytest.mark.parametrize("kind", KINDS)
def test_touched_key_cases(kind):
    dim = 2
    o = Oracle(1 << 8, dim, 1, freq_threshold=2, expire_steps=2, kind=kind, n_filter=1 << 16)
    offs = np.array([0, 1, 2, 3], dtype=np.int64)
    g = np.ones((3, dim), dtype=np.float32)
    k = np.array([10, 10, 20], dtype=np.int64)           # 10 seen twice -> admitted; 20 once -> not
    assert o.lookup_or_insert(k, 0).tolist() == [True, True, False]
    o.apply_grad_adagrad(k, offs, g, 0.1, 1e-8)
    o.apply_grad_adagrad(k, offs, g, 0.1, 1e-8)          # trained twice, reported once; 20 is not stored
    assert o.take_touched().tolist() == [10]
    assert o.lookup_or_insert(k, 1).tolist() == [True, True, True]
    assert o.take_touched().tolist() == []               # looked up, admitted, but not trained
    o.apply_grad_adagrad(k, offs, g * 0, 0.1, 1e-8)      # a zero gradient still counts as trained
    assert o.take_touched().tolist() == [10, 20]
    o.apply_grad_adagrad(k, offs, g, 0.1, 1e-8)
    assert sorted(o.expire_sweep(3).tolist()) == [10, 20]
    assert o.take_touched().tolist() == []               # trained, then expired before the synchronisation


def test_synchronisation_payload_of_the_papers_example():
    """Section 3.2.2 (synchronisation frequency of sparse parameters): 100,000 IDs updated in a minute, embedding
    dimension 1024 -> 4 KB x 100,000, about 400 MB to transfer."""
    dim, ids = 1024, 100000
    o = Oracle(1 << 18, dim, 3, freq_threshold=1, kind="map")
    keys = (np.arange(ids, dtype=np.int64) * 7919) % (1 << 40)
    keys = np.concatenate([keys, keys[:5000]])           # some IDs trained more than once
    offs = np.arange(keys.shape[0] + 1, dtype=np.int64)
    o.lookup_or_insert(keys, 0)
    o.apply_grad_adagrad(keys, offs, np.zeros((keys.shape[0], dim), dtype=np.float32), 0.1, 1e-8)
    touched = o.take_touched()
    assert touched.shape[0] == ids
    payload = touched.shape[0] * dim * 4
    assert payload == 4096 * 100000 and abs(payload / 400e6 - 1) < 0.03


# ---- snapshot / restore ---------------------------------------------------------------------------

def _train(o, rng, steps, first_step, dim, universe=3000):
    out = []
    for step in range(first_step, first_step + steps):
        keys, offs, grad = _batch(rng, 400, universe, dim)
        present = o.lookup_or_insert(keys, step)
        pooled = o.pool(keys, offs)
        o.apply_grad_adagrad(keys, offs, grad, 0.05, 1e-8)
        erased = o.expire_sweep(step)
        out.append((present, pooled, erased))
    return out


@pytest.mark.parametrize("src_kind,dst_kind", [("cuckoo", "cuckoo"), ("map", "cuckoo"), ("cuckoo", "map")])
@pytest.mark.parametrize("bf16", [False, True])
def test_restored_table_equals_the_original_and_trains_on_identically(src_kind, dst_kind, bf16):
    dim, cap, seed = 8, 1 << 12, 5
    mk = lambda kind: Oracle(cap, dim, seed, freq_threshold=2, expire_steps=4, bf16=bf16, kind=kind, n_filter=1 << 14)
    a = mk(src_kind)
    _train(a, np.random.default_rng(1), 5, 0, dim)
    snap, words = a.dump(), a.filter_words()
    assert snap["keys"].shape[0] > 100
    b = mk(dst_kind)
    perm = np.random.default_rng(2).permutation(snap["keys"].shape[0])     # record order must not matter
    assert b.import_entries(snap["keys"][perm], snap["rows"][perm], snap["acc"][perm], snap["last_seen"][perm]) == 0
    b.write_filter_words(words)
    _same_dump(a.dump(), b.dump())
    assert (a.filter_words() == b.filter_words()).all()
    if dst_kind == "cuckoo":
        tc.check_placement(b.dump(), cap, 8, seed)
    # continue-training equivalence: the same further batches give the same outputs and the same state
    ra = _train(a, np.random.default_rng(3), 6, 5, dim)
    rb = _train(b, np.random.default_rng(3), 6, 5, dim)
    for (pa, qa, ea), (pb, qb, eb) in zip(ra, rb):
        assert (pa == pb).all() and (qa.view(np.uint32) == qb.view(np.uint32)).all() and (ea == eb).all()
    _same_dump(a.dump(), b.dump())
    assert (a.filter_words() == b.filter_words()).all()


@pytest.mark.parametrize("kind", KINDS)
def test_import_rejects_stored_and_reserved_keys_and_rounds_bf16(kind):
    dim = 4
    o = Oracle(1 << 8, dim, 9, freq_threshold=1, bf16=True, kind=kind, n_filter=1 << 12)
    o.lookup_or_insert(np.array([5], dtype=np.int64), 0)
    before = o.dump()
    rows = np.array([[1.001, -2.003, 3.14159, 1e-3]] * 3, dtype=np.float32)
    rejected = o.import_entries(np.array([5, -1, 6], dtype=np.int64), rows, np.array([1, 2, 3], dtype=np.float32),
                                np.array([7, 8, 9], dtype=np.uint32))
    assert rejected == 2                                   # 5 is stored, -1 is the reserved key
    d = o.dump()
    assert d["keys"].tolist() == [5, 6]
    assert (d["rows"][0] == before["rows"][0]).all() and d["last_seen"].tolist() == [0, 9] and d["acc"][1] == 3
    want = torch.from_numpy(rows[2]).to(torch.bfloat16).to(torch.float32).numpy()
    assert (d["rows"][1] == want).all()                    # stored in the table's storage type


# ---- rehash / grow --------------------------------------------------------------------------------

def test_rehash_keeps_contents_and_moves_keys_to_the_new_generations_buckets():
    dim, cap, seed = 4, 1 << 10, 13
    o = Oracle(cap, dim, seed, freq_threshold=1, expire_steps=0, kind="cuckoo", n_filter=1 << 12)
    rng = np.random.default_rng(4)
    _train(o, rng, 3, 0, dim, universe=600)
    before, words = o.dump(), o.filter_words()
    tc.check_placement(before, cap, 8, seed, generation=0)
    o.rehash(cap, 1)
    after = o.dump()
    _same_dump(before, after)
    assert (o.filter_words() == words).all()              # same capacity: the counters stay as they are
    tc.check_placement(after, cap, 8, seed, generation=1)
    with pytest.raises(AssertionError):                   # ... and no longer sit where generation 0 puts them
        tc.check_placement(after, cap, 8, seed, generation=0)
    assert o.insert_failures == 0


@pytest.mark.parametrize("kind", KINDS)
def test_grow_spreads_every_counter_over_its_children(kind):
    dim, cap, seed, k = 2, 1 << 8, 17, 2
    o = Oracle(cap, dim, seed, freq_threshold=3, kind=kind, n_filter=1 << 16)
    rng = np.random.default_rng(5)
    keys = rng.integers(0, 1 << 40, size=3000).astype(np.int64)
    idx_old = np.array([o.filter_index(x) for x in keys[:500]])
    o.lookup_or_insert(keys, 0)                            # single occurrences: counted, not admitted
    words = o.filter_words()
    o.rehash(cap << k, 1)
    assert o.capacity == cap << k and o.n_filter == 1 << (16 + k)
    grown = o.filter_words()
    assert (grown == np.repeat(words, 1 << k)).all()
    # a key's new counter is a child of its old one (top-bit addressing), so no count is ever lost
    idx_new = np.array([o.filter_index(x) for x in keys[:500]])
    assert (idx_new >> k == idx_old).all()
    assert (idx_new == tc.filter_index(keys[:500], 1 << (16 + k), seed).astype(np.int64)).all()
    # hence two more sightings still admit (threshold 3), exactly as without the rehash
    twin = Oracle(cap, dim, seed, freq_threshold=3, kind=kind, n_filter=1 << 16)
    twin.lookup_or_insert(keys, 0)
    some = np.concatenate([keys[:100], keys[:100]])
    assert o.lookup_or_insert(some, 1).all() and twin.lookup_or_insert(some, 1).all()


def test_models_agree_through_growth_and_further_training():
    dim, cap, seed = 4, 1 << 9, 19
    a = Oracle(cap, dim, seed, freq_threshold=2, expire_steps=5, kind="cuckoo", n_filter=1 << 16)
    b = Oracle(cap, dim, seed, freq_threshold=2, expire_steps=5, kind="map", n_filter=1 << 16)
    for o in (a, b):
        _train(o, np.random.default_rng(6), 4, 0, dim, universe=2000)
        o.rehash(cap * 4, 3)
    _same_dump(a.dump(), b.dump())
    ra = _train(a, np.random.default_rng(7), 5, 4, dim, universe=2000)
    rb = _train(b, np.random.default_rng(7), 5, 4, dim, universe=2000)
    for (pa, qa, ea), (pb, qb, eb) in zip(ra, rb):
        assert (pa == pb).all() and (qa.view(np.uint32) == qb.view(np.uint32)).all() and (ea == eb).all()
    _same_dump(a.dump(), b.dump())
    assert (a.filter_words() == b.filter_words()).all()
    tc.check_placement(a.dump(), cap * 4, 8, seed, generation=3)


def test_rehash_empties_the_overflow_stash_of_a_one_slot_cuckoo_table():
    """Section 2.1: an insertion that runs into a cycle is answered by a rehash.  One-slot buckets
    (the structure the paper describes) at load 0.45 with a short chain bound overflow; new hash
    functions in a table twice the size place every key."""
    dim, cap, seed = 2, 1 << 8, 23
    o = Oracle(cap, dim, seed, freq_threshold=1, kind="cuckoo", n_filter=1 << 12, bucket=1, max_kicks=6)
    keys = (np.arange(115, dtype=np.int64) + 1) * 2654435761
    assert o.lookup_or_insert(keys, 0).all()
    assert o.insert_failures > 0 and (o.dump()["slot"] == -2).sum() == o.insert_failures
    failures = o.insert_failures
    before = o.dump()
    generation = 1
    o.rehash(cap * 2, generation)
    while o.insert_failures > failures and generation < 8:   # an unlucky generation: rehash again
        failures = o.insert_failures
        generation += 1
        o.rehash(cap * 2, generation)
    after = o.dump()
    _same_dump(before, after)
    assert (after["slot"] >= 0).all()
    tc.check_placement(after, cap * 2, 1, seed, generation=generation)
    assert o.lookup_or_insert(keys, 1).all()


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("thr,hashes", [(0, 1), (1, 2), (3, 1), (3, 3)])
def test_restored_keys_count_as_seen_threshold_times(kind, thr, hashes):
    """Records can be restored without their counters: a placed key's counters are raised to the
    admission threshold (never lowered), so "stored implies counted" holds as after an admission."""
    dim, seed, n_filter = 2, 29, 1 << 16
    o = Oracle(1 << 10, dim, seed, freq_threshold=thr, kind=kind, n_filter=n_filter, filter_hashes=hashes)
    for step in range(6):
        o.lookup_or_insert(np.array([77, 78], dtype=np.int64), step)      # 77 and 78 get counted / admitted
    keys = np.array([5, 6, 7], dtype=np.int64)
    before = o.filter_words()
    assert o.import_entries(keys, np.zeros((3, dim), np.float32), np.zeros(3, np.float32), np.zeros(3, np.uint32)) == 0
    after = o.filter_words()
    least = max(thr, 1)
    touched = set()
    for key in keys.tolist():
        for j in range(hashes):
            i = int(tc.filter_index(np.array([key]), n_filter, seed, j)[0])
            touched.add(i)
            assert after[i] & 255 == max(before[i] & 255, least) and after[i] >> 8 == before[i] >> 8
    others = np.setdiff1d(np.arange(n_filter), np.array(sorted(touched)))
    assert (after[others] == before[others]).all()
    # a restored key is found without being counted again
    assert o.lookup_or_insert(keys, 9).all()
    assert (o.filter_words() == after).all()


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("thr,hashes,expire", [(3, 1, 0), (2, 3, 0), (4, 2, 5)])
def test_counter_words_written_over_a_populated_table_keep_stored_keys_counted(kind, thr, hashes, expire):
    """Counter words may be restored after the records, and they may be anything, all zeros included.  On a
    table that never expires keys every counter of a stored key inside the written range ends at the
    threshold or above (its step field is the written one), every other written counter is exactly the
    written word, and counters outside the range are untouched.  Where counters age (expire > 0) a stored
    key's counter proves nothing, and the words are stored exactly as written: the restored state is the
    snapshot.  The witness indexes the counters with the independent numpy hashes."""
    dim, seed, n_filter = 2, 31, 1 << 12
    o = Oracle(1 << 10, dim, seed, freq_threshold=thr, expire_steps=expire, kind=kind, n_filter=n_filter,
               filter_hashes=hashes)
    keys = (np.arange(200, dtype=np.int64) + 1) * 7919
    for step in range(thr):
        o.lookup_or_insert(keys, step)
    assert o.lookup_or_insert(keys, thr).all()
    before = o.filter_words()
    first, count = 1000, 2000                                  # a window in the middle of the array
    rng = np.random.default_rng(0)
    words = ((rng.integers(0, 50, size=count) << 8) | rng.integers(0, 2, size=count)).astype(np.uint32)
    words[::3] = 0
    o.write_filter_words(words, first)
    after = o.filter_words()
    of_stored = set()
    for j in range(hashes):
        of_stored.update(int(i) for i in tc.filter_index(keys, n_filter, seed, j))
    for i in range(n_filter):
        if not first <= i < first + count:
            assert after[i] == before[i]
            continue
        w = int(words[i - first])
        if i in of_stored and expire == 0:
            assert after[i] >> 8 == w >> 8 and after[i] & 255 == max(w & 255, thr)
        else:
            assert after[i] == w
    # all-zero words over the whole array: every stored key is still counted, nothing else is
    o.write_filter_words(np.zeros(n_filter, dtype=np.uint32))
    z = o.filter_words()
    if expire == 0:
        assert set(np.flatnonzero(z).tolist()) == of_stored and (z[sorted(of_stored)] == thr).all()
    else:
        assert not z.any()
    assert o.lookup_or_insert(keys, thr + 1).all()


@pytest.mark.parametrize("kind", KINDS)
def test_restore_on_a_table_with_ageing_counters_is_the_snapshot_in_either_order(kind):
    """Records then counter words, or counter words then records: a table whose counters age comes back
    exactly as it was snapshotted (a stored key whose counter has restarted since its admission keeps
    that low counter)."""
    dim, seed, n_filter, thr = 2, 33, 1 << 10, 3
    mk = lambda: Oracle(1 << 8, dim, seed, freq_threshold=thr, expire_steps=4, kind=kind, n_filter=n_filter)
    a = mk()
    keys = (np.arange(40, dtype=np.int64) + 1) * 104729
    for step in range(thr):
        a.lookup_or_insert(keys, step)
    # other keys that share counters with stored ones touch them much later: those counters restart at 1
    others = np.arange(5000, 5400, dtype=np.int64)
    a.lookup_or_insert(keys, 9)
    a.lookup_or_insert(others, 9)
    snap, words = a.dump(), a.filter_words()
    idx = tc.filter_index(snap["keys"], n_filter, seed).astype(np.int64)
    assert ((words[idx] & 255) < thr).any()               # the case this test is about does occur
    for records_first in (True, False):
        b = mk()
        if records_first:
            assert b.import_entries(snap["keys"], snap["rows"], snap["acc"], snap["last_seen"]) == 0
            b.write_filter_words(words)
        else:
            b.write_filter_words(words)
            assert b.import_entries(snap["keys"], snap["rows"], snap["acc"], snap["last_seen"]) == 0
        _same_dump(b.dump(), snap)
        assert (b.filter_words() == words).all()
