"""Pins for the multi-hash occurrence filter (the "probabilistic filter" of the paper's section 2.1,
read as a counting filter with k hashes whose count for a key is the minimum of the key's counters).

The oracle is checked against a count-min model written here in Python on the numpy hashes of
tests/table_checks.py (shared with neither implementation), against exact per-key counts when the
array is so large that no two keys share a counter, and against the property that a counting filter
never under-counts (no false negatives).
"""
import collections

import numpy as np
import pytest

from oracle import Oracle
from tests import table_checks as tc

KINDS = ["map", "cuckoo"]


def _stream(rng, steps, n, universe):
    return [rng.zipf(1.2, size=n).astype(np.int64) % universe for _ in range(steps)]


def _count_min_model(batches, seed, n_filter, hashes, thr):
    """Returns per step the set admitted in that step, and the final counters {index: (last step, count)}."""
    present, counters, admitted_at = set(), {}, []
    for step, keys in enumerate(batches):
        idx = [tc.filter_index(keys, n_filter, seed, j).astype(np.int64) for j in range(hashes)]
        missing = [i for i, k in enumerate(keys.tolist()) if k not in present]
        for i in missing:
            for j in range(hashes):
                c = counters.get(int(idx[j][i]), (0, 0))[1]
                counters[int(idx[j][i])] = (step, min(255, c + 1))
        new = set()
        for i in missing:
            if min(counters[int(idx[j][i])][1] for j in range(hashes)) >= max(thr, 1):
                new.add(int(keys[i]))
        present |= new
        admitted_at.append(new)
    return admitted_at, counters


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("hashes,n_filter", [(1, 1 << 9), (2, 1 << 9), (3, 1 << 7), (4, 1 << 10), (2, 2)])
def test_oracle_equals_the_count_min_model(kind, hashes, n_filter):
    seed, thr = 31, 3
    batches = _stream(np.random.default_rng(hashes * 100 + n_filter), steps=6, n=500, universe=900)
    want_sets, want_counters = _count_min_model(batches, seed, n_filter, hashes, thr)
    o = Oracle(1 << 12, 2, seed, freq_threshold=thr, kind=kind, n_filter=n_filter, filter_hashes=hashes)
    stored = set()
    for step, keys in enumerate(batches):
        present = o.lookup_or_insert(keys, step)
        now = set(keys[present].tolist()) | stored
        assert now - stored == want_sets[step], "admitted sets differ at step %d" % step
        stored = now
    words = o.filter_words()
    for index in range(n_filter):
        last, count = want_counters.get(index, (0, 0))
        assert words[index] == (last << 8 | count), "counter %d" % index
    for key in batches[0][:20].tolist():                    # the oracle's own index function, hash by hash
        for j in range(hashes):
            assert o.filter_index(key, j) == int(tc.filter_index(np.array([key]), n_filter, seed, j)[0])


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("hashes", [1, 2, 3, 4])
def test_large_array_gives_exact_counts_and_small_ones_never_under_count(kind, hashes):
    seed, thr = 37, 4
    batches = _stream(np.random.default_rng(9), steps=5, n=400, universe=700)
    # exact admission: a key enters at the step in which its number of missed occurrences reaches thr
    exact_step, seen = {}, collections.Counter()
    for step, keys in enumerate(batches):
        for k in keys.tolist():
            if k not in exact_step:
                seen[k] += 1
        for k in set(keys.tolist()):
            if k not in exact_step and seen[k] >= thr:
                exact_step[k] = step
    for n_filter in (1 << 24, 1 << 8, 1 << 5):
        o = Oracle(1 << 12, 2, seed, freq_threshold=thr, kind=kind, n_filter=n_filter, filter_hashes=hashes)
        got_step = {}
        for step, keys in enumerate(batches):
            present = o.lookup_or_insert(keys, step)
            for k in set(keys[present].tolist()):
                got_step.setdefault(k, step)
        if n_filter == 1 << 24:
            idx = np.concatenate([tc.filter_index(np.array(sorted(seen)), n_filter, seed, j) for j in range(hashes)])
            if np.unique(idx).shape[0] == idx.shape[0]:      # no two (key, hash) pairs share a counter
                assert got_step == exact_step
        # a counting filter may admit early or wrongly, never late: no false negatives
        for k, s in exact_step.items():
            assert k in got_step and got_step[k] <= s
