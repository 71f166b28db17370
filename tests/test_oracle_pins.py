"""Pins of the CPU oracle against things other than itself (CPU only).

What fixes each part: published SplitMix64 outputs (hashing), a hand trace of the insertion
procedure of section 2.1 of the paper (placement), the std::map definition on thousands of tiny
random cases (membership, admission, expiry, pooling, update), library routines (embedding_bag,
index_add, torch.optim.Adagrad, torch's bfloat16 cast) and closed forms.
"""
import os

import numpy as np
import pytest
import torch

from oracle import Oracle, oracle_lib
from tests import table_checks as tc


def test_mixer_matches_published_splitmix64(golden_dir):
    want = [int(l, 16) for l in open(os.path.join(golden_dir, "splitmix64_seed0.txt")) if l.startswith("0x")]
    lib = oracle_lib()
    assert [lib.orc_salt(0, i) for i in range(3)] == want
    # salt i is mix(seed + (i+1) * golden-ratio increment): the generator's definition
    assert lib.orc_mix64(0x9E3779B97F4A7C15) == want[0]
    # numpy witness used by the placement checker agrees as well
    assert [int(tc.salt(0, i)) for i in range(3)] == want
    z = np.random.default_rng(0).integers(0, 2**63, size=1000, dtype=np.int64).astype(np.uint64)
    assert [lib.orc_mix64(int(v)) for v in z[:200]] == [int(v) for v in tc.mix64(z[:200])]


def test_mixer_is_a_bijection_on_a_sample():
    z = np.arange(1 << 16, dtype=np.uint64)
    assert np.unique(tc.mix64(z)).shape[0] == z.shape[0]


def test_init_value_grid_range_and_moments():
    lib = oracle_lib()
    seed, dim = 12345, 64
    keys = np.random.default_rng(1).integers(0, 2**62, size=4000, dtype=np.int64)
    got = np.array([[lib.orc_init_value(seed, int(k), j) for j in range(dim)] for k in keys[:300]], dtype=np.float32)
    # exactly on the 2^-27 grid inside [-2^-4, 2^-4)
    scaled = got.astype(np.float64) * (1 << 27)
    assert (scaled == np.round(scaled)).all()
    assert (got >= -0.0625).all() and (got < 0.0625).all()
    # integer-arithmetic witness: bit-for-bit the same numbers
    assert (tc.init_rows(keys[:300], dim, seed) == got.astype(np.float64)).all()
    # uniform: mean 0, variance a^2/3 (a = 2^-4), over 4000*64 draws
    big = tc.init_rows(keys, dim, seed)
    assert abs(big.mean()) < 4 * 0.0625 / np.sqrt(3 * big.size)
    assert abs(big.var() / (0.0625**2 / 3) - 1) < 0.02
    # different columns and different seeds decorrelate
    assert abs(np.corrcoef(big[:, 0], big[:, 1])[0, 1]) < 0.06
    assert not np.array_equal(tc.init_rows(keys[:10], dim, seed), tc.init_rows(keys[:10], dim, seed + 1))


def test_bf16_round_matches_torch_cast():
    lib = oracle_lib()
    rng = np.random.default_rng(2)
    x = np.concatenate([rng.standard_normal(3000).astype(np.float32) * 0.05,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, -1.00390625, 3.0e38, 1e-40,
                                  np.inf, -np.inf], dtype=np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([lib.orc_bf16_round(float(v)) for v in x], dtype=np.float32)
    assert (got.view(np.uint32) == want.view(np.uint32)).all()
    assert np.isnan(lib.orc_bf16_round(float("nan")))


def test_filter_word_closed_form():
    lib = oracle_lib()
    w = 0
    for i in range(1, 300):  # one touch per call, same step: count = min(255, i)
        w = lib.orc_filter_touch(w, 7, 0)
        assert w == (7 << 8) | min(255, i)
    # ageing: untouched for >= expire steps restarts from zero, otherwise keeps counting
    w = lib.orc_filter_touch(0, 10, 5)
    assert w == (10 << 8) | 1
    assert lib.orc_filter_touch(w, 14, 5) == (14 << 8) | 2   # 4 steps idle: kept
    assert lib.orc_filter_touch(w, 15, 5) == (15 << 8) | 1   # 5 steps idle: restarted
    assert lib.orc_filter_touch(w, 1000, 0) == (1000 << 8) | 2  # expire 0: never aged


def test_cuckoo_insertion_hand_trace(golden_dir):
    """One slot per cell, toy hashes: the oracle's placement follows the paper's procedure."""
    steps = []
    for line in open(os.path.join(golden_dir, "cuckoo_toy_trace.txt")):
        if line.startswith("#") or not line.strip():
            continue
        parts = line.split()
        steps.append((int(parts[0]), {int(p.split(":")[0]): int(p.split(":")[1]) for p in parts[1:]}))
    o = Oracle(8, 4, seed=0, kind="cuckoo", bucket=1, max_kicks=8, hash_mode=1, n_filter=64)
    for t, (key, want) in enumerate(steps):
        present = o.lookup_or_insert(np.array([key]), t)
        assert present.all()
        d = o.dump()
        assert dict(zip(d["keys"].tolist(), d["slot"].tolist())) == want
        assert o.insert_failures == 0
    # 21 hashes to cells already shared by 1, 5 and 17 (T0[1], T1[0], T1[1]): four keys, three cells,
    # the chain cycles; the element left over is kept aside and every key is still found
    assert o.lookup_or_insert(np.array([21]), 10).all()
    assert o.insert_failures == 1
    assert o.lookup_or_insert(np.array([1, 5, 6, 9, 13, 17, 21]), 11).all()
    assert sorted(o.dump()["keys"].tolist()) == [1, 5, 6, 9, 13, 17, 21]


def _random_case(rng):
    cap = int(rng.choice([16, 32, 64, 256]))
    dim = int(rng.choice([1, 4, 8]))
    thr = int(rng.integers(0, 4))
    exp = int(rng.integers(0, 4))
    bf16 = bool(rng.integers(0, 2))
    universe = int(cap * rng.choice([1, 2, 4]))
    bucket = int(rng.choice([1, 2, 4, 8]))
    return cap, dim, thr, exp, bf16, universe, bucket


N_RANDOM = int(os.environ.get("ORACLE_RANDOM_CASES", "6000"))


def test_cuckoo_oracle_equals_map_definition_on_random_tiny_cases():
    """R1 (cuckoo) against R0 (std::map): every observable, bit for bit, on tiny random inputs."""
    master = np.random.default_rng(2024)
    n_steps_total = 0
    for case in range(N_RANDOM):
        rng = np.random.default_rng(master.integers(0, 2**63))
        cap, dim, thr, exp, bf16, universe, bucket = _random_case(rng)
        seed = int(rng.integers(0, 2**62))
        # the filter is wide, so that (almost always) no two test keys share a counter; both models
        # use the same hashed index, so they agree either way
        kw = dict(dim=dim, seed=seed, freq_threshold=thr, expire_steps=exp, bf16=bf16, n_filter=1 << 16)
        r0 = Oracle(cap, kind="map", **kw)
        r1 = Oracle(cap, kind="cuckoo", bucket=bucket, max_kicks=64, **kw)
        step = 0
        for _ in range(int(rng.integers(2, 9))):
            step += int(rng.integers(0, 3))
            n_bags = int(rng.integers(0, 12))
            lens = rng.integers(0, 4, size=n_bags)
            offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
            n = int(offsets[-1])
            # keep the load low enough for the bucket width so that no eviction chain fails
            hi = universe if bucket >= 4 else max(2, min(universe, cap // 4))
            keys = rng.integers(0, hi, size=n).astype(np.int64)
            if n and rng.random() < 0.2:
                keys[rng.integers(0, n)] = -1  # padding key
            p0, p1 = r0.lookup_or_insert(keys, step), r1.lookup_or_insert(keys, step)
            if r1.insert_failures:
                break  # behaviour past a failed chain is not pinned
            assert (p0 == p1).all()
            assert (r0.pool(keys, offsets).view(np.uint32) == r1.pool(keys, offsets).view(np.uint32)).all()
            if rng.random() < 0.7:
                g = rng.standard_normal((n_bags, dim)).astype(np.float32)
                r0.apply_grad_adagrad(keys, offsets, g, 0.05, 1e-8)
                r1.apply_grad_adagrad(keys, offsets, g, 0.05, 1e-8)
            if rng.random() < 0.6:
                now = step + int(rng.integers(0, 2))
                assert r0.expire_sweep(now).tolist() == r1.expire_sweep(now).tolist()
                step = max(step, now)
            d0, d1 = r0.dump(), r1.dump()
            tc.assert_same_table(d1, d0, exact_rows=True)
            if bucket >= 1 and (d1["slot"] >= 0).all():
                tc.check_placement(d1, cap, bucket, seed)
            if n:
                idx = [r0.filter_index(int(k)) for k in keys if k != -1]
                assert [r0.filter_words(i, 1)[0] for i in idx] == [r1.filter_words(i, 1)[0] for i in idx]
            n_steps_total += 1
    assert n_steps_total > 3 * N_RANDOM


def _filled(kind, dim, n_keys, bf16=False, cap=1 << 12):
    o = Oracle(cap, dim, seed=99, freq_threshold=1, kind=kind, bf16=bf16)
    keys = np.arange(1000, 1000 + n_keys, dtype=np.int64) * 7919
    assert o.lookup_or_insert(keys, 0).all()
    return o, keys


@pytest.mark.parametrize("kind", ["map", "cuckoo"])
def test_pool_equals_embedding_bag(kind):
    o, keys = _filled(kind, 16, 500)
    rng = np.random.default_rng(5)
    lens = rng.integers(0, 7, size=200)
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    idx = rng.integers(0, 600, size=int(offsets[-1]))       # indices >= 500 are keys never inserted
    batch_keys = np.where(idx < 500, keys[np.minimum(idx, 499)], 10**15 + idx).astype(np.int64)
    d = o.dump()
    weight = np.zeros((601, 16), dtype=np.float64)           # row 600 = the zero row of absent keys
    pos = {k: i for i, k in enumerate(d["keys"].tolist())}
    for i, k in enumerate(keys.tolist()):
        weight[i] = d["rows"][pos[k]]
    want = torch.nn.functional.embedding_bag(torch.from_numpy(np.where(idx < 500, idx, 600)),
                                             torch.from_numpy(weight), torch.from_numpy(offsets[:-1]),
                                             mode="sum").numpy()
    got = o.pool(batch_keys, offsets)
    assert np.abs(got - want).max() <= 1e-7
    assert (got[lens == 0] == 0).all()


@pytest.mark.parametrize("kind", ["map", "cuckoo"])
@pytest.mark.parametrize("eps", [1e-8, 0.25])               # a large eps tells "outside the root" from "inside"
def test_update_equals_index_add_then_closed_form_adagrad(kind, eps):
    dim, lr = 8, 0.05
    o, keys = _filled(kind, dim, 64)
    before = o.dump()
    rng = np.random.default_rng(6)
    lens = rng.integers(1, 6, size=300)
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    idx = rng.integers(0, 64, size=int(offsets[-1]))
    idx[:40] = 3                                              # a hot key with many duplicates
    grad = rng.standard_normal((300, dim)).astype(np.float32)
    o.apply_grad_adagrad(keys[idx], offsets, grad, lr, eps)
    after = o.dump()
    # library scatter-reduce: expand bag gradients to occurrences and index_add them per key
    bag_of = np.repeat(np.arange(300), lens)
    g = torch.zeros(64, dim, dtype=torch.float64).index_add_(0, torch.from_numpy(idx),
                                                            torch.from_numpy(grad[bag_of].astype(np.float64))).numpy()
    pos = {k: i for i, k in enumerate(before["keys"].tolist())}
    for u in range(64):
        r = pos[int(keys[u])]
        touched = (idx == u).any()
        if not touched:
            assert (after["rows"][r] == before["rows"][r]).all() and after["acc"][r] == 0
            continue
        # one step from acc = 0: acc = |g|^2 / D, dw = -lr g / (|g| / sqrt(D) + eps)
        acc = (g[u] ** 2).sum() / dim
        want = before["rows"][r].astype(np.float64) - lr * g[u] / (np.sqrt(acc) + eps)
        assert np.abs(after["rows"][r] - want).max() <= 1e-7
        assert abs(after["acc"][r] - acc) <= 1e-6 * acc


@pytest.mark.parametrize("kind", ["map", "cuckoo"])
@pytest.mark.parametrize("eps", [1e-8, 0.25])
def test_dim1_equals_torch_adagrad_over_several_steps(kind, eps):
    """With one element per row, row-wise Adagrad is the textbook element-wise optimizer."""
    lr = 0.05
    o, keys = _filled(kind, 1, 32)
    d = o.dump()
    order = np.argsort(np.argsort(keys.astype(np.uint64)))  # position of keys[i] in the sorted dump
    param = torch.tensor(d["rows"][order, 0].astype(np.float64), requires_grad=True)
    opt = torch.optim.Adagrad([param], lr=lr, eps=eps, initial_accumulator_value=0.0, lr_decay=0, weight_decay=0)
    rng = np.random.default_rng(7)
    for step in range(1, 6):
        lens = rng.integers(1, 4, size=50)
        offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        idx = rng.integers(0, 32, size=int(offsets[-1]))
        grad = rng.standard_normal((50, 1)).astype(np.float32)
        o.apply_grad_adagrad(keys[idx], offsets, grad, lr, eps)
        dense = np.zeros(32, dtype=np.float64)
        np.add.at(dense, idx, grad[np.repeat(np.arange(50), lens), 0].astype(np.float64))
        # torch updates every element, also those with zero gradient: those stay put (0 / (0 + eps))
        opt.zero_grad()
        param.grad = torch.from_numpy(dense.copy())
        opt.step()
        got = o.dump()["rows"][order, 0]
        assert np.abs(got - param.detach().numpy()).max() <= 2e-7 * step


def test_bf16_table_rounds_on_every_store():
    o, keys = _filled("cuckoo", 8, 40, bf16=True)
    f, _ = _filled("cuckoo", 8, 40, bf16=False)
    d, df = o.dump(), f.dump()
    want = torch.from_numpy(df["rows"]).to(torch.bfloat16).to(torch.float32).numpy()
    assert (d["rows"] == want).all()
    grad = np.random.default_rng(8).standard_normal((40, 8)).astype(np.float32)
    offsets = np.arange(41, dtype=np.int64)
    o.apply_grad_adagrad(keys, offsets, grad, 0.05, 1e-8)
    rows = o.dump()["rows"]
    assert (rows == torch.from_numpy(rows).to(torch.bfloat16).to(torch.float32).numpy()).all()
    # fp32 update of the widened bf16 value, then one rounding
    pos = {k: i for i, k in enumerate(d["keys"].tolist())}
    for i, k in enumerate(keys.tolist()):
        g = grad[i].astype(np.float64)
        acc = (g**2).sum() / 8
        w = d["rows"][pos[k]].astype(np.float64) - 0.05 * g / (np.sqrt(acc) + 1e-8)
        want = torch.from_numpy(w.astype(np.float32)).to(torch.bfloat16).to(torch.float32).numpy()
        assert (rows[pos[k]] == want).all()
