"""Checks that work on any table dump (the oracle's or the device library's).

The hash functions are written here a third time, in numpy, from the build's written contract
(SplitMix64 output function; salt i = (i+1)-th SplitMix64 output for the table seed; bucket =
top bits), so that the placement invariant of section 2.1 of the paper (every stored element is in
T0[h0(x)] or T1[h1(x)]) is checked by code that shares nothing with either implementation.
"""
import numpy as np

U64 = np.uint64
GOLDEN = U64(0x9E3779B97F4A7C15)


def mix64(z):
    z = np.asarray(z, dtype=U64)
    with np.errstate(over="ignore"):
        z = z ^ (z >> U64(30))
        z = z * U64(0xBF58476D1CE4E5B9)
        z = z ^ (z >> U64(27))
        z = z * U64(0x94D049BB133111EB)
        z = z ^ (z >> U64(31))
    return z


def salt(seed, i):
    with np.errstate(over="ignore"):
        return mix64(U64(seed) + U64(i + 1) * GOLDEN)


def top_bits(h, lg):
    if lg == 0:
        return np.zeros_like(h)
    return h >> U64(64 - lg)


PLACEMENT_STEP = U64(0xD1B54A32D192ED03)


def placement_seed(seed, generation):
    """Seed of the h0 / h1 salts after `generation` rehashes (generation 0: the table as created)."""
    with np.errstate(over="ignore"):
        return U64(seed) + U64(generation) * PLACEMENT_STEP


def bucket_of(side, keys, capacity, bucket, seed, generation=0):
    n_buckets = capacity // 2 // bucket
    lg = int(n_buckets).bit_length() - 1
    keys = np.asarray(keys).astype(U64)
    return top_bits(mix64(keys ^ salt(placement_seed(seed, generation), side)), lg)


def filter_index(keys, n_filter, seed, j=0):
    """Counter j of each key: salt 2 for the first hash, salts 8, 9, 10 for the others."""
    lg = int(n_filter).bit_length() - 1
    keys = np.asarray(keys).astype(U64)
    return top_bits(mix64(keys ^ salt(seed, 2 if j == 0 else 7 + j)), lg)


def init_rows(keys, dim, seed):
    """Initial rows in exact integer arithmetic (value = (u24 - 2^23) * 2^-27)."""
    keys = np.asarray(keys).astype(U64)
    base = mix64(keys ^ salt(seed, 3))
    out = np.empty((keys.shape[0], dim), dtype=np.float64)
    with np.errstate(over="ignore"):
        for j in range(dim):
            u24 = (mix64(base + U64(j)) >> U64(40)).astype(np.int64)
            out[:, j] = (u24 - (1 << 23)) / float(1 << 27)
    return out


def check_placement(dump, capacity, bucket, seed, generation=0):
    """I1 (placement) and I2 (no key twice, no slot twice) on a dump with global slot indices.

    Global slot = side * capacity/2 + bucket_index * bucket + lane; negative slots (stash) are
    exempt from I1 and must not occur in graded runs (the caller asserts that).
    """
    keys, slot = dump["keys"], dump["slot"]
    assert np.unique(keys).shape[0] == keys.shape[0], "a key is stored twice"
    placed = slot >= 0
    s = slot[placed]
    assert np.unique(s).shape[0] == s.shape[0], "two keys share a slot"
    assert (s < capacity).all()
    half = capacity // 2
    side = (s >= half).astype(np.int64)
    bidx = (s - side * half) // bucket
    k = keys[placed]
    for sd in (0, 1):
        m = side == sd
        want = bucket_of(sd, k[m], capacity, bucket, seed, generation).astype(np.int64)
        assert (bidx[m] == want).all(), "a key sits outside its h%d bucket" % sd
    if "row" in dump:
        r = dump["row"]
        assert np.unique(r).shape[0] == r.shape[0], "two keys share an embedding row"
        assert ((r >= 0) & (r < capacity)).all()


def rows_close(got, ref, rtol):
    """Per row: ||got - ref||_inf <= rtol * max(||ref||_inf, tiny).  Returns the worst ratio."""
    if ref.shape[0] == 0:
        assert np.asarray(got).size == 0
        return 0.0
    got = np.asarray(got, dtype=np.float64).reshape(ref.shape[0], -1)
    ref = np.asarray(ref, dtype=np.float64).reshape(ref.shape[0], -1)
    scale = np.maximum(np.abs(ref).max(axis=1), 1e-30)
    err = np.abs(got - ref).max(axis=1) / scale
    worst = float(err.max())
    assert worst <= rtol, "row error %.3e exceeds %.1e (row %d)" % (worst, rtol, int(err.argmax()))
    return worst


def assert_same_table(got, ref, exact_rows, rtol=1e-5):
    """got / ref: dumps sorted by key.  Keys and last_seen bit-exact; rows bit-exact when no
    optimizer step has touched them (`exact_rows`), else within rtol; accumulators within rtol."""
    assert got["keys"].shape == ref["keys"].shape, "admitted sets differ in size: %d vs %d" % (
        got["keys"].shape[0], ref["keys"].shape[0])
    assert (got["keys"] == ref["keys"]).all(), "admitted key sets differ"
    assert (got["last_seen"] == ref["last_seen"]).all(), "last_seen differs"
    if exact_rows:
        assert (got["rows"].view(np.uint32) == ref["rows"].view(np.uint32)).all(), "rows differ bitwise"
        assert (got["acc"].view(np.uint32) == ref["acc"].view(np.uint32)).all(), "accumulators differ bitwise"
    else:
        rows_close(got["rows"], ref["rows"], rtol)
        if ref["acc"].shape[0]:
            a, b = got["acc"].astype(np.float64), ref["acc"].astype(np.float64)
            assert (np.abs(a - b) <= rtol * np.maximum(np.abs(b), 1e-30)).all(), "accumulators differ"
