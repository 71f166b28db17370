"""Pins of the oracle's quotient-remainder pooling (the hashing baseline of the paper's section 3.1,
production-model item: ID_r = ID mod 2^24, ID_q = ID div 2^24, E = E_r + E_q) against things other than
itself: torch's embedding_bag on the two tables, the decomposition's arithmetic in Python integers, and
the sizes the paper states.  CPU only."""
import numpy as np
import torch

from oracle import qr_pool


def _bags(rng, n_bags, lam):
    lens = rng.poisson(lam, size=n_bags).astype(np.int64)
    return np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)


def test_equals_two_embedding_bags():
    rng = np.random.default_rng(0)
    m, dim = 6, 12
    e_r = rng.standard_normal((1 << m, dim)).astype(np.float32)
    e_q = rng.standard_normal((1 << m, dim)).astype(np.float32)
    offs = _bags(rng, 300, 3.0)                          # empty bags included
    ids = rng.integers(0, 1 << (2 * m), size=int(offs[-1]), dtype=np.int64)
    got = qr_pool(e_r, e_q, ids, offs)
    t_ids, t_offs = torch.from_numpy(ids), torch.from_numpy(offs[:-1])
    bag = torch.nn.functional.embedding_bag
    want = (bag(t_ids % (1 << m), torch.from_numpy(e_r).double(), t_offs, mode="sum")
            + bag(t_ids // (1 << m), torch.from_numpy(e_q).double(), t_offs, mode="sum"))
    assert np.allclose(got, want.numpy(), rtol=1e-6, atol=1e-6)
    assert (got[np.diff(offs) == 0] == 0).all()


def test_remainder_and_quotient_are_not_swapped():
    """One ID per bag, tables that hold their own row number: the output names the two rows used."""
    m = 5
    rows = np.arange(1 << m, dtype=np.float32)
    e_r = np.stack([rows, np.zeros_like(rows)], axis=1)   # column 0: remainder row
    e_q = np.stack([np.zeros_like(rows), rows], axis=1)   # column 1: quotient row
    ids = np.array([0, 1, 31, 32, 33, 1023, 700], dtype=np.int64)
    out = qr_pool(e_r, e_q, ids, np.arange(ids.shape[0] + 1, dtype=np.int64))
    assert out[:, 0].tolist() == [int(i) % 32 for i in ids]
    assert out[:, 1].tolist() == [int(i) // 32 for i in ids]


def test_every_id_of_the_space_gets_its_own_pair_and_the_sizes_are_the_papers():
    """The decomposition is a bijection between [0, 2^(2m)) and the pairs (ID_r, ID_q): every ID has a
    combination of its own.  With m = 24 the 2^48 IDs of section 3.1 need 2 * 2^24 = 2^25 rows."""
    m = 24
    rng = np.random.default_rng(1)
    ids = rng.integers(0, 1 << 48, size=10000, dtype=np.int64)
    r, q = ids % (1 << m), ids // (1 << m)
    assert (q < (1 << m)).all() and ((q << m) + r == ids).all()
    assert np.unique(np.stack([r, q], axis=1), axis=0).shape[0] == np.unique(ids).shape[0]
    assert 2 * (1 << m) == 1 << 25 and (1 << m) ** 2 == 1 << 48
    # the same on a space small enough to enumerate
    small = np.arange(1 << 8, dtype=np.int64)
    pairs = set(zip((small % 16).tolist(), (small // 16).tolist()))
    assert len(pairs) == 256


def test_ids_outside_the_space_contribute_nothing():
    m, dim = 4, 4
    e_r = np.ones((1 << m, dim), dtype=np.float32)
    e_q = np.ones((1 << m, dim), dtype=np.float32) * 10
    ids = np.array([3, -1, 1 << 8, (1 << 8) - 1, -(1 << 40)], dtype=np.int64)
    out = qr_pool(e_r, e_q, ids, np.array([0, 2, 3, 5], dtype=np.int64))
    assert (out[0] == 11).all() and (out[1] == 0).all() and (out[2] == 11).all()
