"""The quotient-remainder embedding of the paper's hashing baseline (section 3.1) on the device against
the oracle's plain two-index sum, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

from oracle import qr_pool
from paper_2209_07663_amd import synth
from tests import table_checks as tc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "gpu tests need a GPU"
    return torch.device("cuda:0")


def _tables(rng, m, dim, bf16, dev):
    """Two dense tables as the oracle sees them (fp32 values) and as the device stores them."""
    host, devs = [], []
    for _ in range(2):
        t = torch.from_numpy(rng.standard_normal((1 << m, dim), dtype=np.float32) * 0.05)
        if bf16:
            d = t.to(torch.bfloat16)
            host.append(d.to(torch.float32).numpy())
            devs.append(d.to(dev))
        else:
            host.append(t.numpy())
            devs.append(t.to(dev))
    return host, devs


@pytest.mark.parametrize("dim,bf16,lam", [(4, False, 3.0), (32, False, 3.0), (64, True, 0.0), (100, False, 1.0),
                                          (256, True, 9.0), (512, False, 3.0), (1024, False, 0.5)])
def test_pooled_decomposed_embeddings_match_the_oracle(dev, dim, bf16, lam):
    from paper_2209_07663_amd.binding import mono_qr_gather_pool
    rng = np.random.default_rng(dim)
    m, n_bags = 10, 3000 + dim                          # several waves of bags and a ragged tail
    host, devs = _tables(rng, m, dim, bf16, dev)
    lens = rng.poisson(lam, size=n_bags).astype(np.int64) + (1 if lam == 0.0 else 0)   # empty bags too
    lens[17] = 40                                       # one bag far longer than the indices kept in registers
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    ids = rng.integers(0, 1 << (2 * m), size=int(offs[-1]), dtype=np.int64)
    ids[rng.random(ids.shape[0]) < 0.03] = -1           # padding
    ids[rng.random(ids.shape[0]) < 0.01] = 1 << (2 * m)  # just outside the decomposed space
    got = mono_qr_gather_pool(devs[0], devs[1], torch.from_numpy(ids).to(dev), torch.from_numpy(offs).to(dev))
    want = qr_pool(host[0], host[1], ids, offs)
    tc.rows_close(got.cpu().numpy()[lens > 0], want[lens > 0], 1e-5)
    assert (got.cpu().numpy()[lens == 0] == 0).all()


def test_empty_and_invalid_arguments(dev):
    from paper_2209_07663_amd.binding import mono_qr_gather_pool, MonoError
    t = torch.zeros((16, 8), device=dev)
    ids = torch.empty(0, dtype=torch.int64, device=dev)
    out = mono_qr_gather_pool(t, t, ids, torch.zeros(5, dtype=torch.int64, device=dev))
    assert out.shape == (4, 8) and bool((out == 0).all().item())
    assert mono_qr_gather_pool(t, t, ids, torch.zeros(1, dtype=torch.int64, device=dev)).shape == (0, 8)
    with pytest.raises(ValueError):
        mono_qr_gather_pool(torch.zeros((12, 8), device=dev), torch.zeros((12, 8), device=dev), ids,
                            torch.zeros(2, dtype=torch.int64, device=dev))
    with pytest.raises(MonoError):                       # dim 6 is not a multiple of 4
        mono_qr_gather_pool(torch.zeros((16, 6), device=dev), torch.zeros((16, 6), device=dev), ids,
                            torch.zeros(2, dtype=torch.int64, device=dev))


@pytest.mark.timeout(600)
def test_full_size_two_tables_of_2_to_24_rows(dev):
    """The paper's sizes: IDs of a 2^48 space, two tables of 2^24 rows, with the batch shape of configs[1]
    (65536 samples x 26 slots, Poisson(3)+1 IDs per bag, Zipf IDs), in the launch configuration bench.py times."""
    from paper_2209_07663_amd.binding import mono_qr_gather_pool
    wl = synth.QR_WORKLOAD
    rng = np.random.default_rng(5)
    host, devs = _tables(rng, 24, wl.dim, False, dev)
    b = synth.make_batch(wl, 1, 0)
    assert int(b["keys"].max()) >> 24 > 1000             # the quotient table is really used
    got = mono_qr_gather_pool(devs[0], devs[1], torch.from_numpy(b["keys"]).to(dev),
                              torch.from_numpy(b["offsets"]).to(dev)).cpu().numpy()
    want = qr_pool(host[0], host[1], b["keys"], b["offsets"])
    print("full size: %d IDs in %d bags" % (b["keys"].shape[0], wl.n_bags), flush=True)
    tc.rows_close(got, want, 1e-5)
