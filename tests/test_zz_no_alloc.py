"""The allocation-free variant of the update (its workspace is a fixed array inside the library) against the
ordinary entry point and against the oracle, through the C ABI: two calls in a row, the second with a
smaller batch, so that whatever the first call left in the shared array is seen to do no harm."""
import numpy as np
import pytest
import torch

from oracle import Oracle
from paper_2209_07663_amd import synth
from tests import table_checks as tc

pytestmark = pytest.mark.gpu


def _tables(wl, seed, dev):
    from paper_2209_07663_amd.binding import Table
    mk = lambda: Table(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, max_ids=1 << 18,
                       max_bags=wl.n_bags, device=dev)
    return mk(), mk(), Oracle(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, kind="cuckoo")


@pytest.mark.parametrize("name,dim", [("cfg3", 64), ("cfg5", 64), ("cfg3", 1024)])
def test_noalloc_update_equals_the_ordinary_one_on_two_calls_in_a_row(name, dim):
    from dataclasses import replace
    dev = torch.device("cuda:0")
    seed = 61
    big = replace(synth.scaled(synth.CONFIGS[name], samples=4096 if dim <= 64 else 512, capacity=1 << 18), dim=dim,
                  slots=8)
    small = replace(big, samples=big.samples // 8)                  # the second call: an eighth of the first
    rtol = 1e-2 if big.bf16 else 1e-5
    plain, fixed, orc = _tables(big, seed, dev)
    for step, wl in enumerate([big, small]):
        b = synth.make_batch(wl, seed, step, with_grad=True)
        keys, offs = torch.from_numpy(b["keys"]).to(dev), torch.from_numpy(b["offsets"]).to(dev)
        grad = torch.from_numpy(b["grad"]).to(dev)
        assert keys.shape[0] <= plain.lib.mono_noalloc_max_ids()
        r_plain, r_fixed = plain.mono_lookup_or_insert(keys, step), fixed.mono_lookup_or_insert(keys, step)
        orc.lookup_or_insert(b["keys"], step)
        plain.mono_apply_grad_adagrad(r_plain, offs, grad, wl.lr, wl.eps)
        fixed.mono_apply_grad_adagrad_noalloc(r_fixed, offs, grad, wl.lr, wl.eps)
        orc.apply_grad_adagrad(b["keys"], b["offsets"], b["grad"], wl.lr, wl.eps)
        d_plain, d_fixed = plain.mono_table_export(), fixed.mono_table_export()
        assert d_fixed["keys"].shape[0] > 100
        tc.assert_same_table(d_fixed, d_plain, exact_rows=False, rtol=rtol)      # the existing entry point
        tc.assert_same_table(d_fixed, orc.dump(), exact_rows=False, rtol=rtol)   # and the oracle
        assert (d_fixed["acc"] > 0).sum() == (d_plain["acc"] > 0).sum() > 0
    # the keys trained through either entry point are marked touched alike
    assert (fixed.mono_export_touched(with_values=False)["keys"] == orc.take_touched()).all()
    plain.close()
    fixed.close()


def test_noalloc_update_refuses_a_batch_beyond_its_fixed_workspace():
    from paper_2209_07663_amd.binding import Table, MonoError, MONO_ELIMIT
    dev = torch.device("cuda:0")
    tab = Table(1 << 12, 4, 5, max_ids=1 << 19, max_bags=1 << 19, device=dev)
    limit = tab.lib.mono_noalloc_max_ids()
    assert limit == 1 << 18
    n = limit + 1
    rows = torch.zeros(n, dtype=torch.int32, device=dev)
    offs = torch.arange(n + 1, dtype=torch.int64, device=dev)
    grad = torch.zeros((n, 4), dtype=torch.float32, device=dev)
    with pytest.raises(MonoError) as err:
        tab.mono_apply_grad_adagrad_noalloc(rows, offs, grad, 0.1, 1e-8)
    assert "(%d)" % MONO_ELIMIT in str(err.value) and "fixed workspace" in str(err.value)
    # exactly the limit is accepted: every occurrence names row 0 (in use after the lookup), all gradients are zero
    tab.mono_lookup_or_insert(torch.arange(10, dtype=torch.int64, device=dev), 0)
    tab.mono_apply_grad_adagrad_noalloc(rows[:limit], offs[:limit + 1], grad[:limit], 0.1, 1e-8)
    torch.cuda.synchronize()
    tab.close()
