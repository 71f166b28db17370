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
