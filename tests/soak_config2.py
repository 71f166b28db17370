"""Long full-size run of configs[1] on the device against the oracle (not collected by pytest: it takes
about five minutes, most of it the oracle).  Every step: same presence on both sides, no failed chain;
every eighth step and at the end: whole table equal (keys, last-seen, rows and accumulators within 1e-5),
placement valid, counter words equal.  51 steps take the table from empty to load 0.94.

    python tests/soak_config2.py [steps]
"""
import sys, os, time
sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import numpy as np, torch
from oracle import Oracle
from paper_2209_07663_amd import synth
from paper_2209_07663_amd.binding import Table
from tests import table_checks as tc
wl, seed = synth.CONFIGS["cfg2"], 7
dev = torch.device("cuda:0")
tab = Table(wl.capacity, wl.dim, seed, wl.freq_threshold, 0, False, max_ids=8_000_000, max_bags=wl.n_bags, device=dev)
orc = Oracle(wl.capacity, wl.dim, seed, wl.freq_threshold, 0, False, kind="cuckoo")
steps = int(sys.argv[1]) if len(sys.argv) > 1 else 51
t0 = time.time()
for step in range(steps):
    b = synth.make_batch(wl, seed, step, with_grad=True)
    keys, offs = torch.from_numpy(b["keys"]).to(dev), torch.from_numpy(b["offsets"]).to(dev)
    rows = tab.mono_lookup_or_insert(keys, step)
    present = orc.lookup_or_insert(b["keys"], step)
    assert ((rows.cpu().numpy() >= 0) == present).all(), "presence differs at step %d" % step
    tab.mono_apply_grad_adagrad(rows, offs, torch.from_numpy(b["grad"]).to(dev), wl.lr, wl.eps)
    orc.apply_grad_adagrad(b["keys"], b["offsets"], b["grad"], wl.lr, wl.eps)
    st = tab.mono_table_stats()
    assert st["n_insert_failed"] == 0 and st["n_lost"] == 0 and st["n_full"] == 0
    if step % 8 == 7 or step == steps - 1:
        d = tab.mono_table_export()
        tc.check_placement(d, wl.capacity, 8, seed)
        tc.assert_same_table(d, orc.dump(), exact_rows=False, rtol=1e-5)
        assert (tab.mono_filter_export() == orc.filter_words()).all()
    print("step %d load %.3f max_chain %d  %.0f s" % (step, st["size"] / wl.capacity, st["max_chain"], time.time() - t0), flush=True)
print("soak ok")
