"""Long full-size run of the streaming configuration (frequency filter, expiry, drifting IDs) on the
device against the oracle (not collected by pytest: about four minutes, most of it the oracle).  The
table starts at load 0.75 with the hottest IDs; every step: same presence on both sides, same set of
expired keys, no failed chain, nothing refused; every eighth step and at the end: whole table equal
(keys, last-seen, rows and accumulators within 1e-5), placement valid, counter words equal.  24 steps
take the load to 0.84 and then through the first expiry (18.6 M keys leave at step 20).  A start above
load 0.9 would reach the library's fill limit (31/32 of the rows) before that expiry; the oracle has no
such limit, so from there on the two differ by design and the run is of no use as a comparison.

    python tests/soak_config4.py [steps]
"""
import sys, os, time
sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import numpy as np, torch
from oracle import Oracle
from paper_2209_07663_amd import synth
from paper_2209_07663_amd.binding import Table
from tests import table_checks as tc
wl, seed = synth.CONFIGS["cfg4"], 11
dev = torch.device("cuda:0")
steps = int(sys.argv[1]) if len(sys.argv) > 1 else 24
drift = synth.DriftMap(wl, seed)
hot = synth.hottest_ids(wl, int(0.75 * wl.capacity), drift)
max_ids = 1 << 23
tab = Table(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, False, max_ids=max_ids, max_bags=wl.n_bags, device=dev)
orc = Oracle(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, False, kind="cuckoo")
t0 = time.time()
rows = torch.empty(max_ids, dtype=torch.int32, device=dev)
for lo in range(0, hot.shape[0], max_ids):
    chunk = hot[lo:lo + max_ids]
    dchunk = torch.from_numpy(chunk).to(dev)
    for rep in range(wl.freq_threshold):
        tab.mono_lookup_or_insert(dchunk, 0, rows[:chunk.shape[0]])
        present = orc.lookup_or_insert(chunk, 0)
    assert ((rows[:chunk.shape[0]].cpu().numpy() >= 0) == present).all()
    print("filled chunk at %d  %.0f s" % (lo, time.time() - t0), flush=True)
n_exp = torch.zeros(1, dtype=torch.int64, device=dev)
out = torch.zeros(wl.capacity, dtype=torch.int64, device=dev)
for step in range(1, steps + 1):
    b = synth.make_batch(wl, seed, step, with_grad=True, drift=drift)
    keys, offs = torch.from_numpy(b["keys"]).to(dev), torch.from_numpy(b["offsets"]).to(dev)
    r = tab.mono_lookup_or_insert(keys, step)
    present = orc.lookup_or_insert(b["keys"], step)
    assert ((r.cpu().numpy() >= 0) == present).all(), "presence differs at step %d" % step
    tab.mono_apply_grad_adagrad(r, offs, torch.from_numpy(b["grad"]).to(dev), wl.lr, wl.eps)
    orc.apply_grad_adagrad(b["keys"], b["offsets"], b["grad"], wl.lr, wl.eps)
    tab.mono_expire_sweep(step, n_exp, out)
    want = orc.expire_sweep(step)
    n = int(n_exp.item())
    assert n == want.shape[0], "expired counts differ at step %d: %d vs %d" % (step, n, want.shape[0])
    if n:
        got = np.sort(out[:n].cpu().numpy().view(np.uint64)).view(np.int64)
        assert (got == want).all(), "expired sets differ at step %d" % step
    st = tab.mono_table_stats()
    assert st["n_insert_failed"] == 0 and st["n_lost"] == 0 and st["n_full"] == 0
    if step % 8 == 0 or step == steps:
        d = tab.mono_table_export()
        tc.check_placement(d, wl.capacity, 8, seed)
        tc.assert_same_table(d, orc.dump(), exact_rows=False, rtol=1e-5)
        assert (tab.mono_filter_export() == orc.filter_words()).all()
    print("step %d load %.3f expired %d max_chain %d  %.0f s" % (step, st["size"] / wl.capacity, n, st["max_chain"], time.time() - t0), flush=True)
print("soak ok")
