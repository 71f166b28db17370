"""False admissions of the occurrence filter against its memory, on the device library.

    python -m paper_2209_07663_amd.filter_study [--samples 16384] [--steps 8]

Stream: configs[1] shapes of the benchmark spec (26 slots, Poisson(3)+1 IDs per bag, Zipf(1.05) over 2^32,
threshold 3) at a reduced batch.  For every (hashes per key, number of counters) the script runs
the same batches through a fresh table and reports how many keys were admitted, how many of them
had NOT yet been seen `threshold` times (false admissions: keys that share counters with others),
and the time of lookup_or_insert per step.  A counting filter never refuses a key that has reached
the threshold, so the falsely admitted keys are exactly the surplus over the exact count.
"""
import argparse
import time

import numpy as np
import torch

from . import synth
from .binding import Table


def exact_admitted(batches, thr):
    """Number of distinct keys whose occurrences over the stream reach thr (nothing expires here)."""
    keys, counts = np.unique(np.concatenate(batches), return_counts=True)
    return int((counts >= thr).sum())


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--samples", type=int, default=16384)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--seed", type=int, default=1)
    args = ap.parse_args()
    dev = torch.device("cuda:0")
    capacity = 1 << 22
    wl = synth.scaled(synth.CONFIGS["cfg2"], samples=args.samples, capacity=capacity)
    batches = [synth.make_batch(wl, args.seed, s, with_grad=False)["keys"] for s in range(args.steps)]
    dkeys = [torch.from_numpy(b).to(dev) for b in batches]
    exact = exact_admitted(batches, wl.freq_threshold)
    distinct = np.unique(np.concatenate(batches)).shape[0]
    print("stream: %d steps x %d IDs, %d distinct keys, %d reach the threshold of %d"
          % (args.steps, batches[0].shape[0], distinct, exact, wl.freq_threshold))
    print("| hashes | counters | filter MiB | admitted | false admissions | false / admitted | lookup ms/step |")
    print("|---|---|---|---|---|---|---|")
    for log2 in (18, 20, 22, 24, 26):
        for hashes in (1, 2, 3, 4):
            tab = Table(capacity, wl.dim, args.seed, wl.freq_threshold, 0, False, max_ids=max(b.shape[0] for b in batches),
                        max_bags=wl.n_bags, device=dev, filter_hashes=hashes, filter_log2=log2)
            rows = torch.empty(tab.max_ids, dtype=torch.int32, device=dev)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for s, k in enumerate(dkeys):
                tab.mono_lookup_or_insert(k, s, rows[: k.shape[0]])
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / len(dkeys)
            st = tab.mono_table_stats()
            assert st["n_full"] == 0 and st["n_lost"] == 0 and st["n_admitted"] >= exact
            false = st["n_admitted"] - exact
            print("| %d | 2^%d | %.1f | %d | %d | %.4f | %.3f |" % (hashes, log2, (8 << log2) / 2 ** 20, st["n_admitted"], false,
                                                                 false / max(st["n_admitted"], 1), ms))
            tab.close()


if __name__ == "__main__":
    main()
