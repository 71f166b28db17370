#!/usr/bin/env python3
"""Benchmark of the collisionless-table hot path on one MI355X.

A step = one pass of the whole path over one fresh synthetic batch:
lookup_or_insert -> gather_pool -> apply_grad_adagrad -> expire_sweep.
Default workload: configs[1] of the benchmark spec (capacity 2^24, dim 32 fp32, 65536 samples x 26 slots,
Poisson(3)+1 IDs per bag, Zipf(1.05) over 2^32, threshold 3) on a table that already holds the
workload's hottest IDs up to load 0.5, so that a step admits few new keys (the state after a long run).
Prints ONE JSON line; its `roofline` object is the WHOLE STEP against the HBM peak (compulsory bytes of
the step over the median step time), with the kernel that takes most time as `dominant_kernel`.

    python bench.py --gpus 1 --steps 10 --warmup 3
"""
import argparse
import json
import multiprocessing as mp
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2209_07663_amd import synth  # noqa: E402

# Load factor the table is brought to before the untimed steps.  configs[3] names 0.9, but from there the
# table reaches its fill limit before the first expiry (step 20) and every later batch is refused whole: a
# run from 0.9 measures refusals, so the default stops at 0.75 (--fill-load 0.9 still runs, and reports n_full).
DEFAULT_FILL = {"cfg2": 0.5, "cfg4": 0.75}
OTHER_WORKLOADS = ["cfg3", "cfg4", "cfg5", "qr"]   # reported beside the default workload, a few steps each

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E peak
SECTOR = 32             # bytes: smallest HBM access counted for a random 4/8-byte word
KEY_LINE = 64           # bytes of the eight keys of a bucket (what a probe must read of it)
BUCKET_LINE = 128       # bytes of a bucket as this library stores it (keys + row index / last-seen words)

# HBM bytes (read + written) that rocprofv3's FETCH_SIZE / WRITE_SIZE counters gave for ONE run of this
# script, scaled by the factors a plain 1 GiB copy gives; they are NOT measured by the run that prints
# them.  The figure is attached to a bench line only when workload and fill load are those of the
# profiled command, together with the name of the summary it comes from; otherwise `traffic` is null.
TRAFFIC_FROM_PROFILE = {
    "cfg2": {"profile": "profiles/bench_cfg2_full_step.md", "fill_load": 0.5,
             "step": 3713.1e6,
             "kernels": {"probe_count": 976.5e6, "seg_reduce": 1130.3e6, "gather_pool": 548.7e6,
                         "admit_elect": 280.6e6, "sort_scatter": 140.3e6, "sort_hist": 72.9e6, "insert": 87.7e6}},
}


def _workload(name):
    return synth.QR_WORKLOAD if name == "qr" else synth.CONFIGS[name]


def _gen(args):
    wl_name, seed, step, with_grad = args
    return synth.make_batch(_workload(wl_name), seed, step, with_grad=with_grad)


def generate_batches(wl_name, seed, steps, workers, with_grad=True):
    wl = _workload(wl_name)
    if wl.drift_frac > 0:  # the rotating rank->ID map is sequential state
        drift = synth.DriftMap(wl, seed)
        return [synth.make_batch(wl, seed, s, with_grad=with_grad, drift=drift) for s in steps]
    if workers <= 0:  # in-process (used under profilers, which have initialised the GPU already)
        return [_gen((wl_name, seed, s, with_grad)) for s in steps]
    with mp.get_context("fork").Pool(workers) as pool:
        return pool.map(_gen, [(wl_name, seed, s, with_grad) for s in steps], chunksize=1)


def cpu_baseline(wl, seed, fill_chunks, untimed, timed, budget_s):
    """The oracle as it stands (single thread) on the SAME batches the device is timed on: the fill and
    the untimed batches are replayed first (not timed), then full steps are timed until the budget is used."""
    from oracle import Oracle
    o = Oracle(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, kind="cuckoo")
    t_replay = time.perf_counter()
    for chunk in fill_chunks:
        for _ in range(max(wl.freq_threshold, 1)):
            o.lookup_or_insert(chunk, 0)

    def full_step(b):
        o.lookup_or_insert(b["keys"], b["step"])
        o.pool(b["keys"], b["offsets"])
        o.apply_grad_adagrad(b["keys"], b["offsets"], b["grad"], wl.lr, wl.eps)
        o.expire_sweep(b["step"])

    for b in untimed:
        full_step(b)
    t_replay = time.perf_counter() - t_replay
    ids, t0, used = 0, time.perf_counter(), 0
    for b in timed:
        full_step(b)
        ids += b["keys"].shape[0]
        used += 1
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    return {"value": ids / dt, "unit": "IDs/s", "cores": 1, "kind": "oracle",
            "sample": "full step (lookup_or_insert+pool+adagrad+sweep) on the first %d of the %d timed batches, after "
                      "the same fill and the same %d untimed batches as the device (replayed untimed in %.0f s); %.1f s"
                      % (used, len(timed), len(untimed), t_replay, dt),
            "host_cpus_present": os.cpu_count()}


def algorithmic_bytes(kernel, s, wl):
    """Compulsory bytes of ONE launch of `kernel` for a batch with statistics `s`: what the kernel must move
    if duplicates of a key were served on chip (n occurrences, u_* distinct keys, S = 32-byte sector).  Sort
    scratch and row-index arrays that only exist because of how the work is split into kernels are not counted:
    seg_reduce is charged the backward's compulsory bytes (pooled gradients once, every distinct row and its
    state read and written), not the sorted pairs it reads."""
    e = 2 if wl.bf16 else 4
    row = wl.dim * e
    n, nb = s["n"], s["n_bags"]
    if kernel == "probe_count":
        # keys in, row indices out, one bucket line and a 4-byte stamp per distinct stored key, the counter
        # sector of a distinct missing key read and written; where counters age a miss must also read both
        # of its bucket lines (with expire_steps == 0 a counter below the threshold proves absence)
        if wl.expire_steps == 0:
            return 12 * n + (BUCKET_LINE + 4) * s["u_hit"] + 2 * SECTOR * s["u_miss"]
        return 12 * n + (BUCKET_LINE + 4) * s["u_hit"] + (2 * BUCKET_LINE + 2 * SECTOR) * s["u_miss"]
    if kernel == "admit_elect":
        return 4 * n + 8 * s["n_miss"] + SECTOR * s["u_miss"] + 16 * s["u_new"]
    if kernel == "insert":
        return s["u_new"] * (row + BUCKET_LINE + 4 + 8 + 8 + 4)
    if kernel == "resolve":
        return 4 * n
    if kernel == "gather_pool":
        return 4 * n + 8 * (nb + 1) + row * s["u_present"] + 4 * wl.dim * nb
    if kernel == "seg_reduce":
        return 4 * wl.dim * nb + 2 * row * s["u_present"] + 8 * s["u_present"]
    if kernel == "sweep_find":
        return 4 * s.get("size", wl.capacity)   # the last-seen word of every STORED key (see step_bytes)
    return 0   # the sort kernels and combine move scratch only: no compulsory bytes


def step_bytes(s, wl, sweep_every, bucket_bytes=KEY_LINE):
    """Compulsory bytes of a whole step with perfect on-chip reuse of duplicates: keys, offsets, one bucket
    line per distinct stored key and two per distinct missing key (a miss must look at both buckets), the
    counter sector of a distinct missing key read and written, the stamp, every distinct row read once (and
    written once if new), the pooled output; backward: the pooled gradients, every distinct row read and
    written, its accumulator read and written; sweep: the last-seen word of every STORED key and the removed
    keys (4 bytes per slot of the whole table would be the figure for a sweep that cannot skip empty buckets;
    this library's can, so counting every slot would credit it with bytes it never has to move).
    bucket_bytes = 64: the eight keys of a bucket; 128: the bucket line as this library stores it."""
    e = 2 if wl.bf16 else 4
    row = wl.dim * e
    n, nb = s["n"], s["n_bags"]
    fwd = (8 * n + 8 * (nb + 1) + bucket_bytes * (s["u_hit"] + 2 * s["u_miss"]) + 2 * SECTOR * s["u_miss"]
           + 4 * s["u_present"] + row * s["u_present"] + row * s["u_new"] + 4 * wl.dim * nb)
    bwd = 4 * wl.dim * nb + 2 * row * s["u_present"] + 8 * s["u_present"]
    sweep = (4 * s.get("size", wl.capacity) / sweep_every + 8 * s.get("n_expired", 0)) if wl.expire_steps else 0
    return fwd + bwd + sweep


def time_maintenance(tab, wl, seed, max_ids, dev):
    """Wall time (host clock around calls that synchronise) of the operations around the hot path, on the
    table as the timed steps left it: delta export of the touched keys, full snapshot, restore of that
    snapshot into a fresh table, rehash into a table twice the size.  Bytes are the payloads moved."""
    import ctypes
    import torch
    from paper_2209_07663_amd.binding import Table, check as _check, device_pointer as _p, current_stream as _stream
    size = tab.mono_table_stats()["size"]
    keys = torch.empty(size, dtype=torch.int64, device=dev)
    row = torch.empty(size, dtype=torch.int32, device=dev)
    seen = torch.empty(size, dtype=torch.int32, device=dev)
    vals = torch.empty((size, wl.dim), dtype=torch.float32, device=dev)
    acc = torch.empty(size, dtype=torch.float32, device=dev)
    words = torch.empty(tab.n_filter, dtype=torch.int32, device=dev)
    got = ctypes.c_uint64()
    rec = 8 + 4 * wl.dim + 4 + 4                     # key, fp32 row, accumulator, last-seen / row index
    res = {}

    def timed(fn):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3

    ms = timed(lambda: _check(tab.lib.mono_export_touched(tab.h, _p(keys), _p(row), _p(vals), _p(acc), size,
                                                         ctypes.byref(got), _stream()), "mono_export_touched"))
    n = got.value
    res["export_touched"] = {"keys": n, "ms": round(ms, 3), "payload_GBps": round(n * rec / ms / 1e6, 1),
                             "window": "every update since the table was created"}
    ms = timed(lambda: (_check(tab.lib.mono_table_export(tab.h, _p(keys), _p(row), _p(seen), None, _p(vals), _p(acc),
                                                         size, ctypes.byref(got), _stream()), "mono_table_export"),
                        _check(tab.lib.mono_filter_export(tab.h, _p(words), 0, tab.n_filter, _stream()),
                               "mono_filter_export")))
    snap_bytes = size * rec + 4 * tab.n_filter
    res["snapshot"] = {"keys": size, "ms": round(ms, 3), "payload_GBps": round(snap_bytes / ms / 1e6, 1)}
    fresh = Table(wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, max_ids=max_ids,
                  max_bags=wl.n_bags, device=dev)

    def restore():
        for lo in range(0, size, max_ids):
            hi = min(size, lo + max_ids)
            _check(fresh.lib.mono_table_import(fresh.h, _p(keys[lo:hi]), _p(vals[lo:hi]), _p(acc[lo:hi]), _p(seen[lo:hi]),
                                               hi - lo, None, _stream()), "mono_table_import")
        fresh.mono_filter_import(words)
    ms = timed(restore)
    assert fresh.mono_table_stats()["size"] == size
    res["restore"] = {"keys": size, "ms": round(ms, 3), "payload_GBps": round(snap_bytes / ms / 1e6, 1),
                      "keys_per_s": round(size / ms * 1e3)}
    fresh.close()
    big = Table(2 * wl.capacity, wl.dim, seed, wl.freq_threshold, wl.expire_steps, wl.bf16, max_ids=max_ids,
                max_bags=wl.n_bags, device=dev)
    ms = timed(lambda: big.mono_table_migrate(tab, 1))
    st = big.mono_table_stats()
    assert st["size"] == size and st["stash_size"] == 0
    res["rehash_to_double_capacity"] = {"keys": size, "ms": round(ms, 3), "keys_per_s": round(size / ms * 1e3)}
    big.close()
    return res


def bench_quotient_remainder(args):
    """Second workload: the quotient-remainder embedding of the paper's hashing baseline (section 3.1) through
    the same pooling kernel: no table, no hashing, two dense tables of 2^24 rows.  A step = one pooled
    gather over a fresh batch of the cfg2 shape with IDs of a 2^48 space."""
    import torch
    from paper_2209_07663_amd.binding import mono_qr_gather_pool
    wl = synth.QR_WORKLOAD
    n_steps = args.warmup + args.steps
    batches = generate_batches("qr", args.seed, list(range(n_steps)), args.workers, with_grad=False)
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(args.seed)
    tabs = [torch.randn((1 << 24, wl.dim), generator=gen, device=dev, dtype=torch.float32) * 0.05 for _ in range(2)]
    cpu = None
    if args.cpu_budget > 0:
        from oracle import qr_pool
        host = [t.cpu().numpy() for t in tabs]
        ids, t0, used = 0, time.perf_counter(), 0
        for b in batches[args.warmup:]:
            qr_pool(host[0], host[1], b["keys"], b["offsets"])
            ids += b["keys"].shape[0]
            used += 1
            if time.perf_counter() - t0 > args.cpu_budget:
                break
        dt = time.perf_counter() - t0
        cpu = {"value": ids / dt, "unit": "IDs/s", "cores": 1, "kind": "oracle",
               "sample": "pooled two-table sum on the first %d of the timed batches, %.1f s" % (used, dt),
               "host_cpus_present": os.cpu_count()}
        del host
    dbat = [{"keys": torch.from_numpy(b["keys"]).to(dev), "offsets": torch.from_numpy(b["offsets"]).to(dev)}
            for b in batches]
    out = torch.empty((wl.n_bags, wl.dim), dtype=torch.float32, device=dev)
    for b in dbat[:args.warmup]:
        mono_qr_gather_pool(tabs[0], tabs[1], b["keys"], b["offsets"], out)
    timed = dbat[args.warmup:]
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in timed]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for b, (e0, e1) in zip(timed, ev):
        e0.record()
        mono_qr_gather_pool(tabs[0], tabs[1], b["keys"], b["offsets"], out)
        e1.record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ids = sum(b["keys"].shape[0] for b in timed)
    ms = [e0.elapsed_time(e1) for e0, e1 in ev]
    # compulsory bytes of a launch: IDs, offsets, every distinct row of either table once, the pooled output
    algo = []
    for b in timed:
        k = b["keys"]
        u = torch.unique(k & ((1 << 24) - 1)).numel() + torch.unique(k >> 24).numel()
        algo.append(8 * k.shape[0] + 8 * (wl.n_bags + 1) + 4 * wl.dim * u + 4 * wl.dim * wl.n_bags)
    achieved = float(np.mean(algo)) / (float(np.mean(ms)) * 1e-3) / 1e9
    print(json.dumps({
        "metric": "sparse IDs/sec per pooled gather (quotient-remainder embedding, no table)",
        "value": ids / elapsed, "unit": "IDs/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "qr: two dense tables of 2^24 rows, dim 32 fp32, E = E_r[ID mod 2^24] + E_q[ID div 2^24], "
                               "%d samples x %d slots, Zipf(%.2f) IDs over 2^48" % (wl.samples, wl.slots, wl.alpha),
                   "ids_per_step": ids // args.steps, "step": "qr_gather_pool"},
        "median_step_ms_events": float(np.median(ms)),
        "roofline": {"bound": "hbm", "kernel": "gather_pool (quotient-remainder rows)", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None},
        "cpu_baseline": cpu}))


def run_other_workloads(names, seed, workers):
    """Short runs of the other configurations, each in a child process of its own (its table is gone when it
    ends, and a failure there cannot take the headline figure with it): {name: summary of its JSON line}."""
    import subprocess
    out = {}
    for name in names:
        cmd = [sys.executable, os.path.join(ROOT, "bench.py"), "--workload", name, "--steps", "4", "--warmup", "1",
               "--prefill", "1", "--profile-steps", "1", "--cpu-budget", "0", "--no-maintenance", "--others", "none",
               "--seed", str(seed), "--workers", str(workers)]
        t0 = time.perf_counter()
        try:
            r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, timeout=240)
            line = [l for l in r.stdout.decode().splitlines() if l.startswith("{")]
            if r.returncode != 0 or not line:
                out[name] = {"error": "exit code %d: %s" % (r.returncode, r.stderr.decode()[-300:])}
                continue
            d = json.loads(line[-1])
            roof = d.get("roofline") or {}
            out[name] = {"value": d["value"], "unit": d["unit"], "ms_per_step": round(d["ms_per_step"], 4),
                         "steps": d["steps"], "dtype": d["dtype"], "config": d["config"],
                         "roofline_frac": roof.get("frac"), "roofline_achieved_GBps": roof.get("achieved"),
                         "dominant_kernel": (roof.get("dominant_kernel") or {}).get("kernel", roof.get("kernel")),
                         "table_events": d.get("table_events"), "wall_s": round(time.perf_counter() - t0, 1)}
        except subprocess.TimeoutExpired:
            out[name] = {"error": "no result within 240 s"}
        print("[bench] %s: %s" % (name, {k: out[name].get(k) for k in ("ms_per_step", "value", "error")}),
              file=sys.stderr, flush=True)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg2", choices=sorted(synth.CONFIGS) + ["qr"],
                    help="cfg1..cfg5: the table's training step; qr: the quotient-remainder embedding (pooled gather only)")
    ap.add_argument("--prefill", type=int, default=2, help="untimed steps before the warm-up steps")
    ap.add_argument("--profile-steps", type=int, default=4, help="extra steps run with per-kernel HIP events")
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--cpu-budget", type=float, default=12.0, help="seconds of oracle time; 0 = skip")
    ap.add_argument("--workers", type=int, default=min(16, os.cpu_count() or 8))
    ap.add_argument("--fill-load", type=float, default=-1.0,
                    help="before anything else, admit the workload's hottest IDs until this load factor; default: "
                         "0.5 for cfg2, 0.75 for cfg4 (configs[3] names 0.9: see DEFAULT_FILL), 0 (empty table) for the others")
    ap.add_argument("--no-maintenance", action="store_true",
                    help="skip the timing of delta export, snapshot, restore and rehash after the timed steps")
    ap.add_argument("--others", default="default",
                    help="comma-separated workloads to run for a few steps each after the main one and report in "
                         "`other_workloads`; 'none' = skip; default: cfg3,cfg4,cfg5,qr when the main workload is cfg2")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device copy five times (reference for FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.calibrate_copy:
        import torch
        a = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        b = torch.empty_like(a)
        for _ in range(5):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copied_bytes_per_launch": a.numel() * 4, "launches": 5}))
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives are part of it); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    if args.workload == "qr":
        return bench_quotient_remainder(args)
    wl = synth.CONFIGS[args.workload]
    # Default state of the table: the workload's hottest IDs are admitted first (untimed) up to a load at
    # which a step admits few new keys, as after a long run; --fill-load 0 starts from the empty table.
    fill_load = args.fill_load if args.fill_load >= 0 else DEFAULT_FILL.get(wl.name, 0.0)
    n_untimed = args.prefill + args.warmup
    n_steps = n_untimed + args.steps + args.profile_steps
    t_gen = time.perf_counter()
    batches = generate_batches(args.workload, args.seed, list(range(n_steps)), args.workers)
    t_gen = time.perf_counter() - t_gen
    print("[bench] generated %d batches of %s in %.1f s" % (n_steps, wl.name, t_gen), file=sys.stderr, flush=True)
    max_ids = max(b["keys"].shape[0] for b in batches)
    fill_chunks = []
    if fill_load > 0:
        drift = synth.DriftMap(wl, args.seed) if wl.drift_frac > 0 else None
        hot = synth.hottest_ids(wl, int(fill_load * wl.capacity), drift)
        fill_chunks = [hot[lo:lo + max_ids] for lo in range(0, hot.shape[0], max_ids)]

    cpu = None
    if args.cpu_budget > 0:
        cpu = cpu_baseline(wl, args.seed, fill_chunks, batches[:n_untimed], batches[n_untimed:n_untimed + args.steps],
                           args.cpu_budget)
        print("[bench] oracle: %.3g IDs/s" % cpu["value"], file=sys.stderr, flush=True)

    import torch
    from paper_2209_07663_amd.binding import Table
    dev = torch.device("cuda:0")
    tab = Table(wl.capacity, wl.dim, args.seed, wl.freq_threshold, wl.expire_steps, wl.bf16, max_ids=max_ids,
                max_bags=wl.n_bags, device=dev)
    dbatches = []
    for b in batches:  # inputs resident in HBM before anything is timed
        dbatches.append({"keys": torch.from_numpy(b["keys"]).to(dev), "offsets": torch.from_numpy(b["offsets"]).to(dev),
                         "grad": torch.from_numpy(b["grad"]).to(dev), "step": b["step"], "n": b["keys"].shape[0]})
    rows = torch.empty(max_ids, dtype=torch.int32, device=dev)
    pooled = torch.empty((wl.n_bags, wl.dim), dtype=torch.float32, device=dev)
    n_exp = torch.zeros(1, dtype=torch.int64, device=dev)

    # expiry sweep: every step (configs[3] asks for it; configs[4] leaves the cadence open, and a sweep of its
    # sparsely filled 2^28 slots costs a tenth of its step)
    sweep_every = 1

    def run_step(b):
        r = rows[: b["n"]]
        tab.mono_lookup_or_insert(b["keys"], b["step"], r)
        tab.mono_gather_pool(r, b["offsets"], pooled)
        tab.mono_apply_grad_adagrad(r, b["offsets"], b["grad"], wl.lr, wl.eps)
        if b["step"] % sweep_every == sweep_every - 1:
            tab.mono_expire_sweep(b["step"], n_exp, None)

    for chunk_h in fill_chunks:  # untimed: every hot ID is looked up often enough to pass the occurrence filter
        chunk = torch.from_numpy(chunk_h).to(dev)
        for _ in range(max(wl.freq_threshold, 1)):
            tab.mono_lookup_or_insert(chunk, 0, rows[: chunk.shape[0]])
    if fill_chunks:
        torch.cuda.synchronize()
        print("[bench] filled to load %.3f" % (tab.mono_table_stats()["size"] / wl.capacity), file=sys.stderr, flush=True)
    it = iter(dbatches)
    for _ in range(n_untimed):
        run_step(next(it))
    torch.cuda.synchronize()
    st0 = tab.mono_table_stats()
    load_before = st0["size"] / wl.capacity

    timed = [next(it) for _ in range(args.steps)]
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in timed]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for b, (e0, e1) in zip(timed, ev):
        e0.record()
        run_step(b)
        e1.record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ids = sum(b["n"] for b in timed)
    step_ms = [e0.elapsed_time(e1) for e0, e1 in ev]
    st = tab.mono_table_stats()
    admitted_per_step = (st["n_admitted"] - st0["n_admitted"]) / max(args.steps, 1)

    # per-kernel pass (HIP events inside the library, on the stream the kernels run on) + batch statistics
    stats, prof = [], {}
    tab.mono_profile_enable(True)
    for _ in range(args.profile_steps):
        b = next(it)
        adm0 = tab.mono_table_stats()["n_admitted"]
        r = rows[: b["n"]]
        tab.mono_lookup_or_insert(b["keys"], b["step"], r)
        torch.cuda.synchronize()
        u_all = torch.unique(b["keys"]).numel()
        present = r >= 0
        u_present = torch.unique(b["keys"][present]).numel()
        u_new = tab.mono_table_stats()["n_admitted"] - adm0
        # miss occurrences = occurrences of keys absent before the call: absent now, or admitted in this call
        u_hit = u_present - u_new
        one = {"n": b["n"], "n_bags": wl.n_bags, "u": u_all, "u_present": u_present, "u_new": u_new,
               "u_hit": u_hit, "u_miss": u_all - u_hit, "n_miss": int((~present).sum().item()), "n_expired": 0,
               "size": tab.mono_table_stats()["size"]}
        tab.mono_gather_pool(r, b["offsets"], pooled)
        tab.mono_apply_grad_adagrad(r, b["offsets"], b["grad"], wl.lr, wl.eps)
        if b["step"] % sweep_every == sweep_every - 1:
            tab.mono_expire_sweep(b["step"], n_exp, None)
            one["n_expired"] = int(n_exp.item()) / sweep_every
        stats.append(one)
    prof = tab.mono_profile_read()
    tab.mono_profile_enable(False)
    end = tab.mono_table_stats()

    roofline, kernels, mean = None, {}, None
    med_ms = float(np.median(step_ms))
    if stats:
        mean = {k: float(np.mean([x[k] for x in stats])) for k in stats[0]}
        tp = TRAFFIC_FROM_PROFILE.get(wl.name)
        tp = tp if tp and abs(tp["fill_load"] - fill_load) < 1e-9 else None
        sb, sb_line = step_bytes(mean, wl, sweep_every, KEY_LINE), step_bytes(mean, wl, sweep_every, BUCKET_LINE)
        roofline = {"bound": "hbm", "scope": "whole step: every kernel of lookup_or_insert + gather_pool + "
                                             "apply_grad_adagrad + expire_sweep, compulsory bytes of the step "
                                             "over the median step time (HIP events around each timed step)",
                    "achieved": round(sb / (med_ms * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(sb / (med_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                    "traffic": tp["step"] if tp else None, "traffic_source": tp["profile"] if tp else None,
                    "algorithmic_bytes_per_step": int(sb),
                    "frac_with_128_byte_bucket_lines": round(sb_line / (med_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                    "batch_stats": {k: int(v) for k, v in mean.items()}}
        for name, (ms, launches) in prof.items():
            avg_ms = ms / launches
            ab = algorithmic_bytes(name, mean, wl)
            kernels[name] = {"avg_ms": round(avg_ms, 4), "launches_per_step": launches / len(stats),
                             "ms_per_step": round(ms / len(stats), 4),
                             "algo_GBps": round(ab / avg_ms / 1e6, 1) if ab else None}
        if prof:
            dom = max(prof, key=lambda k: prof[k][0])
            achieved = algorithmic_bytes(dom, mean, wl) / (prof[dom][0] / prof[dom][1]) / 1e6
            roofline["dominant_kernel"] = {
                "kernel": dom, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "avg_launch_ms": round(prof[dom][0] / prof[dom][1], 4),
                "traffic": tp["kernels"].get(dom) if tp else None, "traffic_source": tp["profile"] if tp else None,
                "timing": "HIP events around every launch on the library's stream, over the %d steps that follow "
                          "the timed ones on the same stream of batches (with events in the timed steps the step "
                          "takes longer, so those run without)" % len(stats)}

    maintenance = None if args.no_maintenance else time_maintenance(tab, wl, args.seed, max_ids, dev)
    tab.close()
    del tab, dbatches, rows, pooled
    torch.cuda.empty_cache()
    names = (OTHER_WORKLOADS if wl.name == "cfg2" else []) if args.others == "default" else \
        [w for w in args.others.split(",") if w and w != "none"]
    others = run_other_workloads(names, args.seed, args.workers) if names else None

    out = {
        "metric": "sparse IDs/sec per training step (lookup+pool+update)",
        "value": ids / elapsed, "unit": "IDs/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.bf16 else "f32", "data": "synthetic",
        "config": {"workload": "%s: capacity 2^%d, dim %d, %d samples x %d slots, %s IDs, threshold %d, expire %d"
                               % (wl.name, wl.capacity.bit_length() - 1, wl.dim, wl.samples, wl.slots,
                                  "Zipf(%.2f)" % wl.alpha if wl.dist == "zipf" else "uniform", wl.freq_threshold,
                                  wl.expire_steps),
                   "ids_per_step": ids // args.steps, "fill_load": fill_load, "prefill_steps": args.prefill,
                   "load_factor": round(load_before, 4), "keys_admitted_per_step": round(admitted_per_step),
                   "sweep_every_steps": sweep_every,
                   "step": "lookup_or_insert+gather_pool+apply_grad_adagrad+expire_sweep"},
        "median_step_ms_events": med_ms, "min_step_ms_events": float(np.min(step_ms)),
        "table_events": {k: end[k] for k in ("n_insert_failed", "n_lost", "n_full", "stash_size", "max_chain")},
        "roofline": roofline, "kernels": kernels, "maintenance": maintenance, "cpu_baseline": cpu,
        "other_workloads": others,
    }
    print(json.dumps(out))
    if end["n_lost"]:
        print("bench.py: %d stored elements were lost (stash overflow)" % end["n_lost"], file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
