"""The byte accounting of bench.py on hand-computed cases (CPU only): the roofline fractions it
prints are only as good as these formulas."""
import importlib.util
import os

from paper_2209_07663_amd import synth

_spec = importlib.util.spec_from_file_location("bench", os.path.join(os.path.dirname(__file__), "..", "bench.py"))
bench = importlib.util.module_from_spec(_spec)
_spec.loader.exec_module(bench)

STATS = {"n": 1000, "n_bags": 250, "u": 400, "u_present": 150, "u_new": 50, "u_hit": 100, "u_miss": 300, "n_miss": 600}


def test_kernel_bytes_no_expiry_fp32_dim32():
    wl = synth.CONFIGS["cfg2"]                       # dim 32 fp32 -> 128-byte rows, nothing ages
    S = 32
    b = lambda k: bench.algorithmic_bytes(k, STATS, wl)
    assert b("probe_count") == 12 * 1000 + (128 + 4) * 100 + 2 * S * 300
    assert b("admit_elect") == 4 * 1000 + 8 * 600 + S * 300 + 16 * 50
    assert b("insert") == 50 * (128 + 128 + 24)
    assert b("resolve") == 4 * 1000
    assert b("gather_pool") == 4 * 1000 + 8 * 251 + 128 * 150 + 4 * 32 * 250
    assert b("expand_bags") == 8 * 251 + 4 * 1000
    assert b("sort_hist") == 4 * 1000 and b("sort_scatter") == 16 * 1000
    assert b("seg_reduce") == 8 * 1000 + 4 * 32 * 250 + 2 * 128 * 150 + 8 * 150
    assert b("combine") == 0


def test_kernel_bytes_with_expiry_bf16_dim64():
    wl = synth.CONFIGS["cfg5"]                       # dim 64 bf16 -> 128-byte rows, counters age
    S = 32
    assert bench.algorithmic_bytes("probe_count", STATS, wl) == 12 * 1000 + (128 + 4) * 100 + (256 + 2 * S) * 300
    assert bench.algorithmic_bytes("sweep_find", STATS, wl) == 8 * wl.capacity
    assert bench.algorithmic_bytes("seg_reduce", STATS, wl) == 8 * 1000 + 4 * 64 * 250 + 2 * 128 * 150 + 8 * 150


def test_step_bytes():
    S = 32
    wl = synth.CONFIGS["cfg2"]
    fwd = 8 * 1000 + 8 * 251 + 128 * (100 + 300) + 2 * S * 300 + 4 * 150 + 128 * 150 + 128 * 50 + 4 * 32 * 250
    bwd = 4 * 32 * 250 + 2 * 128 * 150 + 8 * 150
    assert bench.step_bytes(STATS, wl, 1) == fwd + bwd                       # no sweep share without expiry
    wl5 = synth.CONFIGS["cfg5"]
    fwd5 = 8 * 1000 + 8 * 251 + 128 * 400 + 2 * S * 300 + 4 * 150 + 128 * 150 + 128 * 50 + 4 * 64 * 250
    bwd5 = 4 * 64 * 250 + 2 * 128 * 150 + 8 * 150
    assert bench.step_bytes(STATS, wl5, 10) == fwd5 + bwd5 + 8 * wl5.capacity / 10
