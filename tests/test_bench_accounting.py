"""The byte accounting of bench.py on hand-computed cases (CPU only): the roofline fractions it
prints are only as good as these formulas."""
import importlib.util
import os

from paper_2209_07663_amd import synth

_spec = importlib.util.spec_from_file_location("bench", os.path.join(os.path.dirname(__file__), "..", "bench.py"))
bench = importlib.util.module_from_spec(_spec)
_spec.loader.exec_module(bench)

STATS = {"n": 1000, "n_bags": 250, "u": 400, "u_present": 150, "u_new": 50, "u_hit": 100, "u_miss": 300, "n_miss": 600,
         "n_expired": 7, "size": 9000}


def test_kernel_bytes_no_expiry_fp32_dim32():
    wl = synth.CONFIGS["cfg2"]                       # dim 32 fp32 -> 128-byte rows, nothing ages
    S = 32
    b = lambda k: bench.algorithmic_bytes(k, STATS, wl)
    assert b("probe_count") == 12 * 1000 + (128 + 4) * 100 + 2 * S * 300
    assert b("admit_elect") == 4 * 1000 + 8 * 600 + S * 300 + 16 * 50
    assert b("insert") == 50 * (128 + 128 + 24)
    assert b("resolve") == 4 * 1000
    assert b("gather_pool") == 4 * 1000 + 8 * 251 + 128 * 150 + 4 * 32 * 250
    # the backward's compulsory bytes only: the sorted (row, bag) pairs it reads are scratch
    assert b("seg_reduce") == 4 * 32 * 250 + 2 * 128 * 150 + 8 * 150
    # kernels that only move scratch have no compulsory bytes
    assert b("expand_bags") == 0 and b("sort_hist") == 0 and b("sort_scatter") == 0 and b("combine") == 0


def test_kernel_bytes_with_expiry_bf16_dim64():
    wl = synth.CONFIGS["cfg5"]                       # dim 64 bf16 -> 128-byte rows, counters age
    S = 32
    assert bench.algorithmic_bytes("probe_count", STATS, wl) == 12 * 1000 + (128 + 4) * 100 + (256 + 2 * S) * 300
    assert bench.algorithmic_bytes("sweep_find", STATS, wl) == 4 * 9000          # per STORED key, not per slot
    assert bench.algorithmic_bytes("seg_reduce", STATS, wl) == 4 * 64 * 250 + 2 * 128 * 150 + 8 * 150


def test_step_bytes():
    """Whole step: keys, offsets, L bytes of bucket per distinct stored key and 2 L per distinct missing key,
    the counter sector of a missing key read and written, stamp, distinct rows, new rows, pooled output;
    backward: pooled gradients, distinct rows read and written, their state; sweep: 4 bytes per stored key
    per sweep plus 8 per removed key."""
    S = 32
    wl = synth.CONFIGS["cfg2"]
    for L in (64, 128):
        fwd = (8 * 1000 + 8 * 251 + L * (100 + 2 * 300) + 2 * S * 300 + 4 * 150 + 128 * 150 + 128 * 50
               + 4 * 32 * 250)
        bwd = 4 * 32 * 250 + 2 * 128 * 150 + 8 * 150
        assert bench.step_bytes(STATS, wl, 1, L) == fwd + bwd                # no sweep share without expiry
    assert bench.step_bytes(STATS, wl, 1) == bench.step_bytes(STATS, wl, 1, 64)  # the headline counts 64-byte key lines
    wl5 = synth.CONFIGS["cfg5"]
    fwd5 = 8 * 1000 + 8 * 251 + 64 * 700 + 2 * S * 300 + 4 * 150 + 128 * 150 + 128 * 50 + 4 * 64 * 250
    bwd5 = 4 * 64 * 250 + 2 * 128 * 150 + 8 * 150
    assert bench.step_bytes(STATS, wl5, 10) == fwd5 + bwd5 + 4 * 9000 / 10 + 8 * 7


def test_profile_traffic_is_labelled():
    """Counter figures copied from a profile carry the name of that profile and the fill load they hold for."""
    for name, rec in bench.TRAFFIC_FROM_PROFILE.items():
        assert name in synth.CONFIGS
        assert os.path.exists(os.path.join(os.path.dirname(__file__), "..", rec["profile"]))
        assert "fill_load" in rec and rec["step"] > 0 and rec["kernels"]
