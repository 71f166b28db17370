"""The C-ABI library loads without a GPU and exports every symbol include/monotable.h declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "monotable.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mono_[a-z_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib_path():
    from paper_2209_07663_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2209_07663_amd.build import build_library
        build_library()
    return binding.LIB_PATH


def test_header_and_binding_name_the_same_entry_points():
    from paper_2209_07663_amd import binding
    assert declared_symbols() == sorted(binding.SYMBOLS)
    for required in ("mono_table_create", "mono_lookup_or_insert", "mono_gather_pool", "mono_apply_grad_adagrad",
                     "mono_expire_sweep"):
        assert required in binding.SYMBOLS


def test_library_exports_every_declared_symbol(lib_path):
    lib = ctypes.CDLL(lib_path)
    for name in declared_symbols():
        assert hasattr(lib, name), name


def test_size_query_validates_arguments_on_the_host(lib_path):
    from paper_2209_07663_amd import binding
    lib = binding.load_library()
    ok = lib.mono_table_bytes(1 << 16, 16, 0, 4096, 4096)
    rows = (1 << 16) * 16 * 4
    assert ok > rows                                   # rows + buckets + counters + workspace
    assert lib.mono_table_bytes(1 << 16, 16, 1, 4096, 4096) == ok - rows // 2   # bf16 rows are half
    assert lib.mono_table_bytes(1000, 16, 0, 4096, 4096) == 0                   # not a power of two
    assert lib.mono_table_bytes(1 << 16, 6, 0, 4096, 4096) == 0                 # dim not a multiple of 4
    assert lib.mono_table_bytes(1 << 16, 16, 2, 4096, 4096) == 0                # unknown storage flag
    assert lib.mono_table_bytes(1 << 16, 16, 0, 0, 0) == 0
    assert lib.mono_strerror(-1) == b"invalid argument"


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    from paper_2209_07663_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError):
        binding.load_library()
