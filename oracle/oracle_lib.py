"""ctypes front end of the CPU oracle (test infrastructure only; see monolith_oracle.cpp).

`Oracle(kind="cuckoo")` is the sequential cuckoo hashmap of the paper's section 2.1 with the
admission filter and expiry of the same section; `Oracle(kind="map")` is the std::map definition
it is checked against.  Both take the same seeded inputs as the device library.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "monolith_oracle.cpp")
_LIB = os.path.join(_HERE, "libmonolith_oracle.so")

_u64, _u32, _i64p = ctypes.c_uint64, ctypes.c_uint32, ctypes.POINTER(ctypes.c_int64)
_vp, _f32 = ctypes.c_void_p, ctypes.c_float


def build_oracle(force=False):
    """Compile the oracle with g++ -O2 (no tuning flags: it is a baseline, not a product)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", _SRC, "-o", tmp])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def oracle_lib():
    global _lib
    if _lib is None:
        # MONOLITH_ORACLE_LIB: a library built elsewhere from (a variant of) the same source; the
        # test-suite uses it to check that the pins notice mistakes planted in the oracle
        lib = ctypes.CDLL(os.environ.get("MONOLITH_ORACLE_LIB") or build_oracle())
        lib.orc_create.restype = _vp
        lib.orc_create.argtypes = [ctypes.c_int, _u64, _u32, _u64, _u32, _u32, ctypes.c_int, _u64, _u32, _u32,
                                   ctypes.c_int, _u32]
        lib.orc_destroy.argtypes = [_vp]
        lib.orc_lookup_or_insert.argtypes = [_vp, _vp, _u64, _u32, _vp]
        lib.orc_pool.argtypes = [_vp, _vp, _vp, _u64, _vp]
        lib.orc_apply_grad_adagrad.argtypes = [_vp, _vp, _vp, _u64, _vp, _f32, _f32]
        lib.orc_expire_sweep.restype = _u64
        lib.orc_expire_sweep.argtypes = [_vp, _u32]
        lib.orc_erased_keys.argtypes = [_vp, _vp]
        lib.orc_dump.restype = _u64
        lib.orc_dump.argtypes = [_vp]
        lib.orc_dump_read.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp]
        lib.orc_filter_read.argtypes = [_vp, _u64, _u64, _vp]
        lib.orc_filter_index.restype = _u64
        lib.orc_filter_index.argtypes = [_vp, ctypes.c_int64]
        lib.orc_filter_index_j.restype = _u64
        lib.orc_filter_index_j.argtypes = [_vp, ctypes.c_int64, _u32]
        lib.orc_insert_failures.restype = _u64
        lib.orc_insert_failures.argtypes = [_vp]
        lib.orc_refused_full.restype = _u64
        lib.orc_refused_full.argtypes = [_vp]
        lib.orc_max_chain.restype = _u64
        lib.orc_max_chain.argtypes = [_vp]
        lib.orc_take_touched.restype = _u64
        lib.orc_take_touched.argtypes = [_vp]
        lib.orc_touched_keys.argtypes = [_vp, _vp]
        lib.orc_import.restype = _u64
        lib.orc_import.argtypes = [_vp, _vp, _vp, _vp, _vp, _u64]
        lib.orc_filter_write.argtypes = [_vp, _u64, _u64, _vp]
        lib.orc_rehash.restype = ctypes.c_int
        lib.orc_rehash.argtypes = [_vp, _u64, _u32]
        lib.orc_capacity.restype = _u64
        lib.orc_capacity.argtypes = [_vp]
        lib.orc_n_filter.restype = _u64
        lib.orc_n_filter.argtypes = [_vp]
        lib.orc_placement_salt.restype = _u64
        lib.orc_placement_salt.argtypes = [_u64, _u32, ctypes.c_int]
        lib.orc_qr_pool.argtypes = [_vp, _vp, _u32, _u32, _vp, _vp, _u64, _vp]
        lib.orc_mix64.restype = _u64
        lib.orc_mix64.argtypes = [_u64]
        lib.orc_salt.restype = _u64
        lib.orc_salt.argtypes = [_u64, ctypes.c_int]
        lib.orc_init_value.restype = _f32
        lib.orc_init_value.argtypes = [_u64, ctypes.c_int64, _u32]
        lib.orc_bf16_round.restype = _f32
        lib.orc_bf16_round.argtypes = [_f32]
        lib.orc_filter_touch.restype = _u32
        lib.orc_filter_touch.argtypes = [_u32, _u32, _u32]
        _lib = lib
    return _lib


def _ptr(a):
    return a.ctypes.data_as(_vp)


def qr_pool(table_r, table_q, ids, offsets):
    """Quotient-remainder embedding of the paper's hashing baseline, sum-pooled per bag: tables [2^m, dim] fp32."""
    table_r = np.ascontiguousarray(table_r, dtype=np.float32)
    table_q = np.ascontiguousarray(table_q, dtype=np.float32)
    ids = np.ascontiguousarray(ids, dtype=np.int64)
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    rows, dim = table_r.shape
    assert table_q.shape == table_r.shape and rows & (rows - 1) == 0
    out = np.empty((offsets.shape[0] - 1, dim), dtype=np.float32)
    oracle_lib().orc_qr_pool(_ptr(table_r), _ptr(table_q), rows.bit_length() - 1, dim, _ptr(ids), _ptr(offsets),
                             offsets.shape[0] - 1, _ptr(out))
    return out


class Oracle:
    """One table.  Arrays are numpy, C-contiguous; keys int64, offsets int64, grads float32."""

    def __init__(self, capacity, dim, seed, freq_threshold=1, expire_steps=0, bf16=False, kind="cuckoo",
                 n_filter=None, bucket=8, max_kicks=512, hash_mode=0, filter_hashes=1):
        self.lib = oracle_lib()
        self.capacity, self.dim = int(capacity), int(dim)
        self.n_filter = int(n_filter) if n_filter is not None else 4 * self.capacity
        self.h = self.lib.orc_create({"map": 0, "cuckoo": 1}[kind], self.capacity, self.dim, seed, freq_threshold,
                                     expire_steps, int(bf16), self.n_filter, bucket, max_kicks, hash_mode,
                                     filter_hashes)
        if not self.h:
            raise ValueError("oracle: bad table parameters")

    def __del__(self):
        if getattr(self, "h", None):
            self.lib.orc_destroy(self.h)
            self.h = None

    def lookup_or_insert(self, keys, step):
        keys = np.ascontiguousarray(keys, dtype=np.int64)
        present = np.empty(keys.shape[0], dtype=np.uint8)
        self.lib.orc_lookup_or_insert(self.h, _ptr(keys), keys.shape[0], step, _ptr(present))
        return present.astype(bool)

    def pool(self, keys, offsets):
        keys = np.ascontiguousarray(keys, dtype=np.int64)
        offsets = np.ascontiguousarray(offsets, dtype=np.int64)
        n_bags = offsets.shape[0] - 1
        out = np.empty((n_bags, self.dim), dtype=np.float32)
        self.lib.orc_pool(self.h, _ptr(keys), _ptr(offsets), n_bags, _ptr(out))
        return out

    def apply_grad_adagrad(self, keys, offsets, grad, lr, eps):
        keys = np.ascontiguousarray(keys, dtype=np.int64)
        offsets = np.ascontiguousarray(offsets, dtype=np.int64)
        grad = np.ascontiguousarray(grad, dtype=np.float32)
        n_bags = offsets.shape[0] - 1
        assert grad.shape == (n_bags, self.dim)
        self.lib.orc_apply_grad_adagrad(self.h, _ptr(keys), _ptr(offsets), n_bags, _ptr(grad), lr, eps)

    def expire_sweep(self, now):
        n = self.lib.orc_expire_sweep(self.h, now)
        out = np.empty(n, dtype=np.int64)
        if n:
            self.lib.orc_erased_keys(self.h, _ptr(out))
        return out

    def dump(self):
        """Table contents sorted by key (as uint64): keys, rows[n, dim] fp32, acc, last_seen, slot."""
        n = self.lib.orc_dump(self.h)
        keys = np.empty(n, dtype=np.int64)
        rows = np.empty((n, self.dim), dtype=np.float32)
        acc = np.empty(n, dtype=np.float32)
        last_seen = np.empty(n, dtype=np.uint32)
        slot = np.empty(n, dtype=np.int64)
        if n:
            self.lib.orc_dump_read(self.h, _ptr(keys), _ptr(rows), _ptr(acc), _ptr(last_seen), _ptr(slot))
        return {"keys": keys, "rows": rows, "acc": acc, "last_seen": last_seen, "slot": slot}

    def filter_words(self, first=0, count=None):
        count = self.n_filter - first if count is None else count
        out = np.empty(count, dtype=np.uint32)
        self.lib.orc_filter_read(self.h, first, count, _ptr(out))
        return out

    def filter_index(self, key, j=0):
        return self.lib.orc_filter_index_j(self.h, int(key), j)

    # -- maintenance operations --------------------------------------------------------------

    def take_touched(self):
        """Keys trained since the last call (ascending, as uint64 order); clears the set."""
        n = self.lib.orc_take_touched(self.h)
        out = np.empty(n, dtype=np.int64)
        if n:
            self.lib.orc_touched_keys(self.h, _ptr(out))
        return out

    def import_entries(self, keys, rows, acc, last_seen):
        """Restore records in the order given; returns how many were not placed."""
        keys = np.ascontiguousarray(keys, dtype=np.int64)
        rows = np.ascontiguousarray(rows, dtype=np.float32).reshape(keys.shape[0], self.dim)
        acc = np.ascontiguousarray(acc, dtype=np.float32)
        last_seen = np.ascontiguousarray(last_seen, dtype=np.uint32)
        return self.lib.orc_import(self.h, _ptr(keys), _ptr(rows), _ptr(acc), _ptr(last_seen), keys.shape[0])

    def write_filter_words(self, words, first=0):
        words = np.ascontiguousarray(words, dtype=np.uint32)
        self.lib.orc_filter_write(self.h, first, words.shape[0], _ptr(words))

    def rehash(self, new_capacity, generation):
        if self.lib.orc_rehash(self.h, int(new_capacity), int(generation)) != 0:
            raise ValueError("oracle: bad rehash parameters")
        self.capacity = int(self.lib.orc_capacity(self.h))
        self.n_filter = int(self.lib.orc_n_filter(self.h))

    @property
    def insert_failures(self):
        return self.lib.orc_insert_failures(self.h)

    @property
    def refused_full(self):
        """Admissible keys (or restore records) refused because their call would have taken the table past
        its fill limit of capacity - capacity/32 keys."""
        return self.lib.orc_refused_full(self.h)

    @property
    def max_chain(self):
        return self.lib.orc_max_chain(self.h)
