"""Thin ctypes binding of include/monotable.h — argument marshalling only.

Every step of the path runs in the HIP kernels of `libmonotable.so`; torch is used for device
memory and for the current stream.  There is no fallback: if the library is missing, loading fails.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmonotable.so")

MONO_OK, MONO_EINVAL, MONO_ENOMEM, MONO_EHIP, MONO_ELIMIT = 0, -1, -2, -3, -4
MONO_ROWS_FP32, MONO_ROWS_BF16 = 0, 1

_u64, _u32, _vp, _f32 = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_float


class mono_stats(ctypes.Structure):
    _fields_ = [(n, _u64) for n in ("capacity", "size", "n_admitted", "n_expired", "n_insert_failed", "n_lost",
                                    "n_full", "stash_size", "max_chain")]


# every symbol include/monotable.h declares: name -> (restype, argtypes)
SYMBOLS = {
    "mono_table_bytes": (ctypes.c_size_t, [_u64, _u32, _u32, _u64, _u64]),
    "mono_table_create": (ctypes.c_int, [ctypes.POINTER(_vp), _u64, _u32, _u64, _u32, _u32, _u32, _u64, _u64, _vp,
                                         ctypes.c_size_t, _vp]),
    "mono_table_bytes_ex": (ctypes.c_size_t, [_u64, _u32, _u32, _u64, _u64, _u32]),
    "mono_table_create_ex": (ctypes.c_int, [ctypes.POINTER(_vp), _u64, _u32, _u64, _u32, _u32, _u32, _u64, _u64, _u32,
                                            _u32, _vp, ctypes.c_size_t, _vp]),
    "mono_table_destroy": (ctypes.c_int, [_vp]),
    "mono_lookup_or_insert": (ctypes.c_int, [_vp, _vp, _u64, _u32, _vp, _vp]),
    "mono_gather_pool": (ctypes.c_int, [_vp, _vp, _u64, _vp, _u64, _vp, _vp]),
    "mono_qr_gather_pool": (ctypes.c_int, [_vp, _vp, _u32, _u32, _u32, _vp, _u64, _vp, _u64, _vp, _vp]),
    "mono_apply_grad_adagrad": (ctypes.c_int, [_vp, _vp, _u64, _vp, _u64, _vp, _f32, _f32, _vp]),
    "mono_apply_grad_adagrad_noalloc": (ctypes.c_int, [_vp, _vp, _u64, _vp, _u64, _vp, _f32, _f32, _vp]),
    "mono_noalloc_max_ids": (_u64, []),
    "mono_expire_sweep": (ctypes.c_int, [_vp, _u32, _vp, _vp, _u64, _vp]),
    "mono_table_stats": (ctypes.c_int, [_vp, ctypes.POINTER(mono_stats), _vp]),
    "mono_table_export": (ctypes.c_int, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _u64, ctypes.POINTER(_u64), _vp]),
    "mono_export_touched": (ctypes.c_int, [_vp, _vp, _vp, _vp, _vp, _u64, ctypes.POINTER(_u64), _vp]),
    "mono_table_import": (ctypes.c_int, [_vp, _vp, _vp, _vp, _vp, _u64, ctypes.POINTER(_u64), _vp]),
    "mono_filter_import": (ctypes.c_int, [_vp, _vp, _u64, _u64, _vp]),
    "mono_table_migrate": (ctypes.c_int, [_vp, _vp, _u32, _vp]),
    "mono_filter_export": (ctypes.c_int, [_vp, _vp, _u64, _u64, _vp]),
    "mono_profile_enable": (ctypes.c_int, [_vp, ctypes.c_int]),
    "mono_profile_read": (ctypes.c_int, [_vp, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_double),
                                         ctypes.POINTER(_u64), _u32, ctypes.POINTER(_u32)]),
    "mono_strerror": (ctypes.c_char_p, [ctypes.c_int]),
}

_lib = None


def load_library():
    """Loads libmonotable.so (built in-tree by `paper_2209_07663_amd.build`); raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libmonotable.so is not built: run `python -m paper_2209_07663_amd.build` "
                               "(there is no CPU fallback)")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


class MonoError(RuntimeError):
    pass


def _check(rc, what):
    if rc != MONO_OK:
        raise MonoError("%s: %s (%d)" % (what, load_library().mono_strerror(rc).decode(), rc))


def _stream(device=None):
    """torch's current stream on `device` (default: the current device), as a hipStream_t."""
    return torch.cuda.current_stream(device).cuda_stream


def _p(t):
    return None if t is None else t.data_ptr()


# the same helpers under public names, for callers that pass their own buffers straight to the library
check, device_pointer, current_stream = _check, _p, _stream


def _dev(t, dtype):
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError("need a contiguous CUDA tensor of %s" % dtype)


def mono_qr_gather_pool(table_r, table_q, ids, offsets, out=None):
    """Pooled embeddings E_r[id mod 2^m] + E_q[id div 2^m] from two dense tables [2^m, dim] (fp32 or bf16)."""
    if table_r.shape != table_q.shape or table_r.dtype != table_q.dtype or table_r.dim() != 2:
        raise ValueError("the two tables must have the same shape [2^m, dim] and type")
    if table_r.dtype not in (torch.float32, torch.bfloat16):
        raise TypeError("tables must be float32 or bfloat16")
    _dev(table_r, table_r.dtype), _dev(table_q, table_q.dtype), _dev(ids, torch.int64), _dev(offsets, torch.int64)
    rows, dim = table_r.shape
    if rows & (rows - 1):
        raise ValueError("the tables must hold a power-of-two number of rows")
    n_bags = offsets.shape[0] - 1
    if out is None:
        out = torch.empty((n_bags, dim), dtype=torch.float32, device=ids.device)
    _dev(out, torch.float32)
    flags = MONO_ROWS_BF16 if table_r.dtype == torch.bfloat16 else MONO_ROWS_FP32
    _check(load_library().mono_qr_gather_pool(_p(table_r), _p(table_q), rows.bit_length() - 1, dim, flags, _p(ids),
                                              ids.shape[0], _p(offsets), n_bags, _p(out), _stream(ids.device)),
           "mono_qr_gather_pool")
    return out


class Table:
    """One collisionless embedding table on the current device.  Methods carry the C-ABI names."""

    def __init__(self, capacity, dim, seed, freq_threshold=1, expire_steps=0, bf16=False, max_ids=1 << 20,
                 max_bags=None, device="cuda:0", filter_hashes=1, filter_log2=0):
        self.lib = load_library()
        self.capacity, self.dim, self.bf16 = int(capacity), int(dim), bool(bf16)
        self.seed, self.freq_threshold, self.expire_steps = int(seed), int(freq_threshold), int(expire_steps)
        self.max_ids = int(max_ids)
        self.max_bags = int(max_bags) if max_bags is not None else self.max_ids
        self.device = torch.device(device)
        flags = MONO_ROWS_BF16 if bf16 else MONO_ROWS_FP32
        self.filter_hashes, self.filter_log2 = int(filter_hashes), int(filter_log2)
        self.n_filter = (1 << self.filter_log2) if self.filter_log2 else 4 * self.capacity
        nbytes = self.lib.mono_table_bytes_ex(self.capacity, self.dim, flags, self.max_ids, self.max_bags,
                                              self.filter_log2)
        if nbytes == 0:
            raise MonoError("mono_table_bytes: invalid table shape")
        self.arena = torch.empty(nbytes, dtype=torch.uint8, device=self.device)  # torch owns the memory
        h = _vp()
        with torch.cuda.device(self.device):
            _check(self.lib.mono_table_create_ex(ctypes.byref(h), self.capacity, self.dim, seed, freq_threshold,
                                                 expire_steps, flags, self.max_ids, self.max_bags,
                                                 self.filter_hashes, self.filter_log2, self.arena.data_ptr(), nbytes,
                                                 _stream(self.device)), "mono_table_create_ex")
        self.h = h

    def _s(self):
        return _stream(self.device)

    def close(self):
        if getattr(self, "h", None):
            self.lib.mono_table_destroy(self.h)
            self.h = None
            self.arena = None

    def __del__(self):
        self.close()

    def mono_lookup_or_insert(self, keys, step, rows_out=None):
        _dev(keys, torch.int64)
        if rows_out is None:
            rows_out = torch.empty(keys.shape[0], dtype=torch.int32, device=keys.device)
        _dev(rows_out, torch.int32)
        _check(self.lib.mono_lookup_or_insert(self.h, _p(keys), keys.shape[0], step, _p(rows_out), self._s()),
               "mono_lookup_or_insert")
        return rows_out

    def mono_gather_pool(self, rows, offsets, out=None):
        _dev(rows, torch.int32)
        _dev(offsets, torch.int64)
        n_bags = offsets.shape[0] - 1
        if out is None:
            out = torch.empty((n_bags, self.dim), dtype=torch.float32, device=rows.device)
        _dev(out, torch.float32)
        _check(self.lib.mono_gather_pool(self.h, _p(rows), rows.shape[0], _p(offsets), n_bags, _p(out), self._s()),
               "mono_gather_pool")
        return out

    def mono_apply_grad_adagrad(self, rows, offsets, grad, lr, eps):
        _dev(rows, torch.int32)
        _dev(offsets, torch.int64)
        _dev(grad, torch.float32)
        n_bags = offsets.shape[0] - 1
        if grad.numel() != n_bags * self.dim:
            raise ValueError("grad must hold n_bags * dim elements")
        _check(self.lib.mono_apply_grad_adagrad(self.h, _p(rows), rows.shape[0], _p(offsets), n_bags, _p(grad), lr,
                                                eps, self._s()), "mono_apply_grad_adagrad")

    def mono_apply_grad_adagrad_noalloc(self, rows, offsets, grad, lr, eps):
        """The update through the library's fixed workspace (at most mono_noalloc_max_ids() IDs per call)."""
        _dev(rows, torch.int32)
        _dev(offsets, torch.int64)
        _dev(grad, torch.float32)
        n_bags = offsets.shape[0] - 1
        if grad.numel() != n_bags * self.dim:
            raise ValueError("grad must hold n_bags * dim elements")
        with torch.cuda.device(self.device):
            _check(self.lib.mono_apply_grad_adagrad_noalloc(self.h, _p(rows), rows.shape[0], _p(offsets), n_bags,
                                                            _p(grad), lr, eps, self._s()),
                   "mono_apply_grad_adagrad_noalloc")

    def mono_expire_sweep(self, now, n_expired=None, expired_keys=None):
        max_expired = 0
        if expired_keys is not None:
            _dev(expired_keys, torch.int64)
            max_expired = expired_keys.shape[0]
        if n_expired is not None:
            _dev(n_expired, torch.int64)
        _check(self.lib.mono_expire_sweep(self.h, now, _p(n_expired), _p(expired_keys), max_expired, self._s()),
               "mono_expire_sweep")

    def mono_table_stats(self):
        st = mono_stats()
        _check(self.lib.mono_table_stats(self.h, ctypes.byref(st), self._s()), "mono_table_stats")
        return {n: int(getattr(st, n)) for n, _ in mono_stats._fields_}

    def mono_table_export(self, with_values=True):
        """Dump as host numpy arrays sorted by key (as uint64): keys, row, last_seen, slot, rows, acc."""
        n = self.mono_table_stats()["size"]
        dev = self.device
        keys = torch.empty(n, dtype=torch.int64, device=dev)
        row = torch.empty(n, dtype=torch.int32, device=dev)
        seen = torch.empty(n, dtype=torch.int32, device=dev)
        slot = torch.empty(n, dtype=torch.int64, device=dev)
        vals = torch.empty((n, self.dim), dtype=torch.float32, device=dev) if with_values else None
        acc = torch.empty(n, dtype=torch.float32, device=dev) if with_values else None
        got = _u64()
        _check(self.lib.mono_table_export(self.h, _p(keys), _p(row), _p(seen), _p(slot), _p(vals), _p(acc), n,
                                          ctypes.byref(got), self._s()), "mono_table_export")
        if got.value != n:
            raise MonoError("mono_table_export: %d keys stored but %d rows in use" % (got.value, n))
        k = keys.cpu().numpy()
        order = k.view("uint64").argsort(kind="stable")
        d = {"keys": k[order], "row": row.cpu().numpy()[order], "last_seen": seen.cpu().numpy().view("uint32")[order],
             "slot": slot.cpu().numpy()[order]}
        if with_values:
            d["rows"] = vals.cpu().numpy()[order]
            d["acc"] = acc.cpu().numpy()[order]
        return d

    def mono_export_touched(self, max_n=None, with_values=True):
        """Keys trained since the last synchronisation, as host numpy arrays sorted by key: keys, row, rows, acc.
        With max_n below the number of touched keys nothing is taken: returns {"n": count} only."""
        max_n = self.mono_table_stats()["size"] if max_n is None else max_n
        dev = self.device
        keys = torch.empty(max_n, dtype=torch.int64, device=dev)
        row = torch.empty(max_n, dtype=torch.int32, device=dev)
        vals = torch.empty((max_n, self.dim), dtype=torch.float32, device=dev) if with_values else None
        acc = torch.empty(max_n, dtype=torch.float32, device=dev) if with_values else None
        got = _u64()
        _check(self.lib.mono_export_touched(self.h, _p(keys), _p(row), _p(vals), _p(acc), max_n, ctypes.byref(got),
                                            self._s()), "mono_export_touched")
        n = got.value
        if n > max_n:
            return {"n": n}
        k = keys[:n].cpu().numpy()
        order = k.view("uint64").argsort(kind="stable")
        d = {"n": n, "keys": k[order], "row": row[:n].cpu().numpy()[order]}
        if with_values:
            d["rows"] = vals[:n].cpu().numpy()[order]
            d["acc"] = acc[:n].cpu().numpy()[order]
        return d

    def mono_table_import(self, keys, values, acc, last_seen):
        """Restores snapshot records (device tensors: int64, fp32 [n, dim], fp32, int32 holding uint32 steps),
        max_ids at a time; returns how many were refused."""
        _dev(keys, torch.int64), _dev(values, torch.float32), _dev(acc, torch.float32), _dev(last_seen, torch.int32)
        n, refused = keys.shape[0], 0
        if values.shape != (n, self.dim) or acc.shape[0] != n or last_seen.shape[0] != n:
            raise ValueError("values [n, dim], acc [n] and last_seen [n] must match the n keys")
        for lo in range(0, n, self.max_ids):
            hi = min(n, lo + self.max_ids)
            r = _u64()
            _check(self.lib.mono_table_import(self.h, _p(keys[lo:hi]), _p(values[lo:hi]), _p(acc[lo:hi]),
                                              _p(last_seen[lo:hi]), hi - lo, ctypes.byref(r), self._s()),
                   "mono_table_import")
            refused += r.value
        return refused

    def mono_filter_import(self, words, first=0):
        _dev(words, torch.int32)
        _check(self.lib.mono_filter_import(self.h, _p(words), first, words.shape[0], self._s()), "mono_filter_import")

    def mono_table_migrate(self, src, generation):
        """Fills this (fresh) table with everything `src` holds, under the hash functions of `generation`."""
        _check(self.lib.mono_table_migrate(self.h, src.h, generation, self._s()), "mono_table_migrate")

    def rehashed(self, new_capacity, generation):
        """A new table of `new_capacity` >= capacity holding this table's contents (this one stays as it is)."""
        grown = self.n_filter * (new_capacity // self.capacity)          # the counters grow with the table
        dst = Table(new_capacity, self.dim, self.seed, self.freq_threshold, self.expire_steps, self.bf16,
                    max_ids=self.max_ids, max_bags=self.max_bags, device=self.device,
                    filter_hashes=self.filter_hashes, filter_log2=grown.bit_length() - 1)
        dst.mono_table_migrate(self, generation)
        return dst

    def mono_profile_enable(self, on):
        _check(self.lib.mono_profile_enable(self.h, int(on)), "mono_profile_enable")

    def mono_profile_read(self):
        """{kernel name: (total ms, launches)} since the last read."""
        cap = 32
        names, ms, cnt, n = (ctypes.c_char_p * cap)(), (ctypes.c_double * cap)(), (_u64 * cap)(), _u32()
        _check(self.lib.mono_profile_read(self.h, names, ms, cnt, cap, ctypes.byref(n)), "mono_profile_read")
        return {names[i].decode(): (ms[i], int(cnt[i])) for i in range(n.value)}

    def mono_filter_export(self, first=0, count=None):
        count = self.n_filter - first if count is None else count
        words = torch.empty(count, dtype=torch.int32, device=self.device)
        _check(self.lib.mono_filter_export(self.h, _p(words), first, count, self._s()), "mono_filter_export")
        return words.cpu().numpy().view("uint32")
