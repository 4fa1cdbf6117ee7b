"""ctypes front end of the CPU oracle (argument marshalling only; see plora_oracle.cpp)."""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "plora_oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

ELT_BYTES = {0: 2, 1: 2, 2: 4}
STATUS = {0: "OK", -1: "INVAL", -2: "NOMEM", -3: "EXISTS", -4: "NOTFOUND"}


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__("oracle status %s" % STATUS.get(code, code))
        self.code = code


def build(force=True):
    """Compile the oracle with g++ (-O2, no FMA contraction, OpenMP for the timed leg)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-o", _LIB, _SRC]
    subprocess.check_call(cmd)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB):
        build()
    L = C.CDLL(_LIB)
    vp, i32, u32, u64, f32 = C.c_void_p, C.c_int32, C.c_uint32, C.c_uint64, C.c_float
    L.oracle_pool_create.argtypes = [u64, u32, i32, vp, vp, i32, i32, i32, C.POINTER(vp)]
    L.oracle_pool_destroy.argtypes = [vp]
    L.oracle_adapter_bytes.argtypes = [vp, i32]
    L.oracle_adapter_bytes.restype = u64
    L.oracle_load.argtypes = [vp, i32, i32, f32, vp, vp, C.POINTER(u32)]
    L.oracle_evict.argtypes = [vp, i32]
    L.oracle_page_table.argtypes = [vp, i32, vp, u32, C.POINTER(u32)]
    L.oracle_compact.argtypes = [vp, u32, vp, i32, vp]
    L.oracle_stats.argtypes = [vp, vp]
    L.oracle_free_map.argtypes = [vp, vp]
    L.oracle_read_virtual.argtypes = [vp, i32, u64, u64, vp]
    L.oracle_translate.argtypes = [vp, vp, i32, vp, vp, vp, C.POINTER(i32), C.POINTER(i32)]
    L.oracle_shrink.argtypes = [vp, i32, vp, vp, i32, vp, i32, i32, i32, vp]
    L.oracle_expand.argtypes = [vp, i32, vp, vp, i32, vp, i32, i32, i32, vp]
    L.oracle_decode_elt.argtypes = [i32, u32]
    L.oracle_decode_elt.restype = f32
    L.oracle_encode_elt.argtypes = [i32, f32]
    L.oracle_encode_elt.restype = u32
    L.oracle_max_threads.restype = i32
    _lib = L
    return L


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def decode_elt(dtype, bits):
    return _load().oracle_decode_elt(dtype, int(bits))


def encode_elt(dtype, value):
    return _load().oracle_encode_elt(dtype, float(value))


def max_threads():
    return _load().oracle_max_threads()


class OraclePool:
    """The oracle's own host pool: first-fit pages, page tables, paged shrink / expand."""

    def __init__(self, page_bytes, n_pages, d_in, d_out, dtype, max_adapters, max_rank):
        L = _load()
        self._L = L
        self.d_in = np.ascontiguousarray(d_in, dtype=np.int32)
        self.d_out = np.ascontiguousarray(d_out, dtype=np.int32)
        self.n_slots = len(self.d_in)
        self.dtype, self.max_adapters, self.max_rank = dtype, max_adapters, max_rank
        self.page_bytes, self.n_pages = page_bytes, n_pages
        self.elt = ELT_BYTES[dtype]
        h = C.c_void_p()
        rc = L.oracle_pool_create(page_bytes, n_pages, self.n_slots, _ptr(self.d_in), _ptr(self.d_out),
                                  dtype, max_adapters, max_rank, C.byref(h))
        if rc:
            raise OracleError(rc)
        self._h = h

    def close(self):
        if self._h:
            self._L.oracle_pool_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def adapter_bytes(self, rank):
        return self._L.oracle_adapter_bytes(self._h, rank)

    def load(self, aid, rank, scale, blob):
        """Returns the page table (int32 array). Raises OracleError on failure."""
        blob = np.ascontiguousarray(blob)
        need = self.adapter_bytes(rank) if 1 <= rank <= self.max_rank else 0
        if blob.nbytes < need:
            raise ValueError("blob shorter than the adapter")
        cap = (need + self.page_bytes - 1) // self.page_bytes
        pt = np.empty(max(cap, 1), dtype=np.int32)
        n = C.c_uint32(0)
        rc = self._L.oracle_load(self._h, aid, rank, scale, _ptr(blob), _ptr(pt), C.byref(n))
        if rc:
            raise OracleError(rc)
        return pt[: n.value].copy()

    def evict(self, aid):
        rc = self._L.oracle_evict(self._h, aid)
        if rc:
            raise OracleError(rc)

    def compact(self, max_pages=0, skip=()):
        """-> (pages moved, adapters moved)."""
        sk = np.ascontiguousarray(list(skip), dtype=np.int32)
        moved = np.zeros(2, dtype=np.uint32)
        rc = self._L.oracle_compact(self._h, int(max_pages), _ptr(sk) if len(sk) else None, len(sk), _ptr(moved))
        if rc:
            raise OracleError(rc)
        return int(moved[0]), int(moved[1])

    def page_table(self, aid):
        n = C.c_uint32(0)
        rc = self._L.oracle_page_table(self._h, aid, None, 0, C.byref(n))
        if rc:
            raise OracleError(rc)
        pt = np.empty(n.value, dtype=np.int32)
        self._L.oracle_page_table(self._h, aid, _ptr(pt), n.value, C.byref(n))
        return pt

    def stats(self):
        o = np.zeros(8, dtype=np.uint64)
        self._L.oracle_stats(self._h, _ptr(o))
        keys = ["n_pages", "free_pages", "used_pages", "resident_bytes", "loads", "evictions", "nomem", "page_bytes"]
        return dict(zip(keys, (int(v) for v in o)))

    def free_map(self):
        o = np.zeros(self.n_pages, dtype=np.uint8)
        self._L.oracle_free_map(self._h, _ptr(o))
        return o.astype(bool)

    def read_virtual(self, aid, off, nbytes):
        o = np.empty(nbytes, dtype=np.uint8)
        rc = self._L.oracle_read_virtual(self._h, aid, off, nbytes, _ptr(o))
        if rc:
            raise OracleError(rc)
        return o

    def translate(self, tok2adapter):
        t2a = np.ascontiguousarray(tok2adapter, dtype=np.int32)
        T = len(t2a)
        perm = np.empty(max(T, 1), dtype=np.int32)
        seg_adapter = np.empty(max(min(T, self.max_adapters), 1), dtype=np.int32)
        seg_start = np.empty(len(seg_adapter) + 1, dtype=np.int32)
        ns, npm = C.c_int32(0), C.c_int32(0)
        rc = self._L.oracle_translate(self._h, _ptr(t2a), T, _ptr(perm), _ptr(seg_adapter), _ptr(seg_start),
                                      C.byref(ns), C.byref(npm))
        if rc:
            raise OracleError(rc)
        return perm[: npm.value].copy(), seg_adapter[: ns.value].copy(), seg_start[: ns.value + 1].copy()

    def _sel(self, tok_sel):
        if tok_sel is None:
            return None, 0, None
        sel = np.ascontiguousarray(tok_sel, dtype=np.int32)
        return _ptr(sel), len(sel), sel

    def shrink(self, slot, x, tok2adapter, acc64=False, tok_sel=None, threads=1):
        """x: (T, d_in) raw element array (uint16 for fp16/bf16, float32). Returns v (T, max_rank)."""
        t2a = np.ascontiguousarray(tok2adapter, dtype=np.int32)
        x = np.ascontiguousarray(x)
        T = len(t2a)
        assert x.shape == (T, int(self.d_in[slot])) and x.dtype.itemsize == self.elt
        v = np.zeros((T, self.max_rank), dtype=np.float64 if acc64 else np.float32)
        p, n, keep = self._sel(tok_sel)
        rc = self._L.oracle_shrink(self._h, slot, _ptr(x), _ptr(t2a), T, p, n, int(acc64), threads, _ptr(v))
        if rc:
            raise OracleError(rc)
        return v

    def expand(self, slot, v, tok2adapter, y, acc64=False, tok_sel=None, threads=1):
        """Updates y (T, d_out) raw element array in place and returns it."""
        t2a = np.ascontiguousarray(tok2adapter, dtype=np.int32)
        T = len(t2a)
        assert y.flags.c_contiguous and y.shape == (T, int(self.d_out[slot])) and y.dtype.itemsize == self.elt
        v = np.ascontiguousarray(v, dtype=np.float64 if acc64 else np.float32)
        assert v.shape == (T, self.max_rank)
        p, n, keep = self._sel(tok_sel)
        rc = self._L.oracle_expand(self._h, slot, _ptr(v), _ptr(t2a), T, p, n, int(acc64), threads, _ptr(y))
        if rc:
            raise OracleError(rc)
        return y
