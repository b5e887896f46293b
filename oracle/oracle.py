"""ctypes front end of lmc_oracle.c (plain C, built with gcc).  TEST INFRASTRUCTURE ONLY.

Pages are passed as a list of L numpy uint8 arrays, one flat byte array per layer
(paper section 5: a page belongs to one layer), a chunk as a flat uint8 array in the
[L][P][CT][H][D] order, a slot mapping as int64.  A geometry is any object with the
attributes L P H D e BS NB CT plane_stride block_stride token_stride head_stride.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lmc_oracle.c")
_TIMING_SRC = os.path.join(_HERE, "oracle_timing.c")     # thread fan-out for the CPU baseline
_LIB = os.path.join(_HERE, "liblmc_oracle.so")

ORC_OK, ORC_INVAL, ORC_NOMEM, ORC_MISS, ORC_BADSLOT, ORC_BUSY = 0, -1, -2, -3, -4, -6


class _Geom(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("L", "P", "H", "D", "e", "BS", "NB", "CT")] + \
               [(n, ctypes.c_int64) for n in ("plane_stride", "block_stride", "token_stride",
                                              "head_stride")]


def build(force=False):
    """Compile lmc_oracle.c (and the timing driver around it) with gcc into
    liblmc_oracle.so beside it."""
    if not force and os.path.exists(_LIB) and \
            os.path.getmtime(_LIB) >= max(os.path.getmtime(_SRC), os.path.getmtime(_TIMING_SRC)):
        return _LIB
    tmp = _LIB + ".%d.tmp" % os.getpid()
    subprocess.check_call(["gcc", "-std=c11", "-O2", "-Wall", "-Wextra", "-shared", "-fPIC",
                           _SRC, _TIMING_SRC, "-lpthread", "-o", tmp])
    os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        vp, i64, u64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64, ctypes.c_int32
        gp = ctypes.POINTER(_Geom)
        sigs = {
            "orc_chunk_bytes": (i64, [gp]),
            "orc_check_slots": (ctypes.c_int, [gp, vp, i64]),
            "orc_gather_chunk": (ctypes.c_int, [gp, vp, vp, vp]),
            "orc_scatter_chunk": (ctypes.c_int, [gp, vp, vp, vp]),
            "orc_fnv1a64": (u64, [vp, i64]),
            "orc_hash_chunks": (i64, [u64, i32, vp, i64, vp]),
            "orc_store_new": (vp, [gp, i64]),
            "orc_store_free": (None, [vp]),
            "orc_store_set_evict": (None, [vp, ctypes.c_int]),
            "orc_store_drain_evicted": (i64, [vp, vp, i64]),
            "orc_store_find": (i64, [vp, u64]),
            "orc_store_slot_ptr": (vp, [vp, i64]),
            "orc_store_used": (i64, [vp]),
            "orc_lookup": (i64, [vp, vp, i64]),
            "orc_store": (ctypes.c_int, [vp, vp, vp, vp, i64, vp]),
            "orc_retrieve": (ctypes.c_int, [vp, vp, i64, vp, vp]),
            "orc_retrieve_batch": (ctypes.c_int, [vp, i64, vp, vp, vp, vp]),
            "orc_pin": (ctypes.c_int, [vp, vp, i64]),
            "orc_unpin": (ctypes.c_int, [vp, vp, i64]),
            "orc_clear": (ctypes.c_int, [vp, vp, i64]),
            "orc_acquire": (ctypes.c_int, [vp, u64]),
            "orc_release": (ctypes.c_int, [vp, u64]),
            "orc_refs": (i32, [vp, u64]),
            "orc_time_pass": (ctypes.c_double, [gp, vp, vp, vp, vp, i64, vp, vp, ctypes.c_int, ctypes.c_int]),
        }
        for name, (res, args) in sigs.items():
            f = getattr(lib, name)
            f.restype, f.argtypes = res, args
        _lib = lib
    return _lib


def _geom(g):
    return _Geom(*[int(getattr(g, n)) for n, _ in _Geom._fields_])


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data)


def _layer_table(layers):
    for a in layers:
        assert a.dtype == np.uint8 and a.ndim == 1 and a.flags.c_contiguous
    return (ctypes.c_void_p * len(layers))(*[a.ctypes.data for a in layers])


def _i64(a):
    a = np.ascontiguousarray(a, dtype=np.int64)
    return a


def _u64(a):
    return np.ascontiguousarray(a, dtype=np.uint64)


def chunk_bytes(g):
    return int(_L().orc_chunk_bytes(ctypes.byref(_geom(g))))


def gather_chunk(g, layers, slot):
    """One chunk: pages -> new flat uint8 chunk.  Raises on a slot >= NB*BS."""
    slot = _i64(slot)
    assert slot.size == g.CT
    out = np.empty(chunk_bytes(g), dtype=np.uint8)
    tbl = _layer_table(layers)
    rc = _L().orc_gather_chunk(ctypes.byref(_geom(g)), tbl, _ptr(slot), _ptr(out))
    if rc != ORC_OK:
        raise ValueError("oracle gather: status %d" % rc)
    return out


def scatter_chunk(g, chunk, slot, layers):
    """One chunk: flat uint8 chunk -> pages, in place."""
    slot = _i64(slot)
    chunk = np.ascontiguousarray(chunk, dtype=np.uint8)
    assert slot.size == g.CT and chunk.size == chunk_bytes(g)
    tbl = _layer_table(layers)
    rc = _L().orc_scatter_chunk(ctypes.byref(_geom(g)), _ptr(chunk), _ptr(slot), tbl)
    if rc != ORC_OK:
        raise ValueError("oracle scatter: status %d" % rc)


def gather(g, layers, slot_mapping):
    """n chunks -> uint8 array [n, chunk_bytes]."""
    slot_mapping = _i64(slot_mapping).reshape(-1, g.CT)
    return np.stack([gather_chunk(g, layers, s) for s in slot_mapping]) if len(slot_mapping) \
        else np.empty((0, chunk_bytes(g)), dtype=np.uint8)


def scatter(g, chunks, slot_mapping, layers):
    slot_mapping = _i64(slot_mapping).reshape(-1, g.CT)
    chunks = np.asarray(chunks, dtype=np.uint8).reshape(len(slot_mapping), -1)
    for c, s in zip(chunks, slot_mapping):
        scatter_chunk(g, c, s, layers)


def time_pass(g, src_layers, dst_layers, store_slots, load_slots, pool, buffers, n_threads, retrieve):
    """Seconds for one pass of the store analogue (gather_chunk into a buffer, memcpy into
    the pool) or the retrieve analogue (memcpy out of the pool, scatter_chunk) over all
    chunks of the slot mappings, chunks dealt out to n_threads plain threads by
    oracle_timing.c.  pool: uint8[n_chunks * chunk_bytes]; buffers: uint8[n_threads *
    chunk_bytes]; both allocated (and touched) by the caller beforehand."""
    store_slots, load_slots = _i64(store_slots), _i64(load_slots)
    n_chunks = store_slots.size // g.CT
    cb = chunk_bytes(g)
    assert load_slots.size == store_slots.size and pool.size >= n_chunks * cb and buffers.size >= n_threads * cb
    dt = _L().orc_time_pass(ctypes.byref(_geom(g)), _layer_table(src_layers), _layer_table(dst_layers),
                            _ptr(store_slots), _ptr(load_slots), n_chunks, _ptr(pool), _ptr(buffers),
                            int(n_threads), int(bool(retrieve)))
    if dt < 0:
        raise RuntimeError("oracle timing pass failed")
    return dt


def fnv1a64(data: bytes) -> int:
    buf = np.frombuffer(bytes(data), dtype=np.uint8)
    return int(_L().orc_fnv1a64(_ptr(buf) if buf.size else None, buf.size))


def hash_chunks(tokens, CT=256, seed=0):
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    out = np.empty(tokens.size // CT, dtype=np.uint64)
    n = _L().orc_hash_chunks(seed, CT, _ptr(tokens), tokens.size, _ptr(out))
    assert n == out.size
    return out


class OracleStore:
    """The CPU-memory chunk store (pool + index) of lmc_oracle.c."""

    def __init__(self, g, n_slots, evict=False):
        self.g = g
        self._cg = _geom(g)
        self.n_slots = n_slots
        self.chunk_bytes = chunk_bytes(g)
        self._h = ctypes.c_void_p(_L().orc_store_new(ctypes.byref(self._cg), n_slots))
        if not self._h:
            raise MemoryError
        if evict:
            _L().orc_store_set_evict(self._h, 1)

    def drain_evicted(self):
        """Hashes evicted since the last call, oldest eviction first."""
        out = np.empty(max(self.n_slots, 1) * 64, dtype=np.uint64)
        parts = []
        while True:
            n = int(_L().orc_store_drain_evicted(self._h, _ptr(out), out.size))
            parts.append(out[:n].copy())
            if n < out.size:
                return np.concatenate(parts)

    def close(self):
        if self._h:
            _L().orc_store_free(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def find(self, h):
        return int(_L().orc_store_find(self._h, int(h)))

    def used(self):
        return int(_L().orc_store_used(self._h))

    def slot_bytes(self, slot):
        p = _L().orc_store_slot_ptr(self._h, slot)
        return np.ctypeslib.as_array(ctypes.cast(p, ctypes.POINTER(ctypes.c_uint8)),
                                     shape=(self.chunk_bytes,)).copy()

    def lookup(self, hashes):
        hashes = _u64(hashes)
        return int(_L().orc_lookup(self._h, _ptr(hashes), hashes.size))

    def store(self, layers, slot_mapping, hashes):
        """Returns (status, chunks newly written)."""
        hashes, slot_mapping = _u64(hashes), _i64(slot_mapping)
        assert slot_mapping.size == hashes.size * self.g.CT
        n_new = ctypes.c_int64(0)
        rc = _L().orc_store(self._h, _layer_table(layers), _ptr(slot_mapping), _ptr(hashes),
                            hashes.size, ctypes.byref(n_new))
        return rc, n_new.value

    def retrieve(self, hashes, slot_mapping, layers):
        hashes, slot_mapping = _u64(hashes), _i64(slot_mapping)
        assert slot_mapping.size == hashes.size * self.g.CT
        return _L().orc_retrieve(self._h, _ptr(hashes), hashes.size, _ptr(slot_mapping),
                                 _layer_table(layers))

    def retrieve_batch(self, req_chunk_offsets, hashes, slot_mapping, layers):
        off, hashes, slot_mapping = _i64(req_chunk_offsets), _u64(hashes), _i64(slot_mapping)
        return _L().orc_retrieve_batch(self._h, off.size - 1, _ptr(off), _ptr(hashes),
                                       _ptr(slot_mapping), _layer_table(layers))

    def pin(self, hashes):
        hashes = _u64(hashes)
        return _L().orc_pin(self._h, _ptr(hashes), hashes.size)

    def unpin(self, hashes):
        hashes = _u64(hashes)
        return _L().orc_unpin(self._h, _ptr(hashes), hashes.size)

    def clear(self, hashes):
        hashes = _u64(hashes)
        return _L().orc_clear(self._h, _ptr(hashes), hashes.size)

    def acquire(self, h):
        return _L().orc_acquire(self._h, int(h))

    def release(self, h):
        return _L().orc_release(self._h, int(h))

    def refs(self, h):
        return int(_L().orc_refs(self._h, int(h)))
