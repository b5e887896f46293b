"""ctypes binding of liblmc (include/lmc.h).  Argument marshalling only: every step of
the store / retrieve path runs inside the library.

Device buffers are passed as objects with a ``data_ptr()`` method (torch tensors) or as
integer addresses; streams as objects with a ``cuda_stream`` attribute (torch streams;
ROCm PyTorch exposes HIP streams under that name), integer handles, or None for the
null stream.  Host arrays are numpy.  A status other than LMC_OK raises LMCError.

The library must have been built (``python -m paper_2510_09665_amd.build``); there is
no fallback of any kind when it is missing.
"""
import ctypes
import os

import numpy as np

LMC_OK, LMC_ERR_INVAL, LMC_ERR_NOMEM, LMC_ERR_MISS, LMC_ERR_BADSLOT = 0, -1, -2, -3, -4
LMC_ERR_HIP, LMC_ERR_BUSY, LMC_ERR_NODEVICE, LMC_ERR_IO = -5, -6, -7, -8
LMC_MAX_LAYERS = 160
LMC_DEVICE_NONE = -1
LMC_FLAG_VALIDATE_SLOTS, LMC_FLAG_FORCE_SYNC, LMC_FLAG_POISON_STAGING, LMC_FLAG_TIMING = 1, 2, 4, 8
LMC_FLAG_DIRECT = 16
LMC_FLAG_EVICT_LRU = 32
LMC_FLAG_KEEP_STREAMS = 64
LMC_FLAG_TRACE = 128
LMC_STAGE_GATHER, LMC_STAGE_D2H, LMC_STAGE_H2D, LMC_STAGE_SCATTER = 0, 1, 2, 3

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "liblmc.so")

EXPORTS = [
    "lmc_create", "lmc_destroy", "lmc_chunk_bytes", "lmc_chunk_tokens", "lmc_pool_slots",
    "lmc_hash_chunks", "lmc_hash_chunks_from", "lmc_seq_open", "lmc_seq_append",
    "lmc_seq_pending_tokens", "lmc_seq_close", "lmc_block_size", "lmc_test", "lmc_window_create",
    "lmc_window_destroy", "lmc_window_release", "lmc_window_offload", "lmc_window_acquire",
    "lmc_window_get",
    "lmc_lookup", "lmc_store", "lmc_retrieve", "lmc_retrieve_batch", "lmc_retrieve_layerwise",
    "lmc_store_begin", "lmc_store_layers", "lmc_wait_layer", "lmc_wait", "lmc_gather",
    "lmc_scatter", "lmc_store_static", "lmc_put_host", "lmc_get_host", "lmc_find_slot", "lmc_pin", "lmc_unpin",
    "lmc_clear", "lmc_drain_evicted", "lmc_get_stats", "lmc_reset_stats", "lmc_measure_link", "lmc_measure_link_kernel", "lmc_measure_link_duplex", "lmc_measure_link_duplex_kernel",
    "lmc_copy", "lmc_copy_tiles", "lmc_tune", "lmc_trace_read", "lmc_probe_stream", "lmc_chunk_acquire", "lmc_chunk_release", "lmc_tier_open", "lmc_tier_close",
    "lmc_tier_write", "lmc_tier_wait", "lmc_tier_lookup", "lmc_tier_read", "lmc_tier_errno",
    "lmc_tier_get_stats",
    "lmc_strerror", "lmc_last_hip_error",
]


class lmc_kv_geom_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("num_layers", "num_planes", "num_heads", "head_dim", "elem_bytes", "block_size",
                 "num_blocks", "chunk_tokens")] + \
               [(n, ctypes.c_int64) for n in
                ("plane_stride", "block_stride", "token_stride", "head_stride")]


class lmc_config_t(ctypes.Structure):
    _fields_ = [("geom", lmc_kv_geom_t), ("host_pool_bytes", ctypes.c_uint64),
                ("num_staging", ctypes.c_int32), ("staging_chunks", ctypes.c_int32),
                ("device", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("hash_seed", ctypes.c_uint64)]


class lmc_trace_rec_t(ctypes.Structure):
    _fields_ = [("ticket", ctypes.c_uint64), ("stage", ctypes.c_int32), ("chunks", ctypes.c_int32),
                ("bytes", ctypes.c_uint64), ("begin_us", ctypes.c_double), ("end_us", ctypes.c_double)]


class lmc_stats_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint64) for n in
                ("pool_slots_total", "pool_slots_used", "chunks_stored", "chunks_skipped_dup",
                 "chunks_retrieved", "retrieve_misses", "alloc_failures", "chunks_evicted", "d2h_guard_switches", "d2h_guard_active",
                 "bytes_gathered",
                 "bytes_scattered", "bytes_d2h", "bytes_h2d", "gather_launches",
                 "scatter_launches", "timed_gather_launches", "timed_scatter_launches")] + \
               [("gather_ms", ctypes.c_double), ("scatter_ms", ctypes.c_double),
                ("d2h_copy_best_gbps", ctypes.c_double), ("d2h_copy_last_gbps", ctypes.c_double)]


class LMCError(RuntimeError):
    def __init__(self, status, what, ticket=None, hip_error=0):
        self.status, self.ticket, self.hip_error = status, ticket, hip_error
        msg = "%s: %s (%d)" % (what, _lib().lmc_strerror(status).decode(), status)
        if status == LMC_ERR_HIP:
            msg += " hipError_t=%d" % hip_error
        super().__init__(msg)


_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("liblmc.so is not built: run `python -m paper_2510_09665_amd.build` "
                              "(needs hipcc); there is no fallback path")
        # PyTorch wheels ship their own HIP runtime.  A process must not end up with two:
        # if PyTorch is present, let it load its runtime first so that liblmc binds to the
        # same one and device pointers and streams mean the same thing on both sides.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        lib = ctypes.CDLL(LIB_PATH)
        vp, i64, u64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64, ctypes.c_int32
        st = ctypes.c_int32
        sig = {
            "lmc_create": (st, [ctypes.POINTER(lmc_config_t), ctypes.POINTER(vp)]),
            "lmc_destroy": (st, [vp]),
            "lmc_chunk_bytes": (i64, [vp]),
            "lmc_chunk_tokens": (i32, [vp]),
            "lmc_pool_slots": (i64, [vp]),
            "lmc_hash_chunks_from": (st, [vp, u64, vp, i64, vp, ctypes.POINTER(i64)]),
            "lmc_seq_open": (st, [vp, vp, vp, i64, ctypes.POINTER(vp)]),
            "lmc_seq_append": (st, [vp, vp, vp, i64, vp, vp, ctypes.POINTER(i64), ctypes.POINTER(u64)]),
            "lmc_seq_pending_tokens": (st, [vp, ctypes.POINTER(i64)]),
            "lmc_seq_close": (st, [vp]),
            "lmc_block_size": (i32, [vp]),
            "lmc_test": (st, [vp, u64]),
            "lmc_window_create": (st, [vp, i64, i64, ctypes.POINTER(vp)]),
            "lmc_window_destroy": (st, [vp]),
            "lmc_window_release": (st, [vp, vp, vp, i64]),
            "lmc_window_offload": (st, [vp, vp, vp, ctypes.POINTER(i64)]),
            "lmc_window_acquire": (st, [vp, i64, vp, i32]),
            "lmc_window_get": (st, [vp] + [ctypes.POINTER(i64)] * 4 + [ctypes.POINTER(i32)]),
            "lmc_probe_stream": (st, [vp, vp, ctypes.POINTER(ctypes.c_uint32)]),
            "lmc_chunk_acquire": (st, [vp, u64, ctypes.POINTER(vp)]),
            "lmc_chunk_release": (st, [vp, u64]),
            "lmc_tier_open": (st, [vp, ctypes.POINTER(ctypes.c_char_p), i32, i32, ctypes.POINTER(vp)]),
            "lmc_tier_close": (st, [vp]),
            "lmc_tier_write": (st, [vp, vp, i64]),
            "lmc_tier_wait": (st, [vp]),
            "lmc_tier_lookup": (st, [vp, i32, vp, i64, ctypes.POINTER(i64)]),
            "lmc_tier_read": (st, [vp, i32, vp, i64]),
            "lmc_tier_errno": (i32, [vp]),
            "lmc_tier_get_stats": (st, [vp] + [ctypes.POINTER(u64)] * 3),
            "lmc_hash_chunks": (st, [vp, vp, i64, vp, ctypes.POINTER(i64)]),
            "lmc_lookup": (st, [vp, vp, i64, ctypes.POINTER(i64)]),
            "lmc_store": (st, [vp, vp, vp, vp, i64, vp, ctypes.POINTER(u64)]),
            "lmc_retrieve": (st, [vp, vp, i64, vp, vp, vp, ctypes.POINTER(u64)]),
            "lmc_retrieve_batch": (st, [vp, i64, vp, vp, vp, vp, vp, ctypes.POINTER(u64)]),
            "lmc_retrieve_layerwise": (st, [vp, vp, i64, vp, vp, i32, vp, ctypes.POINTER(u64)]),
            "lmc_store_begin": (st, [vp, vp, vp, i64, vp, ctypes.POINTER(u64)]),
            "lmc_store_layers": (st, [vp, u64, i32, i32, vp, vp]),
            "lmc_wait_layer": (st, [vp, u64, i32, vp]),
            "lmc_wait": (st, [vp, u64]),
            "lmc_gather": (st, [vp, vp, vp, i64, vp, vp]),
            "lmc_scatter": (st, [vp, vp, vp, i64, vp, vp]),
            "lmc_store_static": (st, [vp, vp, vp, i64, vp, vp]),
            "lmc_put_host": (st, [vp, vp, i64, vp]),
            "lmc_get_host": (st, [vp, u64, vp]),
            "lmc_find_slot": (st, [vp, u64, ctypes.POINTER(i64)]),
            "lmc_pin": (st, [vp, vp, i64]),
            "lmc_unpin": (st, [vp, vp, i64]),
            "lmc_clear": (st, [vp, vp, i64]),
            "lmc_drain_evicted": (st, [vp, vp, i64, vp]),
            "lmc_get_stats": (st, [vp, ctypes.POINTER(lmc_stats_t)]),
            "lmc_reset_stats": (st, [vp]),
            "lmc_measure_link": (st, [vp, u64, i32, ctypes.POINTER(ctypes.c_double),
                                      ctypes.POINTER(ctypes.c_double)]),
            "lmc_measure_link_kernel": (st, [vp, u64, i32, ctypes.POINTER(ctypes.c_double),
                                      ctypes.POINTER(ctypes.c_double)]),
            "lmc_measure_link_duplex": (st, [vp, u64, i32, ctypes.POINTER(ctypes.c_double)]),
            "lmc_measure_link_duplex_kernel": (st, [vp, u64, i32, ctypes.c_uint32, ctypes.POINTER(ctypes.c_double)]),
            "lmc_copy": (st, [vp, vp, vp, u64, vp]),
            "lmc_copy_tiles": (st, [vp, vp, vp, vp, vp, u64, ctypes.c_uint32, vp]),
            "lmc_tune": (st, [vp, ctypes.c_char_p, i64]),
            "lmc_trace_read": (st, [vp, ctypes.POINTER(lmc_trace_rec_t), i64, ctypes.POINTER(i64), ctypes.POINTER(u64)]),
            "lmc_strerror": (ctypes.c_char_p, [st]),
            "lmc_last_hip_error": (i32, [vp]),
        }
        assert sorted(sig) == sorted(EXPORTS)
        for name, (res, args) in sig.items():
            f = getattr(lib, name)
            f.restype, f.argtypes = res, args
        _LIB = lib
    return _LIB


def _dev(x):
    """device address of a tensor-like or an int"""
    if x is None:
        return None
    return ctypes.c_void_p(x.data_ptr() if hasattr(x, "data_ptr") else int(x))


def _stream(s):
    if s is None:
        return None
    return ctypes.c_void_p(getattr(s, "cuda_stream", s))


def _host(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, ctypes.c_void_p(a.ctypes.data)


def make_geom(g):
    """lmc_kv_geom_t from any object with L P H D e BS NB CT and the four strides."""
    return lmc_kv_geom_t(g.L, g.P, g.H, g.D, g.e, g.BS, g.NB, g.CT, g.plane_stride,
                         g.block_stride, g.token_stride, g.head_stride)


class Context:
    """One lmc_ctx_t.  Methods carry the C names without the lmc_ prefix."""

    def __init__(self, geom, host_pool_bytes, num_staging=2, staging_chunks=16, device=0, flags=0,
                 hash_seed=0):
        """staging_chunks=16 is the measured sweet spot on MI355X (one launch then covers a
        4096-token request); it costs 2 * num_staging * staging_chunks chunks of HBM."""
        self._h = None
        g = geom if isinstance(geom, lmc_kv_geom_t) else make_geom(geom)
        cfg = lmc_config_t(g, host_pool_bytes, num_staging, staging_chunks, device, flags,
                           hash_seed)
        h = ctypes.c_void_p()
        rc = _lib().lmc_create(ctypes.byref(cfg), ctypes.byref(h))
        if rc != LMC_OK:
            raise LMCError(rc, "lmc_create")
        self._h = h
        self.chunk_tokens = g.chunk_tokens
        self.num_layers = g.num_layers

    # -- lifetime ---------------------------------------------------------------
    def destroy(self):
        if self._h is not None:
            _lib().lmc_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.destroy()

    def _check(self, rc, what, ticket=None):
        if rc != LMC_OK:
            raise LMCError(rc, what, ticket, _lib().lmc_last_hip_error(self._h))

    def _layers(self, kv_layers):
        if len(kv_layers) != self.num_layers:
            raise ValueError("expected %d layer pointers" % self.num_layers)
        return (ctypes.c_void_p * len(kv_layers))(
            *[(x.data_ptr() if hasattr(x, "data_ptr") else int(x)) for x in kv_layers])

    # -- sizes ------------------------------------------------------------------
    def chunk_bytes(self):
        return int(_lib().lmc_chunk_bytes(self._h))

    def pool_slots(self):
        return int(_lib().lmc_pool_slots(self._h))

    # -- token processor / index --------------------------------------------------
    def hash_chunks(self, tokens):
        tok, tp = _host(tokens, np.int32)
        out = np.empty(tok.size // self.chunk_tokens, dtype=np.uint64)
        n = ctypes.c_int64()
        self._check(_lib().lmc_hash_chunks(self._h, tp, tok.size, ctypes.c_void_p(out.ctypes.data),
                                           ctypes.byref(n)), "lmc_hash_chunks")
        return out[:n.value]

    def hash_chunks_from(self, prev_id, tokens):
        tok, tp = _host(tokens, np.int32)
        out = np.empty(tok.size // self.chunk_tokens, dtype=np.uint64)
        n = ctypes.c_int64()
        self._check(_lib().lmc_hash_chunks_from(self._h, int(prev_id), tp, tok.size,
                                                ctypes.c_void_p(out.ctypes.data), ctypes.byref(n)),
                    "lmc_hash_chunks_from")
        return out[:n.value]

    def seq_open(self, prompt_tokens, prompt_slots):
        return Sequence(self, prompt_tokens, prompt_slots)

    def lookup(self, chunk_ids):
        ids, ip = _host(chunk_ids, np.uint64)
        n = ctypes.c_int64()
        self._check(_lib().lmc_lookup(self._h, ip, ids.size, ctypes.byref(n)), "lmc_lookup")
        return n.value

    # -- the path -----------------------------------------------------------------
    def store(self, kv_layers, slot_mapping, chunk_ids, stream_to_wait_on=None):
        """Enqueue; returns the ticket.  On LMC_ERR_NOMEM the error carries the ticket."""
        ids, ip = _host(chunk_ids, np.uint64)
        t = ctypes.c_uint64()
        rc = _lib().lmc_store(self._h, self._layers(kv_layers), _dev(slot_mapping), ip, ids.size,
                              _stream(stream_to_wait_on), ctypes.byref(t))
        self._check(rc, "lmc_store", t.value)
        return t.value

    def retrieve(self, chunk_ids, slot_mapping, kv_layers, stream_to_signal=None):
        ids, ip = _host(chunk_ids, np.uint64)
        t = ctypes.c_uint64()
        rc = _lib().lmc_retrieve(self._h, ip, ids.size, _dev(slot_mapping), self._layers(kv_layers),
                                 _stream(stream_to_signal), ctypes.byref(t))
        self._check(rc, "lmc_retrieve", t.value)
        return t.value

    def retrieve_batch(self, req_chunk_offsets, chunk_ids, slot_mapping, kv_layers,
                       stream_to_signal=None):
        off, op = _host(req_chunk_offsets, np.int64)
        ids, ip = _host(chunk_ids, np.uint64)
        t = ctypes.c_uint64()
        rc = _lib().lmc_retrieve_batch(self._h, off.size - 1, op, ip, _dev(slot_mapping),
                                       self._layers(kv_layers), _stream(stream_to_signal),
                                       ctypes.byref(t))
        self._check(rc, "lmc_retrieve_batch", t.value)
        return t.value

    def retrieve_layerwise(self, chunk_ids, slot_mapping, kv_layers, layers_per_step=1,
                           stream_to_wait_on=None):
        ids, ip = _host(chunk_ids, np.uint64)
        t = ctypes.c_uint64()
        rc = _lib().lmc_retrieve_layerwise(self._h, ip, ids.size, _dev(slot_mapping),
                                           self._layers(kv_layers), layers_per_step,
                                           _stream(stream_to_wait_on), ctypes.byref(t))
        self._check(rc, "lmc_retrieve_layerwise", t.value)
        return t.value

    def store_begin(self, slot_mapping, chunk_ids, stream_to_wait_on=None):
        ids, ip = _host(chunk_ids, np.uint64)
        t = ctypes.c_uint64()
        rc = _lib().lmc_store_begin(self._h, _dev(slot_mapping), ip, ids.size,
                                    _stream(stream_to_wait_on), ctypes.byref(t))
        self._check(rc, "lmc_store_begin", t.value)
        return t.value

    def store_layers(self, ticket, first_layer, n_layers, kv_layers, stream_to_wait_on=None):
        self._check(_lib().lmc_store_layers(self._h, ticket, first_layer, n_layers,
                                            self._layers(kv_layers), _stream(stream_to_wait_on)),
                    "lmc_store_layers")

    def wait_layer(self, ticket, layer, stream=None):
        self._check(_lib().lmc_wait_layer(self._h, ticket, layer, _stream(stream)), "lmc_wait_layer")

    def test(self, ticket):
        """True if the ticket's work has finished (never blocks)."""
        rc = _lib().lmc_test(self._h, ticket)
        if rc == LMC_ERR_BUSY:
            return False
        self._check(rc, "lmc_test")
        return True

    def chunk_acquire(self, chunk_id):
        """Raises the chunk's reference counter; returns a read-only numpy view of its
        bytes in the pinned pool, valid until chunk_release."""
        p = ctypes.c_void_p()
        self._check(_lib().lmc_chunk_acquire(self._h, int(chunk_id), ctypes.byref(p)), "lmc_chunk_acquire")
        a = np.ctypeslib.as_array(ctypes.cast(p, ctypes.POINTER(ctypes.c_uint8)), shape=(self.chunk_bytes(),))
        a.flags.writeable = False
        return a

    def chunk_release(self, chunk_id):
        self._check(_lib().lmc_chunk_release(self._h, int(chunk_id)), "lmc_chunk_release")

    def tier_open(self, dirs, n_threads=2):
        return Tier(self, dirs, n_threads)

    def window_create(self, window_pages, max_batch_pages=64):
        return Window(self, window_pages, max_batch_pages)

    def wait(self, ticket=0):
        self._check(_lib().lmc_wait(self._h, ticket), "lmc_wait")

    def gather(self, kv_layers, slot_mapping, n_chunks, staging_dev, stream=None):
        self._check(_lib().lmc_gather(self._h, self._layers(kv_layers), _dev(slot_mapping), n_chunks,
                                      _dev(staging_dev), _stream(stream)), "lmc_gather")

    def scatter(self, staging_dev, slot_mapping, n_chunks, kv_layers, stream=None):
        self._check(_lib().lmc_scatter(self._h, _dev(staging_dev), _dev(slot_mapping), n_chunks,
                                       self._layers(kv_layers), _stream(stream)), "lmc_scatter")

    def store_static(self, kv_layers, slot_mapping, n_chunks, host_dst, stream=None):
        """host_dst: a pinned uint8 tensor (or address) of n_chunks * chunk_bytes."""
        self._check(_lib().lmc_store_static(self._h, self._layers(kv_layers), _dev(slot_mapping), n_chunks,
                                            _dev(host_dst), _stream(stream)), "lmc_store_static")

    # -- host-side chunk access -----------------------------------------------------
    def put_host(self, chunk_ids, host_src):
        ids, ip = _host(chunk_ids, np.uint64)
        src, sp = _host(host_src, np.uint8)
        if src.size != ids.size * self.chunk_bytes():
            raise ValueError("host_src must hold %d chunks" % ids.size)
        self._check(_lib().lmc_put_host(self._h, ip, ids.size, sp), "lmc_put_host")

    def get_host(self, chunk_id):
        out = np.empty(self.chunk_bytes(), dtype=np.uint8)
        self._check(_lib().lmc_get_host(self._h, int(chunk_id), ctypes.c_void_p(out.ctypes.data)),
                    "lmc_get_host")
        return out

    def find_slot(self, chunk_id):
        s = ctypes.c_int64()
        self._check(_lib().lmc_find_slot(self._h, int(chunk_id), ctypes.byref(s)), "lmc_find_slot")
        return s.value

    def pin(self, chunk_ids):
        ids, ip = _host(chunk_ids, np.uint64)
        self._check(_lib().lmc_pin(self._h, ip, ids.size), "lmc_pin")

    def unpin(self, chunk_ids):
        ids, ip = _host(chunk_ids, np.uint64)
        self._check(_lib().lmc_unpin(self._h, ip, ids.size), "lmc_unpin")

    def drain_evicted(self):
        """Ids evicted since the last call (LMC_FLAG_EVICT_LRU), oldest eviction first."""
        out = np.empty(4096, dtype=np.uint64)
        parts = []
        while True:
            n = ctypes.c_int64(0)
            self._check(_lib().lmc_drain_evicted(self._h, out.ctypes.data, out.size, ctypes.byref(n)),
                        "lmc_drain_evicted")
            parts.append(out[:n.value].copy())
            if n.value < out.size:
                return np.concatenate(parts)

    def clear(self, chunk_ids):
        ids, ip = _host(chunk_ids, np.uint64)
        self._check(_lib().lmc_clear(self._h, ip, ids.size), "lmc_clear")

    # -- stats, measurement, tuning ---------------------------------------------------
    def get_stats(self):
        s = lmc_stats_t()
        self._check(_lib().lmc_get_stats(self._h, ctypes.byref(s)), "lmc_get_stats")
        return {n: getattr(s, n) for n, _ in lmc_stats_t._fields_}

    def reset_stats(self):
        self._check(_lib().lmc_reset_stats(self._h), "lmc_reset_stats")

    def measure_link(self, nbytes, reps=3):
        """(h2d GB/s, d2h GB/s) of hipMemcpyAsync between the pinned pool and the GPU."""
        a, b = ctypes.c_double(), ctypes.c_double()
        self._check(_lib().lmc_measure_link(self._h, nbytes, reps, ctypes.byref(a), ctypes.byref(b)),
                    "lmc_measure_link")
        return a.value, b.value

    def measure_link_kernel(self, nbytes, reps=3):
        """(h2d GB/s, d2h GB/s) of the library's link-paced copy kernel over the same link."""
        a, b = ctypes.c_double(), ctypes.c_double()
        self._check(_lib().lmc_measure_link_kernel(self._h, nbytes, reps, ctypes.byref(a), ctypes.byref(b)),
                    "lmc_measure_link_kernel")
        return a.value, b.value

    def measure_link_duplex(self, nbytes, reps=3):
        """sum of both directions, GB/s, with an upload and a download running together"""
        a = ctypes.c_double()
        self._check(_lib().lmc_measure_link_duplex(self._h, nbytes, reps, ctypes.byref(a)),
                    "lmc_measure_link_duplex")
        return a.value

    def measure_link_duplex_kernel(self, nbytes, by_kernel, reps=3):
        """as measure_link_duplex, the upload (bit 0) and / or download (bit 1) made by the copy kernel"""
        a = ctypes.c_double()
        self._check(_lib().lmc_measure_link_duplex_kernel(self._h, nbytes, reps, by_kernel, ctypes.byref(a)),
                    "lmc_measure_link_duplex_kernel")
        return a.value

    def copy(self, dst_dev, src_dev, nbytes, stream=None):
        self._check(_lib().lmc_copy(self._h, _dev(dst_dev), _dev(src_dev), nbytes, _stream(stream)),
                    "lmc_copy")

    def copy_tiles(self, dst_dev, dst_order, src_dev, src_order, n_tiles, mode=0, stream=None):
        """4 KiB tiles in a given order (device uint32 tensors or None); mode 0 copy, 1 read, 2 write"""
        self._check(_lib().lmc_copy_tiles(self._h, _dev(dst_dev), _dev(dst_order), _dev(src_dev), _dev(src_order),
                                          n_tiles, mode, _stream(stream)), "lmc_copy_tiles")

    def probe_stream(self, stream):
        """Bit mask of the library's copy streams that share a hardware queue with `stream`
        (0 = work on it never waits behind the library's copies)."""
        m = ctypes.c_uint32()
        self._check(_lib().lmc_probe_stream(self._h, _stream(stream), ctypes.byref(m)), "lmc_probe_stream")
        return m.value

    def tune(self, key, value):
        self._check(_lib().lmc_tune(self._h, key.encode(), int(value)), "lmc_tune")

    def trace_read(self, cap=65536):
        """Finished records of the trace (LMC_FLAG_TRACE), oldest first: a list of dicts with
        ticket, stage (LMC_STAGE_*), chunks, bytes, begin_us, end_us; and how many were lost."""
        buf = (lmc_trace_rec_t * cap)()
        n, dropped = ctypes.c_int64(0), ctypes.c_uint64(0)
        self._check(_lib().lmc_trace_read(self._h, buf, cap, ctypes.byref(n), ctypes.byref(dropped)), "lmc_trace_read")
        recs = [dict(ticket=r.ticket, stage=r.stage, chunks=r.chunks, bytes=r.bytes, begin_us=r.begin_us,
                     end_us=r.end_us) for r in buf[:n.value]]
        return recs, dropped.value


class Sequence:
    """One lmc_seq_t: the delayed-decode-storing accumulator of one sequence."""

    def __init__(self, ctx, prompt_tokens, prompt_slots):
        self._ctx = ctx
        self._h = None
        tok, tp = _host(prompt_tokens, np.int32)
        sl, sp = _host(prompt_slots, np.int64)
        if tok.size != sl.size:
            raise ValueError("one slot per token")
        h = ctypes.c_void_p()
        ctx._check(_lib().lmc_seq_open(ctx._h, tp, sp, tok.size, ctypes.byref(h)), "lmc_seq_open")
        self._h = h

    def append(self, tokens, slots, kv_layers, stream=None):
        """Returns (chunks completed by this call, ticket of the last store or 0)."""
        tok, tp = _host(tokens, np.int32)
        sl, sp = _host(slots, np.int64)
        if tok.size != sl.size:
            raise ValueError("one slot per token")
        n, t = ctypes.c_int64(), ctypes.c_uint64()
        rc = _lib().lmc_seq_append(self._h, tp, sp, tok.size, self._ctx._layers(kv_layers),
                                   _stream(stream), ctypes.byref(n), ctypes.byref(t))
        self._ctx._check(rc, "lmc_seq_append", t.value)
        return n.value, t.value

    def pending_tokens(self):
        n = ctypes.c_int64()
        self._ctx._check(_lib().lmc_seq_pending_tokens(self._h, ctypes.byref(n)), "lmc_seq_pending_tokens")
        return n.value

    def close(self):
        if self._h is not None:
            _lib().lmc_seq_close(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Tier:
    """One lmc_tier_t: directories under the pool, every chunk written to all of them at once."""

    def __init__(self, ctx, dirs, n_threads):
        self._ctx, self._h = ctx, None
        arr = (ctypes.c_char_p * len(dirs))(*[os.fsencode(d) for d in dirs])
        h = ctypes.c_void_p()
        ctx._check(_lib().lmc_tier_open(ctx._h, arr, len(dirs), n_threads, ctypes.byref(h)), "lmc_tier_open")
        self._h = h

    def write(self, chunk_ids):
        ids, ip = _host(chunk_ids, np.uint64)
        self._ctx._check(_lib().lmc_tier_write(self._h, ip, ids.size), "lmc_tier_write")

    def wait(self):
        self._ctx._check(_lib().lmc_tier_wait(self._h), "lmc_tier_wait")

    def lookup(self, dir_index, chunk_ids):
        ids, ip = _host(chunk_ids, np.uint64)
        n = ctypes.c_int64()
        self._ctx._check(_lib().lmc_tier_lookup(self._h, dir_index, ip, ids.size, ctypes.byref(n)),
                         "lmc_tier_lookup")
        return n.value

    def read(self, dir_index, chunk_ids):
        ids, ip = _host(chunk_ids, np.uint64)
        self._ctx._check(_lib().lmc_tier_read(self._h, dir_index, ip, ids.size), "lmc_tier_read")

    def errno(self):
        return int(_lib().lmc_tier_errno(self._h))

    def get_stats(self):
        v = [ctypes.c_uint64() for _ in range(3)]
        self._ctx._check(_lib().lmc_tier_get_stats(self._h, *[ctypes.byref(x) for x in v]), "lmc_tier_get_stats")
        return dict(files_written=v[0].value, bytes_written=v[1].value, chunks_read=v[2].value)

    def close(self):
        if self._h is not None:
            _lib().lmc_tier_close(self._h)
            self._h = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


class Window:
    """One lmc_window_t: the three-pointer window of dynamic offloading."""

    def __init__(self, ctx, window_pages, max_batch_pages):
        self._ctx, self._h = ctx, None
        h = ctypes.c_void_p()
        ctx._check(_lib().lmc_window_create(ctx._h, window_pages, max_batch_pages, ctypes.byref(h)),
                   "lmc_window_create")
        self._h = h

    def release(self, blocks, chunk_ids):
        b, bp = _host(blocks, np.int64)
        i, ip = _host(chunk_ids, np.uint64)
        if b.size != i.size:
            raise ValueError("one id per block")
        self._ctx._check(_lib().lmc_window_release(self._h, bp, ip, b.size), "lmc_window_release")

    def offload(self, kv_layers, stream=None):
        n = ctypes.c_int64()
        self._ctx._check(_lib().lmc_window_offload(self._h, self._ctx._layers(kv_layers), _stream(stream),
                                                   ctypes.byref(n)), "lmc_window_offload")
        return n.value

    def acquire(self, n, block=False):
        """The n head blocks, or None when the request stalls."""
        out = np.empty(n, dtype=np.int64)
        rc = _lib().lmc_window_acquire(self._h, n, ctypes.c_void_p(out.ctypes.data), 1 if block else 0)
        if rc == LMC_ERR_BUSY:
            return None
        self._ctx._check(rc, "lmc_window_acquire")
        return out

    def get(self):
        v = [ctypes.c_int64() for _ in range(4)]
        st = ctypes.c_int32()
        self._ctx._check(_lib().lmc_window_get(self._h, *[ctypes.byref(x) for x in v], ctypes.byref(st)),
                         "lmc_window_get")
        return dict(start=v[0].value, current=v[1].value, end=v[2].value, tail=v[3].value, state=st.value)

    def destroy(self):
        if self._h is not None:
            _lib().lmc_window_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def strerror(status):
    return _lib().lmc_strerror(status).decode()
