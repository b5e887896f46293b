"""Model check of the whole library against the oracle's chunk store on the GPU: random
sequences of store / retrieve (bulk, batched, layer-wise) / lookup / clear / pin / unpin,
with statuses, slot numbers, pool bytes and page contents compared after every step."""
import numpy as np
import pytest

import oracle
from paper_2510_09665_amd import workloads as W

pytestmark = pytest.mark.gpu


def _status(fn):
    from paper_2510_09665_amd import lmc
    try:
        fn()
        return 0
    except lmc.LMCError as e:
        return e.status


@pytest.mark.parametrize("seed,flags,small_direct", [(1, "poison", 0), (2, "direct", None), (3, "none", 0),
                                                     (4, "none", 2), (5, "poison", 2),
                                                     (6, "evict", 0), (7, "evict", 2)])
def test_random_operation_sequences(seed, flags, small_direct):
    # small_direct: bulk calls of at most that many chunks skip staging (the library's
    # size rule, which at this geometry's 12 KiB chunks would otherwise catch every call);
    # 0 = every call staged, 2 = calls of 1-2 chunks direct and of 3-4 chunks staged
    import torch
    from gpu_util import PagedKV, assert_layers_equal, slots_to_device
    from paper_2510_09665_amd import lmc
    g = W.KVGeometry(L=3, P=2, H=2, D=32, e=2, BS=4, NB=256, CT=16)
    rng = np.random.default_rng(seed)
    kv = PagedKV(g, np.arange(g.NB), rng)                    # source pages, all tracked
    dst = PagedKV(g, np.arange(g.NB), fill="sentinel")       # destination pages
    n_slots = 6
    f = {"poison": lmc.LMC_FLAG_POISON_STAGING, "direct": lmc.LMC_FLAG_DIRECT, "none": 0,
         "evict": lmc.LMC_FLAG_EVICT_LRU | lmc.LMC_FLAG_POISON_STAGING}[flags]
    stream = torch.cuda.current_stream()
    ora = oracle.OracleStore(g, n_slots, evict=flags == "evict")
    keep = []                                                # device slot mappings stay alive
    with lmc.Context(g, n_slots * g.chunk_bytes, staging_chunks=2, flags=f) as c:
        if small_direct is not None:
            c.tune("direct_store_below", small_direct * g.chunk_bytes)
            c.tune("direct_retrieve_below", small_direct * g.chunk_bytes)
        for step in range(150):
            op = rng.choice(["store", "store_lw", "retrieve", "retrieve_lw", "batch", "lookup", "clear",
                             "pin", "unpin"])
            ids = rng.integers(0, 10, rng.integers(1, 5)).astype(np.uint64)
            n = ids.size
            if op in ("store", "store_lw"):
                sl = rng.permutation(g.n_slots)[:n * g.CT].astype(np.int64)
                if rng.random() < 0.3:
                    sl[rng.integers(0, sl.size, 3)] = -1     # tokens without a page
                d = slots_to_device(sl)
                keep.append(d)
                want_rc, _ = ora.store(kv.host, sl, ids)
                if op == "store":
                    got = _status(lambda: c.store(kv.dev, d, ids, stream))
                else:
                    def lw():
                        try:
                            t = c.store_begin(d, ids, stream)
                            rc = 0
                        except lmc.LMCError as e:
                            if e.status != lmc.LMC_ERR_NOMEM:
                                raise
                            t, rc = e.ticket, e.status
                        for l in range(g.L):
                            c.store_layers(t, l, 1, kv.dev, stream)
                        if rc:
                            raise lmc.LMCError(rc, "store_begin", t)
                    got = _status(lw)
                assert got == want_rc, (step, op)
                c.wait()
            elif op in ("retrieve", "retrieve_lw", "batch"):
                tau = rng.permutation(g.n_slots)[:n * g.CT].astype(np.int64)
                d = slots_to_device(tau)
                keep.append(d)
                if op == "batch":
                    cuts = np.sort(rng.integers(0, n + 1, 2))
                    off = [0, int(cuts[0]), int(cuts[1]), n]
                    want_rc = ora.retrieve_batch(off, ids, tau, dst.host)
                    got = _status(lambda: c.retrieve_batch(off, ids, d, dst.dev, stream))
                else:
                    want_rc = ora.retrieve(ids, tau, dst.host)
                    if op == "retrieve":
                        got = _status(lambda: c.retrieve(ids, d, dst.dev, stream))
                    else:
                        got = _status(lambda: c.retrieve_layerwise(ids, d, dst.dev, int(rng.integers(1, 4)), stream))
                assert got == want_rc, (step, op)
                c.wait()
                torch.cuda.synchronize()
                assert_layers_equal(dst.device_blocks_to_host(), dst.host, "step %d %s" % (step, op))
            elif op == "lookup":
                assert c.lookup(ids) == ora.lookup(ids), step
            elif op == "clear":
                assert _status(lambda: c.clear(ids)) == ora.clear(ids), step
            elif op == "pin":
                assert _status(lambda: c.pin(ids)) == ora.pin(ids), step
            else:
                assert _status(lambda: c.unpin(ids)) == ora.unpin(ids), step
            # with eviction on: the same victims in the same order (every call above was
            # waited for, so the library has nothing in flight that it would have to spare)
            assert c.drain_evicted().tolist() == ora.drain_evicted().tolist(), (step, op)
            for i in range(10):
                s = ora.find(i)
                if s < 0:
                    assert _status(lambda: c.find_slot(i)) == lmc.LMC_ERR_MISS, (step, i)
                else:
                    assert c.find_slot(i) == s, (step, i)
                    assert np.array_equal(c.get_host(i), ora.slot_bytes(s)), (step, op, i)
            if len(keep) > 8:
                keep = keep[-4:]
        st = c.get_stats()
        assert st["pool_slots_used"] == ora.used()
        assert (st["chunks_evicted"] > 5) == (flags == "evict")
    ora.close()
