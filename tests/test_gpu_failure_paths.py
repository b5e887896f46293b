"""Error paths and waiting, on the GPU, through the C ABI.

A HIP call that fails in the middle of a store or retrieve must leave lookup, pool slots
and later calls consistent with the CPU oracle (whose store never fails): nothing the
failed call admitted stays behind, and the same call made again gives the oracle's
result.  The failures are injected on the host (lmc_tune "fail_hip_after": the n-th
checked HIP call is not made and counts as failed); nothing on the device goes wrong.

lmc_wait promises that the ticket named *and every earlier one* has finished, although
operations end on streams that are not ordered among each other."""
import numpy as np
import pytest

import oracle
from paper_2510_09665_amd import workloads as W

pytestmark = pytest.mark.gpu

STAGED = (("direct_store_below", 0), ("direct_retrieve_below", 0))


def _setup(n_chunks, L=2, rng_stream=21):
    import torch
    from gpu_util import PagedKV, slots_to_device
    from paper_2510_09665_amd import lmc
    g = W.geometry("llama3_8b", L=L, NB=1024)                 # 2 MiB chunks at L=2
    seq = W.sequence("llama3_8b", g, n_tokens=n_chunks * g.CT, stream=rng_stream)
    rng = W.rng_for("llama3_8b", stream=rng_stream)
    src = PagedKV(g, seq["store_blocks"], rng)
    d_store, d_load = slots_to_device(seq["store_slots"]), slots_to_device(seq["load_slots"])
    return lmc, torch, g, seq, src, d_store, d_load


def _expect_oracle_state(c, g, seq, src, d_load, ids, pool_chunks):
    """Retrieve into fresh pages and compare pool slots, pool bytes and pages with the
    oracle's single, successful store."""
    import torch
    from gpu_util import PagedKV, assert_layers_equal
    ora = oracle.OracleStore(src.gc, pool_chunks)
    rc, n_new = ora.store(src.host, src.compact_slots(seq["store_slots"]), ids)
    assert (rc, n_new) == (0, len(ids))
    dst = PagedKV(g, seq["load_blocks"], fill="sentinel")
    c.wait(c.retrieve(ids, d_load, dst.dev, torch.cuda.current_stream()))
    torch.cuda.synchronize()
    for k, i in enumerate(ids.tolist()):
        assert c.find_slot(i) == ora.find(i)
        assert np.array_equal(c.get_host(i), ora.slot_bytes(ora.find(i))), "pool chunk %d" % k
        oracle.scatter_chunk(dst.gc, ora.slot_bytes(ora.find(i)),
                             dst.compact_slots(seq["load_slots"][k * g.CT:(k + 1) * g.CT]), dst.host)
    assert_layers_equal(dst.device_blocks_to_host(), dst.host, "retrieve after a failed and a repeated store")
    assert dst.untracked_blocks_untouched()
    ora.close()


@pytest.mark.parametrize("mode", ["staged", "direct", "staged_traced"])
def test_store_that_fails_at_any_hip_call_leaves_nothing_behind(mode):
    n = 5
    lmc, torch, g, seq, src, d_store, d_load = _setup(n)
    stream = torch.cuda.current_stream()
    with lmc.Context(g, (n + 2) * g.chunk_bytes, staging_chunks=2) as c:
        if mode != "direct":
            for k, v in STAGED:
                c.tune(k, v)
        if mode == "staged_traced":
            c.tune("trace", 1)                    # the trace's event markers are HIP calls that can fail too
        ids = c.hash_chunks(seq["tokens"])
        failures = 0
        for nth in range(1, 200):
            c.tune("fail_hip_after", nth)
            try:
                t = c.store(src.dev, d_store, ids, stream)
            except lmc.LMCError as e:
                assert e.status == lmc.LMC_ERR_HIP, e
                failures += 1
                # nothing of the failed call is visible, no slot is held, nothing is in flight
                assert c.lookup(ids) == 0
                st = c.get_stats()
                assert st["pool_slots_used"] == 0 and st["chunks_stored"] == 0
                c.wait()
                c.clear(ids)                      # would answer BUSY if a count had leaked
                continue
            c.tune("fail_hip_after", 0)
            c.wait(t)
            break
        else:
            raise AssertionError("the store never got through")
        # one launch without staging is four checked calls; three staged groups are over a dozen
        assert failures >= (3 if mode == "direct" else 12), failures
        _expect_oracle_state(c, g, seq, src, d_load, ids, n + 2)


@pytest.mark.parametrize("traced", [False, True])
def test_retrieve_that_fails_midway_holds_no_counts_and_can_be_repeated(traced):
    n = 5
    lmc, torch, g, seq, src, d_store, d_load = _setup(n, rng_stream=22)
    from gpu_util import PagedKV
    stream = torch.cuda.current_stream()
    with lmc.Context(g, n * g.chunk_bytes, staging_chunks=2) as c:
        for k, v in STAGED:
            c.tune(k, v)
        if traced:
            c.tune("trace", 1)
        ids = c.hash_chunks(seq["tokens"])
        c.wait(c.store(src.dev, d_store, ids, stream))
        scratch_pages = PagedKV(g, seq["load_blocks"], fill="sentinel")
        failures = 0
        for nth in range(1, 200):
            c.tune("fail_hip_after", nth)
            try:
                t = c.retrieve(ids, d_load, scratch_pages.dev, stream)
            except lmc.LMCError as e:
                assert e.status == lmc.LMC_ERR_HIP, e
                failures += 1
                assert c.lookup(ids) == n         # the stored chunks are unharmed
                continue
            c.tune("fail_hip_after", 0)
            c.wait(t)
            break
        else:
            raise AssertionError("the retrieve never got through")
        assert failures >= 5, failures
        # no in-flight count leaked: every chunk can be cleared; then the whole cycle again
        c.wait()
        c.clear(ids)
        assert c.get_stats()["pool_slots_used"] == 0
        c.wait(c.store(src.dev, d_store, ids, stream))
        _expect_oracle_state(c, g, seq, src, d_load, ids, n)


def test_layerwise_store_that_fails_is_taken_back_as_a_whole():
    n = 3
    lmc, torch, g, seq, src, d_store, d_load = _setup(n, L=4, rng_stream=23)
    stream = torch.cuda.current_stream()
    with lmc.Context(g, n * g.chunk_bytes, staging_chunks=2) as c:
        ids = c.hash_chunks(seq["tokens"])
        failures = 0
        for nth in range(1, 200):
            t = c.store_begin(d_store, ids, stream)
            try:
                for l in range(g.L):
                    if l == 2:
                        c.tune("fail_hip_after", nth)   # layers 0 and 1 are on their way already
                    c.store_layers(t, l, 1, src.dev, stream)
            except lmc.LMCError as e:
                assert e.status == lmc.LMC_ERR_HIP, e
                failures += 1
                assert c.lookup(ids) == 0 and c.get_stats()["pool_slots_used"] == 0
                c.wait()
                continue
            c.tune("fail_hip_after", 0)
            c.wait(t)
            break
        else:
            raise AssertionError("the layer-wise store never got through")
        assert failures >= 3, failures
        _expect_oracle_state(c, g, seq, src, d_load, ids, n)


def test_wait_covers_earlier_tickets_that_end_on_other_streams():
    """A large staged store (ends on the D2H stream), then a small store without staging
    (ends on the gather stream) and a retrieve of other chunks (ends on the scatter
    stream).  Waiting for the newest ticket, or for everything, must cover the large
    store as well."""
    n_big = 24
    lmc, torch, g, seq, src, d_store, d_load = _setup(n_big + 1, L=8, rng_stream=24)   # 8 MiB chunks
    from gpu_util import PagedKV, slots_to_device
    stream = torch.cuda.current_stream()
    CT = g.CT
    with lmc.Context(g, (n_big + 3) * g.chunk_bytes, staging_chunks=4) as c:
        c.tune("direct_store_below", 16 << 20)
        ids = c.hash_chunks(seq["tokens"])
        other = np.array([0xABCDEF], dtype=np.uint64)
        c.put_host(other, np.zeros(g.chunk_bytes, dtype=np.uint8))
        dst = PagedKV(g, seq["load_blocks"][:CT // g.BS], fill="sentinel")
        d_one = slots_to_device(seq["load_slots"][:CT])
        for how in ("newest", "everything"):
            t_big = c.store(src.dev, d_store[:n_big * CT], ids[:n_big], stream)        # 192 MiB, staged
            t_small = c.store(src.dev, d_store[n_big * CT:], ids[n_big:], stream)      # 8 MiB, no staging
            t_load = c.retrieve(other, d_one, dst.dev, stream)
            assert t_big < t_small < t_load
            c.wait(t_load if how == "newest" else 0)
            assert c.test(t_big) and c.test(t_small) and c.test(t_load), how
            c.clear(ids)                           # BUSY if the large store were still in flight
        c.clear(other)
        c.wait(c.store(src.dev, d_store, ids, stream))
        _expect_oracle_state(c, g, seq, src, d_load, ids, n_big + 3)
