"""Where the library's streams sit and how a call ties in the caller's stream (paper
section 5.1: the kernels of one group overlap the transfers of another, and stores and
loads run in parallel).  None of it may change a byte: every case is checked against the
CPU oracle."""
import numpy as np
import pytest

import oracle
from paper_2510_09665_amd import workloads as W

pytestmark = pytest.mark.gpu


def _lmc():
    from paper_2510_09665_amd import lmc
    return lmc


def _geom():
    # 8 MiB chunks: pool and staging buffers are large enough for lmc_create to arrange the streams
    return W.geometry("llama3_8b", L=8, NB=2048)


@pytest.mark.parametrize("keep", [False, True])
def test_streams_arranged_or_as_created_same_bytes(keep):
    from test_gpu_store_retrieve import _run_sequence
    lmc = _lmc()
    st = _run_sequence("llama3_8b", geom=_geom(), n_tokens=12 * 256, staging_chunks=2,
                       flags=lmc.LMC_FLAG_KEEP_STREAMS if keep else 0)
    assert st["gather_launches"] >= 6


def _two_requests(g, rng, n):
    from gpu_util import PagedKV
    bpc = g.CT // g.BS
    blocks = rng.permutation(g.NB)
    src_a = PagedKV(g, blocks[:n * bpc], rng)
    src_b = PagedKV(g, blocks[n * bpc:2 * n * bpc], rng)
    dst_b = PagedKV(g, blocks[2 * n * bpc:3 * n * bpc], fill="sentinel")
    sa = W.slots_from_blocks(g, src_a.blocks, n * g.CT)
    sb = W.slots_from_blocks(g, src_b.blocks, n * g.CT)
    tb = W.slots_from_blocks(g, dst_b.blocks, n * g.CT)
    return src_a, src_b, dst_b, sa, sb, tb


def _check_two_requests(c, g, n, ids_a, src_a, src_b, dst_b, sa, sb, tb):
    from gpu_util import assert_layers_equal
    for i, s in zip(ids_a.tolist(), src_a.compact_slots(sa).reshape(n, g.CT)):
        assert np.array_equal(c.get_host(i), oracle.gather_chunk(src_a.gc, src_a.host, s))
    for s, t in zip(src_b.compact_slots(sb).reshape(n, g.CT), dst_b.compact_slots(tb).reshape(n, g.CT)):
        oracle.scatter_chunk(dst_b.gc, oracle.gather_chunk(src_b.gc, src_b.host, s), t, dst_b.host)
    assert_layers_equal(dst_b.device_blocks_to_host(), dst_b.host)
    assert dst_b.untracked_blocks_untouched()


@pytest.mark.parametrize("fragmented", [False, True])
@pytest.mark.parametrize("order", ["store_first", "retrieve_first"])
def test_store_and_retrieve_issued_together_from_one_stream(order, fragmented):
    """Both directions in flight from one caller's stream, in either order of issue; with a
    fragmented pool the second copy streams come into play for the call issued first and
    are left out for the one that finds the other direction busy."""
    import torch
    from gpu_util import slots_to_device
    lmc = _lmc()
    g = _geom()
    n = 10
    src_a, src_b, dst_b, sa, sb, tb = _two_requests(g, np.random.default_rng(77), n)
    ids_a = np.arange(1, n + 1, dtype=np.uint64)
    ids_b = np.arange(101, n + 101, dtype=np.uint64)
    stream = torch.cuda.Stream()        # not the null stream: when it is idle, no event is recorded on it
    with lmc.Context(g, (4 * n + 1) * g.chunk_bytes, staging_chunks=2, flags=lmc.LMC_FLAG_POISON_STAGING) as c:
        for key in ("direct_store_below", "direct_retrieve_below"):
            c.tune(key, 0)
        if fragmented:      # every other slot taken: no two chunks of a request are neighbours
            filler = np.arange(1, 4 * n + 1, dtype=np.uint64) + np.uint64(1 << 40)
            zero = np.zeros(g.chunk_bytes, dtype=np.uint8)
            for f in filler:
                c.put_host([f], zero)
            c.clear(filler[1::2])
        d_sa, d_sb, d_tb = slots_to_device(sa), slots_to_device(sb), slots_to_device(tb)
        torch.cuda.synchronize()            # pages and mappings were made on PyTorch's stream
        c.wait(c.store(src_b.dev, d_sb, ids_b, stream))
        if fragmented:
            assert [c.find_slot(i) for i in ids_b[:3]] == [1, 3, 5]
        for _ in range(2):
            c.clear(ids_a)
            if order == "store_first":
                t1 = c.store(src_a.dev, d_sa, ids_a, stream)
                t2 = c.retrieve(ids_b, d_tb, dst_b.dev, stream)
            else:
                t2 = c.retrieve(ids_b, d_tb, dst_b.dev, stream)
                t1 = c.store(src_a.dev, d_sa, ids_a, stream)
            c.wait(t1)
            c.wait(t2)
        torch.cuda.synchronize()
        _check_two_requests(c, g, n, ids_a, src_a, src_b, dst_b, sa, sb, tb)


def test_rearranging_the_streams_needs_an_idle_context():
    import torch
    from gpu_util import slots_to_device
    lmc = _lmc()
    g = _geom()
    n = 6
    src_a, src_b, dst_b, sa, sb, tb = _two_requests(g, np.random.default_rng(78), n)
    ids_a = np.arange(1, n + 1, dtype=np.uint64)
    ids_b = np.arange(101, n + 101, dtype=np.uint64)
    stream = torch.cuda.current_stream()
    keep = [torch.cuda.Stream() for _ in range(3)]      # the process makes streams of its own in between
    with lmc.Context(g, 2 * n * g.chunk_bytes, staging_chunks=2) as c:
        d_sa, d_sb, d_tb = slots_to_device(sa), slots_to_device(sb), slots_to_device(tb)
        t = c.store(src_b.dev, d_sb, ids_b, stream)
        with pytest.raises(lmc.LMCError) as e:
            c.tune("arrange_streams", 1)
        assert e.value.status == lmc.LMC_ERR_BUSY
        c.wait(t)
        c.tune("arrange_streams", 1)
        with pytest.raises(lmc.LMCError):
            c.tune("arrange_streams", 2)
        t1 = c.store(src_a.dev, d_sa, ids_a, stream)
        t2 = c.retrieve(ids_b, d_tb, dst_b.dev, stream)
        c.wait(t1)
        c.wait(t2)
        torch.cuda.synchronize()
        _check_two_requests(c, g, n, ids_a, src_a, src_b, dst_b, sa, sb, tb)
    del keep


def test_work_pending_on_the_callers_stream_is_waited_for():
    """A store reads what work already on the caller's stream produces, a retrieve does not
    overwrite pages that such work still reads; a stream with nothing pending is not waited
    for at all (every other test).  The caller's stream is kept busy with dense products in
    front of the copy that puts the payload into the pages."""
    import torch
    from gpu_util import PagedKV, assert_layers_equal, slots_to_device
    lmc = _lmc()
    g = _geom()
    n = 4
    rng = np.random.default_rng(79)
    bpc = g.CT // g.BS
    blocks = rng.permutation(g.NB)
    src = PagedKV(g, blocks[:n * bpc], rng)
    dst = PagedKV(g, blocks[n * bpc:2 * n * bpc], fill="sentinel")
    ss = W.slots_from_blocks(g, src.blocks, n * g.CT)
    ts = W.slots_from_blocks(g, dst.blocks, n * g.CT)
    ids = np.arange(1, n + 1, dtype=np.uint64)
    s = torch.cuda.Stream()
    a = torch.randn(4096, 4096, device="cuda", dtype=torch.bfloat16)
    late = [d.clone() for d in src.dev]              # the payload, to arrive late
    for d in src.dev:
        d.zero_()
    copy_of_dst = [torch.empty_like(d) for d in dst.dev]
    torch.cuda.synchronize()
    with lmc.Context(g, n * g.chunk_bytes, staging_chunks=2) as c:
        d_ss, d_ts = slots_to_device(ss), slots_to_device(ts)
        torch.cuda.synchronize()
        with torch.cuda.stream(s):
            for _ in range(40):
                a = (a @ a).clamp_(-1, 1)
            for d, p in zip(src.dev, late):
                d.copy_(p, non_blocking=True)
        assert not s.query()
        t = c.store(src.dev, d_ss, ids, s)
        c.wait(t)
        for i, sl in zip(ids.tolist(), src.compact_slots(ss).reshape(n, g.CT)):
            assert np.array_equal(c.get_host(i), oracle.gather_chunk(src.gc, src.host, sl)), "store ran ahead"
        # retrieve: the caller's stream first takes a copy of the destination pages, late
        with torch.cuda.stream(s):
            for _ in range(40):
                a = (a @ a).clamp_(-1, 1)
            for d, p in zip(dst.dev, copy_of_dst):
                p.copy_(d, non_blocking=True)
        assert not s.query()
        c.wait(c.retrieve(ids, d_ts, dst.dev, s))
        torch.cuda.synchronize()
        for l, p in enumerate(copy_of_dst):
            assert bool((p == p[0]).all()), "retrieve overwrote pages the caller's stream was still reading"
        for sl, tl in zip(src.compact_slots(ss).reshape(n, g.CT), dst.compact_slots(ts).reshape(n, g.CT)):
            oracle.scatter_chunk(dst.gc, oracle.gather_chunk(src.gc, src.host, sl), tl, dst.host)
        assert_layers_equal(dst.device_blocks_to_host(), dst.host)


def test_retrieve_that_does_not_make_the_callers_stream_wait():
    import torch
    from gpu_util import PagedKV, assert_layers_equal, slots_to_device
    lmc = _lmc()
    g = _geom()
    n = 6
    rng = np.random.default_rng(80)
    bpc = g.CT // g.BS
    blocks = rng.permutation(g.NB)
    src = PagedKV(g, blocks[:n * bpc], rng)
    dst = PagedKV(g, blocks[n * bpc:2 * n * bpc], fill="sentinel")
    ss = W.slots_from_blocks(g, src.blocks, n * g.CT)
    ts = W.slots_from_blocks(g, dst.blocks, n * g.CT)
    ids = np.arange(1, n + 1, dtype=np.uint64)
    stream = torch.cuda.current_stream()
    with lmc.Context(g, n * g.chunk_bytes, staging_chunks=2) as c:
        c.tune("caller_waits", 0)
        d_ss, d_ts = slots_to_device(ss), slots_to_device(ts)
        c.wait(c.store(src.dev, d_ss, ids, stream))
        c.wait(c.retrieve(ids, d_ts, dst.dev, stream))     # the host wait is the only ordering
        for sl, tl in zip(src.compact_slots(ss).reshape(n, g.CT), dst.compact_slots(ts).reshape(n, g.CT)):
            oracle.scatter_chunk(dst.gc, oracle.gather_chunk(src.gc, src.host, sl), tl, dst.host)
        assert_layers_equal(dst.device_blocks_to_host(), dst.host)


@pytest.mark.parametrize("at_create", [True, False])
def test_trace_has_one_record_per_step_in_dependency_order(at_create):
    """LMC_FLAG_TRACE: one record per gather launch, per group's copies each way and per
    scatter launch; a group's copy begins after its gather has ended, its scatter after its
    copy; the bytes add up to the payload; the data is what it is without the trace."""
    import torch
    from gpu_util import PagedKV, assert_layers_equal, slots_to_device
    lmc = _lmc()
    g = _geom()
    n, per = 9, 2
    rng = np.random.default_rng(81)
    bpc = g.CT // g.BS
    blocks = rng.permutation(g.NB)
    src = PagedKV(g, blocks[:n * bpc], rng)
    dst = PagedKV(g, blocks[n * bpc:2 * n * bpc], fill="sentinel")
    ss = W.slots_from_blocks(g, src.blocks, n * g.CT)
    ts = W.slots_from_blocks(g, dst.blocks, n * g.CT)
    ids = np.arange(1, n + 1, dtype=np.uint64)
    stream = torch.cuda.current_stream()
    with lmc.Context(g, n * g.chunk_bytes, staging_chunks=per, flags=lmc.LMC_FLAG_TRACE if at_create else 0) as c:
        for key in ("direct_store_below", "direct_retrieve_below"):
            c.tune(key, 0)
        if not at_create:
            assert c.trace_read()[0] == []
            c.tune("trace", 1)
        d_ss, d_ts = slots_to_device(ss), slots_to_device(ts)
        t1 = c.store(src.dev, d_ss, ids, stream)
        c.wait(t1)
        t2 = c.retrieve(ids, d_ts, dst.dev, stream)
        c.wait(t2)
        recs, dropped = c.trace_read()
        assert dropped == 0
        by_stage = {s: [r for r in recs if r["stage"] == s] for s in range(4)}
        # edge groups of one chunk at the exposed ends: 1 + 4 x 2 chunks for the store, 4 x 2 + 1 for the retrieve
        assert [r["chunks"] for r in by_stage[lmc.LMC_STAGE_GATHER]] == [1, 2, 2, 2, 2]
        assert [r["chunks"] for r in by_stage[lmc.LMC_STAGE_D2H]] == [1, 2, 2, 2, 2]
        assert [r["chunks"] for r in by_stage[lmc.LMC_STAGE_H2D]] == [2, 2, 2, 2, 1]
        assert [r["chunks"] for r in by_stage[lmc.LMC_STAGE_SCATTER]] == [2, 2, 2, 2, 1]
        for s in range(4):
            assert sum(r["bytes"] for r in by_stage[s]) == n * g.chunk_bytes
            assert all(r["ticket"] == (t1 if s < 2 else t2) for r in by_stage[s])
            assert all(0 <= r["begin_us"] < r["end_us"] for r in by_stage[s])
        for k_, d in zip(by_stage[lmc.LMC_STAGE_GATHER], by_stage[lmc.LMC_STAGE_D2H]):
            assert d["begin_us"] >= k_["end_us"] - 1.0        # the copy waits for its gather (1 us of clock slack)
        for h, k_ in zip(by_stage[lmc.LMC_STAGE_H2D], by_stage[lmc.LMC_STAGE_SCATTER]):
            assert k_["begin_us"] >= h["end_us"] - 1.0        # the scatter waits for its copy
        assert by_stage[lmc.LMC_STAGE_H2D][0]["begin_us"] >= by_stage[lmc.LMC_STAGE_D2H][-1]["end_us"] - 1.0
        # nothing left, and off means off
        assert c.trace_read()[0] == []
        c.tune("trace", 0)
        c.wait(c.retrieve(ids, d_ts, dst.dev, stream))
        assert c.trace_read()[0] == []
        for i, sl in zip(ids.tolist(), src.compact_slots(ss).reshape(n, g.CT)):
            assert np.array_equal(c.get_host(i), oracle.gather_chunk(src.gc, src.host, sl))
        for sl, tl in zip(src.compact_slots(ss).reshape(n, g.CT), dst.compact_slots(ts).reshape(n, g.CT)):
            oracle.scatter_chunk(dst.gc, oracle.gather_chunk(src.gc, src.host, sl), tl, dst.host)
        assert_layers_equal(dst.device_blocks_to_host(), dst.host)


def _hip():
    import ctypes
    with open("/proc/self/maps") as maps:
        for line in maps:
            if "libamdhip64" in line:
                hip = ctypes.CDLL(line.split()[-1])
                vp = ctypes.c_void_p
                hip.hipStreamCreateWithFlags.argtypes = [ctypes.POINTER(vp), ctypes.c_uint]
                hip.hipStreamQuery.argtypes = [vp]
                hip.hipStreamSynchronize.argtypes = [vp]
                hip.hipStreamDestroy.argtypes = [vp]
                return hip
    pytest.skip("HIP runtime not found in this process")


def test_null_stream_as_the_callers_stream_covers_blocking_streams():
    """A caller that names the null stream relies on its legacy meaning: work recorded there
    waits for what every blocking stream of the process holds.  The KV is produced late on a
    blocking stream; lmc_store(..., NULL) must still store the produced bytes.  (The
    library records no event on an idle stream; that is safe here only because the
    runtime's query of the null stream says "not ready" while a blocking stream is busy,
    which is checked first.)"""
    import ctypes
    import torch
    from gpu_util import PagedKV, slots_to_device
    lmc = _lmc()
    hip = _hip()
    g = _geom()
    n = 4
    rng = np.random.default_rng(82)
    bpc = g.CT // g.BS
    blocks = rng.permutation(g.NB)
    src = PagedKV(g, blocks[:n * bpc], rng)
    ss = W.slots_from_blocks(g, src.blocks, n * g.CT)
    ids = np.arange(1, n + 1, dtype=np.uint64)
    raw = ctypes.c_void_p()
    assert hip.hipStreamCreateWithFlags(ctypes.byref(raw), 0) == 0          # 0: a blocking stream
    producer = torch.cuda.ExternalStream(raw.value)
    a = torch.randn(4096, 4096, device="cuda", dtype=torch.bfloat16)
    late = [d.clone() for d in src.dev]
    for d in src.dev:
        d.zero_()
    try:
        with lmc.Context(g, n * g.chunk_bytes, staging_chunks=2) as c:
            d_ss = slots_to_device(ss)
            torch.cuda.synchronize()
            with torch.cuda.stream(producer):
                for _ in range(40):
                    a = (a @ a).clamp_(-1, 1)
                for d, p in zip(src.dev, late):
                    d.copy_(p, non_blocking=True)
            assert hip.hipStreamQuery(raw) != 0, "the producer finished too early for this test to say anything"
            assert hip.hipStreamQuery(None) != 0, "the null stream's query does not see the blocking stream"
            hip.hipGetLastError()
            t = c.store(src.dev, d_ss, ids, None)                           # NULL: the null stream
            c.wait(t)
            for i, sl in zip(ids.tolist(), src.compact_slots(ss).reshape(n, g.CT)):
                assert np.array_equal(c.get_host(i), oracle.gather_chunk(src.gc, src.host, sl)), "store ran ahead"
            torch.cuda.synchronize()
    finally:
        torch.cuda.synchronize()
        del producer
        hip.hipStreamDestroy(raw)


def test_retrieve_behind_a_store_of_the_same_chunks_follows_it_group_by_group():
    """No host wait between the store of a request and its retrieve: each group's copy to the
    device waits for the store groups that hold its chunks and for nothing more, so the
    two directions overlap (seen in the trace) and the bytes are exact."""
    import torch
    from gpu_util import PagedKV, assert_layers_equal, slots_to_device
    lmc = _lmc()
    g = _geom()
    n, per = 17, 2
    rng = np.random.default_rng(83)
    bpc = g.CT // g.BS
    blocks = rng.permutation(g.NB)
    src = PagedKV(g, blocks[:n * bpc], rng)
    dst = PagedKV(g, blocks[n * bpc:2 * n * bpc], fill="sentinel")
    ss = W.slots_from_blocks(g, src.blocks, n * g.CT)
    ts = W.slots_from_blocks(g, dst.blocks, n * g.CT)
    ids = np.arange(1, n + 1, dtype=np.uint64)
    stream = torch.cuda.Stream()
    with lmc.Context(g, n * g.chunk_bytes, staging_chunks=per, flags=lmc.LMC_FLAG_TRACE | lmc.LMC_FLAG_POISON_STAGING) as c:
        for key in ("direct_store_below", "direct_retrieve_below"):
            c.tune(key, 0)
        d_ss, d_ts = slots_to_device(ss), slots_to_device(ts)
        torch.cuda.synchronize()
        t1 = c.store(src.dev, d_ss, ids, stream)
        t2 = c.retrieve(ids, d_ts, dst.dev, stream)
        c.wait(t1)
        c.wait(t2)
        recs, _ = c.trace_read()
        d2h = [r for r in recs if r["stage"] == lmc.LMC_STAGE_D2H]
        h2d = [r for r in recs if r["stage"] == lmc.LMC_STAGE_H2D]
        assert [r["chunks"] for r in d2h] == [1] + [2] * 8 and [r["chunks"] for r in h2d] == [2] * 8 + [1]
        # chunk ranges of the groups, in order
        def ranges(rs):
            out, a = [], 0
            for r in rs:
                out.append((a, a + r["chunks"], r))
                a += r["chunks"]
            return out
        for a, b, r in ranges(h2d):
            need = max(s["end_us"] for sa, sb, s in ranges(d2h) if sa < b and a < sb)
            assert r["begin_us"] >= need - 1.0, "a group was loaded before its chunks were in the pool"
        # and it did not wait for the whole store: the first load begins before the last store copy ends
        assert h2d[0]["begin_us"] < d2h[-1]["begin_us"]
        for i, sl in zip(ids.tolist(), src.compact_slots(ss).reshape(n, g.CT)):
            assert np.array_equal(c.get_host(i), oracle.gather_chunk(src.gc, src.host, sl))
        for sl, tl in zip(src.compact_slots(ss).reshape(n, g.CT), dst.compact_slots(ts).reshape(n, g.CT)):
            oracle.scatter_chunk(dst.gc, oracle.gather_chunk(src.gc, src.host, sl), tl, dst.host)
        assert_layers_equal(dst.device_blocks_to_host(), dst.host)
        assert dst.untracked_blocks_untouched()


def test_host_reads_of_a_store_under_way_are_exact_chunk_by_chunk():
    """lmc_get_host behind an unfinished store waits for the group of copies that brings in
    the chunk it asks for; every chunk read that way, in order, with no lmc_wait, is exact."""
    import torch
    from gpu_util import PagedKV, slots_to_device
    lmc = _lmc()
    g = _geom()
    n = 17
    rng = np.random.default_rng(84)
    bpc = g.CT // g.BS
    src = PagedKV(g, rng.permutation(g.NB)[:n * bpc], rng)
    ss = W.slots_from_blocks(g, src.blocks, n * g.CT)
    ids = np.arange(1, n + 1, dtype=np.uint64)
    stream = torch.cuda.Stream()
    with lmc.Context(g, n * g.chunk_bytes, staging_chunks=2, flags=lmc.LMC_FLAG_POISON_STAGING) as c:
        c.tune("direct_store_below", 0)
        d_ss = slots_to_device(ss)
        torch.cuda.synchronize()
        t = c.store(src.dev, d_ss, ids, stream)
        for i, sl in zip(ids.tolist(), src.compact_slots(ss).reshape(n, g.CT)):
            assert np.array_equal(c.get_host(i), oracle.gather_chunk(src.gc, src.host, sl)), "chunk %d" % i
        c.wait(t)
