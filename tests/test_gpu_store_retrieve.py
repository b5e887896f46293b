"""GPU parity of the whole path (hash -> lookup -> store -> retrieve, paper sections 4
and 5.1) against the CPU oracle on the benchmark configurations, byte for byte, plus
the pipeline's hazards and error paths.  Everything goes through the C ABI."""
import numpy as np
import pytest

import oracle
from paper_2510_09665_amd import workloads as W

pytestmark = pytest.mark.gpu


def _lmc():
    from paper_2510_09665_amd import lmc
    return lmc


STAGED = (("direct_store_below", 0), ("direct_retrieve_below", 0))


def _run_sequence(name, geom=None, flags=0, num_staging=2, staging_chunks=1, n_tokens=None,
                  pool_chunks=None, tune=(), size_rule=False):
    """Store a whole request, retrieve it into fresh blocks, compare pool and pages.
    Unless size_rule is set the request goes through the staging rings whatever its size
    (most cases here are kept small to be quick, and it is the pipeline they are after)."""
    if not size_rule:
        tune = STAGED + tuple(tune)
    import torch
    from gpu_util import PagedKV, assert_layers_equal, slots_to_device
    lmc = _lmc()
    g = geom or W.geometry(name)
    seq = W.sequence(name, g, n_tokens=n_tokens)
    rng = W.rng_for(name, stream=1)
    src = PagedKV(g, seq["store_blocks"], rng)
    dst = PagedKV(g, seq["load_blocks"], fill="sentinel")
    n_chunks = seq["tokens"].size // g.CT
    pool_chunks = pool_chunks or n_chunks
    stream = torch.cuda.current_stream()
    with lmc.Context(g, pool_chunks * g.chunk_bytes, num_staging=num_staging,
                     staging_chunks=staging_chunks, flags=flags | lmc.LMC_FLAG_TIMING) as c:
        for key, value in tune:
            c.tune(key, value)
        ids = c.hash_chunks(seq["tokens"])
        assert np.array_equal(ids, oracle.hash_chunks(seq["tokens"], g.CT, 0))
        assert c.lookup(ids) == 0
        # the slot mappings must stay alive until lmc_wait: keep the tensors referenced
        d_store, d_load = slots_to_device(seq["store_slots"]), slots_to_device(seq["load_slots"])
        t = c.store(src.dev, d_store, ids, stream)
        assert c.lookup(ids) == n_chunks          # visible at once
        # retrieve is enqueued without waiting for the store: ordered on the device
        t2 = c.retrieve(ids, d_load, dst.dev, stream)
        c.wait(t)
        c.wait(t2)
        torch.cuda.synchronize()

        ora = oracle.OracleStore(src.gc, pool_chunks)
        rc, n_new = ora.store(src.host, src.compact_slots(seq["store_slots"]), ids)
        assert (rc, n_new) == (0, n_chunks)
        for i in ids.tolist():                    # pool image: same slot, same bytes
            assert c.find_slot(i) == ora.find(i)
            assert np.array_equal(c.get_host(i), ora.slot_bytes(ora.find(i))), "pool chunk"
        # the oracle retrieves from its own pool into the compact destination
        for k, i in enumerate(ids.tolist()):
            oracle.scatter_chunk(dst.gc, ora.slot_bytes(ora.find(i)),
                                 dst.compact_slots(seq["load_slots"][k * g.CT:(k + 1) * g.CT]),
                                 dst.host)
        assert_layers_equal(dst.device_blocks_to_host(), dst.host, name + " retrieve")
        assert dst.untracked_blocks_untouched()
        assert src.untracked_blocks_untouched()
        assert_layers_equal(src.device_blocks_to_host(), src.host, name + " source unchanged")
        st = c.get_stats()
        assert st["chunks_stored"] == n_chunks and st["chunks_retrieved"] == n_chunks
        assert st["bytes_d2h"] == st["bytes_h2d"] == n_chunks * g.chunk_bytes
        assert st["timed_gather_launches"] == st["gather_launches"] > 0
        assert st["gather_ms"] > 0 and st["scatter_ms"] > 0
        ora.close()
        return st


def test_config1_tiny():
    # half a MiB: by the library's size rule both directions skip staging ...
    st = _run_sequence("tiny", size_rule=True)
    assert st["gather_launches"] == 1 and st["scatter_launches"] == 1
    # ... and with the rule switched off the same bytes come through the staging ring
    _run_sequence("tiny")
    # 12 chunks of 4 MiB are still below the threshold: one launch each way
    st = _run_sequence("llama3_8b", W.geometry("llama3_8b", L=4, NB=1024), n_tokens=12 * 256, size_rule=True)
    assert st["gather_launches"] == 1 and st["scatter_launches"] == 1


def test_small_direct_and_large_staged_calls_interleaved_without_waiting():
    """Calls below the size threshold skip staging, larger ones use it; they end on
    different streams.  A retrieve enqueued right behind both kinds of store must see
    both complete, and a small retrieve must be ordered behind a large store."""
    import torch
    from gpu_util import PagedKV, assert_layers_equal, slots_to_device
    lmc = _lmc()
    g = W.geometry("llama3_8b", L=2, NB=1024)                # 2 MiB chunks
    rng = np.random.default_rng(11)
    n_big, n_small = 12, 1
    n = n_big + n_small
    blocks = rng.permutation(g.NB)
    bpc = g.CT // g.BS
    sb, lb = blocks[:n * bpc], blocks[n * bpc:2 * n * bpc]
    src = PagedKV(g, sb, rng)
    toks = W.tokens_for(rng, n * g.CT)
    s_slots = W.slots_from_blocks(g, sb, n * g.CT)
    l_slots = W.slots_from_blocks(g, lb, n * g.CT)
    stream = torch.cuda.current_stream()
    for rep in range(3):
        dst = PagedKV(g, lb, fill="sentinel")
        with lmc.Context(g, n * g.chunk_bytes, staging_chunks=2, flags=lmc.LMC_FLAG_POISON_STAGING) as c:
            c.tune("direct_store_below", 4 << 20)
            c.tune("direct_retrieve_below", 2 << 20)
            ids = c.hash_chunks(toks)
            d_s, d_l = slots_to_device(s_slots), slots_to_device(l_slots)
            cut = n_big * g.CT
            # 24 MiB through staging (gather stream, then D2H stream) ...
            c.store(src.dev, d_s[:cut], ids[:n_big], stream)
            # ... and 2 MiB written by the gather kernel itself, which finishes first
            c.store(src.dev, d_s[cut:], ids[n_big:], stream)
            st = c.get_stats()
            assert st["gather_launches"] == 1 + 6 + 1 and st["bytes_d2h"] == n * g.chunk_bytes
            if rep == 0:
                t = c.retrieve(ids, d_l, dst.dev, stream)            # staged; needs both stores
            elif rep == 1:
                c.retrieve(ids[n_big:], d_l[cut:], dst.dev, stream)  # direct; behind the direct store
                t = c.retrieve(ids[:n_big], d_l[:cut], dst.dev, stream)
            else:
                c.retrieve(ids[:1], d_l[:g.CT], dst.dev, stream)     # direct; behind the staged store
                t = c.retrieve(ids[1:], d_l[g.CT:], dst.dev, stream)
            c.wait(t)
            c.wait()
            torch.cuda.synchronize()
            chunks = oracle.gather(src.gc, src.host, src.compact_slots(s_slots))
            oracle.scatter(dst.gc, chunks, dst.compact_slots(l_slots), dst.host)
            for k, i in enumerate(ids.tolist()):
                assert np.array_equal(c.get_host(i), chunks[k]), "pool chunk %d" % k
            assert_layers_equal(dst.device_blocks_to_host(), dst.host, "rep %d" % rep)


def test_config2_llama3_8b_full():
    st = _run_sequence("llama3_8b", staging_chunks=4)
    # 16 chunks: a single-chunk group at the exposed end of each pipeline, then groups of 4
    assert st["gather_launches"] == 1 + 4 and st["scatter_launches"] == 4 + 1


def test_config2_llama3_8b_full_in_the_benchmarks_launch_configuration():
    # bench.py's defaults: two staging buffers of 16 chunks -> launches of 1 and 15 chunks
    st = _run_sequence("llama3_8b", staging_chunks=16, num_staging=2)
    assert st["gather_launches"] == 2 and st["scatter_launches"] == 2
    # the copy-engine guard is on by default: the 480 MiB copy to the host is timed; nothing is wrong with it
    assert 10.0 < st["d2h_copy_best_gbps"] < 80.0 and st["d2h_guard_switches"] == 0
    # switched off, no copy is watched
    st = _run_sequence("llama3_8b", staging_chunks=16, num_staging=2, tune=(("d2h_guard", 0),))
    assert st["d2h_copy_best_gbps"] == 0.0


def test_config5_mla_bf16_full():
    _run_sequence("mla_bf16", staging_chunks=2)
    # bench.py's launch configuration for this shape: the whole request fits one staging buffer
    st = _run_sequence("mla_bf16", staging_chunks=32)
    assert st["gather_launches"] == 2 and st["scatter_launches"] == 2


def test_config5_mla_fp8_full():
    _run_sequence("mla_fp8", staging_chunks=3)      # 32 chunks in groups of 3: ragged last group
    st = _run_sequence("mla_fp8", staging_chunks=32)    # as bench.py launches it
    assert st["gather_launches"] == 2 and st["scatter_launches"] == 2


@pytest.mark.parametrize("flags", ["poison", "force_sync", "validate", "direct"])
def test_pipeline_modes_give_identical_results(flags):
    lmc = _lmc()
    f = {"poison": lmc.LMC_FLAG_POISON_STAGING, "force_sync": lmc.LMC_FLAG_FORCE_SYNC,
         "validate": lmc.LMC_FLAG_VALIDATE_SLOTS, "direct": lmc.LMC_FLAG_DIRECT}[flags]
    # 24 chunks through a ring of 2 single-chunk buffers: every buffer is reused 12 times
    g = W.geometry("llama3_8b", L=4, NB=1024)
    _run_sequence("llama3_8b", g, flags=f, n_tokens=24 * 256)
    _run_sequence("llama3_8b", g, flags=f, n_tokens=24 * 256, num_staging=3, staging_chunks=5)


@pytest.mark.parametrize("engines", [1, 2, 3])
def test_own_copy_kernel_instead_of_the_runtimes_copies(engines):
    """lmc_tune("copy_kernel"): the copies between staging and the pool made by the
    library's link-paced copy kernel (bit 0 to the host, bit 1 from the host)."""
    lmc = _lmc()
    t = (("copy_kernel", engines),)
    g = W.geometry("llama3_8b", L=4, NB=1024)
    _run_sequence("llama3_8b", g, flags=lmc.LMC_FLAG_POISON_STAGING, n_tokens=24 * 256, num_staging=3,
                  staging_chunks=5, tune=t)
    _run_sequence("mla_fp8", W.geometry("mla_fp8", L=7), n_tokens=6 * 256, staging_chunks=2, tune=t)
    # rows that are no multiple of 16 bytes stay with the runtime's copies
    _run_sequence("tiny", W.KVGeometry(L=3, P=2, H=3, D=7, e=2, BS=4, NB=256, CT=32), n_tokens=5 * 32,
                  staging_chunks=2, tune=t)


def test_retrieve_with_scatters_in_destination_order():
    """lmc_tune("scatter_order", 2): every scatter launch of the pipeline visits its rows in
    ascending slot order (built on the device); consecutive launches share that scratch."""
    t = (("scatter_order", 2),)
    g = W.geometry("llama3_8b", L=4, NB=1024)
    lmc = _lmc()
    _run_sequence("llama3_8b", g, flags=lmc.LMC_FLAG_POISON_STAGING, n_tokens=24 * 256, num_staging=3,
                  staging_chunks=5, tune=t)
    _run_sequence("mla_fp8", W.geometry("mla_fp8", L=7), n_tokens=6 * 256, staging_chunks=2, tune=t)
    _run_sequence("llama3_8b", W.geometry("llama3_8b", L=6, NB=512, layout="HND"), n_tokens=8 * 256,
                  staging_chunks=3, tune=t)


def test_direct_mode_full_size_config2_and_mla():
    """LMC_FLAG_DIRECT: the kernels read and write the pinned pool themselves."""
    lmc = _lmc()
    _run_sequence("llama3_8b", flags=lmc.LMC_FLAG_DIRECT, staging_chunks=1)
    _run_sequence("mla_fp8", flags=lmc.LMC_FLAG_DIRECT, staging_chunks=1)


def test_hnd_layout_through_the_pipeline():
    g = W.geometry("llama3_8b", L=6, NB=512, layout="HND")
    _run_sequence("llama3_8b", g, n_tokens=8 * 256, staging_chunks=3)


def test_blocks_outermost_page_order_through_the_pipeline():
    # [NB][P][BS][H][D]: the K and the V page of a block are neighbours (64 KiB apart per block)
    g = W.geometry("llama3_8b", L=6, NB=512, order="NP")
    assert g.plane_stride == 32768 and g.block_stride == 65536
    _run_sequence("llama3_8b", g, n_tokens=8 * 256, staging_chunks=3)
    _run_sequence("llama3_8b", g, n_tokens=8 * 256, staging_chunks=1, flags=_lmc().LMC_FLAG_DIRECT)


@pytest.mark.parametrize("copy_kernel", [0, 3])
def test_fragmented_pool_copies_alternate_between_two_streams(copy_kernel):
    """Every other pool slot is taken, so no two new chunks are neighbours in the pool:
    each group needs one copy per chunk, and those go to two copy streams in turn (or, with
    the library's own copy kernel, follow each other on one).  Pool image and pages must
    equal the oracle's, whose store went through the same history."""
    import torch
    from gpu_util import PagedKV, assert_layers_equal, slots_to_device
    lmc = _lmc()
    name = "llama3_8b"
    g = W.geometry(name, L=4, NB=1024)                       # 4 MiB chunks
    n = 13
    seq = W.sequence(name, g, n_tokens=n * g.CT)
    rng = W.rng_for(name, stream=7)
    src = PagedKV(g, seq["store_blocks"], rng)
    dst = PagedKV(g, seq["load_blocks"], fill="sentinel")
    stream = torch.cuda.current_stream()
    n_pool = 2 * n + 2
    ora = oracle.OracleStore(src.gc, n_pool)
    filler_ids = np.arange(1, 2 * n + 1, dtype=np.uint64) + np.uint64(1 << 40)
    filler_slots = np.tile(src.compact_slots(seq["store_slots"][:g.CT]), 2 * n)
    with lmc.Context(g, n_pool * g.chunk_bytes, staging_chunks=5, num_staging=2,
                     flags=lmc.LMC_FLAG_POISON_STAGING) as c:
        c.tune("copy_kernel", copy_kernel)
        for key, value in STAGED:
            c.tune(key, value)
        # history: 2n filler chunks, then every second one removed, in both stores
        d_fill = slots_to_device(np.tile(seq["store_slots"][:g.CT], 2 * n))
        c.wait(c.store(src.dev, d_fill, filler_ids, stream))
        assert ora.store(src.host, filler_slots, filler_ids) == (0, 2 * n)
        c.clear(filler_ids[1::2])
        assert ora.clear(filler_ids[1::2]) == 0
        ids = c.hash_chunks(seq["tokens"])
        d_store, d_load = slots_to_device(seq["store_slots"]), slots_to_device(seq["load_slots"])
        t = c.store(src.dev, d_store, ids, stream)
        t2 = c.retrieve(ids, d_load, dst.dev, stream)          # behind the store, on the device
        c.wait(t)
        c.wait(t2)
        torch.cuda.synchronize()
        assert ora.store(src.host, src.compact_slots(seq["store_slots"]), ids) == (0, n)
        got_slots = [c.find_slot(i) for i in ids.tolist()]
        assert got_slots == [ora.find(i) for i in ids.tolist()]
        assert got_slots == list(range(1, 2 * n, 2))           # no two are neighbours
        for i in ids.tolist() + filler_ids[0::2].tolist():
            assert np.array_equal(c.get_host(i), ora.slot_bytes(ora.find(i))), "pool chunk"
        assert ora.retrieve(ids, dst.compact_slots(seq["load_slots"]), dst.host) == 0
        assert_layers_equal(dst.device_blocks_to_host(), dst.host, "retrieve from a fragmented pool")
        assert dst.untracked_blocks_untouched()
    ora.close()


def test_eviction_spares_chunks_with_a_transfer_in_flight():
    """LMC_FLAG_EVICT_LRU: request A (32 chunks, 512 MiB: some 9 ms on the link) is being
    retrieved when a store of 10 new chunks needs room in a full pool.  Only request B's
    8 chunks may go, tail first; A's slots are read by the retrieve and must stay, so the
    ninth new chunk finds no room.  The retrieve still delivers A's bytes."""
    import torch
    from gpu_util import PagedKV, assert_layers_equal, slots_to_device
    lmc = _lmc()
    name = "llama3_8b"
    g = W.geometry(name, L=16, NB=2048)                      # 16 MiB chunks
    nA, nB, nC = 32, 8, 10
    seq = W.sequence(name, g, n_tokens=(nA + nB + nC) * g.CT)
    rng = W.rng_for(name, stream=9)
    src = PagedKV(g, seq["store_blocks"], rng)
    dst = PagedKV(g, seq["load_blocks"][:nA * g.CT // g.BS], fill="sentinel")
    stream = torch.cuda.current_stream()
    CT = g.CT
    with lmc.Context(g, (nA + nB) * g.chunk_bytes, staging_chunks=4, flags=lmc.LMC_FLAG_EVICT_LRU) as c:
        ids = c.hash_chunks(seq["tokens"])
        idA, idB, idC = ids[:nA], ids[nA:nA + nB], ids[nA + nB:]
        d_store = slots_to_device(seq["store_slots"])
        d_load = slots_to_device(seq["load_slots"][:nA * CT])
        c.wait(c.store(src.dev, d_store[:nA * CT], idA, stream))
        c.wait(c.store(src.dev, d_store[nA * CT:(nA + nB) * CT], idB, stream))
        assert c.get_stats()["pool_slots_used"] == nA + nB
        t = c.retrieve(idA, d_load, dst.dev, stream)
        with pytest.raises(lmc.LMCError) as e:
            c.store(src.dev, d_store[(nA + nB) * CT:], idC, stream)
        if c.test(t):
            pytest.skip("the retrieve had finished before the store was admitted")
        assert e.value.status == lmc.LMC_ERR_NOMEM
        assert c.drain_evicted().tolist() == idB[::-1].tolist()       # B's tail first
        assert c.lookup(idA) == nA and c.lookup(idC) == nB and c.lookup(idB) == 0
        c.wait()
        torch.cuda.synchronize()
        chunks = oracle.gather(src.gc, src.host, src.compact_slots(seq["store_slots"]))
        oracle.scatter(dst.gc, chunks[:nA], dst.compact_slots(seq["load_slots"][:nA * CT]), dst.host)
        assert_layers_equal(dst.device_blocks_to_host(), dst.host, "retrieve that was in flight")
        for k in list(range(nA)) + list(range(nA + nB, nA + 2 * nB)):
            assert np.array_equal(c.get_host(ids[k]), chunks[k]), k
        st = c.get_stats()
        assert st["chunks_evicted"] == nB and st["pool_slots_used"] == nA + nB


def test_stored_chunks_go_to_two_directories_without_a_copy_and_come_back(tmp_path):
    """Section 5.3: chunks stored from the GPU are written to two lower-tier directories at
    once, straight from the pinned pool, right behind the store (the first count taken on a
    chunk waits for the store that fills it).  Files must equal the oracle's chunks; after
    the pool is emptied they are read back and retrieved into fresh pages."""
    import os
    import torch
    from gpu_util import PagedKV, assert_layers_equal, slots_to_device
    lmc = _lmc()
    name = "llama3_8b"
    g = W.geometry(name, L=4, NB=1024)                       # 4 MiB chunks
    n = 9
    seq = W.sequence(name, g, n_tokens=n * g.CT)
    rng = W.rng_for(name, stream=12)
    src = PagedKV(g, seq["store_blocks"], rng)
    dst = PagedKV(g, seq["load_blocks"], fill="sentinel")
    dirs = [str(tmp_path / "disk"), str(tmp_path / "remote")]
    for d in dirs:
        os.mkdir(d)
    stream = torch.cuda.current_stream()
    chunks = oracle.gather(src.gc, src.host, src.compact_slots(seq["store_slots"]))
    with lmc.Context(g, n * g.chunk_bytes, staging_chunks=2) as c, c.tier_open(dirs, n_threads=4) as t:
        ids = c.hash_chunks(seq["tokens"])
        d_store, d_load = slots_to_device(seq["store_slots"]), slots_to_device(seq["load_slots"])
        c.store(src.dev, d_store, ids, stream)
        t.write(ids)                                          # no lmc_wait in between
        t.wait()
        for d in dirs:
            for k, i in enumerate(ids.tolist()):
                got = np.fromfile(os.path.join(d, "%016x.kv" % i), dtype=np.uint8)
                assert np.array_equal(got, chunks[k]), (d, k)
        c.wait()
        c.clear(ids)
        assert c.lookup(ids) == 0 and t.lookup(1, ids) == n
        t.read(1, ids)
        c.wait(c.retrieve(ids, d_load, dst.dev, stream))
        torch.cuda.synchronize()
        oracle.scatter(dst.gc, chunks, dst.compact_slots(seq["load_slots"]), dst.host)
        assert_layers_equal(dst.device_blocks_to_host(), dst.host, "retrieve of chunks read back from a directory")
        assert t.get_stats() == dict(files_written=2 * n, bytes_written=2 * n * g.chunk_bytes, chunks_read=n)


def test_config3_llama3_70b_full_size_every_chunk_against_the_oracle():
    """Full size: 40 GiB of pages on the device, 128 chunks = 10 GiB through the pinned
    pool with the double-buffered pipeline in the launch configuration bench.py times (2
    staging buffers of 8 chunks: groups of 1, 15 x 8 and 7 chunks).  The oracle
    sees every source block (a compact host copy, payload drawn on the host) and is
    compared byte for byte with all 128 pool chunks and with every destination page;
    blocks that no slot names must still hold the sentinel."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    import torch
    from gpu_util import PagedKV, assert_layers_equal, slots_to_device
    lmc = _lmc()
    name = "llama3_70b"
    g = W.geometry(name)
    seq = W.sequence(name, g)
    n_chunks = seq["tokens"].size // g.CT
    assert n_chunks == 128 and g.chunk_bytes == 80 * 2**20
    threads = max(1, min(16, len(os.sched_getaffinity(0))))
    src = PagedKV(g, seq["store_blocks"], W.rng_for(name, stream=1), threads=threads)
    dst = PagedKV(g, seq["load_blocks"], fill="sentinel")
    s_slots = src.compact_slots(seq["store_slots"]).reshape(n_chunks, g.CT)
    l_slots = dst.compact_slots(seq["load_slots"]).reshape(n_chunks, g.CT)
    stream = torch.cuda.current_stream()
    with lmc.Context(g, n_chunks * g.chunk_bytes, staging_chunks=8, num_staging=2) as c:
        ids = c.hash_chunks(seq["tokens"])
        assert np.array_equal(ids, oracle.hash_chunks(seq["tokens"], g.CT, 0))
        d_store, d_load = slots_to_device(seq["store_slots"]), slots_to_device(seq["load_slots"])
        t = c.store(src.dev, d_store, ids, stream)
        t2 = c.retrieve(ids, d_load, dst.dev, stream)       # no host wait in between
        c.wait(t2)
        torch.cuda.synchronize()
        assert c.test(t)

        # the oracle, chunk by chunk (its C loops run outside the interpreter lock): gather
        # from the compact sources, compare with the pool, scatter into the compact host
        # image of the destination; the chunks' destination blocks are disjoint
        def one(k):
            want = oracle.gather_chunk(src.gc, src.host, s_slots[k])
            assert c.find_slot(ids[k]) == k
            assert np.array_equal(c.get_host(ids[k]), want), "pool chunk %d" % k
            oracle.scatter_chunk(dst.gc, want, l_slots[k], dst.host)
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(one, range(n_chunks)))
        assert_layers_equal(dst.device_blocks_to_host(), dst.host, "llama3_70b retrieve")
        assert dst.untracked_blocks_untouched()
        assert src.untracked_blocks_untouched()
        st = c.get_stats()
        assert st["chunks_stored"] == st["chunks_retrieved"] == n_chunks
        assert st["bytes_d2h"] == st["bytes_h2d"] == n_chunks * g.chunk_bytes
        assert st["gather_launches"] == st["scatter_launches"] == 17


def test_config4_batched_multi_request_retrieve():
    """64 requests, lognormal prefix lengths, only the leading hit chunks are loaded, in
    one lmc_retrieve_batch call; pool slots in shuffled order; every byte checked."""
    import torch
    from gpu_util import PagedKV, assert_layers_equal, slots_to_device
    lmc = _lmc()
    name = "batch_8b"
    g = W.geometry(name)
    reqs = W.request_mix(name, g)
    rng = W.rng_for(name, stream=2)
    n_hit = sum(r["n_hit"] for r in reqs)
    assert 100 < n_hit <= g.NB // (g.CT // g.BS)
    all_blocks = np.concatenate([r["load_blocks"] for r in reqs])
    dst = PagedKV(g, all_blocks, fill="sentinel")
    base = W.payload_bytes(rng, g, g.chunk_bytes).view(np.uint64)
    per = 16                                                 # chunks per launch, as bench.py runs this configuration
    with lmc.Context(g, (n_hit + 3) * g.chunk_bytes, staging_chunks=per) as c:
        ids_per_req = [c.hash_chunks(r["tokens"]) for r in reqs]
        for r, ids in zip(reqs, ids_per_req):
            assert np.array_equal(ids, oracle.hash_chunks(r["tokens"], g.CT, 0))
        # the hit chunks reach the host pool from "a lower tier", in shuffled order
        hit = [(ri, k) for ri, r in enumerate(reqs) for k in range(r["n_hit"])]
        chunk_of = {}
        for j in rng.permutation(len(hit)):
            ri, k = hit[j]
            payload = (base ^ np.uint64((ri * 1000003 + k * 7919 + 1) * 0x9E3779B97F4A7C15 % 2**64)) \
                .view(np.uint8)
            c.put_host([ids_per_req[ri][k]], payload)
            chunk_of[(ri, k)] = payload
        # scheduler side: prefix match per request
        off, ids, slots = [0], [], []
        for ri, r in enumerate(reqs):
            assert c.lookup(ids_per_req[ri]) == r["n_hit"]
            ids.append(ids_per_req[ri][:r["n_hit"]])
            slots.append(r["load_slots"])
            off.append(off[-1] + r["n_hit"])
        ids, slots = np.concatenate(ids), np.concatenate(slots)
        d_slots = slots_to_device(slots)
        t = c.retrieve_batch(off, ids, d_slots, dst.dev, torch.cuda.current_stream())
        c.wait(t)
        torch.cuda.synchronize()
        st = c.get_stats()
        assert st["chunks_retrieved"] == n_hit and st["scatter_launches"] == -(-(n_hit - 1) // per) + 1
        cs = dst.compact_slots(slots)
        j = 0
        for ri, r in enumerate(reqs):
            for k in range(r["n_hit"]):
                oracle.scatter_chunk(dst.gc, chunk_of[(ri, k)], cs[j * g.CT:(j + 1) * g.CT], dst.host)
                j += 1
        assert_layers_equal(dst.device_blocks_to_host(), dst.host, "batched retrieve")
        assert dst.untracked_blocks_untouched()
        # one missing chunk anywhere: nothing is written
        before = dst.device_blocks_to_host()
        bad_ids = ids.copy()
        bad_ids[len(bad_ids) // 2] ^= np.uint64(1)
        with pytest.raises(lmc.LMCError) as e:
            c.retrieve_batch(off, bad_ids, d_slots, dst.dev)
        assert e.value.status == lmc.LMC_ERR_MISS
        torch.cuda.synchronize()
        assert_layers_equal(dst.device_blocks_to_host(), before)


def _status(fn):
    lmc = _lmc()
    try:
        fn()
        return 0
    except lmc.LMCError as e:
        return e.status


def test_store_semantics_against_oracle_store():
    """Duplicate ids are skipped (first writer wins), lowest free slot first, NOMEM keeps
    what was stored, MISS writes nothing, pinned chunks cannot be cleared: statuses, slot
    numbers and pool bytes all equal the oracle's chunk store."""
    import torch
    from gpu_util import PagedKV, assert_layers_equal, slots_to_device
    lmc = _lmc()
    g = W.geometry("tiny")
    rng = np.random.default_rng(77)
    kv = PagedKV(g, np.arange(g.NB), rng)
    slots = rng.permutation(g.n_slots)[:4 * g.CT].reshape(4, g.CT)
    stream = torch.cuda.current_stream()
    ora = oracle.OracleStore(g, 3)

    def both_store(c, ids, sl):
        want_rc, _ = ora.store(kv.host, sl, ids)
        d_sl = slots_to_device(sl)
        got_rc = _status(lambda: c.store(kv.dev, d_sl, ids, stream))
        assert got_rc == want_rc
        c.wait()
        for i in range(1, 12):
            if ora.find(i) < 0:
                assert _status(lambda: c.find_slot(i)) == lmc.LMC_ERR_MISS
            else:
                assert c.find_slot(i) == ora.find(i)
                assert np.array_equal(c.get_host(i), ora.slot_bytes(ora.find(i))), i

    with lmc.Context(g, 3 * g.chunk_bytes) as c:
        both_store(c, [1, 2], slots[:2])
        both_store(c, [1, 3, 1], slots[1:4])          # 1 is present: other pages, not rewritten
        assert c.get_stats()["chunks_skipped_dup"] == 2
        both_store(c, [4], slots[:1])                 # pool full: NOMEM, nothing changes
        assert c.get_stats()["alloc_failures"] == 1
        assert c.clear([2]) is None and ora.clear([2]) == 0
        both_store(c, [5, 6, 7], slots[:3])           # 5 takes slot 1, then NOMEM at 6
        assert c.lookup([1, 5, 9, 3]) == ora.lookup([1, 5, 9, 3]) == 2
        # retrieve with a missing id writes nothing
        dst = PagedKV(g, np.arange(g.NB), fill="sentinel")
        assert _status(lambda: c.retrieve([1, 6], slots_to_device(slots[:2]), dst.dev, stream)) \
            == lmc.LMC_ERR_MISS == ora.retrieve([1, 6], slots[:2], dst.host)
        torch.cuda.synchronize()
        assert_layers_equal(dst.device_blocks_to_host(), dst.host)
        assert c.get_stats()["retrieve_misses"] == 1
        # the same chunk twice in one retrieve, to different pages
        d_sl = slots_to_device(slots[2:4])
        t = c.retrieve([3, 3], d_sl, dst.dev, stream)
        c.wait(t)
        assert ora.retrieve([3, 3], slots[2:4], dst.host) == 0
        assert_layers_equal(dst.device_blocks_to_host(), dst.host)
        # pin / clear / unpin
        c.pin([5])
        assert _status(lambda: c.clear([1, 5])) == lmc.LMC_ERR_BUSY
        assert c.lookup([1]) == 1
        c.unpin([5])
        assert _status(lambda: c.unpin([5])) == lmc.LMC_ERR_INVAL
        c.clear([1, 5, 3, 999])
        assert c.get_stats()["pool_slots_used"] == 0
    ora.close()


@pytest.mark.parametrize("staged", [True, False])
def test_partial_skip_store_launches_per_run_of_new_chunks(staged):
    """Chunks 0,1 and 4 are present; 2,3 and 5,6,7 are new: launches never span a gap, and
    gather from the right parts of the slot mapping."""
    import torch
    from gpu_util import PagedKV, slots_to_device
    lmc = _lmc()
    g = W.geometry("tiny", NB=256)
    rng = np.random.default_rng(5)
    kv = PagedKV(g, np.arange(g.NB), rng)
    toks = W.tokens_for(rng, 8 * g.CT)
    slots = rng.permutation(g.n_slots)[:8 * g.CT].reshape(8, g.CT)
    other = rng.permutation(g.n_slots)[:8 * g.CT].reshape(8, g.CT)
    with lmc.Context(g, 8 * g.chunk_bytes, staging_chunks=4) as c:
        if staged:
            c.tune("direct_store_below", 0)    # 2.5 MiB of new chunks would otherwise skip staging
        ids = c.hash_chunks(toks)
        d_other, d_slots = slots_to_device(other[[0, 1, 4]]), slots_to_device(slots)
        c.store(kv.dev, d_other, ids[[0, 1, 4]], torch.cuda.current_stream())
        c.wait()
        c.reset_stats()
        c.store(kv.dev, d_slots, ids, torch.cuda.current_stream())
        c.wait()
        st = c.get_stats()
        assert st["chunks_stored"] == 5 and st["chunks_skipped_dup"] == 3
        # staged: [2] (single-chunk head), [3], [5, 6, 7]; direct: [2, 3], [5, 6, 7] (the new
        # chunks took pool slots 3..7 in order, so each run is also one run of the pool)
        assert st["gather_launches"] == (3 if staged else 2)
        for k in range(8):
            src_slots = other[k] if k in (0, 1, 4) else slots[k]
            assert np.array_equal(c.get_host(ids[k]), oracle.gather_chunk(g, kv.host, src_slots)), k


def test_store_and_retrieve_run_concurrently_from_two_threads():
    """Full duplex (paper section 5.1, "Parallel Store/load Operations"): one thread stores
    request A while another retrieves request B; afterwards both are exact."""
    import threading
    import torch
    from gpu_util import PagedKV, assert_layers_equal, slots_to_device
    lmc = _lmc()
    g = W.geometry("llama3_8b", L=8, NB=2048)
    rng = np.random.default_rng(41)
    n = 12
    bpc = g.CT // g.BS
    blocks = rng.permutation(g.NB)
    src_a = PagedKV(g, blocks[:n * bpc], rng)
    src_b = PagedKV(g, blocks[n * bpc:2 * n * bpc], rng)
    dst_b = PagedKV(g, blocks[2 * n * bpc:3 * n * bpc], fill="sentinel")
    sa = W.slots_from_blocks(g, src_a.blocks, n * g.CT)
    sb = W.slots_from_blocks(g, src_b.blocks, n * g.CT)
    tb = W.slots_from_blocks(g, dst_b.blocks, n * g.CT)
    ids_a = np.arange(1, n + 1, dtype=np.uint64)
    ids_b = np.arange(101, n + 101, dtype=np.uint64)
    with lmc.Context(g, 2 * n * g.chunk_bytes, staging_chunks=2, flags=lmc.LMC_FLAG_POISON_STAGING) as c:
        d_sa, d_sb, d_tb = slots_to_device(sa), slots_to_device(sb), slots_to_device(tb)
        torch.cuda.synchronize()
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        c.wait(c.store(src_b.dev, d_sb, ids_b, s1))
        errors = []

        def run(fn):
            try:
                for _ in range(3):
                    fn()
            except Exception as e:  # noqa: BLE001
                errors.append(e)

        def do_store():
            c.clear(ids_a)
            c.wait(c.store(src_a.dev, d_sa, ids_a, s1))

        def do_load():
            c.wait(c.retrieve(ids_b, d_tb, dst_b.dev, s2))

        th = [threading.Thread(target=run, args=(f,)) for f in (do_store, do_load)]
        [t.start() for t in th]
        [t.join() for t in th]
        assert not errors, errors
        torch.cuda.synchronize()
        for i, s in zip(ids_a.tolist(), src_a.compact_slots(sa).reshape(n, g.CT)):
            assert np.array_equal(c.get_host(i), oracle.gather_chunk(src_a.gc, src_a.host, s))
        for s, t in zip(src_b.compact_slots(sb).reshape(n, g.CT), dst_b.compact_slots(tb).reshape(n, g.CT)):
            oracle.scatter_chunk(dst_b.gc, oracle.gather_chunk(src_b.gc, src_b.host, s), t, dst_b.host)
        assert_layers_equal(dst_b.device_blocks_to_host(), dst_b.host)


def test_allocation_failures_are_clean_errors():
    """A pool or a staging ring that cannot be allocated gives LMC_ERR_NOMEM and leaves
    nothing behind: a normal context can be created right after."""
    import torch
    lmc = _lmc()
    g = W.geometry("llama3_8b")
    with lmc.Context(g, 2 * g.chunk_bytes):                       # the runtime's own stream resources exist now
        pass
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    with pytest.raises(lmc.LMCError) as e:
        lmc.Context(g, 1 << 50)                                   # a petabyte of pinned memory
    assert e.value.status == lmc.LMC_ERR_NOMEM
    with pytest.raises(lmc.LMCError) as e:
        lmc.Context(g, 2 * g.chunk_bytes, staging_chunks=2000, num_staging=8)   # 16 buffers of 62.5 GiB
    assert e.value.status == lmc.LMC_ERR_NOMEM
    with pytest.raises(lmc.LMCError) as e:
        lmc.Context(g, 2 * g.chunk_bytes, staging_chunks=200000)  # more than one launch can cover
    assert e.value.status == lmc.LMC_ERR_INVAL
    # the failures stay inside the library: the caller's next HIP work sees no stale error
    assert float((torch.full((1024,), 2.0, device="cuda") * 2).sum()) == 4096.0
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] >= free_before - (64 << 20)
    with lmc.Context(g, 2 * g.chunk_bytes) as c:
        assert c.pool_slots() == 2
