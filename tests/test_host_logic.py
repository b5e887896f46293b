"""CPU tests of the library's host side: the C ABI loads and exports what include/lmc.h
declares, and hashing / index / pool bookkeeping of an index-only context agree with
the oracle.  No device call is made here."""
import os
import re

import numpy as np
import pytest

import oracle
from paper_2510_09665_amd import lmc
from paper_2510_09665_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "lmc.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = sorted(set(re.findall(r"\b(lmc_[a-z_]+)\s*\(", header)))
    assert declared == sorted(lmc.EXPORTS)
    lib = lmc._lib()
    for name in declared:
        assert getattr(lib, name) is not None


def test_header_is_plain_c(tmp_path):
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "t.c"
    src.write_text('#include "lmc.h"\nint main(void) { lmc_stats_t s; (void)s; return LMC_OK; }\n')
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only",
                           "-I", os.path.join(ROOT, "include"), str(src)])


def test_struct_sizes_match_the_header_layout():
    import ctypes
    assert ctypes.sizeof(lmc.lmc_kv_geom_t) == 8 * 4 + 4 * 8
    assert ctypes.sizeof(lmc.lmc_config_t) == 64 + 8 + 4 * 4 + 8
    assert ctypes.sizeof(lmc.lmc_stats_t) == 22 * 8


def _ctx(g, n_slots, **kw):
    return lmc.Context(g, n_slots * g.chunk_bytes, device=lmc.LMC_DEVICE_NONE, **kw)


def test_hash_chunks_matches_oracle():
    g = W.geometry("tiny")
    rng = np.random.default_rng(3)
    for seed in (0, 0xDEADBEEFCAFEF00D):
        with _ctx(g, 1, hash_seed=seed) as c:
            for n in (0, 255, 256, 257, 256 * 9 + 3):
                toks = W.tokens_for(rng, n)
                if n:
                    toks[rng.integers(0, n)] = -7
                assert np.array_equal(c.hash_chunks(toks), oracle.hash_chunks(toks, 256, seed))
    g16 = W.KVGeometry(L=1, P=1, H=1, D=16, e=1, BS=4, NB=8, CT=16)
    with _ctx(g16, 1) as c:
        toks = W.tokens_for(rng, 100)
        assert np.array_equal(c.hash_chunks(toks), oracle.hash_chunks(toks, 16, 0))


def test_hash_chain_can_be_continued():
    g = W.geometry("tiny")
    rng = np.random.default_rng(8)
    toks = W.tokens_for(rng, 256 * 7 + 30)
    with _ctx(g, 1, hash_seed=5) as c:
        whole = c.hash_chunks(toks)
        for cut in (1, 3, 6):
            rest = c.hash_chunks_from(whole[cut - 1], toks[256 * cut:])
            assert np.array_equal(rest, whole[cut:])
        assert np.array_equal(c.hash_chunks_from(5, toks), whole)
        assert np.array_equal(whole, oracle.hash_chunks(toks, 256, 5))


def test_sizes_and_bad_configs():
    for name in W.CONFIGS:
        g = W.geometry(name)
        with _ctx(g, 2) as c:
            assert c.chunk_bytes() == g.chunk_bytes == oracle.chunk_bytes(g)
            assert c.pool_slots() == 2
    g = W.geometry("tiny")
    with pytest.raises(lmc.LMCError) as e:
        lmc.Context(g, g.chunk_bytes - 1, device=lmc.LMC_DEVICE_NONE)
    assert e.value.status == lmc.LMC_ERR_INVAL
    with pytest.raises(lmc.LMCError):
        lmc.Context(g, g.chunk_bytes, num_staging=1, device=lmc.LMC_DEVICE_NONE)
    with pytest.raises(lmc.LMCError):
        lmc.Context(W.KVGeometry(L=161, P=1, H=1, D=16, e=1, BS=4, NB=8), 1 << 20,
                    device=lmc.LMC_DEVICE_NONE)
    with pytest.raises(lmc.LMCError):
        lmc.Context(W.KVGeometry(L=1, P=1, H=1, D=16, e=1, BS=1 << 16, NB=1 << 15, CT=16), 1 << 20,
                    device=lmc.LMC_DEVICE_NONE)


def test_data_path_refuses_to_run_without_a_device():
    g = W.geometry("tiny")
    with _ctx(g, 2) as c:
        fake = [0x1000] * g.L
        for call in (lambda: c.store(fake, 0x1000, [1]),
                     lambda: c.retrieve([1], 0x1000, fake),
                     lambda: c.retrieve_batch([0, 1], [1], 0x1000, fake),
                     lambda: c.retrieve_layerwise([1], 0x1000, fake),
                     lambda: c.store_begin(0x1000, [1]),
                     lambda: c.store_layers(1, 0, 1, fake),
                     lambda: c.wait_layer(1, 0),
                     lambda: c.gather(fake, 0x1000, 1, 0x1000),
                     lambda: c.scatter(0x1000, 0x1000, 1, fake),
                     lambda: c.copy(0x1000, 0x2000, 16),
                     lambda: c.measure_link(1024),
                     lambda: c.measure_link_kernel(1024),
                     lambda: c.measure_link_duplex(1024),
                     lambda: c.measure_link_duplex_kernel(1024, 3),
                     lambda: c.store_static(fake, 0x1000, 1, 0x1000),
                     lambda: c.trace_read(4),
                     lambda: c.tune("trace", 1),
                     lambda: c.tune("arrange_streams", 1)):
            with pytest.raises(lmc.LMCError) as e:
                call()
            assert e.value.status == lmc.LMC_ERR_NODEVICE
        c.wait()


def _status(fn):
    try:
        fn()
        return 0
    except lmc.LMCError as e:
        return e.status


@pytest.mark.parametrize("evict", [False, True])
def test_index_and_pool_model_check_against_oracle_store(evict):
    """Random put / lookup / get / pin / unpin / clear sequences: statuses, slot numbers
    (lowest free first), pool bytes and, with eviction on, the evicted ids in order must
    equal the oracle's chunk store."""
    g = W.KVGeometry(L=2, P=2, H=2, D=4, e=2, BS=4, NB=32, CT=16)
    rng = np.random.default_rng(99)
    layers = W.random_layers(rng, g)
    n_slots = 6
    ora = oracle.OracleStore(g, n_slots, evict=evict)
    n_evicted = 0
    with _ctx(g, n_slots, flags=lmc.LMC_FLAG_EVICT_LRU if evict else 0) as c:
        for step in range(600):
            op = rng.choice(["put", "put", "lookup", "pin", "unpin", "clear", "get"])
            ids = rng.integers(0, 12, rng.integers(1, 5)).astype(np.uint64)
            if op == "put":
                slots = rng.permutation(g.n_slots)[:ids.size * g.CT].reshape(ids.size, g.CT)
                chunks = oracle.gather(g, layers, slots)          # the bytes both sides receive
                want_rc, _ = ora.store(layers, slots, ids)
                assert _status(lambda: c.put_host(ids, chunks)) == want_rc, step
                gone = ora.drain_evicted()
                assert c.drain_evicted().tolist() == gone.tolist(), step
                n_evicted += gone.size
            elif op == "lookup":
                assert c.lookup(ids) == ora.lookup(ids)
            elif op == "pin":
                assert _status(lambda: c.pin(ids)) == ora.pin(ids)
            elif op == "unpin":
                assert _status(lambda: c.unpin(ids)) == ora.unpin(ids)
            elif op == "clear":
                assert _status(lambda: c.clear(ids)) == ora.clear(ids)
            else:
                for i in ids.tolist():
                    if ora.find(i) < 0:
                        assert _status(lambda: c.get_host(i)) == lmc.LMC_ERR_MISS
                    else:
                        assert np.array_equal(c.get_host(i), ora.slot_bytes(ora.find(i)))
            for i in range(12):
                want = ora.find(i)
                got = c.find_slot(i) if want >= 0 else -1
                if want < 0:
                    assert _status(lambda: c.find_slot(i)) == lmc.LMC_ERR_MISS
                assert got == want, (step, i)
            st = c.get_stats()
            assert st["pool_slots_used"] == ora.used() and st["pool_slots_total"] == n_slots
            assert st["chunks_evicted"] == n_evicted
    assert (n_evicted > 100) == evict


def test_index_survives_many_inserts_and_erases():
    g = W.KVGeometry(L=1, P=1, H=1, D=16, e=1, BS=4, NB=8, CT=4)   # 64-byte chunks
    n_slots = 5000
    rng = np.random.default_rng(5)
    with _ctx(g, n_slots) as c:
        live = {}
        free = set(range(n_slots))
        for rnd in range(6):
            ids = rng.integers(0, 1 << 63, 3000, dtype=np.uint64)
            for i in ids.tolist():
                if i in live or not free:
                    continue
                c.put_host([i], np.full(64, i & 0xFF, dtype=np.uint8))
                s = min(free)
                free.remove(s)
                live[i] = s
                assert c.find_slot(i) == s
            kill = rng.permutation(list(live))[:len(live) // 2].astype(np.uint64)
            c.clear(kill)
            for i in kill.tolist():
                free.add(live.pop(i))
            for i, s in list(live.items())[::7]:
                assert c.find_slot(i) == s
                assert c.get_host(i)[0] == (i & 0xFF)
            assert c.get_stats()["pool_slots_used"] == len(live)
        with pytest.raises(lmc.LMCError) as e:
            c.put_host(np.arange(1, n_slots + 2, dtype=np.uint64) + (1 << 62),
                       np.zeros((n_slots + 1) * 64, dtype=np.uint8))
        assert e.value.status == lmc.LMC_ERR_NOMEM
        assert c.get_stats()["pool_slots_used"] == n_slots
