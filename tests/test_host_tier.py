"""The reference counter on stored chunks and the directory tier that uses it (paper
section 5.3, "Zero-Copy Operations"), on an index-only context: statuses and counter
behaviour against the oracle's chunk store, file contents against the chunks' bytes.
A write is held open deterministically by making its temporary file a FIFO: the writer
blocks in open() until the test opens the other end."""
import os
import threading

import numpy as np
import pytest

import oracle
from paper_2510_09665_amd import lmc
from paper_2510_09665_amd import workloads as W

G = W.KVGeometry(L=2, P=2, H=2, D=8, e=2, BS=4, NB=32, CT=16)      # 2 KiB chunks


def _status(fn):
    try:
        fn()
        return 0
    except lmc.LMCError as e:
        return e.status


def _ctx(n_slots, **kw):
    return lmc.Context(G, n_slots * G.chunk_bytes, device=lmc.LMC_DEVICE_NONE, **kw)


def _chunks(rng, n):
    layers = W.random_layers(rng, G)
    slots = rng.permutation(G.n_slots)[:n * G.CT].reshape(n, G.CT)
    return layers, slots, oracle.gather(G, layers, slots)


def _name(d, i, tmp=False):
    return os.path.join(d, "%016x.kv" % i + (".tmp" if tmp else ""))


def test_acquire_release_follow_the_oracle_on_random_sequences():
    rng = np.random.default_rng(7)
    n_slots = 5
    ora = oracle.OracleStore(G, n_slots, evict=True)
    with _ctx(n_slots, flags=lmc.LMC_FLAG_EVICT_LRU) as c:
        for step in range(800):
            op = rng.choice(["put", "put", "acquire", "release", "release", "clear", "pin", "unpin"])
            ids = rng.integers(0, 9, rng.integers(1, 4)).astype(np.uint64)
            h = int(ids[0])
            if op == "put":
                layers, slots, chunks = _chunks(rng, ids.size)
                want, _ = ora.store(layers, slots, ids)
                assert _status(lambda: c.put_host(ids, chunks)) == want, step
                assert c.drain_evicted().tolist() == ora.drain_evicted().tolist(), step
            elif op == "acquire":
                want = ora.acquire(h)
                if want == 0:       # the view is the pool itself: same bytes as the oracle's slot
                    assert np.array_equal(c.chunk_acquire(h), ora.slot_bytes(ora.find(h))), step
                else:
                    assert _status(lambda: c.chunk_acquire(h)) == want, step
            elif op == "release":
                assert _status(lambda: c.chunk_release(h)) == ora.release(h), step
            elif op == "clear":
                assert _status(lambda: c.clear(ids)) == ora.clear(ids), step
            elif op == "pin":
                assert _status(lambda: c.pin(ids)) == ora.pin(ids), step
            else:
                assert _status(lambda: c.unpin(ids)) == ora.unpin(ids), step
            for i in range(9):
                want = ora.find(i)
                assert (c.find_slot(i) if want >= 0 else -1) == want, (step, i)
                if want < 0:
                    assert _status(lambda: c.find_slot(i)) == lmc.LMC_ERR_MISS
    ora.close()


def test_every_chunk_goes_to_every_directory_and_comes_back(tmp_path):
    rng = np.random.default_rng(1)
    dirs = [str(tmp_path / "disk"), str(tmp_path / "remote")]
    for d in dirs:
        os.mkdir(d)
    n = 7
    _, _, chunks = _chunks(rng, n)
    ids = rng.integers(1, 1 << 63, n, dtype=np.uint64)
    with _ctx(n) as c, c.tier_open(dirs, n_threads=3) as t:
        c.put_host(ids, chunks)
        assert t.lookup(0, ids) == 0
        t.write(ids)
        t.wait()
        assert t.get_stats() == dict(files_written=2 * n, bytes_written=2 * n * G.chunk_bytes, chunks_read=0)
        for d in dirs:
            assert sorted(os.listdir(d)) == sorted("%016x.kv" % i for i in ids.tolist())
            for k, i in enumerate(ids.tolist()):
                assert np.array_equal(np.fromfile(_name(d, i), dtype=np.uint8), chunks[k].reshape(-1))
        assert t.lookup(1, ids) == n
        # all counts are back: everything can be cleared, then read back from either place
        c.clear(ids)
        assert c.lookup(ids) == 0
        t.read(0, ids[:3])
        t.read(1, ids)                       # the first three are present and skipped
        assert t.get_stats()["chunks_read"] == n and c.lookup(ids) == n
        for k, i in enumerate(ids.tolist()):
            assert np.array_equal(c.get_host(i), chunks[k].reshape(-1))
        # lookup counts the leading run only; a missing file is a miss
        os.remove(_name(dirs[0], int(ids[2])))
        assert t.lookup(0, ids) == 2
        c.clear(ids)
        assert _status(lambda: t.read(0, ids)) == lmc.LMC_ERR_MISS
        assert c.lookup(ids) == 2            # what came before the missing one stays


def test_counts_hold_the_chunk_until_both_destinations_are_done(tmp_path):
    """The oracle's worked example, through the tier: chunk 1 is on its way to two
    directories; one write is held open.  Until it ends, clear is refused and eviction
    passes the chunk over; afterwards it can go."""
    rng = np.random.default_rng(2)
    dirs = [str(tmp_path / "a"), str(tmp_path / "b")]
    for d in dirs:
        os.mkdir(d)
    os.mkfifo(_name(dirs[1], 1, tmp=True))                       # directory b blocks in open()
    _, _, chunks = _chunks(rng, 4)
    with _ctx(2, flags=lmc.LMC_FLAG_EVICT_LRU) as c, c.tier_open(dirs, n_threads=2) as t:
        def put(i):
            return _status(lambda: c.put_host([i], chunks[i - 1]))
        assert put(1) == 0 and put(2) == 0
        assert _status(lambda: t.write([1, 9])) == lmc.LMC_ERR_MISS   # nothing queued, no count left behind
        c.clear([2])
        assert put(2) == 0
        t.write([1])
        # the write to a finishes by itself; the one to b is stuck: one count remains
        for _ in range(2000):
            if os.path.exists(_name(dirs[0], 1)):
                break
            threading.Event().wait(0.005)
        assert os.path.exists(_name(dirs[0], 1))
        assert _status(lambda: c.clear([1])) == lmc.LMC_ERR_BUSY
        assert put(3) == 0 and c.drain_evicted().tolist() == [2]   # 1 is older but counted
        assert _status(lambda: c.pin([3])) == 0
        assert put(4) == lmc.LMC_ERR_NOMEM                          # 3 pinned, 1 counted: no room
        # let the stuck write through: read the FIFO to its end
        got = []
        reader = threading.Thread(target=lambda: got.append(open(_name(dirs[1], 1, tmp=True), "rb").read()))
        reader.start()
        t.wait()
        reader.join()
        assert np.array_equal(np.frombuffer(got[0], dtype=np.uint8), chunks[0].reshape(-1))
        assert os.path.exists(_name(dirs[1], 1))                   # renamed when complete
        assert put(4) == 0 and c.drain_evicted().tolist() == [1]   # the count is back: 1 can go
        assert t.get_stats()["files_written"] == 2


def test_failed_write_is_reported_once_and_gives_the_count_back(tmp_path):
    rng = np.random.default_rng(3)
    good, bad = str(tmp_path / "good"), str(tmp_path / "bad")
    os.mkdir(good)
    os.mkdir(bad)
    _, _, chunks = _chunks(rng, 2)
    with _ctx(2) as c, c.tier_open([good, bad], n_threads=1) as t:
        c.put_host([5, 6], chunks)
        os.mkdir(_name(bad, 5, tmp=True))                          # open() of the temporary file fails: EISDIR
        t.write([5, 6])
        assert _status(t.wait) == lmc.LMC_ERR_IO
        assert t.errno() != 0
        assert _status(t.wait) == 0                                # reported once
        assert sorted(os.listdir(good)) == ["%016x.kv" % 5, "%016x.kv" % 6]
        assert os.path.exists(_name(bad, 6)) and not os.path.exists(_name(bad, 5))
        c.clear([5, 6])                                            # no count is left on either chunk
        # a short file is an I/O error on the way back
        with open(_name(good, 5), "r+b") as f:
            f.truncate(G.chunk_bytes - 1)
        assert _status(lambda: t.read(0, [6, 5])) == lmc.LMC_ERR_IO
        assert c.lookup([6]) == 1 and c.lookup([5]) == 0


def test_bad_arguments(tmp_path):
    with _ctx(2) as c:
        assert _status(lambda: c.tier_open([str(tmp_path / "nowhere")])) == lmc.LMC_ERR_INVAL
        assert _status(lambda: c.tier_open([])) == lmc.LMC_ERR_INVAL
        assert _status(lambda: c.tier_open([str(tmp_path)], n_threads=0)) == lmc.LMC_ERR_INVAL
        with c.tier_open([str(tmp_path)]) as t:
            assert _status(lambda: t.lookup(1, [1])) == lmc.LMC_ERR_INVAL
            assert _status(lambda: t.read(-1, [1])) == lmc.LMC_ERR_INVAL
            t.write([])
            t.wait()
        assert _status(lambda: c.chunk_acquire(1)) == lmc.LMC_ERR_MISS
        assert _status(lambda: c.chunk_release(1)) == lmc.LMC_ERR_MISS
