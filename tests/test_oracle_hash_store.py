"""Pins for the oracle's chunk hashing, prefix lookup and chunk store (paper section 4:
store keeps only new tokens, retrieve serves the prefix-matched tokens)."""
import os
import struct

import numpy as np
import pytest

import oracle
from paper_2510_09665_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "fnv1a64_vectors.txt")


def test_fnv1a64_published_vectors():
    n = 0
    for line in open(GOLDEN):
        if line.startswith("#") or "|" not in line:
            continue
        text, hexval = line.rstrip("\n").split("|")
        assert oracle.fnv1a64(text.encode()) == int(hexval, 16), text
        n += 1
    assert n >= 5


def test_chain_is_fnv_of_previous_hash_and_le32_tokens():
    toks = np.arange(512, dtype=np.int32)
    h = oracle.hash_chunks(toks, CT=256, seed=0)
    m0 = struct.pack("<Q", 0) + struct.pack("<256i", *toks[:256])
    assert int(h[0]) == oracle.fnv1a64(m0)
    m1 = struct.pack("<Q", int(h[0])) + struct.pack("<256i", *toks[256:])
    assert int(h[1]) == oracle.fnv1a64(m1)
    # the seed is the hash "before the first chunk"
    h7 = oracle.hash_chunks(toks, CT=256, seed=7)
    assert int(h7[0]) == oracle.fnv1a64(struct.pack("<Q", 7) + struct.pack("<256i", *toks[:256]))
    assert int(h7[0]) != int(h[0])


def test_chain_worked_example_tokens_0_to_511():
    """Seed 0, tokens 0..511: the two chunk ids, as obtained twice independently of the
    oracle (a byte-at-a-time FNV-1a in plain Python here, and once before when the hash
    was chosen)."""
    def fnv(data):
        x = 0xcbf29ce484222325
        for c in data:
            x = ((x ^ c) * 0x100000001b3) & 0xFFFFFFFFFFFFFFFF
        return x
    h0 = fnv(struct.pack("<Q", 0) + struct.pack("<256i", *range(256)))
    h1 = fnv(struct.pack("<Q", h0) + struct.pack("<256i", *range(256, 512)))
    assert (h0, h1) == (0xc89cc5e687031dc5, 0x8e1d41f5a643ff04)
    got = oracle.hash_chunks(np.arange(512, dtype=np.int32), CT=256, seed=0)
    assert [int(x) for x in got] == [h0, h1]


def test_only_full_chunks_and_prefix_property():
    rng = np.random.default_rng(11)
    a = W.tokens_for(rng, 256 * 6 + 100)
    ha = oracle.hash_chunks(a)
    assert ha.size == 6
    assert np.array_equal(oracle.hash_chunks(a[:256 * 6]), ha)
    for k in range(6):
        b = a.copy()
        b[256 * k + 17] ^= 1
        hb = oracle.hash_chunks(b)
        assert np.array_equal(hb[:k], ha[:k])
        assert np.all(hb[k:] != ha[k:])
    # negative ids and ids above 2^31 hash as their 32-bit two's complement pattern
    c = a.copy()
    c[3] = -5
    assert oracle.hash_chunks(c)[0] != ha[0]
    # chunk length is a parameter
    assert oracle.hash_chunks(a[:64], CT=16).size == 4


def _small():
    g = W.KVGeometry(L=2, P=2, H=2, D=4, e=2, BS=4, NB=32, CT=16)
    return g, np.random.default_rng(21)


def test_lookup_counts_only_the_leading_run():
    g, rng = _small()
    layers = W.random_layers(rng, g)
    st = oracle.OracleStore(g, 8)
    hs = np.array([10, 11, 12, 13], dtype=np.uint64)
    slots = rng.permutation(g.n_slots)[:4 * g.CT]
    assert st.store(layers, slots[:2 * g.CT], hs[:2]) == (0, 2)
    assert st.store(layers, slots[3 * g.CT:], hs[3:]) == (0, 1)
    assert st.lookup(hs) == 2            # 13 is present but 12 is not
    assert st.lookup(hs[2:]) == 0
    assert st.lookup(hs[3:]) == 1
    assert st.lookup(hs[:0]) == 0


def test_store_skips_present_and_fills_lowest_slot_and_nomem():
    g, rng = _small()
    layers = W.random_layers(rng, g)
    st = oracle.OracleStore(g, 3)
    slots = rng.permutation(g.n_slots)[:4 * g.CT].reshape(4, g.CT)
    assert st.store(layers, slots[:2], [1, 2]) == (0, 2)
    assert (st.find(1), st.find(2)) == (0, 1)
    first = st.slot_bytes(0)
    assert np.array_equal(first, oracle.gather_chunk(g, layers, slots[0]))
    # same hash again with other slots: first writer wins, payload is not rewritten
    assert st.store(layers, slots[2:3], [1]) == (0, 0)
    assert np.array_equal(st.slot_bytes(0), first)
    # clear frees slot 0; the next new chunk takes it (lowest free first)
    assert st.clear([1]) == 0 and st.find(1) == -1
    assert st.store(layers, slots[2:4], [3, 4]) == (0, 2)
    assert (st.find(3), st.find(4)) == (0, 2)
    # full: NOMEM, chunks stored before the failing one stay
    assert st.clear([3]) == 0
    rc, n_new = st.store(layers, slots[:3], [7, 8, 9])
    assert (rc, n_new) == (oracle.ORC_NOMEM, 1)
    assert st.find(7) == 0 and st.find(8) == -1 and st.used() == 3


def test_retrieve_miss_writes_nothing_and_batch_is_all_or_nothing():
    g, rng = _small()
    layers = W.random_layers(rng, g)
    st = oracle.OracleStore(g, 8)
    slots = rng.permutation(g.n_slots)[:4 * g.CT].reshape(4, g.CT)
    assert st.store(layers, slots[:3], [1, 2, 3]) == (0, 3)
    dst = [W.sentinel_layer(g, l) for l in range(g.L)]
    before = [a.copy() for a in dst]
    assert st.retrieve([1, 99], slots[:2], dst) == oracle.ORC_MISS
    assert st.retrieve_batch([0, 2, 3], [1, 2, 99], slots[:3], dst) == oracle.ORC_MISS
    assert all(np.array_equal(a, b) for a, b in zip(dst, before))
    tau = rng.permutation(g.n_slots)[:3 * g.CT].reshape(3, g.CT)
    assert st.retrieve_batch([0, 2, 2, 3], [1, 2, 3], tau, dst) == 0
    want = [a.copy() for a in before]
    for i in range(3):
        oracle.scatter_chunk(g, oracle.gather_chunk(g, layers, slots[i]), tau[i], want)
    assert all(np.array_equal(a, b) for a, b in zip(dst, want))
    # a slot beyond the pool is refused before anything happens
    bad = tau.copy()
    bad[2, 5] = g.n_slots
    assert st.retrieve([1, 2, 3], bad, dst) == oracle.ORC_BADSLOT
    assert all(np.array_equal(a, b) for a, b in zip(dst, want))


def test_pin_unpin_clear():
    g, rng = _small()
    layers = W.random_layers(rng, g)
    st = oracle.OracleStore(g, 4)
    slots = rng.permutation(g.n_slots)[:2 * g.CT]
    st.store(layers, slots, [5, 6])
    assert st.pin([5, 77]) == oracle.ORC_MISS
    assert st.clear([5]) == 0 and st.store(layers, slots[:g.CT], [5]) == (0, 1)
    assert st.pin([5]) == 0 and st.pin([5]) == 0
    assert st.clear([6, 5]) == oracle.ORC_BUSY and st.find(6) >= 0
    assert st.unpin([5, 5, 5]) == oracle.ORC_INVAL
    assert st.unpin([5]) == 0
    assert st.clear([5]) == oracle.ORC_BUSY
    assert st.unpin([5]) == 0 and st.unpin([5]) == oracle.ORC_INVAL
    assert st.clear([5, 6, 1234]) == 0 and st.used() == 0


def test_model_check_against_dict_of_bytes():
    """Random op sequences; the reference is a dict hash -> chunk bytes with a set of
    free slot numbers, written here without the oracle's store."""
    g, rng = _small()
    layers = W.random_layers(rng, g)
    n_slots = 5
    st = oracle.OracleStore(g, n_slots)
    model, slot_of, pins = {}, {}, {}
    for step in range(400):
        op = rng.choice(["store", "lookup", "retrieve", "clear", "pin", "unpin"])
        hs = rng.integers(0, 9, rng.integers(1, 4)).astype(np.uint64)
        if op == "store":
            slots = rng.permutation(g.n_slots)[:hs.size * g.CT].reshape(hs.size, g.CT)
            rc, n_new = st.store(layers, slots, hs)
            want_rc, want_new = 0, 0
            for h, s in zip(hs.tolist(), slots):
                if h in model:
                    continue
                free = sorted(set(range(n_slots)) - set(slot_of.values()))
                if not free:
                    want_rc = oracle.ORC_NOMEM
                    break
                model[h] = oracle.gather_chunk(g, layers, s)
                slot_of[h], pins[h] = free[0], 0
                want_new += 1
            assert (rc, n_new) == (want_rc, want_new), step
        elif op == "lookup":
            k = 0
            while k < hs.size and int(hs[k]) in model:
                k += 1
            assert st.lookup(hs) == k
        elif op == "retrieve":
            tau = rng.permutation(g.n_slots)[:hs.size * g.CT].reshape(hs.size, g.CT)
            dst = [W.sentinel_layer(g, l) for l in range(g.L)]
            want = [a.copy() for a in dst]
            rc = st.retrieve(hs, tau, dst)
            if all(int(h) in model for h in hs):
                assert rc == 0
                for h, t in zip(hs.tolist(), tau):
                    oracle.scatter_chunk(g, model[h], t, want)
            else:
                assert rc == oracle.ORC_MISS
            assert all(np.array_equal(a, b) for a, b in zip(dst, want)), step
        elif op == "clear":
            rc = st.clear(hs)
            if any(pins.get(int(h), 0) > 0 for h in hs):
                assert rc == oracle.ORC_BUSY
            else:
                assert rc == 0
                for h in hs.tolist():
                    model.pop(h, None), slot_of.pop(h, None), pins.pop(h, None)
        elif op == "pin":
            rc = st.pin(hs)
            if all(int(h) in model for h in hs):
                assert rc == 0
                for h in hs.tolist():
                    pins[h] += 1
            else:
                assert rc == oracle.ORC_MISS
        else:
            rc = st.unpin(hs)
            if not all(int(h) in model for h in hs):
                assert rc == oracle.ORC_MISS
            elif any(pins[int(h)] < hs.tolist().count(int(h)) for h in hs):
                assert rc == oracle.ORC_INVAL
            else:
                assert rc == 0
                for h in hs.tolist():
                    pins[h] -= 1
        for h, b in model.items():
            assert st.find(h) == slot_of[h]
            assert np.array_equal(st.slot_bytes(slot_of[h]), b)
        assert st.used() == len(model)
