"""Pins for the oracle's optional eviction (the paper says that instances store and evict,
sections 4.2 and 7, without naming a policy; the reading is least recently used, with the
tail of a request going before its head).  Each test fixes the oracle against something
that is not the oracle: the textbook LRU cache built on an ordered dict, a sequence worked
out by hand, and invariants that hold for any sequence."""
from collections import OrderedDict

import numpy as np
import pytest

import oracle
from paper_2510_09665_amd import workloads as W

G = W.KVGeometry(L=1, P=1, H=1, D=8, e=1, BS=2, NB=64, CT=4)


def _layers(rng):
    return W.random_layers(rng, G)


def _slots(rng, n):
    return rng.permutation(G.n_slots)[:n * G.CT].astype(np.int64)


def u64(*xs):
    return np.array(xs, dtype=np.uint64)


def test_one_chunk_per_call_is_the_textbook_lru_cache():
    """With a single chunk per call positions play no part: what remains is the plain LRU
    cache, here modelled by an OrderedDict (use = move to the end, evict = pop the front)."""
    rng = np.random.default_rng(1)
    layers = _layers(rng)
    cap = 5
    s = oracle.OracleStore(G, cap, evict=True)
    model = OrderedDict()
    dst = [np.zeros(G.layer_bytes, dtype=np.uint8)]
    for step in range(600):
        h = int(rng.integers(0, 12))
        if rng.random() < 0.6:
            sl = _slots(rng, 1)
            rc, n_new = s.store(layers, sl, u64(h))
            want_evicted = []
            if h in model:
                model.move_to_end(h)
                assert n_new == 0
            else:
                if len(model) == cap:
                    want_evicted.append(model.popitem(last=False)[0])
                model[h] = oracle.gather_chunk(G, layers, sl)
                assert n_new == 1
            assert rc == 0
            assert s.drain_evicted().tolist() == want_evicted, step
        else:
            rc = s.retrieve(u64(h), _slots(rng, 1), dst)
            if h in model:
                model.move_to_end(h)
                assert rc == 0
            else:
                assert rc == -3
        assert s.used() == len(model)
        for k, v in model.items():
            assert np.array_equal(s.slot_bytes(s.find(k)), v), (step, k)
    s.close()


def test_worked_example_tail_goes_before_head_and_pins_and_own_call_are_safe():
    rng = np.random.default_rng(2)
    layers = _layers(rng)
    s = oracle.OracleStore(G, 6, evict=True)
    st = lambda *h: s.store(layers, _slots(rng, len(h)), u64(*h))
    dst = [np.zeros(G.layer_bytes, dtype=np.uint8)]
    # request A = chunks 1 2 3, request B = chunks 11 12 13: the pool (6 slots) is full
    assert st(1, 2, 3) == (0, 3)
    assert st(11, 12, 13) == (0, 3)
    assert s.drain_evicted().size == 0
    # a new chunk needs room: A is the older call and its tail, chunk 3, is the oldest
    assert st(21) == (0, 1)
    assert s.drain_evicted().tolist() == [3]
    assert s.lookup(u64(1, 2, 3)) == 2          # what is left of A still hits on its head
    # using A's head again makes B the oldest: next out are 13, then 12
    assert s.retrieve(u64(1, 2), _slots(rng, 2), dst) == 0
    assert st(22, 23) == (0, 2)
    assert s.drain_evicted().tolist() == [13, 12]
    # a pinned chunk is passed over: 11 is the oldest but pinned, so 21 goes
    assert s.pin(u64(11)) == 0
    assert st(24) == (0, 1)
    assert s.drain_evicted().tolist() == [21]
    # a call never evicts what it is itself using.  Storing 2 (present) with five new
    # chunks: 1 goes first (oldest call left; its companion 2 belongs to this call), then
    # 23 before 22 (same call, tail first), then 24 -- and then nothing is left to evict:
    # 11 is pinned, everything else is part of this call, so the fifth new chunk fails
    rc, n_new = st(2, 31, 32, 33, 34, 35)
    assert (rc, n_new) == (-2, 4)
    assert s.drain_evicted().tolist() == [1, 23, 22, 24]
    assert sorted(h for h in (2, 11, 31, 32, 33, 34) if s.find(h) >= 0) == [2, 11, 31, 32, 33, 34]
    assert s.find(35) < 0 and s.used() == 6
    # a failed retrieve is no use: 31..34 keep their order, 34 (the tail) goes first
    assert s.unpin(u64(11)) == 0
    assert s.retrieve(u64(34, 99), _slots(rng, 2), dst) == -3
    assert st(41) == (0, 1)
    assert s.drain_evicted().tolist() == [11]   # 11 is older than that whole call
    assert st(42) == (0, 1)
    assert s.drain_evicted().tolist() == [34]
    s.close()


def test_a_chunk_listed_twice_in_a_call_counts_at_its_first_position():
    rng = np.random.default_rng(4)
    layers = _layers(rng)
    s = oracle.OracleStore(G, 3, evict=True)
    dst = [np.zeros(G.layer_bytes, dtype=np.uint8)]
    assert s.store(layers, _slots(rng, 3), u64(51, 52, 51)) == (0, 2)      # 51 at 0 (and 2), 52 at 1
    assert s.store(layers, _slots(rng, 1), u64(53)) == (0, 1)
    assert s.store(layers, _slots(rng, 1), u64(54)) == (0, 1)
    assert s.drain_evicted().tolist() == [52]                              # not 51: its place is 0
    assert s.retrieve(u64(53, 51, 53), _slots(rng, 3), dst) == 0           # 53 at 0, 51 at 1
    assert s.store(layers, _slots(rng, 2), u64(55, 56)) == (0, 2)
    assert s.drain_evicted().tolist() == [54, 51]
    s.close()


def test_reference_counter_two_destinations_hold_the_chunk_until_both_are_done():
    """Section 5.3, zero-copy operations, written out: a chunk on its way to two
    destinations carries two counts; each completion takes one off; only at zero may the
    chunk go (by clear or by eviction)."""
    rng = np.random.default_rng(5)
    layers = _layers(rng)
    s = oracle.OracleStore(G, 2, evict=True)
    assert s.store(layers, _slots(rng, 2), u64(1, 2)) == (0, 2)
    assert s.acquire(9) == -3 and s.release(1) == -1            # absent; nothing to release
    assert s.acquire(1) == 0 and s.acquire(1) == 0              # disk and remote store
    assert s.refs(1) == 2
    assert s.clear(u64(1)) == -6
    # a new chunk needs room: 2 is the tail and goes first anyway; the next one would take
    # 1 (oldest) but cannot, and nothing else may go (3 belongs to the call): no room
    assert s.store(layers, _slots(rng, 2), u64(3, 4)) == (-2, 1)
    assert s.drain_evicted().tolist() == [2]
    assert s.release(1) == 0                                    # first destination done
    assert s.refs(1) == 1 and s.clear(u64(1)) == -6
    assert s.store(layers, _slots(rng, 1), u64(4)) == (0, 1)    # 3 is from an older call now: it goes
    assert s.drain_evicted().tolist() == [3]
    assert s.pin(u64(4)) == 0
    assert s.store(layers, _slots(rng, 1), u64(5)) == (-2, 0)   # 4 pinned, 1 still counted: no room
    assert s.release(1) == 0                                    # second destination done
    assert s.refs(1) == 0 and s.release(1) == -1
    assert s.store(layers, _slots(rng, 1), u64(5)) == (0, 1)    # now 1 can be evicted
    assert s.drain_evicted().tolist() == [1]
    assert s.refs(1) == -1 and s.unpin(u64(4)) == 0 and s.clear(u64(4, 5)) == 0 and s.used() == 0
    s.close()


def test_eviction_off_is_the_old_behaviour():
    rng = np.random.default_rng(3)
    layers = _layers(rng)
    s = oracle.OracleStore(G, 2)
    assert s.store(layers, _slots(rng, 3), u64(1, 2, 3)) == (-2, 2)
    assert s.drain_evicted().size == 0 and s.find(3) < 0
    s.close()


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_invariants_on_random_multi_chunk_sequences(seed):
    """Any sequence: an evicted chunk is gone and was neither pinned nor part of the
    evicting call; the pool never holds more than its slots; a call that fits never
    fails; chunks of the latest call are never evicted by it; the bytes of every chunk
    present are those of the store that brought it in."""
    rng = np.random.default_rng(seed)
    layers = _layers(rng)
    cap = 7
    s = oracle.OracleStore(G, cap, evict=True)
    content, pinned, held = {}, {}, {}
    dst = [np.zeros(G.layer_bytes, dtype=np.uint8)]
    for step in range(400):
        op = rng.choice(["store", "store", "retrieve", "pin", "unpin", "clear", "acquire", "release"])
        ids = rng.integers(0, 20, rng.integers(1, 5))
        hs = u64(*ids.tolist())
        if op == "store":
            sl = _slots(rng, ids.size)
            present_before = {int(h) for h in ids if s.find(int(h)) >= 0}
            rc, n_new = s.store(layers, sl, hs)
            ev = s.drain_evicted().tolist()
            assert len(set(ev)) == len(ev)
            for h in ev:
                assert s.find(h) < 0 or h in ids.tolist()     # gone (unless stored again later in the call)
                assert pinned.get(h, 0) == 0 and held.get(h, 0) == 0, (step, h)
                assert h not in present_before, (step, h)     # the call protects what it found
                content.pop(h, None)
            stored = 0
            for i, h in enumerate(ids.tolist()):
                if h not in content and s.find(h) >= 0:
                    content[h] = oracle.gather_chunk(G, layers, sl[i * G.CT:(i + 1) * G.CT])
                    stored += 1
            assert stored == n_new
            n_unique_new = len(set(ids.tolist()) - present_before)
            evictable = sum(1 for h in list(content) if pinned.get(h, 0) == 0 and h not in ids.tolist())
            if rc == -2:
                # only a call that really cannot fit fails
                assert s.used() == cap
                assert all(pinned.get(h, 0) > 0 or held.get(h, 0) > 0 or h in ids.tolist() for h in content)
            else:
                assert rc == 0 and all(s.find(int(h)) >= 0 for h in ids)
            assert evictable >= 0 and n_unique_new >= n_new
        elif op == "retrieve":
            rc = s.retrieve(hs, _slots(rng, ids.size), dst)
            assert rc == (0 if all(int(h) in content for h in ids) else -3)
        elif op == "pin":
            if s.pin(hs) == 0:
                for h in ids.tolist():
                    pinned[h] = pinned.get(h, 0) + 1
        elif op == "unpin":
            if s.unpin(hs) == 0:
                for h in ids.tolist():
                    pinned[h] -= 1
        elif op == "acquire":
            h = int(ids[0])
            assert s.acquire(h) == (0 if h in content else -3)
            if h in content:
                held[h] = held.get(h, 0) + 1
        elif op == "release":
            h = int(ids[0])
            want = -3 if h not in content else (0 if held.get(h, 0) > 0 else -1)
            assert s.release(h) == want
            if want == 0:
                held[h] -= 1
        else:
            busy = any(h in content and (pinned.get(h, 0) > 0 or held.get(h, 0) > 0) for h in ids.tolist())
            assert s.clear(hs) == (-6 if busy else 0)
            if not busy:
                for h in ids.tolist():
                    content.pop(h, None)
        assert s.used() == len(content) <= cap
        for h, v in content.items():
            assert np.array_equal(s.slot_bytes(s.find(h)), v), (step, h)
    s.close()
