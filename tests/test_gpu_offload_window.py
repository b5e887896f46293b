"""Dynamic offloading through the C ABI (paper section 5.3): free blocks are duplicated to
the pinned pool window by window; a query gets free blocks only once they are duplicated.
Pointer positions follow the oracle's model, and every granted block's KV is in the pool,
byte for byte what the oracle gathers for that block."""
import numpy as np
import pytest

import oracle
from oracle.offload_window import OffloadWindowOracle
from paper_2510_09665_amd import workloads as W

pytestmark = pytest.mark.gpu


def _block_chunk(g, kv, b):
    return oracle.gather_chunk(g, kv.host, np.arange(b * g.BS, (b + 1) * g.BS))


@pytest.mark.parametrize("window,max_batch", [(1, 4), (6, 4), (32, 8)])
def test_window_follows_oracle_and_pool_holds_every_granted_block(window, max_batch):
    import torch
    from gpu_util import PagedKV
    from paper_2510_09665_amd import lmc
    g = W.geometry("llama3_8b", L=4, NB=256, CT=16)            # a chunk is one block
    rng = np.random.default_rng(window)
    kv = PagedKV(g, np.arange(g.NB), rng)
    stream = torch.cuda.current_stream()
    free_order = rng.permutation(g.NB)
    ids = (free_order.astype(np.uint64) + np.uint64(1000))      # id of block b's content
    with lmc.Context(g, g.NB * g.chunk_bytes, staging_chunks=8) as c:
        w = c.window_create(window, max_batch)
        ora = OffloadWindowOracle(window)
        assert w.get()["state"] == 4
        pos, granted = 0, []
        for step in range(120):
            op = rng.integers(0, 3)
            if op == 0 and pos < g.NB:
                n = int(min(rng.integers(1, 12), g.NB - pos))
                w.release(free_order[pos:pos + n], ids[pos:pos + n])
                for b in free_order[pos:pos + n]:
                    ora.release(int(b))
                pos += n
            elif op == 1:
                # duplicate whatever is scheduled, and let it finish: then the oracle's
                # current pointer has reached its end pointer too
                sched = len(ora.scheduled())
                n = w.offload(kv.dev, stream)
                while n < sched:                                 # batch buffers were all busy
                    c.wait()
                    n += w.offload(kv.dev, stream)
                assert n == sched
                c.wait()
                ora.offloaded(sched)
            else:
                n = int(rng.integers(1, 9))
                too_many = n > ora.tail - ora.start              # fewer than n free pages exist
                try:
                    got = w.acquire(n)
                    assert not too_many, step
                except lmc.LMCError as e:
                    assert too_many and e.status == lmc.LMC_ERR_NOMEM, step
                    got = None
                want = ora.take(n)
                if want is None:
                    assert got is None, step
                else:
                    assert got is not None and got.tolist() == want, step
                    granted += want
            st = w.get()
            assert (st["start"], st["current"], st["end"], st["tail"], st["state"]) == \
                (ora.start, ora.current, ora.end, ora.tail, ora.state()), step
        assert len(granted) > 0
        for b in granted:                                        # duplicated before it was handed out
            assert np.array_equal(c.get_host(int(b) + 1000), _block_chunk(g, kv, int(b))), b
        w.destroy()


def test_the_sections_example_through_the_library():
    import torch
    from gpu_util import PagedKV
    from paper_2510_09665_amd import lmc
    g = W.geometry("tiny", CT=16)
    kv = PagedKV(g, np.arange(g.NB), np.random.default_rng(1))
    stream = torch.cuda.current_stream()
    with lmc.Context(g, 16 * g.chunk_bytes) as c:
        w = c.window_create(1, 4)                                # one duplicated page
        w.release(np.arange(10), np.arange(10) + 50)
        assert w.offload(kv.dev, stream) == 1
        c.wait()
        assert w.get() == dict(start=0, current=1, end=1, tail=10, state=4)
        assert w.acquire(3) is None                              # a query needing three pages stalls
        assert w.get()["end"] == 3                               # both pointers must advance by two
        assert w.offload(kv.dev, stream) == 2
        got = w.acquire(3, block=True)                           # waits for the two duplications
        assert got.tolist() == [0, 1, 2]
        assert w.get() == dict(start=3, current=3, end=6, tail=10, state=1)   # end moved forward by three
        with pytest.raises(lmc.LMCError) as e:
            w.acquire(8)
        assert e.value.status == lmc.LMC_ERR_NOMEM               # only seven free pages are left
        for b in (0, 1, 2):
            assert np.array_equal(c.get_host(50 + b), _block_chunk(g, kv, b))
        # a context whose chunk is not one block cannot host a window
        with lmc.Context(W.geometry("tiny"), 2 * W.geometry("tiny").chunk_bytes) as c2:
            with pytest.raises(lmc.LMCError) as e:
                c2.window_create(4, 4)
            assert e.value.status == lmc.LMC_ERR_INVAL
        w.destroy()
