"""GPU parity of the two kernels alone (lmc_gather / lmc_scatter, paper section 5.1)
against the CPU oracle, byte for byte, through the C ABI."""
import zlib

import numpy as np
import pytest

import oracle
from paper_2510_09665_amd import workloads as W

pytestmark = pytest.mark.gpu

# shapes chosen to cross every kernel path: 16-byte vectors with contiguous rows,
# per-head runs (HND), padded blocks, rows that are not a multiple of a wavefront
# (MLA: 72 and 36 vectors), narrow vectors (8/4/2/1 bytes), a block size that is not a
# power of two, planes whose size is not a multiple of a 256-vector tile, P=1 and P=2,
# pages ordered blocks-outermost (the K and V page of a block adjacent in memory).
SHAPES = {
    "tiny_cfg1": dict(L=2, P=2, H=4, D=64, e=2, BS=16, NB=64, CT=256),
    "hnd": dict(L=5, P=2, H=8, D=64, e=2, BS=16, NB=40, CT=64, layout="HND"),
    "padded": dict(L=3, P=2, H=2, D=64, e=2, BS=8, NB=50, CT=64, block_pad=32),
    "mla_bf16_like": dict(L=7, P=1, H=1, D=576, e=2, BS=64, NB=12, CT=256),
    "mla_fp8_like": dict(L=9, P=1, H=1, D=576, e=1, BS=64, NB=12, CT=256),
    "vec8": dict(L=3, P=2, H=3, D=12, e=2, BS=4, NB=64, CT=32),
    "vec4_hnd": dict(L=3, P=2, H=3, D=6, e=2, BS=4, NB=64, CT=32, layout="HND"),
    "vec2": dict(L=2, P=2, H=3, D=7, e=2, BS=4, NB=64, CT=32),
    "vec1_pad": dict(L=2, P=1, H=2, D=5, e=1, BS=3, NB=70, CT=24, block_pad=1),
    "bs_not_pow2": dict(L=17, P=2, H=2, D=32, e=2, BS=12, NB=30, CT=48),
    "many_lp": dict(L=37, P=2, H=1, D=64, e=2, BS=16, NB=32, CT=128),
    "one_token_pages": dict(L=3, P=2, H=8, D=64, e=2, BS=1, NB=4096, CT=64),        # token-granular engines
    "max_layer_planes": dict(L=160, P=2, H=1, D=32, e=2, BS=8, NB=24, CT=32),     # LMC_MAX_LAYERS, K and V
    "blocks_outer": dict(L=4, P=2, H=4, D=64, e=2, BS=16, NB=48, CT=256, order="NP"),
    "blocks_outer_hnd_pad": dict(L=3, P=2, H=3, D=12, e=2, BS=4, NB=64, CT=32, order="NP", layout="HND",
                                 block_pad=8),
}


def _ctx(g, **kw):
    from paper_2510_09665_amd import lmc
    return lmc.Context(g, 4 * g.chunk_bytes, **kw)


@pytest.mark.parametrize("name", list(SHAPES))
@pytest.mark.parametrize("xcd_run", [None, 0, 4])
def test_gather_and_scatter_match_oracle(name, xcd_run):
    import torch
    from gpu_util import PagedKV, assert_layers_equal, slots_to_device
    g = W.KVGeometry(**SHAPES[name])
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    n_chunks = 3
    n_tok = n_chunks * g.CT
    assert n_tok <= g.n_slots
    slots = rng.permutation(g.n_slots)[:n_tok].astype(np.int64)
    slots[rng.integers(0, n_tok, 5)] = -1                 # tokens without a page
    slots[rng.integers(0, n_tok)] = -(2**40)
    src = PagedKV(g, np.arange(g.NB), rng)
    d_slots = slots_to_device(slots)
    with _ctx(g) as c:
        if xcd_run is not None:
            c.tune("xcd_run", xcd_run)
        staging = torch.full((n_chunks * g.chunk_bytes + 64,), 0xCD, dtype=torch.uint8, device="cuda")
        c.gather(src.dev, d_slots, n_chunks, staging, torch.cuda.current_stream())
        torch.cuda.synchronize()
        c.wait()
        want = oracle.gather(g, src.host, slots)
        got = staging.cpu().numpy()
        assert np.array_equal(got[:n_chunks * g.chunk_bytes].reshape(n_chunks, -1), want)
        assert (got[n_chunks * g.chunk_bytes:] == 0xCD).all()      # nothing past the last chunk

        # scatter the oracle's chunks into fresh pages under another mapping
        tau = rng.permutation(g.n_slots)[:n_tok].astype(np.int64)
        tau[rng.integers(0, n_tok, 4)] = -3
        dst = PagedKV(g, np.arange(g.NB), fill="sentinel")
        chunks_dev = torch.from_numpy(want.reshape(-1)).cuda()
        c.scatter(chunks_dev, slots_to_device(tau), n_chunks, dst.dev, torch.cuda.current_stream())
        torch.cuda.synchronize()
        c.wait()
        oracle.scatter(g, want, tau, dst.host)
        assert_layers_equal(dst.device_blocks_to_host(), dst.host, name)


def test_planes_larger_than_4_gib():
    """Offsets inside a layer beyond 32 bits: planes of 5 GiB (163840 pages of 32 KiB), the
    chunks' pages taken from both ends of the planes and from either side of the 4 GiB and
    8 GiB marks of the layer.  The oracle sees a compact copy of those pages; every other
    page must keep its sentinel."""
    import torch
    from gpu_util import PagedKV, assert_layers_equal, slots_to_device
    g = W.KVGeometry(L=1, P=2, H=8, D=128, e=2, BS=16, NB=163840, CT=256)
    assert g.plane_stride > (1 << 32) and g.layer_bytes > (1 << 33)
    rng = np.random.default_rng(4096)
    n_chunks = 3
    marks = [0, 1, 2, 131070, 131071, 131072, 131073, 98302, 98303, 98304, 98305,
             g.NB - 1, g.NB - 2, g.NB - 3]
    rest = rng.permutation(g.NB)
    rest = rest[~np.isin(rest, marks)][:2 * n_chunks * (g.CT // g.BS) - len(marks)]
    blocks = rng.permutation(np.concatenate([np.array(marks), rest]))
    half = blocks.size // 2
    src = PagedKV(g, blocks[:half], rng)
    dst = PagedKV(g, blocks[half:], fill="sentinel")
    slots = W.slots_from_blocks(g, src.blocks, n_chunks * g.CT)
    tau = W.slots_from_blocks(g, dst.blocks, n_chunks * g.CT)
    with _ctx(g) as c:
        staging = torch.full((n_chunks * g.chunk_bytes,), 0xCD, dtype=torch.uint8, device="cuda")
        c.gather(src.dev, slots_to_device(slots), n_chunks, staging, torch.cuda.current_stream())
        torch.cuda.synchronize()
        c.wait()
        want = oracle.gather(src.gc, src.host, src.compact_slots(slots))
        assert np.array_equal(staging.cpu().numpy().reshape(n_chunks, -1), want)
        c.scatter(staging, slots_to_device(tau), n_chunks, dst.dev, torch.cuda.current_stream())
        torch.cuda.synchronize()
        c.wait()
        oracle.scatter(dst.gc, want, dst.compact_slots(tau), dst.host)
        assert_layers_equal(dst.device_blocks_to_host(), dst.host, "planes of 5 GiB")
        assert dst.untracked_blocks_untouched() and src.untracked_blocks_untouched()


@pytest.mark.parametrize("name", list(SHAPES))
@pytest.mark.parametrize("xcd_run", [None, 4])
def test_scatter_in_destination_order_matches_oracle(name, xcd_run):
    """The launch shape for scatters that fill many pages per plane (rows visited in
    ascending slot order, the order built on the device) must write exactly what the
    oracle's scatter writes: every shape, tokens without a page, a slot outside the pages
    (skipped and reported), three calls in a row on the same scratch: a small one, a larger
    one (the scratch grows), a small one again."""
    import torch
    from gpu_util import PagedKV, assert_layers_equal, slots_to_device
    from paper_2510_09665_amd import lmc
    g = W.KVGeometry(**SHAPES[name])
    rng = np.random.default_rng(zlib.crc32(name.encode()) + 1)
    src = PagedKV(g, np.arange(g.NB), rng)
    with _ctx(g) as c:
        c.tune("scatter_order", 2)
        if xcd_run is not None:
            c.tune("xcd_run", xcd_run)
        for n_chunks in (1, 3, 1):
            n_tok = n_chunks * g.CT
            chunks = oracle.gather(g, src.host, rng.permutation(g.n_slots)[:n_tok].astype(np.int64))
            tau = rng.permutation(g.n_slots)[:n_tok].astype(np.int64)
            tau[rng.integers(0, n_tok, 4)] = -3
            tau[rng.integers(0, n_tok)] = -(2**40)
            bad = tau.copy()
            bad[1] = g.n_slots + 5                          # never dereferenced, reported by lmc_wait
            as_skip = tau.copy()
            as_skip[1] = -1
            dst = PagedKV(g, np.arange(g.NB), fill="sentinel")
            c.scatter(torch.from_numpy(chunks.reshape(-1)).cuda(), slots_to_device(bad), n_chunks, dst.dev,
                      torch.cuda.current_stream())
            torch.cuda.synchronize()
            with pytest.raises(lmc.LMCError) as e:
                c.wait()
            assert e.value.status == lmc.LMC_ERR_BADSLOT
            oracle.scatter(g, chunks, as_skip, dst.host)
            assert_layers_equal(dst.device_blocks_to_host(), dst.host, "%s, %d chunks" % (name, n_chunks))


def test_all_layers_in_one_allocation_with_blocks_outermost():
    """[NB][L][P][BS][H][D] in a single allocation: the per-layer base pointers lie inside
    each other's extents and a block's KV over all layers is contiguous.  Same four
    strides, same kernels; gather and scatter against the oracle on the same bytes."""
    import torch
    from gpu_util import slots_to_device
    g = W.BlockMajorKV(W.KVGeometry(L=5, P=2, H=4, D=64, e=2, BS=16, NB=48, CT=256))
    rng = np.random.default_rng(77)
    host = rng.integers(0, 256, g.total_bytes, dtype=np.uint8)
    layers_host = [host[g.layer_offset(l):] for l in range(g.L)]
    dev = torch.from_numpy(host).cuda()
    layers_dev = [dev.data_ptr() + g.layer_offset(l) for l in range(g.L)]
    n_chunks = 2
    slots = rng.permutation(g.n_slots)[:n_chunks * g.CT].astype(np.int64)
    slots[[3, 300]] = -1
    with _ctx(g) as c:
        staging = torch.empty(n_chunks * g.chunk_bytes, dtype=torch.uint8, device="cuda")
        c.gather(layers_dev, slots_to_device(slots), n_chunks, staging, torch.cuda.current_stream())
        torch.cuda.synchronize()
        want = oracle.gather(g, layers_host, slots)
        assert np.array_equal(staging.cpu().numpy().reshape(n_chunks, -1), want)
        tau = rng.permutation(g.n_slots)[:n_chunks * g.CT].astype(np.int64)
        tau[[0, 511]] = -9
        dst_host = np.full(g.total_bytes, 0x6B, dtype=np.uint8)
        dst_dev = torch.from_numpy(dst_host).cuda()
        c.scatter(staging, slots_to_device(tau), n_chunks, [dst_dev.data_ptr() + g.layer_offset(l) for l in range(g.L)],
                  torch.cuda.current_stream())
        torch.cuda.synchronize()
        c.wait()
        oracle.scatter(g, want, tau, [dst_host[g.layer_offset(l):] for l in range(g.L)])
        assert np.array_equal(dst_dev.cpu().numpy(), dst_host)


def test_empty_and_single_token_edge_cases():
    import torch
    from gpu_util import PagedKV, slots_to_device
    g = W.KVGeometry(**SHAPES["tiny_cfg1"])
    rng = np.random.default_rng(0)
    src = PagedKV(g, np.arange(g.NB), rng)
    with _ctx(g) as c:
        staging = torch.full((g.chunk_bytes,), 0x11, dtype=torch.uint8, device="cuda")
        c.gather(src.dev, slots_to_device(np.zeros(0)), 0, staging)       # zero chunks: no-op
        torch.cuda.synchronize()
        assert bool((staging == 0x11).all())
        # every token without a page: the chunk is all zeros
        c.gather(src.dev, slots_to_device(np.full(g.CT, -1)), 1, staging)
        torch.cuda.synchronize()
        assert bool((staging == 0).all())
        # all tokens in one page position (a gather may repeat slots)
        s = np.full(g.CT, 5, dtype=np.int64)
        c.gather(src.dev, slots_to_device(s), 1, staging)
        torch.cuda.synchronize()
        assert np.array_equal(staging.cpu().numpy(), oracle.gather_chunk(g, src.host, s))
        # the last slot of the pool
        s = np.full(g.CT, -1, dtype=np.int64)
        s[-1] = g.n_slots - 1
        c.gather(src.dev, slots_to_device(s), 1, staging)
        torch.cuda.synchronize()
        assert np.array_equal(staging.cpu().numpy(), oracle.gather_chunk(g, src.host, s))
        c.wait()


def test_bad_slot_is_skipped_and_reported():
    import torch
    from gpu_util import PagedKV, assert_layers_equal, slots_to_device
    from paper_2510_09665_amd import lmc
    g = W.KVGeometry(**SHAPES["tiny_cfg1"])
    rng = np.random.default_rng(1)
    src = PagedKV(g, np.arange(g.NB), rng)
    slots = rng.permutation(g.n_slots)[:g.CT].astype(np.int64)
    bad = slots.copy()
    bad[7] = g.n_slots
    bad[100] = 2**45
    as_skip = slots.copy()
    as_skip[[7, 100]] = -1
    chunk = oracle.gather_chunk(g, src.host, slots)
    with _ctx(g) as c:
        staging = torch.empty(g.chunk_bytes, dtype=torch.uint8, device="cuda")
        c.gather(src.dev, slots_to_device(bad), 1, staging)
        torch.cuda.synchronize()
        with pytest.raises(lmc.LMCError) as e:
            c.wait()
        assert e.value.status == lmc.LMC_ERR_BADSLOT
        c.wait()                                           # reported once
        assert np.array_equal(staging.cpu().numpy(), oracle.gather_chunk(g, src.host, as_skip))
        dst = PagedKV(g, np.arange(g.NB), fill="sentinel")
        c.scatter(torch.from_numpy(chunk).cuda(), slots_to_device(bad), 1, dst.dev)
        torch.cuda.synchronize()
        with pytest.raises(lmc.LMCError) as e:
            c.wait()
        assert e.value.status == lmc.LMC_ERR_BADSLOT
        oracle.scatter_chunk(g, chunk, as_skip, dst.host)
        assert_layers_equal(dst.device_blocks_to_host(), dst.host)
    # with validation the call itself fails and nothing is written
    with _ctx(g, flags=lmc.LMC_FLAG_VALIDATE_SLOTS) as c:
        dst = PagedKV(g, np.arange(g.NB), fill="sentinel")
        with pytest.raises(lmc.LMCError) as e:
            c.scatter(torch.from_numpy(chunk).cuda(), slots_to_device(bad), 1, dst.dev)
        assert e.value.status == lmc.LMC_ERR_BADSLOT
        torch.cuda.synchronize()
        assert_layers_equal(dst.device_blocks_to_host(), dst.host)
        c.scatter(torch.from_numpy(chunk).cuda(), slots_to_device(slots), 1, dst.dev)
        torch.cuda.synchronize()
        c.wait()


def test_misaligned_arguments_are_refused():
    import torch
    from gpu_util import PagedKV, slots_to_device
    from paper_2510_09665_amd import lmc
    g = W.KVGeometry(**SHAPES["tiny_cfg1"])
    src = PagedKV(g, np.arange(g.NB), np.random.default_rng(2))
    with _ctx(g) as c:
        staging = torch.empty(g.chunk_bytes + 16, dtype=torch.uint8, device="cuda")
        s = slots_to_device(np.arange(g.CT))
        with pytest.raises(lmc.LMCError) as e:
            c.gather(src.dev, s, 1, staging.data_ptr() + 4)
        assert e.value.status == lmc.LMC_ERR_INVAL
        with pytest.raises(lmc.LMCError) as e:
            c.gather([src.dev[0].data_ptr() + 8, src.dev[1]], s, 1, staging)
        assert e.value.status == lmc.LMC_ERR_INVAL


def test_link_measurements_agree_with_each_other():
    """The link's rate measured by the runtime's copy and by the library's copy kernel, one way
    and both ways at once: sane, close to each other, and the pool's content is preserved."""
    import torch
    from paper_2510_09665_amd import lmc
    g = W.KVGeometry(**SHAPES["tiny_cfg1"])
    n = 64 << 20
    with lmc.Context(g, 2 * n) as c:
        ids = np.arange(1, 9, dtype=np.uint64)
        payload = np.random.default_rng(3).integers(0, 256, 8 * g.chunk_bytes, dtype=np.uint8)
        c.put_host(ids, payload)
        h_rt, d_rt = c.measure_link(n, reps=2)
        h_k, d_k = c.measure_link_kernel(n, reps=2)
        for r in (h_rt, d_rt, h_k, d_k):
            assert 5.0 < r < 200.0
        assert 0.7 < h_k / h_rt < 1.4 and 0.7 < d_k / d_rt < 1.4
        two_way = [c.measure_link_duplex(n, reps=2)] + [c.measure_link_duplex_kernel(n, m, reps=2) for m in (1, 2, 3)]
        for r in two_way:
            assert max(h_rt, d_rt) * 0.9 < r < 2.05 * max(h_rt, d_rt, h_k, d_k)
        for k, i in enumerate(ids):
            assert np.array_equal(c.get_host(i), payload[k * g.chunk_bytes:(k + 1) * g.chunk_bytes])
        for bad in (lambda: c.measure_link_kernel(n + 8), lambda: c.measure_link_duplex_kernel(n, 4),
                    lambda: c.measure_link_duplex_kernel(2 * n, 1)):
            with pytest.raises(lmc.LMCError) as e:
                bad()
            assert e.value.status == lmc.LMC_ERR_INVAL


def test_copy_tiles_moves_tiles_in_the_given_order():
    import torch
    from gpu_util import slots_to_device
    g = W.KVGeometry(**SHAPES["tiny_cfg1"])
    rng = np.random.default_rng(9)
    n_tiles, T = 300, 4096
    with _ctx(g) as c:
        src = torch.randint(0, 256, (n_tiles * T,), dtype=torch.uint8, device="cuda")
        so, do = rng.permutation(n_tiles).astype(np.uint32), rng.permutation(n_tiles).astype(np.uint32)
        d_so, d_do = torch.from_numpy(so.view(np.int32)).cuda(), torch.from_numpy(do.view(np.int32)).cuda()
        for use_s, use_d in ((True, True), (True, False), (False, True), (False, False)):
            dst = torch.zeros(n_tiles * T + T, dtype=torch.uint8, device="cuda")
            c.copy_tiles(dst, d_do if use_d else None, src, d_so if use_s else None, n_tiles, 0, torch.cuda.current_stream())
            torch.cuda.synchronize()
            want = np.zeros((n_tiles + 1, T), dtype=np.uint8)
            s_np = src.cpu().numpy().reshape(n_tiles, T)
            want[do if use_d else np.arange(n_tiles)] = s_np[so if use_s else np.arange(n_tiles)]
            assert np.array_equal(dst.cpu().numpy().reshape(n_tiles + 1, T), want)
        # read-only and write-only modes touch nothing else / write a known pattern
        before = src.clone()
        dst = torch.zeros(n_tiles * T, dtype=torch.uint8, device="cuda")
        c.copy_tiles(dst, None, src, d_so, n_tiles, 1)
        c.copy_tiles(dst, d_do, src, None, 17, 2)
        torch.cuda.synchronize()
        assert torch.equal(src, before)
        got = dst.cpu().numpy().view(np.uint32).reshape(n_tiles, T // 4)
        for w in range(17):
            assert (got[do[w]] == w).all()
        assert (np.delete(got, do[:17], axis=0) == 0).all()


def test_copy_kernel():
    import torch
    g = W.KVGeometry(**SHAPES["tiny_cfg1"])
    with _ctx(g) as c:
        for n in (16, 4096 + 16, 3 * 2**20 + 48):
            src = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda")
            dst = torch.zeros(n + 16, dtype=torch.uint8, device="cuda")
            c.copy(dst, src, n, torch.cuda.current_stream())
            torch.cuda.synchronize()
            assert torch.equal(dst[:n], src) and bool((dst[n:] == 0).all())
