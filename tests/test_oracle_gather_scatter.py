"""Pins for the oracle's gather / scatter (paper section 5.1): each test fixes the
oracle against something that is not the oracle -- a closed form, numpy's own indexing
routines, or exhaustive enumeration on a tiny shape."""
import itertools

import numpy as np
import pytest

import oracle
from paper_2510_09665_amd import workloads as W

SHAPES = [
    dict(L=2, P=2, H=4, D=64, e=2, BS=16, NB=64, CT=256),                  # config 1
    dict(L=3, P=2, H=2, D=8, e=2, BS=4, NB=24, CT=32, layout="HND"),
    dict(L=3, P=2, H=2, D=8, e=2, BS=4, NB=24, CT=32, block_pad=48),
    dict(L=2, P=1, H=1, D=36, e=1, BS=8, NB=16, CT=32),                     # MLA-like, fp8
    dict(L=2, P=2, H=3, D=5, e=1, BS=4, NB=20, CT=16, layout="HND", block_pad=7),
    dict(L=2, P=2, H=2, D=8, e=2, BS=4, NB=24, CT=32, order="NP"),           # K and V page of a block adjacent
    dict(L=2, P=2, H=2, D=6, e=1, BS=4, NB=20, CT=16, order="NP", layout="HND", block_pad=5),
]


def _stamp(l, p, b, o, h, byte):
    """An injective-enough code of a byte's own coordinates (64-bit mix, low byte)."""
    x = (l * 1000003 + p * 10007 + b * 101 + o * 53 + h * 31 + byte * 7 + 0x9E3779B97F4A7C15) \
        & 0xFFFFFFFFFFFFFFFF
    x ^= x >> 29
    x = (x * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
    x ^= x >> 32
    return x & 0xFF


def _stamped_layers(g):
    layers = []
    run = g.D * g.e
    for l in range(g.L):
        a = np.full(g.layer_bytes, 0xEE, dtype=np.uint8)
        for p, b, o, h in itertools.product(range(g.P), range(g.NB), range(g.BS), range(g.H)):
            off = p * g.plane_stride + b * g.block_stride + o * g.token_stride + h * g.head_stride
            a[off:off + run] = [_stamp(l, p, b, o, h, k) for k in range(run)]
        layers.append(a)
    return layers


@pytest.mark.parametrize("kw", SHAPES[1:])
def test_gather_coordinate_stamp_closed_form(kw):
    g = W.KVGeometry(**kw)
    rng = np.random.default_rng(7)
    layers = _stamped_layers(g)
    slot = rng.permutation(g.n_slots)[:g.CT].astype(np.int64)
    slot[rng.integers(0, g.CT, 3)] = -1
    chunk = oracle.gather_chunk(g, layers, slot).reshape(g.L, g.P, g.CT, g.H, g.D * g.e)
    for l, p, t, h in itertools.product(range(g.L), range(g.P), range(g.CT), range(g.H)):
        s = int(slot[t])
        want = [0] * (g.D * g.e) if s < 0 else \
            [_stamp(l, p, s // g.BS, s % g.BS, h, k) for k in range(g.D * g.e)]
        assert chunk[l, p, t, h].tolist() == want, (l, p, t, h)


def test_identity_mapping_is_plain_copy():
    g = W.KVGeometry(**SHAPES[0])
    layers = W.random_layers(np.random.default_rng(1), g)
    slot = np.arange(g.CT, dtype=np.int64)
    chunk = oracle.gather_chunk(g, layers, slot).reshape(g.L, g.P, g.CT * g.R)
    for l in range(g.L):
        for p in range(g.P):
            start = p * g.plane_stride
            assert np.array_equal(chunk[l, p], layers[l][start:start + g.CT * g.R])


def _as_nd(g, layer):
    """numpy view [P][NB][BS][H][run] of an unpadded layer, any layout and page order."""
    run = g.D * g.e
    if g.order == "NP":
        inner = (g.BS, g.H, run) if g.layout == "NHD" else (g.H, g.BS, run)
        v = layer.reshape((g.NB, g.P) + inner).transpose(1, 0, 2, 3, 4)
        return v if g.layout == "NHD" else v.transpose(0, 1, 3, 2, 4)
    if g.layout == "NHD":
        return layer.reshape(g.P, g.NB, g.BS, g.H, run)
    return layer.reshape(g.P, g.NB, g.H, g.BS, run).transpose(0, 1, 3, 2, 4)


@pytest.mark.parametrize("kw", [SHAPES[0], SHAPES[1], SHAPES[3], SHAPES[5]])
def test_gather_equals_numpy_take(kw):
    g = W.KVGeometry(**kw)
    rng = np.random.default_rng(2)
    layers = W.random_layers(rng, g)
    slot = rng.permutation(g.n_slots)[:g.CT].astype(np.int64)
    chunk = oracle.gather_chunk(g, layers, slot).reshape(g.L, g.P, g.CT, g.H, g.D * g.e)
    for l in range(g.L):
        nd = _as_nd(g, layers[l]).reshape(g.P, g.NB * g.BS, g.H, g.D * g.e)
        assert np.array_equal(chunk[l], np.take(nd, slot, axis=1))


@pytest.mark.parametrize("kw", [SHAPES[0], SHAPES[1], SHAPES[3], SHAPES[5]])
def test_scatter_equals_numpy_indexed_assignment(kw):
    g = W.KVGeometry(**kw)
    rng = np.random.default_rng(3)
    chunk = rng.integers(0, 256, g.chunk_bytes, dtype=np.uint8)
    slot = rng.permutation(g.n_slots)[:g.CT].astype(np.int64)
    slot[::5] = -1
    got = [W.sentinel_layer(g, l) for l in range(g.L)]
    want = [a.copy() for a in got]
    oracle.scatter_chunk(g, chunk, slot, got)
    c5 = chunk.reshape(g.L, g.P, g.CT, g.H, g.D * g.e)
    keep = slot >= 0
    for l in range(g.L):
        nd = _as_nd(g, want[l])
        nd[:, slot[keep] // g.BS, slot[keep] % g.BS] = c5[l][:, keep]
        assert np.array_equal(got[l], want[l])


@pytest.mark.parametrize("kw", SHAPES)
def test_round_trip_and_untouched_bytes(kw):
    g = W.KVGeometry(**kw)
    rng = np.random.default_rng(4)
    src = W.random_layers(rng, g)
    sigma = rng.permutation(g.n_slots)[:g.CT].astype(np.int64)
    tau = rng.permutation(g.n_slots)[:g.CT].astype(np.int64)
    chunk = oracle.gather_chunk(g, src, sigma)
    dst = [W.sentinel_layer(g, l) for l in range(g.L)]
    before = [a.copy() for a in dst]
    oracle.scatter_chunk(g, chunk, tau, dst)
    run = g.D * g.e
    touched = [np.zeros(g.layer_bytes, dtype=bool) for _ in range(g.L)]
    for l, p, t, h in itertools.product(range(g.L), range(g.P), range(g.CT), range(g.H)):
        so = p * g.plane_stride + (sigma[t] // g.BS) * g.block_stride + \
            (sigma[t] % g.BS) * g.token_stride + h * g.head_stride
        do = p * g.plane_stride + (tau[t] // g.BS) * g.block_stride + \
            (tau[t] % g.BS) * g.token_stride + h * g.head_stride
        assert np.array_equal(dst[l][do:do + run], src[l][so:so + run])
        touched[l][do:do + run] = True
    for l in range(g.L):
        assert touched[l].sum() == g.P * g.CT * g.R
        assert np.array_equal(dst[l][~touched[l]], before[l][~touched[l]])
    # gather back from where it was scattered: the same chunk, bit for bit
    assert np.array_equal(oracle.gather_chunk(g, dst, tau), chunk)


def test_brute_force_every_injective_mapping():
    g = W.KVGeometry(L=1, P=2, H=1, D=2, e=1, BS=2, NB=3, CT=4)
    rng = np.random.default_rng(5)
    layer = rng.integers(1, 256, g.layer_bytes, dtype=np.uint8)
    pages = layer.reshape(g.P, g.NB, g.BS, g.D)       # [p][b][o][d]; H == 1
    n = 0
    for slot in itertools.permutations(range(g.n_slots), g.CT):
        for skip in (None, n % g.CT):
            s = np.array(slot, dtype=np.int64)
            if skip is not None:
                s[skip] = -1 - skip
            chunk = oracle.gather_chunk(g, [layer], s).reshape(g.P, g.CT, g.D)
            out = np.zeros(g.layer_bytes, dtype=np.uint8)
            oracle.scatter_chunk(g, chunk.reshape(-1), s, [out])
            out = out.reshape(g.P, g.NB, g.BS, g.D)
            want_out = np.zeros_like(out)
            for p in range(g.P):
                for t in range(g.CT):
                    for d in range(g.D):
                        if s[t] < 0:
                            assert chunk[p, t, d] == 0
                        else:
                            assert chunk[p, t, d] == pages[p, s[t] // g.BS, s[t] % g.BS, d]
                            want_out[p, s[t] // g.BS, s[t] % g.BS, d] = pages[p, s[t] // g.BS, s[t] % g.BS, d]
            assert np.array_equal(out, want_out)
        n += 1
    assert n == 360


def test_duplicate_slot_last_token_wins_and_bad_slot_rejected():
    g = W.KVGeometry(L=1, P=1, H=1, D=4, e=1, BS=2, NB=2, CT=4)
    chunk = np.arange(16, dtype=np.uint8)
    out = [np.zeros(g.layer_bytes, dtype=np.uint8)]
    oracle.scatter_chunk(g, chunk, np.array([1, 1, -1, 1]), out)
    assert out[0].reshape(4, 4)[1].tolist() == [12, 13, 14, 15]
    with pytest.raises(ValueError):
        oracle.gather_chunk(g, out, np.array([0, 1, 2, 4]))
    before = out[0].copy()
    with pytest.raises(ValueError):
        oracle.scatter_chunk(g, chunk, np.array([0, 1, 2, 4]), out)
    assert np.array_equal(out[0], before)


def test_size_arithmetic_of_the_paper():
    # Section 3.1 quotes a vLLM page of Llama-3.1-8B as about 62.5 KB and pages of 16-64 KB;
    # 16 tokens x (K and V) x 8 heads x 128 x 2 bytes is 64 KiB.
    g = W.geometry("llama3_8b")
    assert g.BS * g.P * g.R == 65536
    assert g.chunk_bytes == 32 * 2**20 and oracle.chunk_bytes(g) == g.chunk_bytes
    assert W.geometry("llama3_70b").chunk_bytes == 80 * 2**20
    assert W.geometry("mla_bf16").chunk_bytes == 17989632
    assert W.geometry("mla_fp8").chunk_bytes == 8994816
    assert W.geometry("tiny").chunk_bytes == 512 * 1024


def test_timing_driver_only_calls_the_oracle():
    """oracle/oracle_timing.c (the thread fan-out behind the benchmark's CPU baseline) must
    leave exactly what the oracle's own gather and scatter leave, whatever the thread count."""
    import dataclasses
    g = dataclasses.replace(W.geometry("tiny"), NB=48)
    rng = np.random.default_rng(5)
    n = 3
    src = [rng.integers(0, 256, g.layer_bytes, dtype=np.uint8) for _ in range(g.L)]
    blocks = rng.permutation(g.NB)
    s_slots = W.slots_from_blocks(g, blocks, n * g.CT)
    l_slots = W.slots_from_blocks(g, blocks[::-1].copy(), n * g.CT)
    want_pool = oracle.gather(g, src, s_slots)
    want_dst = [np.full(g.layer_bytes, 0x5A, dtype=np.uint8) for _ in range(g.L)]
    oracle.scatter(g, want_pool, l_slots, want_dst)
    for threads in (1, 2, 5):
        pool = np.zeros(n * g.chunk_bytes, dtype=np.uint8)
        buffers = np.zeros(threads * g.chunk_bytes, dtype=np.uint8)
        dst = [np.full(g.layer_bytes, 0x5A, dtype=np.uint8) for _ in range(g.L)]
        assert oracle.time_pass(g, src, dst, s_slots, l_slots, pool, buffers, threads, False) > 0
        assert np.array_equal(pool.reshape(n, -1), want_pool)
        assert oracle.time_pass(g, src, dst, s_slots, l_slots, pool, buffers, threads, True) > 0
        for a, b in zip(dst, want_dst):
            assert np.array_equal(a, b)


def test_layers_that_share_one_allocation_blocks_outermost():
    """[NB][L][P][BS][H][D] in one allocation (W.BlockMajorKV): the oracle, given layer
    pointers that lie inside one another's extents, must equal plain numpy indexing."""
    g = W.BlockMajorKV(W.KVGeometry(L=3, P=2, H=2, D=8, e=2, BS=4, NB=10, CT=8))
    rng = np.random.default_rng(0)
    host = rng.integers(0, 256, g.total_bytes, dtype=np.uint8)
    layers = [host[g.layer_offset(l):] for l in range(g.L)]
    slots = rng.permutation(g.n_slots)[:g.CT].astype(np.int64)
    v = host.reshape(g.NB, g.L, g.P, g.BS, g.R)
    want = np.stack([[v[slots // g.BS, l, p, slots % g.BS] for p in range(g.P)] for l in range(g.L)])
    chunk = oracle.gather_chunk(g, layers, slots)
    assert np.array_equal(chunk, want.reshape(-1))
    out = np.zeros_like(host)
    tau = rng.permutation(g.n_slots)[:g.CT].astype(np.int64)
    oracle.scatter_chunk(g, chunk, tau, [out[g.layer_offset(l):] for l in range(g.L)])
    ref = np.zeros_like(host).reshape(g.NB, g.L, g.P, g.BS, g.R)
    for l in range(g.L):
        for p in range(g.P):
            ref[tau // g.BS, l, p, tau % g.BS] = want[l, p]
    assert np.array_equal(out, ref.reshape(-1))
