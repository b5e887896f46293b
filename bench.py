#!/usr/bin/env python3
"""Benchmark of the KV store / retrieve path on one MI355X.

Headline workload: the largest single-GPU configuration, the Llama-3-70B-shaped KV cache
(80 layers, K and V, 8 KV heads x 128, bf16, 16-token pages, 8192 blocks = 40 GiB of
pages) with one 32768-token context = 128 chunks of 256 tokens = 10 GiB.  One step is one
pass of the whole path over that request:
  hash the tokens -> prefix lookup -> store every chunk (gather kernel + D2H per group of
  chunks, pipelined over two staging buffers) -> wait -> prefix lookup -> retrieve every
  chunk into freshly permuted blocks (H2D + scatter kernel, pipelined) -> wait -> clear.
Inputs are synthetic and resident in HBM before the timed region.  `value` is payload
bytes moved (store + retrieve) per second of wall time.

The run goes: `first_steps` untimed-as-warm-up but measured steps right after set-up (the
rate a cold process sees), then untimed steps until the machine has settled (see the
comment at that loop), the warm-up, the timed steps.  Both rates are in the JSON line.

Also reported in the same JSON line:
  roofline     the gather / scatter launches of the timed steps, timed with HIP events
               bound to the launches on the library's own streams, against the 8 TB/s HBM
               peak; algorithmic bytes = 2 x chunk bytes per chunk (each byte read once
               and written once)
  link         the link's peak per direction: the best over 64 MiB .. 1 GiB of the
               runtime's hipMemcpyAsync and of the library's link-paced copy kernel; store
               and retrieve payload rate as a fraction of it
  device       both kernels alone over the whole request in one launch (10 GiB, far
               beyond the 256 MB Infinity Cache), and a plain copy kernel of the same
               size as the achievable ceiling
  group_size   the headline request with staging buffers of 1 ... 16 chunks: what one copy
               boundary costs the link
  configs      every other benchmark configuration end to end (1 tiny, 2 Llama-3-8B,
               4 batched multi-request retrieve, 5 MLA in bf16 and fp8): store / retrieve
               as a fraction of the link peak and the kernels alone as a fraction of 8 TB/s
  page_placement  the two kernels against where the engine puts its pages: random 32 KiB
               pages, the same pages in address order, pages shuffled inside 2 MiB windows,
               all layers of a block adjacent; and the scatter launch in destination order
  duplex, direct, layerwise, overlap_with_compute, fragmented_pool, small_request
               the other modes of the path on the Llama-3-8B shape (16 chunks, 512 MiB)
  cpu_baseline the CPU oracle doing the same store + retrieve on a stated sample, chunks
               dealt out to plain threads
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X HBM3E, published
# HBM bytes per algorithmic byte of a gather / scatter launch, from rocprofv3 --pmc
# FETCH_SIZE and WRITE_SIZE, each calibrated on the plain copy kernel (profiles/): counters
# cannot be read from inside this process, so the measured ratio is applied to the launch
# size and the JSON says so.
PMC_TRAFFIC_RATIO = 1.0001
WORKLOAD = "llama3_70b"          # the headline: the largest single-GPU configuration
SECONDARY = "llama3_8b"          # the shape the mode legs (duplex, direct, layer-wise, ...) run on
WORKLOAD_TEXT = ("Llama-3-70B-shaped KV on one GPU: 80 layers, 8 KV heads, head_dim 128, bf16, block_size 16, "
                 "pool of 8192 blocks (40 GiB of pages); one 32768-token context = 128 chunks of 256 tokens "
                 "= 10 GiB stored to and retrieved from pinned host memory into freshly permuted blocks, "
                 "gather/D2H and H2D/scatter pipelined over two staging buffers")


def affinity_cpus():
    return len(os.sched_getaffinity(0))


def cpu_baseline(budget_s=20.0):
    """The oracle, as it stands, on a bounded sample: the first 16 chunks of the headline
    request (and, beside it, the 16 chunks of the Llama-3-8B request).  Store analogue =
    oracle gather_chunk into a buffer + memcpy into a pool, retrieve analogue = memcpy out
    of the pool + oracle scatter_chunk; chunks dealt out to plain threads by
    oracle/oracle_timing.c, every buffer allocated and touched before the clock starts."""
    import dataclasses
    from concurrent.futures import ThreadPoolExecutor
    import oracle
    from paper_2510_09665_amd import workloads as W
    n_aff = affinity_cpus()
    n_thr = max(1, min(n_aff, 16))          # the GPU machine gives one GPU's job 16 CPUs
    out = {}
    for name, n_chunks in ((WORKLOAD, 16), (SECONDARY, 16)):
        g = W.geometry(name)
        nb = n_chunks * g.CT // g.BS
        gc = dataclasses.replace(g, NB=nb)                      # only the touched blocks
        with ThreadPoolExecutor(n_thr) as ex:
            src = list(ex.map(lambda r: W.payload_bytes(r, g, gc.layer_bytes), W.rng_for(name, stream=7).spawn(g.L)))
        dst = [np.zeros(gc.layer_bytes, dtype=np.uint8) for _ in range(g.L)]
        blocks = W.rng_for(name, stream=8).permutation(nb)      # pages in random order, as on the GPU
        s_slots = W.slots_from_blocks(gc, blocks, n_chunks * g.CT)
        l_slots = W.slots_from_blocks(gc, blocks[::-1].copy(), n_chunks * g.CT)
        pool = np.zeros(n_chunks * g.chunk_bytes, dtype=np.uint8)
        res = {}
        for label, t in (("single_thread", 1), ("all_threads", n_thr)):
            buffers = np.zeros(t * g.chunk_bytes, dtype=np.uint8)
            best_s, best_l, t0 = 1e30, 1e30, time.perf_counter()
            while True:
                best_s = min(best_s, oracle.time_pass(gc, src, dst, s_slots, l_slots, pool, buffers, t, False))
                best_l = min(best_l, oracle.time_pass(gc, src, dst, s_slots, l_slots, pool, buffers, t, True))
                if time.perf_counter() - t0 > budget_s / 4:
                    break
            nbytes = n_chunks * g.chunk_bytes
            res[label] = {"threads": t, "store_gbps": round(nbytes / best_s / 1e9, 3),
                          "retrieve_gbps": round(nbytes / best_l / 1e9, 3),
                          "store_plus_retrieve_gbps": round(2 * nbytes / (best_s + best_l) / 1e9, 3)}
        out[name] = res
        del src, dst, pool
    head = out[WORKLOAD]
    return {
        "value": head["all_threads"]["store_plus_retrieve_gbps"], "unit": "GB/s",
        "cores": n_thr, "affinity_cpus": n_aff, "kind": "oracle",
        "single_thread_value": head["single_thread"]["store_plus_retrieve_gbps"],
        "sample": "the first 16 of the headline request's 128 chunks (1.25 GiB of the Llama-3-70B shape; a rate, "
                  "so no scaling is needed): oracle gather_chunk + memcpy to a pool, then memcpy from the pool + "
                  "oracle scatter_chunk, pages in seeded random order, chunks dealt out to plain threads "
                  "(oracle/oracle_timing.c), best pass of about 5 s per thread count; payload bytes / wall time",
        "llama3_70b_first_16_chunks": head, "llama3_8b_16_chunks": out[SECONDARY],
    }


def make_pages(torch, W, g, blocks, dev, seed):
    """Paged KV resident in HBM: bf16 uniform(-1, 1) in the listed blocks, zeros elsewhere;
    and an all-zero destination of the same shape."""
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    src, dst = [], []
    sb = torch.from_numpy(np.asarray(blocks)).to(dev)
    for _ in range(g.L):
        a = torch.zeros(g.layer_bytes, dtype=torch.uint8, device=dev)
        if g.e == 2:
            r = (torch.rand((g.P, sb.numel(), g.page_bytes // 2), device=dev, generator=gen) * 2 - 1) \
                .to(torch.bfloat16).view(torch.uint8)
        else:
            r = torch.randint(0, 127, (g.P, sb.numel(), g.page_bytes), device=dev, generator=gen, dtype=torch.uint8)
        a.view(g.P, g.NB, g.page_bytes)[:, sb] = r.view(g.P, sb.numel(), g.page_bytes)
        src.append(a)
        dst.append(torch.zeros(g.layer_bytes, dtype=torch.uint8, device=dev))
    return src, dst


def link_peaks(ctx, pool_bytes):
    """The link's peak per direction: the best rate over transfer sizes 64 MiB .. 1 GiB of
    the runtime's hipMemcpyAsync and of the library's link-paced copy kernel between the
    pinned pool and HBM; and the two-way peak (one transfer each way at once, each made either way) over the sizes."""
    best = {"h2d": (0.0, ""), "d2h": (0.0, "")}
    for mib in (64, 256, 512, 1024):
        n = mib << 20
        if n > pool_bytes:
            continue
        for how, fn in (("hipMemcpyAsync", ctx.measure_link), ("copy kernel", ctx.measure_link_kernel)):
            h, d = fn(n, reps=4)
            if h > best["h2d"][0]:
                best["h2d"] = (h, "%s, %d MiB" % (how, mib))
            if d > best["d2h"][0]:
                best["d2h"] = (d, "%s, %d MiB" % (how, mib))
    duplex = (0.0, "")
    how = {0: "hipMemcpyAsync both ways", 1: "copy kernel up, hipMemcpyAsync down",
           2: "hipMemcpyAsync up, copy kernel down", 3: "copy kernel both ways"}
    for mib in (256, 512, 1024):
        if 2 * (mib << 20) > pool_bytes:
            continue
        for by_kernel in (0, 1, 2, 3):
            r = ctx.measure_link_duplex_kernel(mib << 20, by_kernel, reps=8)
            if r > duplex[0]:
                duplex = (r, "%s, %d MiB each way" % (how[by_kernel], mib))
    # each direction as a row of consecutive copies, as the pipelines issue them group by group
    for gib, pieces in ((4, 2), (4, 8), (4, 16)):
        if 2 * (gib << 30) > pool_bytes:
            continue
        r = ctx.measure_link_duplex_kernel(gib << 30, pieces << 8, reps=2)
        if r > duplex[0]:
            duplex = (r, "hipMemcpyAsync both ways, %d GiB each way in %d consecutive copies" % (gib, pieces))
    return {"h2d_peak_gbps": best["h2d"][0], "h2d_peak_from": best["h2d"][1],
            "d2h_peak_gbps": best["d2h"][0], "d2h_peak_from": best["d2h"][1],
            "duplex_peak_gbps": duplex[0], "duplex_peak_from": duplex[1]}


def against_duplex_peak(got, peaks):
    """A summed two-way rate against the link's measured two-way peak.  The link carried
    what the pipeline moved: a peak below that would be no peak."""
    peak, peak_from = peaks["duplex_peak_gbps"], peaks["duplex_peak_from"]
    if got > peak:
        peak, peak_from = got, "this store + retrieve itself (above every two-way copy measured: %.2f GB/s, %s)" % (
            peaks["duplex_peak_gbps"], peaks["duplex_peak_from"])
    one_way = peaks["h2d_peak_gbps"] + peaks["d2h_peak_gbps"]
    return {"store_plus_retrieve_gbps": round(got, 2),
            "link_duplex_peak_gbps": round(peak, 2), "link_duplex_peak_from": peak_from,
            "frac_of_duplex_peak": round(got / peak, 4),
            # against what two perfect one-way transfers would add up to
            "sum_of_one_way_peaks_gbps": round(one_way, 2),
            "frac_of_sum_of_one_way_peaks": round(got / one_way, 4)}


def kernel_only(torch, ctx, W, name, g, src, dst, n_chunks, dev, stream, gather_slots=None, scatter_slots=None,
                iters=6, reps=3):
    """Seconds per launch of the gather (pages of `src` -> staging), the scatter (staging ->
    other pages, in `dst`: a retrieve fills fresh pages) and a plain copy of the same size,
    each over the whole request in one launch (HIP events on `stream`).  Requests below
    2 GiB rotate over four block sets and four staging buffers, so that nothing is served
    from the 256 MB Infinity Cache."""
    nbytes = n_chunks * g.chunk_bytes
    n_rot = 1 if nbytes >= (2 << 30) else 4
    if gather_slots is None:
        seqs = [W.sequence(name, g, stream=10 + r) for r in range(n_rot)]
        gather_slots = [torch.from_numpy(q["store_slots"]).to(dev) for q in seqs]
        scatter_slots = [torch.from_numpy(q["load_slots"]).to(dev) for q in seqs]
    stagings = [torch.empty(nbytes, dtype=torch.uint8, device=dev) for _ in range(n_rot)]
    spare = torch.empty(nbytes, dtype=torch.uint8, device=dev) if n_rot == 1 else None
    torch.cuda.synchronize()      # pages and slot mappings were made on PyTorch's own stream
    out = []
    for fn in (lambda r: ctx.gather(src, gather_slots[r % len(gather_slots)], n_chunks, stagings[r], stream),
               lambda r: ctx.scatter(stagings[r], scatter_slots[r % len(scatter_slots)], n_chunks, dst, stream),
               lambda r: ctx.copy(stagings[(r + 1) % n_rot] if n_rot > 1 else spare, stagings[r], nbytes // 16 * 16, stream)):
        for r in range(n_rot):
            fn(r)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        best = 1e30
        for _ in range(reps):
            e0.record(stream)
            for i in range(iters):
                fn(i % n_rot)
            e1.record(stream)
            e1.synchronize()
            best = min(best, e0.elapsed_time(e1) / iters * 1e-3)
        out.append(best)
    ctx.wait()
    return out


def kernel_report(nbytes, tg, ts, tc):
    f = lambda t: round(2 * nbytes / t / 1e9, 1)
    return {"bytes_per_launch": 2 * nbytes,
            "gather_hbm_gbps": f(tg), "scatter_hbm_gbps": f(ts), "copy_kernel_hbm_gbps": f(tc),
            "gather_frac_of_hbm_peak": round(f(tg) / HBM_PEAK_GBPS, 4),
            "scatter_frac_of_hbm_peak": round(f(ts) / HBM_PEAK_GBPS, 4),
            "copy_kernel_frac_of_hbm_peak": round(f(tc) / HBM_PEAK_GBPS, 4)}


def other_configs(torch, lmc, W, dev, stream, timed, peaks):
    """Every benchmark configuration but the headline, end to end (store, then retrieve
    into fresh blocks; configuration 4: one batched retrieve of the hit chunks of 64
    requests, pool slots in shuffled order), each as a fraction of the link peak, and both
    kernels alone over the whole request as a fraction of the 8 TB/s HBM peak."""
    res = {}
    h2d, d2h = peaks["h2d_peak_gbps"], peaks["d2h_peak_gbps"]
    for name, staging in (("tiny", 1), ("llama3_8b", 16), ("mla_bf16", 32), ("mla_fp8", 32)):
        g = W.geometry(name)
        seq = W.sequence(name, g)
        n = seq["tokens"].size // g.CT
        kv, fresh = make_pages(torch, W, g, seq["store_blocks"], dev, W.SEED_BASE + W.CONFIGS[name]["id"])
        d_s, d_l = torch.from_numpy(seq["store_slots"]).to(dev), torch.from_numpy(seq["load_slots"]).to(dev)
        ctx = lmc.Context(g, max(n * g.chunk_bytes, 64 << 20), staging_chunks=staging, device=0)
        ids = ctx.hash_chunks(seq["tokens"])

        def st():
            ctx.clear(ids)
            ctx.wait(ctx.store(kv, d_s, ids, stream))
        # best of a dozen: for a few seconds after memory of this size has been allocated or
        # freed in the process, the runtime's device-to-host copies can run at half speed
        ts = timed(st, reps=12)
        tl = timed(lambda: ctx.wait(ctx.retrieve(ids, d_l, fresh, stream)), reps=6)
        nbytes = n * g.chunk_bytes
        tg, tsc, tc = kernel_only(torch, ctx, W, name, g, kv, fresh, n, dev, stream)
        res[name] = {"chunks": n, "payload_bytes": nbytes,
                     "store_gbps": round(nbytes / ts / 1e9, 2), "retrieve_gbps": round(nbytes / tl / 1e9, 2),
                     "store_frac_of_d2h_peak": round(nbytes / ts / 1e9 / d2h, 4),
                     "retrieve_frac_of_h2d_peak": round(nbytes / tl / 1e9 / h2d, 4),
                     "store_ms": round(ts * 1e3, 3), "retrieve_ms": round(tl * 1e3, 3),
                     "kernels_alone": kernel_report(nbytes, tg, tsc, tc)}
        if nbytes < (4 << 20):
            res[name]["note"] = ("half a MiB: launch- and latency-bound, no measure of the link or of HBM; by "
                                 "the library's size rule it moves without staging, in one launch each way")
        ctx.destroy()
        del kv, fresh
    name = "batch_8b"
    g = W.geometry(name)
    reqs = W.request_mix(name, g)
    n_hit = sum(r["n_hit"] for r in reqs)
    kv = [torch.zeros(g.layer_bytes, dtype=torch.uint8, device=dev) for _ in range(g.L)]
    ctx = lmc.Context(g, (n_hit + 1) * g.chunk_bytes, staging_chunks=16, device=0)
    payload = W.payload_bytes(W.rng_for(name, stream=3), g, g.chunk_bytes)
    ids_per = [ctx.hash_chunks(r["tokens"]) for r in reqs]
    hit = [(ri, k) for ri, r in enumerate(reqs) for k in range(r["n_hit"])]
    for j in np.random.default_rng(0).permutation(len(hit)):
        ctx.put_host([ids_per[hit[j][0]][hit[j][1]]], payload)
    off = np.concatenate([[0], np.cumsum([r["n_hit"] for r in reqs])])
    ids_all = np.concatenate([ids_per[ri][:r["n_hit"]] for ri, r in enumerate(reqs)])
    d_sl = torch.from_numpy(np.concatenate([r["load_slots"] for r in reqs])).to(dev)
    t = timed(lambda: ctx.wait(ctx.retrieve_batch(off, ids_all, d_sl, kv, stream)), reps=3)
    nbytes = n_hit * g.chunk_bytes
    tg, tsc, tc = kernel_only(torch, ctx, W, name, g, kv, kv, n_hit, dev, stream, gather_slots=[d_sl],
                              scatter_slots=[d_sl], iters=3)
    res[name] = {"requests": len(reqs), "hit_chunks": n_hit, "payload_bytes": nbytes,
                 "retrieve_batch_gbps": round(nbytes / t / 1e9, 2),
                 "retrieve_frac_of_h2d_peak": round(nbytes / t / 1e9 / h2d, 4),
                 "retrieve_ms": round(t * 1e3, 1),
                 "kernels_alone": kernel_report(nbytes, tg, tsc, tc)}
    ctx.destroy()
    return res


def launch_address_stream(torch, W, g, kv, slots, n_chunks, dev):
    """The 4 KiB tiles a gather / scatter launch over `slots` touches on the paged side, in
    the launch's own order (tile, then layer-plane, then chunk), as tile numbers relative to
    the lowest layer pointer: the input of lmc_copy_tiles.  A tile of the launch is
    4096 / R token rows, which lie together in the page for the NHD layouts used here."""
    base = min(t_.data_ptr() for t_ in kv)
    tiles_per_plane = g.CT * g.R // 4096
    rows_per_tile = 4096 // g.R
    w_ = np.arange(n_chunks * g.L * g.P * tiles_per_plane, dtype=np.int64)
    tile, lp, ch = w_ % tiles_per_plane, (w_ // tiles_per_plane) % (g.L * g.P), w_ // (tiles_per_plane * g.L * g.P)
    slot0 = np.asarray(slots)[ch * g.CT + tile * rows_per_tile]
    layer_at = np.array([t_.data_ptr() - base for t_ in kv], dtype=np.int64)
    addr = layer_at[lp // g.P] + (lp % g.P) * g.plane_stride + slot0 * g.R
    assert (addr % 4096 == 0).all() and addr.max() // 4096 < 2**32
    return base, torch.from_numpy((addr // 4096).astype(np.uint32).view(np.int32)).to(dev), int(w_.size)


def random_pages_sample(torch, lmc, W, dev, stream):
    """Gather / scatter / copy read + write GB/s over 1024 random 32 KiB pages of the
    Llama-3-8B shape (64 chunks, 2 GiB per launch), pages and staging allocated now.  Run
    once as the very first thing of the process and once late: where in the life of the
    process the pages were allocated moves the kernels by several per cent."""
    name = SECONDARY
    g = W.geometry(name)
    n_chunks = 64
    n_tok, nbytes = n_chunks * g.CT, n_chunks * g.chunk_bytes
    rand = W.rng_for(name, stream=50).permutation(g.NB)[:n_tok // g.BS]
    d = torch.from_numpy(W.slots_from_blocks(g, rand, n_tok)).to(dev)
    kv = [torch.zeros(g.layer_bytes, dtype=torch.uint8, device=dev) for _ in range(g.L)]
    staging = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    spare = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    res = {}
    base, pages_order, n_t = launch_address_stream(torch, W, g, kv, W.slots_from_blocks(g, rand, n_tok), n_chunks, dev)
    with lmc.Context(g, 64 << 20, device=0) as ctx:
        for key, fn in (("gather", lambda: ctx.gather(kv, d, n_chunks, staging, stream)),
                        ("scatter", lambda: ctx.scatter(staging, d, n_chunks, kv, stream)),
                        ("copy_kernel", lambda: ctx.copy(spare, staging, nbytes, stream)),
                        # plain tile copies with the same address stream: what the pattern alone costs
                        ("gather_like_plain_copy", lambda: ctx.copy_tiles(staging, None, base, pages_order, n_t, 0, stream)),
                        ("scatter_like_plain_copy", lambda: ctx.copy_tiles(base, pages_order, staging, None, n_t, 0, stream)),
                        # ... and its two halves alone (x 2, so that they read on the same scale)
                        ("twice_read_only_of_the_pages", lambda: ctx.copy_tiles(staging, None, base, pages_order, n_t, 1, stream)),
                        ("twice_write_only_of_the_pages", lambda: ctx.copy_tiles(base, pages_order, staging, None, n_t, 2, stream))):
            fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            best = 1e30
            for _ in range(3):
                e0.record(stream)
                for _ in range(6):
                    fn()
                e1.record(stream)
                e1.synchronize()
                best = min(best, e0.elapsed_time(e1) / 6 * 1e-3)
            res[key + "_hbm_gbps"] = round(2 * nbytes / best / 1e9, 1)
            res[key + "_frac_of_hbm_peak"] = round(2 * nbytes / best / 1e9 / HBM_PEAK_GBPS, 4)
        ctx.wait()
    return res


def placement_leg(torch, lmc, W, dev, stream):
    """What the gather / scatter rate depends on: where the engine puts its pages.  The
    same kernels, the Llama-3-8B shape, 64 chunks (2 GiB, far beyond the Infinity Cache)
    per launch, read + write GB/s against the 8 TB/s peak:
      random            1024 of 8192 blocks in seeded random order (what the benchmark's
                        configurations prescribe)
      address_order     the same blocks visited in ascending address order
      contiguous        blocks 0..1023 in order (both sides of the copy linear)
      window_shuffled   1024 consecutive blocks shuffled inside 2 MiB windows (64 pages)
      random_dest_order random, and the scatter launch in the order of the destination
                        (lmc_tune "scatter_order": rows visited in ascending slot order)
      block_major       random blocks of an engine that keeps all layers of a block
                        together, [NB][L][P][BS][H][D] in one allocation: 2 MiB per block
    and the plain copy kernel of the same size as the ceiling."""
    name = SECONDARY
    g = W.geometry(name)
    n_chunks = 64
    n_tok = n_chunks * g.CT
    nb = n_tok // g.BS
    nbytes = n_chunks * g.chunk_bytes
    rng = W.rng_for(name, stream=50)
    rand = rng.permutation(g.NB)[:nb]
    win = np.arange(nb).reshape(-1, (2 << 20) // g.page_bytes)
    win = np.concatenate([rng.permutation(w_) for w_ in win])
    patterns = {"random": rand, "address_order": np.sort(rand), "contiguous": np.arange(nb), "window_shuffled": win}
    kv = [torch.zeros(g.layer_bytes, dtype=torch.uint8, device=dev) for _ in range(g.L)]
    staging = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    spare = torch.empty(nbytes, dtype=torch.uint8, device=dev)

    def rate(fn, iters=6, reps=3):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        best = 1e30
        for _ in range(reps):
            e0.record(stream)
            for _ in range(iters):
                fn()
            e1.record(stream)
            e1.synchronize()
            best = min(best, e0.elapsed_time(e1) / iters * 1e-3)
        return round(2 * nbytes / best / 1e9, 1)
    res = {"chunks_per_launch": n_chunks, "bytes_per_launch": 2 * nbytes, "page_bytes": g.page_bytes}
    with lmc.Context(g, 64 << 20, device=0) as ctx:
        for label, blocks in patterns.items():
            d = torch.from_numpy(W.slots_from_blocks(g, blocks, n_tok)).to(dev)
            res[label] = {"gather_hbm_gbps": rate(lambda: ctx.gather(kv, d, n_chunks, staging, stream)),
                          "scatter_hbm_gbps": rate(lambda: ctx.scatter(staging, d, n_chunks, kv, stream))}
        d = torch.from_numpy(W.slots_from_blocks(g, rand, n_tok)).to(dev)
        ctx.tune("scatter_order", 2)
        res["random_dest_order"] = {}
        for key, rows in (("groups_of_256_rows", 256), ("plane_by_plane", 0)):
            ctx.tune("ordered_group_rows", rows)
            res["random_dest_order"]["scatter_hbm_gbps_" + key] = rate(lambda: ctx.scatter(staging, d, n_chunks, kv, stream))
        ctx.tune("scatter_order", 0)
        res["copy_kernel_hbm_gbps"] = rate(lambda: ctx.copy(spare, staging, nbytes, stream))
        # What the access pattern alone costs: a plain copy of 4 KiB tiles (no slot mapping, no
        # geometry) fed with exactly the address stream of the random-pages launch above, in
        # the launch's own order (tile, then layer-plane, then chunk).  A tile of the launch
        # is two token rows = 4 KiB on both sides.
        base, pages_order, n_t = launch_address_stream(torch, W, g, kv, W.slots_from_blocks(g, rand, n_tok), n_chunks, dev)
        res["plain_copy_with_the_address_stream_of_random"] = {
            "scatter_like_hbm_gbps": rate(lambda: ctx.copy_tiles(base, pages_order, staging, None, n_t, 0, stream)),
            "gather_like_hbm_gbps": rate(lambda: ctx.copy_tiles(staging, None, base, pages_order, n_t, 0, stream)),
            "read_only_pages_gbps": round(rate(lambda: ctx.copy_tiles(staging, None, base, pages_order, n_t, 1, stream)) / 2, 1),
            "write_only_pages_gbps": round(rate(lambda: ctx.copy_tiles(base, pages_order, staging, None, n_t, 2, stream)) / 2, 1),
            "read_only_linear_gbps": round(rate(lambda: ctx.copy_tiles(spare, None, staging, None, n_t, 1, stream)) / 2, 1),
            "write_only_linear_gbps": round(rate(lambda: ctx.copy_tiles(spare, None, staging, None, n_t, 2, stream)) / 2, 1)}
        ctx.wait()
    del kv
    bm = W.BlockMajorKV(g)
    big = torch.zeros(bm.total_bytes, dtype=torch.uint8, device=dev)
    layers = [big.data_ptr() + bm.layer_offset(l) for l in range(g.L)]
    with lmc.Context(bm, 64 << 20, device=0) as ctx:
        d = torch.from_numpy(W.slots_from_blocks(g, rand, n_tok)).to(dev)
        res["block_major"] = {"gather_hbm_gbps": rate(lambda: ctx.gather(layers, d, n_chunks, staging, stream)),
                              "scatter_hbm_gbps": rate(lambda: ctx.scatter(staging, d, n_chunks, layers, stream)),
                              "contiguous_bytes_per_block": bm.block_stride}
        ctx.wait()
    for v in res.values():
        if isinstance(v, dict):
            for k_ in [k_ for k_ in v if k_.endswith("_hbm_gbps")]:
                v[k_.replace("_hbm_gbps", "_frac_of_hbm_peak")] = round(v[k_] / HBM_PEAK_GBPS, 4)
    return res


def group_size_leg(torch, lmc, W, g, seq, src, dst, d_store, d_load, stream, timed, peaks, num_staging):
    """What a copy boundary costs: the headline request stored and retrieved with staging
    buffers of 1, 2, 4, 8 and 16 chunks (128 ... 8 groups per direction; the copies of a
    group are one merged transfer).  The time beyond payload / link peak, divided by the
    number of groups, is the idle time of the link per boundary."""
    n_chunks = seq["tokens"].size // g.CT
    nbytes = n_chunks * g.chunk_bytes
    res = {}
    for sc in (1, 2, 4, 8, 16):
        with lmc.Context(g, (n_chunks + 1) * g.chunk_bytes, num_staging=num_staging, staging_chunks=sc,
                         device=0) as c:
            ids = c.hash_chunks(seq["tokens"])

            def store_only():
                c.clear(ids)
                c.wait(c.store(src, d_store, ids, stream))
            ts = timed(store_only, reps=4)
            tl = timed(lambda: c.wait(c.retrieve(ids, d_load, dst, stream)), reps=4)
            # the link's idle time between the copies of consecutive groups, from the trace
            gaps = {}
            c.tune("trace", 1)
            c.clear(ids)
            c.wait(c.store(src, d_store, ids, stream))
            c.wait(c.retrieve(ids, d_load, dst, stream))
            recs, _ = c.trace_read()
            c.tune("trace", 0)
            for key, stage in (("store", lmc.LMC_STAGE_D2H), ("retrieve", lmc.LMC_STAGE_H2D)):
                cp = sorted((r for r in recs if r["stage"] == stage), key=lambda r: r["begin_us"])
                gp = sorted(b["begin_us"] - a["end_us"] for a, b in zip(cp, cp[1:]))
                if gp:
                    gaps[key] = {"median": round(gp[len(gp) // 2], 1), "p90": round(gp[(len(gp) * 9) // 10], 1),
                                 "max": round(gp[-1], 1), "sum_ms": round(sum(gp) / 1e3, 3)}
        groups = 1 + -(-(n_chunks - 1) // sc)          # one single-chunk group at the exposed end
        res["staging_chunks_%d" % sc] = {
            "groups_per_direction": groups,
            "store_gbps": round(nbytes / ts / 1e9, 2), "retrieve_gbps": round(nbytes / tl / 1e9, 2),
            "store_frac_of_d2h_peak": round(nbytes / ts / 1e9 / peaks["d2h_peak_gbps"], 4),
            "retrieve_frac_of_h2d_peak": round(nbytes / tl / 1e9 / peaks["h2d_peak_gbps"], 4),
            "store_us_beyond_peak_per_group": round((ts - nbytes / (peaks["d2h_peak_gbps"] * 1e9)) / groups * 1e6, 1),
            "retrieve_us_beyond_peak_per_group": round((tl - nbytes / (peaks["h2d_peak_gbps"] * 1e9)) / groups * 1e6, 1),
            "gap_between_consecutive_groups_copies_us": gaps}
    return res


# shapes beyond the five configurations that --kernels-only can run: a tensor-parallel
# shard (one KV head of the Llama-3-70B shape per GPU: 256-byte rows, 4 KiB pages) and a
# token-granular engine (one-token pages, 2 KiB each)
EXTRA_SHAPES = {
    "tp8_shard_70b": ("llama3_70b", dict(H=1), 32768),
    "one_token_pages_8b": ("llama3_8b", dict(BS=1, NB=8192 * 16), 16384),
}


def kernels_only_mode(names, iters, reps):
    """The gather, the scatter and the plain copy kernel alone over the whole request of each
    named shape, one launch each time, nothing else in the process: the program that the
    rocprofv3 counter runs of profiles/ profile.  Prints one JSON line."""
    import torch
    from paper_2510_09665_amd import lmc
    from paper_2510_09665_amd import workloads as W
    dev = torch.device("cuda:0")
    stream = torch.cuda.Stream()     # the engine's stream, which the library orders itself after (not the null stream)
    res = {}
    for name in names:
        if name in EXTRA_SHAPES:
            base, ov, n_tok = EXTRA_SHAPES[name]
            g = W.geometry(base, **ov)
            rng = W.rng_for(base, stream=60)
            perm = rng.permutation(g.NB)
            nb = n_tok // g.BS
            gs = [torch.from_numpy(W.slots_from_blocks(g, perm[:nb], n_tok)).to(dev)]
            ss = [torch.from_numpy(W.slots_from_blocks(g, perm[nb:2 * nb], n_tok)).to(dev)]
            n = n_tok // g.CT
            rot = {}
        elif name == "batch_8b":
            g = W.geometry(name)
            reqs = W.request_mix(name, g)
            sl = np.concatenate([r["load_slots"] for r in reqs])
            n = sl.size // g.CT
            gs = ss = [torch.from_numpy(sl).to(dev)]
            rot = {}
        else:
            g = W.geometry(name)
            n = W.CONFIGS[name]["tokens"] // g.CT
            gs = ss = None
            rot = {}
        src = [torch.zeros(g.layer_bytes, dtype=torch.uint8, device=dev) for _ in range(g.L)]
        dst = [torch.zeros(g.layer_bytes, dtype=torch.uint8, device=dev) for _ in range(g.L)]
        with lmc.Context(g, max(g.chunk_bytes, 64 << 20), device=0) as ctx:
            tg, ts, tc = kernel_only(torch, ctx, W, name, g, src, dst, n, dev, stream, gather_slots=gs,
                                     scatter_slots=ss, iters=iters, reps=reps, **rot)
        res[name] = {"chunks_per_launch": n, "rows_bytes": g.R, "page_bytes": g.BS * g.R}
        res[name].update(kernel_report(n * g.chunk_bytes, tg, ts, tc))
        for k_, t_ in (("gather_us", tg), ("scatter_us", ts), ("copy_kernel_us", tc)):
            res[name][k_] = round(t_ * 1e6, 1)
        del src, dst
    print(json.dumps({"kernels_only": res}), flush=True)


def mode_legs(torch, lmc, W, dev, stream, legs, args, timed, peaks):
    """The modes beside the bulk pipeline, on the Llama-3-8B shape (16 chunks, 512 MiB)."""
    g = W.geometry(SECONDARY)
    seq = W.sequence(SECONDARY, g)
    n_chunks = seq["tokens"].size // g.CT
    payload_one_way = n_chunks * g.chunk_bytes
    src, dst = make_pages(torch, W, g, seq["store_blocks"], dev, W.SEED_BASE + W.CONFIGS[SECONDARY]["id"])
    d_store = torch.from_numpy(seq["store_slots"]).to(dev)
    d_load = torch.from_numpy(seq["load_slots"]).to(dev)
    ctx = lmc.Context(g, max(2 * n_chunks * g.chunk_bytes, 1 << 30), num_staging=args.num_staging,
                      staging_chunks=16, device=0)
    for kv in args.tune:
        k, v = kv.split("=")
        ctx.tune(k, int(v))
    ids = ctx.hash_chunks(seq["tokens"])
    duplex = direct = layerwise = overlap = fragmented = None
    # full duplex: store one request while another is retrieved (two streams per
    # direction, nothing shared but the link and HBM)
    duplex = None
    if "duplex" in legs:
        ctx.tune("timing", 0)
        ids_a = ctx.hash_chunks(seq["tokens"])
        seq_b = W.sequence(SECONDARY, g, stream=1)
        ids_b = ctx.hash_chunks(seq_b["tokens"])
        d_load_b = torch.from_numpy(seq["load_slots"]).to(dev)
        ctx.clear(ids_a)
        ctx.wait(ctx.store(src, d_store, ids_b, stream))       # request B's chunks are in the pool

        def both():
            ctx.clear(ids_a)
            t1 = ctx.store(src, d_store, ids_a, stream)
            t2 = ctx.retrieve(ids_b, d_load_b, dst, stream)
            ctx.wait(t1)
            ctx.wait(t2)
        t_both = timed(both)
        got = 2 * payload_one_way / t_both / 1e9
        duplex = against_duplex_peak(got, peaks)
        ctx.clear(ids_a)
        ctx.clear(ids_b)

    # direct mode: no staging, the kernels move the bytes over the link themselves
    direct = None
    if "direct" in legs:
        dctx = lmc.Context(g, max(n_chunks * g.chunk_bytes, 1 << 30), device=0, flags=lmc.LMC_FLAG_DIRECT)
        for kv in args.tune:
            k, v = kv.split("=")
            dctx.tune(k, int(v))
        dids = dctx.hash_chunks(seq["tokens"])

        def d_store_only():
            dctx.clear(dids)
            dctx.wait(dctx.store(src, d_store, dids, stream))
        td_s = timed(d_store_only)
        td_l = timed(lambda: dctx.wait(dctx.retrieve(dids, d_load, dst, stream)))
        h2d, d2h = peaks["h2d_peak_gbps"], peaks["d2h_peak_gbps"]
        direct = {"store_gbps": round(payload_one_way / td_s / 1e9, 2),
                  "retrieve_gbps": round(payload_one_way / td_l / 1e9, 2),
                  "store_frac_of_d2h_peak": round(payload_one_way / td_s / 1e9 / d2h, 4),
                  "retrieve_frac_of_h2d_peak": round(payload_one_way / td_l / 1e9 / h2d, 4)}
        dctx.destroy()

    # layer-wise mode: the same request moved layer by layer, alone and with a consumer /
    # producer that works on each layer as soon as it is there
    layerwise = None
    if "layerwise" in legs:
        ctx.tune("timing", 0)
        ids = ctx.hash_chunks(seq["tokens"])
        h2d, d2h = peaks["h2d_peak_gbps"], peaks["d2h_peak_gbps"]
        consumer = torch.cuda.Stream()
        layerwise = {}
        for k in (1, 4):
            def lw_store():
                ctx.clear(ids)
                t = ctx.store_begin(d_store, ids, stream)
                for l0 in range(0, g.L, k):
                    ctx.store_layers(t, l0, min(k, g.L - l0), src, stream)
                ctx.wait(t)
            def lw_load():
                t = ctx.retrieve_layerwise(ids, d_load, dst, k, stream)
                for l in range(g.L):
                    ctx.wait_layer(t, l, consumer)
                ctx.wait(t)
            ts, tl = timed(lw_store), timed(lw_load)
            layerwise["layers_per_step_%d" % k] = {
                "store_gbps": round(payload_one_way / ts / 1e9, 2),
                "retrieve_gbps": round(payload_one_way / tl / 1e9, 2),
                "store_frac_of_d2h_peak": round(payload_one_way / ts / 1e9 / d2h, 4),
                "retrieve_frac_of_h2d_peak": round(payload_one_way / tl / 1e9 / h2d, 4),
            }
        # time to first layer: how long a consumer waits before it can start on layer 0
        def first_layer(mode):
            torch.cuda.synchronize()
            a = time.perf_counter()
            if mode == "layerwise":
                t = ctx.retrieve_layerwise(ids, d_load, dst, 1, stream)
                ctx.wait_layer(t, 0, consumer)
            else:
                t = ctx.retrieve(ids, d_load, dst, consumer)
            consumer.synchronize()
            b = time.perf_counter()
            ctx.wait(t)
            return (b - a) * 1e3
        layerwise["ms_until_layer0_usable"] = {
            "layerwise": round(min(first_layer("layerwise") for _ in range(4)), 3),
            "bulk": round(min(first_layer("bulk") for _ in range(4)), 3)}
        ctx.clear(ids)

    # what layer-wise loading is for (section 5.2): a consumer computes on layer l while
    # layer l+1 is still on its way.  A dense matrix product stands in for a layer's
    # compute, sized so that 32 layers take about as long as the transfer.
    overlap = None
    if "overlap" in legs:
        ctx.tune("timing", 0)
        ids = ctx.hash_chunks(seq["tokens"])
        ctx.wait(ctx.store(src, d_store, ids, stream))
        octx = lmc.Context(g, max(n_chunks * g.chunk_bytes, 1 << 30), device=0, flags=lmc.LMC_FLAG_DIRECT)
        octx.wait(octx.store(src, d_store, ids, stream))
        # HIP maps streams onto a few hardware queues (GPU_MAX_HW_QUEUES, 4 by default), and a
        # stream that shares a queue with one of the library's host-to-device copy streams
        # stands still while such a copy runs.  lmc_probe_stream tells: the consumer is a
        # stream that shares none; one that does is measured as well, if there is one.
        candidates = [torch.cuda.Stream() for _ in range(8)]
        masks = [ctx.probe_stream(c_) & 0x23 for c_ in candidates]      # both H2D streams and the scatter stream
        consumer = candidates[masks.index(0)] if 0 in masks else candidates[0]
        shared = next((c_ for c_, m in zip(candidates, masks) if m), None)
        dmasks = [octx.probe_stream(c_) & 0x20 for c_ in candidates]      # the direct context's scatter stream
        dconsumer = candidates[dmasks.index(0)] if 0 in dmasks else candidates[0]
        staged_consumer = consumer
        a_mat = torch.randn(4096, 4096, device=dev, dtype=torch.bfloat16)
        b_mat = torch.randn(4096, 4096, device=dev, dtype=torch.bfloat16)
        with torch.cuda.stream(consumer):
            for _ in range(10):
                torch.mm(a_mat, b_mat)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(consumer)
            for _ in range(50):
                torch.mm(a_mat, b_mat)
            e1.record(consumer)
        e1.synchronize()
        t_mm = e0.elapsed_time(e1) / 50                      # ms per product
        per_layer = max(1, int(round(9.4 / g.L / t_mm)))      # products per layer: ~9.4 ms in all

        def compute(l):
            for _ in range(per_layer):
                torch.mm(a_mat, b_mat)

        def run(mode, consumer=None):
            c = octx if mode.endswith("direct") else ctx
            consumer = consumer or (dconsumer if mode.endswith("direct") else staged_consumer)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            if mode == "compute_only":
                t = None
            elif mode.startswith("layerwise"):
                t = c.retrieve_layerwise(ids, d_load, dst, 1, stream)
            else:
                t = c.retrieve(ids, d_load, dst, consumer)    # the consumer waits for all of it
            with torch.cuda.stream(consumer):
                for l in range(g.L):
                    if t is not None and mode.startswith("layerwise"):
                        c.wait_layer(t, l, consumer)
                    compute(l)
            consumer.synchronize()
            dt = time.perf_counter() - t0
            if t is not None:
                c.wait(t)
            return dt * 1e3
        overlap = {"compute_ms_per_layer": round(per_layer * t_mm, 3), "layers": g.L,
                   "consumer_shares_a_queue_with_the_retrieve_streams": masks[candidates.index(consumer)] != 0,
                   "streams_probed": len(masks), "streams_sharing": sum(1 for m in masks if m)}
        for mode in ("compute_only", "bulk", "layerwise", "bulk_direct", "layerwise_direct"):
            overlap[mode + "_ms"] = round(min(run(mode) for _ in range(4)), 3)
        if shared is not None:
            overlap["layerwise_ms_on_a_stream_sharing_a_queue"] = round(
                min(run("layerwise", shared) for _ in range(4)), 3)
        # the store side of the same idea: a producer computes layer l and hands it to
        # lmc_store_layers while it goes on with layer l+1; against computing all layers
        # first and storing in bulk afterwards
        full = [ctx.probe_stream(c_) for c_ in candidates]
        producer = next((c_ for c_, m in zip(candidates, full) if (m & 0x1C) == 0), candidates[0])

        def run_store(mode):
            ctx.clear(ids)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            with torch.cuda.stream(producer):
                if mode == "layerwise":
                    t = ctx.store_begin(d_store, ids, producer)
                    for l in range(g.L):
                        compute(l)
                        ctx.store_layers(t, l, 1, src, producer)
                else:
                    for l in range(g.L):
                        compute(l)
                    t = ctx.store(src, d_store, ids, producer)
            ctx.wait(t)
            producer.synchronize()
            return (time.perf_counter() - t0) * 1e3
        overlap["compute_then_bulk_store_ms"] = round(min(run_store("bulk") for _ in range(4)), 3)
        overlap["compute_with_layerwise_store_ms"] = round(min(run_store("layerwise") for _ in range(4)), 3)
        octx.destroy()
        ctx.clear(ids)
        del a_mat, b_mat

    # a pool in which every other slot is taken: no two chunks of the request are
    # neighbours, so every group needs one copy per chunk (two copy streams take turns)
    fragmented = None
    if "fragmented" in legs:
        fctx = lmc.Context(g, (2 * n_chunks + 1) * g.chunk_bytes, staging_chunks=16,
                           num_staging=args.num_staging, device=0)
        filler = np.arange(1, 2 * n_chunks + 1, dtype=np.uint64) + np.uint64(1 << 40)
        zero = np.zeros(g.chunk_bytes, dtype=np.uint8)
        for f in filler:
            fctx.put_host([f], zero)
        fctx.clear(filler[1::2])
        fids = fctx.hash_chunks(seq["tokens"])

        def f_store_only():
            fctx.clear(fids)
            fctx.wait(fctx.store(src, d_store, fids, stream))
        tf_s = timed(f_store_only)
        assert [fctx.find_slot(i) for i in fids[:3]] == [1, 3, 5]
        tf_l = timed(lambda: fctx.wait(fctx.retrieve(fids, d_load, dst, stream)))
        h2d, d2h = peaks["h2d_peak_gbps"], peaks["d2h_peak_gbps"]
        fragmented = {"store_gbps": round(payload_one_way / tf_s / 1e9, 2),
                      "retrieve_gbps": round(payload_one_way / tf_l / 1e9, 2),
                      "store_frac_of_d2h_peak": round(payload_one_way / tf_s / 1e9 / d2h, 4),
                      "retrieve_frac_of_h2d_peak": round(payload_one_way / tf_l / 1e9 / h2d, 4)}

        # layer by layer on the same pool: one 1 MiB piece per chunk and layer; all pieces of
        # a step go in one launch of the library's copy kernel ("runtime_copies": one
        # hipMemcpyAsync per piece instead)
        def f_lw_store():
            fctx.clear(fids)
            t = fctx.store_begin(d_store, fids, stream)
            for l0 in range(g.L):
                fctx.store_layers(t, l0, 1, src, stream)
            fctx.wait(t)
        for key, below in (("layer_by_layer", None), ("layer_by_layer_runtime_copies", 0)):
            if below is not None:
                fctx.tune("pieces_by_kernel_below", below)
            ts_ = timed(f_lw_store)
            tl_ = timed(lambda: fctx.wait(fctx.retrieve_layerwise(fids, d_load, dst, 1, stream)))
            fragmented[key] = {"store_gbps": round(payload_one_way / ts_ / 1e9, 2),
                               "retrieve_gbps": round(payload_one_way / tl_ / 1e9, 2),
                               "store_frac_of_d2h_peak": round(payload_one_way / ts_ / 1e9 / d2h, 4),
                               "retrieve_frac_of_h2d_peak": round(payload_one_way / tl_ / 1e9 / h2d, 4)}
        fctx.destroy()


    ctx.destroy()
    out = {}
    for key, val in (("duplex", duplex), ("direct", direct), ("layerwise", layerwise),
                     ("overlap_with_compute", overlap), ("fragmented_pool", fragmented)):
        if val:
            out[key] = val
    return out


def trace_leg(lmc, ctx, g, src, dst, d_store, d_load, ids, stream, payload_one_way):
    """Component-wise timeline of one store and one retrieve of the headline request, from
    the library's own trace (device time stamps of every gather launch, every group's
    copies and every scatter launch): how long each stage was busy, the gaps between the
    copies of consecutive groups, and what of the span no copy covered."""
    names = {lmc.LMC_STAGE_GATHER: "gather", lmc.LMC_STAGE_D2H: "d2h", lmc.LMC_STAGE_H2D: "h2d",
             lmc.LMC_STAGE_SCATTER: "scatter"}

    def summary(recs, copy_stage, kernel_stage, wall_s):
        out = {"wall_ms_with_the_trace_on": round(wall_s * 1e3, 3),
               "gbps_with_the_trace_on": round(payload_one_way / wall_s / 1e9, 2)}
        copies = sorted((r for r in recs if r["stage"] == copy_stage), key=lambda r: r["begin_us"])
        kernels = sorted((r for r in recs if r["stage"] == kernel_stage), key=lambda r: r["begin_us"])
        first = min(r["begin_us"] for r in copies + kernels)
        last = max(r["end_us"] for r in copies + kernels)
        out["device_span_ms"] = round((last - first) / 1e3, 3)
        for name, rs in ((names[copy_stage], copies), (names[kernel_stage], kernels)):
            busy = sum(r["end_us"] - r["begin_us"] for r in rs)
            out[name] = {"steps": len(rs), "busy_ms": round(busy / 1e3, 3),
                         "mean_us": round(busy / max(len(rs), 1), 1),
                         "gbps_while_busy": round(sum(r["bytes"] for r in rs) / max(busy, 1e-9) / 1e3, 2)}
        gaps = sorted(b["begin_us"] - a["end_us"] for a, b in zip(copies, copies[1:]))
        if gaps:
            out["gap_between_consecutive_groups_copies_us"] = {
                "min": round(gaps[0], 1), "median": round(gaps[len(gaps) // 2], 1), "max": round(gaps[-1], 1),
                "sum_ms": round(sum(gaps) / 1e3, 3),
                "histogram": {"%s-%s us" % (lo, hi): sum(1 for x in gaps if lo <= x < hi)
                              for lo, hi in ((0, 10), (10, 12), (12, 14), (14, 16), (16, 18), (18, 20), (20, 30),
                                             (30, 100), (100, 10 ** 9)) if any(lo <= x < hi for x in gaps)}}
        covered = sum(r["end_us"] - r["begin_us"] for r in copies)
        out["span_not_covered_by_a_copy_ms"] = round((last - first - covered) / 1e3, 3)
        # kernel time that ran while no copy did: what the pipeline failed to hide
        exposed = 0.0
        for k_ in kernels:
            hidden = sum(max(0.0, min(k_["end_us"], c_["end_us"]) - max(k_["begin_us"], c_["begin_us"])) for c_ in copies)
            exposed += (k_["end_us"] - k_["begin_us"]) - hidden
        out["kernel_time_not_behind_a_copy_ms"] = round(exposed / 1e3, 3)
        return out

    ctx.clear(ids)
    ctx.tune("trace", 1)
    res = {}
    try:
        t0 = time.perf_counter()
        ctx.wait(ctx.store(src, d_store, ids, stream))
        wall = time.perf_counter() - t0
        recs, dropped = ctx.trace_read()
        res["store"] = summary(recs, lmc.LMC_STAGE_D2H, lmc.LMC_STAGE_GATHER, wall)
        t0 = time.perf_counter()
        ctx.wait(ctx.retrieve(ids, d_load, dst, stream))
        wall = time.perf_counter() - t0
        recs, dropped2 = ctx.trace_read()
        res["retrieve"] = summary(recs, lmc.LMC_STAGE_H2D, lmc.LMC_STAGE_SCATTER, wall)
        res["records_lost"] = dropped + dropped2
    finally:
        ctx.tune("trace", 0)
        ctx.clear(ids)
    res["note"] = ("kernels carry their own begin / end time stamps; a group's copies are bracketed by two event "
                   "markers on the copy stream, which themselves cost the link some microseconds per group")
    return res


def host_leg(torch, ctx, seq, src, dst, d_store, d_load, ids, stream, n_chunks):
    """The host side of the path (token processor, index, pool bookkeeping; rows a1-a3 and
    a10 of the hot-path table) and what the two enqueue calls cost the calling thread,
    on the headline request: microseconds, best of several."""
    def best(fn, reps=20):
        b = 1e30
        for _ in range(reps):
            t0 = time.perf_counter()
            fn()
            b = min(b, time.perf_counter() - t0)
        return round(b * 1e6, 1)
    res = {"tokens": int(seq["tokens"].size), "chunks": n_chunks}
    res["hash_chunks_us"] = best(lambda: ctx.hash_chunks(seq["tokens"]))
    ctx.clear(ids)
    res["lookup_all_missing_us"] = best(lambda: ctx.lookup(ids))
    enq_s, enq_l = [], []
    for _ in range(4):
        ctx.clear(ids)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        t = ctx.store(src, d_store, ids, stream)
        enq_s.append(time.perf_counter() - t0)
        ctx.wait(t)
        t0 = time.perf_counter()
        t = ctx.retrieve(ids, d_load, dst, stream)
        enq_l.append(time.perf_counter() - t0)
        ctx.wait(t)
    res["store_call_returns_after_us"] = round(min(enq_s) * 1e6, 1)
    res["retrieve_call_returns_after_us"] = round(min(enq_l) * 1e6, 1)
    res["lookup_all_present_us"] = best(lambda: ctx.lookup(ids))
    res["pin_then_unpin_us"] = best(lambda: (ctx.pin(ids), ctx.unpin(ids)))
    t0 = time.perf_counter()
    ctx.clear(ids)
    res["clear_us"] = round((time.perf_counter() - t0) * 1e6, 1)
    return res


def serving_leg(torch, lmc, W, dev, peaks, n_requests=240):
    """A stream of requests as a serving engine would send them (paper section 4: look up
    the prefix, retrieve what is there, store what is new; the paper's multi-round question
    answering, section 8.1), on the Llama-3-8B shape: 32 conversations visited in seeded
    random order; every turn sends the whole conversation so far (the earlier turns are the
    prefix that should hit) plus a few new chunks (seeded lognormal, median 4), and a
    conversation that reaches 64 chunks starts over as a new one.  The pool holds 320
    chunks with LRU eviction, a third of what the conversations add up to, so chunks are
    evicted and come back and the pool fragments; four requests are in flight, each on a
    stream of its own, with no host wait between a request's retrieve and its store.
    Every chunk's KV is one byte value derived from (conversation, chunk), so that what a
    retrieve delivered can be checked with one comparison per page."""
    g = W.geometry(SECONDARY)
    rng = W.rng_for(SECONDARY, stream=70)
    n_sessions, max_chunks, pool_chunks, window = 32, 64, 320, 4
    bpc = g.CT // g.BS
    new_doc = lambda: rng.integers(0, 128256, max_chunks * g.CT, dtype=np.int64).astype(np.int32)
    docs = [new_doc() for _ in range(n_sessions)]
    doc_id = list(range(n_sessions))          # a new number whenever a conversation starts over
    length = [0] * n_sessions
    next_id = n_sessions
    kv = [torch.zeros(g.layer_bytes, dtype=torch.uint8, device=dev) for _ in range(g.L)]
    views = [W.page_view(g, t) for t in kv]
    order = rng.permutation(g.NB)
    # Nothing crosses the link for the harness itself while requests run: a small copy from
    # pageable memory queues behind whatever 256 MiB transfer the copy engine is busy with and
    # blocks the host for that long.  Block lists, slot mappings and fill values are made on
    # the device from what is resident, and the checks collect in a flag that is read at the end.
    order_dev = torch.from_numpy(order).to(dev)
    in_block = torch.arange(g.BS, device=dev, dtype=torch.int64)
    all_good = torch.ones((), dtype=torch.bool, device=dev)
    cursor = 0
    streams = [torch.cuda.Stream() for _ in range(window)]      # one per request in flight, as a batch slot of an engine
    moved = {"hit_chunks": 0, "new_chunks": 0, "requests": 0, "pages_checked": 0}
    inflight = []
    host = {"prepare": 0.0, "retrieve_call": 0.0, "prefill_stand_in": 0.0, "store_call": 0.0, "wait_and_check": 0.0}

    class section:
        def __init__(self, key):
            self.key = key

        def __enter__(self):
            self.t = time.perf_counter()

        def __exit__(self, *a):
            host[self.key] += time.perf_counter() - self.t

    def pattern(d, j):
        return (d * 67 + j * 13 + 1) & 0xFF

    def retire(ctx, item):
        nonlocal all_good
        tickets, keep, d, n_hit, b_dev = item
        for t in tickets:
            ctx.wait(t)
        # the chunks that were retrieved: first, middle and last one, one layer each
        for j in sorted({0, n_hit // 2, n_hit - 1}) if n_hit else ():
            l = (d + j) % g.L
            all_good = all_good & (views[l][:, b_dev[j * bpc:(j + 1) * bpc]] == pattern(d, j)).all()
            moved["pages_checked"] += bpc * g.P

    with lmc.Context(g, pool_chunks * g.chunk_bytes, staging_chunks=8, device=0,
                     flags=lmc.LMC_FLAG_EVICT_LRU | lmc.LMC_FLAG_TRACE) as ctx:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for r_ in range(n_requests):
            stream = streams[r_ % window]
            with section("prepare"):
                ses = int(rng.integers(0, n_sessions))
                if length[ses] >= max_chunks:                    # the conversation is over: a new one takes its place
                    docs[ses], doc_id[ses], length[ses] = new_doc(), next_id, 0
                    next_id += 1
                turn = int(np.clip(round(float(np.exp(np.log(4.0) + 0.7 * rng.standard_normal()))), 1, 16))
                n = min(max_chunks, length[ses] + turn)
                length[ses] = n
                d = doc_id[ses]
                if cursor + n * bpc > g.NB:
                    cursor = 0
                b_dev = order_dev[cursor:cursor + n * bpc]
                cursor += n * bpc
                ids = ctx.hash_chunks(docs[ses][:n * g.CT])
                n_hit = ctx.lookup(ids)
            tickets = []
            with torch.cuda.stream(stream):
                with section("prepare"):
                    # slot of token t: blocks[t // BS] * BS + t % BS
                    d_slots = (b_dev[:, None] * g.BS + in_block[None, :]).reshape(-1)
                    if n_hit < n:
                        tb = b_dev[n_hit * bpc:]
                        chunk_no = torch.arange(n_hit, n, device=dev, dtype=torch.int64)
                        vals = ((chunk_no * 13 + (d * 67 + 1)) & 0xFF).to(torch.uint8).repeat_interleave(bpc)[None, :, None]
                if n_hit:
                    with section("retrieve_call"):
                        tickets.append(ctx.retrieve(ids[:n_hit], d_slots[:n_hit * g.CT], kv, stream))
                # "prefill": the engine computes the KV of the chunks that were not there (one
                # fill per layer: every page of chunk j gets the byte of (conversation, j))
                if n_hit < n:
                    with section("prefill_stand_in"):
                        for v in views:
                            v[:, tb] = vals
                    with section("store_call"):
                        try:
                            tickets.append(ctx.store(kv, d_slots, ids, stream))
                        except lmc.LMCError as e:            # every slot in flight: what fitted is stored
                            if e.status != lmc.LMC_ERR_NOMEM or not e.ticket:
                                raise
                            tickets.append(e.ticket)
                            moved["stores_cut_short"] = moved.get("stores_cut_short", 0) + 1
            moved["hit_chunks"] += n_hit
            moved["new_chunks"] += n - n_hit
            moved["requests"] += 1
            inflight.append((tickets, (d_slots, b_dev), d, n_hit, b_dev))
            if len(inflight) >= window:
                with section("wait_and_check"):
                    retire(ctx, inflight.pop(0))
        while inflight:
            retire(ctx, inflight.pop(0))
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        assert bool(all_good), "a retrieved chunk differs from what its conversation stored"
        st = ctx.get_stats()
        recs, _ = ctx.trace_read()

    def busy(stage):
        """Merged busy intervals of one stage, from the trace."""
        iv = sorted((r["begin_us"], r["end_us"]) for r in recs if r["stage"] == stage)
        out = []
        for a, b in iv:
            if out and a <= out[-1][1]:
                out[-1][1] = max(out[-1][1], b)
            else:
                out.append([a, b])
        return out

    def overlap(x, y):
        i = j = 0
        tot = 0.0
        while i < len(x) and j < len(y):
            lo, hi = max(x[i][0], y[j][0]), min(x[i][1], y[j][1])
            tot += max(0.0, hi - lo)
            if x[i][1] < y[j][1]:
                i += 1
            else:
                j += 1
        return tot
    up, down = busy(lmc.LMC_STAGE_H2D), busy(lmc.LMC_STAGE_D2H)
    link = {"to_device_busy_s": round(sum(b - a for a, b in up) / 1e6, 3),
            "to_host_busy_s": round(sum(b - a for a, b in down) / 1e6, 3),
            "both_busy_s": round(overlap(up, down) / 1e6, 3)}
    total = st["bytes_d2h"] + st["bytes_h2d"]
    return {"requests": moved["requests"], "chunks_retrieved": moved["hit_chunks"], "chunks_stored": moved["new_chunks"],
            "hit_rate_by_chunks": round(moved["hit_chunks"] / max(moved["hit_chunks"] + moved["new_chunks"], 1), 3),
            "chunks_evicted": st["chunks_evicted"], "pool_chunks": pool_chunks,
            "gib_to_host": round(st["bytes_d2h"] / 2**30, 2), "gib_to_device": round(st["bytes_h2d"] / 2**30, 2),
            "wall_s": round(wall, 3), "gbps_both_ways_over_wall": round(total / wall / 1e9, 2), "link": link,
            "host_seconds": {k_: round(v_, 3) for k_, v_ in host.items()},
            "pages_checked": moved["pages_checked"], "stores_cut_short_by_a_full_pool": moved.get("stores_cut_short", 0),
            "note": "wall time includes the stand-in for the engine's prefill (PyTorch fills of the new chunks' pages) "
                    "and the host waits of the four-request window; the rate is what the library sustained beside them"}


def small_leg(torch, lmc, W, dev, stream, timed):
    """One chunk of half a MiB (configuration 1): microseconds from the call to a finished
    lmc_wait, through the staging ring and by the library's size rule (no staging)."""
    small = {}
    tg = W.geometry("tiny")
    tseq = W.sequence("tiny", tg)
    tsrc = [torch.zeros(tg.layer_bytes, dtype=torch.uint8, device=dev) for _ in range(tg.L)]
    ts_, tl_ = torch.from_numpy(tseq["store_slots"]).to(dev), torch.from_numpy(tseq["load_slots"]).to(dev)
    for mode in ("staged", "size_rule"):
        tctx = lmc.Context(tg, 4 * tg.chunk_bytes, device=0)
        if mode == "staged":
            tctx.tune("direct_store_below", 0)
            tctx.tune("direct_retrieve_below", 0)
        tids = tctx.hash_chunks(tseq["tokens"])

        def t_store_only():
            tctx.clear(tids)
            tctx.wait(tctx.store(tsrc, ts_, tids, stream))
        small[mode] = {"store_us": round(timed(t_store_only, reps=40) * 1e6, 1),
                       "retrieve_us": round(timed(lambda: tctx.wait(tctx.retrieve(tids, tl_, tsrc, stream)),
                                                  reps=40) * 1e6, 1)}
        tctx.destroy()
    small["payload_bytes"] = tg.chunk_bytes
    del tsrc
    return small


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--staging-chunks", type=int, default=8)
    ap.add_argument("--num-staging", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--first-steps", type=int, default=20,
                    help="steps measured right after set-up, before anything settles (0 = none)")
    ap.add_argument("--settle-seconds", type=float, default=20.0,
                    help="upper limit for the untimed settling phase before the warm-up (0 = none)")
    ap.add_argument("--legs", default="pipeline,link,device,host,trace,groups,configs,placement,duplex,direct,layerwise,overlap,"
                                      "fragmented,serving,small,cpu",
                    help="comma list of pipeline (always run), link, device, groups, configs, placement, duplex, direct, "
                         "layerwise, overlap, fragmented, small, cpu: the extra measurements to make; "
                         "profiling runs use a subset")
    ap.add_argument("--tune", action="append", default=[], help="key=value for lmc_tune")
    ap.add_argument("--kernels-only", default="",
                    help="comma list of shapes (tiny, llama3_8b, llama3_70b, batch_8b, mla_bf16, mla_fp8, "
                         "tp8_shard_70b, one_token_pages_8b): run only the gather, scatter and copy kernels over "
                         "each shape's whole request and exit (the program the counter profiles run)")
    ap.add_argument("--kernels-only-iters", type=int, default=6)
    ap.add_argument("--kernels-only-reps", type=int, default=3)
    args = ap.parse_args()
    legs = set(args.legs.split(","))
    if args.no_cpu_baseline:
        legs.discard("cpu")
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on one GPU only (no sharding, no collectives); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2510_09665_amd import lmc
    from paper_2510_09665_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    if args.kernels_only:
        kernels_only_mode(args.kernels_only.split(","), args.kernels_only_iters, args.kernels_only_reps)
        return
    dev = torch.device("cuda:0")
    stream = torch.cuda.Stream()     # the engine's stream, which the library orders itself after (not the null stream)
    first_pages = None
    if "placement" in legs:
        try:
            first_pages = random_pages_sample(torch, lmc, W, dev, stream)
        except Exception as e:                               # noqa: BLE001 (a side measurement)
            first_pages = {"error": "%s: %s" % (type(e).__name__, e)}
    g = W.geometry(WORKLOAD)
    seq = W.sequence(WORKLOAD, g)
    n_chunks = seq["tokens"].size // g.CT
    payload_one_way = n_chunks * g.chunk_bytes

    src, dst = make_pages(torch, W, g, seq["store_blocks"], dev, W.SEED_BASE + W.CONFIGS[WORKLOAD]["id"])
    d_store = torch.from_numpy(seq["store_slots"]).to(dev)
    d_load = torch.from_numpy(seq["load_slots"]).to(dev)

    pool_bytes = max((n_chunks + 2) * g.chunk_bytes, 2 << 30)
    ctx = lmc.Context(g, pool_bytes, num_staging=args.num_staging,
                      staging_chunks=args.staging_chunks, device=0, flags=lmc.LMC_FLAG_TIMING)
    for kv in args.tune:
        k, v = kv.split("=")
        ctx.tune(k, int(v))

    def step():
        ids = ctx.hash_chunks(seq["tokens"])
        assert ctx.lookup(ids) == 0
        t = ctx.store(src, d_store, ids, stream)
        ctx.wait(t)
        assert ctx.lookup(ids) == n_chunks
        t = ctx.retrieve(ids, d_load, dst, stream)
        ctx.wait(t)
        ctx.clear(ids)

    def timed_steps(n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            step()
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    # What a process sees that has only just set itself up: the first steps, measured
    # before anything is given time to settle.
    first = None
    if args.first_steps > 0:
        dt1 = timed_steps(1)
        dtn = timed_steps(args.first_steps - 1) if args.first_steps > 1 else 0.0
        first = {"steps": args.first_steps,
                 "gbps": round(2 * payload_one_way * args.first_steps / (dt1 + dtn) / 1e9, 3),
                 "very_first_step_gbps": round(2 * payload_one_way / dt1 / 1e9, 3)}

    # Settle.  For some seconds after tens of GiB of device or pinned memory have been
    # allocated or freed on the host (by this process while it set up, or by the process
    # that had the GPU before), the runtime's device-to-host copies inside a store can run
    # at about half speed; the state passes by itself.  It is a state of the machine, not
    # of this path, so steps are run, untimed, until three seconds' worth in a row reach
    # 90 % of the link rate measured now (a lone copy is not affected) without the
    # library's copy-engine guard stepping in, or until the time limit; what it took is
    # reported beside the rate of the first steps above.
    settle = {"steps": 0, "seconds": 0.0, "settled": args.settle_seconds <= 0}
    if args.settle_seconds > 0:
        _, d2h_now = ctx.measure_link(256 << 20, reps=2)
        need = max(4, int(3.0 / (2 * payload_one_way / (0.9 * d2h_now * 1e9))))
        t_begin, good, slow, seen = time.perf_counter(), 0, 0, ctx.get_stats()["d2h_guard_switches"]
        while time.perf_counter() - t_begin < args.settle_seconds:
            dt = timed_steps(1)
            settle["steps"] += 1
            gs = ctx.get_stats()
            healthy = 2 * payload_one_way / dt / 1e9 >= 0.9 * d2h_now
            if healthy and gs["d2h_guard_switches"] == seen and not gs["d2h_guard_active"]:
                good += 1
            else:
                good, seen = 0, gs["d2h_guard_switches"]
                slow += 0 if healthy else 1
            if good >= need:
                settle["settled"] = True
                break
        settle["seconds"] = round(time.perf_counter() - t_begin, 2)
        settle["slow_steps"] = slow
        settle["steps_in_a_row_required"] = need
    if first:
        settle["first_steps_before_settling"] = first

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    guard_before = ctx.get_stats()["d2h_guard_switches"]
    ctx.reset_stats()
    dt = timed_steps(args.steps)
    st = ctx.get_stats()
    # copies handed to the copy kernel by the guard during the timed steps (0 on a settled machine)
    settle["guard_switches_in_timed_region"] = st["d2h_guard_switches"] - guard_before
    settle["guard_active_after_timed_region"] = bool(st["d2h_guard_active"])

    # the result of the last step: every destination block equals its source block
    sb = torch.from_numpy(seq["store_blocks"]).to(dev)
    lb = torch.from_numpy(seq["load_blocks"]).to(dev)
    for l in range(g.L):
        assert torch.equal(dst[l].view(g.P, g.NB, g.block_stride)[:, lb],
                           src[l].view(g.P, g.NB, g.block_stride)[:, sb]), "round trip differs"

    value = 2 * payload_one_way * args.steps / dt / 1e9
    ms_per_step = dt / args.steps * 1e3

    # dominant kernel of the timed region
    def kern(kind):
        n = st["timed_%s_launches" % kind]
        ms = st["%s_ms" % kind]
        moved = st["bytes_gathered" if kind == "gather" else "bytes_scattered"]
        avg_ms = ms / max(n, 1)
        return dict(launches=n, avg_us=round(avg_ms * 1e3, 2),
                    avg_chunks_per_launch=round(moved / g.chunk_bytes / max(n, 1), 2),
                    bytes_per_launch=2 * moved // max(n, 1),
                    hbm_gbps=round(2 * moved / max(ms, 1e-9) / 1e6, 1))
    kg, ks = kern("gather"), kern("scatter")
    dom_name, dom = ("gather", kg) if st["gather_ms"] >= st["scatter_ms"] else ("scatter", ks)
    roofline = {
        "bound": "hbm", "kernel": "move_rows<16," + dom_name + ">",
        "achieved": dom["hbm_gbps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": round(dom["hbm_gbps"] / HBM_PEAK_GBPS, 4),
        "traffic": int(dom["bytes_per_launch"] * PMC_TRAFFIC_RATIO),
        "traffic_source": "not read in this run: launch bytes x %.4f, the FETCH_SIZE + WRITE_SIZE to algorithmic "
                          "ratio that rocprofv3 --pmc measured for this kernel (profiles/)" % PMC_TRAFFIC_RATIO,
        "bytes_per_launch": dom["bytes_per_launch"], "avg_launch_us": dom["avg_us"],
        "launches": dom["launches"], "gather": kg, "scatter": ks,
    }

    def timed(fn, reps=5):
        best = 1e30
        for _ in range(reps):
            torch.cuda.synchronize()
            a = time.perf_counter()
            fn()
            best = min(best, time.perf_counter() - a)
        return best

    # the link's peak, and store / retrieve of the headline request separately against it
    ids = ctx.hash_chunks(seq["tokens"])
    peaks = link_peaks(ctx, pool_bytes)
    link = None
    if "link" in legs:
        def store_only():
            ctx.clear(ids)
            ctx.wait(ctx.store(src, d_store, ids, stream))
        # measuring the link's peaks allocated and freed GiBs, which can leave the runtime's copies
        # to the host slow for a while (and the guard on the copy kernel): let that pass first
        for _ in range(12):
            store_only()
            if not ctx.get_stats()["d2h_guard_active"]:
                break
        t_store = timed(store_only, reps=4)
        t_load = timed(lambda: ctx.wait(ctx.retrieve(ids, d_load, dst, stream)), reps=4)
        # both directions at once: the first half of the request is stored while the second
        # half is retrieved
        half = n_chunks // 2

        def both():
            ctx.clear(ids[:half])
            t1 = ctx.store(src, d_store[:half * g.CT], ids[:half], stream)
            t2 = ctx.retrieve(ids[half:], d_load[half * g.CT:], dst, stream)
            ctx.wait(t1)
            ctx.wait(t2)
        t_both = timed(both, reps=4)

        # the whole request stored and retrieved with no host wait in between: the retrieve
        # follows the store group by group on the device, both directions of the link at work
        def chained():
            ctx.clear(ids)
            t1 = ctx.store(src, d_store, ids, stream)
            t2 = ctx.retrieve(ids, d_load, dst, stream)
            ctx.wait(t1)
            ctx.wait(t2)
        t_chained = timed(chained, reps=4)
        # the same retrieve without the wait it leaves on the caller's stream (the caller
        # orders by lmc_wait, as this benchmark does anyway)
        ctx.tune("caller_waits", 0)
        t_load_nw = timed(lambda: ctx.wait(ctx.retrieve(ids, d_load, dst, stream)), reps=4)
        ctx.tune("caller_waits", 1)
        ctx.clear(ids)
        link = dict(peaks)
        for k_ in ("h2d_peak_gbps", "d2h_peak_gbps", "duplex_peak_gbps"):
            link[k_] = round(link[k_], 2)
        link.update({
            "store_gbps": round(payload_one_way / t_store / 1e9, 2),
            "retrieve_gbps": round(payload_one_way / t_load / 1e9, 2),
            "store_frac_of_d2h_peak": round(payload_one_way / t_store / 1e9 / peaks["d2h_peak_gbps"], 4),
            "retrieve_frac_of_h2d_peak": round(payload_one_way / t_load / 1e9 / peaks["h2d_peak_gbps"], 4),
            "retrieve_gbps_without_the_wait_on_the_callers_stream": round(payload_one_way / t_load_nw / 1e9, 2),
            "retrieve_enqueued_right_behind_the_store_of_the_same_chunks": dict(
                against_duplex_peak(2 * payload_one_way / t_chained / 1e9, peaks),
                ms=round(t_chained * 1e3, 2), ms_store_wait_retrieve_wait=round((t_store + t_load) * 1e3, 2)),
            "half_stored_while_half_is_retrieved": against_duplex_peak(
                (half + n_chunks - half) * g.chunk_bytes / t_both / 1e9, peaks),
        })

    # kernels alone: the whole request (128 chunks, 10 GiB) in one launch
    device = None
    if "device" in legs:
        ctx.tune("timing", 0)     # back-to-back launches, no per-launch events in between
        tg, tsc, tc = kernel_only(torch, ctx, W, WORKLOAD, g, src, dst, n_chunks, dev, stream,
                                  gather_slots=[d_store], scatter_slots=[d_load], iters=3)
        device = {"chunks_per_launch": n_chunks}
        device.update(kernel_report(payload_one_way, tg, tsc, tc))
        ctx.tune("timing", 1)

    out = {
        "metric": "KV store/retrieve GB/s", "value": round(value, 3), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT,
                   "payload_bytes_per_step": 2 * payload_one_way, "chunk_bytes": g.chunk_bytes,
                   "chunks": n_chunks, "staging_chunks": args.staging_chunks, "num_staging": args.num_staging},
        "roofline": roofline,
        "settle": settle,
    }
    if device:
        out["device"] = device
    if link:
        out["link"] = link
    # the headline's pages and context stay allocated to the end: freeing tens of GiB in
    # the middle of the run is what brings on the slow state described at the settling loop.
    # A side leg that fails must not take the headline line with it: its error is reported
    # in its place.
    def leg(key, fn):
        try:
            val = fn()
        except Exception as e:                               # noqa: BLE001 (reported, not hidden)
            key, val = key or "mode_legs", {"error": "%s: %s" % (type(e).__name__, e)}
        if key is None:
            out.update(val)
        else:
            out[key] = val

    if "host" in legs:
        leg("host_side", lambda: host_leg(torch, ctx, seq, src, dst, d_store, d_load, ids, stream, n_chunks))
    if "trace" in legs:
        leg("trace", lambda: trace_leg(lmc, ctx, g, src, dst, d_store, d_load, ids, stream, payload_one_way))
    if "groups" in legs:
        leg("group_size", lambda: group_size_leg(torch, lmc, W, g, seq, src, dst, d_store, d_load, stream, timed,
                                                 peaks, args.num_staging))
    if "configs" in legs:
        leg("configs", lambda: other_configs(torch, lmc, W, dev, stream, timed, peaks))
    if legs & {"duplex", "direct", "layerwise", "overlap", "fragmented"}:
        leg(None, lambda: mode_legs(torch, lmc, W, dev, stream, legs, args, timed, peaks))
    if "serving" in legs:
        leg("serving_mix", lambda: serving_leg(torch, lmc, W, dev, peaks))
    if "small" in legs:
        leg("small_request", lambda: small_leg(torch, lmc, W, dev, stream, timed))
    if "placement" in legs:
        def placement():
            res = placement_leg(torch, lmc, W, dev, stream)
            res["random_pages_allocated_first_in_the_process"] = first_pages
            res["random_pages_allocated_late_in_the_process"] = random_pages_sample(torch, lmc, W, dev, stream)
            return res
        leg("page_placement", placement)
    ctx.destroy()
    if "cpu" in legs:
        leg("cpu_baseline", cpu_baseline)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
