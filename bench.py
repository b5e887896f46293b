#!/usr/bin/env python3
"""Benchmark of the KV store / retrieve path on one MI355X.

One step is one pass of the whole path over one request of the Llama-3-8B-shaped
configuration (32 layers, K and V, 8 KV heads x 128, bf16, 16-token pages in a pool of
8192 blocks; a 4096-token prefix = 16 chunks of 256 tokens = 512 MiB of KV):
  hash the tokens -> prefix lookup -> store every chunk (gather kernel + D2H per group,
  pipelined) -> wait -> prefix lookup -> retrieve every chunk into freshly permuted
  blocks (H2D + scatter kernel, pipelined) -> wait -> clear the chunks.
Inputs are synthetic and resident in HBM before the timed region.  `value` is payload
bytes moved (store + retrieve) per second of wall time.

Before the warm-up the benchmark settles: it runs untimed steps until 150 in a row reach
90 % of the link rate (see the comment at that loop; `settle` in the JSON says what it
took).  On a machine in its normal state that is three seconds.

Also reported in the same JSON line:
  roofline     the gather / scatter kernel launches of the timed steps, timed with HIP
               events on the library's own streams, against the 8 TB/s HBM peak;
               algorithmic bytes = 2 x chunk bytes per chunk (each byte read once and
               written once)
  device       both kernels alone over all 16 chunks in one launch, sources rotated so
               the working set exceeds the 256 MB Infinity Cache, and a plain copy
               kernel of the same size as the achievable ceiling
  link         hipMemcpyAsync peak between the pinned pool and the GPU per direction,
               and store / retrieve payload rate as a fraction of it
  duplex       a store and a retrieve of different requests running at the same time,
               against the link's measured two-way peak
  direct       the variant without staging: the kernels read / write the pinned pool
  layerwise    the same request moved layer by layer (rectangle copies + kernels over
               one or four layers), as a fraction of the link peak, and how soon layer 0
               is usable compared with the bulk retrieve
  overlap_with_compute  retrieve the request while a consumer stream runs a stand-in for 32
               layers of compute (dense bf16 products, about as long as the transfer):
               compute alone, after a bulk retrieve, and behind a layer-wise retrieve layer
               by layer (section 5.2), each through staging and in direct mode; and the
               store side: compute then bulk store, against layers stored as they are computed
  fragmented_pool  the same request with every other pool slot taken beforehand, so that
               no two of its chunks are neighbours in the pool (one copy per chunk)
  small_request    one 0.5 MiB chunk (configuration 1): microseconds from the call to a
               finished lmc_wait, through the staging ring and by the library's size rule
  cpu_baseline the CPU oracle doing the same store + retrieve on the same 16 chunks,
               chunks fanned out over host threads
  configs      (only with --legs ...,configs) every benchmark configuration end to end
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
# FETCH_SIZE and WRITE_SIZE of this benchmark's device leg, each calibrated on the plain
# copy kernel (profiles/move_rows_llama3_8b_device_leg.md): counters cannot be read from
# inside this process, so the measured ratio is applied to the launch size.
PMC_TRAFFIC_RATIO = 1.0001
WORKLOAD = "llama3_8b"


def cpu_baseline(g, seq, budget_s=12.0):
    """The oracle, as it stands, doing store (gather into a pool) and retrieve (scatter
    from the pool) for the request's 16 chunks; chunks spread over threads."""
    import dataclasses
    from concurrent.futures import ThreadPoolExecutor
    import oracle
    from paper_2510_09665_amd import workloads as W
    rng = W.rng_for(WORKLOAD, stream=7)
    nb = seq["store_blocks"].size
    gc = dataclasses.replace(g, NB=nb)                      # only the touched blocks
    src = [W.payload_bytes(rng, g, gc.layer_bytes) for _ in range(g.L)]
    dst = [np.zeros(gc.layer_bytes, dtype=np.uint8) for _ in range(g.L)]
    n_chunks = seq["tokens"].size // g.CT
    t = np.arange(n_chunks * g.CT, dtype=np.int64)          # block i of the request = compact block i
    s_slots = t.reshape(n_chunks, g.CT)
    d_slots = t[::-1].copy().reshape(n_chunks, g.CT)
    pool = [None] * n_chunks

    def one(i):
        pool[i] = oracle.gather_chunk(gc, src, s_slots[i])
        oracle.scatter_chunk(gc, pool[i], d_slots[i], dst)

    cores = max(1, min(len(os.sched_getaffinity(0)), 16))
    payload = 2 * n_chunks * g.chunk_bytes
    out = {}
    for label, n_thr in (("single", 1), ("all", cores)):
        reps, t0 = 0, time.perf_counter()
        with ThreadPoolExecutor(n_thr) as ex:
            while True:
                list(ex.map(one, range(n_chunks)))
                reps += 1
                dt = time.perf_counter() - t0
                if dt > budget_s / 2:
                    break
        out[label] = payload * reps / dt / 1e9
    return {
        "value": round(out["all"], 3), "unit": "GB/s", "cores": cores, "kind": "oracle",
        "single_thread_value": round(out["single"], 3),
        "sample": "the same 16 chunks (512 MiB) stored and retrieved by oracle gather_chunk + "
                  "scatter_chunk, one chunk per task on a thread pool, repeated for about 6 s per "
                  "thread count; payload bytes / wall time",
    }


def kernel_only(torch, ctx, kv, d_slots, n_chunks, staging, stream, iters=4):
    """Seconds per launch of the gather and of the scatter over n_chunks chunks (HIP events)."""
    out = []
    for fn in (lambda: ctx.gather(kv, d_slots, n_chunks, staging, stream),
               lambda: ctx.scatter(staging, d_slots, n_chunks, kv, stream)):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        best = 1e30
        for _ in range(3):
            e0.record(stream)
            for _ in range(iters):
                fn()
            e1.record(stream)
            e1.synchronize()
            best = min(best, e0.elapsed_time(e1) / iters * 1e-3)
        out.append(best)
    ctx.wait()
    return out


def all_configs(torch, lmc, W, dev, stream, timed):
    """Every benchmark configuration end to end (store, then retrieve into fresh blocks;
    configuration 4: one batched retrieve of the hit chunks of 64 requests, pool slots in
    shuffled order), each as a fraction of the link peak measured in the same context."""
    res = {}
    for name, staging in (("tiny", 1), ("llama3_8b", 16), ("llama3_70b", 8), ("mla_bf16", 32), ("mla_fp8", 32)):
        g = W.geometry(name)
        seq = W.sequence(name, g)
        n = seq["tokens"].size // g.CT
        kv = [torch.zeros(g.layer_bytes, dtype=torch.uint8, device=dev) for _ in range(g.L)]
        d_s, d_l = torch.from_numpy(seq["store_slots"]).to(dev), torch.from_numpy(seq["load_slots"]).to(dev)
        ctx = lmc.Context(g, max(n * g.chunk_bytes, 1 << 30), staging_chunks=staging, device=0)
        ids = ctx.hash_chunks(seq["tokens"])

        def st():
            ctx.clear(ids)
            ctx.wait(ctx.store(kv, d_s, ids, stream))
        # best of a dozen: for a few seconds after memory of this size has been allocated or
        # freed in the process, the runtime's device-to-host copies run at half speed
        ts = timed(st, reps=12)
        tl = timed(lambda: ctx.wait(ctx.retrieve(ids, d_l, kv, stream)), reps=4)
        nbytes = n * g.chunk_bytes
        h2d, d2h = ctx.measure_link(min(512 << 20, nbytes) // 16 * 16, reps=3)
        # the kernels alone: the whole request in one launch, HBM to HBM.  Requests smaller
        # than the 256 MB Infinity Cache are served from it in part, so those are no
        # measure of HBM (configuration 1 and the fp8 variant of 5).
        staging = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        kg, ks = kernel_only(torch, ctx, kv, d_s, n, staging, stream)
        del staging
        res[name] = {"chunks": n, "payload_bytes": nbytes,
                     "kernel_only_gather_hbm_gbps": round(2 * nbytes / kg / 1e9, 1),
                     "kernel_only_scatter_hbm_gbps": round(2 * nbytes / ks / 1e9, 1),
                     "kernel_only_in_cache": nbytes < (512 << 20),
                     "store_gbps": round(nbytes / ts / 1e9, 2), "retrieve_gbps": round(nbytes / tl / 1e9, 2),
                     "store_frac_of_d2h_peak": round(nbytes / ts / 1e9 / d2h, 4),
                     "retrieve_frac_of_h2d_peak": round(nbytes / tl / 1e9 / h2d, 4),
                     "store_ms": round(ts * 1e3, 3), "retrieve_ms": round(tl * 1e3, 3)}
        ctx.destroy()
        del kv
        torch.cuda.empty_cache()
    g = W.geometry("batch_8b")
    reqs = W.request_mix("batch_8b", g)
    n_hit = sum(r["n_hit"] for r in reqs)
    kv = [torch.zeros(g.layer_bytes, dtype=torch.uint8, device=dev) for _ in range(g.L)]
    ctx = lmc.Context(g, (n_hit + 1) * g.chunk_bytes, staging_chunks=16, device=0)
    zero = np.zeros(g.chunk_bytes, dtype=np.uint8)
    ids_per = [ctx.hash_chunks(r["tokens"]) for r in reqs]
    hit = [(ri, k) for ri, r in enumerate(reqs) for k in range(r["n_hit"])]
    for j in np.random.default_rng(0).permutation(len(hit)):
        ctx.put_host([ids_per[hit[j][0]][hit[j][1]]], zero)
    off = np.concatenate([[0], np.cumsum([r["n_hit"] for r in reqs])])
    ids_all = np.concatenate([ids_per[ri][:r["n_hit"]] for ri, r in enumerate(reqs)])
    d_sl = torch.from_numpy(np.concatenate([r["load_slots"] for r in reqs])).to(dev)
    t = timed(lambda: ctx.wait(ctx.retrieve_batch(off, ids_all, d_sl, kv, stream)), reps=3)
    h2d, _ = ctx.measure_link(512 << 20, reps=3)
    nbytes = n_hit * g.chunk_bytes
    staging = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    kg, ks = kernel_only(torch, ctx, kv, d_sl, n_hit, staging, stream)
    del staging
    res["batch_8b"] = {"requests": len(reqs), "hit_chunks": n_hit, "payload_bytes": nbytes,
                       "kernel_only_gather_hbm_gbps": round(2 * nbytes / kg / 1e9, 1),
                       "kernel_only_scatter_hbm_gbps": round(2 * nbytes / ks / 1e9, 1),
                       "retrieve_batch_gbps": round(nbytes / t / 1e9, 2),
                       "retrieve_frac_of_h2d_peak": round(nbytes / t / 1e9 / h2d, 4),
                       "retrieve_ms": round(t * 1e3, 1)}
    ctx.destroy()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--staging-chunks", type=int, default=16)
    ap.add_argument("--num-staging", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--settle-seconds", type=float, default=40.0,
                    help="upper limit for the untimed settling phase before the warm-up (0 = none)")
    ap.add_argument("--legs", default="pipeline,link,device,duplex,direct,layerwise,overlap,fragmented,small,cpu",
                    help="comma list of pipeline (always run), link, device, duplex, direct, layerwise, overlap, "
                         "fragmented, small, cpu, and configs (every benchmark configuration end to end; "
                         "not in the default): the extra measurements to make; profiling runs use a subset")
    ap.add_argument("--tune", action="append", default=[], help="key=value for lmc_tune")
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
    dev = torch.device("cuda:0")
    g = W.geometry(WORKLOAD)
    seq = W.sequence(WORKLOAD, g)
    n_chunks = seq["tokens"].size // g.CT
    payload_one_way = n_chunks * g.chunk_bytes

    # paged KV resident in HBM: bf16 uniform(-1, 1) in the request's blocks
    gen = torch.Generator(device=dev)
    gen.manual_seed(W.SEED_BASE + W.CONFIGS[WORKLOAD]["id"])
    src, dst = [], []
    sb = torch.from_numpy(seq["store_blocks"]).to(dev)
    for _ in range(g.L):
        a = torch.zeros(g.layer_bytes, dtype=torch.uint8, device=dev)
        r = torch.rand((g.P, sb.numel(), g.block_stride // 2), device=dev, generator=gen) * 2 - 1
        a.view(g.P, g.NB, g.block_stride)[:, sb] = \
            r.to(torch.bfloat16).view(torch.uint8).view(g.P, sb.numel(), g.block_stride)
        src.append(a)
        dst.append(torch.zeros(g.layer_bytes, dtype=torch.uint8, device=dev))
    d_store = torch.from_numpy(seq["store_slots"]).to(dev)
    d_load = torch.from_numpy(seq["load_slots"]).to(dev)
    stream = torch.cuda.current_stream()

    ctx = lmc.Context(g, max(2 * n_chunks * g.chunk_bytes, 1 << 30), num_staging=args.num_staging,
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

    # Settle.  For some seconds after tens of GiB of device or pinned memory have been
    # freed on the host (by this process while it set up, or by the process that had the
    # GPU before), the runtime's device-to-host copies inside a store run at about half
    # speed; the state sets in a few steps after the first copies and passes by itself.
    # It is a state of the machine, not of this path, so steps are run, untimed, until 150
    # in a row (three seconds' worth) reach 90 % of the link rate measured now (a lone copy
    # is not affected) without the library's copy-engine guard stepping in, or until the
    # time limit; what it took is reported.  Right after the GPU test suite this takes up
    # to ten seconds, on a machine in its normal state three.
    settle = {"steps": 0, "seconds": 0.0, "settled": args.settle_seconds <= 0}
    if args.settle_seconds > 0:
        _, d2h_now = ctx.measure_link(256 << 20, reps=2)
        t_begin, good, slow, seen = time.perf_counter(), 0, 0, 0
        while time.perf_counter() - t_begin < args.settle_seconds:
            a = time.perf_counter()
            step()
            torch.cuda.synchronize()
            settle["steps"] += 1
            gs = ctx.get_stats()
            healthy = 2 * payload_one_way / (time.perf_counter() - a) / 1e9 >= 0.9 * d2h_now
            if healthy and gs["d2h_guard_switches"] == seen and not gs["d2h_guard_active"]:
                good += 1
            else:
                good, seen = 0, gs["d2h_guard_switches"]
                slow += 0 if healthy else 1
            if good >= 150:
                settle["settled"] = True
                break
        settle["seconds"] = round(time.perf_counter() - t_begin, 2)
        settle["slow_steps"] = slow

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    guard_before = ctx.get_stats()["d2h_guard_switches"]
    ctx.reset_stats()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    st = ctx.get_stats()
    # copies handed to the copy kernel by the guard during the timed steps (0 on a settled machine)
    settle["guard_switches_in_timed_region"] = st["d2h_guard_switches"] - guard_before
    settle["guard_active_after_timed_region"] = bool(st["d2h_guard_active"])

    # the result of the last step: every destination block equals its source block
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
        "bound": "hbm", "kernel": "move_rows<16," + ("gather" if dom_name == "gather" else "scatter") + ">",
        "achieved": dom["hbm_gbps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": round(dom["hbm_gbps"] / HBM_PEAK_GBPS, 4),
        "traffic": int(dom["bytes_per_launch"] * PMC_TRAFFIC_RATIO),
        "bytes_per_launch": dom["bytes_per_launch"], "avg_launch_us": dom["avg_us"],
        "launches": dom["launches"], "gather": kg, "scatter": ks,
    }

    # store and retrieve separately, and the link peak
    def timed(fn, reps=5):
        best = 1e30
        for _ in range(reps):
            torch.cuda.synchronize()
            a = time.perf_counter()
            fn()
            best = min(best, time.perf_counter() - a)
        return best
    ids = ctx.hash_chunks(seq["tokens"])
    link = None
    if "link" in legs:
        def store_only():
            ctx.clear(ids)
            ctx.wait(ctx.store(src, d_store, ids, stream))
        t_store = timed(store_only)
        t_load = timed(lambda: ctx.wait(ctx.retrieve(ids, d_load, dst, stream)))
        ctx.clear(ids)
        h2d, d2h = ctx.measure_link(512 << 20, reps=4)
        link = {
            "h2d_peak_gbps": round(h2d, 2), "d2h_peak_gbps": round(d2h, 2),
            "store_gbps": round(payload_one_way / t_store / 1e9, 2),
            "retrieve_gbps": round(payload_one_way / t_load / 1e9, 2),
            "store_frac_of_d2h_peak": round(payload_one_way / t_store / 1e9 / d2h, 4),
            "retrieve_frac_of_h2d_peak": round(payload_one_way / t_load / 1e9 / h2d, 4),
        }

    # kernels alone: all 16 chunks per launch, rotating over 4 block sets (4 x 512 MiB of
    # sources + 4 staging buffers) so that nothing is served from the Infinity Cache
    device = None
    if "device" in legs:
        n_rot = 4
        rot_slots, stagings = [], []
        for r in range(n_rot):
            s = W.sequence(WORKLOAD, g, stream=10 + r)
            rot_slots.append(torch.from_numpy(s["store_slots"]).to(dev))
            stagings.append(torch.empty(payload_one_way, dtype=torch.uint8, device=dev))

        ctx.tune("timing", 0)     # back-to-back launches, no per-launch events in between

        def dev_time(fn, iters=12, reps=3):
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
            return best
        tg = dev_time(lambda r: ctx.gather(src, rot_slots[r], n_chunks, stagings[r], stream))
        tsc = dev_time(lambda r: ctx.scatter(stagings[r], rot_slots[r], n_chunks, dst, stream))
        tc = dev_time(lambda r: ctx.copy(stagings[r], stagings[(r + 1) % n_rot], payload_one_way, stream))
        ctx.wait()
        device = {
            "chunks_per_launch": n_chunks, "bytes_per_launch": 2 * payload_one_way,
            "gather_us": round(tg * 1e6, 1), "scatter_us": round(tsc * 1e6, 1),
            "copy_kernel_us": round(tc * 1e6, 1),
            "gather_hbm_gbps": round(2 * payload_one_way / tg / 1e9, 1),
            "scatter_hbm_gbps": round(2 * payload_one_way / tsc / 1e9, 1),
            "copy_kernel_hbm_gbps": round(2 * payload_one_way / tc / 1e9, 1),
            "gather_frac_of_hbm_peak": round(2 * payload_one_way / tg / 1e9 / HBM_PEAK_GBPS, 4),
            "scatter_frac_of_hbm_peak": round(2 * payload_one_way / tsc / 1e9 / HBM_PEAK_GBPS, 4),
        }
        del stagings
    # full duplex: store one request while another is retrieved (two streams per
    # direction, nothing shared but the link and HBM)
    duplex = None
    if "duplex" in legs:
        ctx.tune("timing", 0)
        ids_a = ctx.hash_chunks(seq["tokens"])
        seq_b = W.sequence(WORKLOAD, g, stream=1)
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
        peak = ctx.measure_link_duplex(512 << 20, reps=6)
        duplex = {"store_plus_retrieve_gbps": round(2 * payload_one_way / t_both / 1e9, 2),
                  "link_duplex_peak_gbps": round(peak, 2),
                  "frac_of_duplex_peak": round(2 * payload_one_way / t_both / 1e9 / peak, 4)}
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
        h2d, d2h = dctx.measure_link(512 << 20, reps=3)
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
        h2d, d2h = ctx.measure_link(512 << 20, reps=3)
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
        fctx = lmc.Context(g, (2 * n_chunks + 1) * g.chunk_bytes, staging_chunks=args.staging_chunks,
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
        h2d, d2h = fctx.measure_link(512 << 20, reps=3)
        fragmented = {"store_gbps": round(payload_one_way / tf_s / 1e9, 2),
                      "retrieve_gbps": round(payload_one_way / tf_l / 1e9, 2),
                      "store_frac_of_d2h_peak": round(payload_one_way / tf_s / 1e9 / d2h, 4),
                      "retrieve_frac_of_h2d_peak": round(payload_one_way / tf_l / 1e9 / h2d, 4)}
        fctx.destroy()

    ctx.destroy()
    del src, dst
    torch.cuda.empty_cache()

    # a request of one small chunk (config 1, 0.5 MiB): time from the call to a finished
    # lmc_wait, through the staging ring and by the library's size rule (no staging)
    small = None
    if "small" in legs:
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

    configs = all_configs(torch, lmc, W, dev, stream, timed) if "configs" in legs else None

    out = {
        "metric": "KV store/retrieve GB/s", "value": round(value, 3), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": "Llama-3-8B-shaped KV: 32 layers, 8 KV heads, head_dim 128, bf16, "
                               "block_size 16, pool of 8192 blocks; 4096-token prefix = 16 chunks of "
                               "256 tokens; store all chunks then retrieve into freshly permuted blocks",
                   "payload_bytes_per_step": 2 * payload_one_way, "chunk_bytes": g.chunk_bytes,
                   "staging_chunks": args.staging_chunks, "num_staging": args.num_staging},
        "roofline": roofline,
        "settle": settle,
    }
    if device:
        out["device"] = device
    if link:
        out["link"] = link
    if duplex:
        out["duplex"] = duplex
    if direct:
        out["direct"] = direct
    if layerwise:
        out["layerwise"] = layerwise
    if overlap:
        out["overlap_with_compute"] = overlap
    if fragmented:
        out["fragmented_pool"] = fragmented
    if small:
        out["small_request"] = small
    if configs:
        out["configs"] = configs
    if "cpu" in legs:
        out["cpu_baseline"] = cpu_baseline(g, seq)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
