#!/usr/bin/env python3
"""Benchmark of the KV offload / upload hot path on one MI355X.

A step is one pass of the whole path for one agent of the Llama-3-8B-shaped configuration
(32 layers, 8 KV heads, head_dim 128, 16-token blocks, bf16: 2 MiB per block; pool of 16 384
blocks = 32 GiB; 4 096-token context = 256 blocks scattered uniformly at random):

    tc_offload(src blocks -> pinned host records)   gather_pages + D2H DMA
    tc_free(src)                                    pending-free until the copy has completed
    tc_alloc_at(dst) ; tc_upload(host -> dst)       H2D DMA + scatter_pages + rewrite_table

Every step takes a different pair of disjoint block sets out of a seeded partition of the pool
(32 pairs cover all 16 384 blocks), so the gather reads blocks that have been idle and the scatter
writes blocks nobody touched recently, as in serving.  Inputs are synthetic and resident in HBM
before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--tokens", type=int, default=4096, help="context length of the agent")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    return ap.parse_args()


def pinned_link_peak(torch, nbytes, stream, reps=7):
    """Contiguous pinned hipMemcpyAsync of the same byte count, both directions (GB/s)."""
    host = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    dev = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    out = {}
    with torch.cuda.stream(stream):
        for name, fn in (("d2h", lambda: host.copy_(dev, non_blocking=True)),
                         ("h2d", lambda: dev.copy_(host, non_blocking=True))):
            ts = []
            for i in range(reps + 2):
                torch.cuda.synchronize()
                t = time.perf_counter()
                fn()
                stream.synchronize()
                if i >= 2:
                    ts.append(time.perf_counter() - t)
            out[name] = nbytes / float(np.median(ts)) / 1e9
    del host, dev
    return out


def contiguous_copy_reference(torch, K, nbytes, reps=10):
    """The library's contiguous copy kernel on the same byte count: achievable-HBM reference (TB/s of traffic)."""
    a = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    b = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    for _ in range(3):
        K.check(K.tc_copy_contiguous(b, a, nbytes, None))
    e0 = [torch.cuda.Event(enable_timing=True) for _ in range(reps)]
    e1 = [torch.cuda.Event(enable_timing=True) for _ in range(reps)]
    for i in range(reps):
        e0[i].record()
        K.check(K.tc_copy_contiguous(b, a, nbytes, None))
        e1[i].record()
    torch.cuda.synchronize()
    ms = float(np.median([e0[i].elapsed_time(e1[i]) for i in range(reps)]))
    del a, b
    return 2 * nbytes / (ms * 1e-3) / 1e12


def variant(torch, K, pool, shape, pairs, link, note, steps=10, **opts):
    """The same agent through a context with other options, outside the timed region."""
    L, NB, pb = shape.num_layers, shape.num_blocks, shape.page_bytes
    n = len(pairs[0][0])
    payload = n * 2 * L * pb
    rc, ctx = K.tc_create(pool, None, L, NB, pb, shape.block_size, 0, host_arena_bytes=payload + 2 * L * pb, **opts)
    K.check(rc)
    rc, host = K.tc_host_alloc(ctx, n)
    K.check(rc)
    stream = torch.cuda.Stream()
    off, up = [], []
    for k in range(steps + 2):
        src, dst = pairs[(k + 7) % len(pairs)]
        K.check(K.tc_alloc_at(ctx, src))
        K.check(K.tc_alloc_at(ctx, dst))
        if k == 2:
            K.check(K.tc_set_profiling(ctx, 1))
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        ev[0].record(stream)
        K.check(K.tc_offload(ctx, src, host, stream))
        ev[1].record(stream)
        K.check(K.tc_upload(ctx, host, dst, None, stream))
        ev[2].record(stream)
        K.check(K.tc_sync(ctx))
        stream.synchronize()          # ev[2] is recorded after the transfer's own completion event
        K.check(K.tc_free(ctx, src))
        K.check(K.tc_free(ctx, dst))
        if k >= 2:
            off.append(ev[0].elapsed_time(ev[1]))
            up.append(ev[1].elapsed_time(ev[2]))
    st = K.tc_stats(ctx)[1]
    K.check(K.tc_host_free(ctx, host))
    K.check(K.tc_destroy(ctx))
    o, u = float(np.median(off)), float(np.median(up))
    out = {"note": note,
           "offload_GBps": round(payload / o / 1e6, 3), "upload_GBps": round(payload / u / 1e6, 3),
           "offload_ms": round(o, 4), "upload_ms": round(u, 4),
           "pct_of_pinned_link": {"offload": round(100 * payload / o / 1e6 / link["d2h"], 2),
                                  "upload": round(100 * payload / u / 1e6 / link["h2d"], 2)}}
    if st.gather_launches and st.scatter_launches:
        out["avg_launch_us"] = {"gather_pages": round(st.gather_ms / st.gather_launches * 1e3, 1),
                                "scatter_pages": round(st.scatter_ms / st.scatter_launches * 1e3, 1)}
    return out


def cpu_baseline(shape, ids, new_ids, budget_s=12.0):
    """The oracle, as it stands, on the same agent: host mirror with the touched blocks at their true strides."""
    import mmap
    import oracle
    L, NB, pb = shape.num_layers, shape.num_blocks, shape.page_bytes
    P = 2 * L
    n = int(ids.size)
    rec = oracle.record_bytes(L, pb, 0)
    mm = mmap.mmap(-1, P * NB * pb, flags=mmap.MAP_PRIVATE | mmap.MAP_ANONYMOUS | getattr(mmap, "MAP_NORESERVE", 0))
    pool = np.frombuffer(mm, dtype=np.uint8)
    rng = np.random.default_rng(1)
    v = pool.reshape(P, NB, pb)
    fill = rng.integers(0, 256, size=(n, pb), dtype=np.uint8)
    for p in range(P):
        v[p, ids] = fill
        v[p, new_ids] = 0
    host = np.zeros(n * rec, dtype=np.uint8)
    table = np.zeros(n, dtype=np.int32)
    t_off, t_up = [], []
    t_start = time.perf_counter()
    while True:
        t = time.perf_counter()
        oracle.offload(pool, None, L, NB, pb, 0, ids, host)
        t_off.append(time.perf_counter() - t)
        t = time.perf_counter()
        oracle.upload(host, L, NB, pb, 0, new_ids, pool, None, table)
        t_up.append(time.perf_counter() - t)
        if time.perf_counter() - t_start > budget_s or len(t_off) >= 20:
            break
    o, u = float(np.median(t_off)), float(np.median(t_up))
    payload = n * rec

    # the same oracle called from one thread per host core on disjoint runs of blocks (context only)
    from concurrent.futures import ThreadPoolExecutor
    workers = max(1, min(os.cpu_count() or 1, 16))
    cuts = np.linspace(0, n, workers + 1).astype(int)

    def part(k, direction):
        a, b = cuts[k], cuts[k + 1]
        if a == b:
            return
        if direction == 0:
            oracle.offload(pool, None, L, NB, pb, 0, ids[a:b], host[a * rec:b * rec])
        else:
            oracle.upload(host[a * rec:b * rec], L, NB, pb, 0, new_ids[a:b], pool, None, table[a:b])

    par = []
    with ThreadPoolExecutor(workers) as ex:
        for direction in (0, 1):
            ts = []
            for _ in range(5):
                t = time.perf_counter()
                list(ex.map(lambda k: part(k, direction), range(workers)))
                ts.append(time.perf_counter() - t)
            par.append(float(np.median(ts)))
    res = {
        "value": round(2 * payload / (o + u) / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": f"the same agent ({n} blocks, {payload >> 20} MiB each way), offload+upload on a sparse host "
                  f"mirror of the pool, median of {len(t_off)} round trips, single thread",
        "offload_GBps": round(payload / o / 1e9, 3), "upload_GBps": round(payload / u / 1e9, 3),
        "upload_ms_per_1k_tokens": round(u * 1e3 / (n * shape.block_size / 1024), 3),
        "host_cores_available": os.cpu_count(),
        "parallel_calls": {"threads": workers, "value": round(2 * payload / (par[0] + par[1]) / 1e9, 3),
                           "offload_GBps": round(payload / par[0] / 1e9, 3),
                           "upload_GBps": round(payload / par[1] / 1e9, 3)},
    }
    del pool, v
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this library runs on ONE GPU; --gpus must be 1 (no multi-GPU path exists).", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the path has no CPU fallback.", file=sys.stderr)
        sys.exit(2)
    import paper_2510_18586_amd as K
    import tc_workloads as W

    cfg_index = 1
    shape = W.CONFIGS[cfg_index]
    L, NB, pb = shape.num_layers, shape.num_blocks, shape.page_bytes
    n = -(-args.tokens // shape.block_size)
    rng = W.rng_for(cfg_index)
    perm = rng.permutation(NB).astype(np.int32)
    sets = [perm[i * n:(i + 1) * n] for i in range(NB // n)]      # disjoint, each scattered uniformly
    pairs = [(sets[2 * i], sets[2 * i + 1]) for i in range(len(sets) // 2)]
    ids_a, ids_b = pairs[0]

    pool = W.make_pool_device(shape, W.seed_for(cfg_index))
    rec = 2 * L * pb
    payload = n * rec
    rc, ctx = K.tc_create(pool, None, L, NB, pb, shape.block_size, 0, host_arena_bytes=payload + rec)
    K.check(rc)
    assert K.tc_record_bytes(ctx) == rec
    rc, host = K.tc_host_alloc(ctx, n)
    K.check(rc)
    table = torch.full((n,), -1, dtype=torch.int32, device="cuda:0")
    stream = torch.cuda.Stream()

    def step(k, evs=None):
        src, dst = pairs[k % len(pairs)]
        K.check(K.tc_alloc_at(ctx, src))              # the agent owns its blocks
        if evs:
            evs[0].record(stream)
        K.check(K.tc_offload(ctx, src, host, stream))
        K.check(K.tc_free(ctx, src))                  # pending-free until the copy has completed
        if evs:
            evs[1].record(stream)
        K.check(K.tc_alloc_at(ctx, dst))
        K.check(K.tc_upload(ctx, host, dst, table, stream))
        if evs:
            evs[2].record(stream)
        K.check(K.tc_sync(ctx))                       # completion; retires both transfers
        K.check(K.tc_free(ctx, dst))                  # the agent finishes; blocks return to the pool

    link = pinned_link_peak(torch, payload, stream)
    ref_tbps = contiguous_copy_reference(torch, K, payload)

    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()

    K.check(K.tc_set_profiling(ctx, 1))
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(args.warmup + k, evs[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    K.check(K.tc_set_profiling(ctx, 0))

    off_ms = float(np.median([e[0].elapsed_time(e[1]) for e in evs]))
    up_ms = float(np.median([e[1].elapsed_time(e[2]) for e in evs]))
    rc, st = K.tc_stats(ctx)
    K.check(rc)

    ms_per_step = wall * 1e3 / args.steps
    value = 2 * payload * args.steps / wall / 1e9
    off_gbps, up_gbps = payload / (off_ms * 1e-3) / 1e9, payload / (up_ms * 1e-3) / 1e9

    # HBM traffic per launch from the committed rocprofv3 counter runs; valid for this launch size only
    measured = {}
    try:
        with open(os.path.join(os.path.dirname(os.path.abspath(K.library_path())), "measured_traffic.json")) as f:
            measured = json.load(f)
    except OSError:
        pass

    def roof(name, launches, nbytes, ms):
        if not launches:
            return None
        avg_ms = ms / launches
        traffic = measured.get(name) if measured.get("record_bytes_per_launch") == nbytes // launches else None
        achieved = 2.0 * nbytes / launches / (avg_ms * 1e-3) / 1e9   # read + write per payload byte
        return {"kernel": name, "bound": "hbm", "achieved": round(achieved, 1), "peak": 8000.0, "unit": "GB/s",
                "frac": round(achieved / 8000.0, 4), "traffic": traffic,
                "launches": int(launches), "avg_launch_us": round(avg_ms * 1e3, 2),
                "algorithmic_bytes_per_launch": int(2 * nbytes // launches),
                "contiguous_copy_kernel_GBps": round(ref_tbps * 1e3, 1)}

    r_g = roof("gather_pages", st.gather_launches, st.gather_bytes, st.gather_ms)
    r_s = roof("scatter_pages", st.scatter_launches, st.scatter_bytes, st.scatter_ms)
    dominant, other = (r_s, r_g) if st.scatter_ms >= st.gather_ms else (r_g, r_s)

    out = {
        "metric": "KV offload/upload GB/s (% of HBM and host-link peak); upload ms per 1k tokens", "value": round(value, 3), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": "configs[1] llama3-8b-shaped KV: 32 layers x K,V x 8 heads x 128 x 16 tok bf16 "
                               "(2 MiB/block), 16384-block pool (32 GiB), one agent, "
                               f"{args.tokens} tokens = {n} blocks scattered uniformly",
                   "payload_bytes_each_way": payload, "tokens": n * shape.block_size},
        "offload_GBps": round(off_gbps, 3), "upload_GBps": round(up_gbps, 3),
        "offload_ms": round(off_ms, 4), "upload_ms": round(up_ms, 4),
        "upload_ms_per_1k_tokens": round(up_ms / (n * shape.block_size / 1024), 4),
        "pinned_link_GBps": {k: round(v, 3) for k, v in link.items()},
        "pct_of_pinned_link": {"offload": round(100 * off_gbps / link["d2h"], 2),
                               "upload": round(100 * up_gbps / link["h2d"], 2)},
        "roofline": dominant, "roofline_other_kernel": other,
    }
    out["direct_paths"] = variant(torch, K, pool, shape, pairs, link,
                                  "tc_opts.direct_offload = 1 (6 workgroups) / direct_upload = 1 (8 workgroups): no staging, "
                                  "no DMA; not the default", direct_offload=1, direct_upload=1)
    out["host_tail"] = variant(torch, K, pool, shape, pairs, link,
                               "tc_opts.host_tail_div = 64: the last 1/64 of the chunk crosses the link inside the copy "
                               "launch, so the link is not idle while the kernel runs; the launches get longer, the "
                               "transfer shorter; not the default", host_tail_div=64)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, ids_a, ids_b)
    K.check(K.tc_host_free(ctx, host))
    K.check(K.tc_destroy(ctx))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
