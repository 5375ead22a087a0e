#!/usr/bin/env python3
"""Benchmark of the KV offload / upload hot path on one MI355X.

A step is one pass of the whole path for one agent of the Llama-3-8B-shaped configuration
(32 layers, 8 KV heads, head_dim 128, 16-token blocks, bf16: 2 MiB per block; pool of 16 384
blocks = 32 GiB; 4 096-token context = 256 blocks scattered uniformly at random), with the library's
default options (paths chosen by the library):

    tc_offload(src blocks -> pinned host records)   gather_pages into device staging + D2H DMA
    tc_free(src)                                    pending-free until the copy has completed
    tc_alloc_at(dst) ; tc_upload(host -> dst)       scatter_pages reading the pinned records + rewrite_table

Every step takes a different pair of disjoint block sets out of a seeded partition of the pool
(32 pairs cover all 16 384 blocks), so the gather reads blocks that have been idle and the scatter
writes blocks nobody touched recently, as in serving.  Inputs are synthetic and resident in HBM
before the timed region.  Outside the timed region the same agent runs through the two-stage path in
both directions (`staged_path`: both HBM-bound kernels and their roofline fractions), and the other four
benchmark configurations run once each (`configs`).  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBPS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--tokens", type=int, default=4096, help="context length of the agent")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the other four configurations")
    ap.add_argument("--no-overlapped", action="store_true",
                    help="leave the overlap_kernels extras out (under rocprofv3 their kernels run next to the profiler's blit "
                         "copies, which says nothing about them and blurs the per-kernel statistics)")
    ap.add_argument("--config", type=int, default=0, choices=[0, 1, 3, 4, 5],
                    help="run only this one of the other configurations and print its object (for profiler runs)")
    return ap.parse_args()


def pinned_link_peak(torch, nbytes, stream, reps=9):
    """Contiguous pinned hipMemcpyAsync of the same byte count, both directions, timed by events on the stream
    the copy runs on: best and median of `reps` (GB/s).  The best is the denominator of every '% of link'."""
    host = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    dev = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    out = {}
    with torch.cuda.stream(stream):
        for name, fn in (("d2h", lambda: host.copy_(dev, non_blocking=True)),
                         ("h2d", lambda: dev.copy_(host, non_blocking=True))):
            ts = []
            for i in range(reps + 2):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                fn()
                e1.record(stream)
                stream.synchronize()
                if i >= 2:
                    ts.append(e0.elapsed_time(e1) * 1e-3)
            out[name] = nbytes / min(ts) / 1e9
            out[name + "_median"] = nbytes / float(np.median(ts)) / 1e9
    del host, dev
    return out


_hip = None


def plain_copy_on(torch, host_ptr, nbytes, stream, reps=5):
    """The same measurement on memory the library's arena owns: hipMemcpyAsync between the first `nbytes` of the
    pinned buffer at `host_ptr` and a device buffer, best of `reps` per direction (GB/s)."""
    global _hip
    import ctypes
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so")
        _hip.hipMemcpyAsync.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p]
        _hip.hipMemcpyAsync.restype = ctypes.c_int
    dev = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    out = {}
    for name, kind in (("d2h", 2), ("h2d", 1)):
        ts = []
        for i in range(reps + 1):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            dst, src = (host_ptr, dev.data_ptr()) if kind == 2 else (dev.data_ptr(), host_ptr)
            if _hip.hipMemcpyAsync(dst, src, nbytes, kind, stream.cuda_stream) != 0:
                raise RuntimeError("hipMemcpyAsync failed")
            e1.record(stream)
            stream.synchronize()
            if i:
                ts.append(e0.elapsed_time(e1) * 1e-3)
        out[name] = nbytes / min(ts) / 1e9
    del dev
    return out


def contiguous_copy_reference(torch, K, nbytes, reps=10):
    """The library's contiguous copy kernel between cold quarters of a 4 x nbytes buffer: achievable-HBM reference."""
    buf = torch.empty(4 * nbytes, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    ts = []
    for i in range(reps + 2):
        src, dst = buf[(2 * (i % 2)) * nbytes:], buf[(2 * (i % 2) + 1) * nbytes:]
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        K.check(K.tc_copy_contiguous(dst, src, nbytes, None))
        e1.record()
        torch.cuda.synchronize()
        if i >= 2:
            ts.append(e0.elapsed_time(e1))
    del buf
    return 2 * nbytes / (float(np.median(ts)) * 1e-3) / 1e9


def kernel_fracs(st):
    out = {}
    for name, n, nbytes, ms in (("gather_pages", st.gather_launches, st.gather_bytes, st.gather_ms),
                                ("scatter_pages", st.scatter_launches, st.scatter_bytes, st.scatter_ms)):
        if n:
            gbps = 2.0 * nbytes / (ms * 1e-3) / 1e9
            out[name] = {"launches": int(n), "avg_launch_us": round(ms / n * 1e3, 2), "GBps": round(gbps, 1),
                         "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4)}
    # the DMAs themselves, from event pairs around each chunk's copies
    for name, n, nbytes, ms in (("d2h_dma", st.d2h_copies, st.d2h_bytes, st.d2h_ms), ("h2d_dma", st.h2d_copies, st.h2d_bytes, st.h2d_ms)):
        if n and ms > 0:
            out[name] = {"chunks": int(n), "GBps": round(nbytes / ms / 1e6, 3)}
    return out


def timed(torch, K, ctx, stream, fn, reps=3, warm=1):
    """Median of event-timed fn() on `stream` (ms); every repetition is retired before the next."""
    ts = []
    for i in range(reps + warm):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        fn()
        e1.record(stream)
        K.check(K.tc_sync(ctx))
        stream.synchronize()
        if i >= warm:
            ts.append(e0.elapsed_time(e1))
    return float(np.median(ts))


def rates(payload, off_ms, up_ms, link, tokens=None):
    out = {"offload_GBps": round(payload / off_ms / 1e6, 3), "upload_GBps": round(payload / up_ms / 1e6, 3),
           "offload_ms": round(off_ms, 4), "upload_ms": round(up_ms, 4),
           "pct_of_pinned_link": {"offload": round(100 * payload / off_ms / 1e6 / link["d2h"], 2),
                                  "upload": round(100 * payload / up_ms / 1e6 / link["h2d"], 2)}}
    if tokens:
        out["upload_ms_per_1k_tokens"] = round(up_ms / (tokens / 1024), 4)
    return out


def variant(torch, K, pool, shape, pairs, link, note, steps=10, **opts):
    """The same agent through a context with other options, outside the timed region.  Returns (summary, stats)."""
    L, NB, pb = shape.num_layers, shape.num_blocks, shape.page_bytes
    n = len(pairs[0][0])
    rc, ctx = K.tc_create(pool, None, L, NB, pb, shape.block_size, 0, host_arena_bytes=(n + 1) * 2 * L * pb, **opts)
    K.check(rc)
    payload = n * K.tc_record_bytes(ctx)
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
        # each transfer is retired before the next is enqueued: a DMA enqueued behind a running one is sometimes
        # carried out at half rate by the runtime, which would be measured here as the path's own rate
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        ev[0].record(stream)
        K.check(K.tc_offload(ctx, src, host, stream))
        ev[1].record(stream)
        K.check(K.tc_sync(ctx))
        stream.synchronize()          # ev[1] is recorded after the transfer's own completion event
        ev[2].record(stream)
        K.check(K.tc_upload(ctx, host, dst, None, stream))
        ev[3].record(stream)
        K.check(K.tc_sync(ctx))
        stream.synchronize()
        K.check(K.tc_free(ctx, src))
        K.check(K.tc_free(ctx, dst))
        if k >= 2:
            off.append(ev[0].elapsed_time(ev[1]))
            up.append(ev[2].elapsed_time(ev[3]))
    st = K.tc_stats(ctx)[1]
    K.check(K.tc_host_free(ctx, host))
    K.check(K.tc_destroy(ctx))
    out = {"note": note, **rates(payload, float(np.median(off)), float(np.median(up)), link, n * shape.block_size)}
    out["kernels"] = kernel_fracs(st)
    return out, st


# ------------------------------------------------------------------------------------ the other configurations
def fresh_pool(torch, shape):
    """A pool of the configuration's shape filled with seeded random bytes (the path never interprets them)."""
    g = torch.Generator(device="cuda:0")
    g.manual_seed(251018586)
    pool = torch.empty(shape.pool_bytes, dtype=torch.uint8, device="cuda:0")
    pool.view(torch.int32).random_(0, 2 ** 31 - 1, generator=g)
    scales = None
    if shape.scales_per_block:
        scales = torch.rand(shape.scales_per_block * shape.num_blocks, device="cuda:0", generator=g)
    return pool, scales


def host_memory_available():
    try:
        with open("/proc/meminfo") as f:
            for line in f:
                if line.startswith("MemAvailable:"):
                    return int(line.split()[1]) * 1024
    except OSError:
        pass
    return None


class TwoContexts:
    """One pool bound twice: with the default options (paths chosen by the library) and with the two-stage path
    forced, so that the HBM-bound kernels can be timed on the same agents.  Host buffers come from the first
    context's pinned arena; the second takes them as the caller's pinned memory."""

    def __init__(self, torch, K, shape, pool, scales, arena_blocks, overlapped=False):
        self.K, self.shape = K, shape
        a = (shape.num_layers, shape.num_blocks, shape.page_bytes, shape.block_size, shape.scales_per_block)
        # the arena is sized by an upper bound of the record size; what a record is, the library says
        bound = 2 * shape.num_layers * shape.page_bytes + 4 * shape.scales_per_block + 256
        rc, self.auto = K.tc_create(pool, scales, *a, host_arena_bytes=arena_blocks * bound)
        K.check(rc)
        self.rec = K.tc_record_bytes(self.auto)
        rc, self.staged = K.tc_create(pool, scales, *a, direct_offload=K.TC_PATH_STAGED, direct_upload=K.TC_PATH_STAGED,
                                      host_tail_div=1)
        K.check(rc)
        K.check(K.tc_set_profiling(self.staged, 1))
        self.overlapped = None
        if overlapped:   # a third binding: the two-stage path with its kernels on the context's own stream
            rc, self.overlapped = K.tc_create(pool, scales, *a, direct_offload=K.TC_PATH_STAGED, direct_upload=K.TC_PATH_STAGED,
                                              host_tail_div=1, overlap_kernels=1)
            K.check(rc)

    def close(self):
        if self.overlapped:
            self.K.check(self.K.tc_destroy(self.overlapped))
        self.K.check(self.K.tc_destroy(self.staged))
        self.K.check(self.K.tc_destroy(self.auto))


def batch_both_ways(torch, K, two, link, src, dst, tables, stream, tokens):
    """Offload and upload of a batch of agents: default paths, then the forced two-stage path for the kernels."""
    bufs = []
    for s in src:
        rc, b = K.tc_host_alloc(two.auto, len(s))
        K.check(rc)
        bufs.append(b)
    payload = sum(len(s) for s in src) * two.rec
    out = {"agents": len(src), "blocks": int(sum(len(s) for s in src)), "payload_GiB": round(payload / 2 ** 30, 3)}
    # the link's rate on this very arena (a plain pinned copy of up to 512 MiB of it) is the denominator here
    link = plain_copy_on(torch, K.tc_arena_base(two.auto), min(payload, 512 << 20), stream)
    out["pinned_link_GBps_on_this_arena"] = {k: round(v, 3) for k, v in link.items()}
    before = K.tc_stats(two.staged)[1]
    for ctx, key in ((two.auto, "default_paths"), (two.staged, "staged_path"), (two.overlapped, "staged_overlapped")):
        if ctx is None:
            continue
        for s in src:
            K.check(K.tc_alloc_at(ctx, s))
        if dst is not src:
            for d in dst:
                K.check(K.tc_alloc_at(ctx, d))
        off = timed(torch, K, ctx, stream, lambda: K.check(K.tc_offload_batch(ctx, [(src[i], bufs[i]) for i in range(len(src))], stream)), reps=3)
        up = timed(torch, K, ctx, stream, lambda: K.check(K.tc_upload_batch(
            ctx, [(dst[i], bufs[i], tables[i]) for i in range(len(src))], stream)), reps=3)
        out[key] = rates(payload, off, up, link, tokens)
        if ctx == two.staged:
            after = K.tc_stats(ctx)[1]
            for f in ("gather_launches", "gather_bytes", "gather_ms", "scatter_launches", "scatter_bytes", "scatter_ms",
                      "d2h_copies", "d2h_bytes", "d2h_ms", "h2d_copies", "h2d_bytes", "h2d_ms"):
                setattr(after, f, getattr(after, f) - getattr(before, f))      # this batch's launches only
            out[key]["kernels"] = kernel_fracs(after)
        for s in src:
            K.check(K.tc_free(ctx, s))
        if dst is not src:
            for d in dst:
                K.check(K.tc_free(ctx, d))
    return out, bufs


def config1(torch, K, W, link):
    shape = W.CONFIGS[0]
    rng = W.rng_for(0)
    pool = torch.from_numpy(W.make_pool_host(shape, rng)).to("cuda:0")
    ids = W.pick_ids(rng, shape.num_blocks, 8)
    new = W.pick_ids(rng, shape.num_blocks, 8, exclude=ids)
    out = {"workload": "tiny: 2 layers, 8 KiB pages, 256 blocks; one agent of 8 blocks (256 KiB each way); latency-bound"}
    stream = torch.cuda.Stream()
    for key, opts in (("default_paths", {}), ("staged_path", dict(direct_offload=K.TC_PATH_STAGED, direct_upload=K.TC_PATH_STAGED))):
        rc, ctx = K.tc_create(pool, None, shape.num_layers, shape.num_blocks, shape.page_bytes, shape.block_size, 0,
                              host_arena_bytes=16 * 32768, **opts)
        K.check(rc)
        rc, host = K.tc_host_alloc(ctx, 8)
        K.check(K.tc_alloc_at(ctx, ids))
        K.check(K.tc_alloc_at(ctx, new))
        table = torch.zeros(8, dtype=torch.int32, device="cuda:0")
        torch.cuda.synchronize()
        off = timed(torch, K, ctx, stream, lambda: K.check(K.tc_offload(ctx, ids, host, stream)), reps=40, warm=5)
        up = timed(torch, K, ctx, stream, lambda: K.check(K.tc_upload(ctx, host, new, table, stream)), reps=40, warm=5)
        out[key] = {"offload_us": round(off * 1e3, 2), "upload_us": round(up * 1e3, 2),
                    "offload_GBps": round(8 * 32768 / off / 1e6, 3), "upload_GBps": round(8 * 32768 / up / 1e6, 3),
                    "upload_ms_per_1k_tokens": round(up / (8 * 16 / 1024), 4)}
        K.check(K.tc_destroy(ctx))
    return out


WITH_OVERLAPPED = True      # cleared by --no-overlapped


def config3(torch, K, W, link, pool):
    """64 agents of the 8B shape in a fragmented pool, as one batch; alone, next to a memory-bound neighbour on
    another stream, and half of them going out while the other half comes back."""
    shape = W.CONFIGS[2]
    rng = W.rng_for(2)
    tokens = W.lognormal_contexts(rng, 64)
    nblk = W.blocks_of(tokens, shape.block_size).astype(int)
    total = int(nblk.sum())
    two = TwoContexts(torch, K, shape, pool, None, total + 8, overlapped=WITH_OVERLAPPED)

    class B:
        def alloc(self, n):
            rc, ids = K.tc_alloc(two.auto, n)
            return ids if rc == 0 else None

        def free(self, ids):
            K.check(K.tc_free(two.auto, ids))

        def n_free(self):
            return K.tc_stats(two.auto)[1].gpu_blocks_free

    W.fragment_pool(B(), rng, n_ops=50000, need_free=total)
    src = [B().alloc(int(n)) for n in nblk]
    for s in src:
        B().free(s)                       # batch_both_ways claims them again in each context
    tables = torch.full((64, int(nblk.max()) + 1), -1, dtype=torch.int32, device="cuda:0")
    copy, copy2, compute = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    # 2 x total exceeds the pool: the upload claims the original blocks again
    out, bufs = batch_both_ways(torch, K, two, link, src, src, tables, copy, total * shape.block_size)
    out["workload"] = ("8B shape, 64 agents, contexts lognormal(median 2048, sigma 0.8, cap 16384), pool fragmented by "
                       "50 000 seeded alloc/free ops, one tc_offload_batch / tc_upload_batch")
    payload = total * two.rec

    # the neighbour: fp32 triad over 3 x 4 GiB on another stream
    m = 1 << 30
    a, b, c = torch.zeros(m, device="cuda:0"), torch.rand(m, device="cuda:0"), torch.rand(m, device="cuda:0")
    tri_bytes = 3 * 4 * m
    torch.cuda.synchronize()
    ctx = two.auto
    for s in src:
        K.check(K.tc_alloc_at(ctx, s))

    def tri_alone():
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(compute)
        K.check(K.tc_hbm_stream(a, b, c, m, 0.5, 8, compute))
        e1.record(compute)
        compute.synchronize()
        return e0.elapsed_time(e1) / 8

    tri_alone()
    t_tri = tri_alone()

    def overlapped(fn, alone_ms, ctx=two.auto):
        iters = max(1, int(alone_ms / t_tri) + 2)
        e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        torch.cuda.synchronize()
        e[0].record(compute)
        K.check(K.tc_hbm_stream(a, b, c, m, 0.5, iters, compute))
        e[1].record(compute)
        e[2].record(copy)
        fn()
        e[3].record(copy)
        K.check(K.tc_sync(ctx))
        torch.cuda.synchronize()
        return e[2].elapsed_time(e[3]), e[0].elapsed_time(e[1]) / iters

    items_out = [(src[i], bufs[i]) for i in range(64)]
    items_in = [(src[i], bufs[i], tables[i]) for i in range(64)]
    d = out["default_paths"]
    off_ov, tri_off = overlapped(lambda: K.check(K.tc_offload_batch(ctx, items_out, copy)), d["offload_ms"])
    up_ov, tri_up = overlapped(lambda: K.check(K.tc_upload_batch(ctx, items_in, copy)), d["upload_ms"])
    out["next_to_a_memory_bound_kernel"] = {
        "neighbour": "fp32 triad over 3 x 4 GiB (tc_hbm_stream) on another stream",
        "offload_GBps": round(payload / off_ov / 1e6, 3), "upload_GBps": round(payload / up_ov / 1e6, 3),
        "offload_change_pct": round(100 * (d["offload_ms"] / off_ov - 1), 2),
        "upload_change_pct": round(100 * (d["upload_ms"] / up_ov - 1), 2),
        "neighbour_alone_GBps": round(tri_bytes / t_tri / 1e6, 1),
        "neighbour_during_offload_GBps": round(tri_bytes / tri_off / 1e6, 1),
        "neighbour_during_upload_GBps": round(tri_bytes / tri_up / 1e6, 1)}

    # the same next to the neighbour with the copy kernels on the context's own stream (overlap_kernels = 1): what
    # happens depends on which hardware queue the runtime gives that stream
    if two.overlapped:
        for s in src:
            K.check(K.tc_free(two.auto, s))
            K.check(K.tc_alloc_at(two.overlapped, s))
        so = out["staged_overlapped"]
        off_ov2, tri_off2 = overlapped(lambda: K.check(K.tc_offload_batch(two.overlapped, items_out, copy)), so["offload_ms"], two.overlapped)
        out["next_to_a_memory_bound_kernel"]["staged_overlapped"] = {
            "offload_GBps": round(payload / off_ov2 / 1e6, 3), "offload_change_pct": round(100 * (so["offload_ms"] / off_ov2 - 1), 2),
            "neighbour_during_offload_GBps": round(tri_bytes / tri_off2 / 1e6, 1)}
        for s in src:
            K.check(K.tc_free(two.overlapped, s))
            K.check(K.tc_alloc_at(two.auto, s))

    # half of the agents go out while the other half comes back, on two streams
    dup = {}
    moved = (int(nblk[:32].sum()) + int(nblk[32:].sum())) * two.rec
    for cx, key in ((two.auto, "default_paths"), (two.staged, "staged_path")):
        if cx == two.staged:
            for s in src:
                K.check(K.tc_free(two.auto, s))
                K.check(K.tc_alloc_at(two.staged, s))
        ts = []
        for i in range(3):
            torch.cuda.synchronize()
            e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
            e0.record(copy2)
            copy.wait_event(e0)
            K.check(K.tc_upload_batch(cx, items_in[32:], copy2))
            K.check(K.tc_offload_batch(cx, items_out[:32], copy))
            e1.record(copy)
            copy2.wait_event(e1)
            e2.record(copy2)
            K.check(K.tc_sync(cx))
            torch.cuda.synchronize()
            if i:
                ts.append(e0.elapsed_time(e2))
        dup[key] = {"ms": round(float(np.median(ts)), 3), "aggregate_GBps": round(moved / float(np.median(ts)) / 1e6, 3)}
    out["half_out_while_half_in"] = dup
    for s in src:
        K.check(K.tc_free(two.staged, s))
    del a, b, c
    two.close()
    return out


def config4(torch, K, W, link):
    """32B shape (4 MiB per block): agents of the seeded trace at the 5 %, 50 % and 100 % quantile of its sizes."""
    shape = W.CONFIGS[3]
    pool, _ = fresh_pool(torch, shape)
    agents, _ = W.dag_trace(W.rng_for(3), block_size=shape.block_size)
    sizes = sorted(a["blocks"] for a in agents)
    picks = [sizes[int(q * (len(sizes) - 1))] for q in (0.05, 0.5, 1.0)]
    two = TwoContexts(torch, K, shape, pool, None, max(picks) + 2)
    rng = W.rng_for(3, salt=52)
    stream = torch.cuda.Stream()
    rows = []
    for n in picks:
        ids = W.pick_ids(rng, shape.num_blocks, n)
        new = W.pick_ids(rng, shape.num_blocks, n, exclude=ids)
        table = torch.zeros((1, n), dtype=torch.int32, device="cuda:0")
        torch.cuda.synchronize()
        r, bufs = batch_both_ways(torch, K, two, link, [ids], [new], table, stream, n * shape.block_size)
        K.check(K.tc_host_free(two.auto, bufs[0]))
        rows.append(r)
    two.close()
    del pool
    torch.cuda.empty_cache()
    return {"workload": "32B shape: 64 layers, 32 KiB pages (4 MiB per block), 16 384 blocks (64 GiB); single agents of "
                        "the 200-agent trace at the 5 % / 50 % / 100 % quantile of its context lengths",
            "agents": rows}


def config5(torch, K, W, link):
    """70B fp8 shape with one fp32 scale per page: one wave of agents' private blocks as a batch."""
    shape = W.CONFIGS[4]
    pool, scales = fresh_pool(torch, shape)
    rng = W.rng_for(4, salt=53)
    avail = host_memory_available()
    budget = min(16 << 30, int(0.2 * avail)) if avail else 8 << 30
    tokens = W.uniform_contexts(rng, 128)
    private = (W.blocks_of(tokens, shape.block_size) - 32).astype(int)
    bound = shape.planes * shape.page_bytes + 4 * shape.scales_per_block + 256      # what a record can take at most
    arena_blocks = budget // bound
    two = TwoContexts(torch, K, shape, pool, scales.view(torch.int32), arena_blocks, overlapped=WITH_OVERLAPPED)
    wave = []
    for n in private:                 # agents in index order while the arena has room
        if sum(wave) + n + 8 > arena_blocks:
            break
        wave.append(int(n))
    total = sum(wave)
    perm = rng.permutation(shape.num_blocks).astype(np.int32)
    rest = perm[32:]                  # the first 32 stand for the shared prefix blocks, which stay
    cuts = np.cumsum(wave)[:-1]
    src = np.split(rest[:total], cuts)
    dst = np.split(rest[total:2 * total], cuts)
    tables = torch.full((len(wave), 1024), -1, dtype=torch.int32, device="cuda:0")
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    out, _ = batch_both_ways(torch, K, two, link, src, dst, [tables[i].data_ptr() + 128 for i in range(len(wave))], stream,
                             total * shape.block_size)
    out["workload"] = (f"70B fp8 shape: 80 layers, 32-token blocks, 32 KiB pages + 160 fp32 scale words (record {two.rec} B), "
                       f"32 768 blocks (160 GiB); one wave of {len(wave)} of the 128 agents (contexts uniform 1k..32k tokens, "
                       f"32 shared prefix blocks stay), sized to a pinned arena of {budget / 2 ** 30:.0f} GiB")
    two.close()
    del pool, scales
    torch.cuda.empty_cache()
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

    global WITH_OVERLAPPED
    WITH_OVERLAPPED = not args.no_overlapped
    if args.config:
        stream = torch.cuda.Stream()
        link = pinned_link_peak(torch, 512 << 20, stream)
        if args.config == 3:
            one = config3(torch, K, W, link, fresh_pool(torch, W.CONFIGS[2])[0])
        else:
            one = {1: config1, 4: config4, 5: config5}[args.config](torch, K, W, link)
        print(json.dumps({"config": str(args.config), **one}))
        return

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
    rc, ctx = K.tc_create(pool, None, L, NB, pb, shape.block_size, 0, host_arena_bytes=(n + 1) * 2 * L * pb)
    K.check(rc)
    rec = K.tc_record_bytes(ctx)
    payload = n * rec
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
    ref_gbps = contiguous_copy_reference(torch, K, payload)

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
    K.check(K.tc_host_free(ctx, host))
    K.check(K.tc_destroy(ctx))

    ms_per_step = wall * 1e3 / args.steps
    value = 2 * payload * args.steps / wall / 1e9

    # HBM traffic per launch from the committed rocprofv3 counter runs; valid for this launch size only
    measured = {}
    try:
        with open(os.path.join(os.path.dirname(os.path.abspath(K.library_path())), "measured_traffic.json")) as f:
            measured = json.load(f)
    except OSError:
        pass

    def roof(name, launches, nbytes, ms, where):
        if not launches:
            return None
        avg_ms = ms / launches
        # measured per transfer of this size (all launches of the transfer together), spread over its launches
        per_transfer = measured.get("launches_per_transfer", {}).get(name)
        traffic = None
        if per_transfer and measured.get("record_bytes_per_transfer") == nbytes // launches * per_transfer:
            traffic = int(round(measured[name] / per_transfer))
        achieved = 2.0 * nbytes / launches / (avg_ms * 1e-3) / 1e9   # read + write per payload byte
        return {"kernel": name, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                "launches": int(launches), "avg_launch_us": round(avg_ms * 1e3, 2),
                "algorithmic_bytes_per_launch": int(2 * nbytes // launches),
                "contiguous_copy_kernel_GBps": round(ref_gbps, 1), "measured_in": where}

    # the two-stage path forced in both directions, same agent, same launch configuration, after the timed steps
    staged, st2 = variant(torch, K, pool, shape, pairs, link,
                          "direct_offload = direct_upload = TC_PATH_STAGED, no host tail: gather_pages -> DMA, DMA -> scatter_pages",
                          steps=12, direct_offload=K.TC_PATH_STAGED, direct_upload=K.TC_PATH_STAGED, host_tail_div=1)
    # `roofline`: the HBM-bound kernel of the timed steps.  With the default paths that is gather_pages; the upload's
    # scatter reads pinned memory and is bound by the host link (it runs at the link rate, see pct_of_pinned_link).
    # scatter_pages of the two-stage path is listed next to it, timed on the same agent right after.
    dominant = roof("gather_pages", st.gather_launches, st.gather_bytes, st.gather_ms, "the timed steps (default paths)")
    others = [roof("scatter_pages", st2.scatter_launches, st2.scatter_bytes, st2.scatter_ms, "the staged-path run after the timed steps"),
              roof("gather_pages", st2.gather_launches, st2.gather_bytes, st2.gather_ms, "the staged-path run after the timed steps")]
    if dominant is None:        # the path was forced away from staging by an option: fall back to the staged run
        dominant, others = others[0], others[1:]

    out = {
        "metric": "KV offload/upload GB/s (% of HBM and host-link peak); upload ms per 1k tokens", "value": round(value, 3), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": "configs[1] llama3-8b-shaped KV: 32 layers x K,V x 8 heads x 128 x 16 tok bf16 "
                               "(2 MiB/block), 16384-block pool (32 GiB), one agent, "
                               f"{args.tokens} tokens = {n} blocks scattered uniformly",
                   "payload_bytes_each_way": payload, "tokens": n * shape.block_size,
                   "paths": "library defaults: offload staged (gather_pages + D2H DMA), upload direct (scatter_pages reads pinned memory, 16 workgroups)"},
        **rates(payload, off_ms, up_ms, link, n * shape.block_size),
        "pinned_link_GBps": {k: round(v, 3) for k, v in link.items()},
        "roofline": dominant, "roofline_other_kernels": [r for r in others if r],
        "timed_steps_link_bound_kernel": {"kernel": "scatter_pages reading pinned host memory (16 workgroups)",
                                          "launches": int(st.direct_launches),
                                          "avg_launch_ms": round(st.direct_ms / max(1, st.direct_launches), 4),
                                          "GBps": round(st.direct_bytes / max(st.direct_ms, 1e-9) / 1e6, 3), "bound": "host link"},
        "staged_path": staged,
    }
    out["direct_paths"] = variant(torch, K, pool, shape, pairs, link,
                                  "direct_offload = direct_upload = TC_PATH_DIRECT (6 / 16 workgroups): no staging, no DMA",
                                  direct_offload=K.TC_PATH_DIRECT, direct_upload=K.TC_PATH_DIRECT)[0]
    if WITH_OVERLAPPED:
        out["staged_overlapped"] = variant(torch, K, pool, shape, pairs, link,
                                           "two-stage path with overlap_kernels = 1: a short first chunk (32 MiB), then the rest, the "
                                           "copy kernels on the context's own stream under the DMA of the neighbouring chunk",
                                           direct_offload=K.TC_PATH_STAGED, direct_upload=K.TC_PATH_STAGED, host_tail_div=1,
                                           overlap_kernels=1)[0]
    out["host_tail"] = variant(torch, K, pool, shape, pairs, link,
                               "staged both ways with host_tail_div = 64: the last 1/64 of the chunk crosses the link inside "
                               "the copy launch; the launches get longer, the transfer shorter",
                               direct_offload=K.TC_PATH_STAGED, direct_upload=K.TC_PATH_STAGED, host_tail_div=64)[0]
    if not args.no_configs:
        cfgs = {"1": config1(torch, K, W, link), "3": config3(torch, K, W, link, pool)}
        del pool
        torch.cuda.empty_cache()
        cfgs["4"] = config4(torch, K, W, link)
        cfgs["5"] = config5(torch, K, W, link)
        out["configs"] = cfgs
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, ids_a, ids_b)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
