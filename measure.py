#!/usr/bin/env python3
"""Measurements beyond the benchmark line (bench.py covers configurations 1, 2, 3 and 5 and the overlap).

    python3 measure.py [--only hbm_limits,contention,dma_spread,sweep,naive,config4,config4_replay,forecast_noise,lds,host]
                       [--out FILE]

Prints one JSON object per measurement (and writes them to --out).  Needs a GPU.  Kernel and transfer
times are HIP events on the stream of the work unless stated; GB = 1e9 bytes.
  hbm_limits  what HBM gives a streaming kernel on 512 MiB that no cache holds: reading only, writing only
           (non-temporal), a contiguous copy, and the two page kernels on device-resident records.  This is
           the program the counter passes under profiles/ run.
  contention  a 512 MiB transfer of every path and launch width next to a kernel that saturates HBM on
           another stream: how much the transfer slows down, how much the neighbour does
  dma_spread  repeated two-chunk staged transfers of 4 MiB records: spread of the copy engine's per-chunk rate
  sweep    offload / upload time against the number of blocks (64..320, the range of Sec. 7.6), for the 8B
           shape and the paper's 14B shape, with the per-block constants of the linear cost model (Eq. 2)
  naive    the same 256-block transfer done with one hipMemcpyAsync per page and with one
           hipMemcpy2DAsync per block, no gather kernel (comparators)
  config4  32B shape (4 MiB per block): per-agent transfer rates over the trace's agent sizes
  config4_replay  the 200-agent trace in real time (about 27 s): share of uploads that are complete when
           the tool returns, stall otherwise, per-transfer rates
  forecast_noise  that replay with the forecaster of Eq. 1 and noisy user estimates (sigma 0, 0.25, 0.5)
  lds      a contiguous 512 MiB device copy through registers (what the copy kernels do), staged in LDS,
           and with LDS-direct loads: what LDS adds to a copy without reuse
  host     host-side cost of the calls around a 256-block transfer (bookkeeping, enqueue, index, keys),
           median and worst of many repetitions, through the ctypes binding (about 2 us of that is Python)
"""
import argparse
import json
import os
import sys
import time

import numpy as np


def _sync_time(torch, fn, reps=5, warm=1):
    """Median wall time of fn() + device synchronisation (host-side view of a whole call)."""
    ts = []
    for i in range(reps + warm):
        torch.cuda.synchronize()
        t = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        if i >= warm:
            ts.append(time.perf_counter() - t)
    return float(np.median(ts))


def _events(torch, stream, fn, after=None, reps=5, warm=1):
    """Event-timed fn() on `stream`: (median, best, worst) in ms.  after() retires what fn enqueued."""
    ts = []
    for i in range(reps + warm):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        fn()
        e1.record(stream)
        if after:
            after()
        stream.synchronize()
        if i >= warm:
            ts.append(e0.elapsed_time(e1))
    return float(np.median(ts)), float(min(ts)), float(max(ts))


class Ctx:
    def __init__(self, torch, K, W, shape, seed, arena_blocks, fill=True, pool=None, **opts):
        self.torch, self.K, self.shape = torch, K, shape
        if pool is not None:
            self.pool, sc = pool, None
        elif fill:
            self.pool = W.make_pool_device(shape, seed)
            sc = W.make_scales_device(shape, seed)
        else:
            self.pool = torch.empty(shape.pool_bytes, dtype=torch.uint8, device="cuda:0")
            self.pool.view(torch.int32).random_(0, 2 ** 31 - 1)
            sc = torch.rand(shape.scales_per_block * shape.num_blocks, device="cuda:0") if shape.scales_per_block else None
        self.scales = sc
        pb, S = shape.page_bytes, shape.scales_per_block
        # an upper bound of the record size only sizes the arena; the library says what a record is
        rc, self.ctx = K.tc_create(self.pool, sc, shape.num_layers, shape.num_blocks, pb, shape.block_size, S,
                                   host_arena_bytes=arena_blocks * (shape.planes * pb + 4 * S + 256), **opts)
        K.check(rc)
        self.rec = K.tc_record_bytes(self.ctx)

    def close(self):
        self.K.check(self.K.tc_destroy(self.ctx))
        self.pool = self.scales = None
        self.torch.cuda.empty_cache()


def m_hbm_limits(torch, K, W, emit, reps=12):
    """512 MiB per launch, every launch on memory that no cache holds: the regions rotate through 3 GiB, the
    block sets through the whole 32 GiB pool."""
    shape = W.CONFIGS[1]
    c = Ctx(torch, K, W, shape, 1, 1, fill=False)
    n, slots = 256, 6
    nbytes = n * c.rec
    src = torch.empty(slots * nbytes, dtype=torch.uint8, device="cuda:0")
    src.view(torch.int32).random_(0, 2 ** 31 - 1)
    dst = torch.zeros(slots * nbytes, dtype=torch.uint8, device="cuda:0")
    perm = W.rng_for(1, salt=60).permutation(shape.num_blocks).astype(np.int32)
    sets = [np.ascontiguousarray(perm[k * n:(k + 1) * n]) for k in range(shape.num_blocks // n)]
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    k = [0]

    def region(t):
        return t.data_ptr() + (k[0] % slots) * nbytes

    # the same 32 GiB seen as one layer of 32 x as many blocks: every 32 KiB page of a transfer lies at a random
    # place, instead of 64 pages of one block at the same offset in 64 planes
    import dataclasses
    flat_shape = dataclasses.replace(shape, num_layers=1, num_blocks=shape.num_blocks * shape.num_layers)
    flat = Ctx(torch, K, W, flat_shape, 1, 1, pool=c.pool)
    n_flat = nbytes // flat.rec
    perm_flat = W.rng_for(1, salt=63).permutation(flat_shape.num_blocks).astype(np.int32)
    sets_flat = [np.ascontiguousarray(perm_flat[j * n_flat:(j + 1) * n_flat]) for j in range(16)]
    kernels = (
        ("read only (tc_hbm_read)", 1, c, lambda: K.tc_hbm_read(region(src), nbytes, stream)),
        ("write only, non-temporal (tc_hbm_write)", 1, c, lambda: K.tc_hbm_write(region(dst), nbytes, stream)),
        ("contiguous copy (tc_copy_contiguous)", 2, c, lambda: K.tc_copy_contiguous(region(dst), region(src), nbytes, stream)),
        ("gather_pages: scattered pool pages -> device records", 2, c,
         lambda: K.tc_stage_on_device(c.ctx, 0, sets[k[0] % len(sets)], region(dst), stream)),
        ("scatter_pages: device records -> scattered pool pages", 2, c,
         lambda: K.tc_stage_on_device(c.ctx, 1, sets[k[0] % len(sets)], region(src), stream)),
        ("gather_pages, every page at a random place (one-layer view)", 2, flat,
         lambda: K.tc_stage_on_device(flat.ctx, 0, sets_flat[k[0] % 16], region(dst), stream)),
        ("scatter_pages, every page at a random place (one-layer view)", 2, flat,
         lambda: K.tc_stage_on_device(flat.ctx, 1, sets_flat[k[0] % 16], region(src), stream)),
    )
    rows = []
    for name, ways, owner, fn in kernels:
        ts = []
        for i in range(reps + 2):
            k[0] += 1
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            K.check(fn())
            e1.record(stream)
            K.check(K.tc_sync(owner.ctx))
            stream.synchronize()
            if i >= 2:
                ts.append(e0.elapsed_time(e1) * 1e3)
        avg = float(np.mean(ts))
        rows.append(dict(kernel=name, launches=reps + 2, bytes_per_launch=ways * nbytes, avg_us=round(avg, 2),
                         best_us=round(min(ts), 2), worst_us=round(max(ts), 2), TBps=round(ways * nbytes / avg / 1e6, 3),
                         frac_of_8TBps=round(ways * nbytes / avg / 1e6 / 8, 4)))
    K.check(K.tc_destroy(flat.ctx))
    # the scatter on records a kernel has written just before with ordinary (write-back) stores: part of them is
    # still in the 256 MiB memory-side cache, which is the state the scatter finds under rocprofv3 (whose copies are
    # kernels) and never behind a copy engine
    ts = []
    for i in range(reps + 2):
        k[0] += 1
        K.check(K.tc_stage_on_device(c.ctx, 0, sets[(k[0] + 7) % len(sets)], region(dst), stream))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        K.check(K.tc_stage_on_device(c.ctx, 1, sets[k[0] % len(sets)], region(dst), stream))
        e1.record(stream)
        K.check(K.tc_sync(c.ctx))
        stream.synchronize()
        if i >= 2:
            ts.append(e0.elapsed_time(e1) * 1e3)
    avg = float(np.mean(ts))
    rows.append(dict(kernel="scatter_pages on records a gather has just written (write-back stores, partly cached)",
                     launches=reps + 2, bytes_per_launch=2 * nbytes, avg_us=round(avg, 2), best_us=round(min(ts), 2),
                     worst_us=round(max(ts), 2), TBps=round(2 * nbytes / avg / 1e6, 3), frac_of_8TBps=round(2 * nbytes / avg / 1e6 / 8, 4)))
    rd, wr = rows[0]["avg_us"], rows[1]["avg_us"]
    emit(dict(measurement="hbm_limits", MiB_one_way=nbytes / 2 ** 20, reps=reps, rows=rows,
              read_time_plus_write_time_us=round(rd + wr, 2),
              note="a copy takes about as long as reading its bytes and then writing them: the two directions "
                   "share the memory system instead of overlapping"))
    del src, dst
    c.close()


def m_contention(torch, K, W, emit):
    """One 256-block agent (512 MiB), three transfers in a row, while an fp32 triad over 3 x 4 GiB keeps HBM busy
    on another stream.  Against each of them alone."""
    shape = W.CONFIGS[1]
    c0 = Ctx(torch, K, W, shape, 1, 1, fill=False)
    pool = c0.pool
    K.check(K.tc_destroy(c0.ctx))
    m = 1 << 30
    a, b, cc = torch.zeros(m, device="cuda:0"), torch.rand(m, device="cuda:0"), torch.rand(m, device="cuda:0")
    stream, compute = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()

    def tri(iters):
        K.check(K.tc_hbm_stream(a, b, cc, m, 0.5, iters, compute))

    tri(4)
    compute.synchronize()
    t_tri = _events(torch, compute, lambda: tri(8), reps=3)[0] / 8
    n = 256
    perm = W.rng_for(1, salt=61).permutation(shape.num_blocks).astype(np.int32)
    ids = np.ascontiguousarray(perm[:n])
    rows = []
    cases = [("staged", K.TC_PATH_STAGED, 0)] + [("direct", K.TC_PATH_DIRECT, g) for g in (6, 8, 16, 32)]
    for name, mode, grid in cases:
        d = Ctx(torch, K, W, shape, 1, n + 1, pool=pool, direct_offload=mode, direct_upload=mode, host_tail_div=1,
                direct_grid=grid)
        K.check(K.tc_alloc_at(d.ctx, ids))
        rc, buf = K.tc_host_alloc(d.ctx, n)
        K.check(rc)
        row = dict(path=name, workgroups=grid or None)
        for dname, fn in (("offload", lambda: K.check(K.tc_offload(d.ctx, ids, buf, stream))),
                          ("upload", lambda: K.check(K.tc_upload(d.ctx, buf, ids, None, stream)))):
            alone = _events(torch, stream, fn, after=lambda: K.check(K.tc_sync(d.ctx)), reps=3)[0]
            iters = int(4 * alone / t_tri) + 4
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            torch.cuda.synchronize()
            ev[0].record(compute)
            tri(iters)
            ev[1].record(compute)
            time.sleep(0.003)                      # the neighbour is running before the first transfer starts
            ev[2].record(stream)
            for _ in range(3):
                fn()
            ev[3].record(stream)
            K.check(K.tc_sync(d.ctx))
            torch.cuda.synchronize()
            busy = ev[2].elapsed_time(ev[3]) / 3
            lost = ev[0].elapsed_time(ev[1]) - iters * t_tri      # what the neighbour lost, all of it during the overlap
            row[dname] = dict(alone_ms=round(alone, 3), next_to_neighbour_ms=round(busy, 3),
                              transfer_slower_pct=round(100 * (busy / alone - 1), 1),
                              neighbour_slower_pct_while_overlapped=round(100 * lost / (3 * busy), 1))
        rows.append(row)
        K.check(K.tc_free(d.ctx, ids))
        K.check(K.tc_host_free(d.ctx, buf))
        K.check(K.tc_destroy(d.ctx))
    emit(dict(measurement="contention", MiB=n * 2, neighbour="fp32 triad a = b + s c over 3 x 4 GiB",
              neighbour_alone_GBps=round(12 * m / t_tri / 1e6, 1), rows=rows))
    del a, b, cc, pool
    torch.cuda.empty_cache()


class _LinkWatch:
    """Samples what the kernel driver reports about the GPU's PCIe link (sysfs, world-readable) while a transfer
    runs: the distinct values seen, in order of first appearance."""

    FILES = ("current_link_speed", "current_link_width", "pp_dpm_pcie", "pp_dpm_fclk", "pp_dpm_socclk", "pp_dpm_mclk")

    def __init__(self):
        import glob
        import threading
        self.paths = [p for f in self.FILES for p in sorted(glob.glob("/sys/class/drm/card*/device/" + f))]
        self.seen, self.stop, self.thread, self._threading = [], False, None, threading

    def _read(self):
        out = []
        for p in self.paths:
            try:
                with open(p) as f:
                    txt = f.read()
                if "pp_dpm_" in p:
                    txt = " ".join(l.strip() for l in txt.splitlines() if l.rstrip().endswith("*"))
                out.append(txt.strip())
            except OSError:
                out.append("?")
        return tuple(out)

    def __enter__(self):
        self.seen, self.stop = [], False

        def loop():
            while not self.stop:
                v = self._read()
                if v not in self.seen:
                    self.seen.append(v)
                time.sleep(0.002)
        self.thread = self._threading.Thread(target=loop, daemon=True)
        self.thread.start()
        return self

    def __exit__(self, *a):
        self.stop = True
        self.thread.join()


def m_dma_spread(torch, K, W, emit, reps=24):
    """Staged transfers of 1 006 records of 4 MiB, one after the other with nothing else on the GPU, through a
    context with 512 MiB staging slots (eight chunks, eight DMAs each way) and through one with the default 4 GiB
    slots (one chunk, one DMA): the copy engine's rate per transfer, from the event pairs the library puts around
    each chunk, and what the driver said about the PCIe link meanwhile.  A DMA enqueued while the previous one of
    the stream is still running is now and then carried out at about half rate; a single DMA never was."""
    shape = W.CONFIGS[3]
    n = 1006
    staged = dict(direct_offload=K.TC_PATH_STAGED, direct_upload=K.TC_PATH_STAGED, host_tail_div=1)
    one = Ctx(torch, K, W, shape, 3, n + 2, fill=False, **staged)                          # default slots: one chunk
    rec = one.rec
    eight = Ctx(torch, K, W, shape, 3, 0, pool=one.pool, staging_bytes=2 * 128 * rec, staging_slots=2, **staged)
    ids = W.pick_ids(W.rng_for(3, salt=62), shape.num_blocks, n)
    rc, buf = K.tc_host_alloc(one.ctx, n)
    K.check(rc)
    stream = torch.cuda.Stream()
    watch = _LinkWatch()
    out = {}
    for name, c in (("eight_chunks", eight), ("one_chunk", one)):
        K.check(K.tc_alloc_at(c.ctx, ids))
        K.check(K.tc_set_profiling(c.ctx, 1))
    prev = {id(c): K.tc_stats(c.ctx)[1] for c in (eight, one)}
    rows = {"eight_chunks": [], "one_chunk": []}
    for r in range(reps):
        if r % 3 == 2:
            time.sleep(0.5)                  # an idle gap, as between the agents of a trace
        for name, c in (("eight_chunks", eight), ("one_chunk", one)):      # in turn, so that both see the same moments
            with watch:
                off = _events(torch, stream, lambda: K.check(K.tc_offload(c.ctx, ids, buf, stream)),
                              after=lambda: K.check(K.tc_sync(c.ctx)), reps=1, warm=0)[0]
            link_off = list(watch.seen)
            with watch:
                up = _events(torch, stream, lambda: K.check(K.tc_upload(c.ctx, buf, ids, None, stream)),
                             after=lambda: K.check(K.tc_sync(c.ctx)), reps=1, warm=0)[0]
            st, p = K.tc_stats(c.ctx)[1], prev[id(c)]
            rows[name].append(dict(rep=r, after_idle_gap=(r % 3 == 2),
                                   offload_GBps=round(n * rec / off / 1e6, 2), upload_GBps=round(n * rec / up / 1e6, 2),
                                   d2h_dma_GBps=round((st.d2h_bytes - p.d2h_bytes) / max(st.d2h_ms - p.d2h_ms, 1e-9) / 1e6, 2),
                                   h2d_dma_GBps=round((st.h2d_bytes - p.h2d_bytes) / max(st.h2d_ms - p.h2d_ms, 1e-9) / 1e6, 2),
                                   dmas_each_way=int(st.d2h_copies - p.d2h_copies),
                                   link_during_offload=link_off, link_during_upload=list(watch.seen)))
            prev[id(c)] = st
    for name, v in rows.items():
        rates = [x for r_ in v for x in (r_["offload_GBps"], r_["upload_GBps"])]
        out[name] = dict(transfers=len(rates), below_50_GBps=sum(x < 50 for x in rates), slowest_GBps=min(rates),
                         median_GBps=float(np.median(rates)), rows=v)
    emit(dict(measurement="dma_spread", shape=shape.name, blocks=n, GiB=n * rec / 2 ** 30, link_files=watch.paths, **out))
    for c in (eight, one):
        K.check(K.tc_free(c.ctx, ids))
    K.check(K.tc_host_free(one.ctx, buf))
    K.check(K.tc_destroy(eight.ctx))
    one.close()


def m_sweep(torch, K, W, emit):
    for shape in (W.CONFIGS[1], W.PAPER_14B):
        c = Ctx(torch, K, W, shape, 1, 330, fill=False)
        rng = W.rng_for(1, salt=50)
        stream = torch.cuda.Stream()
        rows = []
        for n in (64, 128, 192, 256, 320):
            ids = W.pick_ids(rng, shape.num_blocks, n)
            new = W.pick_ids(rng, shape.num_blocks, n, exclude=ids)
            rc, host = K.tc_host_alloc(c.ctx, n)
            K.check(rc)
            K.check(K.tc_alloc_at(c.ctx, ids))
            K.check(K.tc_alloc_at(c.ctx, new))
            table = torch.zeros(n, dtype=torch.int32, device="cuda:0")
            done = lambda: K.check(K.tc_sync(c.ctx))
            t_off = _events(torch, stream, lambda: K.check(K.tc_offload(c.ctx, ids, host, stream)), done, reps=7)[0] * 1e-3
            t_up = _events(torch, stream, lambda: K.check(K.tc_upload(c.ctx, host, new, table, stream)), done, reps=7)[0] * 1e-3
            K.check(K.tc_sync(c.ctx))
            K.check(K.tc_free(c.ctx, ids))
            K.check(K.tc_free(c.ctx, new))
            K.check(K.tc_host_free(c.ctx, host))
            rows.append(dict(blocks=n, tokens=n * shape.block_size, MiB=n * c.rec / 2 ** 20,
                             offload_ms=t_off * 1e3, upload_ms=t_up * 1e3,
                             offload_GBps=n * c.rec / t_off / 1e9, upload_GBps=n * c.rec / t_up / 1e9))
        N = np.array([r["blocks"] for r in rows], dtype=float)
        fit = {}
        for key in ("offload_ms", "upload_ms"):
            y = np.array([r[key] for r in rows])
            b, a = np.polyfit(N, y, 1)
            ss_res = float(((y - (a + b * N)) ** 2).sum())
            ss_tot = float(((y - y.mean()) ** 2).sum())
            fit[key] = dict(a_ms=float(a), b_ms_per_block=float(b), r2=1 - ss_res / ss_tot)
        emit(dict(measurement="sweep", shape=shape.name, record_MiB=c.rec / 2 ** 20, rows=rows, linear_fit=fit))
        c.close()


def m_naive(torch, K, W, emit):
    shape = W.CONFIGS[1]
    c = Ctx(torch, K, W, shape, 1, 260, fill=False)
    rng = W.rng_for(1, salt=51)
    n = 256
    ids = W.pick_ids(rng, shape.num_blocks, n)
    rc, host = K.tc_host_alloc(c.ctx, n)
    K.check(rc)
    K.check(K.tc_alloc_at(c.ctx, ids))
    stream = torch.cuda.Stream()
    table = torch.zeros(n, dtype=torch.int32, device="cuda:0")
    out = dict(measurement="naive", shape=shape.name, blocks=n, MiB=n * c.rec / 2 ** 20)
    nbytes = n * c.rec
    t = _sync_time(torch, lambda: K.check(K.tc_offload(c.ctx, ids, host, stream)))
    out["library_offload_ms"], out["library_offload_GBps"] = t * 1e3, nbytes / t / 1e9
    t = _sync_time(torch, lambda: K.check(K.tc_upload(c.ctx, host, ids, table, stream)))
    out["library_upload_ms"], out["library_upload_GBps"] = t * 1e3, nbytes / t / 1e9
    for mode, name in ((0, "per_page_memcpy"), (1, "per_block_memcpy2d")):
        for direction, dname in ((0, "offload"), (1, "upload")):
            t = _sync_time(torch, lambda: K.check(K.tc_naive_transfer(c.ctx, ids, host, mode, direction, stream)), reps=3)
            out[f"{name}_{dname}_ms"], out[f"{name}_{dname}_GBps"] = t * 1e3, nbytes / t / 1e9
    emit(out)
    c.close()


def m_config4(torch, K, W, emit):
    shape = W.CONFIGS[3]
    agents, _ = W.dag_trace(W.rng_for(3), block_size=shape.block_size)
    sizes = sorted(a["blocks"] for a in agents)
    picks = [sizes[int(q * (len(sizes) - 1))] for q in (0.05, 0.25, 0.5, 0.75, 0.95, 1.0)]
    c = Ctx(torch, K, W, shape, 3, max(picks) + 2, fill=False)
    rng = W.rng_for(3, salt=52)
    stream = torch.cuda.Stream()
    rows = []
    for n in picks:
        ids = W.pick_ids(rng, shape.num_blocks, n)
        new = W.pick_ids(rng, shape.num_blocks, n, exclude=ids)
        rc, host = K.tc_host_alloc(c.ctx, n)
        K.check(rc)
        K.check(K.tc_alloc_at(c.ctx, ids))
        K.check(K.tc_alloc_at(c.ctx, new))
        table = torch.zeros(n, dtype=torch.int32, device="cuda:0")
        done = lambda: K.check(K.tc_sync(c.ctx))
        t_off = _events(torch, stream, lambda: K.check(K.tc_offload(c.ctx, ids, host, stream)), done)[0] * 1e-3
        t_up = _events(torch, stream, lambda: K.check(K.tc_upload(c.ctx, host, new, table, stream)), done)[0] * 1e-3
        for x in (ids, new):
            K.check(K.tc_free(c.ctx, x))
        K.check(K.tc_host_free(c.ctx, host))
        rows.append(dict(blocks=n, tokens=n * shape.block_size, MiB=n * c.rec / 2 ** 20, offload_ms=t_off * 1e3,
                         upload_ms=t_up * 1e3, offload_GBps=n * c.rec / t_off / 1e9, upload_GBps=n * c.rec / t_up / 1e9,
                         upload_ms_per_1k_tokens=t_up * 1e3 / (n * shape.block_size / 1024)))
    emit(dict(measurement="config4", shape=shape.name, record_MiB=c.rec / 2 ** 20,
              agent_size_quantiles=[0.05, 0.25, 0.5, 0.75, 0.95, 1.0], rows=rows))
    c.close()


def _replay(torch, K, W, ctx_obj, agents, events, speed, predict_ms=None, observe=None, lead_ms=200.0):
    """Real-time replay of a trace on one copy stream.  predict_ms(i) -> predicted call duration at
    call_start (None = the trace's own upload times); observe(i, elapsed_ms) at call_finish."""
    import heapq
    c, shape = ctx_obj, ctx_obj.shape
    stream = torch.cuda.Stream()
    tables = torch.full((len(agents), 1025), -1, dtype=torch.int32, device="cuda:0")
    A = [dict(state="new") for _ in agents]
    ops, stalls, ready, rejected = [], [], 0, 0
    heap = [(t * 1e3, k, kind, i) for k, (t, _, kind, i) in enumerate(events)
            if not (predict_ms and kind == "upload_due")]
    heapq.heapify(heap)
    seq = 10 * len(events)

    def timed(kind, i, nbytes, fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        fn()
        e1.record(stream)
        ops.append((kind, i, nbytes, e0, e1))
        return e1

    def upload(i):
        a, n = A[i], agents[i]["blocks"]
        rc, new = K.tc_alloc(c.ctx, n)
        if rc != 0:
            return False
        a["up_done"] = timed("upload", i, n * c.rec, lambda: K.check(K.tc_upload(c.ctx, a["buf"], new, tables[i], stream)))
        K.check(K.tc_host_free(c.ctx, a["buf"]))
        a.update(state="uploaded", ids=new)
        return True

    t_wall0 = time.perf_counter()
    while heap:
        t, _, kind, i = heapq.heappop(heap)
        delay = t * 1e-3 / speed - (time.perf_counter() - t_wall0)
        if delay > 0:
            time.sleep(delay)
        a, n = A[i], agents[i]["blocks"]
        K.check(K.tc_poll(c.ctx))
        if kind == "start":
            rc, ids = K.tc_alloc(c.ctx, n)
            K.check(rc)
            a.update(state="running", ids=ids)
        elif kind == "call_start":
            a["t_call"] = t
            if predict_ms:
                seq += 1
                heapq.heappush(heap, (t + max(0.0, predict_ms(i) - lead_ms), seq, "upload_due", i))
            rc, buf = K.tc_host_alloc(c.ctx, n)
            if rc != 0:
                rejected += 1
                a["state"] = "kept"
                continue
            a["buf"] = buf
            timed("offload", i, n * c.rec, lambda: K.check(K.tc_offload(c.ctx, a["ids"], buf, stream)))
            K.check(K.tc_free(c.ctx, a["ids"]))
            a["state"] = "offloaded"
        elif kind == "upload_due":
            if a["state"] == "offloaded":
                upload(i)
        elif kind == "call_finish":
            if observe:
                observe(i, t - a["t_call"])
            if a["state"] == "offloaded":
                while not upload(i):            # blocks are still pending-free: wait for the copy stream
                    K.check(K.tc_sync(c.ctx))
            if a["state"] == "uploaded":
                t0 = time.perf_counter()
                if a["up_done"].query():
                    ready += 1
                    stalls.append(0.0)
                else:
                    a["up_done"].synchronize()
                    stalls.append((time.perf_counter() - t0) * 1e3)
                a["state"] = "running"
        elif kind == "finish":
            K.check(K.tc_free(c.ctx, a["ids"]))
    torch.cuda.synchronize()
    K.check(K.tc_sync(c.ctx))
    rates = {k: np.array([nb / (e0.elapsed_time(e1) * 1e-3) / 1e9 for kk, _, nb, e0, e1 in ops if kk == k]) for k in ("offload", "upload")}
    ms1k = np.array([e0.elapsed_time(e1) / (nb / c.rec * shape.block_size / 1024) for kk, _, nb, e0, e1 in ops if kk == "upload"])
    stalls = np.array(stalls)
    q = lambda x: [float(np.percentile(x, p)) for p in (5, 50, 95)]
    late = stalls[stalls > 0]
    return dict(speed=speed, wall_s=time.perf_counter() - t_wall0, offloads=len(rates["offload"]),
                rejected_cpu_capacity=rejected, uploads=len(stalls), uploads_complete_before_call_finish=ready,
                fraction_ready=ready / max(1, len(stalls)), mean_stall_ms=float(stalls.mean()) if len(stalls) else 0.0,
                stall_ms_when_not_ready_p50_p95_max=[float(np.percentile(late, p)) for p in (50, 95, 100)] if len(late) else [0, 0, 0],
                offload_GBps_p5_p50_p95=q(rates["offload"]), upload_GBps_p5_p50_p95=q(rates["upload"]),
                upload_ms_per_1k_tokens_p5_p50_p95=q(ms1k))


def m_config4_replay(torch, K, W, emit, speed=1.0):
    """Real-time replay of the config-4 trace: every call offloads (if the 16 GiB arena has room), the
    upload is issued 200 ms before the predicted finish (constant 2 s prediction) or at the finish when
    the tool returns early.  Reports how often the KV is back when the tool returns, the stall when it
    is not, and the per-transfer rates."""
    shape = W.CONFIGS[3]
    agents, events = W.dag_trace(W.rng_for(3), block_size=shape.block_size)
    c = Ctx(torch, K, W, shape, 3, 4096, fill=False)
    res = _replay(torch, K, W, c, agents, events, speed)
    emit(dict(measurement="config4_replay", agents=len(agents), **res))
    c.close()


def m_forecast_noise(torch, K, W, emit, speed=2.0):
    """The same trace (twice as fast) with the library's forecaster (Eq. 1) in place of the constant
    prediction: the user's estimate of a call is its true duration times lognormal noise of the given
    sigma, the history term is the per-type moving average fed by call_finish."""
    shape = W.CONFIGS[3]
    agents, events = W.dag_trace(W.rng_for(3), block_size=shape.block_size)
    c = Ctx(torch, K, W, shape, 3, 4096, fill=False)
    rows = []
    for sigma in (0.0, 0.25, 0.5):
        rng = W.rng_for(3, salt=70)
        user = [a["call_s"] * 1e3 * float(np.exp(rng.normal(0.0, sigma))) for a in agents]
        rc, f = K.tc_forecaster_create(0.8, 0.3, 2000.0)
        K.check(rc)
        res = _replay(torch, K, W, c, agents, events, speed,
                      predict_ms=lambda i: K.tc_forecaster_estimate(f, i % 4, user[i]),
                      observe=lambda i, ms: K.check(K.tc_forecaster_observe(f, i % 4, ms)))
        K.tc_forecaster_destroy(f)
        rows.append(dict(noise_sigma=sigma, **res))
    emit(dict(measurement="forecast_noise", agents=len(agents), alpha=0.8, gamma=0.3, rows=rows))
    c.close()


def m_lds(torch, K, W, emit):
    n = 512 << 20
    a = torch.empty(n, dtype=torch.uint8, device="cuda:0")
    a.view(torch.int32).random_(0, 2 ** 31 - 1)
    b = torch.zeros(n, dtype=torch.uint8, device="cuda:0")
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()        # a and b were written on torch's stream
    rows = {}
    for name, fn in (("registers (tc_copy_contiguous)", lambda: K.tc_copy_contiguous(b, a, n, stream)),
                     ("registers -> LDS -> registers", lambda: K.tc_copy_via_lds(b, a, n, 0, stream)),
                     ("LDS-direct loads", lambda: K.tc_copy_via_lds(b, a, n, 1, stream))):
        ts = []
        for i in range(14):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            with torch.cuda.stream(stream):
                e0.record(stream)
                K.check(fn())
                e1.record(stream)
            stream.synchronize()
            if i >= 2:
                ts.append(e0.elapsed_time(e1) * 1e3)
        assert torch.equal(a, b)
        b.zero_()
        torch.cuda.synchronize()
        rows[name] = dict(mean_us=round(float(np.mean(ts)), 1), best_us=round(float(min(ts)), 1),
                          TBps_of_traffic=round(2 * n / (float(np.mean(ts)) * 1e-6) / 1e12, 2))
    emit(dict(measurement="lds", MiB=512, rows=rows))


def m_host(torch, K, W, emit):
    """Sec. 6.3 and 7.6 argue that allocation on the migration path has to stay far below a millisecond."""
    shape = W.CONFIGS[1]
    c = Ctx(torch, K, W, shape, 1, 1024, fill=False)
    n = 256
    stream = torch.cuda.Stream()
    out = {}

    def rep(name, fn, reps=2000):
        ts = []
        for _ in range(reps):
            t = time.perf_counter()
            fn()
            ts.append(time.perf_counter() - t)
        ts = np.asarray(ts[reps // 10:]) * 1e6
        out[name] = dict(median_us=round(float(np.median(ts)), 2), p99_us=round(float(np.percentile(ts, 99)), 2),
                         worst_us=round(float(ts.max()), 2))

    def alloc_free():
        rc, ids = K.tc_alloc(c.ctx, n)
        K.tc_free(c.ctx, ids)
    rep("tc_alloc(256) + tc_free", alloc_free)
    rc, ids = K.tc_alloc(c.ctx, n)
    K.check(K.tc_free(c.ctx, ids))

    def prefer_free():
        rc, got = K.tc_alloc_prefer(c.ctx, ids)
        K.tc_free(c.ctx, got)
    rep("tc_alloc_prefer(256) + tc_free", prefer_free)

    def host_alloc_free():
        rc, b = K.tc_host_alloc(c.ctx, n)
        K.tc_host_free(c.ctx, b)
    rep("tc_host_alloc(256) + tc_host_free", host_alloc_free)
    rep("tc_poll, nothing in flight", lambda: K.tc_poll(c.ctx))

    perm = np.random.default_rng(3).permutation(shape.num_blocks).astype(np.int32)
    src, dst = perm[:n].copy(), perm[n:2 * n].copy()
    K.check(K.tc_alloc_at(c.ctx, src))
    K.check(K.tc_alloc_at(c.ctx, dst))
    rc, buf = K.tc_host_alloc(c.ctx, n)
    table = torch.zeros(n, dtype=torch.int32, device="cuda:0")
    torch.cuda.synchronize()
    enq = {"tc_offload(256 blocks): call returns after": [], "tc_upload(256 blocks): call returns after": []}
    for _ in range(40):
        t = time.perf_counter()
        K.tc_offload(c.ctx, src, buf, stream)
        enq["tc_offload(256 blocks): call returns after"].append(time.perf_counter() - t)
        K.check(K.tc_sync(c.ctx))
        t = time.perf_counter()
        K.tc_upload(c.ctx, buf, dst, table, stream)
        enq["tc_upload(256 blocks): call returns after"].append(time.perf_counter() - t)
        K.check(K.tc_sync(c.ctx))
    for k, v in enq.items():
        v = np.asarray(v[4:]) * 1e6
        out[k] = dict(median_us=round(float(np.median(v)), 2), p99_us=round(float(np.percentile(v, 99)), 2),
                      worst_us=round(float(v.max()), 2))

    tokens = np.random.default_rng(4).integers(0, 128000, size=n * shape.block_size, dtype=np.int32)
    rep("tc_chain_hashes(4096 tokens)", lambda: K.tc_chain_hashes(tokens, shape.block_size))
    rc, keys = K.tc_chain_hashes(tokens, shape.block_size)
    rc, ix = K.tc_index_create()

    def index_cycle():
        K.tc_index_insert(ix, keys, src, buf, c.rec)
        K.tc_index_lookup(ix, keys)
        K.tc_index_begin_upload(ix, keys, dst)
        K.tc_index_finish_upload(ix, keys)
    rep("tc_index insert + lookup + begin_upload + finish_upload (256 keys)", index_cycle)
    K.tc_index_destroy(ix)
    emit(dict(measurement="host", blocks=n, calls=out))
    c.close()


ALL = dict(hbm_limits=m_hbm_limits, contention=m_contention, dma_spread=m_dma_spread, sweep=m_sweep, naive=m_naive,
           config4=m_config4, config4_replay=m_config4_replay, forecast_noise=m_forecast_noise, lds=m_lds, host=m_host)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--only", default=",".join(ALL))
    ap.add_argument("--out", default=None)
    ap.add_argument("--reps", type=int, default=0, help="repetitions for hbm_limits / dma_spread (0 = their defaults)")
    args = ap.parse_args()
    import torch
    if not torch.cuda.is_available():
        print("measure: no GPU visible; the path has no CPU fallback.", file=sys.stderr)
        sys.exit(2)
    import paper_2510_18586_amd as K
    import tc_workloads as W
    results = []

    def emit(obj):
        results.append(obj)
        print(json.dumps(obj), flush=True)

    for name in args.only.split(","):
        if args.reps and name in ("hbm_limits", "dma_spread"):
            ALL[name](torch, K, W, emit, reps=args.reps)
        else:
            ALL[name](torch, K, W, emit)
    if args.out:
        with open(args.out, "w") as f:
            json.dump(results, f, indent=1)


if __name__ == "__main__":
    main()
