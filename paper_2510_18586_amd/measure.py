"""Measurements beyond the headline benchmark line, for all five configurations.

    python -m paper_2510_18586_amd.measure [--only sweep,naive,config1,config3,config4,config4_replay,forecast_noise,config5,lds,host] [--out FILE]

Prints one JSON object per measurement (and writes them to --out).  Needs a GPU.  Times are
wall-clock around enqueue + synchronisation unless stated; GB = 1e9 bytes.
  sweep    offload / upload time against the number of blocks (64..320, the paper's Sec. 7.6 range),
           for the 8B shape and the paper's 14B shape, with the per-block constants of the linear
           cost model (Eq. 2): T(N) = a + b N
  naive    the same 256-block transfer done with one hipMemcpyAsync per page and with one
           hipMemcpy2DAsync per block, no gather kernel (comparators)
  config1  the tiny configuration: latency of an 8-block transfer
  config3  64 agents offloaded / uploaded as a batch, alone and while an HBM-streaming kernel
           runs on another stream; the neighbour's own bandwidth alone and overlapped
  config4  32B shape (4 MiB per block): per-agent transfer rates over the trace's agent sizes
  config4_replay  the 200-agent trace in real time (about 27 s): share of uploads that are complete when
           the tool returns, stall otherwise, per-transfer rates
  forecast_noise  that replay with the forecaster of Eq. 1 and noisy user estimates (sigma 0, 0.25, 0.5)
  config5  70B fp8 shape with scales: one wave of private blocks as a batch
  lds      a contiguous 512 MiB device copy through registers (what the copy kernels do), staged in LDS,
           and with LDS-direct loads: what LDS adds to a copy without reuse
  host     host-side cost of the calls around a 256-block transfer (bookkeeping, enqueue, index, keys),
           median and worst of many repetitions, through the ctypes binding (about 2 us of that is Python)
"""
import argparse
import json
import sys
import time

import numpy as np


def _sync_time(torch, fn, reps=5, warm=1):
    """Median wall time of fn() + device synchronisation."""
    ts = []
    for i in range(reps + warm):
        torch.cuda.synchronize()
        t = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        if i >= warm:
            ts.append(time.perf_counter() - t)
    return float(np.median(ts))


def _link_peak(torch, nbytes):
    nbytes = int(min(nbytes, 4 << 30))
    host = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    dev = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    d2h = nbytes / _sync_time(torch, lambda: host.copy_(dev, non_blocking=True)) / 1e9
    h2d = nbytes / _sync_time(torch, lambda: dev.copy_(host, non_blocking=True)) / 1e9
    return d2h, h2d


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
        P, pb, S = shape.planes, shape.page_bytes, shape.scales_per_block
        self.rec = (P * pb + 4 * S + 255) // 256 * 256
        rc, self.ctx = K.tc_create(self.pool, sc, shape.num_layers, shape.num_blocks, pb, shape.block_size, S,
                                   host_arena_bytes=arena_blocks * self.rec, **opts)
        K.check(rc)
        assert K.tc_record_bytes(self.ctx) == self.rec

    def close(self):
        self.K.check(self.K.tc_destroy(self.ctx))
        self.pool = self.scales = None
        self.torch.cuda.empty_cache()


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
            t_off = _sync_time(torch, lambda: K.check(K.tc_offload(c.ctx, ids, host, stream)), reps=7)
            t_up = _sync_time(torch, lambda: K.check(K.tc_upload(c.ctx, host, new, table, stream)), reps=7)
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


def m_config1(torch, K, W, emit):
    shape = W.CONFIGS[0]
    out = dict(measurement="config1", note="latency-bound: 256 KiB per direction")
    for tag, opts in (("", {}), ("direct_", dict(direct_offload=1, direct_upload=1))):
        c = Ctx(torch, K, W, shape, 0, 16, **opts)
        rng = W.rng_for(0)
        ids = W.pick_ids(rng, shape.num_blocks, 8)
        new = W.pick_ids(rng, shape.num_blocks, 8, exclude=ids)
        rc, host = K.tc_host_alloc(c.ctx, 8)
        K.check(rc)
        K.check(K.tc_alloc_at(c.ctx, ids))
        K.check(K.tc_alloc_at(c.ctx, new))
        stream = torch.cuda.Stream()
        table = torch.zeros(8, dtype=torch.int32, device="cuda:0")
        t_off = _sync_time(torch, lambda: K.check(K.tc_offload(c.ctx, ids, host, stream)), reps=50, warm=5)
        t_up = _sync_time(torch, lambda: K.check(K.tc_upload(c.ctx, host, new, table, stream)), reps=50, warm=5)
        out.update({"payload_KiB": 8 * c.rec / 1024, tag + "offload_us": t_off * 1e6, tag + "upload_us": t_up * 1e6,
                    tag + "offload_GBps": 8 * c.rec / t_off / 1e9, tag + "upload_GBps": 8 * c.rec / t_up / 1e9})
        c.close()
    emit(out)


def m_config3(torch, K, W, emit):
    shape = W.CONFIGS[2]
    rng = W.rng_for(2)
    tokens = W.lognormal_contexts(rng, 64)
    nblk = W.blocks_of(tokens, shape.block_size).astype(int)
    total = int(nblk.sum())
    c = Ctx(torch, K, W, shape, 2, total + 8, fill=False)

    class B:
        def alloc(self, n):
            rc, ids = K.tc_alloc(c.ctx, n)
            return ids if rc == 0 else None

        def free(self, ids):
            K.check(K.tc_free(c.ctx, ids))

        def n_free(self):
            return K.tc_stats(c.ctx)[1].gpu_blocks_free

    W.fragment_pool(B(), rng, n_ops=50000, need_free=total)
    src = [B().alloc(int(n)) for n in nblk]
    dst = src            # 2 x total exceeds the pool: the upload claims the original blocks again
    bufs = [K.tc_host_alloc(c.ctx, int(n))[1] for n in nblk]
    tables = torch.full((64, int(nblk.max()) + 1), -1, dtype=torch.int32, device="cuda:0")
    copy, compute = torch.cuda.Stream(), torch.cuda.Stream()
    nbytes = total * c.rec
    d2h, h2d = _link_peak(torch, nbytes)

    # the neighbour: fp32 triad over 3 x 4 GiB
    m = 1 << 30
    a = torch.zeros(m, device="cuda:0")
    b = torch.rand(m, device="cuda:0")
    cc = torch.rand(m, device="cuda:0")
    tri_bytes = 3 * 4 * m

    def offload():
        K.check(K.tc_offload_batch(c.ctx, [(src[i], bufs[i]) for i in range(64)], copy))

    def upload():
        K.check(K.tc_upload_batch(c.ctx, [(dst[i], bufs[i], tables[i]) for i in range(64)], copy))

    def offload_singles():
        for i in range(64):
            K.check(K.tc_offload(c.ctx, src[i], bufs[i], copy))

    t_off = _sync_time(torch, offload, reps=3)
    t_off1 = _sync_time(torch, offload_singles, reps=3)
    t_up = _sync_time(torch, upload, reps=3)
    t_tri = _sync_time(torch, lambda: K.check(K.tc_hbm_stream(a, b, cc, m, 0.5, 4, compute)), reps=3) / 4

    def overlapped(fn, iters):
        # neighbour runs for the whole copy; its rate is taken from its own events
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t = time.perf_counter()
        e0.record(compute)
        K.check(K.tc_hbm_stream(a, b, cc, m, 0.5, iters, compute))
        e1.record(compute)
        fn()
        copy.synchronize()
        t_copy = time.perf_counter() - t
        torch.cuda.synchronize()
        return t_copy, e0.elapsed_time(e1) * 1e-3 / iters

    iters_off = max(1, int(t_off / t_tri))
    iters_up = max(1, int(t_up / t_tri))
    overlapped(offload, iters_off)
    t_off_ov, tri_off = overlapped(offload, iters_off)
    t_up_ov, tri_up = overlapped(upload, iters_up)
    # full duplex: half of the agents go out while the other half comes back, on two streams
    copy2 = torch.cuda.Stream()
    half_bytes_out = int(nblk[:32].sum()) * c.rec
    half_bytes_in = int(nblk[32:].sum()) * c.rec

    def duplex():
        K.check(K.tc_offload_batch(c.ctx, [(src[i], bufs[i]) for i in range(32)], copy))
        K.check(K.tc_upload_batch(c.ctx, [(dst[i], bufs[i], tables[i]) for i in range(32, 64)], copy2))

    t_dup = _sync_time(torch, duplex, reps=3)
    t_out = _sync_time(torch, lambda: K.check(K.tc_offload_batch(c.ctx, [(src[i], bufs[i]) for i in range(32)], copy)), reps=3)
    t_in = _sync_time(torch, lambda: K.check(K.tc_upload_batch(
        c.ctx, [(dst[i], bufs[i], tables[i]) for i in range(32, 64)], copy2)), reps=3)
    # the same with offloads written by the gather kernel straight into pinned memory while uploads are
    # in flight (direct_offload = 2), and the neighbour's rate next to such direct offloads (= 1)
    direct = {}
    for mode in (2, 1):
        d = Ctx(torch, K, W, shape, 2, total + 8, pool=c.pool, direct_offload=mode)
        for i in range(64):
            K.check(K.tc_alloc_at(d.ctx, src[i]))
        dbufs = [K.tc_host_alloc(d.ctx, int(n))[1] for n in nblk]
        K.check(K.tc_offload_batch(d.ctx, [(src[i], dbufs[i]) for i in range(64)], copy))
        K.check(K.tc_sync(d.ctx))

        def dduplex():
            K.check(K.tc_upload_batch(d.ctx, [(src[i], dbufs[i], tables[i]) for i in range(32, 64)], copy2))
            K.check(K.tc_offload_batch(d.ctx, [(src[i], dbufs[i]) for i in range(32)], copy))

        if mode == 2:
            direct["duplex_ms"] = _sync_time(torch, dduplex, reps=3) * 1e3
        else:
            t_d = _sync_time(torch, lambda: K.check(K.tc_offload_batch(d.ctx, [(src[i], dbufs[i]) for i in range(64)], copy)), reps=3)
            direct["offload_batch_GBps"] = nbytes / t_d / 1e9

            def direct_offload():
                K.check(K.tc_offload_batch(d.ctx, [(src[i], dbufs[i]) for i in range(64)], copy))

            iters = max(1, int(t_d / t_tri))
            overlapped(direct_offload, iters)
            t_dov, tri_d = overlapped(direct_offload, iters)
            direct["overlapped_offload_GBps"] = nbytes / t_dov / 1e9
            direct["hbm_stream_during_direct_offload_GBps"] = tri_bytes / tri_d / 1e9
        K.check(K.tc_sync(d.ctx))
        K.check(K.tc_destroy(d.ctx))
    emit(dict(measurement="config3", agents=64, blocks=total, GiB=nbytes / 2 ** 30,
              link_d2h_GBps=d2h, link_h2d_GBps=h2d,
              offload_batch_GBps=nbytes / t_off / 1e9, offload_64_single_calls_GBps=nbytes / t_off1 / 1e9,
              upload_batch_GBps=nbytes / t_up / 1e9,
              offload_pct_link=100 * nbytes / t_off / 1e9 / d2h, upload_pct_link=100 * nbytes / t_up / 1e9 / h2d,
              overlapped_offload_GBps=nbytes / t_off_ov / 1e9, overlapped_upload_GBps=nbytes / t_up_ov / 1e9,
              hbm_stream_alone_GBps=tri_bytes / t_tri / 1e9,
              hbm_stream_during_offload_GBps=tri_bytes / tri_off / 1e9,
              hbm_stream_during_upload_GBps=tri_bytes / tri_up / 1e9,
              upload_ms_per_1k_tokens=t_up * 1e3 / (total * shape.block_size / 1024),
              duplex_half_out_half_in_GBps=(half_bytes_out + half_bytes_in) / t_dup / 1e9,
              duplex_ms=t_dup * 1e3, half_out_alone_ms=t_out * 1e3, half_in_alone_ms=t_in * 1e3,
              duplex_direct_ms=direct["duplex_ms"],
              duplex_direct_GBps=(half_bytes_out + half_bytes_in) / (direct["duplex_ms"] * 1e-3) / 1e9,
              direct_offload_batch_GBps=direct["offload_batch_GBps"],
              direct_overlapped_offload_GBps=direct["overlapped_offload_GBps"],
              hbm_stream_during_direct_offload_GBps=direct["hbm_stream_during_direct_offload_GBps"]))
    del a, b, cc
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
        t_off = _sync_time(torch, lambda: K.check(K.tc_offload(c.ctx, ids, host, stream)))
        t_up = _sync_time(torch, lambda: K.check(K.tc_upload(c.ctx, host, new, table, stream)))
        K.check(K.tc_sync(c.ctx))
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


def m_config5(torch, K, W, emit):
    shape = W.CONFIGS[4]
    rng = W.rng_for(4, salt=53)
    tokens = W.uniform_contexts(rng, 12)
    private = (W.blocks_of(tokens, shape.block_size) - 32).astype(int)
    total = int(private.sum())
    c = Ctx(torch, K, W, shape, 4, total + 8, fill=False)
    perm = rng.permutation(shape.num_blocks).astype(np.int32)
    cuts = np.cumsum(private)[:-1]
    src = np.split(perm[:total], cuts)
    dst = np.split(perm[total:2 * total], cuts)
    for x in src + dst:
        K.check(K.tc_alloc_at(c.ctx, x))
    bufs = [K.tc_host_alloc(c.ctx, int(n))[1] for n in private]
    tables = torch.full((12, 1024), -1, dtype=torch.int32, device="cuda:0")
    stream = torch.cuda.Stream()
    nbytes = total * c.rec
    d2h, h2d = _link_peak(torch, nbytes)
    t_off = _sync_time(torch, lambda: K.check(K.tc_offload_batch(c.ctx, [(src[i], bufs[i]) for i in range(12)], stream)), reps=3)
    t_up = _sync_time(torch, lambda: K.check(K.tc_upload_batch(
        c.ctx, [(dst[i], bufs[i], tables[i].data_ptr() + 128) for i in range(12)], stream)), reps=3)
    K.check(K.tc_set_profiling(c.ctx, 1))
    K.check(K.tc_offload_batch(c.ctx, [(src[i], bufs[i]) for i in range(12)], stream))
    K.check(K.tc_upload_batch(c.ctx, [(dst[i], bufs[i], tables[i].data_ptr() + 128) for i in range(12)], stream))
    K.check(K.tc_sync(c.ctx))
    st = K.tc_stats(c.ctx)[1]
    emit(dict(measurement="config5", agents=12, private_blocks=total, GiB=nbytes / 2 ** 30, record_bytes=c.rec,
              link_d2h_GBps=d2h, link_h2d_GBps=h2d,
              offload_GBps=nbytes / t_off / 1e9, upload_GBps=nbytes / t_up / 1e9,
              offload_pct_link=100 * nbytes / t_off / 1e9 / d2h, upload_pct_link=100 * nbytes / t_up / 1e9 / h2d,
              upload_ms_per_1k_tokens=t_up * 1e3 / (total * shape.block_size / 1024),
              gather_TBps_overlapping_dma=2 * st.gather_bytes / (st.gather_ms * 1e-3) / 1e12,
              scatter_TBps_overlapping_dma=2 * st.scatter_bytes / (st.scatter_ms * 1e-3) / 1e12))
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


ALL = dict(sweep=m_sweep, naive=m_naive, config1=m_config1, config3=m_config3, config4=m_config4,
           config4_replay=m_config4_replay, forecast_noise=m_forecast_noise, config5=m_config5, lds=m_lds, host=m_host)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--only", default=",".join(ALL))
    ap.add_argument("--out", default=None)
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
        ALL[name](torch, K, W, emit)
    if args.out:
        with open(args.out, "w") as f:
            json.dump(results, f, indent=1)


if __name__ == "__main__":
    main()
