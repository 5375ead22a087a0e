"""Benchmark configurations 3, 4 and 5 at full size on the GPU, through the C ABI, with the library's default
options (paths chosen by the library).

Ids, counters and error codes are compared with the oracle's bookkeeping model call by call.
Data: EVERY agent is compared with the oracle byte for byte, streamed through a sparse host mirror of the pool
(harness.OracleStream): the records the library wrote against the oracle's offload of the same blocks, and the
destination blocks (pages and scale words) after the upload against the oracle's upload of the same records.
Blocks outside the destinations are checked through position-sensitive page checksums computed by torch.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_18586_amd as K
import tc_workloads as W
from harness import DEV, GpuPool, OracleStream, host_budget_bytes, host_view

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[configs] {msg}", flush=True)


CODE = {"INVAL": -1, "RANGE": -2, "DUP": -3, "SHARED": -4, "NOMEM": -5, "HOST_NOMEM": -6}


class LockStep:
    """Runs every bookkeeping call on the library and on the model and insists they agree."""

    def __init__(self, gp):
        self.gp, self.ctx = gp, gp.ctx
        self.model = oracle.OracleBlockPool(gp.NB)

    def alloc(self, n):
        rc, ids = K.tc_alloc(self.ctx, n)
        try:
            want = self.model.alloc(n)
        except oracle.OracleError as e:
            assert rc == CODE[e.code]
            return None
        assert rc == 0 and ids.tolist() == want
        return ids

    def free(self, ids):
        assert K.tc_free(self.ctx, ids) == 0
        self.model.free(list(ids))

    def ref(self, ids):
        assert K.tc_ref(self.ctx, ids) == 0
        self.model.ref(list(ids))

    def n_free(self):
        return self.model.n_free()

    def begin(self, ids):
        self.model.begin_op(list(ids))

    def sync(self):
        K.check(K.tc_sync(self.ctx))
        self.model.retire_all()

    def check_counters(self):
        rc, st = K.tc_stats(self.ctx)
        assert rc == 0
        m = self.model
        assert (st.gpu_blocks_free, st.gpu_blocks_used, st.gpu_blocks_pending_free, st.gpu_blocks_shared) == \
               (m.n_free(), m.n_used(), m.n_pending(), m.n_shared())
        return st


# ------------------------------------------------------------------------------------ config 3
def test_config3_64_agents_fragmented_pool_overlapped_with_hbm_stream():
    """8B-shaped pool (32 GiB), 64 agents with lognormal contexts (median 2 048, sigma 0.8, cap 16 384
    tokens), pool fragmented by 50 000 seeded alloc/free ops, all agents offloaded concurrently while
    an HBM-streaming kernel runs on another stream; then uploaded into newly allocated blocks."""
    shape = W.CONFIGS[2]
    rng = W.rng_for(2)
    tokens = W.lognormal_contexts(rng, 64)
    nblk = W.blocks_of(tokens, shape.block_size).astype(int)
    total = int(nblk.sum())
    rec = 2 * shape.num_layers * shape.page_bytes
    gp = GpuPool(shape, seed=W.seed_for(2), host_arena_bytes=(total + 8) * rec)
    chk = None
    try:
        ls = LockStep(gp)
        say(f"config 3: pool ready, {total} blocks to move; fragmenting")
        W.fragment_pool(ls, rng, n_ops=50000, need_free=total)
        ls.check_counters()
        agents = [ls.alloc(int(n)) for n in nblk]
        assert all(a is not None for a in agents)
        spread = np.diff(np.sort(agents[int(np.argmax(nblk))]))
        assert (spread > 1).any(), "fragmentation should scatter an agent's blocks"
        bufs = [K.tc_host_alloc(gp.ctx, int(n)) for n in nblk]
        assert all(rc == 0 for rc, _ in bufs)
        bufs = [addr for _, addr in bufs]

        before = gp.page_checksums(weighted=True)
        chk = OracleStream(gp)
        for i in range(64):
            chk.snapshot(agents[i])
        chk.wait()

        # the neighbour on the compute stream: fp32 triad over 3 x 1 GiB, s = 0.5 keeps it exact
        m = 1 << 28
        b = torch.rand(m, device=DEV)
        c = torch.rand(m, device=DEV)
        a = torch.zeros(m, device=DEV)
        torch.cuda.synchronize()       # torch wrote this on its own stream; the library's calls run on others
        compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        K.check(K.tc_hbm_stream(a, b, c, m, 0.5, 40, compute))
        for i in range(32):                      # back-to-back single calls ...
            K.check(K.tc_offload(gp.ctx, agents[i], bufs[i], copy))
            ls.begin(agents[i])
        K.check(K.tc_offload_batch(gp.ctx, [(agents[i], bufs[i]) for i in range(32, 64)], copy))   # ... and one batch
        ls.begin(np.concatenate(agents[32:]))
        for i in range(64):
            ls.free(agents[i])
        st = ls.check_counters()
        assert st.gpu_blocks_pending_free == total
        ls.sync()
        torch.cuda.synchronize()
        say("config 3: offloads done; checking records")
        assert torch.equal(a, b + 0.5 * c), "the neighbour kernel's result was disturbed"
        assert torch.equal(gp.page_checksums(weighted=True), before), "offload wrote the pool"
        del a, b, c

        # every record of every agent against the oracle, byte for byte
        for i in range(64):
            chk.check_records(agents[i], host_view(bufs[i], int(nblk[i]) * rec), f"agent {i}")
        chk.wait()

        # upload everything into newly allocated blocks, one table row per agent
        say("config 3: uploading")
        new = [ls.alloc(int(n)) for n in nblk]
        tables = torch.full((64, int(nblk.max()) + 1), -1, dtype=torch.int32, device=DEV)
        torch.cuda.synchronize()       # torch wrote this on its own stream; the library's calls run on others
        K.check(K.tc_upload_batch(gp.ctx, [(new[i], bufs[i], tables[i]) for i in range(64)], copy))
        ls.begin(np.concatenate(new))
        ls.sync()
        say("config 3: uploads done; checking every destination block")
        after = gp.page_checksums(weighted=True)
        touched = torch.zeros(gp.NB, dtype=torch.bool, device=DEV)
        rows = tables.cpu().numpy()
        want_rows = [chk.check_upload(host_view(bufs[i], int(nblk[i]) * rec), new[i], f"agent {i}") for i in range(64)]
        chk.wait()
        for i in range(64):
            assert np.array_equal(rows[i, : nblk[i]], want_rows[i]) and (rows[i, nblk[i]:] == -1).all()
            touched[torch.as_tensor(new[i].astype(np.int64), device=DEV)] = True
        assert torch.equal(after[:, ~touched], before[:, ~touched]), "a block outside the destinations changed"
        for i in range(64):
            K.check(K.tc_host_free(gp.ctx, bufs[i]))
        assert chk.bytes_compared == 2 * total * rec
        rc, st = K.tc_stats(gp.ctx)
        assert st.host_slots_used == 0 and st.blocks_offloaded == total and st.blocks_uploaded == total
    finally:
        if chk:
            chk.close()
        gp.close()


# ------------------------------------------------------------------------------------ config 4
def test_config4_trace_replay_200_agents():
    """32B-shaped pool (64 layers, 4 MiB per block, 64 GiB): replay of a seeded trace of 200 agents in
    a random DAG of depth 6; every call offloads, the upload is issued 200 ms (virtual) before the
    predicted finish or at the finish when the tool returns early; a 16 GiB arena forces some
    'CPU capacity insufficient' rejections."""
    shape = W.CONFIGS[3]
    rng = W.rng_for(3)
    agents, events = W.dag_trace(rng, block_size=shape.block_size)
    rec = 2 * shape.num_layers * shape.page_bytes
    gp = GpuPool(shape, seed=W.seed_for(3), host_arena_bytes=4096 * rec)
    chk = None
    try:
        ls = LockStep(gp)
        arena = oracle.OracleHostArena(4096)
        stream = torch.cuda.Stream()
        tables = torch.full((len(agents), 1024 + 1), -1, dtype=torch.int32, device=DEV)
        torch.cuda.synchronize()       # torch wrote this on its own stream; the library's calls run on others
        chk = OracleStream(gp)
        st8 = [dict(state="new") for _ in agents]
        counts = dict(offloads=0, rejected=0, predictive=0, immediate=0)

        def upload(i):
            s = st8[i]
            ls.sync()                                   # retire: deterministic free list on both sides
            new = ls.alloc(agents[i]["blocks"])
            if new is None:
                return False
            # the offload has completed (ls.sync above): its records against the oracle's, byte for byte
            chk.compare(s["want"], host_view(s["buf"], len(new) * rec), f"agent {i}")
            chk.wait()
            K.check(K.tc_upload(gp.ctx, s["buf"], new, tables[i], stream))
            ls.begin(new)
            K.check(K.tc_host_free(gp.ctx, s["buf"]))   # recycled when the upload retires
            arena.begin_op(s["slot"])
            arena.free(s["slot"])
            arena.end_op(s["slot"])                     # the model has no clock: released at once
            s.update(state="uploaded", ids=new)
            return True

        say("config 4: pool ready; replaying 1000 events")
        for e_no, (t, _, kind, i) in enumerate(events):
            if e_no % 100 == 0:
                say(f"config 4: event {e_no}, virtual t = {t:.2f} s, {counts}")
            s, n = st8[i], agents[i]["blocks"]
            if kind == "start":
                ids = ls.alloc(n)
                assert ids is not None, "the pool is sized for the trace's peak"
                tables[i, :n] = torch.from_numpy(ids).to(DEV)
                torch.cuda.synchronize()       # torch wrote this on its own stream; the library's calls run on others
                s.update(state="running", ids=ids)
            elif kind == "call_start":
                ls.sync()                               # finished uploads hand their arena slots back
                rc, buf = K.tc_host_alloc(gp.ctx, n)
                try:
                    slot = arena.alloc(n)
                except oracle.OracleError:
                    assert rc == K.TC_ERR_HOST_NOMEM
                    counts["rejected"] += 1
                    s["state"] = "kept"                 # CPU capacity insufficient: the KV stays on the GPU
                    continue
                assert rc == 0 and buf == K.tc_arena_base(gp.ctx) + slot * rec
                s.update(buf=buf, slot=slot, src=s["ids"])
                # what the oracle makes of these blocks, now: once released they may belong to somebody else
                chk.snapshot(s["ids"])
                chk.wait()
                s["want"] = chk.expected_records(s["ids"])
                chk.drop()                              # nothing else lives in the mirror between two checks
                K.check(K.tc_offload(gp.ctx, s["ids"], buf, stream))
                ls.begin(s["ids"])
                ls.free(s["ids"])
                s["state"] = "offloaded"
                counts["offloads"] += 1
            elif kind == "upload_due":
                if s["state"] == "offloaded" and upload(i):
                    counts["predictive" if not agents[i]["early"] else "immediate"] += 1
            elif kind == "call_finish":
                if s["state"] == "offloaded":           # the tool returned before the upload could be issued
                    assert upload(i), "an immediate upload must find blocks"
                    counts["immediate"] += 1
                if s["state"] == "uploaded":
                    stream.synchronize()
                    row = tables[i].cpu().numpy()
                    want_row = chk.check_upload(s.pop("want"), s["ids"], f"agent {i}")
                    chk.wait()
                    assert np.array_equal(row[:n], want_row) and (row[n:] == -1).all()
                    chk.drop()
                    s["state"] = "running"
            elif kind == "finish":
                assert s["state"] in ("running", "kept")
                ls.free(s["ids"])
                s["state"] = "done"
        ls.sync()
        st = ls.check_counters()
        assert st.gpu_blocks_free == gp.NB and st.host_slots_used == 0 and arena.used_slots() == 0
        assert counts["offloads"] + counts["rejected"] == len(agents)
        assert counts["predictive"] + counts["immediate"] == counts["offloads"]
        assert counts["rejected"] > 0 and counts["predictive"] > 0 and counts["immediate"] > 0
        assert st.n_offloads == counts["offloads"] == st.n_uploads
        moved = sum(agents[i]["blocks"] for i in range(len(agents)) if st8[i].get("src") is not None)
        assert chk.bytes_compared == 2 * moved * rec
    finally:
        if chk:
            chk.close()
        gp.close()


# ------------------------------------------------------------------------------------ config 5
def test_config5_fp8_shared_prefix_waves():
    """70B-shaped fp8 pool (80 layers, 32-token blocks, one fp32 scale per page; 32 768 blocks, 160 GiB):
    128 agents share 32 refcounted prefix blocks that must not move; only private suffix blocks travel;
    contexts uniform 1k..32k tokens; agents run in waves that fit the pool and a 32 GiB arena."""
    shape = W.CONFIGS[4]
    rng = W.rng_for(4)
    rec = oracle.record_bytes(shape.num_layers, shape.page_bytes, shape.scales_per_block)
    arena_slots = host_budget_bytes(16 << 30, share=0.1) // rec        # waves shrink with the host memory at hand
    gp = GpuPool(shape, seed=W.seed_for(4), host_arena_bytes=arena_slots * rec)
    chk = None
    try:
        assert gp.rec == rec == 5 * 1024 * 1024 + 768
        ls = LockStep(gp)
        W.fragment_pool(ls, rng, n_ops=3000, median_blocks=256, need_free=gp.NB)   # scrambles the free list
        ls.check_counters()
        n_agents, n_prefix = 128, 1024 // shape.block_size
        prefix = ls.alloc(n_prefix)
        for _ in range(n_agents - 1):
            ls.ref(prefix)
        assert ls.check_counters().gpu_blocks_shared == n_prefix
        tokens = W.uniform_contexts(rng, n_agents)
        private = (W.blocks_of(tokens, shape.block_size) - n_prefix).astype(int)
        assert private.min() >= 0 and private.max() <= 992
        prefix_sig = gp.block_checksums(prefix)
        stream = torch.cuda.Stream()
        tables = torch.full((n_agents, 1024), -1, dtype=torch.int32, device=DEV)
        tables[:, :n_prefix] = torch.from_numpy(prefix).to(DEV)
        torch.cuda.synchronize()       # torch wrote this on its own stream; the library's calls run on others
        chk = OracleStream(gp)
        i = 0
        n_waves = 0
        while i < n_agents:
            wave, used = [], 0
            while i < n_agents and used + private[i] <= min(arena_slots, ls.n_free()):
                wave.append(i)
                used += int(private[i])
                i += 1
            assert wave, "an agent does not fit an empty pool / arena"
            n_waves += 1
            say(f"config 5: wave {n_waves}: agents {wave[0]}..{wave[-1]}, {used} private blocks")
            ids = {a: ls.alloc(int(private[a])) for a in wave}
            bufs = {}
            for a in wave:
                rc, bufs[a] = K.tc_host_alloc(gp.ctx, int(private[a]))
                assert rc == 0
                tables[a, n_prefix:n_prefix + private[a]] = torch.from_numpy(ids[a]).to(DEV)
                torch.cuda.synchronize()       # torch wrote this on its own stream; the library's calls run on others
            # the whole row must be refused, the private part is what moves
            a0 = max(wave, key=lambda a: private[a])
            row = np.concatenate([prefix, ids[a0]])
            assert K.tc_offload(gp.ctx, row, bufs[a0], stream) == K.TC_ERR_SHARED
            assert K.tc_offload(gp.ctx, prefix[:1], bufs[a0], stream) == K.TC_ERR_SHARED
            rc, priv = K.tc_filter_private(gp.ctx, row)
            assert rc == 0 and np.array_equal(priv, ids[a0])
            for a in wave:
                chk.snapshot(ids[a])
            chk.wait()
            K.check(K.tc_offload_batch(gp.ctx, [(ids[a], bufs[a]) for a in wave], stream))
            ls.begin(np.concatenate([ids[a] for a in wave]))
            for a in wave:
                ls.free(ids[a])
            ls.sync()
            for a in wave:
                chk.check_records(ids[a], host_view(bufs[a], int(private[a]) * rec), f"agent {a}")
            chk.wait()
            new = {a: ls.alloc(int(private[a])) for a in wave}
            K.check(K.tc_upload_batch(
                gp.ctx, [(new[a], bufs[a], tables[a].data_ptr() + 4 * n_prefix) for a in wave], stream))
            ls.begin(np.concatenate([new[a] for a in wave]))
            ls.sync()
            rows = tables[wave[0]: wave[-1] + 1].cpu().numpy()
            want_rows = {a: chk.check_upload(host_view(bufs[a], int(private[a]) * rec), new[a], f"agent {a}") for a in wave}
            chk.wait()
            for k, a in enumerate(wave):
                assert np.array_equal(rows[k, :n_prefix], prefix), "prefix entries were written"
                assert np.array_equal(rows[k, n_prefix:n_prefix + private[a]], want_rows[a])
                assert (rows[k, n_prefix + private[a]:] == -1).all()
                K.check(K.tc_host_free(gp.ctx, bufs[a]))
            chk.drop()
            assert torch.equal(gp.block_checksums(prefix), prefix_sig), "shared prefix blocks changed"
            for a in wave:
                ls.free(new[a])
            ls.check_counters()
        assert n_waves > 1
        rc, st = K.tc_stats(gp.ctx)
        assert st.blocks_offloaded == st.blocks_uploaded == int(private.sum()) and st.host_slots_used == 0
        assert chk.bytes_compared == 2 * int(private.sum()) * rec
    finally:
        if chk:
            chk.close()
        gp.close()
