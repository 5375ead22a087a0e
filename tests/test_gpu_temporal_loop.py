"""The pieces around the copy path working together on the GPU: forecast (Eq. 1) -> hard rejections
incl. ShouldOffload (Sec. 4.2, Alg. 1, with a cost model calibrated on this device, Eq. 2) -> offload -> one
scheduling step of predictive upload at a time (Sec. 4.3: all candidates ranked by P_upload = I + U, the step's
budget from Eq. 3 with critical demand and a shared pool, Eq. 4 in rank order) with piecewise uploads ->
lifecycle (Sec. 6.2) deciding resume / immediate upload.

Every decision the library takes is compared with the oracle's on the spot; every agent that went
through a round trip must find its KV unchanged behind its rewritten block table.
"""
import heapq

import numpy as np
import pytest
import torch

import oracle
import paper_2510_18586_amd as K
import tc_workloads as W
from oracle import lifecycle as L
from oracle import policy
from harness import DEV, GpuPool

pytestmark = pytest.mark.gpu


def test_temporal_loop_on_a_seeded_trace():
    shape = W.CONFIGS[3].with_blocks(3072)                      # 32B-shaped records (4 MiB), 12 GiB pool
    rng = W.rng_for(3, salt=21)
    agents, events = W.dag_trace(rng, n_agents=60, depth=4, median_tokens=1024, cap_tokens=4096,
                                 block_size=shape.block_size)
    rec = 2 * shape.num_layers * shape.page_bytes
    gp = GpuPool(shape, seed=W.seed_for(3, 21), host_arena_bytes=1024 * rec)
    try:
        stream = torch.cuda.Stream()
        rc, model = K.tc_calibrate(gp.ctx, [16, 64, 128], 2, stream)
        assert rc == 0
        m = model.as_tuple()
        rc, fc = K.tc_forecaster_create(0.5, 0.5, 2000.0)
        assert rc == 0
        fc_model = L.Forecaster(0.5, 0.5, 2000.0)
        pool_model = oracle.OracleBlockPool(gp.NB)
        pool_model.free(pool_model.alloc(128))     # the calibration claimed and released its largest size
        lead_ms, step_ms, v_tok_per_ms = 200.0, 50.0, 4.0
        tables = torch.full((len(agents), 260), -1, dtype=torch.int32, device=DEV)
        torch.cuda.synchronize()       # torch wrote this on its own stream; the library's calls run on others
        A = [dict(req=K.tc_req_state(0, 0, 0, 0), model=(L.RUNNING, False, False)) for _ in agents]
        counts = dict(approved=0, rejected=0, resumed_at_once=0, immediate=0, pieces=0, steps=0, steps_with_several=0,
                      steps_budget_binds=0, steps_rank_differs_from_listing=0)
        rng_step = W.rng_for(3, salt=22)                             # draws of the scheduling steps only
        importance = rng_step.uniform(0.0, 1.0, size=len(agents))   # I: what the spatial scheduler would say
        step_pending = [False]

        heap = [(t * 1e3, k, kind, i) for k, (t, _, kind, i) in enumerate(events) if kind != "upload_due"]
        heapq.heapify(heap)
        seq = len(heap) + len(events)

        def push(t, kind, i):
            nonlocal seq
            seq += 1
            heapq.heappush(heap, (t, seq, kind, i))

        def lifecycle(i, event):
            a = A[i]
            rc, act = K.tc_lifecycle_step(a["req"], event)
            a["model"], want = L.step(a["model"], event)
            assert rc == 0 and act == want and a["req"].as_tuple() == a["model"]
            return act

        def alloc(n):
            rc, ids = K.tc_alloc(gp.ctx, n)
            assert rc == 0 and ids.tolist() == pool_model.alloc(n)
            return ids

        def sync():
            K.check(K.tc_sync(gp.ctx))
            pool_model.retire_all()

        def issue_piece(i, t, piece):
            """`piece` more blocks of agent i come back: a contiguous run of its records."""
            a = A[i]
            if a["req"].state == L.OFFLOADED:
                assert lifecycle(i, L.UPLOAD_ISSUED) == L.NONE
            n, done = agents[i]["blocks"], a["done"]
            ids = alloc(piece)
            K.check(K.tc_upload(gp.ctx, a["buf"] + done * rec, ids, tables[i].data_ptr() + 4 * done, stream))
            pool_model.begin_op(ids.tolist())
            a["new"][done:done + piece] = ids
            a["done"] = done + piece
            counts["pieces"] += 1
            if a["done"] == n:
                a["due"] = False
                K.check(K.tc_host_free(gp.ctx, a["buf"]))
                push(t + 0.001, "upload_done", i)

        def upload_rest(i, t):
            """The tool is back: no more waiting, everything that is still missing comes at once."""
            sync()
            issue_piece(i, t, agents[i]["blocks"] - A[i]["done"])

        def scheduling_step(t):
            """Sec. 4.3: every candidate whose upload is due, ranked and served within this step's budget."""
            sync()
            cand_ids = [j for j, b in enumerate(A) if b.get("due") and not b["req"].finish_seen
                        and b["req"].state in (L.OFFLOADED, L.PENDING_UPLOAD) and b["done"] < agents[j]["blocks"]]
            if not cand_ids:
                return False
            # urgency: how close the predicted end of the call is, 0 (far) .. 1 (now or past)
            cands = []
            for j in cand_ids:
                b = A[j]
                urgency = min(1.0, max(0.0, 1.0 - (b["t_call"] + b["t_fc"] - t) / max(b["t_fc"], 1.0)))
                cands.append((float(importance[j]), urgency, agents[j]["blocks"] - b["done"]))
            # critical demand: none, nearly everything that is free (Eq. 3 leaves a small budget), or anything
            gpu_free, shared_free = pool_model.n_free(), int(rng_step.integers(0, 400))
            kind_of_step = int(rng_step.integers(0, 3))
            if kind_of_step == 0:
                d_critical = 0
            elif kind_of_step == 1:
                d_critical = max(0, gpu_free + shared_free - int(rng_step.integers(0, 64)))
            else:
                d_critical = int(rng_step.integers(0, gpu_free + shared_free + 1))
            rc, order, reserve = K.tc_upload_plan(cands, gpu_free, d_critical, shared_free)
            want_order, want_reserve = policy.upload_plan(cands, gpu_free, d_critical, shared_free)
            assert rc == 0 and order == want_order and reserve == want_reserve
            budget = K.tc_upload_budget(gpu_free, d_critical, shared_free)
            assert budget == policy.upload_budget(gpu_free, d_critical, shared_free) and sum(reserve) <= budget
            counts["steps"] += 1
            counts["steps_with_several"] += len(cands) > 1
            counts["steps_budget_binds"] += sum(reserve) < sum(-(-c[2] // 2) for c in cands)
            counts["steps_rank_differs_from_listing"] += order != sorted(order)
            for k in order:
                if reserve[k]:
                    issue_piece(cand_ids[k], t, reserve[k])
            return True

        def verify_and_resume(i):
            a, n = A[i], agents[i]["blocks"]
            stream.synchronize()
            assert np.array_equal(tables[i].cpu().numpy()[:n], a["ids"])
            assert torch.equal(gp.block_checksums(a["ids"]), a["sig"]), f"agent {i}: KV changed"

        while heap:
            t, _, kind, i = heapq.heappop(heap)
            a, n = (A[i], agents[i]["blocks"]) if i >= 0 else (None, 0)
            ftype = i % 4
            user = 2000.0 if ftype < 2 else None
            if kind == "start":
                a["ids"] = alloc(n)
                tables[i, :n] = torch.from_numpy(a["ids"]).to(DEV)
                torch.cuda.synchronize()       # torch wrote this on its own stream; the library's calls run on others
            elif kind == "call_start":
                a["t_call"] = t
                assert lifecycle(i, L.CALL_START) == L.NONE
                t_fc = K.tc_forecaster_estimate(fc, ftype, user)
                assert t_fc == pytest.approx(fc_model.estimate(ftype, user), rel=1e-12)
                queue = [(int(rng.integers(8, 400)), float(rng.uniform(100, 6000))) for _ in range(3)]
                st = K.tc_stats(gp.ctx)[1]
                cpu_free = int(st.host_slots_total - st.host_slots_used)
                gate = (n, cpu_free, pool_model.n_used(), gp.NB, 0.02, t_fc, v_tok_per_ms, queue)
                ok, reason, pick = K.tc_offload_gate(model, *gate)
                assert (reason, pick) == policy.offload_gate(m, *gate) and ok == int(reason == policy.PASS)
                counts["reason_%d" % reason] = counts.get("reason_%d" % reason, 0) + 1
                rc, buf = K.tc_host_alloc(gp.ctx, n) if ok else (K.TC_ERR_HOST_NOMEM, None)
                if not ok or rc != 0:
                    counts["rejected"] += 1
                    continue
                counts["approved"] += 1
                a.update(sig=gp.block_checksums(a["ids"]), buf=buf, done=0, new=np.full(n, -1, dtype=np.int32), t_fc=t_fc,
                         due=False)
                K.check(K.tc_offload(gp.ctx, a["ids"], buf, stream))
                pool_model.begin_op(a["ids"].tolist())
                K.check(K.tc_free(gp.ctx, a["ids"]))
                pool_model.free(a["ids"].tolist())
                assert lifecycle(i, L.OFFLOAD_ISSUED) == L.NONE
                push(t + K.tc_estimate_transfer_ms(model, n) / 2, "offload_done", i)
                push(t + max(0.0, t_fc - lead_ms), "upload_due", i)
            elif kind == "offload_done":
                sync()
                if lifecycle(i, L.OFFLOAD_DONE) == L.UPLOAD_NOW:
                    counts["immediate"] += 1
                    upload_rest(i, t)
            elif kind == "upload_due":
                if a["req"].state in (L.OFFLOADED, L.PENDING_OFFLOAD) and not a["req"].finish_seen:
                    a["due"] = True                       # a candidate from now on (once its offload is through)
                    if not step_pending[0]:
                        step_pending[0] = True
                        push(t, "step", -1)
            elif kind == "step":
                step_pending[0] = False
                scheduling_step(t)
                if any(b.get("due") for b in A):
                    step_pending[0] = True
                    push(t + step_ms, "step", -1)
            elif kind == "upload_done":
                sync()
                a["ids"] = a["new"].copy()
                if lifecycle(i, L.UPLOAD_DONE) == L.RESUME:
                    verify_and_resume(i)
            elif kind == "call_finish":
                elapsed = t - a["t_call"]
                assert K.tc_forecaster_observe(fc, ftype, elapsed) == 0
                fc_model.observe(ftype, elapsed)
                act = lifecycle(i, L.CALL_FINISH)
                if act == L.RESUME:
                    if "sig" in a:
                        counts["resumed_at_once"] += 1
                        verify_and_resume(i)
                elif act == L.UPLOAD_NOW:
                    counts["immediate"] += 1
                    a["due"] = False
                    upload_rest(i, t)
                elif a["req"].state == L.PENDING_UPLOAD and a.get("done", 0) < n:
                    a["due"] = False                      # pieces are in flight and the tool is back: the rest, now
                    upload_rest(i, t)
                # WAIT: a copy is in flight; its completion event takes it from here
            elif kind == "finish":
                if a["req"].state != L.RUNNING:            # still coming back: finish once it has resumed
                    push(t + step_ms, "finish", i)
                    continue
                K.check(K.tc_free(gp.ctx, a["ids"]))
                pool_model.free(a["ids"].tolist())
        sync()
        rc, st = K.tc_stats(gp.ctx)
        assert st.gpu_blocks_free == gp.NB and st.host_slots_used == 0
        assert counts["approved"] > 5 and counts["rejected"] > 0, counts
        assert counts["resumed_at_once"] > 0 and counts["immediate"] > 0, counts
        assert counts["pieces"] > counts["approved"], counts       # uploads really came in pieces
        # Eq. 3 with a binding critical demand, and rankings over several candidates that differ from the order
        # they were listed in, both occurred
        assert counts["steps_with_several"] > 3 and counts["steps_budget_binds"] > 3, counts
        assert counts["steps_rank_differs_from_listing"] > 0, counts
        K.tc_forecaster_destroy(fc)
    finally:
        gp.close()
