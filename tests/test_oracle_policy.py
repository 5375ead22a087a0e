"""Pins for the oracle's scheduling arithmetic (no GPU): the paper's printed transfer times,
numpy's polyfit, hand-worked decisions, and properties that follow from the statements."""
import os

import numpy as np
import pytest

from oracle import policy

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "block_size_anchors.txt")


def _round_trips():
    pts = []
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("round_trip_ms "):
                _, n, t = line.split()
                pts.append((int(n), float(t)))
    return pts


def test_linear_cost_reproduces_the_papers_round_trips():
    pts = dict(_round_trips())
    # a line through the two ends of the printed range predicts the printed middle point
    a, b = policy.fit_linear([64, 320], [pts[64], pts[320]])
    assert abs(b - 0.25) < 1e-12                     # 0.25 ms per block, both directions together
    assert abs((a + b * 256) - pts[256]) <= 0.15     # 63.8 predicted, 63.7 printed
    # offload 32.0 + upload 31.7 = the printed round trip; recompute 1815 ms is 28.5 times it
    model = (0.0, 32.0 / 256, 0.0, 31.7 / 256)
    assert abs(policy.estimate_transfer_ms(model, 256) - pts[256]) < 1e-9
    assert round(1815 / policy.estimate_transfer_ms(model, 256), 1) == 28.5


def test_fit_is_numpy_polyfit():
    rng = np.random.default_rng(3)
    for _ in range(20):
        n = np.sort(rng.choice(np.arange(1, 2000), size=int(rng.integers(2, 9)), replace=False))
        t = 0.3 + 0.037 * n + rng.normal(0, 0.05, size=n.size)
        a, b = policy.fit_linear(list(n), list(t))
        b_np, a_np = np.polyfit(n.astype(float), t, 1)
        assert abs(a - a_np) < 1e-8 and abs(b - b_np) < 1e-10
    with pytest.raises(ValueError):
        policy.fit_linear([5, 5], [1.0, 2.0])


def test_should_offload_hand_worked():
    model = (0.1, 0.04, 0.1, 0.04)                   # 256 blocks -> 20.68 ms round trip
    t_tr = policy.estimate_transfer_ms(model, 256)
    assert abs(t_tr - 20.68) < 1e-12
    queue = [(300, 10), (200, 5000), (100, 900), (50, 100)]
    assert policy.should_offload(model, 256, t_tr, 1.0, [(1, 0.0)]) == (False, -1)  # stall == transfer: "<=" rejects
    assert policy.should_offload(model, 256, float(np.nextafter(t_tr, np.inf)), 1.0, [(1, 0.0)]) == (True, 0)
    assert policy.should_offload(model, 256, 20.0, 1.0, queue) == (False, -1)       # stall too short
    # window 100 ms at 10 tokens/ms = 1 000 tokens: #0 needs too many blocks, #1 too much work, #2 fits
    assert policy.should_offload(model, 256, 120.68, 10.0, queue) == (True, 2)
    # a longer window admits the earlier request: first fit, not best fit
    assert policy.should_offload(model, 256, 620.68, 10.0, queue) == (True, 1)
    assert policy.should_offload(model, 40, 1e6, 10.0, queue) == (False, -1)        # nobody fits 40 freed blocks
    assert policy.should_offload(model, 256, 1e6, 10.0, []) == (False, -1)


def test_should_offload_properties():
    rng = np.random.default_rng(11)
    model = (0.05, 0.0374, 0.07, 0.0374)
    for _ in range(300):
        blocks = int(rng.integers(1, 1025))
        queue = [(int(rng.integers(1, 1200)), float(rng.uniform(1, 50000))) for _ in range(int(rng.integers(0, 8)))]
        v = float(rng.uniform(0.5, 40))
        t_tr = policy.estimate_transfer_ms(model, blocks)
        last = False
        for t_fc in np.linspace(0, 5000, 26):
            ok, k = policy.should_offload(model, blocks, float(t_fc), v, queue)
            if t_fc <= t_tr:
                assert not ok
            if ok:
                cap = (t_fc - t_tr) * v
                assert queue[k][0] <= blocks and queue[k][1] <= cap
                assert all(not (q[0] <= blocks and q[1] <= cap) for q in queue[:k])
            assert ok or not last, "a longer stall can only help"
            last = ok


def test_upload_budget_and_gradual_reserve():
    assert policy.upload_budget(100, 30, 50) == 100          # critical demand covered by the shared pool
    assert policy.upload_budget(100, 80, 50) == 70
    assert policy.upload_budget(20, 80, 50) == 0             # never negative
    assert policy.gradual_reserve(100, 13, 100) == 7         # half of the deficit, rounded up
    assert policy.gradual_reserve(5, 13, 100) == 5
    assert policy.gradual_reserve(100, 13, 3) == 3
    assert policy.gradual_reserve(100, 0, 100) == 0
    # with an ample budget the deficit is gone after ceil(log2(d + 1)) steps
    for d in range(1, 300):
        left, steps = d, 0
        while left:
            r = policy.gradual_reserve(10**9, left, 10**9)
            assert 1 <= r <= left
            left -= r
            steps += 1
        assert steps == int(np.ceil(np.log2(d + 1)))


# ---- hard rejections (Sec. 4.2) and one step of predictive upload (Sec. 4.3) --------------------------

def test_offload_gate_hand_worked():
    m = (0.0, 0.1, 0.0, 0.1)                  # 0.2 ms per block both ways: 100 blocks cost 20 ms
    q = [(150, 10.0), (80, 50.0)]             # the first never fits 100 freed blocks
    args = dict(req_blocks=100, cpu_free_blocks=100, gpu_used_blocks=90, gpu_total_blocks=100,
                pressure_threshold=0.8, t_fc_ms=50.0, v_throughput_tokens_per_ms=2.0, waiting=q)
    assert policy.offload_gate(m, **args) == (policy.PASS, 1)          # window 30 ms -> 60 tokens >= 50
    assert policy.offload_gate(m, **{**args, "cpu_free_blocks": 99}) == (policy.CPU_FULL, -1)
    assert policy.offload_gate(m, **{**args, "t_fc_ms": 20.0}) == (policy.STALL_SHORT, -1)
    assert policy.offload_gate(m, **{**args, "t_fc_ms": 44.0}) == (policy.NO_FIT, -1)     # 48 tokens < 50
    assert policy.offload_gate(m, **{**args, "gpu_used_blocks": 79}) == (policy.LOW_PRESSURE, -1)
    assert policy.offload_gate(m, **{**args, "gpu_used_blocks": 80}) == (policy.PASS, 1)  # "below" is strict
    # several reasons at once: the first in the paper's order is reported
    assert policy.offload_gate(m, **{**args, "cpu_free_blocks": 0, "t_fc_ms": 1.0, "gpu_used_blocks": 0})[0] == policy.CPU_FULL
    assert policy.offload_gate(m, **{**args, "t_fc_ms": 1.0, "gpu_used_blocks": 0})[0] == policy.STALL_SHORT
    assert policy.offload_gate(m, **{**args, "waiting": [], "gpu_used_blocks": 0})[0] == policy.NO_FIT


def test_offload_gate_is_alg1_plus_two_independent_conditions():
    rng = np.random.default_rng(8)
    for _ in range(2000):
        m = tuple(float(x) for x in rng.uniform(0, 0.2, size=4))
        q = [(int(rng.integers(1, 200)), float(rng.uniform(0, 400))) for _ in range(int(rng.integers(0, 5)))]
        req, cpu = int(rng.integers(1, 200)), int(rng.integers(0, 250))
        used, thr = int(rng.integers(0, 101)), float(rng.choice([0.0, 0.5, 0.8, 1.0]))
        t_fc, v = float(rng.uniform(0, 120)), float(rng.uniform(0.5, 4))
        reason, k = policy.offload_gate(m, req, cpu, used, 100, thr, t_fc, v, q)
        alg1 = policy.should_offload(m, req, t_fc, v, q)
        passes = cpu >= req and alg1[0] and used >= thr * 100
        assert (reason == policy.PASS) == passes
        assert k == (alg1[1] if passes else -1)
        if reason in (policy.STALL_SHORT, policy.NO_FIT):
            assert not alg1[0] and cpu >= req


def test_upload_plan_hand_worked():
    # budget: 40 free, critical demand 30 of which 10 fit the shared pool -> 40 - 20 = 20 blocks
    cands = [(0.2, 0.1, 16),      # P = 0.3                    rank 2
             (0.9, 0.5, 10),      # P = 1.4                    rank 0
             (0.1, 0.9, 31)]      # P = 1.0                    rank 1
    order, reserve = policy.upload_plan(cands, 40, 30, 10)
    assert order == [1, 2, 0]
    # rank 0: min(20, ceil(10/2)=5, 20) = 5; rank 1: min(15, 16, 20) = 15; rank 2: min(0, 8, 20) = 0
    assert reserve == [0, 5, 15]
    # equal P: the more urgent first, then the one named first
    assert policy.upload_plan([(0.5, 0.5, 4), (0.2, 0.8, 4), (0.5, 0.5, 4)], 100, 0, 0)[0] == [1, 0, 2]
    assert policy.upload_plan([], 10, 0, 0) == ([], [])
    assert policy.upload_plan([(1.0, 1.0, 9)], 3, 50, 0) == ([0], [0])     # critical demand eats the budget


def test_upload_plan_properties():
    rng = np.random.default_rng(4)
    for _ in range(1000):
        n = int(rng.integers(0, 8))
        cands = [(float(rng.choice([0.0, 0.25, 0.5, 1.0])), float(rng.choice([0.0, 0.25, 0.5, 1.0])), int(rng.integers(0, 40)))
                 for _ in range(n)]
        free, crit, shared = (int(x) for x in rng.integers(0, 60, size=3))
        order, reserve = policy.upload_plan(cands, free, crit, shared)
        budget = policy.upload_budget(free, crit, shared)
        assert sorted(order) == list(range(n))
        p = [cands[i][0] + cands[i][1] for i in order]
        assert all(a >= b for a, b in zip(p, p[1:]))                       # higher priority first
        assert sum(reserve) <= budget and all(r <= -(-c[2] // 2) for r, c in zip(reserve, cands))
        # greedy in rank order: a candidate gets less than half its deficit only when the budget ran out
        left = budget
        for i in order:
            assert reserve[i] == min(left, -(-cands[i][2] // 2))
            left -= reserve[i]
        # the answer does not depend on how the candidates are listed, ties aside
        if len(set(p)) == n:
            perm = [int(x) for x in rng.permutation(n)]
            o2, r2 = policy.upload_plan([cands[j] for j in perm], free, crit, shared)
            assert [perm[j] for j in o2] == order and [r2[perm.index(i)] for i in range(n)] == reserve
