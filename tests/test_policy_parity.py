"""The library's scheduling arithmetic (host only, through the C ABI) against the oracle.

Decisions and integer results must be identical; the fitted constants and the cost estimate are
double-precision sums in a different order (Kahan-free long double vs math.fsum), so they are
compared to 1e-9 relative, well inside the 1e-6 ms a decision could ever depend on.
"""
import numpy as np
import pytest

import paper_2510_18586_amd as K
from oracle import policy


def test_fit_and_estimate_match_oracle():
    rng = np.random.default_rng(5)
    for _ in range(50):
        m = int(rng.integers(2, 10))
        n = np.sort(rng.choice(np.arange(1, 1500), size=m, replace=False)).astype(np.uint32)
        off = 0.06 + 0.0374 * n + rng.normal(0, 0.02, m)
        up = 0.08 + 0.0375 * n + rng.normal(0, 0.02, m)
        rc, model = K.tc_cost_fit(n, off, up)
        assert rc == 0
        want = policy.fit_linear(list(map(int, n)), list(off)) + policy.fit_linear(list(map(int, n)), list(up))
        np.testing.assert_allclose(model.as_tuple(), want, rtol=1e-9, atol=1e-12)
        for blocks in (0, 1, 256, 100000):
            got = K.tc_estimate_transfer_ms(model, blocks)
            assert abs(got - policy.estimate_transfer_ms(model.as_tuple(), blocks)) <= 1e-9 * max(1.0, abs(got))
    assert K.tc_cost_fit([5, 5], [1.0, 2.0], [1.0, 2.0])[0] == K.TC_ERR_INVAL
    assert K.tc_cost_fit([5], [1.0], [1.0])[0] == K.TC_ERR_INVAL


def test_paper_numbers_through_the_abi():
    # Sec. 7.6: 15.8 ms at 64 blocks and 79.8 ms at 320 blocks predict the printed 63.7 ms at 256
    rc, model = K.tc_cost_fit([64, 320], [7.9, 39.9], [7.9, 39.9])
    assert rc == 0 and abs(K.tc_estimate_transfer_ms(model, 256) - 63.7) <= 0.15


def test_should_offload_matches_oracle():
    rng = np.random.default_rng(6)
    model = (0.05, 0.0374, 0.07, 0.0375)
    n_true = 0
    for _ in range(2000):
        blocks = int(rng.integers(0, 1100))
        queue = [(int(rng.integers(0, 1200)), float(rng.uniform(0, 60000))) for _ in range(int(rng.integers(0, 9)))]
        v = float(rng.uniform(0.1, 40))
        t_fc = float(rng.choice([0.0, rng.uniform(0, 100), rng.uniform(0, 5000)]))
        rc, k = K.tc_should_offload(model, blocks, t_fc, v, queue)
        want, k_want = policy.should_offload(model, blocks, t_fc, v, queue)
        assert rc == int(want) and k == k_want
        n_true += rc
    assert 200 < n_true < 1800, "the cases should exercise both outcomes"
    # exactly at the boundary T_fc == T_transfer the stall is too short
    t = policy.estimate_transfer_ms(model, 256)
    assert K.tc_should_offload(model, 256, t, 10.0, [(1, 0.0)]) == (0, -1)
    assert K.tc_should_offload(model, 256, np.nextafter(t, np.inf), 10.0, [(1, 0.0)]) == (1, 0)


def test_budget_and_gradual_reserve_match_oracle():
    rng = np.random.default_rng(7)
    for _ in range(3000):
        a, b, c = (int(x) for x in rng.integers(0, 40000, size=3))
        assert K.tc_upload_budget(a, b, c) == policy.upload_budget(a, b, c)
        assert K.tc_gradual_reserve(a, b, c) == policy.gradual_reserve(a, b, c)
    big = 2**32 - 1
    assert K.tc_gradual_reserve(big, big, big) == policy.gradual_reserve(big, big, big) == 2**31
    assert K.tc_upload_budget(big, big, 0) == 0


def test_offload_gate_matches_oracle():
    rng = np.random.default_rng(12)
    model = (0.05, 0.0374, 0.07, 0.0375)
    seen = set()
    for _ in range(4000):
        req = int(rng.integers(0, 600))
        cpu = int(rng.integers(0, 800))
        total = int(rng.integers(1, 20000))
        used = int(rng.integers(0, total + 1))
        thr = float(rng.choice([0.0, 0.3, 0.5, used / total, 0.9, 1.0]))
        queue = [(int(rng.integers(0, 700)), float(rng.uniform(0, 30000))) for _ in range(int(rng.integers(0, 6)))]
        v = float(rng.uniform(0.1, 40))
        t_fc = float(rng.choice([0.0, rng.uniform(0, 100), rng.uniform(0, 3000)]))
        rc, reason, k = K.tc_offload_gate(model, req, cpu, used, total, thr, t_fc, v, queue)
        want_reason, want_k = policy.offload_gate(model, req, cpu, used, total, thr, t_fc, v, queue)
        assert (reason, k) == (want_reason, want_k) and rc == int(want_reason == policy.PASS)
        seen.add(reason)
    assert seen == {0, 1, 2, 3, 4}, "every outcome should occur"
    assert (K.TC_GATE_PASS, K.TC_GATE_CPU_FULL, K.TC_GATE_STALL_SHORT, K.TC_GATE_NO_FIT, K.TC_GATE_LOW_PRESSURE) == \
        (policy.PASS, policy.CPU_FULL, policy.STALL_SHORT, policy.NO_FIT, policy.LOW_PRESSURE)
    assert K.tc_offload_gate(model, 1, 1, 0, 0, 0.5, 10.0, 1.0, [])[0] == K.TC_ERR_INVAL
    assert K.tc_offload_gate(model, 1, 1, 0, 10, float("nan"), 10.0, 1.0, [])[0] == K.TC_ERR_INVAL


def test_upload_plan_matches_oracle():
    rng = np.random.default_rng(13)
    for _ in range(3000):
        n = int(rng.integers(0, 12))
        grid = rng.random() < 0.5           # coarse values force equal priorities
        cands = [((float(rng.integers(0, 5)) / 4 if grid else float(rng.random())),
                  (float(rng.integers(0, 5)) / 4 if grid else float(rng.random())),
                  int(rng.integers(0, 2000))) for _ in range(n)]
        free, crit, shared = (int(x) for x in rng.integers(0, 3000, size=3))
        rc, order, reserve = K.tc_upload_plan(cands, free, crit, shared)
        assert rc == K.TC_OK and (order, reserve) == policy.upload_plan(cands, free, crit, shared)
    big = 2**32 - 1
    assert K.tc_upload_plan([(0.0, 0.0, big), (1.0, 0.0, big)], big, 0, 0) == (0, [1, 0], [2**31 - 1, 2**31]) == \
        (0,) + policy.upload_plan([(0.0, 0.0, big), (1.0, 0.0, big)], big, 0, 0)
    assert K.tc_upload_plan([(float("nan"), 0.0, 1)], 5, 0, 0)[0] == K.TC_ERR_INVAL


def test_lifecycle_matches_oracle_on_every_state_and_event():
    from oracle import lifecycle as L
    for state in range(5):
        for fin in (False, True):
            for fly in (False, True):
                for event in range(-1, 7):
                    req = K.tc_req_state(state, fin, fly, 0)
                    rc, action = K.tc_lifecycle_step(req, event)
                    try:
                        want, want_action = L.step((state, fin, fly), event)
                    except L.Invalid:
                        assert rc == K.TC_ERR_INVAL and req.as_tuple() == (state, fin, fly)
                        continue
                    assert rc == 0 and req.as_tuple() == want and action == want_action, (state, fin, fly, event)
    assert K.tc_lifecycle_step(K.tc_req_state(9, 0, 0, 0), 0)[0] == K.TC_ERR_INVAL


def test_lifecycle_random_walks_match_oracle():
    from oracle import lifecycle as L
    rng = np.random.default_rng(8)
    resumes = 0
    for _ in range(300):
        req, model = K.tc_req_state(0, 0, 0, 0), (L.RUNNING, False, False)
        for _ in range(40):
            e = int(rng.integers(0, 6))
            rc, action = K.tc_lifecycle_step(req, e)
            try:
                model, want_action = L.step(model, e)
            except L.Invalid:
                assert rc == K.TC_ERR_INVAL
            else:
                assert rc == 0 and action == want_action
                resumes += action == L.RESUME
            assert req.as_tuple() == model
    assert resumes > 100


def test_forecaster_matches_oracle():
    from oracle import lifecycle as L
    rng = np.random.default_rng(9)
    for alpha, gamma, default in ((0.3, 0.25, 5000.0), (0.0, 1.0, 0.0), (1.0, 0.5, 10.0)):
        rc, f = K.tc_forecaster_create(alpha, gamma, default)
        assert rc == 0
        o = L.Forecaster(alpha, gamma, default)
        for _ in range(400):
            t = int(rng.integers(0, 6))
            if rng.random() < 0.5:
                x = float(rng.exponential(2000.0))
                assert K.tc_forecaster_observe(f, t, x) == 0
                o.observe(t, x)
            user = float(rng.uniform(10, 9000)) if rng.random() < 0.5 else None
            got, want = K.tc_forecaster_estimate(f, t, user), o.estimate(t, user)
            assert got == want or abs(got - want) <= 1e-12 * abs(want)
        K.tc_forecaster_destroy(f)
    assert K.tc_forecaster_create(1.5, 0.5, 1.0)[0] == K.TC_ERR_INVAL
    assert K.tc_forecaster_create(0.5, 0.0, 1.0)[0] == K.TC_ERR_INVAL
