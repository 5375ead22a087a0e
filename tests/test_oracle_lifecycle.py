"""Pins for the oracle's lifecycle and forecast (no GPU): the paper's own statements as scenarios,
structural properties over every reachable state, and closed forms of the moving average."""
import itertools

import numpy as np
import pytest

from oracle import lifecycle as L


def run(events, req=(L.RUNNING, False, False)):
    actions = []
    for e in events:
        req, a = L.step(req, e)
        actions.append(a)
    return req, actions


def test_five_states_and_the_ordinary_round_trip():
    assert len({L.RUNNING, L.PENDING_OFFLOAD, L.OFFLOADED, L.PENDING_UPLOAD, L.UPLOADED}) == 5
    req, acts = run([L.CALL_START, L.OFFLOAD_ISSUED, L.OFFLOAD_DONE, L.UPLOAD_ISSUED, L.UPLOAD_DONE, L.CALL_FINISH])
    assert req == (L.RUNNING, False, False)
    assert acts == [L.NONE] * 5 + [L.RESUME]            # uploaded before the tool returned: resumes at once


def test_tool_returns_early_triggers_immediate_upload():
    req, acts = run([L.CALL_START, L.OFFLOAD_ISSUED, L.OFFLOAD_DONE, L.CALL_FINISH])
    assert acts[-1] == L.UPLOAD_NOW and req[0] == L.OFFLOADED
    req, acts = run([L.UPLOAD_ISSUED, L.UPLOAD_DONE], req)
    assert req == (L.RUNNING, False, False) and acts[-1] == L.RESUME


def test_tool_returns_while_a_copy_is_in_flight():
    req, acts = run([L.CALL_START, L.OFFLOAD_ISSUED, L.CALL_FINISH])
    assert acts[-1] == L.WAIT
    req, acts = run([L.OFFLOAD_DONE], req)
    assert acts == [L.UPLOAD_NOW]                        # source blocks are pending-free until the copy is done
    req, acts = run([L.CALL_START, L.OFFLOAD_ISSUED, L.OFFLOAD_DONE, L.UPLOAD_ISSUED, L.CALL_FINISH, L.UPLOAD_DONE])
    assert acts[-2:] == [L.WAIT, L.RESUME] and req == (L.RUNNING, False, False)


def test_offload_not_approved_means_plain_resume():
    req, acts = run([L.CALL_START, L.CALL_FINISH])
    assert req == (L.RUNNING, False, False) and acts[-1] == L.RESUME


def test_reachable_states_are_sound():
    start = (L.RUNNING, False, False)
    seen, frontier = {start}, [start]
    while frontier:
        req = frontier.pop()
        for e in range(6):
            try:
                nxt, act = L.step(req, e)
            except L.Invalid:
                continue
            # an agent only ever resumes with its KV on the GPU and nothing in flight
            if act == L.RESUME:
                assert nxt == start
                assert req[0] in (L.UPLOADED, L.PENDING_UPLOAD, L.PENDING_OFFLOAD)
            if act == L.UPLOAD_NOW:
                assert nxt[0] == L.OFFLOADED and nxt[1]
            if nxt not in seen:
                seen.add(nxt)
                frontier.append(nxt)
    assert {s for s, _, _ in seen} == {0, 1, 2, 3, 4}
    assert len(seen) == 9
    # every reachable state can get back to running
    for req in seen:
        ok = False
        for path in itertools.product(range(6), repeat=5):
            cur = req
            try:
                for e in path:
                    cur, _ = L.step(cur, e)
                    if cur == start:
                        ok = True
                        break
            except L.Invalid:
                pass
            if ok:
                break
        assert ok, req
    for bad in ((L.RUNNING, L.OFFLOAD_DONE), (L.OFFLOADED, L.CALL_START), (L.UPLOADED, L.UPLOAD_ISSUED)):
        with pytest.raises(L.Invalid):
            L.step((bad[0], False, False), bad[1])


def test_forecast_defaults_eq1_and_moving_average():
    f = L.Forecaster(alpha=0.3, gamma=0.25, default_ms=5000.0)
    assert f.estimate("search") == 5000.0                   # nothing known: the system constant
    assert f.estimate("search", 800.0) == 800.0             # the user's estimate
    f.observe("search", 1200.0)
    assert f.estimate("search") == 1200.0                   # first observation taken as is
    assert f.estimate("search", 800.0) == pytest.approx(0.3 * 800 + 0.7 * 1200)   # Eq. 1
    assert f.estimate("other", 50.0) == 50.0                # per function type
    obs = [1200.0, 400.0, 900.0, 100.0, 2500.0]
    for x in obs[1:]:
        f.observe("search", x)
    g = 0.25
    k = len(obs)
    closed = (1 - g) ** (k - 1) * obs[0] + sum(g * (1 - g) ** (k - 1 - j) * obs[j] for j in range(1, k))
    assert f.estimate("search") == pytest.approx(closed, rel=1e-12)
    c = L.Forecaster(0.5, 0.4, 1.0)
    for _ in range(50):
        c.observe(7, 321.0)
    assert c.estimate(7) == pytest.approx(321.0)            # a constant signal is a fixed point
