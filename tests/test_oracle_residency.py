"""Pins for the oracle's residency map / CPU prefix-cache index and its block keys (Sec. 6.3).  CPU only."""
import itertools
import struct

import numpy as np
import pytest

from oracle import residency as R
from oracle import OracleError


# ---- block keys ---------------------------------------------------------------------------------------

def test_fnv1a64_published_vectors():
    """Test vectors of the FNV reference distribution (64-bit FNV-1a)."""
    assert R.fnv1a64(b"") == 0xCBF29CE484222325
    assert R.fnv1a64(b"a") == 0xAF63DC4C8601EC8C
    assert R.fnv1a64(b"foobar") == 0x85944171F73967E8


def test_fnv1a64_is_a_left_fold():
    """Hashing a string equals hashing its tail with the head's hash as the basis."""
    data = bytes(range(1, 200))
    for cut in (0, 1, 7, 100, len(data)):
        assert R.fnv1a64(data) == R.fnv1a64(data[cut:], basis=R.fnv1a64(data[:cut]))


def test_chain_hashes_unrolled_by_hand():
    toks = [3, -1, 70000, 9, 12, 13, 14, 15, 99]            # two whole blocks of 4 and one token over
    h0 = R.fnv1a64(struct.pack("<Q", 5) + struct.pack("<4i", 3, -1, 70000, 9))
    h1 = R.fnv1a64(struct.pack("<Q", h0) + struct.pack("<4i", 12, 13, 14, 15))
    assert R.chain_hashes(toks, 4, parent=5) == [h0, h1]
    assert R.chain_hashes(toks[:3], 4) == []


def test_chain_hashes_cover_the_whole_prefix():
    rng = np.random.default_rng(3)
    a = [int(t) for t in rng.integers(0, 128000, size=16 * 12 + 5)]
    ha = R.chain_hashes(a, 16)
    assert len(ha) == 12 and len(set(ha)) == 12
    for t in (0, 17, 16 * 7 + 15, 16 * 11):
        b = list(a)
        b[t] += 1
        hb = R.chain_hashes(b, 16)
        k = t // 16
        assert hb[:k] == ha[:k]                               # blocks before the change keep their keys
        assert all(x != y for x, y in zip(hb[k:], ha[k:]))    # every block from there on gets a new one
    b = list(a)
    b[-1] += 1                                                # a token of the partial tail has no key
    assert R.chain_hashes(b, 16) == ha
    assert R.chain_hashes(a, 16, parent=1) != ha
    # a continuation hashed from the last key equals hashing the whole sequence
    assert R.chain_hashes(a[16 * 5:], 16, parent=ha[4]) == ha[5:]


# ---- the index ------------------------------------------------------------------------------------------

def test_index_hand_worked_lifecycle():
    ix = R.OracleResidencyIndex()
    ix.insert([10, 11, 12], [7, 3, 9], host_base=0x1000, record_bytes=0x100)
    assert ix.size() == 3
    # prefix lookup: 10, 11 hit; 99 misses and hides 12 behind it
    assert ix.lookup([10, 11, 99, 12]) == [(10, R.CPU, 0x1000, 7), (11, R.CPU, 0x1100, 3)]
    assert ix.lookup([99, 10]) == []
    assert ix.pending([10, 11, 12]) == 0
    ix.begin_upload([10, 11], [7, 4])             # block 7 claimed again, 3 was taken meanwhile
    assert ix.lookup([10, 11, 12]) == [(10, R.H2D, 0x1000, 7), (11, R.H2D, 0x1100, 4), (12, R.CPU, 0x1200, 9)]
    assert ix.pending([10, 11, 12, 99]) == 2      # the request may not run yet
    ix.finish_upload([10, 11])
    assert ix.pending([10, 11, 12]) == 0 and ix.size() == 1
    assert ix.lookup([10]) == [] and ix.lookup([12]) == [(12, R.CPU, 0x1200, 9)]
    ix.remove([12])
    assert ix.size() == 0


def _snapshot(ix):
    return {k: tuple(v) for k, v in ix.entries.items()}


def test_index_errors_leave_no_trace():
    ix = R.OracleResidencyIndex()
    ix.insert([1, 2, 3], [0, 1, 2], 0, 64)
    ix.begin_upload([3], [5])
    snap = _snapshot(ix)
    cases = [
        ("DUP", lambda: ix.insert([4, 2], [8, 9], 4096, 64)),         # 2 is already there; 4 must not appear
        ("DUP", lambda: ix.insert([4, 4], [8, 9], 4096, 64)),
        ("INVAL", lambda: ix.insert([4, 5], [8], 4096, 64)),
        ("INVAL", lambda: ix.begin_upload([1, 9], [4, 5])),           # 9 is absent; 1 must stay CPU-resident
        ("INVAL", lambda: ix.begin_upload([1, 3], [4, 5])),           # 3 is already an H2D entry
        ("DUP", lambda: ix.begin_upload([1, 1], [4, 5])),
        ("INVAL", lambda: ix.finish_upload([3, 1])),                  # 1 has no upload in flight
        ("INVAL", lambda: ix.remove([1, 3])),                         # 3 is being read by its upload
        ("INVAL", lambda: ix.remove([1, 9])),
    ]
    for code, call in cases:
        with pytest.raises(OracleError) as e:
            call()
        assert e.value.code == code
        assert _snapshot(ix) == snap


def test_index_prefix_lookup_against_a_plain_set():
    rng = np.random.default_rng(11)
    for trial in range(300):
        ix = R.OracleResidencyIndex()
        universe = [int(k) for k in rng.choice(1 << 20, size=12, replace=False)]
        present = universe[:int(rng.integers(0, 13))]
        ix.insert(present, list(range(len(present))), 0, 1)
        q = [int(k) for k in rng.choice(universe, size=int(rng.integers(0, 10)))]
        want = list(itertools.takewhile(lambda k: k in set(present), q))
        got = ix.lookup(q)
        assert [h[0] for h in got] == want
        for key, state, rec, blk in got:
            assert state == R.CPU and rec == present.index(key) and blk == present.index(key)


def test_index_random_walk_keeps_the_map_consistent():
    """Every key is in exactly one of {absent, CPU-resident, H2D}; records of live keys never coincide."""
    rng = np.random.default_rng(5)
    ix = R.OracleResidencyIndex()
    model_cpu, model_h2d = {}, {}
    next_rec = 0
    for step in range(3000):
        op = int(rng.integers(0, 4))
        if op == 0:
            keys = [int(k) for k in rng.integers(0, 64, size=int(rng.integers(1, 4)))]
            ok = len(set(keys)) == len(keys) and not any(k in model_cpu or k in model_h2d for k in keys)
            try:
                ix.insert(keys, keys, next_rec, 16)
                assert ok
                for j, k in enumerate(keys):
                    model_cpu[k] = next_rec + 16 * j
                next_rec += 16 * len(keys)
            except OracleError:
                assert not ok
        elif op == 1 and model_cpu:
            keys = [int(k) for k in rng.permutation(list(model_cpu))[:2]]
            ix.begin_upload(keys, [0] * len(keys))
            for k in keys:
                model_h2d[k] = model_cpu.pop(k)
        elif op == 2 and model_h2d:
            keys = [int(k) for k in rng.permutation(list(model_h2d))[:2]]
            ix.finish_upload(keys)
            for k in keys:
                del model_h2d[k]
        elif op == 3 and model_cpu:
            k = int(rng.permutation(list(model_cpu))[0])
            ix.remove([k])
            del model_cpu[k]
        assert ix.size() == len(model_cpu) + len(model_h2d)
        assert ix.pending(range(64)) == len(model_h2d)
        recs = [v[1] for v in ix.entries.values()]
        assert len(set(recs)) == len(recs)
        for k, rec in model_cpu.items():
            assert ix.lookup([k]) == [(k, R.CPU, rec, k)]
