"""The library's residency index and block keys against the oracle model, call for call.  CPU only:
these entry points are host code, reached through the same C ABI as everything else."""
import numpy as np
import pytest

import paper_2510_18586_amd as K
from oracle import OracleError
from oracle import residency as R

CODE = {"INVAL": K.TC_ERR_INVAL, "DUP": K.TC_ERR_DUP}


@pytest.fixture
def index():
    rc, ix = K.tc_index_create()
    assert rc == K.TC_OK and ix
    yield ix
    assert K.tc_index_destroy(ix) == K.TC_OK


def _orc(fn, *a):
    try:
        fn(*a)
        return K.TC_OK
    except OracleError as e:
        return CODE[e.code]


def test_constants_agree():
    assert (K.TC_RES_ABSENT, K.TC_RES_CPU, K.TC_RES_H2D) == (R.ABSENT, R.CPU, R.H2D)
    assert K.TC_FNV_BASIS == R.FNV_BASIS


def test_fnv_and_chain_hashes_match_oracle():
    rng = np.random.default_rng(9)
    for n in (0, 1, 2, 7, 64, 1000):
        data = rng.integers(0, 256, size=n, dtype=np.uint8).tobytes()
        assert K.tc_fnv1a64(data) == R.fnv1a64(data)
        assert K.tc_fnv1a64(data, 12345) == R.fnv1a64(data, 12345)
    for bs, n_tok, parent in ((16, 0, 0), (16, 15, 0), (16, 16, 0), (16, 16 * 9 + 3, 77), (32, 32 * 40, 1 << 63), (1, 5, 2)):
        toks = rng.integers(-5, 200000, size=n_tok, dtype=np.int32)
        rc, keys = K.tc_chain_hashes(toks, bs, parent)
        assert rc == K.TC_OK
        assert [int(k) for k in keys] == R.chain_hashes([int(t) for t in toks], bs, parent)
    assert K.tc_chain_hashes(np.zeros(4, np.int32), 0)[0] == K.TC_ERR_INVAL


def test_hand_worked_lifecycle_matches_oracle(index):
    orc = R.OracleResidencyIndex()
    assert K.tc_index_insert(index, [10, 11, 12], [7, 3, 9], 0x1000, 0x100) == K.TC_OK
    orc.insert([10, 11, 12], [7, 3, 9], 0x1000, 0x100)
    for q in ([10, 11, 99, 12], [99, 10], [], [12, 12, 11]):
        assert K.tc_index_lookup(index, q) == (K.TC_OK, orc.lookup(q))
    assert K.tc_index_begin_upload(index, [10, 11], [7, 4]) == K.TC_OK
    orc.begin_upload([10, 11], [7, 4])
    assert K.tc_index_lookup(index, [10, 11, 12]) == (K.TC_OK, orc.lookup([10, 11, 12]))
    assert K.tc_index_pending(index, [10, 11, 12, 99]) == orc.pending([10, 11, 12, 99]) == 2
    assert K.tc_index_finish_upload(index, [10, 11]) == K.TC_OK
    orc.finish_upload([10, 11])
    assert K.tc_index_size(index) == orc.size() == 1
    assert K.tc_index_remove(index, [12]) == K.TC_OK
    assert K.tc_index_size(index) == 0


def test_errors_match_oracle_and_leave_no_trace(index):
    orc = R.OracleResidencyIndex()
    K.tc_index_insert(index, [1, 2, 3], [0, 1, 2], 4096, 64), orc.insert([1, 2, 3], [0, 1, 2], 4096, 64)
    K.tc_index_begin_upload(index, [3], [5]), orc.begin_upload([3], [5])
    before = K.tc_index_lookup(index, [1, 2, 3])
    cases = [
        (K.tc_index_insert, orc.insert, ([4, 2], [8, 9], 8192, 64)),
        (K.tc_index_insert, orc.insert, ([4, 4], [8, 9], 8192, 64)),
        (K.tc_index_insert, orc.insert, ([4, 5], [8], 8192, 64)),
        (K.tc_index_begin_upload, orc.begin_upload, ([1, 9], [4, 5])),
        (K.tc_index_begin_upload, orc.begin_upload, ([1, 3], [4, 5])),
        (K.tc_index_begin_upload, orc.begin_upload, ([1, 1], [4, 5])),
        (K.tc_index_finish_upload, orc.finish_upload, ([3, 1],)),
        (K.tc_index_remove, orc.remove, ([1, 3],)),
        (K.tc_index_remove, orc.remove, ([1, 9],)),
    ]
    for nat_fn, orc_fn, args in cases:
        rc = nat_fn(index, *args)
        assert rc == _orc(orc_fn, *args) and rc != K.TC_OK
        assert K.tc_index_lookup(index, [1, 2, 3]) == before == (K.TC_OK, orc.lookup([1, 2, 3]))
        assert K.tc_index_size(index) == 3 and K.tc_index_lookup(index, [4])[1] == []


def test_null_arguments(index):
    lib = K.binding._load()
    assert lib.tc_index_create(None) == K.TC_ERR_INVAL
    assert lib.tc_index_insert(None, None, None, None, 0, 0) == K.TC_ERR_INVAL
    assert lib.tc_index_insert(index, None, None, None, 64, 1) == K.TC_ERR_INVAL
    assert lib.tc_index_lookup(index, None, 0, None, None) == K.TC_ERR_INVAL
    assert K.tc_index_pending(None, [1]) == 0 and K.tc_index_size(None) == 0
    assert K.tc_index_destroy(None) == K.TC_OK
    assert K.tc_index_insert(index, [], [], None, 64) == K.TC_OK          # n = 0 is a no-op


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_walk_call_for_call(index, seed):
    rng = np.random.default_rng(seed)
    orc = R.OracleResidencyIndex()
    universe = [int(k) for k in rng.integers(0, 1 << 63, size=48, dtype=np.int64)] + [(1 << 64) - 1, 0]
    base = 1 << 20
    for step in range(4000):
        op = int(rng.integers(0, 6))
        keys = [universe[i] for i in rng.integers(0, len(universe), size=int(rng.integers(0, 5)))]
        if op == 0:
            blocks = [int(b) for b in rng.integers(0, 1000, size=len(keys))]
            rec = int(rng.integers(1, 5)) * 256
            assert K.tc_index_insert(index, keys, blocks, base, rec) == _orc(orc.insert, keys, blocks, base, rec)
            base += 5 * 1280
        elif op == 1:
            blocks = [int(b) for b in rng.integers(0, 1000, size=len(keys))]
            assert K.tc_index_begin_upload(index, keys, blocks) == _orc(orc.begin_upload, keys, blocks)
        elif op == 2:
            assert K.tc_index_finish_upload(index, keys) == _orc(orc.finish_upload, keys)
        elif op == 3:
            assert K.tc_index_remove(index, keys) == _orc(orc.remove, keys)
        elif op == 4:
            assert K.tc_index_lookup(index, keys) == (K.TC_OK, orc.lookup(keys))
        else:
            assert K.tc_index_pending(index, keys) == orc.pending(keys)
        assert K.tc_index_size(index) == orc.size()
    # the whole map, key by key
    for k in universe:
        assert K.tc_index_lookup(index, [k]) == (K.TC_OK, orc.lookup([k]))
