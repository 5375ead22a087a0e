"""Pins for the CPU oracle's data movement (no GPU).

The oracle is checked against things other than itself: values the paper prints
(tests/golden/block_size_anchors.txt), numpy's own indexing routines on a 4-d view
of the pool, the invariants the problem fixes (byte-identical round trip, foreign
blocks untouched, same logical tokens after the remap) and brute force over every
id tuple of tiny pools.  Pool bytes are made position-unique so that a wrong index,
a transposed operand or a dropped plane changes the result.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
import tc_workloads as W

O = oracle      # the oracle under test; test_oracle_mutants.py swaps in deliberately broken builds

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "block_size_anchors.txt")


def _golden(kind):
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith(kind + " "):
                rows.append([int(x) for x in line.split()[1:]])
    assert rows
    return rows


def unique_pool(P, NB, pb, salt=0):
    """uint8 pool where (plane, block, byte) -> value is injective enough to expose index slips."""
    idx = np.arange(P * NB * pb, dtype=np.uint64) + np.uint64(salt)
    v = (idx * np.uint64(2654435761) >> np.uint64(7)) ^ (idx >> np.uint64(3))
    return (v & np.uint64(0xFF)).astype(np.uint8)


# ------------------------------------------------------------------ paper anchors
def test_block_bytes_matches_paper():
    for L, H, D, bs, eb, want in _golden("block_bytes"):
        pb = O.page_bytes(bs, H, D, eb)
        assert 2 * L * pb == want
        assert O.record_bytes(L, pb, 0) == want  # no scales, already a 256-B multiple


def test_tokens_to_blocks_matches_paper():
    for tokens, bs, want in _golden("tokens_to_blocks"):
        assert O.blocks_for_tokens(tokens, bs) == want
    assert O.blocks_for_tokens(1, 16) == 1
    assert O.blocks_for_tokens(17, 16) == 2
    assert O.blocks_for_tokens(0, 16) == 0


def test_benchmark_config_record_sizes():
    # the benchmark configurations: 2 MiB per block for the 8B shape; 4 MiB for 64 layers;
    # 5 MiB of fp8 pages + 160 scale words (640 B), padded to a 256-B multiple
    c = W.CONFIGS
    assert O.record_bytes(c[0].num_layers, c[0].page_bytes, 0) == 32 * 1024
    assert O.record_bytes(c[1].num_layers, c[1].page_bytes, 0) == 2 * 1024 * 1024
    assert O.record_bytes(c[3].num_layers, c[3].page_bytes, 0) == 4 * 1024 * 1024
    assert c[4].page_bytes == 32 * 1024
    assert O.record_bytes(c[4].num_layers, c[4].page_bytes, 160) == 5 * 1024 * 1024 + 768
    assert O.record_bytes(1, 16, 0) == 256   # pad up
    assert O.record_bytes(1, 16, 1) == 256
    assert O.record_bytes(2, 64, 4) == 512   # 256 + 16 -> 512


# ------------------------------------------------------------------ numpy as the definition
@pytest.mark.parametrize("L,NB,pb,S,n", [(2, 64, 48, 0, 9), (3, 37, 80, 6, 11), (1, 19, 16, 1, 5), (4, 128, 256, 0, 40)])
def test_offload_is_numpy_take(L, NB, pb, S, n):
    P = 2 * L
    rng = np.random.default_rng(L * 1000 + NB)
    pool = unique_pool(P, NB, pb)
    scales = rng.integers(0, 2**32, size=S * NB, dtype=np.uint32) if S else None
    ids = W.pick_ids(rng, NB, n)
    rec = O.record_bytes(L, pb, S)
    host = np.full(n * rec, 0xAB, dtype=np.uint8)
    O.offload(pool, scales, L, NB, pb, S, ids, host)

    h = host.reshape(n, rec)
    # pages: the library's own gather along the block axis, blocks moved to the front
    want_pages = np.take(pool.reshape(P, NB, pb), ids, axis=1).transpose(1, 0, 2).reshape(n, P * pb)
    assert np.array_equal(h[:, : P * pb], want_pages)
    if S:
        want_sc = np.take(scales.reshape(S, NB), ids, axis=1).T.copy()
        assert np.array_equal(h[:, P * pb : P * pb + 4 * S].copy().view(np.uint32), want_sc)
    assert not h[:, P * pb + 4 * S :].any(), "pad bytes must be zero"


@pytest.mark.parametrize("L,NB,pb,S,n", [(2, 64, 48, 0, 9), (3, 37, 80, 6, 11), (1, 19, 16, 1, 5)])
def test_upload_is_numpy_put(L, NB, pb, S, n):
    P = 2 * L
    rng = np.random.default_rng(7 + NB)
    rec = O.record_bytes(L, pb, S)
    pool0 = unique_pool(P, NB, pb, salt=5)
    scales0 = rng.integers(0, 2**32, size=S * NB, dtype=np.uint32) if S else None
    host = rng.integers(0, 256, size=n * rec, dtype=np.uint8)
    new_ids = W.pick_ids(rng, NB, n)
    table = np.full(n + 3, -7, dtype=np.int32)

    pool, scales = pool0.copy(), (scales0.copy() if S else None)
    O.upload(host, L, NB, pb, S, new_ids, pool, scales, table[1:])

    want = pool0.reshape(P, NB, pb).copy()
    want[:, new_ids, :] = host.reshape(n, rec)[:, : P * pb].reshape(n, P, pb).transpose(1, 0, 2)
    assert np.array_equal(pool.reshape(P, NB, pb), want)
    if S:
        ws = scales0.reshape(S, NB).copy()
        ws[:, new_ids] = host.reshape(n, rec)[:, P * pb : P * pb + 4 * S].copy().view(np.uint32).T
        assert np.array_equal(scales.reshape(S, NB), ws)
    assert table[0] == -7 and (table[n + 1 :] == -7).all()
    assert np.array_equal(table[1 : n + 1], new_ids)


# ------------------------------------------------------------------ invariants of the problem
def _round_trip(shape, rng, n, scramble=True, same_ids=False):
    L, NB, pb, S = shape.num_layers, shape.num_blocks, shape.page_bytes, shape.scales_per_block
    P = 2 * L
    pool0 = W.make_pool_host(shape, rng)
    scales0 = W.make_scales_host(shape, rng)
    ids = W.pick_ids(rng, NB, n)
    new_ids = ids.copy() if same_ids else W.pick_ids(rng, NB, n, exclude=ids)
    rec = O.record_bytes(L, pb, S)
    host = np.empty(n * rec, dtype=np.uint8)
    pool = pool0.copy()
    scales = scales0.copy() if S else None
    O.offload(pool, scales, L, NB, pb, S, ids, host)
    assert np.array_equal(pool, pool0), "offload must not write the pool"
    scr = np.zeros(NB, dtype=bool)
    if scramble:  # the freed source blocks get reused by somebody else
        pv = pool.reshape(P, NB, pb)
        pv[:, ids, :] = rng.integers(0, 256, size=(P, n, pb), dtype=np.uint8)
        if S:
            scales.reshape(S, NB)[:, ids] = rng.integers(0, 2**32, size=(S, n), dtype=np.uint32)
        scr[ids] = True
    table = np.full(n + 2, -1, dtype=np.int32)
    table[:n] = ids
    table0 = table.copy()
    O.upload(host, L, NB, pb, S, new_ids, pool, scales, table)
    return pool0, scales0, pool, scales, ids, new_ids, table0, table, scr


@pytest.mark.parametrize("same_ids", [False, True])
def test_round_trip_byte_identical_and_foreign_blocks_untouched(same_ids):
    shape = W.CONFIGS[0]
    rng = W.rng_for(0)
    n = 8
    pool0, _, pool, _, ids, new_ids, table0, table, scr = _round_trip(shape, rng, n, same_ids=same_ids)
    P, NB, pb = shape.planes, shape.num_blocks, shape.page_bytes
    a, b = pool0.reshape(P, NB, pb), pool.reshape(P, NB, pb)
    for i in range(n):
        assert np.array_equal(b[:, new_ids[i]], a[:, ids[i]])
    foreign = np.ones(NB, dtype=bool)
    foreign[new_ids] = False
    foreign &= ~scr
    assert np.array_equal(b[:, foreign], a[:, foreign])
    assert (table[n:] == table0[n:]).all()


def test_round_trip_with_scales_and_ragged_page():
    shape = W.PoolShape("odd", 3, 3, 24, 4, 1, 50, 6, "fp8")  # pb = 288: not a power of two
    rng = W.rng_for(4, salt=1)
    n = 7
    pool0, sc0, pool, sc, ids, new_ids, _, _, scr = _round_trip(shape, rng, n)
    S, NB = shape.scales_per_block, shape.num_blocks
    for i in range(n):
        assert np.array_equal(sc.reshape(S, NB)[:, new_ids[i]], sc0.reshape(S, NB)[:, ids[i]])
    foreign = np.ones(NB, dtype=bool)
    foreign[new_ids] = False
    foreign &= ~scr
    assert np.array_equal(sc.reshape(S, NB)[:, foreign], sc0.reshape(S, NB)[:, foreign])


def test_remapped_table_addresses_same_logical_tokens():
    shape = W.CONFIGS[0]
    rng = W.rng_for(0, salt=2)
    n = 8
    pool0, _, pool, _, ids, new_ids, table0, table, _ = _round_trip(shape, rng, n)
    L, NB, pb, bs = shape.num_layers, shape.num_blocks, shape.page_bytes, shape.block_size
    for t in range(n * bs):
        for layer in range(L):
            for kv in (0, 1):
                before = O.read_token(pool0, L, NB, pb, bs, table0, t, layer, kv)
                after = O.read_token(pool, L, NB, pb, bs, table, t, layer, kv)
                assert np.array_equal(before, after)
    # read_token itself against numpy on the 5-d view [L][2][NB][bs][token bytes]
    v = pool0.reshape(L, 2, NB, bs, pb // bs)
    assert np.array_equal(O.read_token(pool0, L, NB, pb, bs, table0, 37, 1, 0), v[1, 0, table0[37 // bs], 37 % bs])


# ------------------------------------------------------------------ brute force on tiny pools
def test_brute_force_all_id_tuples():
    pb = 16
    for L in (1, 2):
        P = 2 * L
        for NB in (1, 3, 6):
            for S in (0, 1, P):
                pool = unique_pool(P, NB, pb, salt=NB)
                scales = (np.arange(S * NB, dtype=np.uint32) * np.uint32(2246822519) + np.uint32(9)) if S else None
                rec = O.record_bytes(L, pb, S)
                for n in range(0, min(3, NB) + 1):
                    for ids in itertools.permutations(range(NB), n):
                        ids_a = np.array(ids, dtype=np.int32)
                        host = np.full(max(n, 1) * rec, 0xEE, dtype=np.uint8)
                        O.offload(pool, scales, L, NB, pb, S, ids_a, host)
                        for j in range(n):
                            for p in range(P):
                                for b in range(pb):
                                    assert host[j * rec + p * pb + b] == pool[(p * NB + ids[j]) * pb + b]
                            for s in range(S):
                                w = int.from_bytes(host[j * rec + P * pb + 4 * s : j * rec + P * pb + 4 * s + 4].tobytes(), "little")
                                assert w == int(scales[s * NB + ids[j]])
                            assert not host[j * rec + P * pb + 4 * S : (j + 1) * rec].any()
                        if n == 0:
                            assert (host == 0xEE).all()
                        # upload into every other ordered tuple, check each byte of the pool
                        for new in itertools.permutations(range(NB), n):
                            if NB == 6 and n == 3 and new[0] > 1:
                                continue  # keep the run short; tuples starting 0/1 still cover every position
                            pool2 = np.zeros_like(pool)
                            sc2 = np.zeros(S * NB, dtype=np.uint32) if S else None
                            tbl = np.full(n + 1, -3, dtype=np.int32)
                            O.upload(host, L, NB, pb, S, np.array(new, dtype=np.int32), pool2, sc2, tbl)
                            want = np.zeros_like(pool)
                            for i in range(n):
                                for p in range(P):
                                    want[(p * NB + new[i]) * pb : (p * NB + new[i] + 1) * pb] = pool[(p * NB + ids[i]) * pb : (p * NB + ids[i] + 1) * pb]
                            assert np.array_equal(pool2, want)
                            assert list(tbl[:n]) == list(new) and tbl[n] == -3
                            if S:
                                ws = np.zeros(S * NB, dtype=np.uint32)
                                for i in range(n):
                                    for s in range(S):
                                        ws[s * NB + new[i]] = scales[s * NB + ids[i]]
                                assert np.array_equal(sc2, ws)


# ------------------------------------------------------------------ degenerate / error cases
def test_empty_and_bad_ids():
    L, NB, pb = 2, 8, 32
    pool = unique_pool(2 * L, NB, pb)
    host = np.full(256, 0x11, dtype=np.uint8)
    O.offload(pool, None, L, NB, pb, 0, np.zeros(0, dtype=np.int32), host)
    assert (host == 0x11).all()
    before = pool.copy()
    for bad in ([-1], [NB], [0, 2**31 - 1]):
        h = np.full(len(bad) * 256, 0x11, dtype=np.uint8)
        with pytest.raises(O.OracleError):
            O.offload(pool, None, L, NB, pb, 0, np.array(bad, dtype=np.int32), h)
        assert (h == 0x11).all(), "nothing may be written when an id is bad"
        with pytest.raises(O.OracleError):
            O.upload(h, L, NB, pb, 0, np.array(bad, dtype=np.int32), pool, None, None)
        assert np.array_equal(pool, before)


def test_opaque_bytes_survive():
    # NaN payloads, -0.0 and denormal patterns are bytes like any other
    L, NB, pb = 1, 4, 16
    pool = np.zeros(2 * L * NB * pb, dtype=np.uint8)
    special = np.array([0x7FC1, 0xFFFF, 0x8000, 0x0001, 0x7F80, 0xFF81, 0x0000, 0x7FFF], dtype=np.uint16).view(np.uint8)
    pool[(0 * NB + 2) * pb : (0 * NB + 2) * pb + 16] = special
    host = np.empty(256, dtype=np.uint8)
    O.offload(pool, None, L, NB, pb, 0, np.array([2], dtype=np.int32), host)
    assert np.array_equal(host[:16], special)
