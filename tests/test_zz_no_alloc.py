"""tc_offload_noalloc (the entry point for callers that cannot allocate) against tc_offload, byte for byte.

Two calls in a row on the same GPU, the second with a smaller input: the fixed device array keeps the
first call's bytes, and nothing of them may show in the second result.  The records are also compared
with the CPU oracle, so both entry points are held to the same bar (bit-exact).
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_18586_amd as K
import tc_workloads as W
from harness import GpuPool, pinned_bytes

pytestmark = pytest.mark.gpu

SHAPES = [
    # 8B-shaped pages (32 KiB, 64 planes: 2 MiB records) in a small pool
    W.PoolShape("8b-pages", 32, 8, 128, 16, 2, 96, 0, "normal"),
    # fp8 pages with one scale word per page and a padded record, ragged tile (10 KiB pages)
    W.PoolShape("scaled-ragged", 3, 5, 64, 32, 1, 200, 6, "fp8"),
    # the tiny configuration
    W.CONFIGS[0],
]


def _noalloc(gp, ids, host, stream):
    s = gp.shape
    return K.tc_offload_noalloc(gp.pool, gp.scales, s.num_layers, s.num_blocks, s.page_bytes, s.block_size,
                                s.scales_per_block, ids, host, stream)


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: s.name)
def test_two_calls_in_a_row_equal_tc_offload(shape):
    rng = W.rng_for(0, salt=77)
    pool_h = W.make_pool_host(shape, rng)
    scales_h = W.make_scales_host(shape, rng)
    gp = GpuPool(shape, pool_h, scales_h)
    try:
        rec = gp.rec
        cap = min(K.TC_NOALLOC_MAX_BLOCKS, K.TC_NOALLOC_STAGING_BYTES // rec, shape.num_blocks)
        stream = torch.cuda.Stream()
        for n in (min(cap, 29), 5):            # the second call is the smaller one
            ids = W.pick_ids(rng, shape.num_blocks, n)
            print(f"[no_alloc] shape={shape.name} n={n} rec={rec}", flush=True)
            want = np.empty(n * rec, dtype=np.uint8)
            oracle.offload(pool_h, scales_h, shape.num_layers, shape.num_blocks, shape.page_bytes,
                           shape.scales_per_block, ids, want)

            ref = pinned_bytes(n * rec)
            ref.fill_(0x5A)
            K.check(K.tc_alloc_at(gp.ctx, ids))
            K.check(K.tc_offload(gp.ctx, ids, ref, stream))
            K.check(K.tc_sync(gp.ctx))
            K.check(K.tc_free(gp.ctx, ids))

            got = pinned_bytes(n * rec + 256)
            got.fill_(0xA5)
            K.check(_noalloc(gp, ids, got, stream))
            stream.synchronize()
            g = got.numpy()
            assert np.array_equal(g[: n * rec], ref.numpy()[: n * rec]), "differs from tc_offload"
            assert np.array_equal(g[: n * rec], want), "differs from the oracle"
            assert (g[n * rec:] == 0xA5).all(), "bytes past the last record were written"
        assert np.array_equal(gp.pool_to_host(), pool_h), "an offload wrote the pool"
    finally:
        gp.close()


def test_limits_and_bad_arguments_enqueue_nothing():
    shape = SHAPES[0]
    rng = W.rng_for(0, salt=78)
    pool_h = W.make_pool_host(shape, rng)
    gp = GpuPool(shape, pool_h, None)
    try:
        rec = gp.rec
        cap = K.TC_NOALLOC_STAGING_BYTES // rec
        host = pinned_bytes((cap + 1) * rec)
        host.fill_(0x11)
        ids = np.arange(cap + 1, dtype=np.int32)
        assert _noalloc(gp, ids, host, None) == K.TC_ERR_LIMIT              # one record too many for the array
        assert _noalloc(gp, ids[:cap], host, None) == K.TC_OK               # exactly the maximum
        torch.cuda.synchronize()
        want = np.empty(cap * rec, dtype=np.uint8)
        oracle.offload(pool_h, None, shape.num_layers, shape.num_blocks, shape.page_bytes, 0, ids[:cap], want)
        assert np.array_equal(host.numpy()[: cap * rec], want)
        host.fill_(0x11)
        assert _noalloc(gp, np.array([3, 3], dtype=np.int32), host, None) == K.TC_ERR_DUP
        assert _noalloc(gp, np.array([shape.num_blocks], dtype=np.int32), host, None) == K.TC_ERR_RANGE
        assert _noalloc(gp, np.array([-1], dtype=np.int32), host, None) == K.TC_ERR_RANGE
        pageable = np.zeros(rec, dtype=np.uint8)
        assert _noalloc(gp, np.array([1], dtype=np.int32), pageable, None) == K.TC_ERR_NOT_PINNED
        assert _noalloc(gp, np.zeros(0, dtype=np.int32), host, None) == K.TC_OK
        torch.cuda.synchronize()
        assert (host.numpy() == 0x11).all(), "a rejected call wrote the host buffer"
    finally:
        gp.close()


def test_more_ids_than_one_id_launch_carries():
    """n above 256 takes several id launches; small pages keep the records inside the array."""
    shape = W.PoolShape("many-small", 2, 1, 8, 16, 2, 1500, 1, "normal")    # 256-B pages, S = 1
    rng = W.rng_for(0, salt=79)
    pool_h = W.make_pool_host(shape, rng)
    scales_h = W.make_scales_host(shape, rng)
    gp = GpuPool(shape, pool_h, scales_h)
    try:
        rec = gp.rec
        host = pinned_bytes(K.TC_NOALLOC_MAX_BLOCKS * rec)
        for n in (K.TC_NOALLOC_MAX_BLOCKS, 300):
            ids = W.pick_ids(rng, shape.num_blocks, n)
            want = np.empty(n * rec, dtype=np.uint8)
            oracle.offload(pool_h, scales_h, shape.num_layers, shape.num_blocks, shape.page_bytes, 1, ids, want)
            host.fill_(0)
            K.check(_noalloc(gp, ids, host, None))
            torch.cuda.synchronize()
            assert np.array_equal(host.numpy()[: n * rec], want)
        assert _noalloc(gp, W.pick_ids(rng, shape.num_blocks, K.TC_NOALLOC_MAX_BLOCKS + 1), host, None) == K.TC_ERR_LIMIT
    finally:
        gp.close()
