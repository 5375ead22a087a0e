"""The measurement helpers of the library are kernels too: the contiguous copies must be exact and
must reject what their kernels cannot take."""
import numpy as np
import pytest
import torch

import paper_2510_18586_amd as K
from harness import DEV

pytestmark = pytest.mark.gpu


def _src(nbytes, seed):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    return torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device=DEV, generator=g)


@pytest.mark.parametrize("nbytes", [16, 4096 - 16, 32768, 32768 * 5 + 48, 64 << 20])
def test_copy_contiguous_is_exact_including_a_ragged_tail(nbytes):
    guard = 4096
    a = _src(nbytes, 1)
    b = torch.full((guard + nbytes + guard,), 0xEE, dtype=torch.uint8, device=DEV)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())      # a and b were filled on torch's current stream
    K.check(K.tc_copy_contiguous(b[guard:], a, nbytes, stream))
    stream.synchronize()
    assert torch.equal(b[guard:guard + nbytes], a)
    assert bool((b[:guard] == 0xEE).all()) and bool((b[guard + nbytes:] == 0xEE).all())


@pytest.mark.parametrize("direct_loads", [0, 1])
@pytest.mark.parametrize("nbytes", [16384, 16384 * 7, 48 << 20])
def test_copy_via_lds_is_exact(direct_loads, nbytes):
    guard = 4096
    a = _src(nbytes, 2 + direct_loads)
    b = torch.full((guard + nbytes + guard,), 0xEE, dtype=torch.uint8, device=DEV)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    K.check(K.tc_copy_via_lds(b[guard:], a, nbytes, direct_loads, stream))
    stream.synchronize()
    assert torch.equal(b[guard:guard + nbytes], a)
    assert bool((b[:guard] == 0xEE).all()) and bool((b[guard + nbytes:] == 0xEE).all())


def test_helpers_reject_sizes_and_alignments_their_kernels_cannot_take():
    a = torch.zeros(1 << 16, dtype=torch.uint8, device=DEV)
    b = torch.zeros(1 << 16, dtype=torch.uint8, device=DEV)
    assert K.tc_copy_contiguous(b, a, 24) == K.TC_ERR_INVAL                 # not a multiple of 16
    assert K.tc_copy_contiguous(b[8:], a, 32) == K.TC_ERR_INVAL             # misaligned
    assert K.tc_copy_contiguous(None, a, 32) == K.TC_ERR_INVAL
    assert K.tc_copy_contiguous(b, a, 0) == K.TC_OK
    assert K.tc_copy_via_lds(b, a, 16384 + 16, 0) == K.TC_ERR_INVAL         # whole tiles only
    assert K.tc_copy_via_lds(b[16:], a[8:], 16384, 1) == K.TC_ERR_INVAL
    assert K.tc_copy_via_lds(b, a, 0, 1) == K.TC_OK
    torch.cuda.synchronize()


def test_hbm_stream_computes_the_triad():
    n = (1 << 20) + 4 * 37
    g = torch.Generator(device=DEV)
    g.manual_seed(9)
    b = torch.randn(n, device=DEV, generator=g)
    c = torch.randn(n, device=DEV, generator=g)
    a = torch.zeros(n, device=DEV)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    K.check(K.tc_hbm_stream(a, b, c, n, 0.5, 2, stream))
    stream.synchronize()
    # a = b + 0.5 * c in fp32: multiplying by 0.5 is exact, so fused or not the result is the rounded sum
    assert torch.equal(a, b + 0.5 * c)
    assert K.tc_hbm_stream(a, b, c, n + 1, 0.5, 1, stream) == K.TC_ERR_INVAL


def test_one_way_streams_write_everything_and_read_without_side_effects():
    nbytes = 4096 * 2051                       # not a multiple of 8 tiles: the last run is short
    guard = 4096
    buf = torch.full((guard + nbytes + guard,), 0xEE, dtype=torch.uint8, device=DEV)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    K.check(K.tc_hbm_write(buf[guard:], nbytes, stream))
    stream.synchronize()
    words = buf[guard:guard + nbytes].view(torch.int32).view(-1, 256, 4)      # [tile][lane][4 words]
    tiles = torch.arange(words.shape[0], dtype=torch.int32, device=DEV)
    assert torch.equal(words[:, :, 0], tiles[:, None].expand(-1, 256))        # every tile written, by its own workgroup
    assert torch.equal(words[:, :, 2], torch.arange(256, dtype=torch.int32, device=DEV)[None, :].expand(words.shape[0], -1))
    assert bool((buf[:guard] == 0xEE).all()) and bool((buf[guard + nbytes:] == 0xEE).all())
    before = buf.clone()
    K.check(K.tc_hbm_read(buf[guard:], nbytes, stream))
    stream.synchronize()
    assert torch.equal(buf, before)
    assert K.tc_hbm_write(buf[guard:], 4096 + 16, stream) == K.TC_ERR_INVAL
    assert K.tc_hbm_read(buf[guard + 8:], 4096, stream) == K.TC_ERR_INVAL
    assert K.tc_hbm_read(None, 0, stream) == K.TC_OK


def test_stage_on_device_is_the_staged_kernel_on_device_records():
    """tc_stage_on_device against the oracle: gather into device records, scatter from them into other blocks."""
    import oracle
    import tc_workloads as W
    from harness import GpuPool
    shape = W.PoolShape("fp8-small", 3, 2, 32, 8, 1, 80, 6, "fp8")
    rng = W.rng_for(4, salt=91)
    pool_h, scales_h = W.make_pool_host(shape, rng), W.make_scales_host(shape, rng)
    gp = GpuPool(shape, pool_h, scales_h)
    try:
        n, rec = 23, gp.rec
        ids = W.pick_ids(rng, shape.num_blocks, n)
        new_ids = W.pick_ids(rng, shape.num_blocks, n, exclude=ids)
        records = torch.full((n * rec + 256,), 0x77, dtype=torch.uint8, device=DEV)
        stream = torch.cuda.Stream()
        stream.wait_stream(torch.cuda.current_stream())
        K.check(K.tc_stage_on_device(gp.ctx, 0, ids, records, stream))
        want = np.empty(n * rec, dtype=np.uint8)
        oracle.offload(pool_h, scales_h, shape.num_layers, shape.num_blocks, shape.page_bytes, shape.scales_per_block, ids, want)
        K.check(K.tc_sync(gp.ctx))
        got = records.cpu().numpy()
        assert np.array_equal(got[: n * rec], want) and (got[n * rec:] == 0x77).all()
        K.check(K.tc_stage_on_device(gp.ctx, 1, new_ids, records, stream))
        K.check(K.tc_sync(gp.ctx))
        oracle.upload(want, shape.num_layers, shape.num_blocks, shape.page_bytes, shape.scales_per_block, new_ids, pool_h, scales_h, None)
        assert np.array_equal(gp.pool_to_host(), pool_h) and np.array_equal(gp.scales_all_to_host(), scales_h)
        assert K.tc_stage_on_device(gp.ctx, 0, [1, 1], records, stream) == K.TC_ERR_DUP
        assert K.tc_stage_on_device(gp.ctx, 0, [80], records, stream) == K.TC_ERR_RANGE
        assert K.tc_stage_on_device(gp.ctx, 2, [1], records, stream) == K.TC_ERR_INVAL
        assert K.tc_stage_on_device(gp.ctx, 0, [1], np.zeros(rec, dtype=np.uint8), stream) == K.TC_ERR_INVAL
        rc, st = K.tc_stats(gp.ctx)
        assert st.ops_in_flight == 0 and st.gpu_blocks_free == shape.num_blocks
    finally:
        gp.close()
