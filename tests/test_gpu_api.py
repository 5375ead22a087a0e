"""GPU tests of the C ABI around the copies: validation, bookkeeping with real transfers in
flight, batches, the pinned arena, partial uploads and shared prefix blocks.  Data is always
compared with the oracle; ids and counters with the oracle's bookkeeping model."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_18586_amd as K
import tc_workloads as W
from harness import DEV, GpuPool, pinned_bytes

pytestmark = pytest.mark.gpu

SMALL = W.PoolShape("small", 4, 2, 64, 16, 2, 64, 0, "normal")      # 4 KiB pages, 32 KiB records


def _stats(gp):
    rc, st = K.tc_stats(gp.ctx)
    assert rc == 0
    return st


def _staged_launches(n, rec, num_blocks, overlap_kernels=0):
    """How many copy launches a staged transfer of n records takes (4 GiB slots; with overlap_kernels a short
    first chunk of 32 MiB for transfers that have something to overlap), from the planning model."""
    from oracle import transfer_plan as T
    return len(T.plan_staged(n, min((4096 << 20) // rec, num_blocks), False, max(1, (32 << 20) // rec), overlap_kernels)[0])


def test_validation_errors_have_no_effect():
    rng = W.rng_for(0, salt=11)
    pool_h = W.make_pool_host(SMALL, rng)
    gp = GpuPool(SMALL, pool_h, None)
    try:
        rec = gp.rec
        host = pinned_bytes(8 * rec)
        host.fill_(0x5A)
        table = torch.full((8,), -9, dtype=torch.int32, device=DEV)
        torch.cuda.synchronize()       # torch wrote this on its own stream; the library's calls run on others
        K.check(K.tc_alloc_at(gp.ctx, [3, 4, 5, 6]))
        K.check(K.tc_ref(gp.ctx, [6]))
        before = _stats(gp).as_dict()
        cases = [
            ([3, 64], K.TC_ERR_RANGE), ([-1, 3], K.TC_ERR_RANGE), ([3, 4, 3], K.TC_ERR_DUP),
            ([3, 7], K.TC_ERR_INVAL), ([3, 6], K.TC_ERR_SHARED),
        ]
        for ids, code in cases:
            assert K.tc_offload(gp.ctx, ids, host) == code
            assert K.tc_upload(gp.ctx, host, ids, table) == code
            assert K.tc_offload_batch(gp.ctx, [([5], host), (ids, host.data_ptr() + rec)]) == code
        pageable = np.zeros(4 * rec, dtype=np.uint8)
        assert K.tc_offload(gp.ctx, [3, 4], pageable) == K.TC_ERR_NOT_PINNED
        assert K.tc_upload(gp.ctx, pageable, [3, 4], table) == K.TC_ERR_NOT_PINNED
        assert K.tc_upload(gp.ctx, host, [3, 4], np.zeros(2, dtype=np.int32)) == K.TC_ERR_NOT_PINNED  # table not device
        assert K.tc_offload(gp.ctx, [3], None) == K.TC_ERR_INVAL
        assert K.tc_free(gp.ctx, [7]) == K.TC_ERR_INVAL
        assert K.tc_free(gp.ctx, [64]) == K.TC_ERR_RANGE
        assert K.tc_ref(gp.ctx, [7]) == K.TC_ERR_INVAL
        assert K.tc_alloc(gp.ctx, 61)[0] == K.TC_ERR_NOMEM
        assert K.tc_alloc_at(gp.ctx, [10, 3]) == K.TC_ERR_NOMEM
        torch.cuda.synchronize()
        assert _stats(gp).as_dict() == before
        assert (host.numpy() == 0x5A).all()
        assert np.array_equal(gp.pool_to_host(), pool_h)
        assert (table.cpu().numpy() == -9).all()
    finally:
        gp.close()


def test_create_rejects_bad_descriptions():
    pool = torch.zeros(1 << 20, dtype=torch.uint8, device=DEV)
    host = np.zeros(1 << 20, dtype=np.uint8)
    assert K.tc_create(pool, None, 0, 8, 4096, 16)[0] == K.TC_ERR_INVAL           # no layers
    assert K.tc_create(pool, None, 2, 8, 4100, 16)[0] == K.TC_ERR_INVAL           # page not a 16-B multiple
    assert K.tc_create(pool, None, 2, 8, 4096, 16, 3)[0] == K.TC_ERR_INVAL        # scales_per_block not in {0,1,P}
    assert K.tc_create(pool, None, 2, 8, 4096, 16, 4)[0] == K.TC_ERR_INVAL        # scales announced, none given
    assert K.tc_create(pool.data_ptr() + 16, None, 2, 8, 4096, 16)[0] == K.TC_ERR_INVAL   # misaligned
    assert K.tc_create(pinned_bytes(1 << 20), None, 2, 8, 4096, 16)[0] == K.TC_ERR_NOT_PINNED   # pool is host memory


def test_pending_free_blocks_are_not_handed_out_while_the_copy_runs():
    # 8B-shaped pages; 256 of 300 blocks move (512 MiB, ~10 ms on the link)
    shape = W.CONFIGS[1].with_blocks(300)
    gp = GpuPool(shape, seed=5)
    model = oracle.OracleBlockPool(shape.num_blocks)
    try:
        n = 256
        rc, ids = K.tc_alloc(gp.ctx, 300)
        assert rc == 0 and list(ids) == model.alloc(300)
        move = ids[:n]
        host = pinned_bytes(n * gp.rec)
        stream = torch.cuda.Stream()
        K.check(K.tc_offload(gp.ctx, move, host, stream))
        model.begin_op(list(move))
        K.check(K.tc_free(gp.ctx, move))
        model.free(list(move))
        st = _stats(gp)
        assert (st.gpu_blocks_pending_free, st.gpu_blocks_free, st.gpu_blocks_used) == (n, 0, 44)
        assert (model.n_pending(), model.n_free(), model.n_used()) == (n, 0, 44)
        # the copy was enqueued microseconds ago and takes milliseconds
        assert K.tc_alloc(gp.ctx, 1)[0] == K.TC_ERR_NOMEM
        assert K.tc_alloc_at(gp.ctx, move[:1]) == K.TC_ERR_NOMEM
        assert K.tc_alloc_prefer(gp.ctx, move[:1])[0] == K.TC_ERR_NOMEM
        stream.synchronize()
        model.retire_all()
        # the finished transfer is retired by the call itself, so the original blocks can be claimed again
        want = [int(move[3]), -1, int(ids[299]), int(move[0])]
        rc, got = K.tc_alloc_prefer(gp.ctx, want)
        assert rc == 0 and list(got) == model.alloc_prefer(want) and got[0] == move[3] and got[3] == move[0]
        K.check(K.tc_free(gp.ctx, got))
        model.free(list(got))
        rc, again = K.tc_alloc(gp.ctx, n)      # retires the finished transfer itself
        assert rc == 0 and list(again) == model.alloc(n)
        assert _stats(gp).gpu_blocks_pending_free == 0
    finally:
        gp.close()


@pytest.mark.parametrize("direct,tail,overlap_kernels", [(3, 1, 0), (1, 0, 0), (3, 2, 0), (3, 4, 0), (0, 0, 0), (3, 1, 1), (3, 4, 1)],
                         ids=["staged", "direct", "staged-tail2", "staged-tail4", "auto", "staged-overlapped", "staged-tail4-overlapped"])
def test_batch_of_agents_shares_chunks(direct, tail, overlap_kernels):
    rng = W.rng_for(2, salt=3)
    shape = W.CONFIGS[1].with_blocks(128)
    L, NB, pb, P = shape.num_layers, shape.num_blocks, shape.page_bytes, shape.planes
    pool_h = W.make_pool_host(shape, rng)
    sizes = [5, 0, 17, 1, 9, 3]
    perm = W.pick_ids(rng, NB, 2 * sum(sizes))
    src = np.split(perm[: sum(sizes)], np.cumsum(sizes)[:-1])
    dst = np.split(perm[sum(sizes):], np.cumsum(sizes)[:-1])
    # staging: 3 slots of 4 records, so chunks straddle agents
    gp = GpuPool(shape, pool_h, None, staging_bytes=3 * 4 * 2 * 1024 * 1024, staging_slots=3,
                 host_arena_bytes=40 * 2 * 1024 * 1024, direct_offload=direct, direct_upload=direct,
                 host_tail_div=tail,      # chunk tails inside one agent's buffer skip staging, the others do not
                 overlap_kernels=overlap_kernels)
    try:
        rec = gp.rec
        bufs = []
        for s in sizes:
            rc, addr = K.tc_host_alloc(gp.ctx, s)
            assert rc == 0 and (addr is None) == (s == 0)
            bufs.append(addr)
        assert _stats(gp).host_slots_used == sum(sizes)
        assert K.tc_host_alloc(gp.ctx, 6)[0] == K.TC_ERR_HOST_NOMEM     # 40 slots, 35 taken
        stream = torch.cuda.Stream()
        K.check(K.tc_alloc_at(gp.ctx, perm[: sum(sizes)]))
        K.check(K.tc_offload_batch(gp.ctx, list(zip(src, bufs)), stream))
        K.check(K.tc_free(gp.ctx, perm[: sum(sizes)]))
        K.check(K.tc_sync(gp.ctx))
        wants = []
        for ids, addr, s in zip(src, bufs, sizes):
            want = np.empty(max(s * rec, 1), dtype=np.uint8)
            oracle.offload(pool_h, None, L, NB, pb, 0, ids, want)
            wants.append(want)
            if s:
                got = np.ctypeslib.as_array((np.ctypeslib.ctypes.c_uint8 * (s * rec)).from_address(addr))
                assert np.array_equal(got, want[: s * rec])
        # upload the whole batch into other blocks, one table row per agent
        tables = torch.full((len(sizes), 20), -1, dtype=torch.int32, device=DEV)
        torch.cuda.synchronize()       # torch wrote this on its own stream; the library's calls run on others
        tables_h = np.full((len(sizes), 20), -1, dtype=np.int32)
        K.check(K.tc_alloc_at(gp.ctx, perm[sum(sizes):]))
        K.check(K.tc_upload_batch(gp.ctx, [(dst[i], bufs[i], tables[i]) for i in range(len(sizes))], stream))
        for i, s in enumerate(sizes):
            oracle.upload(wants[i], L, NB, pb, 0, dst[i], pool_h, None, tables_h[i])
            K.check(K.tc_host_free(gp.ctx, bufs[i]))      # while the upload may still be reading it
        stream.synchronize()
        assert np.array_equal(gp.pool_to_host(), pool_h)
        assert np.array_equal(tables.cpu().numpy(), tables_h)
        K.check(K.tc_sync(gp.ctx))
        st = _stats(gp)
        assert st.host_slots_used == 0 and st.n_offloads == 1 and st.n_uploads == 1
        assert st.blocks_offloaded == sum(sizes) and st.bytes_uploaded == sum(sizes) * rec
    finally:
        gp.close()


def test_partial_uploads_restore_an_agent_piecewise():
    """Destination blocks arrive in pieces (gradual reservation): records [a, b) of the host buffer
    are uploaded as they get their blocks; the result equals one whole upload."""
    rng = W.rng_for(3, salt=4)
    shape = SMALL
    L, NB, pb = shape.num_layers, shape.num_blocks, shape.page_bytes
    pool_h = W.make_pool_host(shape, rng)
    n = 13
    ids = W.pick_ids(rng, NB, n)
    new_ids = W.pick_ids(rng, NB, n, exclude=ids)
    gp = GpuPool(shape, pool_h, None)
    try:
        rec = gp.rec
        host = pinned_bytes(n * rec)
        K.check(K.tc_alloc_at(gp.ctx, ids))
        K.check(K.tc_offload(gp.ctx, ids, host))
        K.check(K.tc_free(gp.ctx, ids))
        K.check(K.tc_sync(gp.ctx))
        want = np.empty(n * rec, dtype=np.uint8)
        oracle.offload(pool_h, None, L, NB, pb, 0, ids, want)
        table = torch.full((n,), -1, dtype=torch.int32, device=DEV)
        torch.cuda.synchronize()       # torch wrote this on its own stream; the library's calls run on others
        table_h = np.full(n, -1, dtype=np.int32)
        oracle.upload(want, L, NB, pb, 0, new_ids, pool_h, None, table_h)
        done = 0
        for piece in (7, 3, 2, 1):      # ceil(deficit / 2) each step
            part = new_ids[done: done + piece]
            K.check(K.tc_alloc_at(gp.ctx, part))
            K.check(K.tc_upload(gp.ctx, host.data_ptr() + done * rec, part, table.data_ptr() + 4 * done))
            done += piece
        torch.cuda.synchronize()
        assert np.array_equal(gp.pool_to_host(), pool_h)
        assert np.array_equal(table.cpu().numpy(), table_h)
    finally:
        gp.close()


def test_shared_prefix_blocks_stay_put():
    rng = W.rng_for(4, salt=5)
    shape = W.PoolShape("fp8-small", 3, 2, 32, 8, 1, 80, 6, "fp8")
    L, NB, pb, S = shape.num_layers, shape.num_blocks, shape.page_bytes, shape.scales_per_block
    pool_h = W.make_pool_host(shape, rng)
    scales_h = W.make_scales_host(shape, rng)
    gp = GpuPool(shape, pool_h, scales_h)
    model = oracle.OracleBlockPool(NB)
    try:
        rc, prefix = K.tc_alloc(gp.ctx, 4)
        assert list(prefix) == model.alloc(4)
        agents = []
        for a in range(3):
            if a:
                K.check(K.tc_ref(gp.ctx, prefix))
                model.ref(list(prefix))
            rc, priv = K.tc_alloc(gp.ctx, 5 + a)
            assert list(priv) == model.alloc(5 + a)
            agents.append(np.concatenate([prefix, priv]))
        assert _stats(gp).gpu_blocks_shared == 4
        row = agents[1]
        host = pinned_bytes(len(row) * gp.rec)
        assert K.tc_offload(gp.ctx, row, host) == K.TC_ERR_SHARED
        rc, private = K.tc_filter_private(gp.ctx, row)
        assert rc == 0 and list(private) == model.filter_private(list(row)) == list(row[4:])
        K.check(K.tc_offload(gp.ctx, private, host))
        K.check(K.tc_free(gp.ctx, private))
        K.check(K.tc_sync(gp.ctx))
        want = np.empty(len(private) * gp.rec, dtype=np.uint8)
        oracle.offload(pool_h, scales_h, L, NB, pb, S, private, want)
        assert np.array_equal(host.numpy()[: want.size], want)
        model.free(list(private))
        # back into fresh blocks; the table's prefix entries are never written
        rc, fresh = K.tc_alloc(gp.ctx, len(private))
        assert list(fresh) == model.alloc(len(private))
        table = torch.from_numpy(row.copy()).to(DEV)
        table_h = row.copy()
        oracle.upload(want, L, NB, pb, S, fresh, pool_h, scales_h, table_h[4:])
        K.check(K.tc_upload(gp.ctx, host, fresh, table.data_ptr() + 4 * 4))
        torch.cuda.synchronize()
        assert np.array_equal(table.cpu().numpy(), table_h) and list(table_h[:4]) == list(prefix)
        assert np.array_equal(gp.pool_to_host(), pool_h)
        assert np.array_equal(gp.scales_all_to_host(), scales_h)
    finally:
        gp.close()


def test_calibrated_cost_model_predicts_a_transfer_and_leaves_the_pool_alone():
    """Eq. 2 closed on this platform: tc_calibrate fits T(N) from its own transfers and leaves the pool as it
    was; the per-block constants are those of a host link (between 40 and 70 GB/s); the estimate for a size it
    did not measure agrees with transfers timed here by events on the stream to within 15 % (a bound that
    catches a wrong unit or a dropped term of Eq. 2, not the link's run-to-run noise); the gate of Alg. 1
    then uses it."""
    shape = W.CONFIGS[1].with_blocks(400)
    gp = GpuPool(shape, seed=9, host_arena_bytes=330 * 2 * 1024 * 1024)
    try:
        before = gp.page_checksums(weighted=True)
        stream = torch.cuda.Stream()
        rc, model = K.tc_calibrate(gp.ctx, [32, 64, 128, 256], 3, stream)
        assert rc == 0
        assert torch.equal(gp.page_checksums(weighted=True), before), "calibration must not change the pool"
        st = _stats(gp)
        assert st.gpu_blocks_free == 400 and st.host_slots_used == 0
        # 2 MiB per block at 40 .. 70 GB/s is 0.030 .. 0.052 ms per block and direction
        assert 0.030 < model.off_b_ms_per_block < 0.052 and 0.030 < model.up_b_ms_per_block < 0.052
        assert abs(model.off_a_ms) < 0.5 and abs(model.up_a_ms) < 0.5
        # linear in the number of blocks (Eq. 2), increasing, and additive over the two directions
        e = [K.tc_estimate_transfer_ms(model, k) for k in (0, 100, 200, 300)]
        assert e[1] < e[2] < e[3] and abs((e[3] - e[2]) - (e[2] - e[1])) < 1e-9
        assert abs(e[0] - (model.off_a_ms + model.up_a_ms)) < 1e-12
        n = 192
        rc, ids = K.tc_alloc(gp.ctx, n)
        rc, host = K.tc_host_alloc(gp.ctx, n)
        ts = []
        for _ in range(6):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            K.check(K.tc_offload(gp.ctx, ids, host, stream))
            K.check(K.tc_upload(gp.ctx, host, ids, None, stream))
            e1.record(stream)
            stream.synchronize()
            ts.append(e0.elapsed_time(e1))
        measured = float(np.median(ts[1:]))
        predicted = K.tc_estimate_transfer_ms(model, n)
        assert abs(predicted - measured) / measured < 0.15, (predicted, measured)
        # a 2 s tool call leaves a window; a 10 ms one does not cover the round trip of 192 blocks
        assert K.tc_should_offload(model, n, 2000.0, 5.0, [(500, 10.0), (100, 4000.0)]) == (1, 1)
        assert K.tc_should_offload(model, n, 10.0, 5.0, [(100, 1.0)]) == (0, -1)
        assert K.tc_calibrate(gp.ctx, [32, 500], 1, stream)[0] == K.TC_ERR_NOMEM
    finally:
        gp.close()


@pytest.mark.parametrize("overlap_kernels", [0, 1], ids=["in-line", "kernels-on-the-engines-stream"])
def test_whole_pool_moves_in_one_call_over_many_chunks(overlap_kernels):
    """Maximum size: every block of the pool is a source, then a destination (reversed order)."""
    rng = W.rng_for(1, salt=31)
    shape = W.CONFIGS[1].with_blocks(160)                       # 320 MiB pool
    L, NB, pb = shape.num_layers, shape.num_blocks, shape.page_bytes
    pool_h = W.make_pool_host(shape, rng)
    ids = rng.permutation(NB).astype(np.int32)
    gp = GpuPool(shape, pool_h, None, staging_bytes=2 * 7 * 2 * 1024 * 1024, staging_slots=2,   # 7 records per chunk
                 direct_offload=K.TC_PATH_STAGED, direct_upload=K.TC_PATH_STAGED, overlap_kernels=overlap_kernels)
    try:
        host = pinned_bytes(NB * gp.rec)
        rc, got = K.tc_alloc(gp.ctx, NB)
        assert rc == 0 and K.tc_alloc(gp.ctx, 1)[0] == K.TC_ERR_NOMEM
        K.check(K.tc_offload(gp.ctx, ids, host))
        want = np.empty(NB * gp.rec, dtype=np.uint8)
        oracle.offload(pool_h, None, L, NB, pb, 0, ids, want)
        torch.cuda.synchronize()
        assert np.array_equal(host.numpy(), want)
        new_ids = ids[::-1].copy()
        table = torch.full((NB,), -1, dtype=torch.int32, device=DEV)
        torch.cuda.synchronize()       # torch wrote this on its own stream; the library's calls run on others
        table_h = np.full(NB, -1, dtype=np.int32)
        oracle.upload(want, L, NB, pb, 0, new_ids, pool_h, None, table_h)
        K.check(K.tc_upload(gp.ctx, host, new_ids, table))
        torch.cuda.synchronize()
        assert np.array_equal(gp.pool_to_host(), pool_h)
        assert np.array_equal(table.cpu().numpy(), table_h)
        # one id too many can only be a repeat
        assert K.tc_offload(gp.ctx, np.concatenate([ids, ids[:1]]), host) == K.TC_ERR_DUP
    finally:
        gp.close()


@pytest.mark.parametrize("overlap_kernels", [0, 1], ids=["in-line", "kernels-on-the-engines-stream"])
def test_two_streams_share_one_staging_slot(overlap_kernels):
    """An offload and an upload of different agents issued back to back on different streams must not
    trample each other's chunk in the single staging slot."""
    rng = W.rng_for(1, salt=32)
    shape = W.CONFIGS[1].with_blocks(128)
    L, NB, pb = shape.num_layers, shape.num_blocks, shape.page_bytes
    pool_h = W.make_pool_host(shape, rng)
    perm = W.pick_ids(rng, NB, 90)
    a_src, b_src, b_dst = perm[:30], perm[30:60], perm[60:90]
    gp = GpuPool(shape, pool_h, None, staging_bytes=4 * 2 * 1024 * 1024, staging_slots=1,       # 4 records per chunk
                 direct_offload=K.TC_PATH_STAGED, direct_upload=K.TC_PATH_STAGED, overlap_kernels=overlap_kernels)
    try:
        rec = gp.rec
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        K.check(K.tc_alloc_at(gp.ctx, perm))
        host_a, host_b = pinned_bytes(30 * rec), pinned_bytes(30 * rec)
        K.check(K.tc_offload(gp.ctx, b_src, host_b, s1))
        s1.synchronize()
        want_b = np.empty(30 * rec, dtype=np.uint8)
        oracle.offload(pool_h, None, L, NB, pb, 0, b_src, want_b)
        assert np.array_equal(host_b.numpy(), want_b)
        want_a = np.empty(30 * rec, dtype=np.uint8)
        oracle.offload(pool_h, None, L, NB, pb, 0, a_src, want_a)       # a_src is not touched by b's upload
        for _ in range(3):
            host_a.fill_(0)
            K.check(K.tc_offload(gp.ctx, a_src, host_a, s1))            # chunks of the two transfers
            K.check(K.tc_upload(gp.ctx, host_b, b_dst, None, s2))       # interleave in the one slot
            torch.cuda.synchronize()
            assert np.array_equal(host_a.numpy(), want_a)
        oracle.upload(want_b, L, NB, pb, 0, b_dst, pool_h, None, None)
        assert np.array_equal(gp.pool_to_host(), pool_h)
    finally:
        gp.close()


@pytest.mark.parametrize("overlap_kernels", [0, 1], ids=["in-line", "kernels-on-the-engines-stream"])
def test_calls_from_several_host_threads(overlap_kernels):
    """The context serialises callers: four threads, each with its own stream and agent."""
    import threading
    rng = W.rng_for(1, salt=33)
    shape = W.CONFIGS[1].with_blocks(256)
    L, NB, pb = shape.num_layers, shape.num_blocks, shape.page_bytes
    pool_h = W.make_pool_host(shape, rng)
    perm = W.pick_ids(rng, NB, 4 * 2 * 24)
    gp = GpuPool(shape, pool_h, None, staging_bytes=2 * 8 * 2 * 1024 * 1024, staging_slots=2,
                 host_arena_bytes=100 * 2 * 1024 * 1024, direct_offload=K.TC_PATH_STAGED, direct_upload=K.TC_PATH_STAGED,
                 overlap_kernels=overlap_kernels)
    try:
        rec = gp.rec
        K.check(K.tc_alloc_at(gp.ctx, perm))
        errors, bufs = [], [None] * 4
        tables = torch.full((4, 24), -1, dtype=torch.int32, device=DEV)
        torch.cuda.synchronize()       # torch wrote this on its own stream; the library's calls run on others

        def worker(k):
            try:
                torch.cuda.set_device(0)
                stream = torch.cuda.Stream()
                src, dst = perm[48 * k: 48 * k + 24], perm[48 * k + 24: 48 * k + 48]
                rc, buf = K.tc_host_alloc(gp.ctx, 24)
                K.check(rc)
                bufs[k] = buf
                for _ in range(3):
                    K.check(K.tc_offload(gp.ctx, src, buf, stream))
                    K.check(K.tc_upload(gp.ctx, buf, dst, tables[k], stream))
                    K.check(K.tc_poll(gp.ctx))
                stream.synchronize()
            except Exception as e:      # noqa: BLE001
                errors.append(e)

        threads = [threading.Thread(target=worker, args=(k,)) for k in range(4)]
        for t in threads:
            t.start()
        for t in threads:
            t.join()
        assert not errors, errors
        K.check(K.tc_sync(gp.ctx))
        for k in range(4):
            src, dst = perm[48 * k: 48 * k + 24], perm[48 * k + 24: 48 * k + 48]
            want = np.empty(24 * rec, dtype=np.uint8)
            oracle.offload(pool_h, None, L, NB, pb, 0, src, want)
            from harness import host_view
            assert np.array_equal(host_view(bufs[k], 24 * rec), want)
            oracle.upload(want, L, NB, pb, 0, dst, pool_h, None, None)
            assert np.array_equal(tables[k].cpu().numpy(), dst)
        assert np.array_equal(gp.pool_to_host(), pool_h)
        assert _stats(gp).ops_in_flight == 0
    finally:
        gp.close()


def test_auto_mode_goes_direct_only_while_an_upload_is_in_flight():
    """direct_offload = 2: an offload issued while an upload of the same context is in flight is written
    by the gather kernel straight into pinned memory (so the two directions overlap on the link);
    otherwise it takes the staged path.  Same bytes either way."""
    rng = W.rng_for(1, salt=34)
    shape = W.CONFIGS[1].with_blocks(512)
    L, NB, pb = shape.num_layers, shape.num_blocks, shape.page_bytes
    gp = GpuPool(shape, seed=34, direct_offload=K.TC_PATH_DIRECT_IF_DUPLEX, direct_upload=K.TC_PATH_STAGED)
    mirror = None
    try:
        from harness import SparseMirror
        rec = gp.rec
        perm = W.pick_ids(rng, NB, 3 * 128)
        a, b, c = perm[:128], perm[128:256], perm[256:]
        K.check(K.tc_alloc_at(gp.ctx, perm))
        K.check(K.tc_set_profiling(gp.ctx, 1))
        mirror = SparseMirror(gp, perm)
        host_a, host_b = pinned_bytes(128 * rec), pinned_bytes(128 * rec)
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        K.check(K.tc_offload(gp.ctx, b, host_b, s1))                 # nothing in flight: staged
        K.check(K.tc_sync(gp.ctx))
        st = _stats(gp)
        g = _staged_launches(128, rec, NB)
        assert g == 1 and st.direct_launches == 0 and st.gather_launches == g and st.transfers_overlapped == 0
        K.check(K.tc_upload(gp.ctx, host_b, c, None, s2))            # 256 MiB coming in ...
        K.check(K.tc_offload(gp.ctx, a, host_a, s1))                 # ... while 256 MiB go out: direct
        K.check(K.tc_sync(gp.ctx))
        st = _stats(gp)
        assert st.direct_launches == 1 and st.direct_bytes == 128 * rec and st.gather_launches == g
        want = np.empty(128 * rec, dtype=np.uint8)
        oracle.offload(mirror.pool, None, L, NB, pb, 0, a, want)
        assert np.array_equal(host_a.numpy(), want)
        oracle.offload(mirror.pool, None, L, NB, pb, 0, b, want)
        assert np.array_equal(host_b.numpy(), want)
        oracle.upload(want, L, NB, pb, 0, c, mirror.pool, None, None)
        assert np.array_equal(gp.blocks_to_host(c), mirror.blocks(c))
    finally:
        if mirror:
            mirror.close()
        gp.close()


def test_transfers_on_different_streams_respect_block_and_buffer_hazards():
    """An upload into blocks that an offload on another stream is still reading, and an upload from an
    arena buffer that an offload on another stream is still writing, must each wait for that offload."""
    shape = W.CONFIGS[1].with_blocks(600)
    L, NB, pb = shape.num_layers, shape.num_blocks, shape.page_bytes
    rng = W.rng_for(1, salt=35)
    gp = GpuPool(shape, seed=35, host_arena_bytes=520 * 2 * 1024 * 1024)
    mirror = None
    try:
        from harness import SparseMirror, host_view
        rec = gp.rec
        n = 256                                            # 512 MiB: each transfer takes ~10 ms
        perm = W.pick_ids(rng, NB, 2 * n)
        a, b = perm[:n], perm[n:]
        K.check(K.tc_alloc_at(gp.ctx, perm))
        mirror = SparseMirror(gp, perm)
        rc, buf_a = K.tc_host_alloc(gp.ctx, n)
        rc, buf_b = K.tc_host_alloc(gp.ctx, n)
        s1, s2, s3 = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
        want_a = np.empty(n * rec, dtype=np.uint8)
        want_b = np.empty(n * rec, dtype=np.uint8)
        oracle.offload(mirror.pool, None, L, NB, pb, 0, a, want_a)
        oracle.offload(mirror.pool, None, L, NB, pb, 0, b, want_b)
        K.check(K.tc_offload(gp.ctx, b, buf_b, s1))
        K.check(K.tc_sync(gp.ctx))
        for _ in range(3):
            K.check(K.tc_offload(gp.ctx, a, buf_a, s1))        # reads blocks a, writes buf_a (s1)
            K.check(K.tc_upload(gp.ctx, buf_b, a, None, s2))   # overwrites blocks a with b's bytes (s2): must wait
            K.check(K.tc_upload(gp.ctx, buf_a, b, None, s3))   # reads buf_a (s3): must wait for the offload too
            K.check(K.tc_sync(gp.ctx))
            assert np.array_equal(host_view(buf_a, n * rec), want_a), "the upload overtook the offload's reads"
            assert np.array_equal(gp.blocks_to_host(b), mirror.blocks(a)), "the upload read buf_a before it was written"
            assert np.array_equal(gp.blocks_to_host(a), mirror.blocks(b))
            # put the pool back the way the mirror has it
            K.check(K.tc_upload(gp.ctx, buf_a, a, None, s1))
            K.check(K.tc_upload(gp.ctx, buf_b, b, None, s1))
            K.check(K.tc_sync(gp.ctx))
    finally:
        if mirror:
            mirror.close()
        gp.close()


def test_thousands_of_small_transfers_wrap_the_id_ring():
    """3 000 one- and two-block transfers on one stream with no host synchronisation in between: the id
    rings (1 024 entries here) wrap several times and the calls have to wait for old transfers to retire.
    The KV contents rotate through the pool; the end state must equal the oracle's."""
    rng = W.rng_for(0, salt=41)
    pool_host = W.make_pool_host(SMALL, rng)
    mirror = pool_host.copy()
    gp = GpuPool(SMALL, pool_host=pool_host, host_arena_bytes=8 * 2 * SMALL.num_layers * SMALL.page_bytes)
    L, NB, pb = gp.L, gp.NB, gp.pb
    try:
        rc, ids = K.tc_alloc(gp.ctx, NB)
        assert rc == 0
        order = rng.permutation(NB).astype(np.int32)
        bufs = [K.tc_host_alloc(gp.ctx, 2)[1] for _ in range(4)]
        host_o = np.zeros(2 * gp.rec, dtype=np.uint8)
        stream = torch.cuda.Stream()
        table = torch.full((4,), -1, dtype=torch.int32, device=DEV)
        torch.cuda.synchronize()       # torch wrote this on its own stream; the library's calls run on others
        for i in range(1500):
            n = 1 + i % 2
            src = np.array([order[(i + k) % NB] for k in range(n)], dtype=np.int32)
            dst = np.array([order[(i + 7 + 3 * k) % NB] for k in range(n)], dtype=np.int32)
            buf = bufs[i % 4]
            K.check(K.tc_offload(gp.ctx, src, buf, stream))
            K.check(K.tc_upload(gp.ctx, buf, dst, table, stream))
            oracle.offload(mirror, None, L, NB, pb, 0, src, host_o[:n * gp.rec])
            oracle.upload(host_o[:n * gp.rec], L, NB, pb, 0, dst, mirror, None)
        K.check(K.tc_sync(gp.ctx))
        st = _stats(gp)
        assert st.n_offloads == st.n_uploads == 1500 and st.ops_in_flight == 0
        assert np.array_equal(gp.pool_to_host(), mirror)
        assert table.cpu().numpy()[:2].tolist() == dst.tolist()
    finally:
        gp.close()


def test_the_librarys_own_choice_of_path():
    """Default options: an upload goes through the scatter kernel that reads pinned memory itself, an offload
    through device staging and DMA, unless an upload is in flight: then it goes direct as well.  With
    auto_direct_bytes set, offloads below it go direct, the threshold itself does not.  Same bytes whichever way."""
    rng = W.rng_for(1, salt=36)
    shape = W.CONFIGS[1].with_blocks(400)
    L, NB, pb = shape.num_layers, shape.num_blocks, shape.page_bytes
    mirror = None
    for auto_bytes in (0, 128 << 20):
        gp = GpuPool(shape, seed=36, auto_direct_bytes=auto_bytes)
        try:
            from harness import SparseMirror
            rec = gp.rec
            perm = W.pick_ids(rng, NB, 63 + 64 + 100 + 100)
            small, edge, big, dst = perm[:63], perm[63:127], perm[127:227], perm[227:]
            K.check(K.tc_alloc_at(gp.ctx, perm))
            K.check(K.tc_set_profiling(gp.ctx, 1))
            mirror = SparseMirror(gp, perm)
            bufs = {k: pinned_bytes(len(v) * rec) for k, v in (("small", small), ("edge", edge), ("big", big))}
            s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()

            def counts():
                K.check(K.tc_sync(gp.ctx))
                st = _stats(gp)
                return st.direct_launches, st.gather_launches, st.scatter_launches

            K.check(K.tc_offload(gp.ctx, small, bufs["small"], s1))          # 126 MiB
            assert counts() == ((1, 0, 0) if auto_bytes else (0, _staged_launches(63, rec, NB), 0))
            d, g = counts()[:2]
            K.check(K.tc_offload(gp.ctx, edge, bufs["edge"], s1))            # 128 MiB, the threshold itself: staged
            g += _staged_launches(64, rec, NB)
            assert counts() == (d, g, 0)
            K.check(K.tc_upload(gp.ctx, bufs["edge"], dst[:64], None, s2))   # uploads: direct
            assert counts() == (d + 1, g, 0)
            junk = pinned_bytes(100 * rec)
            K.check(K.tc_upload(gp.ctx, junk, dst, None, s2))                # 200 MiB coming in (whatever bytes) ...
            K.check(K.tc_offload(gp.ctx, big, bufs["big"], s1))              # ... while 200 MiB go out: direct
            assert counts() == (d + 3, g, 0)
            for ids, key in ((small, "small"), (edge, "edge"), (big, "big")):
                want = np.empty(len(ids) * rec, dtype=np.uint8)
                oracle.offload(mirror.pool, None, L, NB, pb, 0, ids, want)
                assert np.array_equal(bufs[key].numpy(), want), key
        finally:
            if mirror:
                mirror.close()
                mirror = None
            gp.close()


def test_an_agent_of_4_GiB_is_one_launch_and_one_dma_by_default():
    """The default staging slot holds 4 GiB of records: the largest agent of the config-4 trace (1 006 blocks of
    4 MiB) goes out and comes back as one chunk (a DMA enqueued behind a running one is what the runtime sometimes
    carries out at half rate; a single DMA never was)."""
    shape = W.CONFIGS[3].with_blocks(1100)
    gp = GpuPool(shape, seed=41, direct_offload=K.TC_PATH_STAGED, direct_upload=K.TC_PATH_STAGED)
    try:
        n, rec = 1006, gp.rec
        rng = W.rng_for(3, salt=41)
        ids = W.pick_ids(rng, shape.num_blocks, n)
        K.check(K.tc_alloc_at(gp.ctx, ids))
        K.check(K.tc_set_profiling(gp.ctx, 1))
        host = pinned_bytes(n * rec)
        stream = torch.cuda.Stream()
        sig = gp.block_checksums(ids)
        K.check(K.tc_offload(gp.ctx, ids, host, stream))
        K.check(K.tc_sync(gp.ctx))
        # a few records against the oracle's definition, page by page (the whole agent is compared in the config-4 test)
        P, pb = shape.planes, shape.page_bytes
        pool_v = gp.pool.view(P, shape.num_blocks, pb)
        for j in (0, 1, 517, n - 1):
            want = pool_v[:, int(ids[j]), :].reshape(-1).cpu()
            assert torch.equal(host[j * rec: j * rec + P * pb], want)
        K.check(K.tc_upload(gp.ctx, host, ids, None, stream))
        K.check(K.tc_sync(gp.ctx))
        assert torch.equal(gp.block_checksums(ids), sig)
        st = _stats(gp)
        assert (st.gather_launches, st.d2h_copies, st.h2d_copies, st.scatter_launches) == (1, 1, 1, 1)
        assert st.d2h_bytes == n * rec and st.transfers_overlapped == 0
    finally:
        gp.close()


def test_default_staging_shrinks_where_device_memory_is_short():
    """With less device memory free than the default ring of 2 x 4 GiB, tc_create takes a smaller ring instead of
    failing, and transfers are cut into more chunks; a ring size the caller asked for is taken literally."""
    shape = W.CONFIGS[3].with_blocks(1100)                 # 4 MiB records, 4.3 GiB pool
    gp = GpuPool(shape, seed=42, direct_offload=K.TC_PATH_STAGED, direct_upload=K.TC_PATH_STAGED)
    gp.close()                                             # (the pool's memory is known to fit; now take the rest away)
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    leave = shape.pool_bytes + (3 << 30)                   # room for the pool and about 3 GiB more: not for 8 GiB of staging
    hog = torch.empty(free - leave, dtype=torch.uint8, device=DEV)
    gp = None
    try:
        pool = W.make_pool_device(shape, 42, DEV)
        torch.cuda.synchronize()       # torch filled the pool on its own stream; the library's calls run on others
        a = (shape.num_layers, shape.num_blocks, shape.page_bytes, shape.block_size, 0)
        rc, ctx = K.tc_create(pool, None, *a, staging_bytes=8 << 30, staging_slots=2)
        assert rc == K.TC_ERR_HIP and ctx is None          # asked for: not there
        rc, ctx = K.tc_create(pool, None, *a, direct_offload=K.TC_PATH_STAGED, direct_upload=K.TC_PATH_STAGED, host_tail_div=1)
        assert rc == K.TC_OK
        try:
            n, rec = 600, K.tc_record_bytes(ctx)
            ids = W.pick_ids(W.rng_for(3, salt=42), shape.num_blocks, n)
            K.check(K.tc_alloc_at(ctx, ids))
            K.check(K.tc_set_profiling(ctx, 1))
            host = pinned_bytes(n * rec)
            stream = torch.cuda.Stream()
            K.check(K.tc_offload(ctx, ids, host, stream))
            K.check(K.tc_sync(ctx))
            st = K.tc_stats(ctx)[1]
            assert st.gather_launches >= 2 and st.d2h_bytes == n * rec      # a smaller ring: several chunks
            P, pb = shape.planes, shape.page_bytes
            pool_v = pool.view(P, shape.num_blocks, pb)
            for j in (0, 299, 300, n - 1):
                assert torch.equal(host[j * rec: j * rec + P * pb], pool_v[:, int(ids[j]), :].reshape(-1).cpu())
        finally:
            K.check(K.tc_destroy(ctx))
    finally:
        del hog
        torch.cuda.empty_cache()
