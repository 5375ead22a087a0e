"""GPU parity: tc_offload / tc_upload through the C ABI against the CPU oracle, bit for bit.

Every case feeds the same seeded inputs to both sides.  Integer / byte work: the bar is
exact equality of every host-record byte, every pool byte, every scale word and every
block-table entry.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_18586_amd as K
import tc_workloads as W
from harness import DEV, GpuPool, SparseMirror, pinned_bytes

pytestmark = pytest.mark.gpu


def _round_trip_case(shape, seed_idx, n, salt=0, same_ids=False, auto=False, **opts):
    """auto = False: the staged path (gather / scatter through device staging) unless opts name another;
    auto = True: the library's own choice of path (its default options)."""
    if not auto:
        opts.setdefault("direct_offload", K.TC_PATH_STAGED)
        opts.setdefault("direct_upload", K.TC_PATH_STAGED)
    rng = W.rng_for(seed_idx, salt)
    L, NB, pb, S, P = shape.num_layers, shape.num_blocks, shape.page_bytes, shape.scales_per_block, shape.planes
    pool_h = W.make_pool_host(shape, rng)
    scales_h = W.make_scales_host(shape, rng)
    ids = W.pick_ids(rng, NB, n)
    new_ids = ids.copy() if same_ids else W.pick_ids(rng, NB, n, exclude=ids)
    rec = oracle.record_bytes(L, pb, S)

    # ---- oracle
    want_host = np.empty(max(n * rec, 1), dtype=np.uint8)
    oracle.offload(pool_h, scales_h, L, NB, pb, S, ids, want_host)

    # ---- GPU
    gp = GpuPool(shape, pool_h, scales_h, **opts)
    try:
        stream = torch.cuda.Stream()
        host = pinned_bytes(n * rec + 512)
        host.fill_(0xA5)
        K.check(K.tc_alloc_at(gp.ctx, ids))
        K.check(K.tc_offload(gp.ctx, ids, host, stream))
        K.check(K.tc_free(gp.ctx, ids))          # released right after the copy is issued
        rc, st = K.tc_stats(gp.ctx)
        assert st.gpu_blocks_free + st.gpu_blocks_used + st.gpu_blocks_pending_free == NB
        K.check(K.tc_sync(gp.ctx))
        got = host.numpy()
        assert np.array_equal(got[: n * rec], want_host[: n * rec]), "offload records differ from the oracle"
        assert (got[n * rec:] == 0xA5).all(), "bytes past the last record were written"
        assert np.array_equal(gp.pool_to_host(), pool_h), "offload wrote the pool"
        rc, st = K.tc_stats(gp.ctx)
        assert st.gpu_blocks_pending_free == 0 and st.gpu_blocks_free == NB

        # somebody else reuses the freed blocks: scramble them on both sides with the same bytes
        junk = rng.integers(0, 256, size=(P, n, pb), dtype=np.uint8)
        if n and not same_ids:
            pool_h.reshape(P, NB, pb)[:, ids] = junk
            gp.pool3()[:, torch.as_tensor(ids.astype(np.int64), device=DEV)] = torch.from_numpy(junk).to(DEV)
            torch.cuda.synchronize()       # torch wrote this on its own stream; the library's calls run on others

        table_h = np.full(n + 4, -1, dtype=np.int32)
        table_h[:n] = ids
        table_d = torch.from_numpy(table_h.copy()).to(DEV)
        oracle.upload(want_host, L, NB, pb, S, new_ids, pool_h, scales_h, table_h)

        K.check(K.tc_alloc_at(gp.ctx, new_ids))
        K.check(K.tc_upload(gp.ctx, host, new_ids, table_d, stream))
        stream.synchronize()
        assert np.array_equal(gp.pool_to_host(), pool_h), "pool after upload differs from the oracle"
        if S:
            assert np.array_equal(gp.scales_all_to_host(), scales_h), "scales after upload differ"
        assert np.array_equal(table_d.cpu().numpy(), table_h), "block table differs"
        K.check(K.tc_sync(gp.ctx))
    finally:
        gp.close()


@pytest.mark.parametrize("auto", [False, True], ids=["staged", "auto"])
def test_config1_tiny(auto):
    # 2 layers, 4 KV heads, head_dim 64, 16-token blocks, bf16, 256 blocks, one agent with 8 blocks
    _round_trip_case(W.CONFIGS[0], 0, 8, auto=auto)


def test_config1_tiny_same_ids():
    # the original blocks are claimed again on upload
    _round_trip_case(W.CONFIGS[0], 0, 8, salt=1, same_ids=True)


@pytest.mark.parametrize("overlap_kernels", [0, 1], ids=["in-line", "kernels-on-the-engines-stream"])
@pytest.mark.parametrize("slots", [1, 3])
def test_8b_pages_many_chunks_ragged_tail(slots, overlap_kernels):
    # 8B-shaped pages (32 KiB, 64 planes); staging slots of 5 records -> 8 chunks, the last one ragged; everything
    # in line on the caller's stream, or the copy kernels on the context's own stream under the DMAs of their
    # neighbours (with one slot: strictly taking turns)
    shape = W.CONFIGS[1].with_blocks(96)
    _round_trip_case(shape, 1, 37, salt=slots, staging_bytes=slots * 5 * 2 * 1024 * 1024, staging_slots=slots,
                     overlap_kernels=overlap_kernels)


@pytest.mark.parametrize("div,slots", [(2, 1), (4, 2), (5, 3)])
def test_host_tail_of_every_chunk_skips_staging(div, slots):
    # chunks of 5 records: with div <= 5 the last 5 // div blocks of each full chunk go straight to / from the
    # pinned buffer inside the same launch; the ragged last chunk (2 records) is too small for div > 2
    shape = W.CONFIGS[1].with_blocks(96)
    _round_trip_case(shape, 1, 37, salt=60 + div, staging_bytes=slots * 5 * 2 * 1024 * 1024, staging_slots=slots,
                     host_tail_div=div)
    # the automatic tail: 1/64 of a chunk, so chunks of 70 records carry one record each through the launch itself
    if div == 2:
        _round_trip_case(W.CONFIGS[0].with_blocks(512), 0, 200, salt=63, staging_bytes=70 * 32 * 1024, staging_slots=1, host_tail_div=0)
    # scales and a zero pad in the tail records, capped grid, one chunk
    _round_trip_case(W.PoolShape("fp8-small", 3, 2, 32, 8, 1, 80, 6, "fp8"), 4, 23, salt=61 + div, host_tail_div=div, max_grid=5)
    # ragged tiles
    _round_trip_case(W.PoolShape("odd-ragged", 2, 5, 128, 16, 1, 40, 1, "fp8"), 4, 9, salt=62 + div, host_tail_div=div)


def test_capped_grid_strides_over_items():
    shape = W.CONFIGS[1].with_blocks(64)
    _round_trip_case(shape, 1, 21, salt=7, max_grid=37)


@pytest.mark.parametrize("shape,n", [
    (W.PoolShape("odd-small", 3, 3, 24, 4, 1, 50, 6, "fp8"), 7),        # 288-B pages, one scale per plane
    (W.PoolShape("odd-ragged", 2, 5, 128, 16, 1, 40, 1, "fp8"), 9),     # 10 KiB pages: ragged second tile; 1 scale
    (W.PoolShape("fp8-70b-pages", 80, 8, 128, 32, 1, 24, 160, "fp8"), 10),  # config-5 record: 5 MiB + 640 B + pad
    (W.PoolShape("min", 1, 1, 8, 1, 2, 10, 0, "normal"), 5),            # 16-B pages, every block is a source or a destination
])
def test_odd_shapes_and_scales(shape, n):
    _round_trip_case(shape, 4, n, salt=n)


@pytest.mark.parametrize("off,up,grid", [(1, 3, 0), (1, 1, 3), (3, 1, 0), (2, 1, 0), (0, 0, 0), (2, 0, 0)])
def test_direct_paths_move_the_same_bytes(off, up, grid):
    # the gather kernel stores straight into the pinned host buffer / the scatter kernel reads straight
    # from it (no staging, no DMA)
    opts = dict(direct_offload=off, direct_upload=up, direct_grid=grid)
    _round_trip_case(W.CONFIGS[1].with_blocks(96), 1, 37, salt=40 + off + 3 * up + grid, **opts)
    _round_trip_case(W.PoolShape("fp8-small", 3, 2, 32, 8, 1, 80, 6, "fp8"), 4, 11, salt=41, **opts)
    _round_trip_case(W.PoolShape("odd-ragged", 2, 5, 128, 16, 1, 40, 1, "fp8"), 4, 9, salt=42, **opts)
    _round_trip_case(W.CONFIGS[0], 0, 8, salt=43, **opts)


def _random_case(k):
    """A seeded random small shape + options: page sizes from 16 B to 48 KiB (whole tiles, ragged tiles,
    less than one tile), every scale layout, chunked and unchunked staging, capped grids, direct paths."""
    rng = W.rng_for(0, salt=1000 + k)
    L = int(rng.integers(1, 6))
    elem = int(rng.choice([1, 2]))
    pb = 16 * int(rng.choice([1, 2, 3, 17, 64, 255, 256, 257, 512, 640, 1024, 2048, 3072]))
    S = int(rng.choice([0, 1, 2 * L]))
    NB = int(rng.integers(4, 70))
    n = int(rng.integers(1, NB // 2 + 1))
    # a shape whose page_bytes is exactly pb: 1 token per block, 1 head, head_dim = pb / elem
    shape = W.PoolShape(f"rand{k}", L, 1, pb // elem, 1, elem, NB, S, "fp8" if elem == 1 else "normal")
    assert shape.page_bytes == pb
    rec = (2 * L * pb + 4 * S + 255) // 256 * 256
    opts = {}
    if rng.random() < 0.6:
        slots = int(rng.integers(1, 4))
        opts.update(staging_slots=slots, staging_bytes=slots * int(rng.integers(1, 5)) * rec)
    if rng.random() < 0.4:
        opts["max_grid"] = int(rng.choice([1, 2, 7, 64]))
    mode = int(rng.integers(0, 4))
    if mode == 1:
        opts.update(direct_offload=1, direct_upload=1, direct_grid=int(rng.choice([0, 1, 5])))
    elif mode == 2:
        opts.update(direct_offload=2, direct_upload=int(rng.choice([1, 3])))
    if rng.random() < 0.5:
        opts["host_tail_div"] = int(rng.choice([2, 3, 4, 8]))
    if rng.random() < 0.4:
        opts["overlap_kernels"] = 1
    return shape, n, opts


@pytest.mark.parametrize("k", range(24))
def test_random_small_shapes_and_options(k):
    shape, n, opts = _random_case(k)
    print(f"case {k}: L={shape.num_layers} pb={shape.page_bytes} S={shape.scales_per_block} NB={shape.num_blocks} n={n} {opts}", flush=True)
    _round_trip_case(shape, 0, n, salt=2000 + k, **opts)


@pytest.mark.parametrize("k", range(24))
def test_random_small_shapes_with_the_librarys_choice_of_path(k):
    """The same 24 shapes with the path left to the library (the default): uploads go through the scatter kernel
    that reads pinned memory itself, offloads through staging with the automatic host tail on transfers of several
    chunks; a large auto_direct_bytes in every third case sends the offload through the direct gather as well."""
    shape, n, opts = _random_case(k)
    for key in ("direct_offload", "direct_upload"):
        opts.pop(key, None)
    if k % 3 == 0:
        opts["auto_direct_bytes"] = 1 << 40
    else:
        opts.pop("host_tail_div", None)
    print(f"case {k} (auto): L={shape.num_layers} pb={shape.page_bytes} S={shape.scales_per_block} NB={shape.num_blocks} n={n} {opts}", flush=True)
    _round_trip_case(shape, 0, n, salt=2000 + k, auto=True, **opts)


def test_zero_blocks_is_a_no_op():
    _round_trip_case(W.CONFIGS[0], 0, 0, salt=3)


@pytest.mark.parametrize("host_tail_div,paths", [(1, "staged"), (64, "staged"), (0, "auto"), (1, "staged-overlapped")])
def test_config2_full_size_llama3_8b(host_tail_div, paths):
    """32 layers x 8 heads x 128 x 16 tokens bf16 (2 MiB per block), 16 384 blocks (32 GiB), one agent
    with a 4 096-token context = 256 blocks scattered uniformly; default launch configuration, and the
    one with the last 1/64 of the chunk moved over the link by the copy launch itself."""
    shape = W.CONFIGS[1]
    rng = W.rng_for(1)
    n = oracle.blocks_for_tokens(4096, shape.block_size)
    L, NB, pb, S, P = shape.num_layers, shape.num_blocks, shape.page_bytes, 0, shape.planes
    ids = W.pick_ids(rng, NB, n)
    new_ids = W.pick_ids(rng, NB, n, exclude=ids)
    path = {} if paths == "auto" else dict(direct_offload=K.TC_PATH_STAGED, direct_upload=K.TC_PATH_STAGED)
    if paths == "staged-overlapped":
        path["overlap_kernels"] = 1
    gp = GpuPool(shape, seed=W.seed_for(1), host_tail_div=host_tail_div, **path)
    try:
        rec = gp.rec
        before = gp.page_checksums(weighted=True)       # position-sensitive: a word that moved inside a page shows
        mirror = SparseMirror(gp, np.concatenate([ids, new_ids]))
        want_host = np.empty(n * rec, dtype=np.uint8)
        oracle.offload(mirror.pool, None, L, NB, pb, S, ids, want_host)

        stream = torch.cuda.Stream()
        host = pinned_bytes(n * rec)
        K.check(K.tc_alloc_at(gp.ctx, ids))
        K.check(K.tc_offload(gp.ctx, ids, host, stream))
        K.check(K.tc_free(gp.ctx, ids))
        K.check(K.tc_sync(gp.ctx))
        assert np.array_equal(host.numpy(), want_host)
        assert torch.equal(gp.page_checksums(weighted=True), before), "offload wrote the pool"

        table_d = torch.full((n + 2,), -1, dtype=torch.int32, device=DEV)
        torch.cuda.synchronize()       # torch wrote this on its own stream; the library's calls run on others
        table_h = np.full(n + 2, -1, dtype=np.int32)
        oracle.upload(want_host, L, NB, pb, S, new_ids, mirror.pool, None, table_h)
        K.check(K.tc_alloc_at(gp.ctx, new_ids))
        K.check(K.tc_upload(gp.ctx, host, new_ids, table_d, stream))
        stream.synchronize()
        assert np.array_equal(gp.blocks_to_host(new_ids), mirror.blocks(new_ids)), "uploaded blocks differ"
        assert np.array_equal(table_d.cpu().numpy(), table_h)
        # every block outside new_ids: untouched (per-page checksums by torch, not by the library)
        after = gp.page_checksums(weighted=True)
        keep = torch.ones(NB, dtype=torch.bool, device=DEV)
        keep[torch.as_tensor(new_ids.astype(np.int64), device=DEV)] = False
        assert torch.equal(after[:, keep], before[:, keep])
        # the remapped table addresses the same logical tokens (sampled)
        t0 = np.full(n, -1, dtype=np.int32)
        t0[:] = ids
        src_blocks = mirror.blocks(ids)  # still the pre-offload bytes: sources were not scrambled here
        for t in rng.integers(0, n * shape.block_size, size=64):
            j, slot = divmod(int(t), shape.block_size)
            tok = pb // shape.block_size
            for layer, kv in ((0, 0), (17, 1), (31, 1)):
                got = oracle.read_token(mirror.pool, L, NB, pb, shape.block_size, table_h, int(t), layer, kv)
                assert np.array_equal(got, src_blocks[2 * layer + kv, j, slot * tok:(slot + 1) * tok])
    finally:
        gp.close()
