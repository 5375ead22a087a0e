"""Residency map + CPU prefix-cache index driving real transfers (Sec. 6.3): an offload enters the
blocks' keys, a later request with the same prefix hits them on the CPU side, takes back the original
GPU blocks that are still free, uploads, and may run only when no H2D entry is left.  The library's
answers are compared with the oracle models call for call, the bytes with the oracle's copy."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_18586_amd as K
import tc_workloads as W
from oracle import residency as R
from harness import DEV, GpuPool, host_view

pytestmark = pytest.mark.gpu


def test_cpu_hit_reclaims_original_blocks_and_uploads():
    shape = W.CONFIGS[0]
    rng = W.rng_for(0, salt=31)
    pool_host = W.make_pool_host(shape, rng)
    mirror = pool_host.copy()
    gp = GpuPool(shape, pool_host=pool_host, host_arena_bytes=64 * 2 * shape.num_layers * shape.page_bytes)
    L, NB, pb, bs = gp.L, gp.NB, gp.pb, shape.block_size
    rc, ix = K.tc_index_create()
    assert rc == 0
    ixm = R.OracleResidencyIndex()
    bpm = oracle.OracleBlockPool(NB)
    try:
        stream = torch.cuda.Stream()
        tokens_a = rng.integers(0, 128000, size=10 * bs + 5, dtype=np.int32)        # 10 whole blocks + a tail
        rc, keys_a = K.tc_chain_hashes(tokens_a, bs)
        assert rc == 0 and [int(k) for k in keys_a] == R.chain_hashes([int(t) for t in tokens_a], bs)

        # agent A owns 11 scattered blocks (the last one partly filled: it has no key and is not cached)
        ids_a = W.pick_ids(rng, NB, 11)
        assert K.tc_alloc_at(gp.ctx, ids_a) == 0
        bpm.alloc_at(ids_a)
        cached = ids_a[:10]
        rc, buf = K.tc_host_alloc(gp.ctx, 10)
        assert rc == 0
        assert K.tc_offload(gp.ctx, cached, buf, stream) == 0
        assert K.tc_index_insert(ix, keys_a, cached, buf, gp.rec) == 0
        ixm.insert(keys_a, cached, buf, gp.rec)
        host_o = np.zeros(10 * gp.rec, dtype=np.uint8)
        oracle.offload(mirror, None, L, NB, pb, 0, np.asarray(cached, dtype=np.int32), host_o)
        assert K.tc_free(gp.ctx, ids_a) == 0
        bpm.begin_op(cached), bpm.free(ids_a)
        assert K.tc_sync(gp.ctx) == 0
        bpm.retire_all()
        assert np.array_equal(host_view(buf, 10 * gp.rec), host_o)

        # somebody else takes the four most recently freed blocks and overwrites them
        rc, other = K.tc_alloc(gp.ctx, 4)
        assert rc == 0 and list(other) == bpm.alloc(4)
        assert set(other) <= set(int(b) for b in ids_a)
        junk = rng.integers(0, 256, size=(gp.P, 4, pb), dtype=np.uint8)
        gp.pool3()[:, torch.as_tensor(other.astype(np.int64), device=DEV)] = torch.from_numpy(junk).to(DEV)
        torch.cuda.synchronize()       # torch wrote this on its own stream; the library's calls run on others
        mirror.reshape(gp.P, NB, pb)[:, other.astype(np.int64)] = junk

        # a request sharing only the first three blocks sees exactly those on the CPU side
        tokens_b = np.concatenate([tokens_a[:3 * bs], rng.integers(0, 128000, size=4 * bs, dtype=np.int32)])
        rc, keys_b = K.tc_chain_hashes(tokens_b, bs)
        rc, hits_b = K.tc_index_lookup(ix, keys_b)
        assert rc == 0 and hits_b == ixm.lookup(keys_b) and len(hits_b) == 3

        # the same conversation comes back two blocks longer: ten CPU hits
        tokens_a2 = np.concatenate([tokens_a[:10 * bs], rng.integers(0, 128000, size=2 * bs, dtype=np.int32)])
        rc, keys_a2 = K.tc_chain_hashes(tokens_a2, bs)
        rc, hits = K.tc_index_lookup(ix, keys_a2)
        assert rc == 0 and hits == ixm.lookup(keys_a2) and len(hits) == 10
        assert all(h[1] == K.TC_RES_CPU for h in hits) and hits[0][2] == buf
        prefer = [h[3] for h in hits] + [-1, -1]
        rc, new_ids = K.tc_alloc_prefer(gp.ctx, prefer)
        assert rc == 0 and list(new_ids) == bpm.alloc_prefer(prefer)
        reclaimed = sum(int(a) == int(b) for a, b in zip(new_ids[:10], cached))
        assert reclaimed == 10 - len(set(int(b) for b in other) & set(int(b) for b in cached)) and 0 < reclaimed < 10

        table = torch.full((16,), -7, dtype=torch.int32, device=DEV)
        torch.cuda.synchronize()       # torch wrote this on its own stream; the library's calls run on others
        hit_keys = [h[0] for h in hits]
        assert K.tc_upload(gp.ctx, hits[0][2], new_ids[:10], table, stream) == 0
        assert K.tc_index_begin_upload(ix, hit_keys, new_ids[:10]) == 0
        ixm.begin_upload(hit_keys, new_ids[:10])
        assert K.tc_index_pending(ix, keys_a2) == ixm.pending(keys_a2) == 10      # the request has to wait
        assert K.tc_index_remove(ix, hit_keys[:1]) == K.TC_ERR_INVAL              # no eviction under the copy
        assert K.tc_sync(gp.ctx) == 0
        assert K.tc_index_finish_upload(ix, hit_keys) == 0
        ixm.finish_upload(hit_keys)
        assert K.tc_index_pending(ix, keys_a2) == 0 and K.tc_index_size(ix) == ixm.size() == 0
        assert K.tc_index_lookup(ix, keys_b) == (0, [])
        assert K.tc_host_free(gp.ctx, buf) == 0

        table_o = np.full(16, -7, dtype=np.int32)
        oracle.upload(host_o, L, NB, pb, 0, np.asarray(new_ids[:10], dtype=np.int32), mirror, None, table_o[:10])
        assert np.array_equal(gp.pool_to_host(), mirror)
        assert np.array_equal(table.cpu().numpy(), table_o)
        # the logical tokens read through the new table are the ones the agent wrote before the offload
        for t in (0, bs - 1, 3 * bs + 2, 10 * bs - 1):
            got = oracle.read_token(mirror, L, NB, pb, bs, table_o[:10], t, 1, 0)
            want = oracle.read_token(pool_host, L, NB, pb, bs, np.asarray(cached, dtype=np.int32), t, 1, 0)
            assert np.array_equal(got, want)
    finally:
        K.tc_index_destroy(ix)
        gp.close()
