"""Shared plumbing of the GPU parity tests: device memory via torch, calls via the C-ABI binding.

Nothing here computes any part of the path; it allocates, copies inputs in and results out
(torch copies), and drives the library and the oracle with the same seeded inputs.
"""
import os

import numpy as np
import torch

import oracle
import paper_2510_18586_amd as K
import tc_workloads as W

DEV = "cuda:0"
GUARD_BYTES = 1 << 16          # keeps the pool 256-B aligned
GUARD_VALUE = 0xC3


class GpuPool:
    """A KV pool (+ scales) in device memory bound to a library context."""

    def __init__(self, shape, pool_host=None, scales_host=None, seed=None, **opts):
        self.shape = shape
        self.L, self.NB, self.pb = shape.num_layers, shape.num_blocks, shape.page_bytes
        self.P, self.S = shape.planes, shape.scales_per_block
        self._guarded = None
        if pool_host is not None:
            # guard bytes in front of and behind the pool: a kernel that writes outside it is caught at close()
            g = GUARD_BYTES
            self._guarded = torch.full((g + pool_host.size + g,), GUARD_VALUE, dtype=torch.uint8, device=DEV)
            self.pool = self._guarded[g:g + pool_host.size]
            self.pool.copy_(torch.from_numpy(pool_host))
            self.scales = torch.from_numpy(scales_host.view(np.int32)).to(DEV) if self.S else None
        else:
            self.pool = W.make_pool_device(shape, seed, DEV)
            sc = W.make_scales_device(shape, seed, DEV)
            self.scales = sc.view(torch.int32) if sc is not None else None
        rc, self.ctx = K.tc_create(self.pool, self.scales, self.L, self.NB, self.pb, shape.block_size, self.S, **opts)
        K.check(rc)
        self.rec = K.tc_record_bytes(self.ctx)
        assert self.rec == oracle.record_bytes(self.L, self.pb, self.S)

    def close(self):
        if self.ctx:
            K.check(K.tc_destroy(self.ctx))
            self.ctx = None
        if self._guarded is not None:
            g, n = GUARD_BYTES, self._guarded.numel()
            ok = bool((self._guarded[:g] == GUARD_VALUE).all()) and bool((self._guarded[n - g:] == GUARD_VALUE).all())
            self._guarded = None
            assert ok, "bytes outside the pool were written"
        self.pool = self.scales = None
        torch.cuda.empty_cache()


    # ---- views / copies (torch only) --------------------------------------
    def pool3(self):
        return self.pool.view(self.P, self.NB, self.pb)

    def blocks_to_host(self, ids):
        """[P][len(ids)][pb] uint8 numpy copy of the given blocks."""
        idx = torch.as_tensor(np.asarray(ids, dtype=np.int64), device=DEV)
        return self.pool3()[:, idx].cpu().numpy()

    def scales_to_host(self, ids):
        idx = torch.as_tensor(np.asarray(ids, dtype=np.int64), device=DEV)
        return self.scales.view(self.S, self.NB)[:, idx].cpu().numpy().view(np.uint32)

    def pool_to_host(self):
        return self.pool.cpu().numpy()

    def scales_all_to_host(self):
        return self.scales.cpu().numpy().view(np.uint32) if self.S else None

    def _weights(self):
        # odd, position-dependent multipliers: a sum that notices words that moved inside a page
        i = torch.arange(self.pb // 4, dtype=torch.int64, device=DEV)
        return i * 2654435761 + 0x9E3779B1 | 1

    def page_checksums(self, weighted=False):
        """One int64 per (plane, block): a torch reduction, independent of the library.  weighted:
        position-sensitive (wrapping) sum instead of the plain sum of the page's 32-bit words."""
        v = self.pool.view(torch.int32).view(self.P, self.NB, self.pb // 4)
        if not weighted:
            return v.sum(dim=2, dtype=torch.int64)
        w = self._weights()
        return torch.stack([(v[p].to(torch.int64) * w).sum(dim=1) for p in range(self.P)])

    def block_checksums(self, ids, weighted=True):
        """[P][len(ids)] int64 page checksums (+ scale words as extra rows): torch only."""
        idx = torch.as_tensor(np.asarray(ids, dtype=np.int64), device=DEV)
        v = self.pool.view(torch.int32).view(self.P, self.NB, self.pb // 4)
        if weighted:
            w = self._weights()
            cs = torch.stack([(v[p, idx].to(torch.int64) * w).sum(dim=1) for p in range(self.P)])
        else:
            cs = v[:, idx].sum(dim=2, dtype=torch.int64)
        if self.S:
            cs = torch.cat([cs, self.scales.view(self.S, self.NB)[:, idx].to(torch.int64)], dim=0)
        return cs


def host_budget_bytes(want, share=0.25):
    """Pinned-arena size for a test: `want`, but never more than `share` of the host memory that is
    available right now (read from /proc/meminfo at run time); prints what it chose."""
    avail = None
    try:
        with open("/proc/meminfo") as f:
            for line in f:
                if line.startswith("MemAvailable:"):
                    avail = int(line.split()[1]) * 1024
    except OSError:
        pass
    got = int(want) if avail is None else int(min(want, share * avail))
    print(f"[harness] host memory available {'?' if avail is None else f'{avail / 2**30:.0f} GiB'}, "
          f"{os.cpu_count()} cpus: pinned arena {got / 2**30:.1f} GiB (wanted {want / 2**30:.1f})", flush=True)
    return got


def pinned_bytes(n):
    return torch.empty(max(int(n), 1), dtype=torch.uint8, pin_memory=True)


class SparseMirror:
    """Host mirror of a full-size pool holding only the blocks a test touches, at their true
    offsets: an anonymous no-reserve mapping, so untouched pages are never materialised.
    close() returns the memory."""

    def __init__(self, gp, ids=()):
        import mmap
        self.gp = gp
        flags = mmap.MAP_PRIVATE | mmap.MAP_ANONYMOUS | getattr(mmap, "MAP_NORESERVE", 0)
        self._mm = [mmap.mmap(-1, gp.P * gp.NB * gp.pb, flags=flags)]
        self.pool = np.frombuffer(self._mm[0], dtype=np.uint8)
        self.scales = None
        if gp.S:
            self._mm.append(mmap.mmap(-1, 4 * gp.S * gp.NB, flags=flags))
            self.scales = np.frombuffer(self._mm[1], dtype=np.uint32)
        if len(ids):
            self.load(ids)

    def load(self, ids):
        """Copies the current device content of these blocks (and their scale words) into the mirror."""
        gp = self.gp
        ids = np.asarray(ids, dtype=np.int64)
        v = self.pool.reshape(gp.P, gp.NB, gp.pb)
        for a in range(0, ids.size, 64):
            sub = ids[a:a + 64]
            v[:, sub] = gp.blocks_to_host(sub)
            if gp.S:
                self.scales.reshape(gp.S, gp.NB)[:, sub] = gp.scales_to_host(sub)

    def blocks(self, ids):
        return self.pool.reshape(self.gp.P, self.gp.NB, self.gp.pb)[:, np.asarray(ids, dtype=np.int64)]

    def scale_words(self, ids):
        return self.scales.reshape(self.gp.S, self.gp.NB)[:, np.asarray(ids, dtype=np.int64)]

    def close(self):
        self.pool = self.scales = None
        for m in self._mm:
            try:
                m.close()
            except BufferError:
                pass
        self._mm = []


def host_view(addr, nbytes):
    """numpy view of pinned memory the library handed out (tc_host_alloc)."""
    import ctypes
    return np.ctypeslib.as_array((ctypes.c_uint8 * int(nbytes)).from_address(int(addr)))
