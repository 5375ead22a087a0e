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


class OracleStream:
    """Byte-for-byte comparison of whole configurations with the oracle, streamed: the blocks an agent owns are
    pulled into a sparse host mirror at their true strides (through pinned memory, in pieces of at most `piece`
    blocks), the oracle offloads them from the mirror and its records are compared with the library's; the oracle
    uploads the library's records into the mirror and the destination blocks are pulled and compared; then the
    mirror's pages are given back.  The CPU work of each piece runs on a small thread pool (the oracle's C code,
    numpy copies and comparisons all release the interpreter lock), the GPU copies on the calling thread."""

    def __init__(self, gp, workers=None, piece=192, max_pending=10):
        from concurrent.futures import ThreadPoolExecutor
        self.gp, self.piece, self.max_pending = gp, piece, max_pending
        self.mirror = SparseMirror(gp)
        self.pool = ThreadPoolExecutor(workers or max(2, min(12, (os.cpu_count() or 4) - 2)))
        self.pending = []
        self.stream = torch.cuda.Stream()
        self.bytes_compared = 0

    # ---- plumbing
    def _submit(self, fn, *a):
        self.pending.append(self.pool.submit(fn, *a))
        while len(self.pending) > self.max_pending:
            self.pending.pop(0).result()

    def wait(self):
        while self.pending:
            self.pending.pop(0).result()

    def _pieces(self, n):
        return [(a, min(n, a + self.piece)) for a in range(0, n, self.piece)]

    def _pull(self, ids):
        """(pages [P][n][pb], scale words [S][n] or None) of these blocks in pinned host memory + the event that
        says the copies have landed.  Runs on its own stream after everything enqueued so far on the device."""
        gp = self.gp
        host = torch.empty((gp.P, len(ids), gp.pb), dtype=torch.uint8, pin_memory=True)
        sc = torch.empty((gp.S, len(ids)), dtype=torch.int32, pin_memory=True) if gp.S else None
        torch.cuda.synchronize()
        with torch.cuda.stream(self.stream):
            # every temporary is made on this stream: a tensor made on another stream could be recycled, and
            # overwritten, while the gather enqueued here still reads it
            idx = torch.as_tensor(np.asarray(ids, dtype=np.int64)).to(DEV, non_blocking=False)
            host.copy_(gp.pool3()[:, idx], non_blocking=True)
            if gp.S:
                sc.copy_(gp.scales.view(gp.S, gp.NB)[:, idx], non_blocking=True)
            ev = torch.cuda.Event()
            ev.record(self.stream)
        return host, sc, ev

    @staticmethod
    def _same(a, b):
        a, b = np.ascontiguousarray(a).reshape(-1), np.ascontiguousarray(b).reshape(-1)
        if a.size != b.size:
            return False
        k = a.size // 8 * 8
        return bool((a[:k].view(np.uint64) == b[:k].view(np.uint64)).all()) and bool((a[k:] == b[k:]).all())

    # ---- the three steps
    def snapshot(self, ids):
        """Before the offload: the agent's blocks, as they are on the device now, go into the mirror."""
        ids = np.asarray(ids, dtype=np.int32)
        for a, b in self._pieces(len(ids)):
            host, sc, ev = self._pull(ids[a:b])

            def work(sub=ids[a:b].astype(np.int64), host=host, sc=sc, ev=ev):
                ev.synchronize()
                gp = self.gp
                self.mirror.pool.reshape(gp.P, gp.NB, gp.pb)[:, sub] = host.numpy()
                if gp.S:
                    self.mirror.scales.reshape(gp.S, gp.NB)[:, sub] = sc.numpy().view(np.uint32)
            self._submit(work)

    def check_records(self, ids, records, what=""):
        """After the offload has completed: the oracle's records of these blocks against the library's
        (`records`: numpy view of the host buffer).  The caller has waited for the snapshot (wait())."""
        gp = self.gp
        ids = np.asarray(ids, dtype=np.int32)
        for a, b in self._pieces(len(ids)):
            def work(a=a, b=b):
                want = np.empty((b - a) * gp.rec, dtype=np.uint8)
                oracle.offload(self.mirror.pool, self.mirror.scales, gp.L, gp.NB, gp.pb, gp.S, ids[a:b], want)
                assert self._same(want, records[a * gp.rec:b * gp.rec]), f"{what}: records of blocks {a}..{b} differ from the oracle"
            self._submit(work)
            self.bytes_compared += (b - a) * gp.rec

    def expected_records(self, ids):
        """The oracle's records of these blocks, from the mirror as it is now (complete on return)."""
        gp = self.gp
        ids = np.asarray(ids, dtype=np.int32)
        want = np.empty(len(ids) * gp.rec, dtype=np.uint8)
        for a, b in self._pieces(len(ids)):
            self._submit(lambda a=a, b=b: oracle.offload(self.mirror.pool, self.mirror.scales, gp.L, gp.NB, gp.pb, gp.S,
                                                         ids[a:b], want[a * gp.rec:b * gp.rec]))
        self.wait()
        return want

    def compare(self, want, got, what=""):
        """Two byte arrays of whole records, piece by piece on the pool (complete after wait())."""
        gp = self.gp
        assert want.size == got.size, f"{what}: {want.size} bytes expected, {got.size} there"
        for a, b in self._pieces(want.size // gp.rec):
            def work(a=a, b=b):
                assert self._same(want[a * gp.rec:b * gp.rec], got[a * gp.rec:b * gp.rec]), \
                    f"{what}: records of blocks {a}..{b} differ from the oracle"
            self._submit(work)
            self.bytes_compared += (b - a) * gp.rec

    def check_upload(self, records, new_ids, what="", table=None):
        """After the upload has completed: the oracle uploads the same records into the mirror, and the
        destination blocks on the device must equal the mirror's, pages and scale words.  Returns the table
        row the oracle wrote, complete after wait() (if `table`, an int32 array of len(new_ids), is given it is
        filled).  The caller has waited for the steps before."""
        gp = self.gp
        new_ids = np.asarray(new_ids, dtype=np.int32)
        if table is None:
            table = np.full(len(new_ids), -1, dtype=np.int32)
        for a, b in self._pieces(len(new_ids)):
            host, sc, ev = self._pull(new_ids[a:b])

            def work(a=a, b=b, host=host, sc=sc, ev=ev):
                oracle.upload(records[a * gp.rec:b * gp.rec], gp.L, gp.NB, gp.pb, gp.S, new_ids[a:b], self.mirror.pool,
                              self.mirror.scales, table[a:b])
                ev.synchronize()
                sub = new_ids[a:b].astype(np.int64)
                assert self._same(host.numpy(), self.mirror.pool.reshape(gp.P, gp.NB, gp.pb)[:, sub]), \
                    f"{what}: uploaded blocks {a}..{b} differ from the oracle"
                if gp.S:
                    assert self._same(sc.numpy().view(np.uint32), self.mirror.scales.reshape(gp.S, gp.NB)[:, sub]), \
                        f"{what}: scale words of blocks {a}..{b} differ from the oracle"
            self._submit(work)
            self.bytes_compared += (b - a) * gp.rec
        return table

    def drop(self, ids=None):
        """Gives the mirror's pages of these blocks (all of them without `ids`) back to the system; they read
        as zeros afterwards."""
        import mmap
        self.wait()
        gp = self.gp
        mm = self.mirror._mm[0]
        if gp.pb % mmap.PAGESIZE or not hasattr(mm, "madvise"):
            return
        if ids is None:
            mm.madvise(mmap.MADV_DONTNEED)
            return
        blocks = np.sort(np.asarray(ids, dtype=np.int64))
        if blocks.size == 0:
            return
        cuts = np.flatnonzero(np.diff(blocks) != 1) + 1            # runs of consecutive ids: one call per run and plane
        for run in np.split(blocks, cuts):
            for p in range(gp.P):
                mm.madvise(mmap.MADV_DONTNEED, int((p * gp.NB + run[0]) * gp.pb), int(run.size) * gp.pb)

    def close(self):
        try:
            self.wait()
        finally:
            self.pool.shutdown(wait=True)
            self.mirror.close()
