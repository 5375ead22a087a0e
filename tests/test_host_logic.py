"""The library's host bookkeeping (csrc/tc_blocks.h) against the oracle's model, without a GPU.

The C++ classes are compiled with g++ (address + undefined-behaviour sanitizers on) behind a
test-only C shim and driven with the same seeded op streams as the oracle's OracleBlockPool /
OracleHostArena; every returned id, status code and counter must agree.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest

import tc_workloads as W
from oracle import OracleBlockPool, OracleHostArena, OracleError

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CODE = {"INVAL": -1, "RANGE": -2, "DUP": -3, "SHARED": -4, "NOMEM": -5, "HOST_NOMEM": -6}


@pytest.fixture(scope="module")
def shim(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("shim") / "libblocks_shim.so")
    subprocess.run(
        ["g++", "-std=c++17", "-O1", "-g", "-fPIC", "-shared", "-Wall", "-Wextra", "-Werror",
         "-fsanitize=undefined", "-fno-sanitize-recover=undefined",
         "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2510_18586_amd", "csrc"),
         os.path.join(HERE, "csrc", "blocks_shim.cpp"), "-o", out],
        check=True)
    lib = ctypes.CDLL(out)
    vp, u32, u64 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64
    lib.tcb_pool_new.restype, lib.tcb_pool_new.argtypes = vp, [u32]
    lib.tcb_pool_del.argtypes = [vp]
    for f in ("tcb_alloc_at", "tcb_ref", "tcb_free", "tcb_check_transfer", "tcb_begin", "tcb_end"):
        getattr(lib, f).argtypes = [vp, vp, u32]
    lib.tcb_alloc.argtypes = [vp, u32, vp]
    lib.tcb_alloc_prefer.argtypes = [vp, vp, u32, vp]
    lib.tcb_filter_private.argtypes = [vp, vp, u32, vp, ctypes.POINTER(u32)]
    lib.tcb_counts.argtypes = [vp, vp]
    lib.tcb_arena_new.restype, lib.tcb_arena_new.argtypes = vp, [u64]
    lib.tcb_arena_del.argtypes = [vp]
    lib.tcb_arena_alloc.restype, lib.tcb_arena_alloc.argtypes = ctypes.c_int64, [vp, u64]
    lib.tcb_arena_free.argtypes = [vp, u64]
    lib.tcb_arena_used.restype, lib.tcb_arena_used.argtypes = u64, [vp]
    lib.tcb_arena_locate.argtypes = [vp, u64, ctypes.POINTER(u64), ctypes.POINTER(u64)]
    lib.tcb_arena_begin.argtypes = [vp, u64]
    lib.tcb_arena_end.argtypes = [vp, u64]
    return lib


class NativePool:
    def __init__(self, lib, nb):
        self.lib, self.p = lib, lib.tcb_pool_new(nb)

    def __del__(self):
        self.lib.tcb_pool_del(self.p)

    @staticmethod
    def _a(ids):
        a = np.ascontiguousarray(ids, dtype=np.int32)
        return a, (a.ctypes.data if a.size else None), int(a.size)

    def call(self, name, ids):
        a, p, n = self._a(ids)
        return getattr(self.lib, name)(self.p, p, n)

    def alloc(self, n):
        out = np.empty(max(n, 1), dtype=np.int32)
        rc = self.lib.tcb_alloc(self.p, n, out.ctypes.data)
        return rc, list(out[:n]) if rc == 0 else []

    def alloc_prefer(self, pref):
        a, p, n = self._a(pref)
        out = np.empty(max(n, 1), dtype=np.int32)
        rc = self.lib.tcb_alloc_prefer(self.p, p, n, out.ctypes.data)
        return rc, [int(x) for x in out[:n]] if rc == 0 else []

    def counts(self):
        c = np.zeros(4, dtype=np.uint32)
        self.lib.tcb_counts(self.p, c.ctypes.data)
        return tuple(int(x) for x in c)

    def filter_private(self, ids):
        a, p, n = self._a(ids)
        out = np.empty(max(n, 1), dtype=np.int32)
        m = ctypes.c_uint32()
        rc = self.lib.tcb_filter_private(self.p, p, n, out.ctypes.data, ctypes.byref(m))
        return rc, list(out[:m.value])


def _oracle_rc(fn, *a):
    try:
        return 0, fn(*a)
    except OracleError as e:
        return CODE[e.code], None


def _same_counts(nat, orc):
    assert nat.counts() == (orc.n_free(), orc.n_used(), orc.n_pending(), orc.n_shared())


def test_hand_worked_sequence_matches_oracle(shim):
    nat, orc = NativePool(shim, 8), OracleBlockPool(8)
    assert nat.alloc(3) == (0, [0, 1, 2]) and orc.alloc(3) == [0, 1, 2]
    assert nat.call("tcb_free", [1]) == 0
    orc.free([1])
    assert nat.alloc(2)[1] == orc.alloc(2) == [1, 3]
    assert nat.call("tcb_free", [0, 2]) == 0
    orc.free([0, 2])
    assert nat.alloc(3)[1] == orc.alloc(3) == [2, 0, 4]
    assert nat.alloc(4)[0] == CODE["NOMEM"]
    _same_counts(nat, orc)


def test_alloc_prefer_hand_worked_matches_oracle(shim):
    nat, orc = NativePool(shim, 8), OracleBlockPool(8)
    nat.alloc(8), orc.alloc(8)
    nat.call("tcb_free", [5, 2, 7]), orc.free([5, 2, 7])
    assert nat.alloc_prefer([2, 4, 5]) == (0, orc.alloc_prefer([2, 4, 5])) == (0, [2, 7, 5])
    assert nat.alloc_prefer([1])[0] == _oracle_rc(orc.alloc_prefer, [1])[0] == CODE["NOMEM"]
    # a block that is pending-free behind a running copy is not claimed
    nat.call("tcb_begin", [2, 7]), orc.begin_op([2, 7])
    nat.call("tcb_free", [2, 7, 5]), orc.free([2, 7, 5])
    assert nat.alloc_prefer([7])[1] == orc.alloc_prefer([7]) == [5]
    _same_counts(nat, orc)


def test_error_codes_and_no_side_effects(shim):
    nat, orc = NativePool(shim, 8), OracleBlockPool(8)
    nat.alloc(3), orc.alloc(3)
    for ids in ([0, 8], [-1], [0, 1, 0], [0, 5], []):
        assert nat.call("tcb_check_transfer", ids) == _oracle_rc(orc.check_transfer, ids)[0]
    assert nat.call("tcb_free", [0, 0]) == _oracle_rc(orc.free, [0, 0])[0] == CODE["INVAL"]
    assert nat.call("tcb_ref", [4]) == _oracle_rc(orc.ref, [4])[0] == CODE["INVAL"]
    assert nat.call("tcb_ref", [0, 1]) == 0
    orc.ref([0, 1])
    assert nat.call("tcb_check_transfer", [2, 1]) == _oracle_rc(orc.check_transfer, [2, 1])[0] == CODE["SHARED"]
    assert nat.filter_private([0, 1, 2]) == (0, orc.filter_private([0, 1, 2]))
    assert nat.call("tcb_alloc_at", [4, 0]) == _oracle_rc(orc.alloc_at, [4, 0])[0] == CODE["NOMEM"]
    assert nat.call("tcb_alloc_at", [4, 4]) == _oracle_rc(orc.alloc_at, [4, 4])[0] == CODE["DUP"]
    _same_counts(nat, orc)
    assert nat.call("tcb_free", [0, 0]) == 0   # two references now: both may be dropped at once
    orc.free([0, 0])
    _same_counts(nat, orc)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_op_stream_id_for_id(shim, seed):
    rng = np.random.default_rng(seed)
    NB = 113
    nat, orc = NativePool(shim, NB), OracleBlockPool(NB)
    held, ops = [], []
    for _ in range(8000):
        r = rng.random()
        if r < 0.30:
            n = int(rng.integers(0, 14))
            rc, got = nat.alloc(n)
            rco, want = _oracle_rc(orc.alloc, n)
            assert rc == rco and (rc != 0 or got == want)
            if rc == 0 and got:
                held.append(got)
        elif r < 0.40 and orc.n_free():
            k = int(rng.integers(1, 6))
            ids = [int(x) for x in rng.choice(NB, size=k, replace=bool(rng.random() < 0.2))]
            rc, rco = nat.call("tcb_alloc_at", ids), _oracle_rc(orc.alloc_at, ids)[0]
            assert rc == rco
            if rc == 0:
                held.append(ids)
        elif r < 0.45:
            k = int(rng.integers(0, 9))
            pref = [int(x) for x in rng.integers(-1, NB + 1, size=k)]      # repeats, held and bad ids included
            rc, got = nat.alloc_prefer(pref)
            rco, want = _oracle_rc(orc.alloc_prefer, pref)
            assert rc == rco and (rc != 0 or got == want), pref
            if rc == 0 and got:
                held.append(got)
        elif r < 0.52 and held:
            ids = held[int(rng.integers(len(held)))]
            assert nat.call("tcb_ref", ids) == 0
            orc.ref(ids)
            held.append(list(ids))
        elif r < 0.75 and held:
            ids = held.pop(int(rng.integers(len(held))))
            if rng.random() < 0.5:
                rc, rco = nat.call("tcb_check_transfer", ids), _oracle_rc(orc.check_transfer, ids)[0]
                assert rc == rco
                if rc == 0:
                    nat.call("tcb_begin", ids)
                    orc.begin_op(ids)
                    ops.append(ids)
            assert nat.call("tcb_free", ids) == 0
            orc.free(ids)
        elif r < 0.90 and ops:
            ids = ops.pop(0)
            nat.call("tcb_end", ids)
            orc.retire_oldest()
        _same_counts(nat, orc)
        f, u, p, _ = nat.counts()
        assert f + u + p == NB
    while ops:
        nat.call("tcb_end", ops.pop(0))
        orc.retire_oldest()
    # whatever is free now comes out in the same order on both sides
    n = orc.n_free()
    assert nat.alloc(n)[1] == orc.alloc(n)


def test_fragmentation_script_same_ids_on_both_sides(shim):
    """The config-3 fragmentation recipe (seeded alloc/free ops) run against both allocators."""
    NB = 2048
    nat, orc = NativePool(shim, NB), OracleBlockPool(NB)

    class Nat:
        def alloc(self, n):
            rc, ids = nat.alloc(n)
            return ids if rc == 0 else None

        def free(self, ids):
            assert nat.call("tcb_free", ids) == 0

        def n_free(self):
            return nat.counts()[0]

    class Orc:
        def alloc(self, n):
            try:
                return orc.alloc(n)
            except OracleError:
                return None

        def free(self, ids):
            orc.free(ids)

        def n_free(self):
            return orc.n_free()

    a = W.fragment_pool(Nat(), W.rng_for(2, salt=9), n_ops=4000, median_blocks=16, need_free=900)
    b = W.fragment_pool(Orc(), W.rng_for(2, salt=9), n_ops=4000, median_blocks=16, need_free=900)
    assert a == b
    _same_counts(nat, orc)
    n = orc.n_free()
    ids_n, ids_o = nat.alloc(n)[1], orc.alloc(n)
    assert ids_n == ids_o
    assert ids_n != sorted(ids_n), "the free list should be fragmented, not ascending"


def test_host_arena_matches_oracle(shim):
    rng = np.random.default_rng(5)
    N = 300
    a, o = shim.tcb_arena_new(N), OracleHostArena(N)
    live, busy = [], []
    try:
        for _ in range(5000):
            r = rng.random()
            if r < 0.45:
                n = int(rng.integers(1, 40))
                got = shim.tcb_arena_alloc(a, n)
                rco, want = _oracle_rc(o.alloc, n)
                assert (got < 0) == (rco != 0)
                if rco == 0:
                    assert got == want
                    live.append((got, n))
            elif r < 0.60 and live:
                s, n = live[int(rng.integers(len(live)))]
                slot = s + int(rng.integers(n))
                st, room = ctypes.c_uint64(), ctypes.c_uint64()
                assert shim.tcb_arena_locate(a, slot, ctypes.byref(st), ctypes.byref(room)) == 1
                assert st.value == o.owner_of(slot) == s and room.value == s + n - slot
                shim.tcb_arena_begin(a, s)
                o.begin_op(s)
                busy.append(s)
            elif r < 0.85 and live:
                s, n = live.pop(int(rng.integers(len(live))))
                assert shim.tcb_arena_free(a, s) == 0
                o.free(s)
                assert shim.tcb_arena_free(a, s) == CODE["INVAL"]     # second release is refused
            elif busy:
                s = busy.pop(0)
                shim.tcb_arena_end(a, s)
                o.end_op(s)
            assert shim.tcb_arena_used(a) == o.used_slots()
    finally:
        shim.tcb_arena_del(a)


@pytest.mark.parametrize("sanitizer", ["address,undefined", "thread"])
def test_host_code_under_sanitizers(tmp_path, sanitizer):
    """tests/csrc/host_sanitize.cpp + the library's host-only sources as a plain executable, built with
    AddressSanitizer + UBSan and with ThreadSanitizer: seeded op streams on the block pool and the arena,
    four threads on one residency index and one forecaster, random inputs to the scheduling arithmetic."""
    csrc = os.path.join(ROOT, "paper_2510_18586_amd", "csrc")
    exe = str(tmp_path / "host_sanitize")
    subprocess.run(
        ["g++", "-std=c++17", "-O1", "-g", "-Wall", "-Wextra", "-Werror", "-pthread",
         "-fsanitize=" + sanitizer, "-fno-sanitize-recover=all",
         "-static-libasan" if "address" in sanitizer else "-static-libtsan",     # no dependence on library load order
         "-I", os.path.join(ROOT, "include"), "-I", csrc,
         os.path.join(HERE, "csrc", "host_sanitize.cpp"), os.path.join(csrc, "tc_index.cpp"),
         os.path.join(csrc, "tc_policy.cpp"), "-o", exe],
        check=True)
    out = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0 and out.stdout.strip().endswith("ok"), (out.returncode, out.stdout[-2000:], out.stderr[-4000:])


# ---------------------------------------------------------------------------------- transfer planning
def _plan_sigs(lib):
    vp, u32, u64, i64, ci = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_int64, ctypes.c_int
    lib.tcp_book_new.restype, lib.tcp_book_new.argtypes = vp, [u64, u32]
    lib.tcp_book_del.argtypes = [vp]
    lib.tcp_book_begin.restype = i64
    lib.tcp_book_begin.argtypes = [vp, u64, vp, u32, vp, u32, ci, vp, ctypes.POINTER(u32), vp]
    lib.tcp_book_publish.restype = u64
    lib.tcp_book_publish.argtypes = [vp, u64, vp, u32, vp, u32, ci, ci, vp]
    lib.tcp_book_cancel.argtypes = [vp, vp]
    lib.tcp_book_retire.restype, lib.tcp_book_retire.argtypes = u64, [vp]
    lib.tcp_book_ring_used.restype, lib.tcp_book_ring_used.argtypes = u64, [vp]
    lib.tcp_book_upload_in_flight.argtypes = [vp]
    lib.tcp_plan_chunks.restype, lib.tcp_plan_chunks.argtypes = u32, [u64, u32, ci, u32, vp, u32]
    lib.tcp_chunk_pieces.restype, lib.tcp_chunk_pieces.argtypes = u32, [vp, vp, u32, u64, u64, vp, u32]
    lib.tcp_host_tail.argtypes = [u32, u64, u32, vp, vp, u32, vp]
    lib.tcp_offload_direct.argtypes = [u32, u64, ci, u64]
    lib.tcp_upload_direct.argtypes = [u32]
    lib.tcp_tail_divisor.restype, lib.tcp_tail_divisor.argtypes = u32, [u32, u64, ci]
    lib.tcp_kernels_overlap.argtypes = [u32, u64]
    lib.tcp_plan_staged.restype, lib.tcp_plan_staged.argtypes = u32, [u64, u32, ci, u32, u32, ctypes.POINTER(ci), vp, u32]
    return lib


def test_transfer_book_matches_the_model_step_for_step(shim):
    """Id ring, hazards and what a failed transfer holds (csrc/tc_plan.h) against oracle/transfer_plan.py on
    seeded streams of begin / publish / publish-failed / cancel / retire: every ring start, every set of
    transfers to wait for, every ticket and the ring's fill level agree."""
    import oracle.transfer_plan as T
    lib = _plan_sigs(shim)
    rng = np.random.default_rng(W.seed_for(0, 91))
    for cap, nb in ((16, 12), (64, 40), (1000, 300)):
        book = lib.tcp_book_new(cap, nb)
        model = T.OracleTransferBook(cap)
        for _ in range(3000):
            r = rng.random()
            if r < 0.6:
                n = int(rng.integers(1, max(2, min(nb, cap // 3))))
                ids = rng.choice(nb, size=n, replace=False).astype(np.int32)
                arena = rng.choice(8, size=int(rng.integers(0, 3)), replace=False).astype(np.uint64)
                stream, up = int(rng.integers(1, 4)), int(rng.integers(0, 2))
                waits = np.zeros(64, dtype=np.uint64)
                n_waits, span = ctypes.c_uint32(0), np.zeros(3, dtype=np.uint64)
                got = lib.tcp_book_begin(book, stream, ids.ctypes.data, n, arena.ctypes.data if arena.size else None,
                                         int(arena.size), up, waits.ctypes.data, ctypes.byref(n_waits), span.ctypes.data)
                want_start, want_waits = model.begin(stream, ids.tolist(), arena.tolist(), upload=bool(up))
                assert set(int(x) for x in waits[: n_waits.value]) == want_waits
                assert got == (-1 if want_start is None else want_start)
                if want_start is None:
                    continue
                if rng.random() < 0.1:
                    lib.tcp_book_cancel(book, span.ctypes.data)
                    model.cancel()
                else:
                    failed = int(rng.random() < 0.2)
                    t = lib.tcp_book_publish(book, stream, ids.ctypes.data, n, arena.ctypes.data if arena.size else None,
                                             int(arena.size), up, failed, span.ctypes.data)
                    assert t == model.publish(failed=bool(failed))
            elif model.ops:
                assert lib.tcp_book_retire(book) == model.retire_oldest()["ticket"]
            assert lib.tcp_book_ring_used(book) == model.ring.used()
            assert bool(lib.tcp_book_upload_in_flight(book)) == model.upload_in_flight()
        lib.tcp_book_del(book)


def test_chunks_pieces_tail_and_paths_match_the_model(shim):
    import oracle.transfer_plan as T
    lib = _plan_sigs(shim)
    rng = np.random.default_rng(W.seed_for(0, 92))
    for _ in range(2000):
        lens = rng.integers(1, 300, size=int(rng.integers(1, 8))).astype(np.uint32)
        firsts = np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.uint64)
        segs = [(int(f), int(n)) for f, n in zip(firsts, lens)]
        total, slot, up = int(lens.sum()), int(rng.integers(1, 400)), int(rng.integers(0, 2))
        out = np.zeros(2048, dtype=np.uint32)
        head = int(rng.choice([0, 0, 1, 7, 64, 500]))
        k = lib.tcp_plan_chunks(total, slot, up, head, out.ctypes.data, out.size)
        sizes = T.plan_chunks(total, slot, bool(up), head)
        assert out[:k].tolist() == sizes
        ov = ctypes.c_int(0)
        k2 = lib.tcp_plan_staged(total, slot, up, head, opt01 := int(rng.integers(0, 2)), ctypes.byref(ov), out.ctypes.data, out.size)
        assert (out[:k2].tolist(), bool(ov.value)) == T.plan_staged(total, slot, bool(up), head, opt01)
        c0 = 0
        for size in sizes[:6]:
            buf = np.zeros(4 * 16, dtype=np.uint64)
            m = lib.tcp_chunk_pieces(firsts.ctypes.data, lens.ctypes.data, len(segs), c0, c0 + size, buf.ctypes.data, 16)
            assert [tuple(int(x) for x in buf[4 * i:4 * i + 4]) for i in range(m)] == T.chunk_pieces(segs, c0, c0 + size)
            div = int(rng.choice([0, 1, 2, 3, 64, 1000]))
            o3 = np.zeros(3, dtype=np.int64)
            lib.tcp_host_tail(div, c0, size, firsts.ctypes.data, lens.ctypes.data, len(segs), o3.ctypes.data)
            staged, seg, in_seg = T.host_tail_split(div, c0, size, segs)
            assert (int(o3[0]), int(o3[1]), int(o3[2])) == (staged, -1 if seg is None else seg, 0 if in_seg is None else in_seg)
            c0 += size
        mode, nbytes, dup, auto = int(rng.integers(0, 4)), int(rng.integers(0, 1 << 30)), int(rng.integers(0, 2)), int(rng.integers(1, 1 << 30))
        assert bool(lib.tcp_offload_direct(mode, nbytes, dup, auto)) == (T.offload_path(mode, nbytes, bool(dup), auto) == T.DIRECT)
        assert bool(lib.tcp_upload_direct(mode)) == (T.upload_path(mode) == T.DIRECT)
        opt, nch = int(rng.choice([0, 1, 2, 48])), int(rng.integers(1, 5))
        ov = int(rng.integers(0, 2))
        assert lib.tcp_tail_divisor(opt, nch, ov) == T.tail_divisor(opt, nch, bool(ov))
        assert bool(lib.tcp_kernels_overlap(opt if opt < 2 else 1, nch)) == T.kernels_overlap_copies(opt if opt < 2 else 1, nch)


def test_engine_on_a_cpu_stand_in_under_sanitizers(tmp_path):
    """tests/csrc/engine_emul.cpp: the whole transfer engine (csrc/tc_engine_core.h) with a stand-in device that
    queues work per stream and runs it in adversarial orders on exact-size heap buffers, walking a launch through
    the kernels' own index arithmetic.  Built with AddressSanitizer + UBSan, compared byte for byte with the
    oracle's C file, with every fallible device call failing in turn."""
    import oracle
    csrc = os.path.join(ROOT, "paper_2510_18586_amd", "csrc")
    exe, obj = str(tmp_path / "engine_emul"), str(tmp_path / "tc_oracle.o")
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all"]
    subprocess.run(["gcc", "-std=c11", "-O1", "-g", *san, "-c", os.path.join(os.path.dirname(oracle.__file__), "tc_oracle.c"),
                    "-o", obj], check=True)
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-Wall", "-Wextra", "-Werror", *san, "-static-libasan",
                    "-I", os.path.join(ROOT, "include"), "-I", csrc, os.path.join(HERE, "csrc", "engine_emul.cpp"), obj,
                    "-o", exe], check=True)
    out = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    assert out.returncode == 0 and out.stdout.strip().endswith("ok"), (out.returncode, out.stdout[-2000:], out.stderr[-4000:])


ORDERING_MISTAKES = {
    "an offload's DMA does not wait for its gather": (
        "                    TC_DEV(dev.stream_wait(stream, slot->ready));\n                }\n                TC_RC(time_begin(&op, stream, uint64_t(split) * rec, kD2H));",
        "                }\n                TC_RC(time_begin(&op, stream, uint64_t(split) * rec, kD2H));"),
    "a gather overwrites a slot whose DMA is still to come": ("if (slot->used) TC_DEV(dev.stream_wait(ks, slot->last));", ";"),
    "a scatter does not wait for its DMA": ("                    TC_DEV(dev.stream_wait(kstream, slot->ready));", ""),
    "the table is rewritten before the last scatter": (
        "            if (overlapped && final_slot) TC_DEV(dev.stream_wait(stream, final_slot->last));", ""),
    "the engine's stream starts before the ids are in place": ("                TC_DEV(dev.stream_wait(kstream, op.payload.entry));", ""),
    "a transfer on another stream is not waited for": (
        "            if (dev.stream_wait(stream, book->entries()[at].payload.done)) return TC_ERR_HIP;", ";"),
    "an upload's DMA overwrites a slot whose scatter is still to come": ("if (slot->used) TC_DEV(dev.stream_wait(stream, slot->last));", ";"),
    "a failed transfer's completion does not cover the engine's stream": (
        "covered = dev.event_record(op.payload.entry, kstream) == 0 && dev.stream_wait(stream, op.payload.entry) == 0;", "covered = true;"),
}


def test_ordering_mistakes_planted_in_the_engine_are_caught(tmp_path):
    """The stand-in device of tests/csrc/engine_emul.cpp runs queued work in adversarial orders.  That this finds a
    missing event wait is itself checked: each wait the engine relies on is taken out of a copy of
    csrc/tc_engine_core.h in turn, and every such build must fail the stand-in's tests (CPU only, memory-safe:
    the stand-in works on heap buffers)."""
    import shutil
    from concurrent.futures import ThreadPoolExecutor
    import oracle
    csrc = os.path.join(ROOT, "paper_2510_18586_amd", "csrc")
    obj = str(tmp_path / "tc_oracle.o")
    subprocess.run(["gcc", "-std=c11", "-O1", "-c", os.path.join(os.path.dirname(oracle.__file__), "tc_oracle.c"), "-o", obj], check=True)
    text = open(os.path.join(csrc, "tc_engine_core.h")).read()

    def build_and_run(item):
        k, (name, (old, new)) = item
        d = tmp_path / f"m{k}"
        d.mkdir()
        for h in os.listdir(csrc):
            if h.endswith(".h"):
                shutil.copy(os.path.join(csrc, h), d / h)
        assert text.count(old) >= 1, name
        (d / "tc_engine_core.h").write_text(text.replace(old, new, 1))
        exe = str(d / "emul")
        subprocess.run(["g++", "-std=c++17", "-O1", "-I", os.path.join(ROOT, "include"), "-I", str(d),
                        os.path.join(HERE, "csrc", "engine_emul.cpp"), obj, "-o", exe], check=True)
        out = subprocess.run([exe], capture_output=True, text=True, timeout=300)
        return name, out.returncode, out.stdout[-300:]

    with ThreadPoolExecutor(4) as pool:
        results = list(pool.map(build_and_run, enumerate(ORDERING_MISTAKES.items())))
    for name, rc, tail in results:
        assert rc != 0 and "FAILED" in tail, f"not caught: {name}: {tail}"
