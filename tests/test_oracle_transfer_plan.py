"""Pins for the oracle's model of the host-side transfer planning (oracle/transfer_plan.py), CPU only.

Hand-worked cases, brute force over every record, and invariants that any correct ring / chunk plan /
hazard rule has to keep (no ring entry with two owners, every record carried exactly once, a transfer
never overtakes the last one that touched its blocks from another stream).  Paper Sec. 6.3 fixes only
the principle (nothing a copy may still read is reused before the copy is done); the readings are
listed at the top of the model.
"""
import numpy as np

import oracle.transfer_plan as T


# ---------------------------------------------------------------- id ring
def test_ring_hand_worked():
    r = T.OracleIdRing(10)
    assert r.alloc(4) == 0 and r.alloc(4) == 4
    assert r.alloc(4) is None                      # 2 entries left before the end, 4 do not fit after wrapping either
    assert r.alloc(2) == 8 and r.used() == 10
    assert r.alloc(1) is None
    assert r.release_oldest() == (0, 4, 0)
    assert r.alloc(3) == 0 and r.used() == 9       # the tail is at 0 again: nothing skipped
    assert r.release_oldest() == (4, 4, 0) and r.release_oldest() == (8, 2, 0)
    assert r.alloc(7) == 3 and r.used() == 10
    assert r.release_oldest() == (0, 3, 0)
    assert r.alloc(3) == 0 and r.live[-1] == (0, 3, 0)
    r = T.OracleIdRing(10)
    assert r.alloc(6) == 0 and r.release_oldest() and r.alloc(3) == 0   # an empty ring starts at 0 again
    assert r.alloc(6) == 3 and r.release_oldest() == (0, 3, 0)
    assert r.alloc(3) == 0 and r.live[-1] == (0, 3, 1)                  # entry 9 is skipped and stays held
    assert r.used() == 10 and r.alloc(1) is None
    assert r.release_oldest() == (3, 6, 0) and r.alloc(1) == 3 and r.used() == 5
    assert r.cancel_newest() == (3, 1, 0) and r.alloc(2) == 3           # a cancelled span leaves no trace
    try:
        r.alloc(11)
        assert False
    except ValueError:
        pass


def test_ring_entries_never_have_two_owners():
    rng = np.random.default_rng(5)
    for cap in (7, 16, 100):
        r = T.OracleIdRing(cap)
        for _ in range(4000):
            if rng.random() < 0.55 or not r.live:
                n = int(rng.integers(1, max(2, cap // 2)))
                before = list(r.live)
                start = r.alloc(n)
                if start is None:
                    assert r.live == before and r.live          # refused: nothing changed, and a release will help
                else:
                    assert 0 <= start and start + n <= cap      # contiguous, inside the ring
            elif rng.random() < 0.9:
                r.release_oldest()
            else:
                r.cancel_newest()
            held = r.entries_held()
            assert len(held) == len(set(held)) and r.used() <= cap
            assert r.used() >= len(held)
        while r.live:
            r.release_oldest()
        assert r.alloc(cap) == 0                                # an empty ring takes a request of its whole size


# ---------------------------------------------------------------- chunks and pieces
def test_chunks_hand_worked():
    assert T.plan_chunks(0, 4, False) == []
    assert T.plan_chunks(10, 4, False) == [4, 4, 2] and T.plan_chunks(10, 4, True) == [2, 4, 4]
    assert T.plan_chunks(8, 4, True) == [4, 4] and T.plan_chunks(3, 4, False) == [3]
    for total in range(0, 40):
        for slot in (1, 3, 8):
            for up in (False, True):
                sizes = T.plan_chunks(total, slot, up)
                assert sum(sizes) == total and all(0 < s <= slot for s in sizes)
                assert len(sizes) == -(-total // slot)
    # the two directions cut the record list at mirrored places
    cuts = lambda sizes: set(np.cumsum(sizes).tolist())
    assert cuts(T.plan_chunks(10, 4, False)) != cuts(T.plan_chunks(10, 4, True))   # 4,8,10 against 2,6,10: mirrored
    assert cuts(T.plan_chunks(10, 4, False)) == {10 - c for c in cuts(T.plan_chunks(10, 4, True)) if c != 10} | {10}


def test_chunks_with_a_short_first_chunk():
    # hand-worked: 2 records ahead of full slots of 4; nothing changes for lists of at most twice the head
    assert T.plan_chunks(10, 4, False, 2) == [2, 4, 4] and T.plan_chunks(10, 4, True, 2) == [4, 4, 2]
    assert T.plan_chunks(11, 4, False, 2) == [2, 4, 4, 1] and T.plan_chunks(11, 4, True, 2) == [1, 4, 4, 2]
    assert T.plan_chunks(4, 4, False, 2) == [4] and T.plan_chunks(5, 4, False, 2) == [2, 3]
    assert T.plan_chunks(3, 8, False, 1) == [1, 2] and T.plan_chunks(2, 8, False, 1) == [2]
    assert T.plan_chunks(20, 4, False, 6) == [4, 4, 4, 4, 4]            # a head is never longer than a slot
    assert T.plan_chunks(9, 4, False, 0) == [4, 4, 1]
    for total in range(0, 60):
        for slot in (1, 3, 8):
            for head in (0, 1, 2, 5, 9):
                off, up = T.plan_chunks(total, slot, False, head), T.plan_chunks(total, slot, True, head)
                assert up == off[::-1] and sum(off) == total and all(0 < s <= slot for s in off)
                h = min(head, slot)
                if h and total > 2 * h:
                    assert off[0] == h and off[1:] == T.plan_chunks(total - h, slot, False)
                else:
                    assert off == T.plan_chunks(total, slot, False)


def test_a_staged_transfer_overlaps_only_if_there_is_something_to_overlap():
    assert T.plan_staged(4, 8, False, 2, 1) == ([4], False)              # at most twice the head: one chunk, in line
    assert T.plan_staged(5, 8, False, 2, 1) == ([2, 3], True) and T.plan_staged(5, 8, True, 2, 1) == ([3, 2], True)
    assert T.plan_staged(5, 8, False, 2, 0) == ([5], False)              # not asked for: the plain cut
    assert T.plan_staged(20, 8, False, 2, 0) == ([8, 8, 4], False) and T.plan_staged(20, 8, True, 2, 1) == ([2, 8, 8, 2], True)
    assert T.plan_staged(20, 8, False, 0, 1) == ([8, 8, 4], True) and T.plan_staged(8, 8, False, 0, 1) == ([8], False)
    assert T.plan_staged(0, 8, False, 2, 1) == ([], False)


def test_pieces_carry_every_record_once():
    rng = np.random.default_rng(6)
    assert T.chunk_pieces([(0, 5), (5, 3)], 3, 7) == [(0, 3, 0, 2), (1, 0, 2, 2)]
    assert T.chunk_pieces([(0, 5), (5, 3)], 5, 8) == [(1, 0, 0, 3)]
    for _ in range(300):
        lens = rng.integers(1, 9, size=int(rng.integers(1, 7)))
        segs, first = [], 0
        for n in lens:
            segs.append((first, int(n)))
            first += int(n)
        total, slot = first, int(rng.integers(1, 10))
        up = bool(rng.integers(0, 2))
        seen = {}
        c0 = 0
        for size in T.plan_chunks(total, slot, up):
            in_chunk = set()
            for k, in_seg, in_ch, n in T.chunk_pieces(segs, c0, c0 + size):
                for j in range(n):
                    rec = segs[k][0] + in_seg + j              # position in the list, by way of the buffer
                    assert rec == c0 + in_ch + j               # and by way of the chunk: the same record
                    assert 0 <= in_seg + j < segs[k][1] and 0 <= in_ch + j < size
                    assert rec not in seen
                    seen[rec] = True
                    in_chunk.add(in_ch + j)
            assert in_chunk == set(range(size))
            c0 += size
        assert sorted(seen) == list(range(total))


def test_host_tail_hand_worked():
    assert T.host_tail_split(0, 0, 16, [(0, 16)]) == (16, None, None)
    assert T.host_tail_split(4, 0, 16, [(0, 16)]) == (12, 0, 12)
    assert T.host_tail_split(4, 8, 16, [(0, 40)]) == (12, 0, 20)          # chunk [8, 24), tail [20, 24)
    assert T.host_tail_split(4, 0, 3, [(0, 3)]) == (3, None, None)        # fewer records than the divisor
    assert T.host_tail_split(4, 0, 16, [(0, 13), (13, 3)]) == (16, None, None)     # tail [12, 16) straddles two buffers
    assert T.host_tail_split(4, 0, 16, [(0, 12), (12, 10)]) == (12, 1, 0)          # tail starts the second buffer
    assert T.host_tail_split(64, 0, 256, [(0, 256)]) == (252, 0, 252)
    assert T.host_tail_split(3, 0, 8, [(0, 8)]) == (6, 0, 6)              # 8 // 3 = 2 records


# ---------------------------------------------------------------- hazards
def test_hazards_hand_worked():
    ops = [(1, "a", {1, 2}, {0}), (2, "b", {2, 3}, set()), (3, "a", {9}, {40})]
    assert T.hazard_waits(ops, "a", [1], []) == set()            # same stream: order is implicit
    assert T.hazard_waits(ops, "b", [1], []) == {1}
    assert T.hazard_waits(ops, "a", [2], []) == {2}              # the LAST toucher counts, not the first
    assert T.hazard_waits(ops, "b", [2], []) == set()            # ... and it is on the caller's stream
    assert T.hazard_waits(ops, "c", [2, 9], [0]) == {1, 2, 3}
    assert T.hazard_waits(ops, "c", [7], [8]) == set()
    assert T.hazard_waits([], "a", [1], [0]) == set()
    assert T.hazard_waits(ops, "b", [], [40]) == {3}


def test_hazard_waits_cover_every_conflict():
    """Waiting for the returned tickets (plus stream order) puts the new transfer after EVERY earlier transfer
    that touched one of its blocks or its host allocation."""
    rng = np.random.default_rng(8)
    for _ in range(300):
        book = T.OracleTransferBook(10000)
        order_after = {}                       # ticket -> set of tickets it is ordered after (transitively)
        for _ in range(int(rng.integers(1, 12))):
            stream = int(rng.integers(0, 3))
            ids = rng.choice(12, size=int(rng.integers(1, 5)), replace=False).tolist()
            arena = [int(rng.integers(0, 4))]
            start, waits = book.begin(stream, ids, arena)
            earlier = [o for o in book.ops]
            t = book.publish()
            after = set()
            for o in earlier:
                if o["stream"] == stream or o["ticket"] in waits:
                    after |= {o["ticket"]} | order_after[o["ticket"]]
            order_after[t] = after
            for o in earlier:
                if set(o["ids"]) & set(ids) or set(o["arena"]) & set(arena):
                    assert o["ticket"] in after, "a conflicting transfer may still be running"


# ---------------------------------------------------------------- paths
def test_paths_truth_table():
    MiB = 1 << 20
    assert T.upload_path(T.PATH_AUTO) == T.DIRECT and T.upload_path(T.PATH_DIRECT) == T.DIRECT
    assert T.upload_path(T.PATH_STAGED) == T.STAGED
    for up in (False, True):
        assert T.offload_path(T.PATH_DIRECT, 1 << 40, up, 128 * MiB) == T.DIRECT
        assert T.offload_path(T.PATH_STAGED, 1, up, 128 * MiB) == T.STAGED
    assert T.offload_path(T.PATH_DIRECT_IF_DUPLEX, 1, False, 128 * MiB) == T.STAGED
    assert T.offload_path(T.PATH_DIRECT_IF_DUPLEX, 1 << 40, True, 128 * MiB) == T.DIRECT
    assert T.offload_path(T.PATH_AUTO, 128 * MiB - 1, False, 128 * MiB) == T.DIRECT
    assert T.offload_path(T.PATH_AUTO, 128 * MiB, False, 128 * MiB) == T.STAGED      # the threshold itself is staged
    assert T.offload_path(T.PATH_AUTO, 1 << 40, True, 128 * MiB) == T.DIRECT
    assert T.tail_divisor(0, 1) == 0 and T.tail_divisor(0, 2) == 64 and T.tail_divisor(0, 9, auto_div=32) == 32
    assert T.tail_divisor(1, 5) == 0 and T.tail_divisor(48, 1) == 48 and T.tail_divisor(2, 3) == 2
    # kernels on their own stream already keep the link busy: no automatic tail then, an explicit one stays
    assert T.tail_divisor(0, 2, overlapped=True) == 0 and T.tail_divisor(0, 9, True) == 0
    assert T.tail_divisor(16, 2, overlapped=True) == 16 and T.tail_divisor(1, 2, True) == 0
    assert [T.kernels_overlap_copies(1, n) for n in (1, 2, 7)] == [False, True, True]
    assert [T.kernels_overlap_copies(0, n) for n in (1, 2, 7)] == [False, False, False]


# ---------------------------------------------------------------- what a failed enqueue keeps
def test_a_half_enqueued_transfer_keeps_what_it_holds():
    book = T.OracleTransferBook(8)
    start, waits = book.begin("s", [3, 4, 5], [0])
    assert start == 0 and waits == set()
    book.publish(failed=True)                    # part of it reached the stream before the runtime refused
    start2, waits2 = book.begin("t", [4], [0])   # the kernels of the failed transfer may still read block 4 and entries 0..2
    assert start2 == 3 and waits2 == {1}
    book.publish()
    assert sorted(book.ring.entries_held()) == [0, 1, 2, 3]
    assert book.begin("s", [1, 2, 6, 7, 0], [])[0] is None       # 4 entries left, 5 wanted: retire first
    assert book.retire_oldest()["failed"] is True
    assert book.begin("s", [1, 2, 6, 7, 0], [])[0] is None       # entries 4..7 are free, but a span does not wrap around
    assert book.retire_oldest()["ticket"] == 2
    assert book.begin("s", [1, 2, 6, 7, 0], [])[0] == 0          # empty ring: from the start
    book.cancel()                                                # nothing reached the stream: the span goes back at once
    assert book.ring.entries_held() == [] and book.begin("s", [9], [])[0] == 0


def test_upload_in_flight_is_what_switches_the_offload_path():
    book = T.OracleTransferBook(64)
    book.begin("s", [1], [], upload=False)
    book.publish()
    assert not book.upload_in_flight()
    book.begin("t", [2], [], upload=True)
    book.publish()
    assert book.upload_in_flight()
    book.retire_oldest()
    assert book.upload_in_flight()
    book.retire_oldest()
    assert not book.upload_in_flight()
