"""Pins for the oracle's bookkeeping model (no GPU).

What the paper fixes (Sec. 6.3): a block released while a copy that reads it is in flight
is *pending-free* and goes back on the free list no earlier than the end of that copy; CPU
blocks are recycled through a free list; the original GPU block can be claimed again.
The rest are conservation laws checked against plain sets under seeded random op streams,
plus hand-worked examples of the LIFO order chosen here.
"""
import numpy as np
import pytest

from oracle import OracleBlockPool, OracleHostArena, OracleError


def test_hand_worked_lifo_order():
    bp = OracleBlockPool(8)
    assert bp.alloc(3) == [0, 1, 2]
    bp.free([1])
    assert bp.alloc(2) == [1, 3]
    bp.free([0, 2])            # pushed in the order given: 2 ends on top
    assert bp.alloc(3) == [2, 0, 4]
    with pytest.raises(OracleError) as e:
        bp.alloc(4)            # 5, 6, 7 left only
    assert e.value.code == "NOMEM"
    assert bp.n_free() == 3    # all-or-nothing: nothing was taken
    assert bp.alloc(3) == [5, 6, 7]


def test_pending_free_until_transfer_completes():
    bp = OracleBlockPool(4)
    ids = bp.alloc(4)
    bp.begin_op(ids[:2])       # copy of blocks 0, 1 issued
    bp.free(ids[:2])           # released right away, as the paper does
    assert bp.n_pending() == 2 and bp.n_free() == 0
    with pytest.raises(OracleError):
        bp.alloc(1)            # not reusable while still being read
    bp.retire_oldest()
    assert bp.n_pending() == 0 and bp.n_free() == 2
    assert bp.alloc(2) == [1, 0]


def test_two_reads_of_one_block_both_must_finish():
    bp = OracleBlockPool(2)
    bp.alloc(2)
    bp.begin_op([0])
    bp.begin_op([0, 1])
    bp.free([0])
    bp.retire_oldest()
    assert bp.n_pending() == 1 and bp.n_free() == 0
    bp.retire_oldest()
    assert bp.n_pending() == 0 and bp.n_free() == 1


def test_shared_prefix_blocks_do_not_move():
    bp = OracleBlockPool(8)
    prefix = bp.alloc(2)
    bp.ref(prefix)             # second owner
    private = bp.alloc(3)
    with pytest.raises(OracleError) as e:
        bp.check_transfer(prefix + private)
    assert e.value.code == "SHARED"
    assert bp.filter_private(prefix + private) == private
    bp.free(prefix)
    bp.check_transfer(prefix)  # one owner left: movable again
    assert bp.n_shared() == 0


def test_transfer_validation_codes():
    bp = OracleBlockPool(8)
    ids = bp.alloc(3)
    for bad, code in (([0, 8], "RANGE"), ([-1], "RANGE"), ([0, 1, 0], "DUP"), ([0, 5], "INVAL")):
        with pytest.raises(OracleError) as e:
            bp.begin_op(bad)
        assert e.value.code == code
    assert not bp.ops and bp.inflight == [0] * 8
    with pytest.raises(OracleError) as e:
        bp.free([0, 0])
    assert e.value.code == "INVAL" and bp.refcount[0] == 1
    bp.begin_op(ids)


def test_alloc_at_reclaims_original_blocks():
    bp = OracleBlockPool(8)
    a = bp.alloc(4)
    bp.free(a[1:3])
    bp.alloc_at([2, 1])
    assert bp.refcount[1] == 1 and bp.refcount[2] == 1
    with pytest.raises(OracleError) as e:
        bp.alloc_at([4, 0])    # 0 is held
    assert e.value.code == "NOMEM" and bp.refcount[4] == 0 and 4 in bp.free_stack
    assert bp.alloc(2) == [4, 5]


def test_random_ops_conserve_blocks():
    rng = np.random.default_rng(20251018)
    NB = 97
    bp = OracleBlockPool(NB)
    held = []                  # list of lists
    in_flight = []             # ids of unretired ops, oldest first
    handed_out = set()
    for step in range(6000):
        r = rng.random()
        if r < 0.35:
            n = int(rng.integers(0, 12))
            try:
                got = bp.alloc(n)
            except OracleError as e:
                assert e.code == "NOMEM" and n > bp.n_free()
            else:
                assert len(got) == n and not (set(got) & handed_out)
                for op in in_flight:      # never a block that is still being read
                    assert not (set(got) & op)
                handed_out |= set(got)
                if got:
                    held.append(got)
        elif r < 0.6 and held:
            k = int(rng.integers(len(held)))
            ids = held.pop(k)
            if rng.random() < 0.5:
                bp.begin_op(ids)
                in_flight.append(set(ids))
            bp.free(ids)
            handed_out -= set(ids)
        elif r < 0.8 and in_flight:
            bp.retire_oldest()
            in_flight.pop(0)
        assert bp.n_free() + bp.n_used() + bp.n_pending() == NB
        assert bp.n_used() == len(handed_out)
        assert len(set(bp.free_stack)) == len(bp.free_stack)
        assert min(bp.refcount) >= 0
    bp.retire_all()
    for ids in held:
        bp.free(ids)
    assert bp.n_free() == NB and bp.n_pending() == 0


def test_host_arena_first_fit_and_merge():
    ar = OracleHostArena(10)
    a = ar.alloc(3)
    b = ar.alloc(4)
    c = ar.alloc(3)
    assert (a, b, c) == (0, 3, 7) and ar.used_slots() == 10
    with pytest.raises(OracleError) as e:
        ar.alloc(1)
    assert e.value.code == "HOST_NOMEM"
    ar.free(a)
    ar.free(c)
    with pytest.raises(OracleError):
        ar.alloc(4)            # 3 + 3 free but not adjacent
    assert ar.alloc(2) == 0    # lowest address that fits
    ar.free(b)                 # merges with [2,3) and [7,10)
    assert ar.free_runs == [(2, 8)]
    assert ar.alloc(8) == 2
    assert ar.alloc(0) is None
    ar.free(None)
    with pytest.raises(OracleError):
        ar.free(5)             # not the start of an allocation


def test_host_arena_deferred_release():
    ar = OracleHostArena(4)
    a = ar.alloc(4)
    ar.begin_op(a)
    ar.free(a)
    assert ar.used_slots() == 4
    with pytest.raises(OracleError):
        ar.free(a)             # already released once
    ar.end_op(a)
    assert ar.used_slots() == 0 and ar.free_runs == [(0, 4)]


def test_host_arena_random_ops_no_overlap():
    rng = np.random.default_rng(77)
    N = 200
    ar = OracleHostArena(N)
    live = {}
    for _ in range(3000):
        if rng.random() < 0.55:
            n = int(rng.integers(1, 30))
            try:
                s = ar.alloc(n)
            except OracleError:
                # no free run of n slots may exist
                occ = np.zeros(N, dtype=bool)
                for st, ln in live.items():
                    occ[st:st + ln] = True
                run = best = 0
                for o in occ:
                    run = 0 if o else run + 1
                    best = max(best, run)
                assert best < n
            else:
                for st, ln in live.items():
                    assert s + n <= st or st + ln <= s
                live[s] = n
        elif live:
            s = list(live)[int(rng.integers(len(live)))]
            ar.free(s)
            del live[s]
        assert ar.used_slots() == sum(live.values())
        assert ar.used_slots() + sum(l for _, l in ar.free_runs) == N


# ---- alloc_prefer: an upload takes its original GPU blocks again where it still can (Sec. 6.3) ----

def test_alloc_prefer_hand_worked():
    bp = OracleBlockPool(8)
    bp.alloc(8)
    bp.free([5, 2, 7])                       # stack top: 7, then 2, then 5
    assert bp.alloc_prefer([2, 4, 5]) == [2, 7, 5]    # 2 and 5 are free again, 4 is taken: fresh block 7
    assert bp.n_free() == 0
    with pytest.raises(OracleError) as e:
        bp.alloc_prefer([1])
    assert e.value.code == "NOMEM"


def test_alloc_prefer_reduces_to_alloc_at_plus_alloc():
    """Against routines pinned above: claiming the free preferred ids with alloc_at and popping the rest
    with alloc gives the same ids in the same places and leaves the same free list."""
    rng = np.random.default_rng(77)
    for trial in range(200):
        NB = int(rng.integers(1, 24))
        a, b = OracleBlockPool(NB), OracleBlockPool(NB)
        taken = [int(x) for x in rng.permutation(NB)[:int(rng.integers(0, NB + 1))]]
        for bp in (a, b):
            bp.alloc_at(taken)
        back = [int(x) for x in rng.permutation(taken)[:int(rng.integers(0, len(taken) + 1))]]
        for bp in (a, b):
            bp.free(back)
        n = int(rng.integers(0, NB + 2))
        pref = [int(x) for x in rng.integers(-2, NB + 2, size=n)]       # repeats, taken and bad ids included
        if n > a.n_free():
            before = list(a.free_stack)
            with pytest.raises(OracleError):
                a.alloc_prefer(pref)
            assert a.free_stack == before and a.refcount == b.refcount  # all or nothing
            continue
        got = a.alloc_prefer(pref)
        seen, claim = set(), []
        for x in pref:
            ok = 0 <= x < NB and b.refcount[x] == 0 and not b.pending[x] and x not in seen
            claim.append(ok)
            if ok:
                seen.add(x)
        b.alloc_at([x for x, ok in zip(pref, claim) if ok])
        fresh = iter(b.alloc(n - sum(claim)))
        want = [x if ok else next(fresh) for x, ok in zip(pref, claim)]
        assert got == want, (trial, pref)
        assert a.free_stack == b.free_stack and a.refcount == b.refcount


def test_alloc_prefer_never_takes_a_pending_free_block():
    bp = OracleBlockPool(4)
    ids = bp.alloc(2)                        # 0, 1
    bp.begin_op(ids)
    bp.free(ids)                             # both pending-free while the copy reads them
    assert bp.alloc_prefer([0, 1]) == [2, 3]
    bp.retire_all()
    assert sorted(bp.free_stack) == [0, 1]
