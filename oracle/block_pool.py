"""Bookkeeping model for the oracle.  TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

A deliberately naive model of the block bookkeeping around KV migration
(paper Sec. 6.3 "CPU Migration Infrastructure"):

* source GPU blocks of an issued copy become *pending-free* when released and go
  back to the free pool only once the transfer has completed;
* the CPU side is a pool of fixed-size blocks recycled through a free list and
  never handed back to the operating system;
* on upload the original GPU block may be claimed again when it is still free.

Readings where the paper is silent: the GPU free list is a LIFO stack that first
hands out 0, 1, 2, ...; a release pushes ids in the order given; transfers retire
in issue order; the host arena hands out the lowest-addressed run of contiguous
fixed-size slots that fits (first fit) and merges neighbours on release.
"""


class OracleError(Exception):
    def __init__(self, code, msg=""):
        super().__init__(f"{code}: {msg}" if msg else code)
        self.code = code


class OracleBlockPool:
    def __init__(self, num_blocks):
        self.NB = int(num_blocks)
        self.refcount = [0] * self.NB
        self.inflight = [0] * self.NB
        self.pending = [False] * self.NB
        self.free_stack = list(range(self.NB - 1, -1, -1))  # top of stack = end of list
        self.ops = []          # [(ticket, [ids])] in issue order
        self.next_ticket = 1

    # ---- queries ---------------------------------------------------------
    def n_free(self):
        return len(self.free_stack)

    def n_used(self):
        return sum(1 for r in self.refcount if r > 0)

    def n_pending(self):
        return sum(1 for p in self.pending if p)

    def n_shared(self):
        return sum(1 for r in self.refcount if r > 1)

    # ---- helpers ---------------------------------------------------------
    def _check_range(self, ids):
        for b in ids:
            if b < 0 or b >= self.NB:
                raise OracleError("RANGE", f"block id {b}")

    @staticmethod
    def _check_dup(ids):
        if len(set(ids)) != len(ids):
            raise OracleError("DUP")

    # ---- allocation ------------------------------------------------------
    def alloc(self, n):
        if n > len(self.free_stack):
            raise OracleError("NOMEM")
        out = [self.free_stack.pop() for _ in range(n)]
        for b in out:
            self.refcount[b] = 1
        return out

    def alloc_at(self, ids):
        ids = [int(b) for b in ids]
        self._check_range(ids)
        self._check_dup(ids)
        for b in ids:
            if self.refcount[b] != 0 or self.pending[b]:
                raise OracleError("NOMEM", f"block {b} is not free")
        for b in ids:
            self.free_stack.remove(b)
            self.refcount[b] = 1

    def alloc_prefer(self, preferred):
        """n blocks, all or nothing: preferred[i] itself wherever it is still free (the original GPU
        block is taken again where it still can be), a fresh block from the free list for the rest.  The
        preferred ids are claimed first, in order; the gaps are then filled in order.  An id that is
        out of range, taken, pending-free or named earlier in the call is simply no preference."""
        preferred = [int(b) for b in preferred]
        if len(preferred) > len(self.free_stack):
            raise OracleError("NOMEM")
        out = [None] * len(preferred)
        for i, b in enumerate(preferred):
            if 0 <= b < self.NB and b in self.free_stack:
                self.free_stack.remove(b)
                self.refcount[b] = 1
                out[i] = b
        for i in range(len(out)):
            if out[i] is None:
                out[i] = self.free_stack.pop()
                self.refcount[out[i]] = 1
        return out

    def ref(self, ids):
        ids = [int(b) for b in ids]
        self._check_range(ids)
        for b in ids:
            if self.refcount[b] < 1:
                raise OracleError("INVAL", f"block {b} is not allocated")
        for b in ids:
            self.refcount[b] += 1

    def free(self, ids):
        ids = [int(b) for b in ids]
        self._check_range(ids)
        drop = {}
        for b in ids:
            drop[b] = drop.get(b, 0) + 1
            if drop[b] > self.refcount[b]:
                raise OracleError("INVAL", f"block {b} released more often than held")
        for b in ids:
            self.refcount[b] -= 1
            if self.refcount[b] == 0:
                if self.inflight[b] > 0:
                    self.pending[b] = True
                else:
                    self.free_stack.append(b)

    # ---- transfers -------------------------------------------------------
    def check_transfer(self, ids):
        """A block can move only if it is allocated and held by exactly one owner."""
        ids = [int(b) for b in ids]
        self._check_range(ids)
        self._check_dup(ids)
        for b in ids:
            if self.refcount[b] == 0:
                raise OracleError("INVAL", f"block {b} is not allocated")
            if self.refcount[b] > 1:
                raise OracleError("SHARED", f"block {b} has {self.refcount[b]} owners")
        return ids

    def begin_op(self, ids):
        ids = self.check_transfer(ids)
        for b in ids:
            self.inflight[b] += 1
        t = self.next_ticket
        self.next_ticket += 1
        self.ops.append((t, ids))
        return t

    def retire_oldest(self):
        """The oldest in-flight transfer has completed."""
        _, ids = self.ops.pop(0)
        for b in ids:
            self.inflight[b] -= 1
            if self.inflight[b] == 0 and self.pending[b]:
                self.pending[b] = False
                self.free_stack.append(b)

    def retire_all(self):
        while self.ops:
            self.retire_oldest()

    def filter_private(self, ids):
        """ids held by exactly one owner, order kept (shared prefix blocks never move)."""
        ids = [int(b) for b in ids]
        self._check_range(ids)
        return [b for b in ids if self.refcount[b] == 1]


class OracleHostArena:
    """Fixed-size host slots; an allocation is a run of contiguous slots."""

    def __init__(self, n_slots):
        self.n_slots = int(n_slots)
        self.free_runs = [(0, self.n_slots)] if self.n_slots else []  # sorted (start, length)
        self.live = {}       # start -> length
        self.inflight = {}   # start -> count
        self.pending = set()

    def used_slots(self):
        return sum(self.live.values())

    def alloc(self, n):
        if n == 0:
            return None
        for k, (start, length) in enumerate(self.free_runs):
            if length >= n:
                if length == n:
                    del self.free_runs[k]
                else:
                    self.free_runs[k] = (start + n, length - n)
                self.live[start] = n
                return start
        raise OracleError("HOST_NOMEM")

    def _release(self, start):
        n = self.live.pop(start)
        runs = sorted(self.free_runs + [(start, n)])
        merged = []
        for s, l in runs:
            if merged and merged[-1][0] + merged[-1][1] == s:
                merged[-1] = (merged[-1][0], merged[-1][1] + l)
            else:
                merged.append((s, l))
        self.free_runs = merged

    def free(self, start):
        if start is None:
            return
        if start not in self.live or start in self.pending:
            raise OracleError("INVAL", f"slot {start} is not the start of a live allocation")
        if self.inflight.get(start, 0) > 0:
            self.pending.add(start)
        else:
            self._release(start)

    def owner_of(self, slot):
        for s, n in self.live.items():
            if s <= slot < s + n:
                return s
        return None

    def begin_op(self, start):
        self.inflight[start] = self.inflight.get(start, 0) + 1

    def end_op(self, start):
        self.inflight[start] -= 1
        if self.inflight[start] == 0 and start in self.pending:
            self.pending.discard(start)
            self._release(start)
