"""Model of the host-side planning around a transfer.  TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Deliberately naive Python for what the library decides on the host before and after it enqueues the
copies of paper Sec. 6.3 (asynchronous migration on a dedicated stream; nothing a copy may still read
is reused before that copy has completed): where a transfer's ids sit in the fixed ring of device ids,
how its records are cut into staging chunks and per-buffer copies, which earlier transfers a new one
has to wait for, which path it takes, and what stays held when enqueueing fails half-way.

Readings where the paper is silent (it describes no mechanism at this level):
* id ring: entries are handed out in address order; a request that does not fit before the end of the
  ring starts again at entry 0 and the skipped tail stays unusable until that request is released; an
  empty ring starts at 0; releases come oldest first; a held span is never handed out again.
* chunks: full staging slots first, the remainder last; an upload takes the remainder first, so both
  directions cut the record list at the same places.
* hazards: a transfer waits for the LAST earlier transfer, still in flight, that touched one of its
  blocks or its host allocation, if that one was put on another stream (same-stream order is implicit).
* paths: an upload goes through the copy kernel that reads pinned memory itself unless told otherwise;
  an offload does so while an upload of the same context is in flight (the two then share the link
  instead of taking turns) or when it is below a size the caller may set (none by default), and through
  device staging plus DMA otherwise.
* a transfer whose enqueue failed after part of it was handed to the stream keeps everything it holds
  (ring span, in-flight marks, host allocation) until it is retired like any other transfer.
"""

PATH_AUTO, PATH_DIRECT, PATH_DIRECT_IF_DUPLEX, PATH_STAGED = 0, 1, 2, 3
STAGED, DIRECT = "staged", "direct"


class OracleIdRing:
    """cap entries; spans are (start, n, skipped) oldest first."""

    def __init__(self, cap):
        self.cap = int(cap)
        self.live = []

    def used(self):
        return sum(n + skipped for _, n, skipped in self.live)

    def _tail(self):
        if not self.live:
            return 0
        start, n, _ = self.live[-1]
        return (start + n) % self.cap

    def alloc(self, n):
        """Start entry of n consecutive entries, or None when they do not fit right now."""
        n = int(n)
        if n > self.cap:
            raise ValueError("larger than the ring")
        tail = self._tail()
        skipped = 0
        start = tail
        if tail + n > self.cap:
            skipped = self.cap - tail
            start = 0
        if self.used() + skipped + n > self.cap:
            return None
        self.live.append((start, n, skipped))
        return start

    def release_oldest(self):
        return self.live.pop(0)

    def cancel_newest(self):
        return self.live.pop()

    def entries_held(self):
        """Every ring entry some live span owns (the pins check that no entry has two owners)."""
        out = []
        for start, n, _ in self.live:
            out.extend(range(start, start + n))
        return out


def plan_chunks(total, slot_blocks, upload, head_blocks=0):
    """Sizes, in blocks, of the staging chunks a list of `total` records is cut into: full slots, then what is
    left.  With head_blocks > 0 a list of more than twice that many records starts with a short chunk of
    head_blocks records (at most a slot): while it crosses the link the copy kernel is already at work on the
    next one, so only a short kernel runs with the link idle.  An upload takes the same sizes in reverse order:
    its last kernel, the one nothing hides, is the short one."""
    left = int(total)
    sizes = []
    head = min(int(head_blocks), int(slot_blocks))
    if head > 0 and left > 2 * head:
        sizes.append(head)
        left -= head
    while left > 0:
        take = min(int(slot_blocks), left)
        sizes.append(take)
        left -= take
    return sizes[::-1] if upload else sizes


def chunk_pieces(segments, c0, c1):
    """segments: [(first_record_in_list, n_records)] per host buffer, in list order.  The copies that carry
    records [c0, c1) of the list: (segment index, first record inside the segment's buffer, first record
    inside the chunk, how many), one per buffer the chunk touches."""
    out = []
    for k, (first, n) in enumerate(segments):
        a, b = max(first, c0), min(first + n, c1)
        if a < b:
            out.append((k, a - first, a - c0, b - a))
    return out


def host_tail_split(div, c0, nblk, segments):
    """With a tail divisor `div` >= 2 the last nblk // div records of the chunk [c0, c0 + nblk) cross the link
    inside the copy launch, if the chunk has at least div records and those records lie in one host buffer.
    Returns (records that still go through staging, segment index, first record inside that buffer), the last
    two None when there is no tail."""
    if div < 2 or nblk < div:
        return nblk, None, None
    m = nblk // div
    first = c0 + nblk - m
    for k, (s_first, s_n) in enumerate(segments):
        if first >= s_first and c0 + nblk <= s_first + s_n:
            return nblk - m, k, first - s_first
    return nblk, None, None


def hazard_waits(in_flight, stream, block_ids, arena_starts):
    """in_flight: [(ticket, stream, set(block ids), set(arena starts))] oldest first.  The tickets the new
    transfer has to wait for."""
    waits = set()
    for what, index in ((block_ids, 2), (arena_starts, 3)):
        for x in what:
            last = None
            for op in in_flight:
                if x in op[index]:
                    last = op
            if last is not None and last[1] != stream:
                waits.add(last[0])
    return waits


def offload_path(mode, total_bytes, upload_in_flight, auto_direct_bytes):
    if mode == PATH_DIRECT:
        return DIRECT
    if mode == PATH_STAGED:
        return STAGED
    if mode == PATH_DIRECT_IF_DUPLEX:
        return DIRECT if upload_in_flight else STAGED
    return DIRECT if (upload_in_flight or total_bytes < auto_direct_bytes) else STAGED


def upload_path(mode):
    return STAGED if mode == PATH_STAGED else DIRECT


def kernels_overlap_copies(option, n_chunks):
    """Whether a staged transfer runs its copy kernels on the engine's own stream, so that the kernel of one chunk
    overlaps with the link copy of its neighbour: option 1 asks for it, and it happens for transfers of more than
    one chunk (a single chunk has nothing to overlap with, and the hop between streams would only delay it);
    option 0 (the default) keeps everything in line on the caller's stream."""
    return option == 1 and n_chunks > 1


def plan_staged(total, slot_blocks, upload, head_blocks, overlap_option):
    """(chunk sizes, whether the kernels overlap with the copies) of a staged transfer: the cut with a short first
    chunk if that yields something to overlap, else the plain cut with everything in line."""
    sizes = plan_chunks(total, slot_blocks, upload, head_blocks)
    if kernels_overlap_copies(overlap_option, len(sizes)):
        return sizes, True
    return plan_chunks(total, slot_blocks, upload, 0), False


def tail_divisor(option, n_chunks, overlapped=False, auto_div=64):
    """option 0 = automatic, 1 = never, N >= 2 = 1/N.  Automatic: a tail where the link would otherwise idle once
    per chunk, i.e. in transfers of more than one chunk whose kernels run in line with their copies."""
    if option == 0:
        return auto_div if (n_chunks > 1 and not overlapped) else 0
    return 0 if option == 1 else option


class OracleTransferBook:
    """Transfers in flight, oldest first, and what each of them holds."""

    def __init__(self, ring_cap):
        self.ring = OracleIdRing(ring_cap)
        self.ops = []            # dicts: ticket, stream, ids, arena, failed
        self.next_ticket = 1

    def begin(self, stream, ids, arena_starts, upload=False):
        """Returns (ring start or None when the oldest transfer has to be retired first, tickets to wait for).
        Nothing is held yet when the start is None."""
        waits = hazard_waits([(o["ticket"], o["stream"], set(o["ids"]), set(o["arena"])) for o in self.ops],
                             stream, ids, arena_starts)
        start = self.ring.alloc(len(ids))
        if start is None:
            return None, waits
        self._pending = dict(stream=stream, ids=list(ids), arena=list(arena_starts), start=start, upload=bool(upload))
        return start, waits

    def publish(self, failed=False):
        op = self._pending
        op.update(ticket=self.next_ticket, failed=failed)
        self.next_ticket += 1
        self.ops.append(op)
        self._pending = None
        return op["ticket"]

    def cancel(self):
        """Nothing of the transfer reached the stream: its ring span goes back at once."""
        self.ring.cancel_newest()
        self._pending = None

    def retire_oldest(self):
        self.ring.release_oldest()
        return self.ops.pop(0)

    def upload_in_flight(self):
        return any(o.get("upload") for o in self.ops)
