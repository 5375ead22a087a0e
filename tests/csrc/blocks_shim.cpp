// Test-only C shim over the library's host bookkeeping classes (tc_blocks.h), so that the
// free list, reference counts, pending-free rule and host arena can be exercised without a GPU.
#include "tc_blocks.h"
#include "tc_plan.h"

extern "C" {
void *tcb_pool_new(uint32_t nb) { return new tc::BlockPool(nb); }
void tcb_pool_del(void *p) { delete static_cast<tc::BlockPool *>(p); }
int tcb_alloc(void *p, uint32_t n, int32_t *out) { return static_cast<tc::BlockPool *>(p)->alloc(n, out); }
int tcb_alloc_at(void *p, const int32_t *ids, uint32_t n) { return static_cast<tc::BlockPool *>(p)->alloc_at(ids, n); }
int tcb_alloc_prefer(void *p, const int32_t *pref, uint32_t n, int32_t *out) { return static_cast<tc::BlockPool *>(p)->alloc_prefer(pref, n, out); }
int tcb_ref(void *p, const int32_t *ids, uint32_t n) { return static_cast<tc::BlockPool *>(p)->ref(ids, n); }
int tcb_free(void *p, const int32_t *ids, uint32_t n) { return static_cast<tc::BlockPool *>(p)->free(ids, n); }
int tcb_check_transfer(void *p, const int32_t *ids, uint32_t n) { return static_cast<tc::BlockPool *>(p)->check_transfer(ids, n); }
void tcb_begin(void *p, const int32_t *ids, uint32_t n) { static_cast<tc::BlockPool *>(p)->begin_transfer(ids, n); }
void tcb_end(void *p, const int32_t *ids, uint32_t n) { static_cast<tc::BlockPool *>(p)->end_transfer(ids, n); }
int tcb_filter_private(void *p, const int32_t *ids, uint32_t n, int32_t *out, uint32_t *m)
{
    return static_cast<tc::BlockPool *>(p)->filter_private(ids, n, out, m);
}
void tcb_counts(void *p, uint32_t *out4)
{
    auto *b = static_cast<tc::BlockPool *>(p);
    out4[0] = b->n_free(); out4[1] = b->n_used(); out4[2] = b->n_pending(); out4[3] = b->n_shared();
}

// ---- transfer planning (tc_plan.h)
struct NoPayload {};
typedef tc::TransferBook<NoPayload> Book;
void *tcp_book_new(uint64_t ring_cap, uint32_t nb) { return new Book(ring_cap, nb); }
void tcp_book_del(void *b) { delete static_cast<Book *>(b); }
// Returns the ring start, or -1 when the oldest transfer has to be retired first; waits: tickets, *n_waits of them.
int64_t tcp_book_begin(void *bp, uint64_t stream, const int32_t *ids, uint32_t n, const uint64_t *arena, uint32_t n_arena,
                       int upload, uint64_t *waits, uint32_t *n_waits, uint64_t *span3)
{
    Book *b = static_cast<Book *>(bp);
    std::vector<int32_t> v(ids, ids + n);
    std::vector<uint64_t> a(arena, arena + n_arena);
    std::vector<size_t> at;
    b->waits(reinterpret_cast<const void *>(uintptr_t(stream)), v, a, &at);
    *n_waits = uint32_t(at.size());
    for (size_t i = 0; i < at.size(); ++i) waits[i] = b->entries()[at[i]].ticket;
    tc::IdRing::Span s;
    if (!b->ring().alloc(n, &s)) return -1;
    span3[0] = s.start; span3[1] = s.consumed; span3[2] = s.prev_tail;
    (void)upload;
    return int64_t(s.start);
}
uint64_t tcp_book_publish(void *bp, uint64_t stream, const int32_t *ids, uint32_t n, const uint64_t *arena, uint32_t n_arena,
                          int upload, int failed, const uint64_t *span3)
{
    Book::Entry e;
    e.stream = reinterpret_cast<const void *>(uintptr_t(stream));
    e.upload = upload != 0;
    e.failed = failed != 0;
    e.ids.assign(ids, ids + n);
    e.arena_starts.assign(arena, arena + n_arena);
    e.span.start = span3[0]; e.span.consumed = span3[1]; e.span.prev_tail = span3[2];
    return static_cast<Book *>(bp)->publish(std::move(e));
}
void tcp_book_cancel(void *bp, const uint64_t *span3)
{
    tc::IdRing::Span s;
    s.start = span3[0]; s.consumed = span3[1]; s.prev_tail = span3[2];
    static_cast<Book *>(bp)->ring().cancel(s);
}
uint64_t tcp_book_retire(void *bp)
{
    Book *b = static_cast<Book *>(bp);
    const uint64_t t = b->front().ticket;
    b->pop_front();
    return t;
}
uint64_t tcp_book_ring_used(void *bp) { return static_cast<Book *>(bp)->ring().used(); }
int tcp_book_upload_in_flight(void *bp) { return static_cast<Book *>(bp)->upload_in_flight() ? 1 : 0; }
uint32_t tcp_plan_chunks(uint64_t total, uint32_t slot_blocks, int upload, uint32_t head_blocks, uint32_t *out, uint32_t room)
{
    const std::vector<uint32_t> v = tc::plan_chunks(total, slot_blocks, upload != 0, head_blocks);
    for (size_t i = 0; i < v.size() && i < room; ++i) out[i] = v[i];
    return uint32_t(v.size());
}
uint32_t tcp_chunk_pieces(const uint64_t *seg_first, const uint32_t *seg_n, uint32_t n_segs, uint64_t c0, uint64_t c1,
                          uint64_t *out4, uint32_t room)
{
    std::vector<tc::SegSpan> segs;
    for (uint32_t i = 0; i < n_segs; ++i) segs.push_back(tc::SegSpan{seg_first[i], seg_n[i]});
    std::vector<tc::Piece> p;
    tc::chunk_pieces(segs, c0, c1, &p);
    for (size_t i = 0; i < p.size() && i < room; ++i) {
        out4[4 * i] = p[i].seg; out4[4 * i + 1] = p[i].in_seg; out4[4 * i + 2] = p[i].in_chunk; out4[4 * i + 3] = p[i].n;
    }
    return uint32_t(p.size());
}
void tcp_host_tail(uint32_t div, uint64_t c0, uint32_t nblk, const uint64_t *seg_first, const uint32_t *seg_n, uint32_t n_segs,
                   int64_t *out3)
{
    std::vector<tc::SegSpan> segs;
    for (uint32_t i = 0; i < n_segs; ++i) segs.push_back(tc::SegSpan{seg_first[i], seg_n[i]});
    const tc::TailSplit t = tc::host_tail_split(div, c0, nblk, segs);
    out3[0] = t.staged; out3[1] = t.seg; out3[2] = int64_t(t.in_seg);
}
int tcp_offload_direct(uint32_t mode, uint64_t bytes, int upload_in_flight, uint64_t auto_bytes)
{
    return tc::offload_goes_direct(mode, bytes, upload_in_flight != 0, auto_bytes) ? 1 : 0;
}
int tcp_upload_direct(uint32_t mode) { return tc::upload_goes_direct(mode) ? 1 : 0; }
uint32_t tcp_tail_divisor(uint32_t option, uint64_t n_chunks, int overlapped) { return tc::tail_divisor(option, size_t(n_chunks), overlapped != 0); }
uint32_t tcp_plan_staged(uint64_t total, uint32_t slot_blocks, int upload, uint32_t head_blocks, uint32_t option, int *overlapped,
                         uint32_t *out, uint32_t room)
{
    bool ov = false;
    const std::vector<uint32_t> v = tc::plan_staged(total, slot_blocks, upload != 0, head_blocks, option, &ov);
    *overlapped = ov ? 1 : 0;
    for (size_t i = 0; i < v.size() && i < room; ++i) out[i] = v[i];
    return uint32_t(v.size());
}
int tcp_kernels_overlap(uint32_t option, uint64_t n_chunks) { return tc::kernels_overlap_copies(option, size_t(n_chunks)) ? 1 : 0; }

void *tcb_arena_new(uint64_t slots) { return new tc::HostArena(slots); }
void tcb_arena_del(void *a) { delete static_cast<tc::HostArena *>(a); }
int64_t tcb_arena_alloc(void *a, uint64_t n) { return static_cast<tc::HostArena *>(a)->alloc(n); }
int tcb_arena_free(void *a, uint64_t start) { return static_cast<tc::HostArena *>(a)->free(start); }
uint64_t tcb_arena_used(void *a) { return static_cast<tc::HostArena *>(a)->used(); }
int tcb_arena_locate(void *a, uint64_t slot, uint64_t *start, uint64_t *room)
{
    return static_cast<tc::HostArena *>(a)->locate(slot, start, room) ? 1 : 0;
}
void tcb_arena_begin(void *a, uint64_t start) { static_cast<tc::HostArena *>(a)->begin_transfer(start); }
void tcb_arena_end(void *a, uint64_t start) { static_cast<tc::HostArena *>(a)->end_transfer(start); }
}
