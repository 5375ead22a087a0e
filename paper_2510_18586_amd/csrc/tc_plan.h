// Host-side planning around a transfer; no GPU types, so that all of it runs in CPU tests.
//
// Paper Sec. 6.3: migrations are issued asynchronously on a dedicated stream, and nothing a copy may
// still read is reused before that copy has completed.  Here that rule covers, besides the KV blocks
// (tc_blocks.h), the ring of device-side block ids a transfer's kernels read, the host allocation its
// copies touch, and the order between transfers that callers put on different streams.
#pragma once

#include <algorithm>
#include <cstdint>
#include <deque>
#include <unordered_map>
#include <vector>

namespace tc {

// ---------------------------------------------------------------------------------------- id ring
// `cap` entries handed out in address order as spans of consecutive entries.  A request that does not
// fit before the end of the ring starts again at entry 0; the entries it skipped stay unusable until the
// request itself is released.  An empty ring starts at 0.  Spans are released oldest first; the newest
// may be cancelled (nothing was enqueued that could read it).
class IdRing {
public:
    struct Span {
        uint64_t start = 0;      // first entry
        uint64_t consumed = 0;   // entries held: skipped + n
        uint64_t prev_tail = 0;  // where the ring stood before, to cancel the newest span
    };

    explicit IdRing(uint64_t cap) : cap_(cap) {}
    uint64_t cap() const { return cap_; }
    uint64_t used() const { return used_; }

    // false: n entries do not fit right now (the caller retires the oldest transfer and tries again).
    // n must not exceed cap().
    bool alloc(uint64_t n, Span *out)
    {
        if (used_ == 0) tail_ = 0;
        uint64_t skipped = 0, at = tail_;
        if (at + n > cap_) {
            skipped = cap_ - at;
            at = 0;
        }
        if (used_ + skipped + n > cap_) return false;
        out->start = at;
        out->consumed = skipped + n;
        out->prev_tail = tail_;
        used_ += skipped + n;
        tail_ = (at + n) % cap_;
        return true;
    }
    void release(const Span &s) { used_ -= s.consumed; }
    void cancel(const Span &s)
    {
        used_ -= s.consumed;
        tail_ = s.prev_tail;
    }

private:
    uint64_t cap_, tail_ = 0, used_ = 0;
};

// ------------------------------------------------------------------------------ chunks and pieces
// Chunk sizes (in blocks) for `total` records: full slots, then the remainder.  With head_blocks > 0 a list of
// more than twice that many records starts with a short chunk of head_blocks records (at most a slot): while it
// crosses the link the copy kernel is already at work on the next chunk, so only a short kernel runs with the
// link idle.  An upload takes the same sizes in reverse order: its last kernel, which nothing hides, is the
// short one.
inline std::vector<uint32_t> plan_chunks(uint64_t total, uint32_t slot_blocks, bool upload, uint32_t head_blocks = 0)
{
    std::vector<uint32_t> out;
    const uint32_t head = std::min(head_blocks, slot_blocks);
    if (head > 0 && total > 2ull * head) {
        out.push_back(head);
        total -= head;
    }
    while (total) {
        const uint32_t take = uint32_t(std::min<uint64_t>(slot_blocks, total));
        out.push_back(take);
        total -= take;
    }
    if (upload) std::reverse(out.begin(), out.end());
    return out;
}

// One host buffer's run of records inside the concatenated list of a (batched) transfer.
struct SegSpan {
    uint64_t first;  // index of its first record in the list
    uint32_t n;
};

// One contiguous copy between a staging chunk and a host buffer.
struct Piece {
    uint32_t seg;        // which buffer
    uint64_t in_seg;     // first record inside that buffer
    uint64_t in_chunk;   // first record inside the chunk
    uint64_t n;          // records
};

// The copies that carry records [c0, c1) of the list: one per buffer the chunk touches.
inline void chunk_pieces(const std::vector<SegSpan> &segs, uint64_t c0, uint64_t c1, std::vector<Piece> *out)
{
    out->clear();
    for (size_t k = 0; k < segs.size(); ++k) {
        const uint64_t a = std::max<uint64_t>(segs[k].first, c0), b = std::min<uint64_t>(segs[k].first + segs[k].n, c1);
        if (a < b) out->push_back(Piece{uint32_t(k), a - segs[k].first, a - c0, b - a});
    }
}

// The host link is idle while a chunk's copy kernel runs.  With a tail divisor N >= 2 the last nblk / N
// records of the chunk [c0, c0 + nblk) skip staging and cross the link inside the copy launch, provided
// the chunk has at least N records and the tail lies in one host buffer.
struct TailSplit {
    uint32_t staged;   // leading records of the chunk that still go through staging (nblk = no tail)
    int32_t seg;       // buffer that holds the tail, -1 = no tail
    uint64_t in_seg;   // first tail record inside that buffer
};
inline TailSplit host_tail_split(uint32_t div, uint64_t c0, uint32_t nblk, const std::vector<SegSpan> &segs)
{
    if (div < 2 || nblk < div) return TailSplit{nblk, -1, 0};
    const uint32_t m = nblk / div;
    const uint64_t first = c0 + nblk - m;
    for (size_t k = 0; k < segs.size(); ++k)
        if (first >= segs[k].first && c0 + nblk <= segs[k].first + segs[k].n)
            return TailSplit{nblk - m, int32_t(k), first - segs[k].first};
    return TailSplit{nblk, -1, 0};
}

// ------------------------------------------------------------------------------------------ paths
// Values of tc_opts.direct_offload / direct_upload.
enum : uint32_t { kPathAuto = 0, kPathDirect = 1, kPathDirectIfDuplex = 2, kPathStaged = 3 };
constexpr uint32_t kAutoTailDivisor = 64;

// Direct = the copy kernel writes / reads the pinned host buffer itself.  Measured on MI355X, 512 MiB next to a
// kernel that saturates HBM on another stream (transfer time / that kernel's rate, against each alone):
//   staged                      offload +14 %, upload +22 %     neighbour -2 %
//   direct, 6 / 8 workgroups    offload +80 %, upload +63 %     neighbour -4 % / -1 %
//   direct, 16 workgroups       offload +31 %, upload  +4 %     neighbour -42 % / -4 %
//   direct, 32 workgroups       offload  +5 %, upload  +2 %     neighbour -66 % / -22 %
// Host-bound stores (direct offload) clog the memory pipeline for everybody once there are enough of them to
// keep the link busy under load; host-bound loads (direct upload) do not.  So, left to the library:
// an upload goes direct (16 workgroups: as fast as the link when the GPU is idle, the least disturbed when it
// is busy, one pass through HBM instead of three); an offload goes through device staging and the copy engine,
// except while an upload of the same context is in flight: kernel-driven D2H traffic overlaps with H2D traffic
// on the link, two DMAs of opposite direction take turns.  auto_direct_bytes > 0 adds a size rule for callers
// whose GPU is otherwise idle: an offload below that many bytes goes direct too (one kernel beats kernel + DMA
// by ~19 us).
inline bool offload_goes_direct(uint32_t mode, uint64_t total_bytes, bool upload_in_flight, uint64_t auto_direct_bytes)
{
    if (mode == kPathDirect) return true;
    if (mode == kPathStaged) return false;
    if (mode == kPathDirectIfDuplex) return upload_in_flight;
    return upload_in_flight || total_bytes < auto_direct_bytes;
}
inline bool upload_goes_direct(uint32_t mode) { return mode != kPathStaged; }
// tc_opts.overlap_kernels: 1 = a staged transfer of more than one chunk runs its copy kernels on the engine's own
// stream, so that the kernel of one chunk overlaps with the link copy of its neighbour (a single chunk has nothing
// to overlap with, and the hop between streams would only delay it); 0 (the default) = everything in line on the
// caller's stream.  Measured on MI355X with an otherwise idle GPU: 512 MiB go out at 98.6 % instead of 98.1 % of
// the link, a batch of 20 GiB at 99.4 % instead of 97.5 %.  It is not the default because the engine's stream is
// one more stream for the runtime to place on its few hardware queues: where it lands behind a caller's stream
// that runs long kernels, every copy kernel waits for the kernel in front (a 20 GiB batch next to back-to-back
// 2.4 ms kernels went out at half rate), and the caller cannot steer that.
inline bool kernels_overlap_copies(uint32_t option, size_t n_chunks) { return option == 1 && n_chunks > 1; }
// The short first chunk of such a transfer: 32 MiB of records.  Measured on 512 MiB: 16 + 240 blocks of 2 MiB
// reach 99.5 % of the link, 8 + 248 99.4 %, 2 + 6 + 24 + 96 + 128 99.1 %, four equal chunks 98.9 %, one chunk 98.3 %.
constexpr uint64_t kHeadBytes = 32ull << 20;
inline uint32_t head_blocks_of(uint64_t record_bytes)
{
    const uint64_t n = kHeadBytes / record_bytes;
    return uint32_t(n < 1 ? 1 : (n > 0xffffffffull ? 0xffffffffull : n));
}
// Chunk sizes of a staged transfer and whether its kernels overlap with its copies: the cut with a short first
// chunk if that yields something to overlap, else the plain cut with everything in line.
inline std::vector<uint32_t> plan_staged(uint64_t total, uint32_t slot_blocks, bool upload, uint32_t head_blocks,
                                         uint32_t overlap_option, bool *overlapped)
{
    std::vector<uint32_t> sizes = plan_chunks(total, slot_blocks, upload, head_blocks);
    *overlapped = kernels_overlap_copies(overlap_option, sizes.size());
    return *overlapped ? sizes : plan_chunks(total, slot_blocks, upload, 0);
}
// tc_opts.host_tail_div: 0 = automatic (a tail where the link would otherwise idle once per chunk: transfers of
// more than one chunk whose kernels run in line with their copies), 1 = never, N >= 2 = 1/N of every chunk.
inline uint32_t tail_divisor(uint32_t option, size_t n_chunks, bool overlapped = false)
{
    if (option == 0) return (n_chunks > 1 && !overlapped) ? kAutoTailDivisor : 0;
    return option == 1 ? 0 : option;
}

// --------------------------------------------------------------------------- transfers in flight
// What the engine remembers of every transfer until it is retired, oldest first, and the hazards between
// transfers on different streams: a new transfer waits for the LAST earlier one, still in flight, that
// touched one of its blocks or its host allocation, unless that one is on the same stream (implicit
// order).  A transfer whose enqueue failed after part of it reached the stream is published like any
// other (failed = true): its kernels may still run, so everything it holds stays held until it retires.
template <class Payload>
class TransferBook {
public:
    struct Entry {
        uint64_t ticket = 0;             // consecutive in issue order
        const void *stream = nullptr;    // where it was enqueued
        bool upload = false, failed = false;
        std::vector<int32_t> ids;
        std::vector<uint64_t> arena_starts;
        IdRing::Span span;
        Payload payload{};
    };

    TransferBook(uint64_t ring_cap, uint32_t num_blocks) : ring_(ring_cap), block_ticket_(num_blocks, 0) {}

    IdRing &ring() { return ring_; }
    bool empty() const { return ops_.empty(); }
    size_t size() const { return ops_.size(); }
    Entry &front() { return ops_.front(); }
    const std::deque<Entry> &entries() const { return ops_; }
    bool upload_in_flight() const
    {
        for (const Entry &e : ops_)
            if (e.upload) return true;
        return false;
    }

    // Entries (by position in entries()) the new transfer has to wait for.
    void waits(const void *stream, const std::vector<int32_t> &ids, const std::vector<uint64_t> &arena_starts,
               std::vector<size_t> *out) const
    {
        out->clear();
        if (ops_.empty()) return;
        const uint64_t front = ops_.front().ticket;
        auto consider = [&](uint64_t t) {
            if (t < front) return;  // retired (or never set)
            const size_t at = size_t(t - front);
            if (ops_[at].stream == stream) return;
            if (std::find(out->begin(), out->end(), at) == out->end()) out->push_back(at);
        };
        for (int32_t id : ids) consider(block_ticket_[size_t(id)]);
        for (uint64_t s : arena_starts) {
            auto it = arena_ticket_.find(s);
            if (it != arena_ticket_.end()) consider(it->second);
        }
    }

    // The transfer is enqueued (or failed half-way): remember it as the last one on its blocks and
    // host allocations.  Returns its ticket.
    uint64_t publish(Entry &&e)
    {
        e.ticket = next_ticket_++;
        for (int32_t id : e.ids) block_ticket_[size_t(id)] = e.ticket;
        for (uint64_t s : e.arena_starts) arena_ticket_[s] = e.ticket;
        ops_.push_back(std::move(e));
        return ops_.back().ticket;
    }

    // The oldest transfer is complete: its ring span goes back; the caller releases blocks and arena runs.
    void pop_front()
    {
        Entry &e = ops_.front();
        for (uint64_t s : e.arena_starts) {
            auto it = arena_ticket_.find(s);
            if (it != arena_ticket_.end() && it->second == e.ticket) arena_ticket_.erase(it);
        }
        ring_.release(e.span);
        ops_.pop_front();
    }

private:
    IdRing ring_;
    std::deque<Entry> ops_;
    uint64_t next_ticket_ = 1;
    std::vector<uint64_t> block_ticket_;
    std::unordered_map<uint64_t, uint64_t> arena_ticket_;
};

}  // namespace tc
