// The transfer engine of tokencake_kv, written against a small device interface `Dev` so that the whole of
// it (validation, id ring, chunking, hazards, path choice, enqueue order, what a failed enqueue keeps) runs
// in CPU tests against a recording device.  The library instantiates it with the HIP runtime (tc_engine.cpp).
//
// Offload (paper Sec. 4.1 / 6.3: a stalled agent's KV is copied to CPU memory asynchronously on a
// dedicated stream) runs in two stages per staging chunk:
//     gather_pages  ->  one contiguous D2H DMA per agent segment of the chunk
// Upload is the mirror image:
//     H2D DMA  ->  scatter_pages  (... last chunk)  ->  rewrite_table
// or, on the direct paths, one copy kernel per agent that writes / reads the pinned host buffer itself.
// The caller's stream is the paper's dedicated copy stream: it carries every DMA, the table rewrite and the
// completion event; kernels of other streams overlap freely.  By default the copy kernels run on that stream
// too, in line with the DMAs.  With tc_opts.overlap_kernels a transfer of several chunks puts its copy kernels
// on the engine's own stream, tied to the caller's by events in both directions:
//     offload   caller: ids, entry event ............ wait ready[c], DMA c, record last[c] ...... done
//               engine: wait entry; per chunk c: wait last[slot], gather c, record ready[c]
//     upload    caller: ids; per chunk c: wait last[slot], DMA c, record ready[c] .... wait last[final], tables, done
//               engine: per chunk c: wait ready[c], scatter c, record last[c]
// so the kernel of one chunk runs under the link copy of its neighbour, every DMA of a transfer stays on one
// stream, in order, and the completion event on the caller's stream covers everything.  `last` of a slot is its
// last consumer's event whoever that was; it orders the slot's reuse across transfers and streams.  The block
// bookkeeping (tc_blocks.h) is updated under the context's mutex; a transfer holds its blocks "in
// flight" until poll / sync see its completion event.
//
// Dev supplies (every int result: 0 = ok):
//   types   Stream, Event
//   events  event_create(Event*, bool timing), event_destroy, event_record(Event, Stream),
//           event_query(Event) (0 done, 1 not yet, < 0 error), event_sync(Event),
//           event_elapsed_ms(float*, Event, Event), stream_wait(Stream, Event), stream_sync(Stream)
//   copies  copy_ids(int32_t *dev, const int32_t *host, uint64_t n, Stream),
//           copy_d2h(void *host, const void *dev, uint64_t bytes, Stream), copy_h2d(void *dev, const void *host, ...)
//   kernels gather(...), scatter(...), rewrite(...) with the arguments of the launchers in tc_kernels.h
//   memory  device_view(void **out, void *host), is_pinned_host(const void *, uint64_t), is_device_ptr(const void *)
#pragma once

#include <cstring>
#include <vector>

#include "tc_blocks.h"
#include "tc_geom.h"
#include "tc_plan.h"
#include "tokencake_kv.h"

namespace tc {

// A handful of workgroups saturate the host link.  More host-bound stores (gather) only deepen the queue that
// other kernels' memory traffic has to wait behind; host-bound loads (scatter) are harmless up to about 24
// workgroups, and 16 keep a direct upload at the link rate next to a kernel that saturates HBM.  A chunk's host
// tail shares its launch with thousands of staged workgroups and stays small either way.
constexpr uint32_t kDefaultDirectGatherGrid = 6;
constexpr uint32_t kDefaultDirectScatterGrid = 16;
constexpr uint32_t kDefaultTailScatterGrid = 8;

enum TimedKind { kGather = 0, kScatter = 1, kD2H = 2, kH2D = 3, kDirect = 4 };

template <class Dev>
class Engine {
public:
    using Stream = typename Dev::Stream;
    using Event = typename Dev::Event;

    struct Slot {
        char *buf = nullptr;
        Event last{};   // last consumer finished: the slot may be overwritten
        Event ready{};  // the slot's producer finished (transfers whose kernels run on the engine's stream)
        bool used = false;
    };
    struct Timed {
        Event t0, t1;
        uint64_t bytes;
        int kind;
    };
    struct OpPayload {
        Event done{};
        Event entry{};           // ties the engine's stream to the caller's (overlapped transfers only)
        bool overlapped = false;
        std::vector<Timed> timed;
    };
    using Book = TransferBook<OpPayload>;
    using Entry = typename Book::Entry;

    Dev dev;
    tc_pool_desc pool{};
    tc_opts opts{};
    PageGeom geom{};
    uint64_t rec = 0;
    BlockPool *blocks = nullptr;
    HostArena *arena = nullptr;
    char *arena_base = nullptr;
    uint64_t arena_bytes = 0;
    uint32_t slot_blocks = 0;
    Stream kstream{};             // the engine's own stream for copy kernels; valid if has_kstream
    bool has_kstream = false;
    std::vector<Slot> slots;
    uint32_t next_slot = 0;
    int32_t *ids_host = nullptr;  // pinned ring
    int32_t *ids_dev = nullptr;   // device ring
    Book *book = nullptr;
    std::vector<Event> sync_events, time_events;  // recycled
    bool profiling = false;
    tc_stats_t st{};

    // ------------------------------------------------------------------------------ events
    int get_event(bool timing, Event *out)
    {
        auto &poolv = timing ? time_events : sync_events;
        if (!poolv.empty()) {
            *out = poolv.back();
            poolv.pop_back();
            return TC_OK;
        }
        return dev.event_create(out, timing) ? TC_ERR_HIP : TC_OK;
    }
    void put_event(bool timing, Event e) { (timing ? time_events : sync_events).push_back(e); }

    // --------------------------------------------------------------------------- retirement
    // The oldest transfer is known to be complete (or can no longer run): release what it held.
    void retire_front()
    {
        Entry &op = book->front();
        blocks->end_transfer(op.ids.data(), uint32_t(op.ids.size()));
        for (uint64_t s : op.arena_starts) arena->end_transfer(s);
        for (Timed &t : op.payload.timed) {
            float ms = 0.f;
            if (!op.failed && dev.event_elapsed_ms(&ms, t.t0, t.t1) == 0) {
                switch (t.kind) {
                case kGather: st.gather_launches++; st.gather_bytes += t.bytes; st.gather_ms += ms; break;
                case kScatter: st.scatter_launches++; st.scatter_bytes += t.bytes; st.scatter_ms += ms; break;
                case kDirect: st.direct_launches++; st.direct_bytes += t.bytes; st.direct_ms += ms; break;
                case kD2H: st.d2h_copies++; st.d2h_bytes += t.bytes; st.d2h_ms += ms; break;
                default: st.h2d_copies++; st.h2d_bytes += t.bytes; st.h2d_ms += ms; break;
                }
            }
            put_event(true, t.t0);
            put_event(true, t.t1);
        }
        put_event(false, op.payload.done);
        if (op.payload.overlapped) put_event(false, op.payload.entry);
        book->pop_front();
    }

    int poll()
    {
        while (!book->empty()) {
            const int q = dev.event_query(book->front().payload.done);
            if (q == 1) break;
            if (q != 0) return TC_ERR_HIP;
            retire_front();
        }
        return TC_OK;
    }

    int sync()
    {
        while (!book->empty()) {
            if (dev.event_sync(book->front().payload.done)) return TC_ERR_HIP;
            retire_front();
        }
        return TC_OK;
    }

    // --------------------------------------------------------------------------- validation
    struct Segment {  // one agent's run of records inside the concatenated list
        uint64_t first;  // index of its first record in the list
        uint32_t n;
        char *host;
        int32_t *table;
    };
    struct Plan {
        std::vector<Segment> segs;
        std::vector<SegSpan> spans;   // the same runs without the pointers
        std::vector<int32_t> ids;
        uint64_t total = 0;
    };

    bool in_arena(const char *p) const { return arena_base && p >= arena_base && p < arena_base + arena_bytes; }

    bool pinned(const void *p, uint64_t bytes)
    {
        const char *b = static_cast<const char *>(p);
        if (arena_base && b >= arena_base && b + bytes <= arena_base + arena_bytes) return true;
        return dev.is_pinned_host(p, bytes);
    }

    // Validation of a whole batch; no state is changed.
    int validate(const tc_xfer_desc *descs, uint32_t n_descs, Plan *plan)
    {
        if (n_descs && !descs) return TC_ERR_INVAL;
        uint64_t total = 0;
        for (uint32_t d = 0; d < n_descs; ++d) {
            if (descs[d].n == 0) continue;
            if (!descs[d].block_ids || !descs[d].host_buf) return TC_ERR_INVAL;
            total += descs[d].n;
        }
        if (total > blocks->total()) {
            // more ids than blocks: there is a bad or repeated id among them; find out which
            for (uint32_t d = 0; d < n_descs; ++d)
                if (int rc = blocks->check_range(descs[d].block_ids, descs[d].n)) return rc;
            return TC_ERR_DUP;
        }
        plan->ids.reserve(total);
        for (uint32_t d = 0; d < n_descs; ++d) {
            if (descs[d].n == 0) continue;
            plan->segs.push_back(Segment{plan->ids.size(), descs[d].n, static_cast<char *>(descs[d].host_buf),
                                         descs[d].block_table});
            plan->spans.push_back(SegSpan{plan->ids.size(), descs[d].n});
            plan->ids.insert(plan->ids.end(), descs[d].block_ids, descs[d].block_ids + descs[d].n);
        }
        plan->total = total;
        if (int rc = blocks->check_transfer(plan->ids.data(), uint32_t(total))) return rc;
        for (const Segment &s : plan->segs) {
            if (reinterpret_cast<uintptr_t>(s.host) % 16) return TC_ERR_INVAL;
            if (!pinned(s.host, uint64_t(s.n) * rec)) return TC_ERR_NOT_PINNED;
            if (in_arena(s.host)) {
                const uint64_t off = uint64_t(s.host - arena_base);
                uint64_t start, room;
                if (off % rec) return TC_ERR_INVAL;
                if (!arena->locate(off / rec, &start, &room) || room < s.n) return TC_ERR_INVAL;
            }
        }
        return TC_OK;
    }

    // ------------------------------------------------------------------ start / end of a transfer
    // Orders the transfer after conflicting ones on other streams, puts its ids into the rings and marks
    // blocks and arena runs in flight.  On an error nothing is held and nothing of this transfer is enqueued.
    int begin_op(Plan &plan, Stream stream, bool upload, Entry *op, uint64_t *ring_start)
    {
        op->stream = reinterpret_cast<const void *>(stream);
        op->upload = upload;
        for (const Segment &s : plan.segs) {
            if (!in_arena(s.host)) continue;
            uint64_t start, room;
            arena->locate(uint64_t(s.host - arena_base) / rec, &start, &room);
            op->arena_starts.push_back(start);
        }
        std::vector<size_t> waits;
        book->waits(op->stream, plan.ids, op->arena_starts, &waits);
        for (size_t at : waits)
            if (dev.stream_wait(stream, book->entries()[at].payload.done)) return TC_ERR_HIP;
        if (int rc = get_event(false, &op->payload.done)) return rc;
        if (plan.total > book->ring().cap()) {
            put_event(false, op->payload.done);
            return TC_ERR_INVAL;
        }
        while (!book->ring().alloc(plan.total, &op->span)) {
            // the ring is full of ids that transfers in flight still read: wait for the oldest
            if (book->empty() || dev.event_sync(book->front().payload.done)) {
                put_event(false, op->payload.done);
                return TC_ERR_HIP;
            }
            retire_front();
        }
        *ring_start = op->span.start;
        std::memcpy(ids_host + *ring_start, plan.ids.data(), plan.total * sizeof(int32_t));
        if (dev.copy_ids(ids_dev + *ring_start, ids_host + *ring_start, plan.total, stream)) {
            book->ring().cancel(op->span);   // the copy was refused: nothing reads the span
            put_event(false, op->payload.done);
            return TC_ERR_HIP;
        }
        blocks->begin_transfer(plan.ids.data(), uint32_t(plan.total));
        for (uint64_t s : op->arena_starts) arena->begin_transfer(s);
        op->ids = std::move(plan.ids);
        return TC_OK;
    }

    // Enqueueing failed after begin_op: work already on the stream (the id copy at least, perhaps kernels and
    // DMAs) may still read the id span, the blocks and the host buffers.  If a completion event can still be
    // recorded, the transfer is kept in flight, marked failed, and everything it holds is released when it
    // retires.  Otherwise the streams are drained here, after which nothing of it can run, and all is rolled back.
    // Kernels of an overlapped transfer may sit on the engine's stream with nothing on the caller's stream
    // waiting for them yet: the caller's stream is made to, before its completion event means anything.
    int fail_op(Entry &&op, Stream stream, int rc)
    {
        st.transfers_failed++;
        bool covered = true;
        if (op.payload.overlapped)
            covered = dev.event_record(op.payload.entry, kstream) == 0 && dev.stream_wait(stream, op.payload.entry) == 0;
        if (covered && dev.event_record(op.payload.done, stream) == 0) {
            op.failed = true;
            book->publish(std::move(op));
            return rc;
        }
        if (op.payload.overlapped) (void)dev.stream_sync(kstream);
        (void)dev.stream_sync(stream);
        blocks->end_transfer(op.ids.data(), uint32_t(op.ids.size()));
        for (uint64_t s : op.arena_starts) arena->end_transfer(s);
        book->ring().cancel(op.span);   // still the newest span: the mutex is held since begin_op
        for (Timed &t : op.payload.timed) {
            put_event(true, t.t0);
            put_event(true, t.t1);
        }
        put_event(false, op.payload.done);
        if (op.payload.overlapped) put_event(false, op.payload.entry);
        return rc;
    }

    int time_begin(Entry *op, Stream stream, uint64_t bytes, int kind)
    {
        if (!profiling) return TC_OK;
        Timed t{Event{}, Event{}, bytes, kind};
        if (int rc = get_event(true, &t.t0)) return rc;
        if (int rc = get_event(true, &t.t1)) {
            put_event(true, t.t0);
            return rc;
        }
        op->payload.timed.push_back(t);
        return dev.event_record(t.t0, stream) ? TC_ERR_HIP : TC_OK;
    }
    int time_end(Entry *op, Stream stream)
    {
        if (!profiling) return TC_OK;
        return dev.event_record(op->payload.timed.back().t1, stream) ? TC_ERR_HIP : TC_OK;
    }

#define TC_DEV(expr)                   \
    do {                               \
        if ((expr) != 0) return TC_ERR_HIP; \
    } while (0)
#define TC_RC(expr)                    \
    do {                               \
        if (int rc_ = (expr)) return rc_; \
    } while (0)

    // DMA of the parts of every segment that fall into records [c0, c1) of the list.
    int dma_chunk(const Plan &plan, uint64_t c0, uint64_t c1, char *slot_buf, bool to_host, Stream stream)
    {
        std::vector<Piece> pieces;
        chunk_pieces(plan.spans, c0, c1, &pieces);
        for (const Piece &p : pieces) {
            char *host = plan.segs[p.seg].host + p.in_seg * rec;
            char *devp = slot_buf + p.in_chunk * rec;
            if (to_host) TC_DEV(dev.copy_d2h(host, devp, p.n * rec, stream));
            else TC_DEV(dev.copy_h2d(devp, host, p.n * rec, stream));
        }
        return TC_OK;
    }

    // Where the chunk [c0, c0 + nblk) is split between staging and the host tail; *host_part is the GPU's
    // view of the tail's first record (nullptr = no tail).
    uint32_t host_tail(const Plan &plan, uint32_t div, uint64_t c0, uint32_t nblk, void **host_part)
    {
        *host_part = nullptr;
        const TailSplit t = host_tail_split(div, c0, nblk, plan.spans);
        if (t.seg < 0) return nblk;
        void *view = nullptr;
        if (dev.device_view(&view, plan.segs[size_t(t.seg)].host + t.in_seg * rec)) return nblk;
        *host_part = view;
        return t.staged;
    }

    // The GPU's view of every segment's host buffer, or false if one of them cannot be mapped.
    bool device_views(const Plan &plan, std::vector<void *> *out)
    {
        out->resize(plan.segs.size());
        for (size_t k = 0; k < plan.segs.size(); ++k)
            if (dev.device_view(&(*out)[k], plan.segs[k].host)) return false;
        return true;
    }

    // ---------------------------------------------------------------------------------- offload
    int offload(const tc_xfer_desc *descs, uint32_t n_descs, Stream stream)
    {
        Plan plan;
        TC_RC(validate(descs, n_descs, &plan));
        if (plan.total == 0) return TC_OK;
        (void)poll();

        // Direct path: the gather kernel writes each agent's records straight into its pinned host buffer.
        // Kernel-driven D2H traffic overlaps with H2D traffic, which two DMAs of opposite direction do not;
        // otherwise the staged path is the polite one (see offload_goes_direct).
        bool direct = offload_goes_direct(opts.direct_offload, plan.total * rec, book->upload_in_flight(), opts.auto_direct_bytes);
        std::vector<void *> dev_view;
        if (direct && !device_views(plan, &dev_view)) {
            if (opts.direct_offload == kPathDirect) return TC_ERR_NOT_PINNED;
            direct = false;   // left to the library: pinned but not mapped memory goes through staging
        }

        Entry op;
        uint64_t ring_start = 0;
        TC_RC(begin_op(plan, stream, false, &op, &ring_start));

        auto enqueue_direct = [&]() -> int {
            const uint32_t grid = opts.direct_grid ? opts.direct_grid : kDefaultDirectGatherGrid;
            for (size_t k = 0; k < plan.segs.size(); ++k) {
                const Segment &s = plan.segs[k];
                TC_RC(time_begin(&op, stream, uint64_t(s.n) * rec, kDirect));
                TC_DEV(dev.gather(pool.kv_base, static_cast<const uint32_t *>(pool.scales), dev_view[k],
                                  ids_dev + ring_start + s.first, s.n, geom, grid, true, stream, nullptr, s.n, 0));
                TC_RC(time_end(&op, stream));
            }
            TC_DEV(dev.event_record(op.payload.done, stream));
            return TC_OK;
        };
        auto enqueue = [&]() -> int {
            bool overlapped = false;
            const std::vector<uint32_t> chunks =
                plan_staged(plan.total, slot_blocks, false, head_blocks_of(rec), has_kstream ? opts.overlap_kernels : 0, &overlapped);
            const uint32_t div = tail_divisor(opts.host_tail_div, chunks.size(), overlapped);
            const Stream ks = overlapped ? kstream : stream;
            if (overlapped) {
                // the engine's stream starts after the ids are in place and after whatever begin_op waited for
                TC_RC(get_event(false, &op.payload.entry));
                op.payload.overlapped = true;
                TC_DEV(dev.event_record(op.payload.entry, stream));
                TC_DEV(dev.stream_wait(kstream, op.payload.entry));
            }
            uint64_t c0 = 0;
            for (uint32_t nblk : chunks) {
                Slot *slot = &slots[next_slot];
                next_slot = (next_slot + 1) % uint32_t(slots.size());
                if (slot->used) TC_DEV(dev.stream_wait(ks, slot->last));
                void *host_part = nullptr;
                const uint32_t split = host_tail(plan, div, c0, nblk, &host_part);
                TC_RC(time_begin(&op, ks, uint64_t(nblk) * rec, kGather));
                TC_DEV(dev.gather(pool.kv_base, static_cast<const uint32_t *>(pool.scales), slot->buf,
                                  ids_dev + ring_start + c0, nblk, geom, opts.max_grid, false, ks, host_part, split,
                                  opts.direct_grid ? opts.direct_grid : kDefaultDirectGatherGrid));
                TC_RC(time_end(&op, ks));
                if (overlapped) {
                    TC_DEV(dev.event_record(slot->ready, kstream));
                    TC_DEV(dev.stream_wait(stream, slot->ready));
                }
                TC_RC(time_begin(&op, stream, uint64_t(split) * rec, kD2H));
                TC_RC(dma_chunk(plan, c0, c0 + split, slot->buf, true, stream));
                TC_RC(time_end(&op, stream));
                TC_DEV(dev.event_record(slot->last, stream));
                slot->used = true;
                c0 += nblk;
            }
            TC_DEV(dev.event_record(op.payload.done, stream));
            if (overlapped) st.transfers_overlapped++;
            return TC_OK;
        };
        const uint64_t total = op.ids.size();
        if (int rc = direct ? enqueue_direct() : enqueue()) return fail_op(std::move(op), stream, rc);

        st.n_offloads++;
        st.blocks_offloaded += total;
        st.bytes_offloaded += total * rec;
        book->publish(std::move(op));
        return TC_OK;
    }

    // ----------------------------------------------------------------------------------- upload
    int upload(const tc_xfer_desc *descs, uint32_t n_descs, Stream stream)
    {
        Plan plan;
        TC_RC(validate(descs, n_descs, &plan));
        for (const Segment &s : plan.segs)
            if (s.table && !dev.is_device_ptr(s.table)) return TC_ERR_NOT_PINNED;
        if (plan.total == 0) return TC_OK;
        (void)poll();

        // Direct path: the scatter kernel reads each agent's records straight from its pinned host buffer.
        bool direct = upload_goes_direct(opts.direct_upload);
        std::vector<void *> dev_view;
        if (direct && !device_views(plan, &dev_view)) {
            if (opts.direct_upload == kPathDirect) return TC_ERR_NOT_PINNED;
            direct = false;
        }

        Entry op;
        uint64_t ring_start = 0;
        TC_RC(begin_op(plan, stream, true, &op, &ring_start));

        // the mapping is restored only after the data it points to is in place
        auto rewrite_tables = [&]() -> int {
            for (const Segment &s : plan.segs)
                if (s.table) TC_DEV(dev.rewrite(s.table, ids_dev + ring_start + s.first, s.n, stream));
            TC_DEV(dev.event_record(op.payload.done, stream));
            return TC_OK;
        };
        auto enqueue_direct = [&]() -> int {
            const uint32_t grid = opts.direct_grid ? opts.direct_grid : kDefaultDirectScatterGrid;
            for (size_t k = 0; k < plan.segs.size(); ++k) {
                const Segment &s = plan.segs[k];
                TC_RC(time_begin(&op, stream, uint64_t(s.n) * rec, kDirect));
                TC_DEV(dev.scatter(dev_view[k], pool.kv_base, static_cast<uint32_t *>(pool.scales),
                                   ids_dev + ring_start + s.first, s.n, geom, grid, true, stream, nullptr, s.n, 0));
                TC_RC(time_end(&op, stream));
            }
            return rewrite_tables();
        };
        auto enqueue = [&]() -> int {
            bool overlapped = false;
            const std::vector<uint32_t> chunks =
                plan_staged(plan.total, slot_blocks, true, head_blocks_of(rec), has_kstream ? opts.overlap_kernels : 0, &overlapped);
            const uint32_t div = tail_divisor(opts.host_tail_div, chunks.size(), overlapped);
            const Stream ks = overlapped ? kstream : stream;
            if (overlapped) {
                TC_RC(get_event(false, &op.payload.entry));   // only a failed enqueue records it (fail_op)
                op.payload.overlapped = true;
            }
            Slot *final_slot = nullptr;
            uint64_t c0 = 0;
            for (uint32_t nblk : chunks) {
                Slot *slot = &slots[next_slot];
                next_slot = (next_slot + 1) % uint32_t(slots.size());
                if (slot->used) TC_DEV(dev.stream_wait(stream, slot->last));
                void *host_part = nullptr;
                const uint32_t split = host_tail(plan, div, c0, nblk, &host_part);
                TC_RC(time_begin(&op, stream, uint64_t(split) * rec, kH2D));
                TC_RC(dma_chunk(plan, c0, c0 + split, slot->buf, false, stream));
                TC_RC(time_end(&op, stream));
                if (overlapped) {
                    // the scatter also needs the ids and whatever begin_op waited for: both precede this event
                    TC_DEV(dev.event_record(slot->ready, stream));
                    TC_DEV(dev.stream_wait(kstream, slot->ready));
                }
                TC_RC(time_begin(&op, ks, uint64_t(nblk) * rec, kScatter));
                TC_DEV(dev.scatter(slot->buf, pool.kv_base, static_cast<uint32_t *>(pool.scales),
                                   ids_dev + ring_start + c0, nblk, geom, opts.max_grid, false, ks, host_part, split,
                                   opts.direct_grid ? opts.direct_grid : kDefaultTailScatterGrid));
                TC_RC(time_end(&op, ks));
                TC_DEV(dev.event_record(slot->last, ks));
                slot->used = true;
                final_slot = slot;
                c0 += nblk;
            }
            // the engine's stream runs in order: its last scatter is done when all are
            if (overlapped && final_slot) TC_DEV(dev.stream_wait(stream, final_slot->last));
            if (overlapped) st.transfers_overlapped++;
            return rewrite_tables();
        };
        const uint64_t total = op.ids.size();
        if (int rc = direct ? enqueue_direct() : enqueue()) return fail_op(std::move(op), stream, rc);

        st.n_uploads++;
        st.blocks_uploaded += total;
        st.bytes_uploaded += total * rec;
        book->publish(std::move(op));
        return TC_OK;
    }
    // Measurement helper: the staged path's copy kernel alone on records in device memory (no DMA, no
    // bookkeeping of blocks); the ids take the usual way through the id ring.
    int stage_on_device(int direction, const int32_t *ids, uint32_t n, void *dev_records, Stream stream)
    {
        if (direction < 0 || direction > 1 || (n && (!ids || !dev_records))) return TC_ERR_INVAL;
        if (n == 0) return TC_OK;
        TC_RC(blocks->check_range(ids, n));
        TC_RC(blocks->check_distinct(ids, n));
        if (!dev.is_device_ptr(dev_records) || n > book->ring().cap()) return TC_ERR_INVAL;
        (void)poll();
        Entry op;
        op.stream = reinterpret_cast<const void *>(stream);
        TC_RC(get_event(false, &op.payload.done));
        while (!book->ring().alloc(n, &op.span)) {
            if (book->empty() || dev.event_sync(book->front().payload.done)) {
                put_event(false, op.payload.done);
                return TC_ERR_HIP;
            }
            retire_front();
        }
        std::memcpy(ids_host + op.span.start, ids, uint64_t(n) * sizeof(int32_t));
        if (dev.copy_ids(ids_dev + op.span.start, ids_host + op.span.start, n, stream)) {
            book->ring().cancel(op.span);
            put_event(false, op.payload.done);
            return TC_ERR_HIP;
        }
        auto enqueue = [&]() -> int {
            TC_RC(time_begin(&op, stream, uint64_t(n) * rec, direction == 0 ? kGather : kScatter));
            if (direction == 0)
                TC_DEV(dev.gather(pool.kv_base, static_cast<const uint32_t *>(pool.scales), dev_records,
                                  ids_dev + op.span.start, n, geom, opts.max_grid, false, stream, nullptr, n, 0));
            else
                TC_DEV(dev.scatter(dev_records, pool.kv_base, static_cast<uint32_t *>(pool.scales),
                                   ids_dev + op.span.start, n, geom, opts.max_grid, false, stream, nullptr, n, 0));
            TC_RC(time_end(&op, stream));
            TC_DEV(dev.event_record(op.payload.done, stream));
            return TC_OK;
        };
        if (int rc = enqueue()) return fail_op(std::move(op), stream, rc);
        book->publish(std::move(op));
        return TC_OK;
    }
#undef TC_DEV
#undef TC_RC

    void fill_stats(tc_stats_t *out) const
    {
        tc_stats_t s = st;
        s.gpu_blocks_total = blocks->total();
        s.gpu_blocks_free = blocks->n_free();
        s.gpu_blocks_used = blocks->n_used();
        s.gpu_blocks_pending_free = blocks->n_pending();
        s.gpu_blocks_shared = blocks->n_shared();
        s.ops_in_flight = uint32_t(book->size());
        s.host_slots_total = arena->total();
        s.host_slots_used = arena->used();
        *out = s;
    }
};

}  // namespace tc
