// Transfer engine and C ABI of tokencake_kv (see include/tokencake_kv.h for the contract).
//
// Offload (paper Sec. 4.1 / 6.3: a stalled agent's KV is copied to CPU memory asynchronously on a
// dedicated stream) runs in two stages per staging chunk, all on the caller's stream:
//     gather_pages  ->  one contiguous D2H DMA per agent segment of the chunk
// Upload is the mirror image:
//     H2D DMA  ->  scatter_pages  (... last chunk)  ->  rewrite_table
// The stream is the paper's dedicated copy stream; kernels of other streams overlap freely.  The
// gather is ~50x faster than the host link, so running it in line with the DMAs costs under 2 %;
// a second, private DMA stream (gather of chunk c+1 under the DMA of chunk c) was measured and
// dropped: with two copies queued across streams the runtime at random ran the DMAs at half rate.
// A slot's `last` event orders its reuse when callers bring different streams.  The block
// bookkeeping (tc_blocks.h) is updated under one mutex; a transfer holds its blocks "in flight"
// until tc_poll / tc_sync see its completion event.
#include <cstdio>
#include <cstring>
#include <deque>
#include <mutex>
#include <new>
#include <unordered_map>
#include <vector>

#include <hip/hip_runtime_api.h>

#include "tc_blocks.h"
#include "tc_geom.h"
#include "tc_kernels.h"
#include "tokencake_kv.h"

namespace {

constexpr uint64_t kDefaultSlotBytes = 512ull << 20;
constexpr uint32_t kDefaultSlots = 2;
// A handful of workgroups saturate the host link; more only deepen the queue of host-bound requests
// that other kernels' memory traffic has to wait behind.
constexpr uint32_t kDefaultDirectGatherGrid = 6;
constexpr uint32_t kDefaultDirectScatterGrid = 8;

struct Slot {
    char *buf = nullptr;
    hipEvent_t last = nullptr;  // last consumer finished: the slot may be overwritten
    bool used = false;
};

enum TimedKind { kGather = 0, kScatter = 1, kD2H = 2, kH2D = 3, kDirect = 4 };

struct Timed {
    hipEvent_t t0, t1;
    uint64_t bytes;
    int kind;
};

struct Op {
    hipEvent_t done = nullptr;
    uint64_t ticket = 0;           // consecutive in issue order
    hipStream_t stream = nullptr;  // where it was enqueued
    bool is_upload = false;
    std::vector<int32_t> ids;
    std::vector<uint64_t> arena_starts;
    uint64_t ring_consumed = 0;
    uint64_t ring_prev_tail = 0;  // to undo the newest allocation
    std::vector<Timed> timed;
};

struct Segment {  // one agent's run of records inside the concatenated list
    uint64_t first;  // index of its first record in the list
    uint32_t n;
    char *host;
    int32_t *table;
};

}  // namespace

struct tc_ctx {
    std::mutex mu;
    tc_pool_desc pool{};
    tc_opts opts{};
    tc::PageGeom geom{};
    uint64_t rec = 0;
    tc::BlockPool *blocks = nullptr;
    tc::HostArena *arena = nullptr;
    char *arena_base = nullptr;
    uint64_t arena_bytes = 0;

    char *staging = nullptr;
    uint64_t slot_bytes = 0;
    uint32_t slot_blocks = 0;
    std::vector<Slot> slots;
    uint32_t next_slot = 0;

    int32_t *ids_host = nullptr;  // pinned ring
    int32_t *ids_dev = nullptr;   // device ring
    uint64_t ring_cap = 0, ring_tail = 0, ring_used = 0;

    std::deque<Op> ops;
    uint64_t next_ticket = 1;
    // Hazards between transfers that callers put on different streams: the last transfer that
    // touched a block / an arena allocation; a later one on another stream waits for its event.
    std::vector<uint64_t> block_ticket;
    std::unordered_map<uint64_t, uint64_t> arena_ticket;
    std::vector<hipEvent_t> sync_events, time_events;  // recycled
    bool profiling = false;
    tc_stats_t st{};
};

namespace {

#define HIP_TRY(expr)                                                                              \
    do {                                                                                           \
        hipError_t e_ = (expr);                                                                    \
        if (e_ != hipSuccess) {                                                                    \
            std::fprintf(stderr, "tokencake_kv: %s failed: %s (%s:%d)\n", #expr, hipGetErrorString(e_), \
                         __FILE__, __LINE__);                                                      \
            return TC_ERR_HIP;                                                                     \
        }                                                                                          \
    } while (0)

int get_event(tc_ctx *c, bool timing, hipEvent_t *out)
{
    auto &poolv = timing ? c->time_events : c->sync_events;
    if (!poolv.empty()) {
        *out = poolv.back();
        poolv.pop_back();
        return TC_OK;
    }
    HIP_TRY(hipEventCreateWithFlags(out, timing ? hipEventDefault : hipEventDisableTiming));
    return TC_OK;
}

void put_event(tc_ctx *c, bool timing, hipEvent_t e)
{
    if (e) (timing ? c->time_events : c->sync_events).push_back(e);
}

bool is_pinned_host(tc_ctx *c, const void *p, uint64_t bytes)
{
    const char *b = static_cast<const char *>(p);
    if (c->arena_base && b >= c->arena_base && b + bytes <= c->arena_base + c->arena_bytes) return true;
    for (const char *q : {b, b + (bytes ? bytes - 1 : 0)}) {
        hipPointerAttribute_t a;
        if (hipPointerGetAttributes(&a, q) != hipSuccess) {
            (void)hipGetLastError();
            return false;
        }
        if (a.type != hipMemoryTypeHost) return false;
    }
    return true;
}

bool is_device_ptr(const void *p)
{
    hipPointerAttribute_t a;
    if (hipPointerGetAttributes(&a, p) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return a.type == hipMemoryTypeDevice;
}

// The oldest transfer is known to be complete: release what it held.
int retire_front(tc_ctx *c)
{
    Op &op = c->ops.front();
    c->blocks->end_transfer(op.ids.data(), uint32_t(op.ids.size()));
    for (uint64_t s : op.arena_starts) {
        c->arena->end_transfer(s);
        auto it = c->arena_ticket.find(s);
        if (it != c->arena_ticket.end() && it->second == op.ticket) c->arena_ticket.erase(it);
    }
    c->ring_used -= op.ring_consumed;
    for (Timed &t : op.timed) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, t.t0, t.t1) == hipSuccess) {
            switch (t.kind) {
            case kGather: c->st.gather_launches++; c->st.gather_bytes += t.bytes; c->st.gather_ms += ms; break;
            case kScatter: c->st.scatter_launches++; c->st.scatter_bytes += t.bytes; c->st.scatter_ms += ms; break;
            case kDirect: c->st.direct_launches++; c->st.direct_bytes += t.bytes; c->st.direct_ms += ms; break;
            case kD2H: c->st.d2h_copies++; c->st.d2h_bytes += t.bytes; c->st.d2h_ms += ms; break;
            default: c->st.h2d_copies++; c->st.h2d_bytes += t.bytes; c->st.h2d_ms += ms; break;
            }
        } else {
            (void)hipGetLastError();
        }
        put_event(c, true, t.t0);
        put_event(c, true, t.t1);
    }
    put_event(c, false, op.done);
    c->ops.pop_front();
    return TC_OK;
}

int poll_locked(tc_ctx *c)
{
    while (!c->ops.empty()) {
        hipError_t e = hipEventQuery(c->ops.front().done);
        if (e == hipErrorNotReady) {
            (void)hipGetLastError();
            break;
        }
        if (e != hipSuccess) return TC_ERR_HIP;
        retire_front(c);
    }
    return TC_OK;
}

int sync_locked(tc_ctx *c)
{
    while (!c->ops.empty()) {
        HIP_TRY(hipEventSynchronize(c->ops.front().done));
        retire_front(c);
    }
    return TC_OK;
}

// n consecutive entries of the id rings; waits for old transfers when the ring is full.
int ring_alloc(tc_ctx *c, uint64_t n, uint64_t *start, uint64_t *consumed, uint64_t *prev_tail)
{
    if (n > c->ring_cap) return TC_ERR_INVAL;
    for (;;) {
        if (c->ring_used == 0) c->ring_tail = 0;
        uint64_t waste = 0, at = c->ring_tail;
        if (at + n > c->ring_cap) {
            waste = c->ring_cap - at;
            at = 0;
        }
        if (c->ring_used + waste + n <= c->ring_cap) {
            *prev_tail = c->ring_tail;
            c->ring_used += waste + n;
            c->ring_tail = (at + n) % c->ring_cap;
            *start = at;
            *consumed = waste + n;
            return TC_OK;
        }
        if (c->ops.empty()) return TC_ERR_INVAL;  // cannot happen: an empty ring fits n <= cap
        HIP_TRY(hipEventSynchronize(c->ops.front().done));
        retire_front(c);
    }
}

// Chunk sizes (in blocks) for `total` records: full slots, then the remainder.  An upload takes
// the remainder first, so both directions end with the same chunk boundaries.
std::vector<uint32_t> plan_chunks(uint64_t total, uint32_t slot_blocks, bool reversed)
{
    std::vector<uint32_t> out;
    while (total) {
        uint32_t take = uint32_t(std::min<uint64_t>(slot_blocks, total));
        out.push_back(take);
        total -= take;
    }
    if (reversed) std::reverse(out.begin(), out.end());
    return out;
}

struct Plan {
    std::vector<Segment> segs;
    std::vector<int32_t> ids;
    uint64_t total = 0;
};

// Validation of a whole batch; no state is changed.
int validate(tc_ctx *c, const tc_xfer_desc *descs, uint32_t n_descs, Plan *plan)
{
    if (n_descs && !descs) return TC_ERR_INVAL;
    uint64_t total = 0;
    for (uint32_t d = 0; d < n_descs; ++d) {
        if (descs[d].n == 0) continue;
        if (!descs[d].block_ids || !descs[d].host_buf) return TC_ERR_INVAL;
        total += descs[d].n;
    }
    if (total > c->blocks->total()) {
        // more ids than blocks: there is a bad or repeated id among them; find out which
        for (uint32_t d = 0; d < n_descs; ++d)
            if (int rc = c->blocks->check_range(descs[d].block_ids, descs[d].n)) return rc;
        return TC_ERR_DUP;
    }
    plan->ids.reserve(total);
    for (uint32_t d = 0; d < n_descs; ++d) {
        if (descs[d].n == 0) continue;
        plan->segs.push_back(Segment{plan->ids.size(), descs[d].n, static_cast<char *>(descs[d].host_buf),
                                     descs[d].block_table});
        plan->ids.insert(plan->ids.end(), descs[d].block_ids, descs[d].block_ids + descs[d].n);
    }
    plan->total = total;
    if (int rc = c->blocks->check_transfer(plan->ids.data(), uint32_t(total))) return rc;
    for (const Segment &s : plan->segs) {
        if (reinterpret_cast<uintptr_t>(s.host) % 16) return TC_ERR_INVAL;
        if (!is_pinned_host(c, s.host, uint64_t(s.n) * c->rec)) return TC_ERR_NOT_PINNED;
        if (c->arena_base && s.host >= c->arena_base && s.host < c->arena_base + c->arena_bytes) {
            uint64_t off = uint64_t(s.host - c->arena_base);
            uint64_t start, room;
            if (off % c->rec) return TC_ERR_INVAL;
            if (!c->arena->locate(off / c->rec, &start, &room) || room < s.n) return TC_ERR_INVAL;
        }
    }
    return TC_OK;
}

// Common start of a transfer: ids into the rings, blocks and arena runs marked in flight.
// Orders this transfer after unretired transfers on OTHER streams that touched the same blocks or
// the same arena allocations (same-stream order is implicit).
int wait_for_hazards(tc_ctx *c, const Plan &plan, hipStream_t stream)
{
    if (c->ops.empty()) return TC_OK;
    const uint64_t front = c->ops.front().ticket;
    std::vector<uint64_t> waits;
    auto consider = [&](uint64_t t) {
        if (t < front) return;  // retired (or never set)
        const Op &o = c->ops[size_t(t - front)];
        if (o.stream == stream) return;
        for (uint64_t w : waits)
            if (w == t) return;
        waits.push_back(t);
    };
    for (int32_t id : plan.ids) consider(c->block_ticket[size_t(id)]);
    for (const Segment &s : plan.segs) {
        if (c->arena_base && s.host >= c->arena_base && s.host < c->arena_base + c->arena_bytes) {
            uint64_t start, room;
            if (c->arena->locate(uint64_t(s.host - c->arena_base) / c->rec, &start, &room)) {
                auto it = c->arena_ticket.find(start);
                if (it != c->arena_ticket.end()) consider(it->second);
            }
        }
    }
    for (uint64_t t : waits) HIP_TRY(hipStreamWaitEvent(stream, c->ops[size_t(t - front)].done, 0));
    return TC_OK;
}

// The transfer is enqueued: remember it as the last one on its blocks and arena allocations.
void publish_op(tc_ctx *c, Op &&op, hipStream_t stream)
{
    op.ticket = c->next_ticket++;
    op.stream = stream;
    for (int32_t id : op.ids) c->block_ticket[size_t(id)] = op.ticket;
    for (uint64_t s : op.arena_starts) c->arena_ticket[s] = op.ticket;
    c->ops.push_back(std::move(op));
}

int begin_op(tc_ctx *c, Plan &plan, hipStream_t stream, Op *op, uint64_t *ring_start)
{
    if (int rc = wait_for_hazards(c, plan, stream)) return rc;
    if (int rc = get_event(c, false, &op->done)) return rc;
    if (int rc = ring_alloc(c, plan.total, ring_start, &op->ring_consumed, &op->ring_prev_tail)) {
        put_event(c, false, op->done);
        return rc;
    }
    std::memcpy(c->ids_host + *ring_start, plan.ids.data(), plan.total * sizeof(int32_t));
    if (hipMemcpyAsync(c->ids_dev + *ring_start, c->ids_host + *ring_start, plan.total * sizeof(int32_t),
                       hipMemcpyHostToDevice, stream) != hipSuccess) {
        (void)hipGetLastError();
        c->ring_used -= op->ring_consumed;
        c->ring_tail = op->ring_prev_tail;
        put_event(c, false, op->done);
        return TC_ERR_HIP;
    }
    c->blocks->begin_transfer(plan.ids.data(), uint32_t(plan.total));
    for (const Segment &s : plan.segs) {
        if (c->arena_base && s.host >= c->arena_base && s.host < c->arena_base + c->arena_bytes) {
            uint64_t start, room;
            c->arena->locate(uint64_t(s.host - c->arena_base) / c->rec, &start, &room);
            c->arena->begin_transfer(start);
            op->arena_starts.push_back(start);
        }
    }
    op->ids = std::move(plan.ids);
    return TC_OK;
}

int abort_op(tc_ctx *c, Op *op, int rc)
{
    c->blocks->end_transfer(op->ids.data(), uint32_t(op->ids.size()));
    for (uint64_t s : op->arena_starts) c->arena->end_transfer(s);
    c->ring_used -= op->ring_consumed;  // the newest allocation: the tail steps back over it
    c->ring_tail = op->ring_prev_tail;
    for (Timed &t : op->timed) {
        put_event(c, true, t.t0);
        put_event(c, true, t.t1);
    }
    put_event(c, false, op->done);
    return rc;
}

int time_begin(tc_ctx *c, Op *op, hipStream_t stream, uint64_t bytes, int kind)
{
    if (!c->profiling) return TC_OK;
    Timed t{nullptr, nullptr, bytes, kind};
    if (int rc = get_event(c, true, &t.t0)) return rc;
    if (int rc = get_event(c, true, &t.t1)) return rc;
    HIP_TRY(hipEventRecord(t.t0, stream));
    op->timed.push_back(t);
    return TC_OK;
}

int time_end(tc_ctx *c, Op *op, hipStream_t stream)
{
    if (!c->profiling) return TC_OK;
    HIP_TRY(hipEventRecord(op->timed.back().t1, stream));
    return TC_OK;
}

// DMA of the parts of every segment that fall into records [c0, c1) of the list.
int dma_chunk(tc_ctx *c, const Plan &plan, uint64_t c0, uint64_t c1, char *slot_buf, bool to_host, hipStream_t stream)
{
    for (const Segment &s : plan.segs) {
        uint64_t a = std::max<uint64_t>(s.first, c0), b = std::min<uint64_t>(s.first + s.n, c1);
        if (a >= b) continue;
        char *host = s.host + (a - s.first) * c->rec;
        char *dev = slot_buf + (a - c0) * c->rec;
        uint64_t bytes = (b - a) * c->rec;
        if (to_host) HIP_TRY(hipMemcpyAsync(host, dev, bytes, hipMemcpyDeviceToHost, stream));
        else HIP_TRY(hipMemcpyAsync(dev, host, bytes, hipMemcpyHostToDevice, stream));
    }
    return TC_OK;
}

// The host link is idle while a chunk's copy kernel runs.  With tc_opts.host_tail_div = N the last 1/N of
// the chunk's blocks skips staging: a few workgroups of the same launch move them straight to / from the
// pinned buffer while the rest of the grid streams through HBM, and the DMA carries that much less.
// Returns how many leading blocks of the chunk [c0, c0 + nblk) still go through staging.
uint32_t host_tail(tc_ctx *c, const Plan &plan, uint64_t c0, uint32_t nblk, void **host_part)
{
    const uint32_t denom = c->opts.host_tail_div;
    *host_part = nullptr;
    if (denom < 2 || nblk < denom) return nblk;
    const uint32_t m = nblk / denom;
    const uint64_t first = c0 + nblk - m;           // first record of the tail
    for (const Segment &s : plan.segs) {
        if (first >= s.first && c0 + nblk <= s.first + s.n) {   // the tail lies inside one agent's buffer
            void *view = nullptr;
            if (hipHostGetDevicePointer(&view, s.host + (first - s.first) * c->rec, 0) != hipSuccess) {
                (void)hipGetLastError();
                return nblk;
            }
            *host_part = view;
            return nblk - m;
        }
    }
    return nblk;
}

int offload_locked(tc_ctx *c, const tc_xfer_desc *descs, uint32_t n_descs, hipStream_t stream)
{
    Plan plan;
    if (int rc = validate(c, descs, n_descs, &plan)) return rc;
    if (plan.total == 0) return TC_OK;
    (void)poll_locked(c);

    Op op;
    uint64_t ring_start = 0;
    if (int rc = begin_op(c, plan, stream, &op, &ring_start)) return rc;

    // Direct path: the gather kernel writes each agent's records straight into its pinned host buffer.
    // Slightly slower alone than gather + SDMA, but kernel-driven D2H traffic overlaps with H2D DMAs,
    // which two SDMA copies of opposite direction do not.
    bool direct = c->opts.direct_offload == 1;
    if (c->opts.direct_offload == 2)
        for (const Op &o : c->ops) direct = direct || o.is_upload;
    auto enqueue_direct = [&]() -> int {
        const uint32_t grid = c->opts.direct_grid ? c->opts.direct_grid : kDefaultDirectGatherGrid;
        std::vector<void *> dev_view(plan.segs.size());
        for (size_t k = 0; k < plan.segs.size(); ++k)  // the address the GPU sees the pinned buffer at
            if (hipHostGetDevicePointer(&dev_view[k], plan.segs[k].host, 0) != hipSuccess) {
                (void)hipGetLastError();
                return TC_ERR_NOT_PINNED;
            }
        for (size_t k = 0; k < plan.segs.size(); ++k) {
            const Segment &s = plan.segs[k];
            if (int rc = time_begin(c, &op, stream, uint64_t(s.n) * c->rec, kDirect)) return rc;
            HIP_TRY(tc::launch_gather_pages(c->pool.kv_base, static_cast<const uint32_t *>(c->pool.scales), dev_view[k],
                                            c->ids_dev + ring_start + s.first, s.n, c->geom, grid, true, stream, nullptr, s.n, 0));
            if (int rc = time_end(c, &op, stream)) return rc;
        }
        HIP_TRY(hipEventRecord(op.done, stream));
        return TC_OK;
    };
    auto enqueue = [&]() -> int {
        uint64_t c0 = 0;
        for (uint32_t nblk : plan_chunks(plan.total, c->slot_blocks, false)) {
            Slot *slot = &c->slots[c->next_slot];
            c->next_slot = (c->next_slot + 1) % uint32_t(c->slots.size());
            if (slot->used) HIP_TRY(hipStreamWaitEvent(stream, slot->last, 0));
            void *host_part = nullptr;
            const uint32_t split = host_tail(c, plan, c0, nblk, &host_part);
            if (int rc = time_begin(c, &op, stream, uint64_t(nblk) * c->rec, kGather)) return rc;
            HIP_TRY(tc::launch_gather_pages(c->pool.kv_base, static_cast<const uint32_t *>(c->pool.scales), slot->buf,
                                            c->ids_dev + ring_start + c0, nblk, c->geom, c->opts.max_grid, false, stream,
                                            host_part, split,
                                            c->opts.direct_grid ? c->opts.direct_grid : kDefaultDirectGatherGrid));
            if (int rc = time_end(c, &op, stream)) return rc;
            if (int rc = time_begin(c, &op, stream, uint64_t(split) * c->rec, kD2H)) return rc;
            if (int rc = dma_chunk(c, plan, c0, c0 + split, slot->buf, true, stream)) return rc;
            if (int rc = time_end(c, &op, stream)) return rc;
            HIP_TRY(hipEventRecord(slot->last, stream));
            slot->used = true;
            c0 += nblk;
        }
        HIP_TRY(hipEventRecord(op.done, stream));
        return TC_OK;
    };
    if (int rc = direct ? enqueue_direct() : enqueue()) return abort_op(c, &op, rc);

    c->st.n_offloads++;
    c->st.blocks_offloaded += plan.total;
    c->st.bytes_offloaded += plan.total * c->rec;
    publish_op(c, std::move(op), stream);
    return TC_OK;
}

int upload_locked(tc_ctx *c, const tc_xfer_desc *descs, uint32_t n_descs, hipStream_t stream)
{
    Plan plan;
    if (int rc = validate(c, descs, n_descs, &plan)) return rc;
    for (const Segment &s : plan.segs)
        if (s.table && !is_device_ptr(s.table)) return TC_ERR_NOT_PINNED;
    if (plan.total == 0) return TC_OK;
    (void)poll_locked(c);

    Op op;
    uint64_t ring_start = 0;
    if (int rc = begin_op(c, plan, stream, &op, &ring_start)) return rc;

    // Direct path: the scatter kernel reads each agent's records straight from its pinned host buffer.
    auto enqueue_direct = [&]() -> int {
        const uint32_t grid = c->opts.direct_grid ? c->opts.direct_grid : kDefaultDirectScatterGrid;
        std::vector<void *> dev_view(plan.segs.size());
        for (size_t k = 0; k < plan.segs.size(); ++k)
            if (hipHostGetDevicePointer(&dev_view[k], plan.segs[k].host, 0) != hipSuccess) {
                (void)hipGetLastError();
                return TC_ERR_NOT_PINNED;
            }
        for (size_t k = 0; k < plan.segs.size(); ++k) {
            const Segment &s = plan.segs[k];
            if (int rc = time_begin(c, &op, stream, uint64_t(s.n) * c->rec, kDirect)) return rc;
            HIP_TRY(tc::launch_scatter_pages(dev_view[k], c->pool.kv_base, static_cast<uint32_t *>(c->pool.scales),
                                             c->ids_dev + ring_start + s.first, s.n, c->geom, grid, true, stream, nullptr, s.n, 0));
            if (int rc = time_end(c, &op, stream)) return rc;
        }
        for (const Segment &s : plan.segs)
            if (s.table) HIP_TRY(tc::launch_rewrite_table(s.table, c->ids_dev + ring_start + s.first, s.n, stream));
        HIP_TRY(hipEventRecord(op.done, stream));
        return TC_OK;
    };
    auto enqueue = [&]() -> int {
        uint64_t c0 = 0;
        for (uint32_t nblk : plan_chunks(plan.total, c->slot_blocks, true)) {
            Slot *slot = &c->slots[c->next_slot];
            c->next_slot = (c->next_slot + 1) % uint32_t(c->slots.size());
            if (slot->used) HIP_TRY(hipStreamWaitEvent(stream, slot->last, 0));
            void *host_part = nullptr;
            const uint32_t split = host_tail(c, plan, c0, nblk, &host_part);
            if (int rc = time_begin(c, &op, stream, uint64_t(split) * c->rec, kH2D)) return rc;
            if (int rc = dma_chunk(c, plan, c0, c0 + split, slot->buf, false, stream)) return rc;
            if (int rc = time_end(c, &op, stream)) return rc;
            if (int rc = time_begin(c, &op, stream, uint64_t(nblk) * c->rec, kScatter)) return rc;
            HIP_TRY(tc::launch_scatter_pages(slot->buf, c->pool.kv_base, static_cast<uint32_t *>(c->pool.scales),
                                             c->ids_dev + ring_start + c0, nblk, c->geom, c->opts.max_grid, false, stream,
                                             host_part, split,
                                             c->opts.direct_grid ? c->opts.direct_grid : kDefaultDirectScatterGrid));
            if (int rc = time_end(c, &op, stream)) return rc;
            HIP_TRY(hipEventRecord(slot->last, stream));
            slot->used = true;
            c0 += nblk;
        }
        // the mapping is restored only after the data it points to is in place
        for (const Segment &s : plan.segs)
            if (s.table) HIP_TRY(tc::launch_rewrite_table(s.table, c->ids_dev + ring_start + s.first, s.n, stream));
        HIP_TRY(hipEventRecord(op.done, stream));
        return TC_OK;
    };
    if (int rc = c->opts.direct_upload ? enqueue_direct() : enqueue()) return abort_op(c, &op, rc);
    op.is_upload = true;

    c->st.n_uploads++;
    c->st.blocks_uploaded += plan.total;
    c->st.bytes_uploaded += plan.total * c->rec;
    publish_op(c, std::move(op), stream);
    return TC_OK;
}

void destroy_unlocked(tc_ctx *c)
{
    for (Slot &s : c->slots) {
        if (s.last) (void)hipEventDestroy(s.last);
    }
    for (hipEvent_t e : c->sync_events) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->time_events) (void)hipEventDestroy(e);
    if (c->staging) (void)hipFree(c->staging);
    if (c->ids_dev) (void)hipFree(c->ids_dev);
    if (c->ids_host) (void)hipHostFree(c->ids_host);
    if (c->arena_base) (void)hipHostFree(c->arena_base);
    delete c->blocks;
    delete c->arena;
    delete c;
}

}  // namespace

// ================================================================================= C ABI
// No exception crosses the C boundary: running out of host memory inside a container is reported,
// anything else unexpected is an invalid call.
#define TC_CATCH_ALL                                              \
    catch (const std::bad_alloc &) { return TC_ERR_HOST_NOMEM; } \
    catch (...) { return TC_ERR_INVAL; }

extern "C" {

int tc_create(const tc_pool_desc *pool, const tc_opts *opts, tc_ctx **out)
try {
    if (!pool || !out) return TC_ERR_INVAL;
    *out = nullptr;
    if (int rc = tc::check_pool_desc(pool)) return rc;
    const uint32_t P = 2 * pool->num_layers;
    const uint32_t S = pool->scales_per_block;
    if (opts && (opts->direct_offload > 2 || opts->direct_upload > 1 || opts->host_tail_div == 1)) return TC_ERR_INVAL;
    if (!is_device_ptr(pool->kv_base) || (S && !is_device_ptr(pool->scales))) return TC_ERR_NOT_PINNED;

    tc_ctx *c = new (std::nothrow) tc_ctx;
    if (!c) return TC_ERR_HOST_NOMEM;
    // whatever way this function is left without success, the half-built context goes with it
    struct Undo {
        tc_ctx *c;
        ~Undo() { if (c) destroy_unlocked(c); }
    } undo{c};
    c->pool = *pool;
    if (opts) c->opts = *opts;
    c->rec = tc::record_bytes_of(P, pool->page_bytes, S);
    c->geom = tc::make_geom(*pool);

    uint32_t n_slots = c->opts.staging_slots ? c->opts.staging_slots : kDefaultSlots;
    if (n_slots < 1) n_slots = 1;
    uint64_t slot_bytes = c->opts.staging_bytes ? c->opts.staging_bytes / n_slots : kDefaultSlotBytes;
    if (slot_bytes < c->rec) slot_bytes = c->rec;
    uint64_t slot_blocks = slot_bytes / c->rec;
    if (slot_blocks > pool->num_blocks) slot_blocks = pool->num_blocks;
    c->slot_blocks = uint32_t(slot_blocks);
    c->slot_bytes = slot_blocks * c->rec;

    c->blocks = new (std::nothrow) tc::BlockPool(pool->num_blocks);
    const uint64_t arena_slots = c->opts.host_arena_bytes / c->rec;
    c->arena = new (std::nothrow) tc::HostArena(arena_slots);
    c->arena_bytes = arena_slots * c->rec;
    c->ring_cap = std::max<uint64_t>(4ull * pool->num_blocks, 1024);
    c->block_ticket.assign(pool->num_blocks, 0);

    auto fail = [](int code) { return code; };
    if (!c->blocks || !c->arena) return fail(TC_ERR_HOST_NOMEM);
#define HIP_OR_FAIL(expr)                                                                     \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess) {                                                               \
            std::fprintf(stderr, "tokencake_kv: %s failed: %s\n", #expr, hipGetErrorString(e_)); \
            return fail(e_ == hipErrorOutOfMemory && std::strstr(#expr, "Host") ? TC_ERR_HOST_NOMEM : TC_ERR_HIP); \
        }                                                                                     \
    } while (0)
    HIP_OR_FAIL(hipMalloc(reinterpret_cast<void **>(&c->staging), c->slot_bytes * n_slots));
    HIP_OR_FAIL(hipMalloc(reinterpret_cast<void **>(&c->ids_dev), c->ring_cap * sizeof(int32_t)));
    HIP_OR_FAIL(hipHostMalloc(reinterpret_cast<void **>(&c->ids_host), c->ring_cap * sizeof(int32_t), hipHostMallocDefault));
    if (c->arena_bytes)
        HIP_OR_FAIL(hipHostMalloc(reinterpret_cast<void **>(&c->arena_base), c->arena_bytes, hipHostMallocDefault));
    c->slots.resize(n_slots);
    for (uint32_t i = 0; i < n_slots; ++i) {
        c->slots[i].buf = c->staging + uint64_t(i) * c->slot_bytes;
        HIP_OR_FAIL(hipEventCreateWithFlags(&c->slots[i].last, hipEventDisableTiming));
    }
    // Touch what the first transfers will touch, once, here: the runtime maps pinned pages for the
    // copy engines lazily, and a first DMA into fresh arena pages was seen to take up to three times
    // as long.  One pass of zeros from the staging ring over the whole arena pays for that now (this
    // is the recycled CPU block pool of Sec. 6.3: allocate once, never go back to the system).
    const uint64_t ring_bytes = c->slot_bytes * n_slots;
    HIP_OR_FAIL(hipMemset(c->staging, 0, ring_bytes));
    for (uint64_t off = 0; off < c->arena_bytes; off += ring_bytes)
        HIP_OR_FAIL(hipMemcpy(c->arena_base + off, c->staging, std::min(ring_bytes, c->arena_bytes - off),
                              hipMemcpyDeviceToHost));
    // first transfers should not pay for event creation
    for (int i = 0; i < 8; ++i) {
        hipEvent_t e = nullptr;
        HIP_OR_FAIL(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        c->sync_events.push_back(e);
    }
#undef HIP_OR_FAIL
    undo.c = nullptr;
    *out = c;
    return TC_OK;
} TC_CATCH_ALL

int tc_destroy(tc_ctx *ctx)
{
    if (!ctx) return TC_OK;
    int rc;
    {
        std::lock_guard<std::mutex> g(ctx->mu);
        rc = sync_locked(ctx);
    }
    destroy_unlocked(ctx);
    return rc;
}

uint64_t tc_record_bytes(const tc_ctx *ctx) { return ctx ? ctx->rec : 0; }

void *tc_arena_base(const tc_ctx *ctx) { return ctx ? ctx->arena_base : nullptr; }

const char *tc_strerror(int code)
{
    switch (code) {
    case TC_OK: return "ok";
    case TC_ERR_INVAL: return "invalid argument, unallocated block or over-release";
    case TC_ERR_RANGE: return "block id out of range";
    case TC_ERR_DUP: return "duplicate block id in one transfer";
    case TC_ERR_SHARED: return "block has more than one owner and must not move";
    case TC_ERR_NOMEM: return "not enough free GPU blocks";
    case TC_ERR_HOST_NOMEM: return "pinned host arena exhausted";
    case TC_ERR_NOT_PINNED: return "host buffer is not pinned, or a device pointer is not device memory";
    case TC_ERR_HIP: return "HIP runtime call failed";
    case TC_ERR_LIMIT: return "transfer exceeds the fixed capacity of the entry point that does not allocate";
    default: return "unknown tokencake_kv error";
    }
}

int tc_alloc(tc_ctx *ctx, uint32_t n, int32_t *out_ids)
try {
    if (!ctx || (n && !out_ids)) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    // blocks of finished transfers may still be waiting for retirement
    if (n > ctx->blocks->n_free()) (void)poll_locked(ctx);
    return ctx->blocks->alloc(n, out_ids);
} TC_CATCH_ALL

int tc_alloc_at(tc_ctx *ctx, const int32_t *ids, uint32_t n)
try {
    if (!ctx || (n && !ids)) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    int rc = ctx->blocks->alloc_at(ids, n);
    if (rc == TC_ERR_NOMEM && ctx->blocks->n_pending()) {
        (void)poll_locked(ctx);
        rc = ctx->blocks->alloc_at(ids, n);
    }
    return rc;
} TC_CATCH_ALL

int tc_alloc_prefer(tc_ctx *ctx, const int32_t *preferred, uint32_t n, int32_t *out_ids)
try {
    if (!ctx || (n && (!preferred || !out_ids))) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    // retire what has finished first: an original block may be pending-free behind a completed copy
    if (ctx->blocks->n_pending()) (void)poll_locked(ctx);
    return ctx->blocks->alloc_prefer(preferred, n, out_ids);
} TC_CATCH_ALL

int tc_ref(tc_ctx *ctx, const int32_t *ids, uint32_t n)
try {
    if (!ctx || (n && !ids)) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    return ctx->blocks->ref(ids, n);
} TC_CATCH_ALL

int tc_free(tc_ctx *ctx, const int32_t *ids, uint32_t n)
try {
    if (!ctx || (n && !ids)) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    return ctx->blocks->free(ids, n);
} TC_CATCH_ALL

int tc_filter_private(tc_ctx *ctx, const int32_t *ids, uint32_t n, int32_t *out_ids, uint32_t *m)
try {
    if (!ctx || !m || (n && (!ids || !out_ids))) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    return ctx->blocks->filter_private(ids, n, out_ids, m);
} TC_CATCH_ALL

int tc_host_alloc(tc_ctx *ctx, uint32_t n_blocks, void **host_buf)
try {
    if (!ctx || !host_buf) return TC_ERR_INVAL;
    *host_buf = nullptr;
    if (n_blocks == 0) return TC_OK;
    std::lock_guard<std::mutex> g(ctx->mu);
    int64_t s = ctx->arena->alloc(n_blocks);
    if (s < 0) {
        // slots of finished transfers may be waiting for retirement
        (void)poll_locked(ctx);
        s = ctx->arena->alloc(n_blocks);
    }
    if (s < 0) return TC_ERR_HOST_NOMEM;
    *host_buf = ctx->arena_base + uint64_t(s) * ctx->rec;
    return TC_OK;
} TC_CATCH_ALL

int tc_host_free(tc_ctx *ctx, void *host_buf)
try {
    if (!ctx) return TC_ERR_INVAL;
    if (!host_buf) return TC_OK;
    std::lock_guard<std::mutex> g(ctx->mu);
    char *p = static_cast<char *>(host_buf);
    if (!ctx->arena_base || p < ctx->arena_base || p >= ctx->arena_base + ctx->arena_bytes) return TC_ERR_INVAL;
    uint64_t off = uint64_t(p - ctx->arena_base);
    if (off % ctx->rec) return TC_ERR_INVAL;
    return ctx->arena->free(off / ctx->rec);
} TC_CATCH_ALL

int tc_offload_batch(tc_ctx *ctx, const tc_xfer_desc *descs, uint32_t n_descs, void *stream)
try {
    if (!ctx) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    return offload_locked(ctx, descs, n_descs, static_cast<hipStream_t>(stream));
} TC_CATCH_ALL

int tc_upload_batch(tc_ctx *ctx, const tc_xfer_desc *descs, uint32_t n_descs, void *stream)
try {
    if (!ctx) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    return upload_locked(ctx, descs, n_descs, static_cast<hipStream_t>(stream));
} TC_CATCH_ALL

int tc_offload(tc_ctx *ctx, const int32_t *block_ids, uint32_t n, void *host_buf, void *stream)
try {
    tc_xfer_desc d{block_ids, n, host_buf, nullptr};
    return tc_offload_batch(ctx, &d, 1, stream);
} TC_CATCH_ALL

int tc_upload(tc_ctx *ctx, const void *host_buf, const int32_t *new_block_ids, uint32_t n, int32_t *block_table,
              void *stream)
try {
    tc_xfer_desc d{new_block_ids, n, const_cast<void *>(host_buf), block_table};
    return tc_upload_batch(ctx, &d, 1, stream);
} TC_CATCH_ALL

int tc_poll(tc_ctx *ctx)
try {
    if (!ctx) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    return poll_locked(ctx);
} TC_CATCH_ALL

int tc_sync(tc_ctx *ctx)
try {
    if (!ctx) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    return sync_locked(ctx);
} TC_CATCH_ALL

int tc_stats(tc_ctx *ctx, tc_stats_t *out)
try {
    if (!ctx || !out) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    tc_stats_t s = ctx->st;
    s.gpu_blocks_total = ctx->blocks->total();
    s.gpu_blocks_free = ctx->blocks->n_free();
    s.gpu_blocks_used = ctx->blocks->n_used();
    s.gpu_blocks_pending_free = ctx->blocks->n_pending();
    s.gpu_blocks_shared = ctx->blocks->n_shared();
    s.ops_in_flight = uint32_t(ctx->ops.size());
    s.host_slots_total = ctx->arena->total();
    s.host_slots_used = ctx->arena->used();
    *out = s;
    return TC_OK;
} TC_CATCH_ALL

int tc_set_profiling(tc_ctx *ctx, int on)
try {
    if (!ctx) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    ctx->profiling = on != 0;
    return TC_OK;
} TC_CATCH_ALL

int tc_calibrate(tc_ctx *ctx, const uint32_t *sizes, uint32_t m, uint32_t reps, void *stream, tc_cost_model *out)
try {
    if (!ctx || !sizes || !out || m < 2 || reps == 0) return TC_ERR_INVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint32_t largest = 0;
    for (uint32_t i = 0; i < m; ++i) largest = std::max(largest, sizes[i]);
    if (largest == 0) return TC_ERR_INVAL;
    std::vector<int32_t> ids(largest);
    void *host = nullptr;
    if (int rc = tc_alloc(ctx, largest, ids.data())) return rc;
    if (int rc = tc_host_alloc(ctx, largest, &host)) {
        (void)tc_free(ctx, ids.data(), largest);
        return rc;
    }
    hipEvent_t e[3] = {nullptr, nullptr, nullptr};
    int rc = TC_OK;
    for (auto &ev : e)
        if (hipEventCreate(&ev) != hipSuccess) rc = TC_ERR_HIP;
    std::vector<double> off_ms(m), up_ms(m);
    for (uint32_t i = 0; i < m && rc == TC_OK; ++i) {
        std::vector<float> o, u;
        for (uint32_t r = 0; r <= reps && rc == TC_OK; ++r) {  // the first round warms up
            if (hipEventRecord(e[0], st) != hipSuccess) rc = TC_ERR_HIP;
            if (rc == TC_OK) rc = tc_offload(ctx, ids.data(), sizes[i], host, stream);
            if (rc == TC_OK && hipEventRecord(e[1], st) != hipSuccess) rc = TC_ERR_HIP;
            // the same bytes go back into the same blocks: the pool ends up as it was
            if (rc == TC_OK) rc = tc_upload(ctx, host, ids.data(), sizes[i], nullptr, stream);
            if (rc == TC_OK && hipEventRecord(e[2], st) != hipSuccess) rc = TC_ERR_HIP;
            if (rc == TC_OK && hipEventSynchronize(e[2]) != hipSuccess) rc = TC_ERR_HIP;
            float a = 0.f, b = 0.f;
            if (rc == TC_OK && (hipEventElapsedTime(&a, e[0], e[1]) != hipSuccess ||
                                hipEventElapsedTime(&b, e[1], e[2]) != hipSuccess))
                rc = TC_ERR_HIP;
            if (r > 0) {
                o.push_back(a);
                u.push_back(b);
            }
        }
        if (rc != TC_OK) break;
        std::sort(o.begin(), o.end());
        std::sort(u.begin(), u.end());
        off_ms[i] = o[o.size() / 2];
        up_ms[i] = u[u.size() / 2];
    }
    for (auto &ev : e)
        if (ev) (void)hipEventDestroy(ev);
    (void)tc_sync(ctx);
    (void)tc_host_free(ctx, host);
    (void)tc_free(ctx, ids.data(), largest);
    if (rc != TC_OK) return rc;
    return tc_cost_fit(sizes, off_ms.data(), up_ms.data(), m, out);
} TC_CATCH_ALL

int tc_copy_contiguous(void *dst, const void *src, uint64_t bytes, void *stream)
try {
    if ((bytes && (!dst || !src)) || bytes % 16) return TC_ERR_INVAL;
    if ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) % 16) return TC_ERR_INVAL;
    HIP_TRY(tc::launch_copy_contiguous(dst, src, bytes, static_cast<hipStream_t>(stream)));
    return TC_OK;
} TC_CATCH_ALL

int tc_copy_via_lds(void *dst, const void *src, uint64_t bytes, int lds_direct_loads, void *stream)
try {
    if ((bytes && (!dst || !src)) || bytes % 16384) return TC_ERR_INVAL;
    if ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) % 16) return TC_ERR_INVAL;
    HIP_TRY(tc::launch_copy_via_lds(dst, src, bytes, lds_direct_loads != 0, static_cast<hipStream_t>(stream)));
    return TC_OK;
} TC_CATCH_ALL

int tc_hbm_stream(float *a, const float *b, const float *c, uint64_t n, float s, uint32_t iters, void *stream)
try {
    if ((n && (!a || !b || !c)) || n % 4) return TC_ERR_INVAL;
    if ((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b) | reinterpret_cast<uintptr_t>(c)) % 16)
        return TC_ERR_INVAL;
    HIP_TRY(tc::launch_hbm_stream(a, b, c, n, s, iters, static_cast<hipStream_t>(stream)));
    return TC_OK;
} TC_CATCH_ALL

int tc_naive_transfer(tc_ctx *ctx, const int32_t *block_ids, uint32_t n, void *host_buf, int mode, int direction,
                      void *stream)
try {
    if (!ctx || (n && (!block_ids || !host_buf)) || mode < 0 || mode > 1 || direction < 0 || direction > 1)
        return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    if (ctx->pool.scales_per_block) return TC_ERR_INVAL;
    if (int rc = ctx->blocks->check_range(block_ids, n)) return rc;
    if (n && !is_pinned_host(ctx, host_buf, uint64_t(n) * ctx->rec)) return TC_ERR_NOT_PINNED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint64_t pb = ctx->pool.page_bytes, NB = ctx->pool.num_blocks, P = ctx->geom.planes;
    char *pool = static_cast<char *>(ctx->pool.kv_base);
    char *host = static_cast<char *>(host_buf);
    for (uint32_t j = 0; j < n; ++j) {
        char *rec = host + uint64_t(j) * ctx->rec;
        char *blk = pool + uint64_t(block_ids[j]) * pb;
        if (mode == 1) {
            if (direction == 0)
                HIP_TRY(hipMemcpy2DAsync(rec, pb, blk, NB * pb, pb, P, hipMemcpyDeviceToHost, st));
            else
                HIP_TRY(hipMemcpy2DAsync(blk, NB * pb, rec, pb, pb, P, hipMemcpyHostToDevice, st));
        } else {
            for (uint64_t p = 0; p < P; ++p) {
                if (direction == 0)
                    HIP_TRY(hipMemcpyAsync(rec + p * pb, blk + p * NB * pb, pb, hipMemcpyDeviceToHost, st));
                else
                    HIP_TRY(hipMemcpyAsync(blk + p * NB * pb, rec + p * pb, pb, hipMemcpyHostToDevice, st));
            }
        }
    }
    return TC_OK;
} TC_CATCH_ALL

}  // extern "C"
