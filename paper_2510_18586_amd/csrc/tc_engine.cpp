// C ABI of tokencake_kv (see include/tokencake_kv.h for the contract): the transfer engine of
// tc_engine_core.h instantiated with the HIP runtime, plus what only exists with a real device
// (allocation of staging, rings and arena; calibration; the measurement helpers).
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include <hip/hip_runtime_api.h>

#include "tc_engine_core.h"
#include "tc_kernels.h"
#include "tokencake_kv.h"
#include "tokencake_kv_bench.h"

namespace {

// A staging slot holds what one DMA carries.  4 GiB (8 GiB of staging out of 288 GB) makes one agent one chunk
// and one DMA in every shape this was measured on (a 32k-token context of an 8B model, 16k tokens of a 32B one).
// That matters beyond launch counts: a hipMemcpyAsync that is enqueued while the previous copy of the stream is
// still running, with a kernel in between, now and then runs at about half the link's rate (31-46 GB/s instead of 57;
// 3.9 GiB transfers in eight chunks: roughly every second repetition on some machines).  With the host waiting for
// the previous chunk's DMA before enqueueing the next, 72 of 72 such transfers ran at full rate, and so did every
// single-chunk transfer ever measured; the runtime picks its copy engine at enqueue time by what is busy then.
// An asynchronous call cannot wait, so the library keeps the number of DMAs per transfer small instead.
constexpr uint64_t kDefaultSlotBytes = 4096ull << 20;
constexpr uint32_t kDefaultSlots = 2;

bool report(hipError_t e, const char *what)
{
    if (e == hipSuccess) return false;
    std::fprintf(stderr, "tokencake_kv: %s failed: %s\n", what, hipGetErrorString(e));
    return true;
}
#define HIP_FAILED(expr) report((expr), #expr)

// The device interface of tc::Engine on the HIP runtime.
struct HipDev {
    using Stream = hipStream_t;
    using Event = hipEvent_t;

    int event_create(Event *out, bool timing)
    {
        return HIP_FAILED(hipEventCreateWithFlags(out, timing ? hipEventDefault : hipEventDisableTiming));
    }
    void event_destroy(Event e) { (void)hipEventDestroy(e); }
    int event_record(Event e, Stream s) { return HIP_FAILED(hipEventRecord(e, s)); }
    int event_query(Event e)
    {
        const hipError_t r = hipEventQuery(e);
        if (r == hipSuccess) return 0;
        (void)hipGetLastError();
        return r == hipErrorNotReady ? 1 : -1;
    }
    int event_sync(Event e) { return HIP_FAILED(hipEventSynchronize(e)); }
    int event_elapsed_ms(float *ms, Event a, Event b)
    {
        if (hipEventElapsedTime(ms, a, b) == hipSuccess) return 0;
        (void)hipGetLastError();
        return 1;
    }
    int stream_wait(Stream s, Event e) { return HIP_FAILED(hipStreamWaitEvent(s, e, 0)); }
    int stream_sync(Stream s) { return HIP_FAILED(hipStreamSynchronize(s)); }
    int copy_ids(int32_t *dev, const int32_t *host, uint64_t n, Stream s)
    {
        return HIP_FAILED(hipMemcpyAsync(dev, host, n * sizeof(int32_t), hipMemcpyHostToDevice, s));
    }
    int copy_d2h(void *host, const void *dev, uint64_t bytes, Stream s)
    {
        return HIP_FAILED(hipMemcpyAsync(host, dev, bytes, hipMemcpyDeviceToHost, s));
    }
    int copy_h2d(void *dev, const void *host, uint64_t bytes, Stream s)
    {
        return HIP_FAILED(hipMemcpyAsync(dev, host, bytes, hipMemcpyHostToDevice, s));
    }
    int gather(const void *pool, const uint32_t *scales, void *staging, const int32_t *ids_dev, uint32_t n,
               const tc::PageGeom &g, uint32_t max_grid, bool direct, Stream s, void *host_part, uint32_t split,
               uint32_t host_wgs)
    {
        return HIP_FAILED(tc::launch_gather_pages(pool, scales, staging, ids_dev, n, g, max_grid, direct, s, host_part,
                                                  split, host_wgs));
    }
    int scatter(const void *staging, void *pool, uint32_t *scales, const int32_t *ids_dev, uint32_t n,
                const tc::PageGeom &g, uint32_t max_grid, bool direct, Stream s, const void *host_part, uint32_t split,
                uint32_t host_wgs)
    {
        return HIP_FAILED(tc::launch_scatter_pages(staging, pool, scales, ids_dev, n, g, max_grid, direct, s, host_part,
                                                   split, host_wgs));
    }
    int rewrite(int32_t *table, const int32_t *ids_dev, uint32_t n, Stream s)
    {
        return HIP_FAILED(tc::launch_rewrite_table(table, ids_dev, n, s));
    }
    int device_view(void **out, void *host)
    {
        if (hipHostGetDevicePointer(out, host, 0) == hipSuccess) return 0;
        (void)hipGetLastError();
        return 1;
    }
    bool is_pinned_host(const void *p, uint64_t bytes)
    {
        const char *b = static_cast<const char *>(p);
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
};

}  // namespace

struct tc_ctx {
    std::mutex mu;
    tc::Engine<HipDev> e;
    char *staging = nullptr;
};

namespace {

#define HIP_TRY(expr)                          \
    do {                                       \
        if (HIP_FAILED(expr)) return TC_ERR_HIP; \
    } while (0)

void destroy_unlocked(tc_ctx *c)
{
    auto &e = c->e;
    for (auto &s : e.slots) {
        if (s.last) (void)hipEventDestroy(s.last);
        if (s.ready) (void)hipEventDestroy(s.ready);
    }
    if (e.has_kstream) (void)hipStreamDestroy(e.kstream);
    for (hipEvent_t ev : e.sync_events) (void)hipEventDestroy(ev);
    for (hipEvent_t ev : e.time_events) (void)hipEventDestroy(ev);
    if (c->staging) (void)hipFree(c->staging);
    if (e.ids_dev) (void)hipFree(e.ids_dev);
    if (e.ids_host) (void)hipHostFree(e.ids_host);
    if (e.arena_base) (void)hipHostFree(e.arena_base);
    delete e.book;
    delete e.blocks;
    delete e.arena;
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
    if (opts && (opts->direct_offload > tc::kPathStaged || opts->direct_upload > tc::kPathStaged ||
                 opts->direct_upload == tc::kPathDirectIfDuplex || opts->overlap_kernels > 1 || opts->reserved0 != 0))
        return TC_ERR_INVAL;
    HipDev probe;
    if (!probe.is_device_ptr(pool->kv_base) || (S && !probe.is_device_ptr(pool->scales))) return TC_ERR_NOT_PINNED;

    tc_ctx *c = new (std::nothrow) tc_ctx;
    if (!c) return TC_ERR_HOST_NOMEM;
    // whatever way this function is left without success, the half-built context goes with it
    struct Undo {
        tc_ctx *c;
        ~Undo() { if (c) destroy_unlocked(c); }
    } undo{c};
    auto &e = c->e;
    e.pool = *pool;
    if (opts) e.opts = *opts;
    e.rec = tc::record_bytes_of(P, pool->page_bytes, S);
    e.geom = tc::make_geom(*pool);

    uint32_t n_slots = e.opts.staging_slots ? e.opts.staging_slots : kDefaultSlots;
    uint64_t slot_bytes = e.opts.staging_bytes ? e.opts.staging_bytes / n_slots : kDefaultSlotBytes;
    if (slot_bytes < e.rec) slot_bytes = e.rec;
    uint64_t slot_blocks = slot_bytes / e.rec;
    if (slot_blocks > pool->num_blocks) slot_blocks = pool->num_blocks;
    e.slot_blocks = uint32_t(slot_blocks);
    slot_bytes = slot_blocks * e.rec;

    const uint64_t ring_cap = std::max<uint64_t>(4ull * pool->num_blocks, 1024);
    e.blocks = new (std::nothrow) tc::BlockPool(pool->num_blocks);
    const uint64_t arena_slots = e.opts.host_arena_bytes / e.rec;
    e.arena = new (std::nothrow) tc::HostArena(arena_slots);
    e.arena_bytes = arena_slots * e.rec;
    e.book = new (std::nothrow) tc::Engine<HipDev>::Book(ring_cap, pool->num_blocks);
    if (!e.blocks || !e.arena || !e.book) return TC_ERR_HOST_NOMEM;

#define HIP_OR_FAIL(expr)                                                                     \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess) {                                                               \
            std::fprintf(stderr, "tokencake_kv: %s failed: %s\n", #expr, hipGetErrorString(e_)); \
            return e_ == hipErrorOutOfMemory && std::strstr(#expr, "Host") ? TC_ERR_HOST_NOMEM : TC_ERR_HIP; \
        }                                                                                     \
    } while (0)
    // The default ring is generous (see kDefaultSlotBytes).  Where the pool leaves less room than that, a default
    // ring shrinks by halves (down to 64 MiB per slot) rather than failing; a size the caller asked for is taken
    // literally.
    for (;;) {
        const hipError_t err = hipMalloc(reinterpret_cast<void **>(&c->staging), slot_bytes * n_slots);
        if (err == hipSuccess) break;
        c->staging = nullptr;
        (void)hipGetLastError();
        if (err != hipErrorOutOfMemory || e.opts.staging_bytes != 0 || slot_blocks < 2 || slot_bytes <= (64ull << 20)) {
            std::fprintf(stderr, "tokencake_kv: hipMalloc of %llu B of staging failed: %s\n",
                         static_cast<unsigned long long>(slot_bytes * n_slots), hipGetErrorString(err));
            return TC_ERR_HIP;
        }
        slot_blocks = (slot_blocks + 1) / 2;
        e.slot_blocks = uint32_t(slot_blocks);
        slot_bytes = slot_blocks * e.rec;
    }
    HIP_OR_FAIL(hipMalloc(reinterpret_cast<void **>(&e.ids_dev), ring_cap * sizeof(int32_t)));
    HIP_OR_FAIL(hipHostMalloc(reinterpret_cast<void **>(&e.ids_host), ring_cap * sizeof(int32_t), hipHostMallocDefault));
    if (e.arena_bytes)
        HIP_OR_FAIL(hipHostMalloc(reinterpret_cast<void **>(&e.arena_base), e.arena_bytes, hipHostMallocDefault));
    e.slots.resize(n_slots);
    for (uint32_t i = 0; i < n_slots; ++i) {
        e.slots[i].buf = c->staging + uint64_t(i) * slot_bytes;
        HIP_OR_FAIL(hipEventCreateWithFlags(&e.slots[i].last, hipEventDisableTiming));
        HIP_OR_FAIL(hipEventCreateWithFlags(&e.slots[i].ready, hipEventDisableTiming));
    }
    // the engine's own stream for the copy kernels of multi-chunk transfers; default priority, like every stream here
    if (e.opts.overlap_kernels == 1) {
        HIP_OR_FAIL(hipStreamCreateWithFlags(&e.kstream, hipStreamNonBlocking));
        e.has_kstream = true;
    }
    // Touch what the first transfers will touch, once, here: the runtime maps pinned pages for the
    // copy engines lazily, and a first DMA into fresh arena pages was seen to take up to three times
    // as long.  One pass of zeros from the staging ring over the whole arena pays for that now (this
    // is the recycled CPU block pool of Sec. 6.3: allocate once, never go back to the system).
    const uint64_t ring_bytes = slot_bytes * n_slots;
    HIP_OR_FAIL(hipMemset(c->staging, 0, ring_bytes));
    for (uint64_t off = 0; off < e.arena_bytes; off += ring_bytes)
        HIP_OR_FAIL(hipMemcpy(e.arena_base + off, c->staging, std::min(ring_bytes, e.arena_bytes - off),
                              hipMemcpyDeviceToHost));
    // first transfers should not pay for event creation
    for (int i = 0; i < 8; ++i) {
        hipEvent_t ev = nullptr;
        HIP_OR_FAIL(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
        e.sync_events.push_back(ev);
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
        rc = ctx->e.sync();
    }
    destroy_unlocked(ctx);
    return rc;
}

uint64_t tc_record_bytes(const tc_ctx *ctx) { return ctx ? ctx->e.rec : 0; }

void *tc_arena_base(const tc_ctx *ctx) { return ctx ? ctx->e.arena_base : nullptr; }

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
    if (n > ctx->e.blocks->n_free()) (void)ctx->e.poll();
    return ctx->e.blocks->alloc(n, out_ids);
} TC_CATCH_ALL

int tc_alloc_at(tc_ctx *ctx, const int32_t *ids, uint32_t n)
try {
    if (!ctx || (n && !ids)) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    int rc = ctx->e.blocks->alloc_at(ids, n);
    if (rc == TC_ERR_NOMEM && ctx->e.blocks->n_pending()) {
        (void)ctx->e.poll();
        rc = ctx->e.blocks->alloc_at(ids, n);
    }
    return rc;
} TC_CATCH_ALL

int tc_alloc_prefer(tc_ctx *ctx, const int32_t *preferred, uint32_t n, int32_t *out_ids)
try {
    if (!ctx || (n && (!preferred || !out_ids))) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    // retire what has finished first: an original block may be pending-free behind a completed copy
    if (ctx->e.blocks->n_pending()) (void)ctx->e.poll();
    return ctx->e.blocks->alloc_prefer(preferred, n, out_ids);
} TC_CATCH_ALL

int tc_ref(tc_ctx *ctx, const int32_t *ids, uint32_t n)
try {
    if (!ctx || (n && !ids)) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    return ctx->e.blocks->ref(ids, n);
} TC_CATCH_ALL

int tc_free(tc_ctx *ctx, const int32_t *ids, uint32_t n)
try {
    if (!ctx || (n && !ids)) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    return ctx->e.blocks->free(ids, n);
} TC_CATCH_ALL

int tc_filter_private(tc_ctx *ctx, const int32_t *ids, uint32_t n, int32_t *out_ids, uint32_t *m)
try {
    if (!ctx || !m || (n && (!ids || !out_ids))) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    return ctx->e.blocks->filter_private(ids, n, out_ids, m);
} TC_CATCH_ALL

int tc_host_alloc(tc_ctx *ctx, uint32_t n_blocks, void **host_buf)
try {
    if (!ctx || !host_buf) return TC_ERR_INVAL;
    *host_buf = nullptr;
    if (n_blocks == 0) return TC_OK;
    std::lock_guard<std::mutex> g(ctx->mu);
    auto &e = ctx->e;
    int64_t s = e.arena->alloc(n_blocks);
    if (s < 0) {
        // slots of finished transfers may be waiting for retirement
        (void)e.poll();
        s = e.arena->alloc(n_blocks);
    }
    if (s < 0) return TC_ERR_HOST_NOMEM;
    *host_buf = e.arena_base + uint64_t(s) * e.rec;
    return TC_OK;
} TC_CATCH_ALL

int tc_host_free(tc_ctx *ctx, void *host_buf)
try {
    if (!ctx) return TC_ERR_INVAL;
    if (!host_buf) return TC_OK;
    std::lock_guard<std::mutex> g(ctx->mu);
    auto &e = ctx->e;
    char *p = static_cast<char *>(host_buf);
    if (!e.in_arena(p)) return TC_ERR_INVAL;
    const uint64_t off = uint64_t(p - e.arena_base);
    if (off % e.rec) return TC_ERR_INVAL;
    return e.arena->free(off / e.rec);
} TC_CATCH_ALL

int tc_offload_batch(tc_ctx *ctx, const tc_xfer_desc *descs, uint32_t n_descs, void *stream)
try {
    if (!ctx) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    return ctx->e.offload(descs, n_descs, static_cast<hipStream_t>(stream));
} TC_CATCH_ALL

int tc_upload_batch(tc_ctx *ctx, const tc_xfer_desc *descs, uint32_t n_descs, void *stream)
try {
    if (!ctx) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    return ctx->e.upload(descs, n_descs, static_cast<hipStream_t>(stream));
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
    return ctx->e.poll();
} TC_CATCH_ALL

int tc_sync(tc_ctx *ctx)
try {
    if (!ctx) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    return ctx->e.sync();
} TC_CATCH_ALL

int tc_stats(tc_ctx *ctx, tc_stats_t *out)
try {
    if (!ctx || !out) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    ctx->e.fill_stats(out);
    return TC_OK;
} TC_CATCH_ALL

int tc_set_profiling(tc_ctx *ctx, int on)
try {
    if (!ctx) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    ctx->e.profiling = on != 0;
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

int tc_hbm_write(void *dst, uint64_t bytes, void *stream)
try {
    if ((bytes && !dst) || bytes % 4096 || reinterpret_cast<uintptr_t>(dst) % 16) return TC_ERR_INVAL;
    HIP_TRY(tc::launch_hbm_one_way(dst, bytes, true, static_cast<hipStream_t>(stream)));
    return TC_OK;
} TC_CATCH_ALL

int tc_hbm_read(const void *src, uint64_t bytes, void *stream)
try {
    if ((bytes && !src) || bytes % 4096 || reinterpret_cast<uintptr_t>(src) % 16) return TC_ERR_INVAL;
    HIP_TRY(tc::launch_hbm_one_way(const_cast<void *>(src), bytes, false, static_cast<hipStream_t>(stream)));
    return TC_OK;
} TC_CATCH_ALL

int tc_stage_on_device(tc_ctx *ctx, int direction, const int32_t *block_ids, uint32_t n, void *dev_records, void *stream)
try {
    if (!ctx) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ctx->mu);
    return ctx->e.stage_on_device(direction, block_ids, n, dev_records, static_cast<hipStream_t>(stream));
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
    auto &e = ctx->e;
    if (e.pool.scales_per_block) return TC_ERR_INVAL;
    if (int rc = e.blocks->check_range(block_ids, n)) return rc;
    if (n && !e.pinned(host_buf, uint64_t(n) * e.rec)) return TC_ERR_NOT_PINNED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint64_t pb = e.pool.page_bytes, NB = e.pool.num_blocks, P = e.geom.planes;
    char *pool = static_cast<char *>(e.pool.kv_base);
    char *host = static_cast<char *>(host_buf);
    for (uint32_t j = 0; j < n; ++j) {
        char *rec = host + uint64_t(j) * e.rec;
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
