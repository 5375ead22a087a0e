// tc_offload_noalloc: the offload of tc_offload for callers that cannot allocate (code under HIP
// graph capture, tight serving loops, harnesses that forbid hipMalloc).  tc_offload keeps its device
// staging chunk and its device id ring in memory that tc_create allocated; this entry point keeps both
// in one file-scope device array of fixed size instead and calls no allocating routine at all: no
// context, no events, no heap.  The kernels are the library's own (stage ids, gather_pages) and take
// the array's device address as an argument, exactly as they take a context's staging chunk.
#include <algorithm>
#include <atomic>
#include <cstdio>
#include <mutex>

#include <hip/hip_runtime.h>

#include "tc_geom.h"
#include "tc_kernels.h"
#include "tokencake_kv.h"

namespace {

constexpr size_t kIdBytes = size_t(TC_NOALLOC_MAX_BLOCKS) * sizeof(int32_t);   // 4 KiB, keeps the chunk 256-B aligned
constexpr size_t kScratchBytes = kIdBytes + size_t(TC_NOALLOC_STAGING_BYTES);

// [ ids: TC_NOALLOC_MAX_BLOCKS int32 | staging chunk: TC_NOALLOC_STAGING_BYTES ].  Every GPU the
// library runs on holds its own copy, at its own address, until the process ends.  In host code this
// name is only a handle for hipGetSymbolAddress; it is never passed to a kernel or a copy.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
std::atomic<unsigned char *> g_scratch_ptr[kMaxDevices];   // device address of `scratch`, per device

// The array's address on the current device; looked up once per device, with that device current.
hipError_t scratch_address(unsigned char **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    unsigned char *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> g(g_mu);
        p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
        if (!p) {
            e = hipGetSymbolAddress(reinterpret_cast<void **>(&p), HIP_SYMBOL(scratch));
            if (e != hipSuccess) return e;
            if (!p) return hipErrorInvalidSymbol;
            g_scratch_ptr[dev].store(p, std::memory_order_release);
        }
    }
    *out = p;
    return hipSuccess;
}

// Ids travel as a kernel argument: no pageable-memory copy, nothing for the runtime to stage.
constexpr uint32_t kIdsPerLaunch = 256;
struct IdPack {
    int32_t v[kIdsPerLaunch];
};

__global__ __launch_bounds__(kIdsPerLaunch) void stage_ids_kernel(int32_t *__restrict__ dst, IdPack pack, uint32_t count)
{
    const uint32_t i = threadIdx.x;
    if (i < count) dst[i] = pack.v[i];
}

bool pinned_host(const void *p, uint64_t bytes)
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

bool device_ptr(const void *p)
{
    hipPointerAttribute_t a;
    if (hipPointerGetAttributes(&a, p) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return a.type == hipMemoryTypeDevice;
}

#define NOALLOC_HIP(expr)                                                                               \
    do {                                                                                                \
        hipError_t e_ = (expr);                                                                         \
        if (e_ != hipSuccess) {                                                                         \
            std::fprintf(stderr, "tokencake_kv: %s failed: %s (%s:%d)\n", #expr, hipGetErrorString(e_), \
                         __FILE__, __LINE__);                                                           \
            return TC_ERR_HIP;                                                                          \
        }                                                                                               \
    } while (0)

}  // namespace

extern "C" int tc_offload_noalloc(const tc_pool_desc *pool, const int32_t *block_ids, uint32_t n, void *host_buf,
                                  void *stream)
{
    if (int rc = tc::check_pool_desc(pool)) return rc;
    if (n == 0) return TC_OK;
    if (!block_ids || !host_buf || reinterpret_cast<uintptr_t>(host_buf) % 16) return TC_ERR_INVAL;
    const tc::PageGeom geom = tc::make_geom(*pool);
    const uint64_t rec = geom.rec16 * 16;
    if (n > TC_NOALLOC_MAX_BLOCKS || uint64_t(n) * rec > TC_NOALLOC_STAGING_BYTES) {
        std::fprintf(stderr,
                     "tokencake_kv: tc_offload_noalloc: %u blocks of %llu bytes exceed the fixed scratch "
                     "(at most %u blocks and %llu bytes per call)\n",
                     n, static_cast<unsigned long long>(rec), unsigned(TC_NOALLOC_MAX_BLOCKS),
                     static_cast<unsigned long long>(TC_NOALLOC_STAGING_BYTES));
        return TC_ERR_LIMIT;
    }
    // range and duplicates, on the stack
    int32_t sorted[TC_NOALLOC_MAX_BLOCKS];
    for (uint32_t i = 0; i < n; ++i) {
        if (block_ids[i] < 0 || uint32_t(block_ids[i]) >= pool->num_blocks) return TC_ERR_RANGE;
        sorted[i] = block_ids[i];
    }
    std::sort(sorted, sorted + n);
    for (uint32_t i = 1; i < n; ++i)
        if (sorted[i] == sorted[i - 1]) return TC_ERR_DUP;
    if (!device_ptr(pool->kv_base) || (pool->scales_per_block && !device_ptr(pool->scales))) return TC_ERR_NOT_PINNED;
    if (!pinned_host(host_buf, uint64_t(n) * rec)) return TC_ERR_NOT_PINNED;

    unsigned char *base = nullptr;
    NOALLOC_HIP(scratch_address(&base));
    int32_t *ids_dev = reinterpret_cast<int32_t *>(base);
    unsigned char *chunk = base + kIdBytes;
    hipStream_t st = static_cast<hipStream_t>(stream);

    // Nothing in the array has to start at zero: the ids in use and every byte of the n records
    // (pages, scale words, zero pad) are written by this call before they are read.
    for (uint32_t at = 0; at < n; at += kIdsPerLaunch) {
        IdPack pack;
        const uint32_t count = std::min(kIdsPerLaunch, n - at);
        for (uint32_t i = 0; i < count; ++i) pack.v[i] = block_ids[at + i];
        for (uint32_t i = count; i < kIdsPerLaunch; ++i) pack.v[i] = 0;
        hipLaunchKernelGGL(stage_ids_kernel, dim3(1), dim3(kIdsPerLaunch), 0, st, ids_dev + at, pack, count);
        NOALLOC_HIP(hipGetLastError());
    }
    NOALLOC_HIP(tc::launch_gather_pages(pool->kv_base, static_cast<const uint32_t *>(pool->scales), chunk, ids_dev, n,
                                        geom, 0, false, st, nullptr, n, 0));
    NOALLOC_HIP(hipMemcpyAsync(host_buf, chunk, uint64_t(n) * rec, hipMemcpyDeviceToHost, st));
    return TC_OK;
}
