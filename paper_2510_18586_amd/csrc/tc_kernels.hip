// gfx950 kernels of the KV offload / upload path (paper Sec. 6.3: KV blocks migrate between GPU
// blocks and CPU blocks; Sec. 7.6: a block is block_size tokens of every layer's K and V).
//
// gather_pages   pool (plane-major, pages of one block strided by NB*page_bytes) -> staging
//                chunk (block-major records, the host layout), so that one contiguous DMA can
//                carry many blocks over the host link.
// scatter_pages  the inverse, into the destination blocks of an upload.
// rewrite_table  block_table[i] = new_ids[i] once the data is in place.
//
// Both copy kernels are pure HBM streaming: a workgroup of four wave64 moves one tile of a page,
// every lane with U independent 16-byte loads in flight before the first store (a wave
// instruction covers 1 KiB of consecutive addresses).  There is no arithmetic on the payload and
// no reuse, so neither LDS nor MFMA has anything to add; bytes are never reinterpreted.
#include <hip/hip_runtime.h>

#include "tc_kernels.h"

namespace tc {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kThreads = kCopyThreads;

template <bool NT>
__device__ __forceinline__ u32x4 ld16(const u32x4 *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT>
__device__ __forceinline__ void st16(u32x4 *p, u32x4 v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// One work item = (block k of the chunk, plane p, tile t of the page).  Items are ordered with
// the tile fastest, then the plane: consecutive workgroups write (gather) or read (scatter)
// consecutive staging addresses.
// DIRECT marks the launches whose "staging" side is pinned host memory: the same code, but a
// distinct kernel for the profiler, because those launches are bound by the host link, not by HBM.
// TAIL marks the launches that also carry a host part (see below); without it that code is not there.
template <int U, bool NTL, bool NTS, bool GATHER, bool DIRECT, bool TAIL>
__global__ __launch_bounds__(kThreads) void page_copy_kernel(
    u32x4 *__restrict__ pool, uint32_t *__restrict__ scales, u32x4 *__restrict__ staging,
    const int32_t *__restrict__ ids, uint32_t n_items, uint32_t tiles, PageGeom g,
    u32x4 *__restrict__ host_part, uint32_t split, uint32_t host_wgs)
{
    constexpr uint32_t kTile = kThreads * U;  // 16-byte units per tile
    // Records of blocks [0, split) live in `staging`; records of blocks [split, n) in `host_part` (pinned
    // host memory seen from the GPU).  The first host_wgs workgroups take the host-side items, so that the
    // link is busy from the start of the launch; everybody else takes the staging-side items.
    uint32_t first = blockIdx.x, last = n_items, step = gridDim.x;
    if constexpr (TAIL) {
        const uint32_t items_staged = split * g.planes * tiles;
        if (blockIdx.x < host_wgs) { first = items_staged + blockIdx.x; last = n_items; step = host_wgs; }
        else { first = blockIdx.x - host_wgs; last = items_staged; step = gridDim.x - host_wgs; }
    }
    for (uint32_t item = first; item < last; item += step) {
        const uint32_t t = item % tiles;
        const uint32_t kp = item / tiles;
        const uint32_t p = kp % g.planes;
        const uint32_t k = kp / g.planes;
        const uint64_t blk = uint64_t(uint32_t(ids[k]));

        // wave-uniform bases; the lane offset stays 32-bit so loads use scalar-base addressing
        u32x4 *in_pool = pool + (uint64_t(p) * g.num_blocks + blk) * g.page16 + t * kTile;
        u32x4 *record = staging + uint64_t(k) * g.rec16;
        if constexpr (TAIL)
            if (k >= split) record = host_part + uint64_t(k - split) * g.rec16;
        u32x4 *in_stag = record + uint64_t(p) * g.page16 + t * kTile;
        const u32x4 *src = GATHER ? in_pool : in_stag;
        u32x4 *dst = GATHER ? in_stag : in_pool;
        const uint32_t lane = threadIdx.x;
        const uint32_t left = g.page16 - t * kTile;  // 16-byte units from the tile start to the page end

        u32x4 v[U];
        if (left >= kTile) {  // full tile: U loads in flight, then U stores, no predicates
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = ld16<NTL>(src + lane + u * kThreads);
#pragma unroll
            for (int u = 0; u < U; ++u) st16<NTS>(dst + lane + u * kThreads, v[u]);
        } else {              // ragged last tile of a page
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (lane + u * kThreads < left) st16<NTS>(dst + lane + u * kThreads, ld16<NTL>(src + lane + u * kThreads));
        }

        // the record's tail: S scale words gathered from their planes, then zero pad
        if (g.tail_words && p == 0 && t == 0) {
            uint32_t *tail = reinterpret_cast<uint32_t *>(record + uint64_t(g.planes) * g.page16);
            for (uint32_t w = threadIdx.x; w < g.tail_words; w += kThreads) {
                if (GATHER) tail[w] = (w < g.scales) ? scales[uint64_t(w) * g.num_blocks + blk] : 0u;
                else if (w < g.scales) scales[uint64_t(w) * g.num_blocks + blk] = tail[w];
            }
        }
    }
}

__global__ __launch_bounds__(kThreads) void rewrite_table_kernel(int32_t *__restrict__ table,
                                                                  const int32_t *__restrict__ ids, uint32_t n)
{
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i < n) table[i] = ids[i];
}

template <int U, bool NT>
__global__ __launch_bounds__(kThreads) void copy_contiguous_kernel(u32x4 *__restrict__ dst,
                                                                    const u32x4 *__restrict__ src, uint64_t n16)
{
    const uint64_t tile = uint64_t(blockIdx.x) * (kThreads * U);
    const u32x4 *s = src + tile;
    u32x4 *d = dst + tile;
    const uint32_t lane = threadIdx.x;
    const uint64_t left = n16 - tile;
    if (left >= kThreads * U) {
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = ld16<NT>(s + lane + u * kThreads);
#pragma unroll
        for (int u = 0; u < U; ++u) st16<NT>(d + lane + u * kThreads, v[u]);
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (lane + u * kThreads < left) st16<NT>(d + lane + u * kThreads, ld16<NT>(s + lane + u * kThreads));
    }
}

// The same contiguous copy with the tile staged in LDS, kept to measure what LDS adds to a copy that
// has no reuse.  DMA = false: loads into registers, ds_write, barrier, ds_read, stores.  DMA = true:
// LDS-direct loads (each lane names its own global address; a wave's 64 x 16 bytes land consecutively
// at a wave-uniform LDS address), then ds_read and stores.  Whole tiles only.
template <int U, bool DMA>
__global__ __launch_bounds__(kThreads) void copy_via_lds_kernel(u32x4 *__restrict__ dst, const u32x4 *__restrict__ src)
{
    __shared__ u32x4 buf[kThreads * U];
    const uint64_t base = uint64_t(blockIdx.x) * (kThreads * U) + threadIdx.x;
    if constexpr (DMA) {
        const uint32_t wave = threadIdx.x / 64;
#pragma unroll
        for (int u = 0; u < U; ++u)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src + base + u * kThreads),
                                             (__attribute__((address_space(3))) void *)(buf + u * kThreads + wave * 64),
                                             16, 0, 0);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    } else {
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = ld16<true>(src + base + u * kThreads);
#pragma unroll
        for (int u = 0; u < U; ++u) buf[u * kThreads + threadIdx.x] = v[u];
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < U; ++u) st16<true>(dst + base + u * kThreads, buf[u * kThreads + threadIdx.x]);
}

typedef float f32x4 __attribute__((ext_vector_type(4)));

// One pass of a = b + s*c; a workgroup covers 4 consecutive 4 KiB rows and retires, so that
// workgroups of other streams interleave with it as they would with an ordinary memory-bound kernel.
__global__ __launch_bounds__(kThreads) void hbm_stream_kernel(f32x4 *__restrict__ a, const f32x4 *__restrict__ b,
                                                               const f32x4 *__restrict__ c, uint64_t n4, float s)
{
    const uint64_t base = uint64_t(blockIdx.x) * (kThreads * 4) + threadIdx.x;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const uint64_t i = base + u * kThreads;
        if (i < n4) {
            f32x4 x = b[i], y = c[i];
            a[i] = x + s * y;
        }
    }
}

// ---------------------------------------------------------------------------------------------
template <bool GATHER>
static hipError_t launch_page_copy(void *pool, uint32_t *scales, void *staging, const int32_t *ids_dev, uint32_t n,
                                   const PageGeom &g, uint32_t max_grid, bool direct, hipStream_t stream,
                                   void *host_part, uint32_t split, uint32_t host_wgs)
{
    if (n == 0) return hipSuccess;
    const uint32_t U = tile_units(g.page16);  // widest tile that a page still fills
    // Cache policy, measured on MI355X with cold 512 MiB launches in the offload -> upload sequence:
    // non-temporal loads help both directions.  The gather's staging writes stay ordinary
    // write-back stores: they are absorbed by the memory-side cache and drain to HBM while the
    // slow host-link DMA that follows reads them.  The scatter's page writes are non-temporal, so
    // it leaves no dirty lines for the next kernel to evict (with ordinary stores the scatter looks
    // faster and the following gather pays for it; the sum is worse).
    const uint32_t tiles = tiles_per_page(g.page16);
    const uint64_t items64 = uint64_t(n) * g.planes * tiles;
    if (items64 > 0x7fffffffull) return hipErrorInvalidValue;
    const uint32_t n_items = uint32_t(items64);
    if (split > n || (split < n && (!host_part || host_wgs == 0 || direct))) return hipErrorInvalidValue;
    if (split == n) host_wgs = 0;
    const uint32_t items_staged = split * g.planes * tiles;
    uint32_t grid = items_staged;
    if (max_grid && grid > max_grid) grid = max_grid;
    if (grid == 0 && host_wgs == 0) return hipSuccess;
    grid += host_wgs;

#define TC_LAUNCH(UU, NL, NS, DR, TL)                                                                          \
    hipLaunchKernelGGL((page_copy_kernel<UU, NL, NS, GATHER, DR, TL>), dim3(grid), dim3(kThreads), 0, stream,    \
                       static_cast<u32x4 *>(pool), scales, static_cast<u32x4 *>(staging), ids_dev, n_items, \
                       tiles, g, static_cast<u32x4 *>(host_part), split, host_wgs)
#define TC_LAUNCH_U(NL, NS, DR, TL)                  \
    switch (U) {                                     \
    case 8: TC_LAUNCH(8, NL, NS, DR, TL); break;     \
    case 4: TC_LAUNCH(4, NL, NS, DR, TL); break;     \
    case 2: TC_LAUNCH(2, NL, NS, DR, TL); break;     \
    default: TC_LAUNCH(1, NL, NS, DR, TL); break;    \
    }
    const bool tail = host_wgs != 0;
    if (direct) { TC_LAUNCH_U(true, true, true, false) }
    else if (GATHER && tail) { TC_LAUNCH_U(true, false, false, true) }
    else if (GATHER) { TC_LAUNCH_U(true, false, false, false) }
    else if (tail) { TC_LAUNCH_U(true, true, false, true) }
    else { TC_LAUNCH_U(true, true, false, false) }
#undef TC_LAUNCH_U
#undef TC_LAUNCH
    return hipGetLastError();
}

hipError_t launch_gather_pages(const void *pool, const uint32_t *scales, void *staging, const int32_t *ids_dev,
                               uint32_t n, const PageGeom &g, uint32_t max_grid, bool direct, hipStream_t stream,
                               void *host_part, uint32_t split, uint32_t host_wgs)
{
    return launch_page_copy<true>(const_cast<void *>(pool), const_cast<uint32_t *>(scales), staging, ids_dev, n, g,
                                  max_grid, direct, stream, host_part, split, host_wgs);
}

hipError_t launch_scatter_pages(const void *staging, void *pool, uint32_t *scales, const int32_t *ids_dev,
                                uint32_t n, const PageGeom &g, uint32_t max_grid, bool direct, hipStream_t stream,
                                const void *host_part, uint32_t split, uint32_t host_wgs)
{
    return launch_page_copy<false>(pool, scales, const_cast<void *>(staging), ids_dev, n, g, max_grid, direct, stream,
                                   const_cast<void *>(host_part), split, host_wgs);
}

hipError_t launch_rewrite_table(int32_t *table, const int32_t *ids_dev, uint32_t n, hipStream_t stream)
{
    if (n == 0 || table == nullptr) return hipSuccess;
    hipLaunchKernelGGL(rewrite_table_kernel, dim3((n + kThreads - 1) / kThreads), dim3(kThreads), 0, stream, table,
                       ids_dev, n);
    return hipGetLastError();
}

hipError_t launch_copy_contiguous(void *dst, const void *src, uint64_t bytes, hipStream_t stream)
{
    if (bytes == 0) return hipSuccess;
    const uint64_t n16 = bytes / 16;
    const uint64_t grid = (n16 + kThreads * 8 - 1) / (kThreads * 8);
    if (grid > 0x7fffffffull) return hipErrorInvalidValue;
    hipLaunchKernelGGL((copy_contiguous_kernel<8, true>), dim3(uint32_t(grid)), dim3(kThreads), 0, stream,
                       static_cast<u32x4 *>(dst), static_cast<const u32x4 *>(src), n16);
    return hipGetLastError();
}

hipError_t launch_copy_via_lds(void *dst, const void *src, uint64_t bytes, bool lds_direct_loads, hipStream_t stream)
{
    constexpr int U = 4;                                   // 16 KiB of LDS per workgroup
    constexpr uint64_t kTileBytes = uint64_t(kThreads) * U * 16;
    if (bytes == 0) return hipSuccess;
    if (bytes % kTileBytes) return hipErrorInvalidValue;   // the kernel has no ragged path
    const uint64_t grid = bytes / kTileBytes;
    if (grid > 0x7fffffffull) return hipErrorInvalidValue;
    if (lds_direct_loads)
        hipLaunchKernelGGL((copy_via_lds_kernel<U, true>), dim3(uint32_t(grid)), dim3(kThreads), 0, stream,
                           static_cast<u32x4 *>(dst), static_cast<const u32x4 *>(src));
    else
        hipLaunchKernelGGL((copy_via_lds_kernel<U, false>), dim3(uint32_t(grid)), dim3(kThreads), 0, stream,
                           static_cast<u32x4 *>(dst), static_cast<const u32x4 *>(src));
    return hipGetLastError();
}

hipError_t launch_hbm_stream(float *a, const float *b, const float *c, uint64_t n, float s, uint32_t iters,
                             hipStream_t stream)
{
    if (n == 0 || iters == 0) return hipSuccess;
    const uint64_t n4 = n / 4;
    const uint64_t grid = (n4 + kThreads * 4 - 1) / (kThreads * 4);
    if (grid > 0x7fffffffull) return hipErrorInvalidValue;
    for (uint32_t it = 0; it < iters; ++it)
        hipLaunchKernelGGL(hbm_stream_kernel, dim3(uint32_t(grid)), dim3(kThreads), 0, stream,
                           reinterpret_cast<f32x4 *>(a), reinterpret_cast<const f32x4 *>(b),
                           reinterpret_cast<const f32x4 *>(c), n4, s);
    return hipGetLastError();
}

}  // namespace tc
