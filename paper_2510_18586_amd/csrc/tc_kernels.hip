// gfx950 kernels of the KV offload / upload path (paper Sec. 6.3: KV blocks migrate between GPU
// blocks and CPU blocks; Sec. 7.6: a block is block_size tokens of every layer's K and V).
//
// gather_pages   pool (plane-major, pages of one block strided by NB*page_bytes) -> staging
//                chunk (block-major records, the host layout), so that one contiguous DMA can
//                carry many blocks over the host link.
// scatter_pages  the inverse, into the destination blocks of an upload.
// rewrite_table  block_table[i] = new_ids[i] once the data is in place.
//
// Both copy kernels are pure HBM streaming: a workgroup of four wave64 moves 4 KiB tiles of pages,
// every lane 16 bytes per tile (a wave instruction covers 1 KiB of consecutive addresses).  There is
// no arithmetic on the payload and no reuse, so neither LDS nor MFMA has anything to add; bytes are
// never reinterpreted.
#include <algorithm>
#include <type_traits>

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

// One work item = (block k of the chunk, plane p, 4 KiB tile t of the page), ordered with the tile
// fastest, then the plane: consecutive items are consecutive addresses on the record side.
//
// Item -> workgroup.  HBM sustains more when each XCD streams a region of its own than when the eight
// XCDs interleave 4 KiB pieces of one region, and more with many small workgroups than with few large
// ones (measured on MI355X: scatter 196 -> 177 us, gather 158 -> 150 us per 512 MiB).  So the staged
// launches cut the items into `chunks` = 8 contiguous runs; workgroup b (on XCD b mod 8) walks run
// b mod 8, and V = 1: one tile per iteration, one iteration per workgroup unless the grid is capped.
// The launches that touch pinned host memory are bound by the host link and run on a handful of
// workgroups; those need many loads in flight per lane instead: V = 8 consecutive tiles per iteration,
// no cut (DIRECT), or the first host_wgs workgroups of a staged launch (TAIL).
//
// DIRECT marks the launches whose "staging" side is pinned host memory: the same code, but a distinct
// kernel for the profiler, because those launches are bound by the host link, not by HBM.
// TAIL marks the launches that also carry a host part; without it that code is not there.
template <bool NTL, bool NTS, bool GATHER, bool DIRECT, bool TAIL>
__global__ __launch_bounds__(kThreads) void page_copy_kernel(
    u32x4 *__restrict__ pool, uint32_t *__restrict__ scales, u32x4 *__restrict__ staging,
    const int32_t *__restrict__ ids, u32x4 *__restrict__ host_part, CopyPlan c)
{
    const PageGeom &g = c.g;
    const uint32_t lane = threadIdx.x;

    // where item `at` lives on both sides
    struct Place {
        const u32x4 *src;
        u32x4 *dst;
        u32x4 *record;
        uint32_t left;   // 16-byte units from the tile start to the page end
    };
    auto place = [&](const ItemPos &at, uint64_t blk) -> Place {
        // wave-uniform bases; the lane offset stays 32-bit so loads use scalar-base addressing
        const ItemPlace w = item_place(at, blk, g, TAIL ? c.split : 0xffffffffu);
        u32x4 *in_pool = pool + w.pool16;
        u32x4 *record = (TAIL && w.in_host_part ? host_part : staging) + w.record16;
        u32x4 *in_stag = record + w.tile16;
        return Place{GATHER ? in_pool : in_stag, GATHER ? in_stag : in_pool, record, w.left};
    };
    // the record's tail, moved by the workgroup that has the block's first item: S scale words gathered from
    // (scattered to) their planes, then zero pad
    auto move_tail = [&](const ItemPos &at, uint64_t blk, u32x4 *record) {
        if (g.tail_words == 0 || at.p != 0 || at.t != 0) return;
        uint32_t *tail = reinterpret_cast<uint32_t *>(record + uint64_t(g.planes) * g.page16);
        for (uint32_t w = lane; w < g.tail_words; w += kThreads) {
            if (GATHER) tail[w] = (w < g.scales) ? scales[uint64_t(w) * g.num_blocks + blk] : 0u;
            else if (w < g.scales) scales[uint64_t(w) * g.num_blocks + blk] = tail[w];
        }
    };

    // moves items [item, item + count), count <= V, all loads issued before the first store
    auto move = [&](uint32_t item, uint32_t count, auto vtag) {
        constexpr int V = decltype(vtag)::value;
        u32x4 v[V];
        const ItemPos first = item_pos(item, c.tiles, c.planes);
        if (V == 1 || (count == V && first.t + V <= c.tiles.d)) {
            // all V tiles lie in one page: one look-up, consecutive addresses
            const uint64_t blk = uint64_t(uint32_t(ids[first.k]));
            const Place pl = place(first, blk);
            if (pl.left >= uint32_t(V) * kThreads) {   // and all of them are full: V loads in flight, then V stores, no predicates
#pragma unroll
                for (int u = 0; u < V; ++u) v[u] = ld16<NTL>(pl.src + lane + u * kThreads);
#pragma unroll
                for (int u = 0; u < V; ++u) st16<NTS>(pl.dst + lane + u * kThreads, v[u]);
            } else {
#pragma unroll
                for (int u = 0; u < V; ++u)
                    if (lane + u * kThreads < pl.left) v[u] = ld16<NTL>(pl.src + lane + u * kThreads);
#pragma unroll
                for (int u = 0; u < V; ++u)
                    if (lane + u * kThreads < pl.left) st16<NTS>(pl.dst + lane + u * kThreads, v[u]);
            }
            move_tail(first, blk, pl.record);
        } else {
            ItemPos at[V];
            uint32_t blk[V];
            Place pl[V];
#pragma unroll
            for (int u = 0; u < V; ++u) {   // the id look-ups first, together
                at[u] = item_pos(item + (uint32_t(u) < count ? u : 0), c.tiles, c.planes);
                blk[u] = uint32_t(ids[at[u].k]);
            }
            bool all_full = count == V;
#pragma unroll
            for (int u = 0; u < V; ++u) {
                pl[u] = place(at[u], uint64_t(blk[u]));
                if (uint32_t(u) >= count) pl[u].left = 0;
                all_full = all_full && pl[u].left >= kThreads;
            }
            if (all_full) {   // V full tiles of several pages: no predicates, so the stores need not wait for one another
#pragma unroll
                for (int u = 0; u < V; ++u) v[u] = ld16<NTL>(pl[u].src + lane);
#pragma unroll
                for (int u = 0; u < V; ++u) st16<NTS>(pl[u].dst + lane, v[u]);
            } else {
#pragma unroll
                for (int u = 0; u < V; ++u)
                    if (lane < pl[u].left) v[u] = ld16<NTL>(pl[u].src + lane);
#pragma unroll
                for (int u = 0; u < V; ++u)
                    if (lane < pl[u].left) st16<NTS>(pl[u].dst + lane, v[u]);
            }
#pragma unroll
            for (int u = 0; u < V; ++u)
                if (uint32_t(u) < count) move_tail(at[u], uint64_t(blk[u]), pl[u].record);
        }
    };
    using One = std::integral_constant<int, 1>;
    using Eight = std::integral_constant<int, 8>;

    const WgWalk ww = workgroup_walk(c, blockIdx.x);
    if constexpr (TAIL || DIRECT) {
        if (ww.width == 8) {
            for (uint32_t item = ww.w.first; item < ww.w.end; item += ww.w.step) move(item, min(8u, ww.w.end - item), Eight{});
            return;
        }
    }
    for (uint32_t item = ww.w.first; item < ww.w.end; item += ww.w.step) move(item, 1, One{});
}

__global__ __launch_bounds__(kThreads) void rewrite_table_kernel(int32_t *__restrict__ table,
                                                                  const int32_t *__restrict__ ids, uint32_t n)
{
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i < n) table[i] = ids[i];
}

// dst[i] = src[i] with the staged launches' mapping: 4 KiB tiles, XCD b mod 8 streams the (b mod 8)-th eighth.
template <bool NT>
__global__ __launch_bounds__(kThreads) void copy_contiguous_kernel(u32x4 *__restrict__ dst,
                                                                    const u32x4 *__restrict__ src, uint64_t n16,
                                                                    uint32_t n_tiles)
{
    const uint32_t r = blockIdx.x % kXcds;
    const uint32_t per = (n_tiles + kXcds - 1) / kXcds;
    const uint32_t tile = r * per + blockIdx.x / kXcds;
    if (blockIdx.x / kXcds >= per || tile >= n_tiles) return;
    const uint64_t at = uint64_t(tile) * kThreads + threadIdx.x;
    if (at < n16) st16<NT>(dst + at, ld16<NT>(src + at));
}

// One-way streams with the same tiles and mapping: what HBM sustains in each direction alone.
template <bool WRITE>
__global__ __launch_bounds__(kThreads) void hbm_one_way_kernel(u32x4 *__restrict__ p, uint32_t n_tiles)
{
    const uint32_t r = blockIdx.x % kXcds;
    const uint32_t per = (n_tiles + kXcds - 1) / kXcds;
    const uint32_t tile = r * per + blockIdx.x / kXcds;
    if (tile >= n_tiles) return;
    u32x4 *at = p + uint64_t(tile) * kThreads + threadIdx.x;
    if constexpr (WRITE) {
        const u32x4 v = {tile, 0x9E3779B9u, threadIdx.x, ~tile};
        st16<true>(at, v);
    } else {
        const u32x4 v = ld16<true>(at);
        asm volatile("" ::"v"(v.x), "v"(v.y), "v"(v.z), "v"(v.w));   // the value is used: the load stays
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
    // Cache policy, measured on MI355X with cold 512 MiB launches in the offload -> upload sequence:
    // non-temporal loads help both directions.  The gather's staging writes stay ordinary
    // write-back stores: they are absorbed by the memory-side cache and drain to HBM while the
    // slow host-link DMA that follows reads them.  The scatter's page writes are non-temporal, so
    // it leaves no dirty lines for the next kernel to evict (with ordinary stores the scatter looks
    // faster and the following gather pays for it; the sum is worse).
    CopyPlan c;
    if (!make_copy_plan(n, g, max_grid, direct, host_part != nullptr, split, host_wgs, &c)) return hipErrorInvalidValue;
    if (c.grid == 0) return hipSuccess;
    const uint32_t grid = c.grid;
    host_wgs = c.host_wgs;

#define TC_LAUNCH(NL, NS, DR, TL)                                                                             \
    hipLaunchKernelGGL((page_copy_kernel<NL, NS, GATHER, DR, TL>), dim3(grid), dim3(kThreads), 0, stream,     \
                       static_cast<u32x4 *>(pool), scales, static_cast<u32x4 *>(staging), ids_dev,           \
                       static_cast<u32x4 *>(host_part), c)
    const bool tail = host_wgs != 0;
    if (direct) TC_LAUNCH(true, true, true, false);
    else if (GATHER && tail) TC_LAUNCH(true, false, false, true);
    else if (GATHER) TC_LAUNCH(true, false, false, false);
    else if (tail) TC_LAUNCH(true, true, false, true);
    else TC_LAUNCH(true, true, false, false);
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
    const uint64_t n_tiles = (n16 + kThreads - 1) / kThreads;
    const uint64_t grid = (n_tiles + kXcds - 1) / kXcds * kXcds;
    if (grid > 0x7fffffffull) return hipErrorInvalidValue;
    hipLaunchKernelGGL((copy_contiguous_kernel<true>), dim3(uint32_t(grid)), dim3(kThreads), 0, stream,
                       static_cast<u32x4 *>(dst), static_cast<const u32x4 *>(src), n16, uint32_t(n_tiles));
    return hipGetLastError();
}

hipError_t launch_hbm_one_way(void *p, uint64_t bytes, bool write, hipStream_t stream)
{
    if (bytes == 0) return hipSuccess;
    const uint64_t n_tiles = bytes / (kThreads * 16);
    const uint64_t grid = (n_tiles + kXcds - 1) / kXcds * kXcds;
    if (bytes % (kThreads * 16) || grid > 0x7fffffffull) return hipErrorInvalidValue;
    if (write)
        hipLaunchKernelGGL((hbm_one_way_kernel<true>), dim3(uint32_t(grid)), dim3(kThreads), 0, stream,
                           static_cast<u32x4 *>(p), uint32_t(n_tiles));
    else
        hipLaunchKernelGGL((hbm_one_way_kernel<false>), dim3(uint32_t(grid)), dim3(kThreads), 0, stream,
                           static_cast<u32x4 *>(p), uint32_t(n_tiles));
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
