// Work-item arithmetic of the page copy kernels: which (block, plane, tile) an item is and which items a
// workgroup takes.  Plain inline code shared by the kernels and the host (launchers, limits, and the
// CPU tests that walk every mapping), so the index arithmetic that decides what a kernel touches can be
// checked without a GPU.
#pragma once

#include <cstdint>

#if defined(__HIPCC__)
#define TC_HD __host__ __device__ __forceinline__
#else
#define TC_HD inline
#endif

namespace tc {

// Geometry shared by gather and scatter; all "16" fields count 16-byte units.
struct PageGeom {
    uint32_t planes;       // P = 2 * layers
    uint32_t page16;       // page_bytes / 16
    uint64_t num_blocks;   // NB
    uint64_t rec16;        // host-record bytes / 16
    uint32_t scales;       // S: scale words per block (0, 1 or P)
    uint32_t tail_words;   // 32-bit words from the end of the pages to the end of the record
};

// A copy tile is 256 lanes x 16 B = 4 KiB; a page is cut into ceil(page16 / 256) tiles, the last one
// possibly ragged.  The launchers and the limit on a pool description both go by this function.
constexpr uint32_t kCopyThreads = 256;
TC_HD uint32_t tiles_per_page(uint32_t page16) { return (page16 + kCopyThreads - 1) / kCopyThreads; }

// Workgroups are dealt round-robin over the 8 XCDs of the chip (workgroup b runs on XCD b mod 8), each
// with its own L2.  The staged launches give every XCD one contiguous eighth of the work items.
constexpr uint32_t kXcds = 8;

// floor(n / d) for n < 2^31 as one widening multiply and a shift (Granlund & Montgomery, "Division by
// invariant integers using multiplication", 1994): with l = ceil(log2 d) and mul = ceil(2^(31+l) / d),
// floor(n * mul / 2^(31+l)) = floor(n / d) for every n < 2^31, and mul < 2^32.
struct FastDiv {
    uint32_t d, mul, shift;
};
inline FastDiv make_fastdiv(uint32_t d)
{
    uint32_t l = 0;
    while ((uint64_t(1) << l) < d) ++l;
    const uint64_t mul = ((uint64_t(1) << (31 + l)) + d - 1) / d;   // d <= 2^31, so l <= 31: no overflow
    return FastDiv{d, uint32_t(mul), 31 + l};
}
TC_HD uint32_t fastdiv(uint32_t n, const FastDiv &f) { return uint32_t((uint64_t(n) * f.mul) >> f.shift); }

// One work item = (block k of the chunk, plane p, tile t of the page), ordered with the tile fastest,
// then the plane: consecutive items are consecutive addresses on the record side.
struct ItemPos {
    uint32_t k, p, t;
};
TC_HD ItemPos item_pos(uint32_t item, const FastDiv &tiles, const FastDiv &planes)
{
    const uint32_t kp = fastdiv(item, tiles);
    const uint32_t k = fastdiv(kp, planes);
    return ItemPos{k, kp - k * planes.d, item - kp * tiles.d};
}

// Where an item's tile lies, in 16-byte units: from the pool's base, and from the base of the record side
// (the staging chunk, or the host part when the launch carries a host tail and the block belongs to it).
struct ItemPlace {
    uint64_t pool16;     // offset of the tile in the pool
    uint64_t record16;   // offset of the block's record in its buffer
    uint64_t tile16;     // offset of the tile inside the record
    uint32_t left;       // 16-byte units from the tile start to the page end (the tile covers min(left, 256))
    bool in_host_part;   // the record lives in the host part, counted from block `split`
};
TC_HD ItemPlace item_place(const ItemPos &at, uint64_t blk, const PageGeom &g, uint32_t split)
{
    const bool host = at.k >= split;
    return ItemPlace{(uint64_t(at.p) * g.num_blocks + blk) * g.page16 + uint64_t(at.t) * kCopyThreads,
                     uint64_t(host ? at.k - split : at.k) * g.rec16,
                     uint64_t(at.p) * g.page16 + uint64_t(at.t) * kCopyThreads, g.page16 - at.t * kCopyThreads, host};
}

// The items a workgroup takes: first, first + step, ... below end; `width` consecutive items at each stop.
struct ItemWalk {
    uint32_t first, end, step;
};

// Staged launches.  Items [0, n_items) are cut into `chunks` contiguous runs of per = ceil(n_items / chunks);
// workgroup b of `grid` walks run r = b mod chunks, in turn with the other workgroups of that run
// (b = r, r + chunks, ...), one item at a stop.  Needs 1 <= chunks <= grid.
TC_HD ItemWalk staged_walk(uint32_t b, uint32_t grid, uint32_t n_items, uint32_t chunks)
{
    const uint32_t r = b % chunks;
    const uint32_t per = (n_items + chunks - 1) / chunks;
    const uint32_t wgs_of_run = (grid - r + chunks - 1) / chunks;
    const uint64_t run_end = uint64_t(r + 1) * per;
    return ItemWalk{r * per + b / chunks, run_end < n_items ? uint32_t(run_end) : n_items, wgs_of_run};
}

// Launches that are bound by the host link: a few workgroups, `width` consecutive items per stop,
// grid-stride over items [first_item, end_item).
TC_HD ItemWalk strided_walk(uint32_t b, uint32_t grid, uint32_t first_item, uint32_t end_item, uint32_t width)
{
    const uint64_t first = uint64_t(first_item) + uint64_t(b) * width;
    return ItemWalk{first < end_item ? uint32_t(first) : end_item, end_item, grid * width};
}

// Everything a page-copy launch is told besides its pointers, and its grid: decided in one place for the
// launcher and for the CPU tests that walk a launch.
struct CopyPlan {
    PageGeom g;
    FastDiv tiles;       // tiles per page
    FastDiv planes;      // planes per block
    uint32_t n_items;    // blocks * planes * tiles
    uint32_t split;      // records of blocks [0, split) live in staging, the rest in the host part (n = none)
    uint32_t host_wgs;   // the first host_wgs workgroups take the host-side items, 8 per stop
    uint32_t chunks;     // the staged items are cut into this many contiguous runs, one per XCD (1 = no cut)
    uint32_t grid;       // workgroups, host_wgs included; 0 = nothing to launch
    bool direct;         // the record side is pinned host memory: few workgroups, 8 items per stop, no cut
};
// false: the request does not fit a launch (more than 2^31 - 1 items, or a split that makes no sense).
inline bool make_copy_plan(uint32_t n, const PageGeom &g, uint32_t max_grid, bool direct, bool has_host_part,
                           uint32_t split, uint32_t host_wgs, CopyPlan *out)
{
    const uint32_t tiles = tiles_per_page(g.page16);
    const uint64_t items64 = uint64_t(n) * g.planes * tiles;
    if (items64 > 0x7fffffffull) return false;
    if (split > n || (split < n && (!has_host_part || host_wgs == 0 || direct))) return false;
    if (split == n) host_wgs = 0;
    CopyPlan c{};
    c.g = g;
    c.tiles = make_fastdiv(tiles);
    c.planes = make_fastdiv(g.planes);
    c.n_items = uint32_t(items64);
    c.split = split;
    c.direct = direct;
    const uint32_t items_staged = split * g.planes * tiles;
    // the host part and a direct launch move 8 tiles per workgroup and stop: more workgroups than stops are no use
    // (and the walk's step, workgroups * 8, stays far below 2^32)
    if (host_wgs) host_wgs = host_wgs < (c.n_items - items_staged + 7) / 8 ? host_wgs : (c.n_items - items_staged + 7) / 8;
    c.host_wgs = host_wgs;
    uint32_t grid = direct ? (items_staged + 7) / 8 : items_staged;
    if (max_grid && grid > max_grid) grid = max_grid;
    // every run needs a workgroup of its own; a grid below 8 walks the items as one run
    c.chunks = (!direct && grid >= kXcds) ? kXcds : 1;
    c.grid = grid + host_wgs;
    *out = c;
    return true;
}

// The walk of workgroup b of a launch: the first host_wgs workgroups take the host part, 8 items a stop;
// the workgroups of a direct launch take everything 8 items a stop; all others walk their XCD's run.
struct WgWalk {
    ItemWalk w;
    uint32_t width;   // items per stop: 1 or 8
};
TC_HD WgWalk workgroup_walk(const CopyPlan &c, uint32_t b)
{
    const uint32_t staged_end = c.split * c.planes.d * c.tiles.d < c.n_items ? c.split * c.planes.d * c.tiles.d : c.n_items;
    if (b < c.host_wgs) return WgWalk{strided_walk(b, c.host_wgs, staged_end, c.n_items, 8), 8};
    b -= c.host_wgs;
    const uint32_t grid = c.grid - c.host_wgs;
    if (c.direct) return WgWalk{strided_walk(b, grid, 0, staged_end, 8), 8};
    return WgWalk{staged_walk(b, grid, staged_end, c.chunks), 1};
}

}  // namespace tc
