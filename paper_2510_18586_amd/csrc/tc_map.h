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

}  // namespace tc
