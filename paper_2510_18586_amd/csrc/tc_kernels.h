// Launchers of the gfx950 kernels behind tc_offload / tc_upload.  Internal to the library.
#pragma once

#include <cstdint>
#include <hip/hip_runtime_api.h>

#include "tc_map.h"

namespace tc {

// staging[k] <- record of block ids[k] for k < n (pages, scale words, zero pad).  `staging` is a
// device staging chunk, or (direct = true) the GPU's view of pinned host memory.
// A launch may be split: records of blocks [0, split) go to `staging`, those of [split, n) to
// `host_part` (the GPU's view of pinned host memory, record split first), handled by the first
// `host_wgs` workgroups so that the host link works while the rest of the grid streams through HBM.
// split = n (the default) means no host part.
hipError_t launch_gather_pages(const void *pool, const uint32_t *scales, void *staging, const int32_t *ids_dev,
                               uint32_t n, const PageGeom &g, uint32_t max_grid, bool direct, hipStream_t stream,
                               void *host_part, uint32_t split, uint32_t host_wgs);
// block ids[k] <- record k of staging (same meaning of `direct` and of the split).
hipError_t launch_scatter_pages(const void *staging, void *pool, uint32_t *scales, const int32_t *ids_dev,
                                uint32_t n, const PageGeom &g, uint32_t max_grid, bool direct, hipStream_t stream,
                                const void *host_part, uint32_t split, uint32_t host_wgs);
// table[i] = ids[i], i < n.
hipError_t launch_rewrite_table(int32_t *table, const int32_t *ids_dev, uint32_t n, hipStream_t stream);

hipError_t launch_copy_contiguous(void *dst, const void *src, uint64_t bytes, hipStream_t stream);
// One-way stream over `bytes` (a multiple of 4 KiB): non-temporal stores of a pattern, or loads alone.
hipError_t launch_hbm_one_way(void *p, uint64_t bytes, bool write, hipStream_t stream);
// The same copy staged through LDS (bytes must be a multiple of 16 KiB); measurement only.
hipError_t launch_copy_via_lds(void *dst, const void *src, uint64_t bytes, bool lds_direct_loads, hipStream_t stream);
hipError_t launch_hbm_stream(float *a, const float *b, const float *c, uint64_t n, float s, uint32_t iters,
                             hipStream_t stream);

}  // namespace tc
