// Pool description -> record size and kernel geometry, and the one place where the limits on a pool
// description are checked (paper Sec. 7.6: a block is block_size tokens of every layer's K and V;
// the host keeps one record per block).  Host only; shared by tc_create and the entry point that
// works without a context.
#pragma once

#include <cstdint>

#include "tc_map.h"
#include "tokencake_kv.h"

namespace tc {

// Host bytes per block: P pages, S scale words, rounded up to 256 B.
inline uint64_t record_bytes_of(uint32_t planes, uint32_t page_bytes, uint32_t scales)
{
    const uint64_t raw = uint64_t(planes) * page_bytes + 4ull * scales;
    return (raw + 255) / 256 * 256;
}

// Everything about a pool description that can be judged without a device call.
inline int check_pool_desc(const tc_pool_desc *pool)
{
    if (!pool) return TC_ERR_INVAL;
    if (!pool->kv_base || pool->num_layers == 0 || pool->num_blocks == 0 || pool->page_bytes == 0) return TC_ERR_INVAL;
    if (pool->page_bytes % 16 || (reinterpret_cast<uintptr_t>(pool->kv_base) % 256)) return TC_ERR_INVAL;
    if (pool->num_blocks > 0x7fffffffu || pool->num_layers > (1u << 20)) return TC_ERR_INVAL;
    const uint32_t P = 2 * pool->num_layers;
    const uint32_t S = pool->scales_per_block;
    if (S != 0 && S != 1 && S != P) return TC_ERR_INVAL;
    if ((S != 0) != (pool->scales != nullptr)) return TC_ERR_INVAL;
    if (S && (reinterpret_cast<uintptr_t>(pool->scales) % 4)) return TC_ERR_INVAL;
    // one launch may cover every block of the pool: its work items (block x plane x tile) are counted in 31 bits
    if (uint64_t(pool->num_blocks) * P * tiles_per_page(pool->page_bytes / 16) > 0x7fffffffull) return TC_ERR_INVAL;
    return TC_OK;
}

inline PageGeom make_geom(const tc_pool_desc &pool)
{
    const uint32_t P = 2 * pool.num_layers;
    const uint64_t rec = record_bytes_of(P, pool.page_bytes, pool.scales_per_block);
    PageGeom g{};
    g.planes = P;
    g.page16 = pool.page_bytes / 16;
    g.num_blocks = pool.num_blocks;
    g.rec16 = rec / 16;
    g.scales = pool.scales_per_block;
    g.tail_words = uint32_t((rec - uint64_t(P) * pool.page_bytes) / 4);
    return g;
}

}  // namespace tc
