// Residency map and CPU prefix-cache index (paper Sec. 6.3, "CPU Migration Infrastructure"): which
// block key lives in which CPU record, which GPU block it came from or is going to, and whether an
// H2D transfer for it is still outstanding.  Host only; no HIP.
//
// The paper fixes neither the hash nor the index structure.  Keys are opaque 64-bit values here; a
// lookup answers for the longest leading run of keys that are present, because a block's key covers
// the whole prefix before it.  The convenience key function is a parent-chained 64-bit FNV-1a over
// whole blocks of token ids.
#include <cstring>
#include <mutex>
#include <new>
#include <unordered_map>
#include <unordered_set>
#include <vector>

#include "tokencake_kv.h"

namespace {

struct Entry {
    void *cpu_record;
    int32_t gpu_block;
    int32_t state;
};

bool distinct(const uint64_t *keys, uint32_t n)
{
    if (n < 2) return true;
    std::unordered_set<uint64_t> seen;
    seen.reserve(n * 2);
    for (uint32_t i = 0; i < n; ++i)
        if (!seen.insert(keys[i]).second) return false;
    return true;
}

}  // namespace

struct tc_index {
    mutable std::mutex mu;
    std::unordered_map<uint64_t, Entry> map;

    // every key present and in `state`
    bool all_in(const uint64_t *keys, uint32_t n, int state) const
    {
        for (uint32_t i = 0; i < n; ++i) {
            auto it = map.find(keys[i]);
            if (it == map.end() || it->second.state != state) return false;
        }
        return true;
    }
};

// No exception crosses the C boundary: running out of host memory inside a container is reported,
// anything else unexpected is an invalid call.
#define TC_CATCH_ALL                                              \
    catch (const std::bad_alloc &) { return TC_ERR_HOST_NOMEM; } \
    catch (...) { return TC_ERR_INVAL; }

extern "C" {

uint64_t tc_fnv1a64(const void *data, uint64_t len, uint64_t basis)
{
    const unsigned char *p = static_cast<const unsigned char *>(data);
    uint64_t h = basis;
    for (uint64_t i = 0; i < len; ++i) {
        h ^= p[i];
        h *= 0x100000001B3ull;
    }
    return h;
}

int tc_chain_hashes(const int32_t *tokens, uint64_t n_tokens, uint32_t block_size, uint64_t parent,
                    uint64_t *out, uint64_t *n_out)
try {
    if (!block_size || !n_out || (n_tokens && !tokens)) return TC_ERR_INVAL;
    uint64_t blocks = n_tokens / block_size;
    if (blocks && !out) return TC_ERR_INVAL;
    uint64_t h = parent;
    for (uint64_t b = 0; b < blocks; ++b) {
        unsigned char le[8];
        for (int k = 0; k < 8; ++k) le[k] = (unsigned char)(h >> (8 * k));
        uint64_t x = tc_fnv1a64(le, 8, TC_FNV_BASIS);
        // token ids are hashed as 32-bit little-endian words, which is their layout in memory here
        h = tc_fnv1a64(tokens + b * block_size, uint64_t(block_size) * 4, x);
        out[b] = h;
    }
    *n_out = blocks;
    return TC_OK;
} TC_CATCH_ALL

int tc_index_create(tc_index **out)
try {
    if (!out) return TC_ERR_INVAL;
    *out = new (std::nothrow) tc_index();
    return *out ? TC_OK : TC_ERR_HOST_NOMEM;
} TC_CATCH_ALL

int tc_index_destroy(tc_index *ix)
{
    delete ix;
    return TC_OK;
}

int tc_index_insert(tc_index *ix, const uint64_t *keys, const int32_t *gpu_blocks, void *host_buf,
                    uint64_t record_bytes, uint32_t n)
try {
    if (!ix || (n && (!keys || !gpu_blocks || !host_buf))) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ix->mu);
    if (!distinct(keys, n)) return TC_ERR_DUP;
    for (uint32_t i = 0; i < n; ++i)
        if (ix->map.count(keys[i])) return TC_ERR_DUP;
    ix->map.reserve(ix->map.size() + n);
    for (uint32_t i = 0; i < n; ++i)
        ix->map[keys[i]] = Entry{static_cast<char *>(host_buf) + uint64_t(i) * record_bytes, gpu_blocks[i], TC_RES_CPU};
    return TC_OK;
} TC_CATCH_ALL

int tc_index_lookup(const tc_index *ix, const uint64_t *keys, uint32_t n, tc_index_hit *out, uint32_t *hits)
try {
    if (!ix || !hits || (n && (!keys || !out))) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ix->mu);
    uint32_t k = 0;
    for (; k < n; ++k) {
        auto it = ix->map.find(keys[k]);
        if (it == ix->map.end()) break;
        out[k].key = keys[k];
        out[k].cpu_record = it->second.cpu_record;
        out[k].gpu_block = it->second.gpu_block;
        out[k].state = it->second.state;
    }
    *hits = k;
    return TC_OK;
} TC_CATCH_ALL

int tc_index_begin_upload(tc_index *ix, const uint64_t *keys, const int32_t *new_gpu_blocks, uint32_t n)
try {
    if (!ix || (n && (!keys || !new_gpu_blocks))) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ix->mu);
    if (!distinct(keys, n)) return TC_ERR_DUP;
    if (!ix->all_in(keys, n, TC_RES_CPU)) return TC_ERR_INVAL;
    for (uint32_t i = 0; i < n; ++i) {
        Entry &e = ix->map[keys[i]];
        e.state = TC_RES_H2D;
        e.gpu_block = new_gpu_blocks[i];
    }
    return TC_OK;
} TC_CATCH_ALL

int tc_index_finish_upload(tc_index *ix, const uint64_t *keys, uint32_t n)
try {
    if (!ix || (n && !keys)) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ix->mu);
    if (!distinct(keys, n)) return TC_ERR_DUP;
    if (!ix->all_in(keys, n, TC_RES_H2D)) return TC_ERR_INVAL;
    for (uint32_t i = 0; i < n; ++i) ix->map.erase(keys[i]);
    return TC_OK;
} TC_CATCH_ALL

int tc_index_remove(tc_index *ix, const uint64_t *keys, uint32_t n)
try {
    if (!ix || (n && !keys)) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(ix->mu);
    if (!distinct(keys, n)) return TC_ERR_DUP;
    if (!ix->all_in(keys, n, TC_RES_CPU)) return TC_ERR_INVAL;
    for (uint32_t i = 0; i < n; ++i) ix->map.erase(keys[i]);
    return TC_OK;
} TC_CATCH_ALL

uint32_t tc_index_pending(const tc_index *ix, const uint64_t *keys, uint32_t n)
{
    if (!ix || (n && !keys)) return 0;
    std::lock_guard<std::mutex> g(ix->mu);
    uint32_t c = 0;
    for (uint32_t i = 0; i < n; ++i) {
        auto it = ix->map.find(keys[i]);
        if (it != ix->map.end() && it->second.state == TC_RES_H2D) ++c;
    }
    return c;
}

uint64_t tc_index_size(const tc_index *ix)
{
    if (!ix) return 0;
    std::lock_guard<std::mutex> g(ix->mu);
    return ix->map.size();
}

}  // extern "C"
