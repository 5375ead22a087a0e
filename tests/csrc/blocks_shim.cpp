// Test-only C shim over the library's host bookkeeping classes (tc_blocks.h), so that the
// free list, reference counts, pending-free rule and host arena can be exercised without a GPU.
#include "tc_blocks.h"

extern "C" {
void *tcb_pool_new(uint32_t nb) { return new tc::BlockPool(nb); }
void tcb_pool_del(void *p) { delete static_cast<tc::BlockPool *>(p); }
int tcb_alloc(void *p, uint32_t n, int32_t *out) { return static_cast<tc::BlockPool *>(p)->alloc(n, out); }
int tcb_alloc_at(void *p, const int32_t *ids, uint32_t n) { return static_cast<tc::BlockPool *>(p)->alloc_at(ids, n); }
int tcb_alloc_prefer(void *p, const int32_t *pref, uint32_t n, int32_t *out) { return static_cast<tc::BlockPool *>(p)->alloc_prefer(pref, n, out); }
int tcb_ref(void *p, const int32_t *ids, uint32_t n) { return static_cast<tc::BlockPool *>(p)->ref(ids, n); }
int tcb_free(void *p, const int32_t *ids, uint32_t n) { return static_cast<tc::BlockPool *>(p)->free(ids, n); }
int tcb_check_transfer(void *p, const int32_t *ids, uint32_t n) { return static_cast<tc::BlockPool *>(p)->check_transfer(ids, n); }
void tcb_begin(void *p, const int32_t *ids, uint32_t n) { static_cast<tc::BlockPool *>(p)->begin_transfer(ids, n); }
void tcb_end(void *p, const int32_t *ids, uint32_t n) { static_cast<tc::BlockPool *>(p)->end_transfer(ids, n); }
int tcb_filter_private(void *p, const int32_t *ids, uint32_t n, int32_t *out, uint32_t *m)
{
    return static_cast<tc::BlockPool *>(p)->filter_private(ids, n, out, m);
}
void tcb_counts(void *p, uint32_t *out4)
{
    auto *b = static_cast<tc::BlockPool *>(p);
    out4[0] = b->n_free(); out4[1] = b->n_used(); out4[2] = b->n_pending(); out4[3] = b->n_shared();
}

void *tcb_arena_new(uint64_t slots) { return new tc::HostArena(slots); }
void tcb_arena_del(void *a) { delete static_cast<tc::HostArena *>(a); }
int64_t tcb_arena_alloc(void *a, uint64_t n) { return static_cast<tc::HostArena *>(a)->alloc(n); }
int tcb_arena_free(void *a, uint64_t start) { return static_cast<tc::HostArena *>(a)->free(start); }
uint64_t tcb_arena_used(void *a) { return static_cast<tc::HostArena *>(a)->used(); }
int tcb_arena_locate(void *a, uint64_t slot, uint64_t *start, uint64_t *room)
{
    return static_cast<tc::HostArena *>(a)->locate(slot, start, room) ? 1 : 0;
}
void tcb_arena_begin(void *a, uint64_t start) { static_cast<tc::HostArena *>(a)->begin_transfer(start); }
void tcb_arena_end(void *a, uint64_t start) { static_cast<tc::HostArena *>(a)->end_transfer(start); }
}
