// Host-side block bookkeeping for the KV migration path (paper Sec. 6.3):
//   * GPU blocks: LIFO free list, reference counts, and the pending-free rule — a block
//     released while a transfer touching it is in flight re-enters the free list only when
//     that transfer retires;
//   * CPU blocks: fixed-size slots of one pinned arena, handed out as first-fit runs of
//     consecutive slots and recycled, never returned to the operating system.
// Pure C++17, no HIP: the transfer engine owns one of each and drives them under its mutex.
#pragma once

#include <algorithm>
#include <cstdint>
#include <iterator>
#include <map>
#include <vector>

#include "tokencake_kv.h"

namespace tc {

class BlockPool {
public:
    explicit BlockPool(uint32_t num_blocks)
        : nb_(num_blocks), next_(num_blocks), prev_(num_blocks), ref_(num_blocks, 0),
          inflight_(num_blocks, 0), stamp_(num_blocks, 0), state_(num_blocks, kFree)
    {
        // free list in ascending order from the head: the first hand-out is 0, 1, 2, ...
        for (uint32_t b = 0; b < nb_; ++b) {
            next_[b] = (b + 1 < nb_) ? int32_t(b + 1) : -1;
            prev_[b] = int32_t(b) - 1;
        }
        head_ = nb_ ? 0 : -1;
        n_free_ = nb_;
    }

    uint32_t total() const { return nb_; }
    uint32_t n_free() const { return n_free_; }
    uint32_t n_used() const { return n_used_; }
    uint32_t n_pending() const { return n_pending_; }
    uint32_t n_shared() const { return n_shared_; }

    int alloc(uint32_t n, int32_t *out)
    {
        if (n > n_free_) return TC_ERR_NOMEM;
        for (uint32_t i = 0; i < n; ++i) {
            int32_t b = head_;
            unlink(b);
            take(b);
            out[i] = b;
        }
        return TC_OK;
    }

    int alloc_at(const int32_t *ids, uint32_t n)
    {
        if (int rc = check_range(ids, n)) return rc;
        if (int rc = check_distinct(ids, n)) return rc;
        for (uint32_t i = 0; i < n; ++i)
            if (state_[ids[i]] != kFree) return TC_ERR_NOMEM;
        for (uint32_t i = 0; i < n; ++i) {
            unlink(ids[i]);
            take(ids[i]);
        }
        return TC_OK;
    }

    // n blocks, all or nothing: preferred[i] itself where it is still on the free list (the original
    // GPU block is taken again where it still can be, Sec. 6.3), a fresh block otherwise.  All claims happen
    // before the first fresh block is popped, so a pop can never take a block a later entry asks for.
    int alloc_prefer(const int32_t *preferred, uint32_t n, int32_t *out)
    {
        if (n > n_free_) return TC_ERR_NOMEM;
        for (uint32_t i = 0; i < n; ++i) {
            int32_t b = preferred[i];
            if (b >= 0 && uint32_t(b) < nb_ && state_[b] == kFree) {
                unlink(b);
                take(b);
                out[i] = b;
            } else {
                out[i] = -1;
            }
        }
        for (uint32_t i = 0; i < n; ++i) {
            if (out[i] >= 0) continue;
            int32_t b = head_;
            unlink(b);
            take(b);
            out[i] = b;
        }
        return TC_OK;
    }

    int ref(const int32_t *ids, uint32_t n)
    {
        if (int rc = check_range(ids, n)) return rc;
        for (uint32_t i = 0; i < n; ++i)
            if (ref_[ids[i]] == 0) return TC_ERR_INVAL;
        for (uint32_t i = 0; i < n; ++i)
            if (++ref_[ids[i]] == 2) ++n_shared_;
        return TC_OK;
    }

    int free(const int32_t *ids, uint32_t n)
    {
        if (int rc = check_range(ids, n)) return rc;
        // an id may appear several times as long as it holds that many references
        bump_epoch();
        for (uint32_t i = 0; i < n; ++i) {
            uint32_t b = uint32_t(ids[i]);
            if (stamp_[b] != epoch_) { stamp_[b] = epoch_; count_[b] = 0; }
            if (++count_[b] > ref_[b]) return TC_ERR_INVAL;
        }
        for (uint32_t i = 0; i < n; ++i) {
            uint32_t b = uint32_t(ids[i]);
            uint32_t r = --ref_[b];
            if (r == 1) --n_shared_;
            if (r == 0) {
                --n_used_;
                if (inflight_[b]) {
                    state_[b] = kPending;
                    ++n_pending_;
                } else {
                    push_free(int32_t(b));
                }
            }
        }
        return TC_OK;
    }

    // A block may move only if it is allocated and has exactly one owner.
    int check_transfer(const int32_t *ids, uint32_t n)
    {
        if (int rc = check_range(ids, n)) return rc;
        if (int rc = check_distinct(ids, n)) return rc;
        for (uint32_t i = 0; i < n; ++i) {
            uint32_t r = ref_[ids[i]];
            if (r == 0) return TC_ERR_INVAL;
            if (r > 1) return TC_ERR_SHARED;
        }
        return TC_OK;
    }

    void begin_transfer(const int32_t *ids, uint32_t n)
    {
        for (uint32_t i = 0; i < n; ++i) ++inflight_[ids[i]];
    }

    void end_transfer(const int32_t *ids, uint32_t n)
    {
        for (uint32_t i = 0; i < n; ++i) {
            uint32_t b = uint32_t(ids[i]);
            if (--inflight_[b] == 0 && state_[b] == kPending) {
                --n_pending_;
                push_free(int32_t(b));
            }
        }
    }

    int filter_private(const int32_t *ids, uint32_t n, int32_t *out, uint32_t *m)
    {
        if (int rc = check_range(ids, n)) return rc;
        uint32_t k = 0;
        for (uint32_t i = 0; i < n; ++i)
            if (ref_[ids[i]] == 1) out[k++] = ids[i];
        *m = k;
        return TC_OK;
    }

    int check_range(const int32_t *ids, uint32_t n) const
    {
        for (uint32_t i = 0; i < n; ++i)
            if (ids[i] < 0 || uint32_t(ids[i]) >= nb_) return TC_ERR_RANGE;
        return TC_OK;
    }

    int check_distinct(const int32_t *ids, uint32_t n)
    {
        bump_epoch();
        for (uint32_t i = 0; i < n; ++i) {
            if (stamp_[ids[i]] == epoch_) return TC_ERR_DUP;
            stamp_[ids[i]] = epoch_;
        }
        return TC_OK;
    }

private:
    enum : uint8_t { kFree = 0, kUsed = 1, kPending = 2 };

    void bump_epoch()
    {
        if (count_.empty()) count_.assign(nb_, 0);
        if (++epoch_ == 0) {  // wrapped: old stamps could alias
            std::fill(stamp_.begin(), stamp_.end(), 0u);
            epoch_ = 1;
        }
    }
    void unlink(int32_t b)
    {
        int32_t p = prev_[b], q = next_[b];
        if (p >= 0) next_[p] = q; else head_ = q;
        if (q >= 0) prev_[q] = p;
        --n_free_;
    }
    void take(int32_t b)
    {
        state_[b] = kUsed;
        ref_[b] = 1;
        ++n_used_;
    }
    void push_free(int32_t b)
    {
        state_[b] = kFree;
        prev_[b] = -1;
        next_[b] = head_;
        if (head_ >= 0) prev_[head_] = b;
        head_ = b;
        ++n_free_;
    }

    uint32_t nb_;
    std::vector<int32_t> next_, prev_;
    std::vector<uint32_t> ref_, inflight_, stamp_, count_;
    std::vector<uint8_t> state_;
    int32_t head_ = -1;
    uint32_t epoch_ = 0;
    uint32_t n_free_ = 0, n_used_ = 0, n_pending_ = 0, n_shared_ = 0;
};

// Slots are record-sized; an allocation is identified by its first slot.
class HostArena {
public:
    explicit HostArena(uint64_t n_slots) : n_slots_(n_slots)
    {
        if (n_slots_) free_runs_[0] = n_slots_;
    }

    uint64_t total() const { return n_slots_; }
    uint64_t used() const { return used_; }

    // first fit from the lowest address; returns the first slot or -1
    int64_t alloc(uint64_t n)
    {
        for (auto it = free_runs_.begin(); it != free_runs_.end(); ++it) {
            if (it->second < n) continue;
            uint64_t start = it->first, len = it->second;
            free_runs_.erase(it);
            if (len > n) free_runs_[start + n] = len - n;
            live_[start] = Live{n, 0, false};
            used_ += n;
            return int64_t(start);
        }
        return -1;
    }

    // TC_OK, or TC_ERR_INVAL when `start` is not the first slot of a live, unreleased allocation
    int free(uint64_t start)
    {
        auto it = live_.find(start);
        if (it == live_.end() || it->second.released) return TC_ERR_INVAL;
        if (it->second.inflight) it->second.released = true;
        else release(it);
        return TC_OK;
    }

    // the live allocation that contains `slot`; returns its first slot and the slots left from `slot` on
    bool locate(uint64_t slot, uint64_t *start, uint64_t *room) const
    {
        auto it = live_.upper_bound(slot);
        if (it == live_.begin()) return false;
        --it;
        if (slot >= it->first + it->second.len) return false;
        *start = it->first;
        *room = it->first + it->second.len - slot;
        return true;
    }

    void begin_transfer(uint64_t start) { ++live_.at(start).inflight; }

    void end_transfer(uint64_t start)
    {
        auto it = live_.find(start);
        if (--it->second.inflight == 0 && it->second.released) release(it);
    }

private:
    struct Live { uint64_t len; uint32_t inflight; bool released; };

    void release(std::map<uint64_t, Live>::iterator it)
    {
        uint64_t start = it->first, len = it->second.len;
        live_.erase(it);
        used_ -= len;
        auto nx = free_runs_.lower_bound(start);
        if (nx != free_runs_.end() && start + len == nx->first) {
            len += nx->second;
            nx = free_runs_.erase(nx);
        }
        if (nx != free_runs_.begin()) {
            auto pv = std::prev(nx);
            if (pv->first + pv->second == start) {
                pv->second += len;
                return;
            }
        }
        free_runs_[start] = len;
    }

    uint64_t n_slots_;
    uint64_t used_ = 0;
    std::map<uint64_t, uint64_t> free_runs_;
    std::map<uint64_t, Live> live_;
};

}  // namespace tc
