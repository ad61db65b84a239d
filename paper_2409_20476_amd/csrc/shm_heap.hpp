// Host-side symmetric-heap allocator.  One instance serves every PE: an offset it hands out
// names the same block in every PE's partition (paper section "OpenSHMEM Memory and Execution
// Model": identical layout of the symmetric segments; section "Proposed Device APIs": memory
// management is host-only).  Lowest-address first fit over a map of free extents, with
// coalescing on release.  No HIP calls; usable without a device.
#pragma once

#include <cstddef>
#include <cstdint>
#include <iterator>
#include <map>

class shm_heap_allocator {
public:
    static constexpr uint64_t GRANULE = 16;          // block sizes are rounded up to the vector width
    static constexpr uint64_t NPOS = UINT64_MAX;

    void reset(uint64_t bytes)
    {
        free_.clear();
        live_.clear();
        if (bytes) free_[0] = bytes;
    }

    // Returns the offset, or NPOS when no free extent can hold `bytes` at `align` (a power of two).
    uint64_t allocate(uint64_t bytes, uint64_t align)
    {
        const uint64_t need = (bytes + GRANULE - 1) / GRANULE * GRANULE;
        if (need < bytes) return NPOS;               // overflow
        for (auto it = free_.begin(); it != free_.end(); ++it) {
            const uint64_t beg = it->first, end = beg + it->second;
            const uint64_t start = (beg + align - 1) & ~(align - 1);
            if (start < beg || start > end || end - start < need) continue;
            free_.erase(it);
            if (start > beg) free_[beg] = start - beg;
            if (start + need < end) free_[start + need] = end - (start + need);
            live_[start] = need;
            return start;
        }
        return NPOS;
    }

    // Size of the live block at `off`, or 0 if there is none.
    uint64_t live_size(uint64_t off) const
    {
        auto it = live_.find(off);
        return it == live_.end() ? 0 : it->second;
    }

    bool release(uint64_t off)
    {
        auto it = live_.find(off);
        if (it == live_.end()) return false;
        uint64_t beg = off, len = it->second;
        live_.erase(it);
        auto next = free_.lower_bound(beg);
        if (next != free_.end() && next->first == beg + len) {
            len += next->second;
            next = free_.erase(next);
        }
        if (next != free_.begin()) {
            auto prev = std::prev(next);
            if (prev->first + prev->second == beg) {
                beg = prev->first;
                len += prev->second;
                free_.erase(prev);
            }
        }
        free_[beg] = len;
        return true;
    }

    size_t live_blocks() const { return live_.size(); }
    size_t free_extents() const { return free_.size(); }

private:
    std::map<uint64_t, uint64_t> free_;   // offset -> length of each free extent
    std::map<uint64_t, uint64_t> live_;   // offset -> length of each live block
};
