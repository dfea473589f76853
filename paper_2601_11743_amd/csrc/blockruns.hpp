// Free block runs of the shim's address space: first fit, neighbours merged on release.
// (Paper, "Granularity of Memory Management": memory is handed out in whole fixed-size blocks.)
// Header only and free of HIP, so it is tested on the CPU.
#pragma once
#include <cstdint>
#include <iterator>
#include <map>

namespace nixie {

class BlockRuns {
public:
    explicit BlockRuns(uint64_t blocks = 0) { if (blocks) free_[0] = blocks; }
    static constexpr uint64_t kNone = ~0ull;

    // first block of the lowest run of at least n free blocks, or kNone; nothing changes
    uint64_t find(uint64_t n) const {
        if (n == 0) return kNone;
        for (const auto &r : free_)
            if (r.second >= n) return r.first;
        return kNone;
    }
    // takes [first, first + n) out of the free run that starts at first (as returned by find)
    void take(uint64_t first, uint64_t n) {
        auto it = free_.find(first);
        const uint64_t rest = it->second - n;
        free_.erase(it);
        if (rest) free_[first + n] = rest;
    }
    // gives [first, first + n) back and merges it with free neighbours
    void give(uint64_t first, uint64_t n) {
        auto next = free_.lower_bound(first);
        if (next != free_.end() && next->first == first + n) { n += next->second; next = free_.erase(next); }
        if (next != free_.begin()) {
            auto prev = std::prev(next);
            if (prev->first + prev->second == first) { first = prev->first; n += prev->second; free_.erase(prev); }
        }
        free_[first] = n;
    }
    uint64_t free_blocks() const {
        uint64_t t = 0;
        for (const auto &r : free_) t += r.second;
        return t;
    }
    size_t runs() const { return free_.size(); }

private:
    std::map<uint64_t, uint64_t> free_;   // first block -> number of blocks
};

}  // namespace nixie
