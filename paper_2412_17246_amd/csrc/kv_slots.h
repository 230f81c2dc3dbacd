// Host-side bookkeeping of KV-cache slots: each slot owns one contiguous run of token positions
// inside the per-layer KV arena (the same run in every layer).  First-fit with coalescing.
#pragma once

#include <stdint.h>

#include <algorithm>
#include <vector>

namespace bz {

class KvSlots {
  public:
    KvSlots(int max_seqs, int64_t capacity_tokens)
        : off_(max_seqs, -1), cap_(max_seqs, 0) {
        if (capacity_tokens > 0) free_.push_back({0, capacity_tokens});
    }
    bool reserved(int slot) const { return off_[slot] >= 0; }
    int64_t offset(int slot) const { return off_[slot]; }
    int64_t capacity(int slot) const { return cap_[slot]; }
    int64_t largest_free() const {
        int64_t best = 0;
        for (const auto& e : free_) best = std::max(best, e.len);
        return best;
    }
    // returns false when no free run is long enough
    bool reserve(int slot, int64_t tokens) {
        for (size_t i = 0; i < free_.size(); ++i) {
            if (free_[i].len >= tokens) {
                off_[slot] = free_[i].off;
                cap_[slot] = tokens;
                free_[i].off += tokens;
                free_[i].len -= tokens;
                if (free_[i].len == 0) free_.erase(free_.begin() + i);
                return true;
            }
        }
        return false;
    }
    void release(int slot) {
        Extent e{off_[slot], cap_[slot]};
        off_[slot] = -1;
        cap_[slot] = 0;
        auto it = std::lower_bound(free_.begin(), free_.end(), e,
                                   [](const Extent& a, const Extent& b) { return a.off < b.off; });
        it = free_.insert(it, e);
        // merge with the next and the previous run
        if (it + 1 != free_.end() && it->off + it->len == (it + 1)->off) {
            it->len += (it + 1)->len;
            free_.erase(it + 1);
        }
        if (it != free_.begin() && (it - 1)->off + (it - 1)->len == it->off) {
            (it - 1)->len += it->len;
            free_.erase(it);
        }
    }

  private:
    struct Extent {
        int64_t off, len;
    };
    std::vector<Extent> free_;     // sorted by offset, no two adjacent
    std::vector<int64_t> off_, cap_;
};

}  // namespace bz
