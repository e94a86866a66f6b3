// Eviction policy of the aggregate cache (paper Section 3.3, "Eviction Policy"): which cached aggregates stay when
// memory is limited.  Host-side bookkeeping only: keys, sizes and scores; the owner maps keys to device buffers.
//
//   score(Agg) = F(Agg) / S(Agg) - I(Agg)     F = accesses still to come, S = size, I = imminence (timesteps
//                                             that pass before the next access); the lowest score leaves first
//   expiration: an entry whose F reaches 0 leaves at once, whatever its score
// and, for comparison (Section 5, "Effectiveness of Caching Policy"), least-recently-used and least-frequently-used.
#pragma once
#include <cstdint>
#include <map>
#include <vector>

#include "reinc.h"

namespace reinc {

class CachePolicy {
   public:
    struct Counters {
        int64_t hits = 0, misses = 0, admitted = 0, refused = 0, evicted = 0, expired = 0, used = 0, peak_used = 0;
    };

    CachePolicy(int32_t policy, int64_t budget) : policy_(policy), budget_(budget) {}

    int32_t policy() const { return policy_; }
    int64_t budget() const { return budget_; }
    const Counters &counters() const { return n_; }
    bool contains(int64_t key) const { return items_.count(key) != 0; }

    // Look-up.  A hit refreshes recency and frequency and consumes one future access; *expired tells the owner that
    // the entry left on this hit (score policy, F reached 0): its buffer is free once the current use is over.
    bool access(int64_t key, bool *expired);
    // A freshly computed aggregate asks for room.  Returns whether it was admitted; keys that had to leave are
    // appended to *evicted.  A refused offer evicts nothing.  An offer of a present key only replaces its F and I.
    bool offer(int64_t key, int64_t size, int64_t future, int64_t imminence, std::vector<int64_t> *evicted);
    // Replaces F and I of a present key; returns true if that expired it.
    bool rescore(int64_t key, int64_t future, int64_t imminence);
    void clear();

   private:
    struct Item {
        int64_t size, future, imminence;
        uint64_t last_use, uses;
    };
    // a leaves before b
    bool leaves_first(int64_t ka, const Item &a, int64_t kb, const Item &b) const;
    static int compare_score(const Item &a, const Item &b);
    void erase(std::map<int64_t, Item>::iterator it);

    int32_t policy_;
    int64_t budget_;
    uint64_t tick_ = 0;
    std::map<int64_t, Item> items_;
    Counters n_;
};

}  // namespace reinc
