// Eviction policy of the aggregate cache (paper Section 3.3, "Eviction Policy") and its stand-alone C entry points.
// Host code only: nothing here touches the device.
#include "cache_policy.h"

#include <algorithm>
#include <new>

namespace reinc {

// Sign of score(a) - score(b) with score = F/S - I, exact: both sides are multiplied by S_a * S_b > 0.
// Sizes, counts and imminences below 2^40 cannot overflow the 128-bit products.
int CachePolicy::compare_score(const Item &a, const Item &b)
{
    using wide = __int128;
    const wide sa = a.size, sb = b.size;
    const wide lhs = wide(a.future) * sb - wide(a.imminence) * sa * sb;
    const wide rhs = wide(b.future) * sa - wide(b.imminence) * sa * sb;
    return lhs < rhs ? -1 : (lhs > rhs ? 1 : 0);
}

bool CachePolicy::leaves_first(int64_t ka, const Item &a, int64_t kb, const Item &b) const
{
    if (policy_ == REINC_POLICY_SCORE) {
        const int c = compare_score(a, b);
        if (c != 0) return c < 0;
    } else if (policy_ == REINC_POLICY_LFU) {
        if (a.uses != b.uses) return a.uses < b.uses;
    }
    if (a.last_use != b.last_use) return a.last_use < b.last_use;
    return ka < kb;
}

void CachePolicy::erase(std::map<int64_t, Item>::iterator it)
{
    n_.used -= it->second.size;
    items_.erase(it);
}

bool CachePolicy::access(int64_t key, bool *expired)
{
    ++tick_;
    if (expired) *expired = false;
    auto it = items_.find(key);
    if (it == items_.end()) {
        ++n_.misses;
        return false;
    }
    ++n_.hits;
    Item &e = it->second;
    e.last_use = tick_;
    ++e.uses;
    if (e.future > 0) --e.future;
    if (policy_ == REINC_POLICY_SCORE && e.future == 0) {
        erase(it);
        ++n_.expired;
        if (expired) *expired = true;
    }
    return true;
}

bool CachePolicy::rescore(int64_t key, int64_t future, int64_t imminence)
{
    auto it = items_.find(key);
    if (it == items_.end()) return false;
    it->second.future = std::max<int64_t>(future, 0);
    it->second.imminence = imminence;
    if (policy_ == REINC_POLICY_SCORE && it->second.future == 0) {
        erase(it);
        ++n_.expired;
        return true;
    }
    return false;
}

bool CachePolicy::offer(int64_t key, int64_t size, int64_t future, int64_t imminence, std::vector<int64_t> *evicted)
{
    ++tick_;
    auto present = items_.find(key);
    if (present != items_.end()) {
        present->second.future = future;
        present->second.imminence = imminence;
        return true;
    }
    const Item fresh{size, future, imminence, tick_, 1};
    auto admit = [&]() {
        items_.emplace(key, fresh);
        n_.used += size;
        n_.peak_used = std::max(n_.peak_used, n_.used);
        ++n_.admitted;
        return true;
    };
    if (policy_ == REINC_POLICY_KEEP_ALL) return admit();
    if (size > budget_ || (policy_ == REINC_POLICY_SCORE && future <= 0)) {
        ++n_.refused;
        return false;
    }
    // choose who leaves: the entry that leaves first among those not chosen yet, until there is room; under the
    // score policy every one of them must score strictly below the newcomer, or nobody leaves
    std::vector<std::map<int64_t, Item>::iterator> out;
    int64_t room = budget_ - n_.used;
    while (room < size) {
        auto worst = items_.end();
        for (auto it = items_.begin(); it != items_.end(); ++it) {
            if (std::find(out.begin(), out.end(), it) != out.end()) continue;
            if (worst == items_.end() || leaves_first(it->first, it->second, worst->first, worst->second)) worst = it;
        }
        if (worst == items_.end()) break;  // cannot happen: size <= budget
        if (policy_ == REINC_POLICY_SCORE && compare_score(worst->second, fresh) >= 0) {
            ++n_.refused;
            return false;
        }
        out.push_back(worst);
        room += worst->second.size;
    }
    for (auto it : out) {
        if (evicted) evicted->push_back(it->first);
        erase(it);
    }
    n_.evicted += int64_t(out.size());
    return admit();
}

void CachePolicy::clear()
{
    items_.clear();
    n_.used = 0;
}

}  // namespace reinc

struct reinc_policy {
    reinc::CachePolicy store;
    reinc_policy(int32_t policy, int64_t budget) : store(policy, budget) {}
};

extern "C" {

int reinc_policy_create(reinc_policy **out, int32_t policy, int64_t budget)
{
    if (!out) return REINC_E_ARG;
    *out = nullptr;
    if (policy < REINC_POLICY_KEEP_ALL || policy > REINC_POLICY_LFU || budget < 0) return REINC_E_ARG;
    reinc_policy *p = new (std::nothrow) reinc_policy(policy, budget);
    if (!p) return REINC_E_NOMEM;
    *out = p;
    return REINC_OK;
}

int reinc_policy_destroy(reinc_policy *p)
{
    delete p;
    return REINC_OK;
}

int reinc_policy_access(reinc_policy *p, int64_t key, int32_t *hit)
{
    if (!p || !hit) return REINC_E_ARG;
    *hit = p->store.access(key, nullptr) ? 1 : 0;
    return REINC_OK;
}

int reinc_policy_offer(reinc_policy *p, int64_t key, int64_t size, int64_t future, int64_t imminence, int32_t *admitted,
                       int64_t *evicted, int32_t evicted_cap, int32_t *n_evicted)
{
    if (!p || !admitted || size <= 0 || evicted_cap < 0 || (evicted_cap > 0 && !evicted)) return REINC_E_ARG;
    try {
        std::vector<int64_t> gone;
        *admitted = p->store.offer(key, size, future, imminence, &gone) ? 1 : 0;
        if (n_evicted) *n_evicted = int32_t(gone.size());
        for (size_t i = 0; i < gone.size() && i < size_t(evicted_cap); ++i) evicted[i] = gone[i];
    } catch (const std::bad_alloc &) {  // no exception crosses the C boundary
        return REINC_E_NOMEM;
    }
    return REINC_OK;
}

int reinc_policy_rescore(reinc_policy *p, int64_t key, int64_t future, int64_t imminence)
{
    if (!p) return REINC_E_ARG;
    p->store.rescore(key, future, imminence);
    return REINC_OK;
}

int reinc_policy_contains(const reinc_policy *p, int64_t key, int32_t *present)
{
    if (!p || !present) return REINC_E_ARG;
    *present = p->store.contains(key) ? 1 : 0;
    return REINC_OK;
}

int reinc_policy_counters(const reinc_policy *p, int64_t *out)
{
    if (!p || !out) return REINC_E_ARG;
    const reinc::CachePolicy::Counters &n = p->store.counters();
    const int64_t v[REINC_POLICY_COUNTERS] = {n.hits, n.misses, n.admitted, n.refused, n.evicted, n.expired, n.used, n.peak_used};
    std::copy(v, v + REINC_POLICY_COUNTERS, out);
    return REINC_OK;
}

}  // extern "C"
