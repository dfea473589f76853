// Registry behind spaces.hpp: a small sorted table under one mutex (plans are rare events).
#include "spaces.hpp"

#include <algorithm>
#include <mutex>

namespace nixie {

namespace {
std::mutex g_mu;
std::vector<SpaceSpan> g_spaces;          // sorted by base, disjoint
uint64_t g_pools = 0;

SpaceSpan *find_locked(uint64_t addr) {
    auto it = std::upper_bound(g_spaces.begin(), g_spaces.end(), addr, [](uint64_t v, const SpaceSpan &s) { return v < s.base; });
    if (it == g_spaces.begin()) return nullptr;
    --it;
    return addr < it->base + it->bytes ? &*it : nullptr;
}
}  // namespace

namespace {
std::vector<TierSpan> g_tiers;            // sorted by host_base, disjoint; under g_mu
}

bool tier_register(const TierSpan &t) {
    std::lock_guard<std::mutex> g(g_mu);
    auto it = std::upper_bound(g_tiers.begin(), g_tiers.end(), t.host_base, [](uint64_t v, const TierSpan &x) { return v < x.host_base; });
    if (it != g_tiers.end() && it->host_base < t.host_base + t.bytes) return false;
    if (it != g_tiers.begin() && (it - 1)->host_base + (it - 1)->bytes > t.host_base) return false;
    g_tiers.insert(it, t);
    return true;
}

bool tier_unregister(uint64_t host_base) {
    std::lock_guard<std::mutex> g(g_mu);
    for (auto it = g_tiers.begin(); it != g_tiers.end(); ++it)
        if (it->host_base == host_base) { g_tiers.erase(it); return true; }
    return false;
}

bool tier_translate(uint64_t host_addr, uint64_t bytes, uint64_t *dev_addr) {
    std::lock_guard<std::mutex> g(g_mu);
    if (g_tiers.empty() || bytes == 0) return false;
    auto it = std::upper_bound(g_tiers.begin(), g_tiers.end(), host_addr, [](uint64_t v, const TierSpan &x) { return v < x.host_base; });
    if (it == g_tiers.begin()) return false;
    --it;
    if (host_addr + bytes > it->host_base + it->bytes) return false;
    *dev_addr = it->dev_base + (host_addr - it->host_base);
    return true;
}

std::shared_mutex &switch_lock() {
    static std::shared_mutex mu;
    return mu;
}

uint64_t next_pool_key() {
    std::lock_guard<std::mutex> g(g_mu);
    return kKeyOrigin + (g_pools++) * kKeyStride;
}

void space_register(const SpaceSpan &s) {
    std::lock_guard<std::mutex> g(g_mu);
    auto it = std::upper_bound(g_spaces.begin(), g_spaces.end(), s.base, [](uint64_t v, const SpaceSpan &x) { return v < x.base; });
    g_spaces.insert(it, s);
}

void space_unregister(uint64_t base) {
    std::lock_guard<std::mutex> g(g_mu);
    g_spaces.erase(std::remove_if(g_spaces.begin(), g_spaces.end(), [&](const SpaceSpan &s) { return s.base == base; }), g_spaces.end());
}

void space_set_mapped(uint64_t base, uint64_t first, uint64_t count, bool on) {
    std::lock_guard<std::mutex> g(g_mu);
    SpaceSpan *s = find_locked(base);
    if (!s || s->base != base) return;
    for (uint64_t b = first; b < first + count && b < s->mapped.size(); b++) s->mapped[b] = on ? 1 : 0;
}

bool space_translate(uint64_t addr, uint64_t bytes, uint64_t *key, SpaceUse *use) {
    std::lock_guard<std::mutex> g(g_mu);
    if (use) *use = SpaceUse{0, 0, 0};
    *key = addr;
    if (bytes == 0) return true;
    SpaceSpan *s = find_locked(addr);
    if (!s) {
        // outside every space: must not reach into one that starts behind addr
        auto it = std::upper_bound(g_spaces.begin(), g_spaces.end(), addr, [](uint64_t v, const SpaceSpan &x) { return v < x.base; });
        return it == g_spaces.end() || addr + bytes <= it->base;
    }
    if (addr + bytes > s->base + s->bytes) return false;
    *key = s->key_base + (addr - s->base);
    if (use) {
        use->base = s->base;
        use->first = (addr - s->base) / s->block_bytes;
        use->count = (addr + bytes - 1 - s->base) / s->block_bytes - use->first + 1;
    }
    return true;
}

bool space_uses_mapped(const std::vector<SpaceUse> &uses) {
    std::lock_guard<std::mutex> g(g_mu);
    for (const SpaceUse &u : uses) {
        SpaceSpan *s = find_locked(u.base);
        if (!s || s->base != u.base) return false;
        for (uint64_t b = u.first; b < u.first + u.count; b++)
            if (b >= s->mapped.size() || !s->mapped[b]) return false;
    }
    return true;
}

}  // namespace nixie
