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
struct TierEntry { TierSpan span; uint64_t id; uint64_t users; };
std::vector<TierEntry> g_tiers;           // sorted by host_base, disjoint; under g_mu
uint64_t g_tier_ids = 0;
}

bool tier_register(const TierSpan &t) {
    std::lock_guard<std::mutex> g(g_mu);
    auto it = std::upper_bound(g_tiers.begin(), g_tiers.end(), t.host_base, [](uint64_t v, const TierEntry &x) { return v < x.span.host_base; });
    if (it != g_tiers.end() && it->span.host_base < t.host_base + t.bytes) return false;
    if (it != g_tiers.begin() && (it - 1)->span.host_base + (it - 1)->span.bytes > t.host_base) return false;
    g_tiers.insert(it, TierEntry{t, ++g_tier_ids, 0});
    return true;
}

TierDrop tier_unregister(uint64_t host_base) {
    std::lock_guard<std::mutex> g(g_mu);
    for (auto it = g_tiers.begin(); it != g_tiers.end(); ++it)
        if (it->span.host_base == host_base) {
            if (it->users) return kTierInUse;
            g_tiers.erase(it);
            return kTierDropped;
        }
    return kTierUnknown;
}

bool tier_translate(uint64_t host_addr, uint64_t bytes, uint64_t *dev_addr, uint64_t *span_id) {
    std::lock_guard<std::mutex> g(g_mu);
    if (g_tiers.empty() || bytes == 0) return false;
    auto it = std::upper_bound(g_tiers.begin(), g_tiers.end(), host_addr, [](uint64_t v, const TierEntry &x) { return v < x.span.host_base; });
    if (it == g_tiers.begin()) return false;
    --it;
    if (host_addr + bytes > it->span.host_base + it->span.bytes) return false;
    *dev_addr = it->span.dev_base + (host_addr - it->span.host_base);
    if (span_id) *span_id = it->id;
    return true;
}

bool tier_acquire(const std::vector<uint64_t> &span_ids) {
    std::lock_guard<std::mutex> g(g_mu);
    for (uint64_t id : span_ids)
        if (std::none_of(g_tiers.begin(), g_tiers.end(), [&](const TierEntry &e) { return e.id == id; })) return false;
    for (uint64_t id : span_ids)
        for (TierEntry &e : g_tiers)
            if (e.id == id) e.users++;
    return true;
}

void tier_release(const std::vector<uint64_t> &span_ids) {
    std::lock_guard<std::mutex> g(g_mu);
    for (uint64_t id : span_ids)
        for (TierEntry &e : g_tiers)
            if (e.id == id && e.users) e.users--;
}

void registry_counts(uint64_t *spaces, uint64_t *tier_spans) {
    std::lock_guard<std::mutex> g(g_mu);
    *spaces = g_spaces.size();
    *tier_spans = g_tiers.size();
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

bool space_assign(uint64_t base, uint64_t first, const uint64_t *pool_blocks, uint64_t count) {
    std::lock_guard<std::mutex> g(g_mu);
    SpaceSpan *s = find_locked(base);
    if (!s || s->base != base || first > s->assigned.size() || count > s->assigned.size() - first) return false;
    for (uint64_t i = 0; i < count; i++)
        if (pool_blocks[i] >= s->assigned.size() || (s->mapped[first + i] && s->assigned[first + i] != pool_blocks[i])) return false;
    for (uint64_t i = 0; i < count; i++) s->assigned[first + i] = pool_blocks[i];
    return true;
}

bool space_translate(uint64_t addr, uint64_t bytes, std::vector<KeyPiece> *pieces, std::vector<SpaceUse> *uses) {
    std::lock_guard<std::mutex> g(g_mu);
    if (bytes == 0) return true;
    SpaceSpan *s = find_locked(addr);
    if (!s) {
        // outside every space: must not reach into one that starts behind addr
        auto it = std::upper_bound(g_spaces.begin(), g_spaces.end(), addr, [](uint64_t v, const SpaceSpan &x) { return v < x.base; });
        if (it != g_spaces.end() && addr + bytes > it->base) return false;
        if (pieces) pieces->push_back(KeyPiece{addr, bytes});
        return true;
    }
    if (addr + bytes > s->base + s->bytes) return false;
    const uint64_t B = s->block_bytes;
    uint64_t off = addr - s->base, left = bytes;
    bool first_piece = true;
    while (left) {
        const uint64_t blk = off / B, in = off % B, take = std::min(left, B - in);
        const uint64_t key = s->key_base + s->assigned[blk] * B + in;
        if (pieces) {
            if (!first_piece && pieces->back().key + pieces->back().len == key) pieces->back().len += take;
            else pieces->push_back(KeyPiece{key, take});
        }
        if (uses) uses->push_back(SpaceUse{s->base, blk, s->assigned[blk]});
        first_piece = false;
        off += take;
        left -= take;
    }
    return true;
}

int space_range_state(uint64_t addr, uint64_t bytes) {
    std::lock_guard<std::mutex> g(g_mu);
    if (bytes == 0) return 0;
    SpaceSpan *s = find_locked(addr);
    if (!s) {
        auto it = std::upper_bound(g_spaces.begin(), g_spaces.end(), addr, [](uint64_t v, const SpaceSpan &x) { return v < x.base; });
        return it != g_spaces.end() && addr + bytes > it->base ? 2 : 0;
    }
    if (addr + bytes > s->base + s->bytes) return 2;
    for (uint64_t blk = (addr - s->base) / s->block_bytes; blk <= (addr + bytes - 1 - s->base) / s->block_bytes; blk++)
        if (!s->mapped[blk]) return 1;
    return 0;
}

bool space_uses_valid(const std::vector<SpaceUse> &uses) {
    std::lock_guard<std::mutex> g(g_mu);
    for (const SpaceUse &u : uses) {
        SpaceSpan *s = find_locked(u.base);
        if (!s || s->base != u.base || u.index >= s->mapped.size()) return false;
        if (!s->mapped[u.index] || s->assigned[u.index] != u.pool_block) return false;
    }
    return true;
}

}  // namespace nixie
