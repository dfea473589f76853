// Placement planner: which chunks leave the GPU for the incoming application, and to which host
// tier they go.  Pure host code.
//
// Paper, "Speeding Up Context Switches" (the global plan): the chunks the incoming application
// needs are collected, the chunks to evict are computed -- only as many as needed --, and then
// the tiers are visited from the top to decide how much evicted data may stay in each without
// being pushed further down; transfers that cross several tiers are issued first.
// "Hierarchical Memory": one copy per chunk, so capacities are plain sums.
// Choices the paper leaves open: victims go application by application in the caller's order
// (the scheduler's), inside one in table order; pinned space is claimed first-fit in eviction
// order.
#include <algorithm>
#include <cstdint>
#include <numeric>
#include <vector>

#include "nixie.h"

extern "C" int nixie_place(const nixie_capacity_t *cap, const nixie_chunk_state_t *chunks, uint64_t n,
                           uint32_t incoming_app, const uint32_t *victim_apps, uint32_t n_victims,
                           uint32_t *new_tier, uint64_t *order, uint64_t *n_moved, nixie_placement_t *summary) {
    if (!cap || (n && (!chunks || !new_tier)) || (n_victims && !victim_apps)) return NIXIE_EINVAL;
    uint64_t in_tier[3] = {0, 0, 0};
    uint64_t need = 0, from_pageable = 0;
    for (uint64_t i = 0; i < n; i++) {
        const nixie_chunk_state_t &c = chunks[i];
        if (c.tier > NIXIE_TIER_PAGEABLE) return NIXIE_EINVAL;
        if (in_tier[c.tier] + c.bytes < in_tier[c.tier]) return NIXIE_EINVAL;
        in_tier[c.tier] += c.bytes;
    }
    if (in_tier[NIXIE_TIER_GPU] > cap->gpu_bytes || in_tier[NIXIE_TIER_PINNED] > cap->pinned_bytes) return NIXIE_EINVAL;
    for (uint32_t v = 0; v < n_victims; v++)
        if (victim_apps[v] == incoming_app) return NIXIE_EINVAL;

    // Both directions of a switch run at once, so evicted data can only take pinned room that is
    // free before anything moves: the incoming application's pinned chunks still hold theirs.
    uint64_t pinned_room = cap->pinned_bytes - in_tier[NIXIE_TIER_PINNED];
    // the incoming application moves up, whatever tier it is in
    for (uint64_t i = 0; i < n; i++) {
        const nixie_chunk_state_t &c = chunks[i];
        new_tier[i] = c.tier;
        if (c.app != incoming_app || c.tier == NIXIE_TIER_GPU) continue;
        new_tier[i] = NIXIE_TIER_GPU;
        need += c.bytes;
        in_tier[c.tier] -= c.bytes;
        if (c.tier == NIXIE_TIER_PAGEABLE) from_pageable += c.bytes;
    }
    nixie_placement_t s{};
    s.restored_bytes = need;
    s.restored_from_pageable_bytes = from_pageable;

    // victims: one scan of the table per victim application keeps table order inside it
    uint64_t free_gpu = cap->gpu_bytes - in_tier[NIXIE_TIER_GPU];
    for (uint32_t v = 0; v < n_victims && free_gpu < need; v++) {
        for (uint64_t i = 0; i < n && free_gpu < need; i++) {
            const nixie_chunk_state_t &c = chunks[i];
            if (c.app != victim_apps[v] || c.tier != NIXIE_TIER_GPU || c.bytes == 0 || new_tier[i] != NIXIE_TIER_GPU) continue;
            free_gpu += c.bytes;
            s.evicted_bytes += c.bytes;
            if (c.bytes <= pinned_room) {          // may stay in the upper host tier
                new_tier[i] = NIXIE_TIER_PINNED;
                pinned_room -= c.bytes;
                s.kept_pinned_bytes += c.bytes;
            } else {
                new_tier[i] = NIXIE_TIER_PAGEABLE;
                s.to_pageable_bytes += c.bytes;
            }
        }
    }
    if (free_gpu < need) return NIXIE_ENOMEM;      // does not fit even with every victim gone
    s.gpu_used_after = cap->gpu_bytes - (free_gpu - need);
    s.pinned_used_after = in_tier[NIXIE_TIER_PINNED] + s.kept_pinned_bytes;

    // migration order: two-tier moves, then one-tier moves, table order inside each
    uint64_t moved = 0;
    for (int hops = 2; hops >= 1; hops--)
        for (uint64_t i = 0; i < n; i++) {
            const int d = (int)new_tier[i] - (int)chunks[i].tier;
            if ((d < 0 ? -d : d) != hops) continue;
            if (order) order[moved] = i;
            moved++;
        }
    if (n_moved) *n_moved = moved;
    if (summary) *summary = s;
    return NIXIE_OK;
}
