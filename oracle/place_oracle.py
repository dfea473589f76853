"""CPU oracle of the placement planner (which chunks leave the GPU, and to which host tier).
TEST INFRASTRUCTURE.  Plain Python, shares nothing with the library and never imports it.

What it follows -- paper, "Speeding Up Context Switches", the global plan:
  1. collect the chunks of the incoming application that are not in GPU memory: they all go there;
  2. compute which chunks now in GPU memory must be evicted to make room -- no more than needed;
  3. go through the host tiers, upper one first, and decide how much of the evicted data can stay
     in a tier without being moved further down: what fits in the room the pinned tier has now
     stays there, the rest goes to pageable memory (both directions of a switch run at once, so
     the incoming application's pinned chunks still hold their space while evicted data arrives);
  4. transfers that cross several tiers come first in the migration order.
"Hierarchical Memory": every chunk has exactly one copy, so a tier's usage is the sum of the
chunks placed in it and a capacity is never exceeded.

Readings where the paper is silent (also listed in the design notes) -- "parity unpinned" by the
paper for these, pinned here only by the invariants and by exhaustive search on tiny inputs:
victims are taken application by application in an order the caller supplies (the scheduler's:
lowest priority first), inside an application in table order; eviction stops at the first chunk
boundary at which the incoming application fits; evicted chunks claim pinned space in eviction
order, a chunk that does not fit goes to pageable memory and later, smaller ones may still fit.
"""
from __future__ import annotations

GPU, PINNED, PAGEABLE = 0, 1, 2


class PlacementError(ValueError):
    pass


def place(gpu_capacity: int, pinned_capacity: int, chunks, incoming_app: int, victim_apps):
    """chunks: list of (bytes, app, tier).  Returns (new_tier list, summary dict, order list).

    order: indices of the chunks that move, in migration order (step 4)."""
    used = {GPU: 0, PINNED: 0, PAGEABLE: 0}
    for b, _, t in chunks:
        if t not in used:
            raise PlacementError("unknown tier")
        used[t] += b
    if used[GPU] > gpu_capacity or used[PINNED] > pinned_capacity:
        raise PlacementError("current placement exceeds a capacity")
    if incoming_app in victim_apps:
        raise PlacementError("the incoming application cannot be a victim")
    new_tier = [t for _, _, t in chunks]

    # step 1: everything of the incoming application goes to the GPU
    need = 0
    room = pinned_capacity - used[PINNED]      # step 3 works with the room there is before anything moves
    for i, (b, app, t) in enumerate(chunks):
        if app == incoming_app and t != GPU:
            need += b
            new_tier[i] = GPU
            used[t] -= b
    # step 2: evict until it fits, no further
    free = gpu_capacity - used[GPU]
    evicted = []
    for v in victim_apps:
        for i, (b, app, t) in enumerate(chunks):
            if free >= need:
                break
            if app == v and t == GPU and b > 0:
                evicted.append(i)
                free += b
    if free < need:
        raise PlacementError("the incoming application does not fit even with every victim evicted")
    # step 3: tier by tier, keep what fits
    for i in evicted:
        b = chunks[i][0]
        if b <= room:
            new_tier[i] = PINNED
            room -= b
        else:
            new_tier[i] = PAGEABLE
    # step 4: moves that cross two tiers first; otherwise table order
    moved = [i for i in range(len(chunks)) if new_tier[i] != chunks[i][2]]
    order = sorted(moved, key=lambda i: (-abs(new_tier[i] - chunks[i][2]), i))

    s = dict(restored_bytes=need,
             restored_from_pageable_bytes=sum(chunks[i][0] for i in moved if new_tier[i] == GPU and chunks[i][2] == PAGEABLE),
             evicted_bytes=sum(chunks[i][0] for i in evicted),
             kept_pinned_bytes=sum(chunks[i][0] for i in evicted if new_tier[i] == PINNED),
             to_pageable_bytes=sum(chunks[i][0] for i in evicted if new_tier[i] == PAGEABLE))
    s["gpu_used_after"] = sum(b for (b, _, _), t in zip(chunks, new_tier) if t == GPU)
    s["pinned_used_after"] = sum(b for (b, _, _), t in zip(chunks, new_tier) if t == PINNED)
    return new_tier, s, order
