"""Pins of the placement oracle, run against the oracle and against the library (nixie_place).

The paper gives the steps but no worked numbers, so the pins are hand-worked instances of those
steps, the invariants that "exactly one copy" and the capacities impose, and an exhaustive check
on tiny inputs that the eviction is minimal for the given victim order."""
import itertools

import pytest

from oracle import place_oracle as po

GPU, PIN, PAGE = po.GPU, po.PINNED, po.PAGEABLE
GiB = 1 << 30


def oracle_place(gpu, pinned, chunks, incoming, victims):
    return po.place(gpu, pinned, chunks, incoming, victims)


def library_place(gpu, pinned, chunks, incoming, victims):
    import paper_2601_11743_amd as nx
    try:
        return nx.place(gpu, pinned, chunks, incoming, victims)
    except nx.NixieError as e:
        raise po.PlacementError(str(e))


IMPLS = {"oracle": oracle_place, "library": library_place}


@pytest.fixture(params=list(IMPLS))
def place(request):
    return IMPLS[request.param]


def test_worked_example_partial_eviction(place):
    """32 GiB GPU, 8 GiB pinned.  A (app 0) holds 4 x 6 GiB on the GPU, B (app 1) needs 2 x 7 GiB from
    pageable memory.  Free: 8 GiB; need 14: evict A's chunks in order until >= 14 free: one chunk
    (6 GiB) gives exactly 14.  It fits the pinned tier (8 GiB), so it stays there."""
    chunks = [(6 * GiB, 0, GPU)] * 4 + [(7 * GiB, 1, PAGE)] * 2
    tier, s, order = place(32 * GiB, 8 * GiB, chunks, 1, [0])
    assert tier == [PIN, GPU, GPU, GPU, GPU, GPU]
    assert s["evicted_bytes"] == 6 * GiB and s["kept_pinned_bytes"] == 6 * GiB and s["to_pageable_bytes"] == 0
    assert s["restored_bytes"] == 14 * GiB and s["gpu_used_after"] == 32 * GiB and s["pinned_used_after"] == 6 * GiB
    assert order == [4, 5, 0]            # pageable -> GPU crosses two tiers and goes first


def test_worked_example_pinned_overflow_and_first_fit(place):
    """24 GiB GPU, 10 GiB pinned of which B's 4 GiB chunk still holds its place while the switch runs.
    A holds 8 + 8 + 2 + 6 GiB; B needs 4 (pinned) + 16 (pageable) = 20; free 0 -> evict 8, 8, 2, 6 until
    >= 20 free: 8 + 8 + 2 = 18 < 20, so all four (24).  Pinned room = 10 - 4 = 6: 8 does not fit -> pageable,
    8 -> pageable, 2 fits (room 4), 6 -> pageable."""
    chunks = [(8 * GiB, 0, GPU), (8 * GiB, 0, GPU), (2 * GiB, 0, GPU), (6 * GiB, 0, GPU),
              (4 * GiB, 1, PIN), (16 * GiB, 1, PAGE)]
    tier, s, order = place(24 * GiB, 10 * GiB, chunks, 1, [0])
    assert tier == [PAGE, PAGE, PIN, PAGE, GPU, GPU]
    assert s["kept_pinned_bytes"] == 2 * GiB and s["to_pageable_bytes"] == 22 * GiB
    assert s["restored_from_pageable_bytes"] == 16 * GiB
    assert s["gpu_used_after"] == 20 * GiB and s["pinned_used_after"] == 2 * GiB
    assert order == [0, 1, 3, 5, 2, 4]   # the two-tier moves in table order, then the one-tier moves


def test_pinned_room_counts_the_incoming_chunks_that_are_still_there(place):
    """Both directions of a switch run at once: the space of B's pinned chunk is not free for A's
    evicted chunk, although it will be once the switch is over."""
    chunks = [(4, 0, GPU), (4, 1, PIN)]
    tier, s, _ = place(4, 4, chunks, 1, [0])
    assert tier == [PAGE, GPU] and s["pinned_used_after"] == 0
    tier, s, _ = place(4, 8, chunks, 1, [0])
    assert tier == [PIN, GPU] and s["pinned_used_after"] == 4


def test_nothing_to_do_and_victim_order(place):
    chunks = [(5, 0, GPU), (5, 1, GPU), (5, 2, GPU)]
    tier, s, order = place(20, 0, chunks, 1, [0, 2])
    assert tier == [GPU, GPU, GPU] and order == [] and s["evicted_bytes"] == 0
    # C (app 2) comes first in the victim order: it is the one to go, A stays
    chunks = [(5, 0, GPU), (5, 2, GPU), (7, 1, PAGE)]
    tier, s, _ = place(12, 0, chunks, 1, [2, 0])
    assert tier == [GPU, PAGE, GPU]
    tier, s, _ = place(12, 0, chunks, 1, [0, 2])
    assert tier == [PAGE, GPU, GPU]
    # an application that is not listed is never touched
    with pytest.raises(po.PlacementError):
        place(12, 0, chunks, 1, [0][:0])


def test_errors(place):
    with pytest.raises(po.PlacementError):
        place(10, 0, [(11, 0, GPU)], 1, [0])                       # already over capacity
    with pytest.raises(po.PlacementError):
        place(10, 0, [(6, 0, GPU), (11, 1, PAGE)], 1, [0])         # can never fit
    with pytest.raises(po.PlacementError):
        place(10, 0, [(6, 0, GPU), (5, 1, PAGE)], 1, [1])          # the incoming application as its own victim
    with pytest.raises(po.PlacementError):
        place(10, 0, [(6, 0, 7)], 1, [0])                          # no such tier


def test_invariants_and_minimal_eviction_exhaustively(place):
    """Every instance with 2 applications, up to 3 + 2 chunks of sizes 1..3 on a small machine: one copy
    each, capacities respected, the incoming application entirely on the GPU, untouched chunks
    untouched, and the eviction minimal: without its last victim chunk the GPU would overflow."""
    count = 0
    for na, nb in itertools.product(range(0, 4), range(1, 3)):
        for sizes in itertools.product((1, 2, 3), repeat=na + nb):
            for b_tiers in itertools.product((PIN, PAGE), repeat=nb):
                chunks = [(sizes[i], 0, GPU) for i in range(na)] + [(sizes[na + j], 1, b_tiers[j]) for j in range(nb)]
                for gpu_cap, pin_cap in ((6, 3), (9, 0), (7, 6)):
                    used_g = sum(b for b, _, t in chunks if t == GPU)
                    used_p = sum(b for b, _, t in chunks if t == PIN)
                    b_total = sum(b for b, a, _ in chunks if a == 1)
                    if used_g > gpu_cap or used_p > pin_cap:
                        continue
                    if b_total > gpu_cap:
                        with pytest.raises(po.PlacementError):
                            place(gpu_cap, pin_cap, chunks, 1, [0])
                        continue
                    tier, s, order = place(gpu_cap, pin_cap, chunks, 1, [0])
                    count += 1
                    g = sum(b for (b, _, _), t in zip(chunks, tier) if t == GPU)
                    p = sum(b for (b, _, _), t in zip(chunks, tier) if t == PIN)
                    assert g <= gpu_cap and p <= pin_cap and g == s["gpu_used_after"] and p == s["pinned_used_after"]
                    assert all(t == GPU for (_, a, _), t in zip(chunks, tier) if a == 1)
                    ev = [i for i in range(na) if tier[i] != GPU]
                    assert ev == list(range(len(ev)))              # table order, a prefix of A
                    if ev:                                          # minimal: one chunk fewer would not fit
                        assert g + chunks[ev[-1]][0] > gpu_cap
                    # a chunk goes to pageable memory only if it did not fit the pinned room left at its turn
                    room = pin_cap - sum(b for b, a, t in chunks if t == PIN)
                    for i in ev:
                        if tier[i] == PIN:
                            room -= chunks[i][0]
                        else:
                            assert chunks[i][0] > room
                    assert sorted(order) == [i for i in range(len(chunks)) if tier[i] != chunks[i][2]]
                    hops = [abs(tier[i] - chunks[i][2]) for i in order]
                    assert hops == sorted(hops, reverse=True)
    assert count > 1000
