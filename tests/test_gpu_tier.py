"""GPU parity for the pinned tier (paper, "Hierarchical Memory"): allocations whose host side lies
in registered pinned memory move directly between HBM and that memory, the others through the
ring, in one switch.  The result is the same plain definition the oracle computes."""
import numpy as np
import pytest

from tests.helpers import HostSet, AliasedPair

pytestmark = pytest.mark.gpu

KiB, MiB = 1 << 10, 1 << 20
S = 64 * KiB

SIZES_A = [5 * S + 1, 300, 2 * S, 9 * S + 77, 15, 16, 17, 3 * S - 1, 0, 20 * S + 5]
SIZES_B = [4 * S, 11, 3 * S + 9, 7 * S, 1, 12 * S + 3, 999]


@pytest.fixture(scope="module")
def nx():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2601_11743_amd as nx
    nx.lib()
    return nx


class Pinned:
    """A pinned (GPU-addressable) host buffer from torch, as a numpy array."""

    def __init__(self, nbytes: int):
        import torch
        self.t = torch.empty(max(1, nbytes), dtype=torch.uint8, pin_memory=True)
        self.a = self.t.numpy()
        assert self.a.ctypes.data % 4096 == 0


def move_host_arena(hs, pin: Pinned):
    """Relocate a HostSet's pageable arena into pinned memory (same bytes, same alignment)."""
    pin.a[:hs.host.size] = hs.host
    hs.host = pin.a[:hs.host.size]


def test_registration_errors(nx):
    import torch
    pageable = np.zeros(1 << 20, dtype=np.uint8)
    with pytest.raises(nx.NixieError) as e:
        nx.tier_register(pageable.ctypes.data, pageable.size)
    assert e.value.code == nx.EINVAL
    dev = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(nx.NixieError) as e:
        nx.tier_register(dev.data_ptr(), 1 << 20)
    assert e.value.code == nx.EINVAL
    pin = Pinned(1 << 20)
    base = pin.a.ctypes.data
    with pytest.raises(nx.NixieError):
        nx.tier_register(base, 0)
    nx.tier_register(base, 1 << 19)
    for lo, n in [(base, 1 << 19), (base + 4096, 4096), (base + (1 << 19) - 1, 4096)]:
        with pytest.raises(nx.NixieError) as e:
            nx.tier_register(lo, n)                       # overlaps what is registered
        assert e.value.code == nx.EINVAL
    nx.tier_register(base + (1 << 19), 1 << 19)           # adjacent is fine
    with pytest.raises(nx.NixieError):
        nx.tier_unregister(base + 4096)                   # not a registered base
    nx.tier_unregister(base)
    nx.tier_unregister(base + (1 << 19))
    with pytest.raises(nx.NixieError):
        nx.tier_unregister(base)


def test_registration_in_use_cannot_be_dropped(nx):
    """A plan with direct chunks holds GPU addresses of the registered memory: while it lives the
    registration stays (NIXIE_EBUSY), so a later switch can never touch freed pinned memory.  A plan
    whose chunks are all staged holds nothing."""
    from tests.gpu_helpers import GpuSet
    g = GpuSet([3 * S + 5, 100], 5, "dev")
    pin = Pinned(g.hs.host.size)
    move_host_arena(g.hs, pin)
    base = pin.a.ctypes.data
    nx.tier_register(base, g.hs.host.size)
    staged = nx.Plan(g.rows(), [], 8 * S, nx.Opts(slot_bytes=S, flags=nx.NO_DIRECT))
    nx.tier_unregister(base)                              # nothing points into it
    nx.tier_register(base, g.hs.host.size)
    plan = nx.Plan(g.rows(), [], 0, nx.Opts(slot_bytes=S))
    assert plan.info()["direct_bytes_out"] == sum(g.hs.sizes)
    second = nx.Plan(g.rows(), [], 0, nx.Opts(slot_bytes=S))
    for _ in range(2):
        with pytest.raises(nx.NixieError) as e:
            nx.tier_unregister(base)
        assert e.value.code == nx.EBUSY
    plan.switch()                                         # still valid, still correct
    g.hs.check_moved()
    plan.close()
    with pytest.raises(nx.NixieError) as e:
        nx.tier_unregister(base)                          # the second plan still holds it
    assert e.value.code == nx.EBUSY
    second.close()
    staged.close()
    nx.tier_unregister(base)


CASES = {
    # name: (A pinned fraction, B pinned fraction, skew (dev, host), ring bytes, flags, expectation)
    "all_direct_no_ring": (1.0, 1.0, (0, 0), 0, 0, "direct"),
    "all_direct_skewed": (1.0, 1.0, (5, 5), 0, 0, "direct"),
    "out_direct_in_staged": (1.0, 0.0, (3, 3), 8 * S, 0, "mixed"),
    "in_direct_out_staged": (0.0, 1.0, (0, 0), 8 * S, 0, "mixed"),
    "half_and_half": (0.5, 0.5, (7, 7), 8 * S, 0, "mixed"),
    "not_congruent_falls_back": (1.0, 1.0, (1, 2), 8 * S, 0, "staged"),
    "tier_switched_off": (1.0, 1.0, (0, 0), 8 * S, "NO_DIRECT", "staged"),
    "serialized": (0.5, 1.0, (0, 0), 8 * S, "SERIALIZE", "mixed"),
}


@pytest.mark.parametrize("case", list(CASES))
def test_switch_with_pinned_tier_matches_oracle(nx, oracle, case):
    import torch
    from tests.gpu_helpers import GpuSet, first_diff
    fa, fb, skew, ring, flag, expect = CASES[case]
    kw = dict(skew_dev=skew[0], skew_host=skew[1])
    rA, rB = HostSet(SIZES_A, 21, "dev", **kw), HostSet(SIZES_B, 22, "host", **kw)
    h_a, h_b = oracle.hash_table(rA.pairs(), "dev"), oracle.hash_table(rB.pairs(), "host")
    oracle.switch_direct(rA.pairs(), rB.pairs())

    gA, gB = GpuSet(SIZES_A, 21, "dev", **kw), GpuSet(SIZES_B, 22, "host", **kw)
    pins, registered = [], []
    for g, frac in ((gA, fa), (gB, fb)):
        pin = Pinned(g.hs.host.size)
        pins.append(pin)
        move_host_arena(g.hs, pin)
        n = int(g.hs.host.size * frac) // 4096 * 4096 if frac < 1.0 else g.hs.host.size
        if n:
            nx.tier_register(pin.a.ctypes.data, n)
            registered.append(pin.a.ctypes.data)
    try:
        flags = getattr(nx, flag) if flag else 0
        plan = nx.Plan(gA.rows(), gB.rows(), ring, nx.Opts(slot_bytes=S, flags=flags))
        info = plan.info()
        total = sum(SIZES_A) + sum(SIZES_B)
        direct = info["direct_bytes_out"] + info["direct_bytes_in"]
        if expect == "direct":
            assert direct == total and info["pinned_ring_bytes"] == 0
            assert info["drain_threads"] == 0 and info["fill_threads"] == 0
        elif expect == "staged":
            assert direct == 0
        else:
            assert 0 < direct < total
        h_out, h_in = plan.hash_tables()
        assert np.array_equal(h_out, h_a) and np.array_equal(h_in, h_b)
        for _ in range(2):                                   # a plan is reusable
            st = plan.switch()
            assert st["bytes_out"] == sum(SIZES_A) and st["bytes_in"] == sum(SIZES_B)
            if _ == 0:
                dev_B = gB.download()
                assert np.array_equal(gA.hs.host, rA.host), "evicted set: " + first_diff(gA.hs.host, rA.host)
                assert np.array_equal(dev_B, rB.dev), "restored set: " + first_diff(dev_B, rB.dev)
                assert np.array_equal(gA.download(), gA.hs.dev), "device arena of the evicted set was written"
                # second round: the same move again must give the same bytes
                gA.hs.host[:] = 0x11
        dev_B = gB.download()
        assert np.array_equal(dev_B, rB.dev)
        for i, (o, b) in enumerate(zip(gA.hs.lhost.offsets, gA.hs.sizes)):
            assert np.array_equal(gA.hs.host[o:o + b], rA.host[o:o + b]), f"allocation {i} after the second switch"
        plan.verify(h_a, h_b)
        plan.close()
    finally:
        for r in registered:
            nx.tier_unregister(r)


@pytest.mark.parametrize("pinned", ["a", "b", "both"])
def test_in_place_switch_with_pinned_tier(nx, oracle, pinned):
    import torch
    from tests.gpu_helpers import first_diff
    sa, sb, shift = [20 * S + 5, 999, 13 * S, 6 * S], [17 * S, 4, 15 * S + 1, 2 * S], 256
    ref = AliasedPair(sa, sb, 31, shift_b=shift)
    oracle.switch_direct(ref.pairs_a(), ref.pairs_b())
    ref.check()
    g = AliasedPair(sa, sb, 31, shift_b=shift)
    pins, registered = [], []
    for which, name in (("a", "host_a"), ("b", "host_b")):
        if pinned in (which, "both"):
            arr = getattr(g, name)
            pin = Pinned(arr.size)
            pin.a[:arr.size] = arr
            setattr(g, name, pin.a[:arr.size])
            pins.append(pin)
            nx.tier_register(pin.a.ctypes.data, arr.size)
            registered.append(pin.a.ctypes.data)
    try:
        dev_t = torch.from_numpy(g.dev).to("cuda:0")
        base = dev_t.data_ptr()
        rows_a = [(base + od, g.host_a.ctypes.data + oh, b) for od, oh, b in zip(g.la.offsets, g.lha.offsets, g.sizes_a)]
        rows_b = [(base + od, g.host_b.ctypes.data + oh, b) for od, oh, b in zip(g.lb.offsets, g.lhb.offsets, g.sizes_b)]
        plan = nx.Plan(rows_a, rows_b, 8 * S, nx.Opts(slot_bytes=S, flags=nx.IN_PLACE))
        info = plan.info()
        assert info["direct_bytes_out"] == (sum(sa) if pinned in ("a", "both") else 0)
        assert info["direct_bytes_in"] == (sum(sb) if pinned in ("b", "both") else 0)
        plan.switch()
        torch.cuda.synchronize()
        dev_after = dev_t.cpu().numpy()
        assert np.array_equal(g.host_a, ref.host_a), "evicted set: " + first_diff(g.host_a, ref.host_a)
        assert np.array_equal(dev_after, ref.dev), "device arena: " + first_diff(dev_after, ref.dev)
        plan.close()
    finally:
        for r in registered:
            nx.tier_unregister(r)


def test_prefetch_into_the_pinned_tier_then_switch(nx, oracle):
    """The incoming application waits in pageable memory, is brought into the pinned tier ahead of
    the switch (nixie_host_copy, the scheduler's prefetch candidate), and then moves directly;
    the evicted one lands in the pinned tier and is demoted to pageable memory afterwards."""
    from tests.gpu_helpers import GpuSet, first_diff
    rA, rB = HostSet(SIZES_A, 21, "dev"), HostSet(SIZES_B, 22, "host")
    oracle.switch_direct(rA.pairs(), rB.pairs())
    gA, gB = GpuSet(SIZES_A, 21, "dev"), GpuSet(SIZES_B, 22, "host")
    pin_a, pin_b = Pinned(gA.hs.host.size), Pinned(gB.hs.host.size)
    pin_a.a[:] = 0xEE
    pin_b.a[:] = 0xEE
    nx.tier_register(pin_a.a.ctypes.data, pin_a.a.size)
    nx.tier_register(pin_b.a.ctypes.data, pin_b.a.size)
    try:
        offs_a, offs_b = gA.hs.lhost.offsets, gB.hs.lhost.offsets
        pageable_b, pageable_a = gB.hs.host.ctypes.data, gA.hs.host.ctypes.data
        nx.host_copy([pin_b.a.ctypes.data + o for o in offs_b], [pageable_b + o for o in offs_b], SIZES_B, 3)
        dev_a, dev_b = gA.dev_t.data_ptr(), gB.dev_t.data_ptr()
        rows_a = [(dev_a + od, pin_a.a.ctypes.data + oh, b) for od, oh, b in zip(gA.hs.ldev.offsets, offs_a, SIZES_A)]
        rows_b = [(dev_b + od, pin_b.a.ctypes.data + oh, b) for od, oh, b in zip(gB.hs.ldev.offsets, offs_b, SIZES_B)]
        plan = nx.Plan(rows_a, rows_b, 0)
        info = plan.info()
        assert info["direct_bytes_out"] == sum(SIZES_A) and info["direct_bytes_in"] == sum(SIZES_B)
        plan.switch()
        plan.close()
        nx.host_copy([pageable_a + o for o in offs_a], [pin_a.a.ctypes.data + o for o in offs_a], SIZES_A)
        dev_B = gB.download()
        assert np.array_equal(dev_B, rB.dev), "restored set: " + first_diff(dev_B, rB.dev)
        assert np.array_equal(gA.hs.host, rA.host), "evicted set: " + first_diff(gA.hs.host, rA.host)
    finally:
        nx.tier_unregister(pin_a.a.ctypes.data)
        nx.tier_unregister(pin_b.a.ctypes.data)


def test_placement_drives_a_partial_eviction(nx, oracle):
    """Three applications on a GPU too small for all: nixie_place picks the victims (C before A,
    only as far as needed) and their host tiers, the tables of the switch are read off its answer,
    and the switch is checked against the oracle run on CPU mirrors of the same buffers."""
    import torch
    from tests.gpu_helpers import GpuSet, first_diff
    sizes = {0: [6 * S, 3 * S + 5, 4 * S], 2: [5 * S, 2 * S, 7 * S + 1, 900], 1: [8 * S, 4 * S + 3, 6 * S, 10]}
    seeds = {0: 51, 1: 52, 2: 53}
    B_TIERS = [nx.TIER_PINNED, nx.TIER_PAGEABLE, nx.TIER_PAGEABLE, nx.TIER_PINNED]
    resident = {a: sum(sizes[a]) for a in (0, 2)}
    gpu_cap = resident[0] + resident[2] + 3 * S           # B needs ~18 S: about 15 S must go
    pin_cap = 12 * S + 4096

    chunks, index = [], []
    for a in (0, 2, 1):
        for i, b in enumerate(sizes[a]):
            chunks.append((b, a, nx.TIER_GPU if a != 1 else B_TIERS[i]))
            index.append((a, i))
    tier, summ, order = nx.place(gpu_cap, pin_cap, chunks, 1, [2, 0])
    evicted = {index[j] for j in range(len(chunks)) if chunks[j][2] == nx.TIER_GPU and tier[j] != nx.TIER_GPU}
    assert evicted == {(2, i) for i in range(len(sizes[2]))} | {(0, 0)}      # all of C, then A's first chunk only
    assert summ["kept_pinned_bytes"] > 0 and summ["to_pageable_bytes"] > 0 and summ["gpu_used_after"] <= gpu_cap

    def build(make_set, pinned_arena):
        """Tables of the switch for one copy of the world (GPU or CPU mirror)."""
        sets = {a: make_set(sizes[a], seeds[a], "host" if a == 1 else "dev") for a in (0, 1, 2)}
        cursor = 0
        rows_out, rows_in, pairs_out, pairs_in = [], [], [], []
        for j, (a, i) in enumerate(index):
            hs = sets[a].hs if hasattr(sets[a], "hs") else sets[a]
            b = chunks[j][0]
            od, oh = hs.ldev.offsets[i], hs.lhost.offsets[i]
            dev_base = sets[a].dev_t.data_ptr() if hasattr(sets[a], "dev_t") else None
            was, now = chunks[j][2], tier[j]
            if was == now:
                continue
            host_in_pinned = (now if was == nx.TIER_GPU else was) == nx.TIER_PINNED
            if host_in_pinned:                       # a place in the pinned tier, congruent with the device address
                cursor = (cursor + 255) // 256 * 256 + (od % 16)
                host_view = pinned_arena[cursor:cursor + b]
                cursor += b
                if was == nx.TIER_PINNED:
                    host_view[:] = hs.host[oh:oh + b]          # B's chunk waits in the pinned tier
            else:
                host_view = hs.host[oh:oh + b]
            pair = (hs.dev[od:od + b], host_view)
            row = ((dev_base + od) if dev_base is not None else 0, host_view.ctypes.data, b)
            (rows_out if was == nx.TIER_GPU else rows_in).append(row)
            (pairs_out if was == nx.TIER_GPU else pairs_in).append(pair)
        assert cursor <= pin_cap
        return sets, rows_out, rows_in, pairs_out, pairs_in

    ref_pinned = np.full(pin_cap, 0xEE, dtype=np.uint8)
    ref_sets, _, _, ref_out, ref_in = build(lambda s, seed, res: HostSet(s, seed, res), ref_pinned)
    oracle.switch_direct(ref_out, ref_in)

    pin = Pinned(pin_cap)
    pin.a[:] = 0xEE
    nx.tier_register(pin.a.ctypes.data, pin_cap)
    try:
        sets, rows_out, rows_in, _, _ = build(lambda s, seed, res: GpuSet(s, seed, res), pin.a)
        plan = nx.Plan(rows_out, rows_in, 8 * S, nx.Opts(slot_bytes=S))
        info = plan.info()
        assert info["bytes_out"] == summ["evicted_bytes"] and info["bytes_in"] == summ["restored_bytes"]
        assert info["direct_bytes_out"] == summ["kept_pinned_bytes"]
        assert info["direct_bytes_in"] == summ["restored_bytes"] - summ["restored_from_pageable_bytes"]
        plan.switch()
        plan.close()
        assert np.array_equal(pin.a, ref_pinned), "pinned tier: " + first_diff(pin.a, ref_pinned)
        for a in (0, 1, 2):
            got_dev = sets[a].download()
            assert np.array_equal(got_dev, ref_sets[a].dev), f"app {a} device arena: " + first_diff(got_dev, ref_sets[a].dev)
            assert np.array_equal(sets[a].hs.host, ref_sets[a].host), f"app {a} pageable arena"
        import workloads as W
        dev_b = sets[1].download()                   # B is entirely on the GPU, bytes as generated
        for i, (o, b) in enumerate(zip(sets[1].hs.ldev.offsets, sizes[1])):
            assert np.array_equal(dev_b[o:o + b], W.content_bytes(seeds[1], i, b)), f"B's allocation {i}"
    finally:
        nx.tier_unregister(pin.a.ctypes.data)
