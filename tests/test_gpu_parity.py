"""GPU parity: libnixie (through its C ABI) against the CPU oracle, bit for bit.

Every case builds the same seeded inputs twice: one copy goes through the oracle on the CPU,
the other has its device arena uploaded to HBM and goes through nixie_switch.  Destination
arenas are compared whole (contents and red zones); hashes are compared per allocation."""
import numpy as np
import pytest

import workloads as W
from tests.helpers import HostSet

pytestmark = pytest.mark.gpu

KiB, MiB = 1 << 10, 1 << 20


@pytest.fixture(scope="module")
def nx():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2601_11743_amd as nx
    nx.lib()     # raises if the HIP library is missing: no fallback
    return nx


def run_case(nx, oracle, sizes_a, sizes_b, ring, opts=None, seed=7, skew=(0, 0), switches=1,
             oracle_staged=None):
    from tests.gpu_helpers import GpuSet, first_diff
    kw = dict(skew_dev=skew[0], skew_host=skew[1])
    # oracle side
    rA, rB = HostSet(sizes_a, seed, "dev", **kw), HostSet(sizes_b, seed + 1, "host", **kw)
    h_out_ref = oracle.hash_table(rA.pairs(), "dev")
    h_in_ref = oracle.hash_table(rB.pairs(), "host")
    if oracle_staged:
        oracle.switch_staged(rA.pairs(), rB.pairs(), **oracle_staged)
    else:
        oracle.switch_direct(rA.pairs(), rB.pairs())
    # GPU side
    gA, gB = GpuSet(sizes_a, seed, "dev", **kw), GpuSet(sizes_b, seed + 1, "host", **kw)
    plan = nx.Plan(gA.rows(), gB.rows(), ring, opts)
    try:
        info = plan.info()
        assert info["pinned_ring_bytes"] <= ring
        assert info["bytes_out"] == sum(sizes_a) and info["bytes_in"] == sum(sizes_b)
        h_out, h_in = plan.hash_tables()
        assert np.array_equal(h_out, h_out_ref), "pre-switch device hashes differ from the oracle"
        assert np.array_equal(h_in, h_in_ref), "pre-switch host hashes differ from the oracle"
        for _ in range(switches):
            st = plan.switch()
            assert st["bytes_out"] == sum(sizes_a) and st["bytes_in"] == sum(sizes_b)
        dev_B = gB.download()
        assert np.array_equal(gA.hs.host, rA.host), "evicted set: " + first_diff(gA.hs.host, rA.host)
        assert np.array_equal(dev_B, rB.dev), "restored set: " + first_diff(dev_B, rB.dev)
        # the source device arena of A keeps its red zones too (nothing strays on the device side)
        dev_A = gA.download()
        assert np.array_equal(dev_A, gA.hs.dev), "device arena of the evicted set was written"
        rep = plan.verify(h_out_ref, h_in_ref)
        assert rep["mismatched_out"] == 0 and rep["mismatched_in"] == 0
        assert rep["checked_out"] == len(sizes_a) and rep["checked_in"] == len(sizes_b)
        return info, st
    finally:
        plan.close()


def test_config1_tiny(nx, oracle):
    cf = W.config(1)
    sa, sb = [b for _, b in cf["A"]], [b for _, b in cf["B"]]
    info, st = run_case(nx, oracle, sa, sb, cf["ring_bytes"][0], nx.Opts(slot_bytes=cf["slot_bytes"]),
                        seed=cf["seed_A"])
    assert info["slot_bytes"] == 256 * KiB and info["out_slots"] == 8 and info["in_slots"] == 8


S = 64 * KiB


@pytest.mark.parametrize("order", [0, 1, 2, 3])
def test_edge_sizes_every_order(nx, oracle, order):
    sizes_a = [1, 15, 16, 17, 255, 4096, S - 1, S, S + 1, 3 * S + 5, 0, 10 * S + 333, 7]
    sizes_b = [S + 1, 2, 7 * S - 3, 0, 31, 5 * S, 16]
    run_case(nx, oracle, sizes_a, sizes_b, 8 * S, nx.Opts(slot_bytes=S, order=order))


@pytest.mark.parametrize("skew", [(1, 0), (0, 7), (15, 9), (3, 3), (8, 12)])
def test_unaligned_bases(nx, oracle, skew):
    sizes_a = [100, 1000, S + 3, 5, 2 * S, 40000]
    sizes_b = [999, 16, 3 * S + 1, 77777]
    run_case(nx, oracle, sizes_a, sizes_b, 8 * S, nx.Opts(slot_bytes=S), skew=skew)


def test_pure_evict_and_pure_restore(nx, oracle):
    run_case(nx, oracle, [3 * S + 1, 5, 900000], [], 4 * S, nx.Opts(slot_bytes=S))
    run_case(nx, oracle, [], [2 * S, 9, 1234567], 4 * S, nx.Opts(slot_bytes=S))
    run_case(nx, oracle, [], [], 4 * S, nx.Opts(slot_bytes=S))
    run_case(nx, oracle, [0, 0], [0], 4 * S, nx.Opts(slot_bytes=S))


@pytest.mark.parametrize("team,wgs", [(1, 1), (1, 7), (2, 8), (4, 64), (8, 64), (3, 5)])
def test_launch_shapes(nx, oracle, team, wgs):
    sizes_a = [5 * S + 1, 300, 2 * S, 11 * S + 17]
    sizes_b = [4 * S, 11, 6 * S + 9, 200000]
    run_case(nx, oracle, sizes_a, sizes_b, 8 * S,
             nx.Opts(slot_bytes=S, team=team, gather_wgs=wgs, scatter_wgs=wgs, drain_threads=2, fill_threads=3))


@pytest.mark.parametrize("g,s,flex,flags", [(1, 1, 1, 0), (1, 1, 32, 0), (3, 2, 7, 0), (16, 8, 64, 0), (8, 8, 0, "NO_FLEX_WGS"),
                                           (2, 5, 9, "IN_ORDER_ADDRESS")])
def test_workgroups_that_serve_either_direction(nx, oracle, g, s, flex, flags):
    """Workgroups without a fixed role take units of whichever direction has more left; with one fixed
    workgroup per direction they do nearly all the work, in both roles, one unit after the other."""
    sizes_a = [5 * S + 1, 300, 2 * S, 11 * S + 17, 7]
    sizes_b = [4 * S, 11, 6 * S + 9, 200000, 3 * S - 5, 15 * S]
    o = nx.Opts(slot_bytes=S, team=4, gather_wgs=g, scatter_wgs=s, flex_wgs=flex, drain_threads=2, fill_threads=2,
                flags=nx.NO_FLEX_WGS if flags == "NO_FLEX_WGS" else 0, order=nx.ORDER_ADDRESS if flags == "IN_ORDER_ADDRESS" else 0)
    info, st = run_case(nx, oracle, sizes_a, sizes_b, 8 * S, o, switches=2)
    assert info["flex_wgs"] == (0 if flags == "NO_FLEX_WGS" else flex)
    # very unequal sets, and one of them empty: the roles collapse to one
    run_case(nx, oracle, [30 * S + 1], [100], 8 * S, o)
    run_case(nx, oracle, [100], [30 * S + 1], 8 * S, o)
    info, st = run_case(nx, oracle, [9 * S], [], 8 * S, o)
    assert info["flex_wgs"] == 0


def test_uneven_ring_split_and_staged_oracle(nx, oracle):
    sizes_a = [9 * S + 1, 77, 3 * S]
    sizes_b = [5 * S, 3, 2 * S + 2]
    run_case(nx, oracle, sizes_a, sizes_b, 8 * S, nx.Opts(slot_bytes=S, out_slots=6),
             oracle_staged=dict(ring_bytes=8 * S, slot_bytes=S, n_out_slots=6, seed=3, check_bytes=True))
    run_case(nx, oracle, sizes_a, sizes_b, 8 * S, nx.Opts(slot_bytes=S, flags=nx.SPLIT_BY_BYTES))


def test_serialized_and_plain_memcpy_modes(nx, oracle):
    sizes_a = [9 * S + 1, 77, 3 * S]
    sizes_b = [5 * S, 3, 2 * S + 2]
    info, st = run_case(nx, oracle, sizes_a, sizes_b, 8 * S, nx.Opts(slot_bytes=S, flags=nx.SERIALIZE))
    assert st["kernels"] == 2
    run_case(nx, oracle, sizes_a, sizes_b, 8 * S, nx.Opts(slot_bytes=S, flags=nx.HOST_PLAIN_MEMCPY))


def test_statistics_are_filled_in(nx, oracle):
    """Timers and counters of a switch: plausible and complete (every slot is used many times over, so
    the pump has made rounds and has seen credit round trips in both directions)."""
    info, st = run_case(nx, oracle, [60 * S + 5, 999], [55 * S, 4], 4 * S, nx.Opts(slot_bytes=S))
    assert st["bytes_out"] == 60 * S + 5 + 999 and st["bytes_in"] == 55 * S + 4 and st["kernels"] == 1
    assert 0 < st["ns_launch"] < st["ns_total"] and 0 < st["ns_kernel"] <= st["ns_total"]
    assert 0 < st["ns_in_done"] <= st["ns_total"] and 0 < st["ns_out_done"] <= st["ns_total"]
    assert st["pump_rounds_out"] > 10 and st["pump_rounds_in"] > 10
    for rtt in (st["credit_rtt_ticks_out"], st["credit_rtt_ticks_in"]):
        assert 50 < rtt < 100_000_000          # between half a microsecond and a second, in 100 MHz ticks
    assert st["gpu_status"] == 0


def test_repeated_switch_same_plan(nx, oracle):
    """A plan is reusable: flags and counters start clean every time."""
    run_case(nx, oracle, [20 * S + 5, 999], [17 * S, 4], 4 * S, nx.Opts(slot_bytes=S), switches=3)


def test_many_small_allocations(nx, oracle):
    sa = W.log_uniform_sizes(5, 3000, 256, 64 * KiB, 1)
    sb = W.log_uniform_sizes(6, 3000, 256, 64 * KiB, 1)
    run_case(nx, oracle, sa, sb, 4 * MiB, None)   # default slot: halves down from 2 MiB


def test_hash_buffers_device_and_host(nx, oracle):
    import torch
    sizes = [0, 1, 7, 8, 9, 4095, 32768, 32769, 100000, 3 * MiB + 5]
    for skew in (0, 3, 8):
        hs = HostSet(sizes, 99, "dev", skew_dev=skew)
        ref = oracle.hash_table(hs.pairs(), "dev")
        t = torch.from_numpy(hs.dev).to("cuda:0")
        ptrs = [t.data_ptr() + o for o in hs.ldev.offsets]
        got_d = nx.hash_buffers(ptrs, sizes, True)
        got_h = nx.hash_buffers([hs.dev.ctypes.data + o for o in hs.ldev.offsets], sizes, False)
        assert np.array_equal(got_d, ref) and np.array_equal(got_h, ref)


def test_verify_reports_mismatch(nx, oracle):
    from tests.gpu_helpers import GpuSet
    gA, gB = GpuSet([5000, 6000], 1, "dev"), GpuSet([7000], 2, "host")
    plan = nx.Plan(gA.rows(), gB.rows(), 4 * S, nx.Opts(slot_bytes=S))
    ho, hi = plan.hash_tables()
    plan.switch()
    bad = ho.copy(); bad[1] ^= np.uint64(1)
    rep = plan.verify(bad, hi, check=False)
    assert rep["rc"] == nx.EMISMATCH and rep["first_bad_out"] == 1 and rep["mismatched_in"] == 0
    plan.close()


def test_errors(nx):
    from tests.gpu_helpers import GpuSet
    g = GpuSet([5000, 6000], 1, "dev")
    rows = g.rows()
    with pytest.raises(nx.NixieError) as e:
        nx.Plan(rows, [], 64 * KiB, nx.Opts(slot_bytes=64 * KiB))        # one slot only
    assert e.value.code == nx.EINVAL
    with pytest.raises(nx.NixieError) as e:
        nx.Plan(rows + [(rows[0][0] + 10, rows[0][1] + 100000, 100)], [], 4 * S)   # device overlap
    assert e.value.code == nx.EOVERLAP
    with pytest.raises(nx.NixieError) as e:
        nx.Plan(rows, [], 4 * S, nx.Opts(slot_bytes=1000))              # slot not a multiple of 4096
    assert e.value.code == nx.EINVAL


def test_stalled_drain_times_out_cleanly(nx):
    """Credits are withheld by the host on purpose: the kernel's bounded wait expires, every
    workgroup leaves, and the switch reports a timeout instead of hanging."""
    from tests.gpu_helpers import GpuSet
    gA, gB = GpuSet([40 * S], 1, "dev"), GpuSet([3 * S], 2, "host")
    plan = nx.Plan(gA.rows(), gB.rows(), 4 * S,
                   nx.Opts(slot_bytes=S, timeout_ms=300, flags=nx.DIAG_STALL_DRAIN))
    st = plan.switch(check=False)
    assert st["rc"] == nx.ETIMEOUT
    assert st["ns_total"] < 5e9
    plan.close()
    # the device is still healthy: a normal switch works right after
    gA2, gB2 = GpuSet([40 * S], 1, "dev"), GpuSet([3 * S], 2, "host")
    plan = nx.Plan(gA2.rows(), gB2.rows(), 4 * S, nx.Opts(slot_bytes=S))
    plan.switch()
    gA2.hs.check_moved()
    plan.close()


# ---- in-place switch: B's device ranges reuse the GPU memory A gives up -----------------------

ALIAS_CASES = [
    ([5 * S + 1, 300, 2 * S, 9 * S + 77], [4 * S, 11, 3 * S + 9, 7 * S], 0),
    ([3 * S, 3 * S, 3 * S, 3 * S], [3 * S, 3 * S, 3 * S, 3 * S], 0),
    ([2 * S + 7, 900, 5 * S], [S, S, 500, 4 * S + 3], 1000),
    ([4 * S], [100, 200, 6 * S], 3 * S),
    ([20 * S + 5, 999, 13 * S], [17 * S, 4, 15 * S + 1], 256),
]


def run_in_place(nx, oracle, sa, sb, shift, skew_a, skew_b, ring, opts, extra_flags=0):
    import torch
    from tests.helpers import AliasedPair
    from tests.gpu_helpers import first_diff
    ref = AliasedPair(sa, sb, 31, shift_b=shift, skew_a=skew_a, skew_b=skew_b)
    h_out_ref = oracle.hash_table(ref.pairs_a(), "dev")
    h_in_ref = oracle.hash_table(ref.pairs_b(), "host")
    oracle.switch_direct(ref.pairs_a(), ref.pairs_b())           # the definition: evict all, then restore
    ref.check()

    g = AliasedPair(sa, sb, 31, shift_b=shift, skew_a=skew_a, skew_b=skew_b)
    dev_t = torch.from_numpy(g.dev).to("cuda:0")
    base = dev_t.data_ptr()
    rows_a = [(base + od, g.host_a.ctypes.data + oh, b) for od, oh, b in zip(g.la.offsets, g.lha.offsets, g.sizes_a)]
    rows_b = [(base + od, g.host_b.ctypes.data + oh, b) for od, oh, b in zip(g.lb.offsets, g.lhb.offsets, g.sizes_b)]
    plan = nx.Plan(rows_a, rows_b, ring, nx.Opts(flags=nx.IN_PLACE | extra_flags, **opts))
    try:
        h_out, h_in = plan.hash_tables()
        assert np.array_equal(h_out, h_out_ref) and np.array_equal(h_in, h_in_ref)
        st = plan.switch()
        torch.cuda.synchronize()
        dev_after = dev_t.cpu().numpy()
        assert np.array_equal(g.host_a, ref.host_a), "evicted set: " + first_diff(g.host_a, ref.host_a)
        assert np.array_equal(dev_after, ref.dev), "device arena: " + first_diff(dev_after, ref.dev)
        plan.verify(h_out_ref, h_in_ref)
    finally:
        plan.close()
    return rows_a, rows_b, st


@pytest.mark.parametrize("case", range(len(ALIAS_CASES)))
@pytest.mark.parametrize("mode", ["default", "small_units", "serialized", "either"])
def test_in_place_switch(nx, oracle, case, mode):
    sa, sb, shift = ALIAS_CASES[case]
    kw = dict(default={}, small_units=dict(team=8, gather_wgs=16, scatter_wgs=24, drain_threads=2, fill_threads=2),
              serialized={}, either=dict(team=4, gather_wgs=1, scatter_wgs=1, flex_wgs=24))[mode]
    rows_a, rows_b, _ = run_in_place(nx, oracle, sa, sb, shift, case % 3, (case * 5) % 16, 8 * S, dict(slot_bytes=S, **kw),
                                     nx.SERIALIZE if mode == "serialized" else 0)
    with pytest.raises(nx.NixieError):
        nx.Plan(rows_a, rows_b, 8 * S, nx.Opts(slot_bytes=S))     # without the flag aliasing is an error


def _random_alias_case(seed):
    """Seeded draw of aliased tables: sizes, how far B's ranges are shifted against A's, alignment of either
    side, slot and ring size, order, launch shape, flags (as names)."""
    rng = np.random.default_rng(7000 + seed)
    slot = int(rng.choice([4 * KiB, 16 * KiB, 64 * KiB]))
    draw = lambda n: [int(rng.choice([1, 16, slot - 1, slot, slot + 1])) if rng.random() < 0.25
                      else int(np.exp(rng.uniform(0, np.log(8 * slot)))) for _ in range(n)]
    sa, sb = draw(int(rng.integers(1, 25))), draw(int(rng.integers(1, 25)))
    shift = int(rng.choice([0, 16, 1000, slot, 3 * slot + 48, int(rng.integers(0, max(1, sum(sa))))]))
    o = dict(slot_bytes=slot, order=int(rng.integers(0, 4)), drain_threads=int(rng.integers(1, 4)),
             fill_threads=int(rng.integers(1, 4)))
    if rng.random() < 0.5: o["team"] = int(rng.integers(1, 9))
    if rng.random() < 0.6: o["gather_wgs"], o["scatter_wgs"] = int(rng.integers(1, 25)), int(rng.integers(1, 25))
    if rng.random() < 0.5: o["flex_wgs"] = int(rng.integers(1, 33))
    extra = 0
    if rng.random() < 0.2: extra |= 2          # SERIALIZE
    if rng.random() < 0.3: extra |= 1          # SPLIT_BY_BYTES
    if rng.random() < 0.2: extra |= 256        # NO_FLEX_WGS
    ring = int(rng.integers(4, 20)) * slot
    return sa, sb, shift, int(rng.integers(0, 16)), int(rng.integers(0, 16)), ring, o, extra


@pytest.mark.parametrize("seed", range(16))
def test_random_in_place_plans(nx, oracle, seed):
    sa, sb, shift, skew_a, skew_b, ring, o, extra = _random_alias_case(seed)
    print(f"seed {seed}: {len(sa)} + {len(sb)} allocations, {sum(sa)} + {sum(sb)} bytes, shift {shift}, ring {ring}, {o}, "
          f"extra flags {extra}", flush=True)
    run_in_place(nx, oracle, sa, sb, shift, skew_a, skew_b, ring, o, extra)


def test_in_place_small_incoming_set_is_ready_early(nx, oracle):
    """768 MiB leave, 128 MiB come in where the LAST eight outgoing allocations are: the planner evicts those
    first, so the incoming application is ready after a fraction of the switch (it would be ready only at the
    very end if the outgoing table were walked as listed)."""
    import workloads as W
    sa = [16 * MiB] * 48
    sb = [16 * MiB - 4096] * 8
    la, lb = W.make_layout(sa, redzone=256), W.make_layout(sb, redzone=256)
    shift = la.offsets[40] - lb.offsets[0]
    _, _, st = run_in_place(nx, oracle, sa, sb, shift, 0, 0, 64 * MiB, {})
    print(f"in-place 768 MiB out / 128 MiB in over the tail: B ready after {st['ns_in_done'] / 1e6:.2f} ms of "
          f"{st['ns_total'] / 1e6:.2f} ms", flush=True)
    assert 0 < st["ns_in_done"] < 0.5 * st["ns_total"], st


# ---- one ring for many plans --------------------------------------------------------------------

def test_plans_share_one_ring(nx, oracle):
    """Three plans made on one ring object, switched one after the other: each matches the oracle;
    the pinned payload memory is the ring's; a ring in use cannot be destroyed, nor serve two
    switches at once."""
    from tests.gpu_helpers import GpuSet, first_diff
    ring = nx.Ring(8 * S)
    plans, sets, refs = [], [], []
    for k, (sa, sb) in enumerate([([5 * S + 1, 300, 2 * S], [4 * S, 11]), ([S, S, S - 1], [7 * S + 3]),
                                  ([9 * S + 77], [3 * S + 9, 7 * S, 15])]):
        rA, rB = HostSet(sa, 80 + k, "dev"), HostSet(sb, 90 + k, "host")
        oracle.switch_direct(rA.pairs(), rB.pairs())
        gA, gB = GpuSet(sa, 80 + k, "dev"), GpuSet(sb, 90 + k, "host")
        p = nx.Plan(gA.rows(), gB.rows(), ring, nx.Opts(slot_bytes=S))
        assert p.info()["ring_bytes"] == 8 * S and p.info()["pinned_ring_bytes"] <= 8 * S
        plans.append(p); sets.append((gA, gB)); refs.append((rA, rB))
    with pytest.raises(nx.NixieError) as e:
        ring.close()                                             # three plans still use it
    assert e.value.code == nx.EBUSY
    plans[0].switch_begin()
    assert plans[1].switch(check=False)["rc"] == nx.EBUSY        # the ring is busy with another plan's switch
    plans[0].switch_end()
    for p in plans[1:] + plans[:1]:                              # plan 0 a second time, in another order
        p.switch()
    for (gA, gB), (rA, rB) in zip(sets, refs):
        dev_B = gB.download()
        assert np.array_equal(gA.hs.host, rA.host), "evicted set: " + first_diff(gA.hs.host, rA.host)
        assert np.array_equal(dev_B, rB.dev), "restored set: " + first_diff(dev_B, rB.dev)
    with pytest.raises(nx.NixieError):
        nx.Plan(sets[0][0].rows(), sets[0][1].rows(), ring, nx.Opts(slot_bytes=4 * S))   # 2 slots: too small a ring
    for p in plans:
        p.close()
    ring.close()


# ---- special cases that reduce to a library routine ---------------------------------------------

def test_single_allocation_equals_a_plain_device_copy(nx):
    """One allocation each way, ring larger than both: the switch is one D2H and one H2D copy, and
    must give what torch's own copies (the runtime's hipMemcpy path) give."""
    import torch
    n_a, n_b = 3 * MiB + 17, 2 * MiB + 5
    g = torch.Generator(device="cuda:0")
    g.manual_seed(5)
    dev_a = torch.randint(0, 256, (n_a,), dtype=torch.uint8, device="cuda:0", generator=g)
    host_b = np.random.default_rng(6).integers(0, 256, n_b, dtype=np.uint8)
    host_a = np.zeros(n_a, dtype=np.uint8)
    dev_b = torch.zeros(n_b, dtype=torch.uint8, device="cuda:0")
    want_a = dev_a.cpu().numpy()                                    # library D2H
    want_b = torch.from_numpy(host_b).to("cuda:0")                  # library H2D
    torch.cuda.synchronize()
    plan = nx.Plan([(dev_a.data_ptr(), host_a.ctypes.data, n_a)], [(dev_b.data_ptr(), host_b.ctypes.data, n_b)], 16 * MiB)
    plan.switch()
    plan.close()
    assert np.array_equal(host_a, want_a)
    assert torch.equal(dev_b, want_b)


def test_pure_eviction_equals_concatenation_copied_to_the_host(nx):
    """Empty incoming table: the gather of many allocations into one host buffer is torch.cat(...).cpu()."""
    import torch
    g = torch.Generator(device="cuda:0")
    g.manual_seed(9)
    sizes = [5 * S + 1, 300, 2 * S, 9 * S + 77, 15, 16, 17, 1, 3 * S - 1]
    parts = [torch.randint(0, 256, (b,), dtype=torch.uint8, device="cuda:0", generator=g) for b in sizes]
    want = torch.cat(parts).cpu().numpy()
    host = np.full(sum(sizes), 0x5A, dtype=np.uint8)
    offs = np.concatenate([[0], np.cumsum(sizes)[:-1]]).astype(int)
    rows_out = [(p.data_ptr(), host.ctypes.data + int(o), b) for p, o, b in zip(parts, offs, sizes)]
    plan = nx.Plan(rows_out, [], 4 * S, nx.Opts(slot_bytes=S))
    assert plan.info()["in_slots"] == 0
    plan.switch()
    plan.close()
    assert np.array_equal(host, want)


def _random_case(seed):
    """One seeded draw over everything a caller can choose: table shapes, sizes around the slot
    boundaries, slot and ring size, ring split, order, launch shape, host threads, host-side modes."""
    rng = np.random.default_rng(1000 + seed)
    slot = int(rng.choice([4 * KiB, 16 * KiB, 64 * KiB, 256 * KiB]))
    edge = [0, 1, 15, 16, 17, slot - 1, slot, slot + 1, 2 * slot + 5]

    def sizes(n):
        out = []
        for _ in range(n):
            if rng.random() < 0.3:
                out.append(int(rng.choice(edge)))
            else:
                out.append(int(np.exp(rng.uniform(0, np.log(6 * slot)))))
        return out

    na, nb = int(rng.integers(0, 40)), int(rng.integers(0, 40))
    if seed % 8 == 5: na = 0
    if seed % 8 == 6: nb = 0
    sa, sb = sizes(na), sizes(nb)
    n_slots = int(rng.integers(4, 25))
    o = dict(slot_bytes=slot, order=int(rng.integers(0, 4)), drain_threads=int(rng.integers(1, 5)),
             fill_threads=int(rng.integers(1, 5)))
    if rng.random() < 0.5: o["team"] = int(rng.integers(1, 9))
    if rng.random() < 0.6:
        o["gather_wgs"], o["scatter_wgs"] = int(rng.integers(1, 33)), int(rng.integers(1, 33))
    if rng.random() < 0.5: o["flex_wgs"] = int(rng.integers(1, 41))
    flags = 0
    for f, pr in (("SPLIT_BY_BYTES", 0.3), ("SERIALIZE", 0.15), ("HOST_PLAIN_MEMCPY", 0.3), ("HOST_SPIN", 0.3),
                  ("NO_FLEX_WGS", 0.2)):
        if rng.random() < pr: flags |= {"SPLIT_BY_BYTES": 1, "SERIALIZE": 2, "HOST_PLAIN_MEMCPY": 16, "HOST_SPIN": 128,
                                        "NO_FLEX_WGS": 256}[f]
    o["flags"] = flags
    if not (flags & 1) and sum(sa) and sum(sb) and rng.random() < 0.4:
        o["out_slots"] = int(rng.integers(2, n_slots - 1))
    skew = (int(rng.integers(0, 16)), int(rng.integers(0, 16))) if rng.random() < 0.5 else (0, 0)
    return sa, sb, n_slots * slot, o, skew, int(rng.integers(1, 3))


@pytest.mark.parametrize("seed", range(32))
def test_random_plans(nx, oracle, seed):
    """Seeded sweep over the option space (no aliasing, no pinned tier: those have sweeps of their own)."""
    sa, sb, ring, o, skew, switches = _random_case(seed)
    print(f"seed {seed}: {len(sa)} + {len(sb)} allocations, {sum(sa)} + {sum(sb)} bytes, ring {ring}, {o}, skew {skew}, "
          f"{switches} switches", flush=True)
    run_case(nx, oracle, sa, sb, ring, nx.Opts(**o), seed=50 + seed, skew=skew, switches=switches)


def test_link_peak_probe_is_plausible(nx):
    """nixie_link_peak (the roofline's denominator): every figure is a rate this link can have, one direction
    alone is never slower than the same direction with the other one busy, and bad arguments are refused."""
    p = nx.link_peak(64 * MiB, 2)
    for k in ("sdma_d2h", "sdma_h2d", "sdma_d2h_both", "sdma_h2d_both", "kernel_d2h", "kernel_h2d", "kernel_d2h_both",
              "kernel_h2d_both"):
        assert 5.0 < p[k] < 70.0, (k, p)
    assert p["sdma_d2h_both"] <= 1.05 * p["sdma_d2h"] and p["sdma_h2d_both"] <= 1.05 * p["sdma_h2d"], p
    for bad in ((1 << 20) - 16, (1 << 20) + 8):
        with pytest.raises(nx.NixieError) as e:
            nx.link_peak(bad, 1)
        assert e.value.code == nx.EINVAL
    with pytest.raises(nx.NixieError):
        nx.link_peak(1 << 20, 0)


@pytest.mark.parametrize("slots,threads", [(1024, 4), (640, 3), (2048, 1)])
def test_more_slots_than_the_pump_keeps_in_registers(nx, oracle, slots, threads):
    """A direction with more than 256 slots: the pump wave keeps the last-seen flag values of the first 256 in
    registers and the others in device memory.  4 KiB slots, several turns of the ring, both directions; then
    one direction alone with all the slots."""
    slot = 4 * KiB
    sizes_a = [700 * slot + 1, 3, 555 * slot, 17 * slot - 9] + [slot + 1] * 40
    sizes_b = [900 * slot - 5, slot, 311 * slot + 77] + [3 * slot - 1] * 30
    o = nx.Opts(slot_bytes=slot, drain_threads=threads, fill_threads=threads)
    info, st = run_case(nx, oracle, sizes_a, sizes_b, slots * slot, o, seed=91, switches=2)
    assert info["out_slots"] == slots // 2 and info["in_slots"] == slots // 2 and info["out_slots"] > 256
    info, st = run_case(nx, oracle, sizes_a, [], slots * slot, o, seed=92)
    assert info["out_slots"] == slots and info["in_slots"] == 0
    info, st = run_case(nx, oracle, [], sizes_b, slots * slot, o, seed=93)
    assert info["in_slots"] == slots


@pytest.mark.parametrize("mask", [0x01, 0xAA, 0xF0, 0xFF])
def test_workgroups_restricted_to_some_xcds(nx, oracle, mask):
    """xcd_mask (a tuning aid): workgroups that land on an XCD outside the mask leave at once, the others do
    all the work; 64 + 64 + 16 workgroups are dealt over the 8 XCDs, so every mask keeps some."""
    sizes_a = [5 * S + 1, 300, 2 * S, 11 * S + 17, 7]
    sizes_b = [4 * S, 11, 6 * S + 9, 200000, 3 * S - 5]
    o = nx.Opts(slot_bytes=S, gather_wgs=64, scatter_wgs=64, flex_wgs=16, xcd_mask=mask, timeout_ms=5000)
    run_case(nx, oracle, sizes_a, sizes_b, 8 * S, o, seed=70 + mask % 7)


def test_ring_only_diagnostic_mode_completes(nx):
    """NIXIE_DIAG_RING_ONLY (measurement: the host threads recycle credits without touching pageable memory):
    the switch completes and reports its figures; the incoming bytes are whatever the ring held."""
    from tests.gpu_helpers import GpuSet
    gA, gB = GpuSet([20 * S + 3, 77], 1, "dev"), GpuSet([9 * S, 5], 2, "host")
    plan = nx.Plan(gA.rows(), gB.rows(), 8 * S, nx.Opts(slot_bytes=S, flags=nx.DIAG_RING_ONLY))
    st = plan.switch()
    assert st["bytes_out"] == 20 * S + 80 and st["bytes_in"] == 9 * S + 5 and st["kernels"] == 1
    assert st["ns_total"] > 0 and st["gpu_status"] == 0
    plan.close()
