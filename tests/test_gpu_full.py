"""Full-size parity on the GPU: the five benchmark configs at their real sizes, in the launch
configuration bench.py times.

The oracle cannot move 17-24 GiB in test time, so it is applied to a sample of allocations
(first, last, smallest, largest and seeded random picks): for each sampled allocation the
oracle's direct definition produces the expected destination bytes and its hash, which are
compared bit for bit with what nixie_switch left.  On top of that every destination arena is
compared whole against its (untouched) source arena, red zones included, and nixie_verify
checks all per-allocation hashes against the pre-switch snapshot."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu
MiB, GiB = 1 << 20, 1 << 30


@pytest.fixture(scope="module")
def nx():
    import torch
    assert torch.cuda.is_available()
    import paper_2601_11743_amd as nx
    nx.lib()
    return nx


def sample_indices(sizes, seed, n_random=16, cap_bytes=1200 * MiB):
    order = np.argsort(sizes)
    picks = {0, len(sizes) - 1, int(order[0]), int(order[-1]), int(order[len(order) // 2])}
    rng = np.random.default_rng(seed)
    picks.update(int(i) for i in rng.integers(0, len(sizes), size=n_random))
    out, acc = [], 0
    for i in sorted(picks, key=lambda i: sizes[i]):
        if acc + sizes[i] > cap_bytes and out:
            continue
        out.append(i)
        acc += sizes[i]
    return sorted(out)


def oracle_expectation(oracle, S, idx, src_side):
    """Oracle's direct definition on the sampled allocations of set S: returns the destination
    bytes it produces and the oracle hash of each."""
    pairs, dst = [], []
    for i in idx:
        if src_side == "dev":
            src = S.dev_view(i).cpu().numpy().copy()
            d = np.zeros_like(src)
            pairs.append((src, d))        # (dev stand-in, host stand-in)
        else:
            src = S.host_view(i).copy()
            d = np.zeros_like(src)
            pairs.append((d, src))
        dst.append(d)
    if src_side == "dev":
        oracle.switch_direct(pairs, [])
    else:
        oracle.switch_direct([], pairs)
    return dst, [oracle.hash64(d) for d in dst]


def full_case(nx, oracle, cfg, ring, round_trips=0, opts_kw=None):
    import torch
    from workloads.device import BigSet
    cf = W.config(cfg)
    A = BigSet(cf["A"], cf["seed_A"], "dev", cf["content"])
    B = BigSet(cf["B"], cf["seed_B"], "host", cf["content"])
    ia, ib = sample_indices(A.sizes, 1), sample_indices(B.sizes, 2)
    exp_a, hash_a = oracle_expectation(oracle, A, ia, "dev")
    exp_b, hash_b = oracle_expectation(oracle, B, ib, "host")
    opts = nx.Opts(slot_bytes=cf["slot_bytes"] or 0, **(opts_kw or {}))
    plan = nx.Plan(A.rows(), B.rows(), ring, opts)
    info = plan.info()
    assert info["pinned_ring_bytes"] <= ring
    assert info["bytes_out"] == A.total_bytes and info["bytes_in"] == B.total_bytes
    h_out, h_in = plan.hash_tables()
    assert [int(h_out[i]) for i in ia] == hash_a, "GPU hash kernel differs from the oracle hash"
    assert [int(h_in[i]) for i in ib] == hash_b, "host hash differs from the oracle hash"

    st = plan.switch()
    for i, e in zip(ia, exp_a):
        assert np.array_equal(A.host_view(i), e), f"evicted allocation {i} differs from the oracle"
    for i, e in zip(ib, exp_b):
        assert np.array_equal(B.dev_view(i).cpu().numpy(), e), f"restored allocation {i} differs from the oracle"
    assert A.arenas_equal(), "evicted set: pageable arena differs from the HBM source arena"
    assert B.arenas_equal(), "restored set: HBM arena differs from the pageable source arena"
    rep = plan.verify(h_out, h_in)
    assert rep["checked_out"] == len(A.sizes) and rep["checked_in"] == len(B.sizes)

    if round_trips:
        back = nx.Plan(B.rows(), A.rows(), ring, opts)
        for t in range(round_trips):
            # sources are "don't care" after a switch: overwrite them before the way back
            for S, side in ((A, "dev"), (B, "host")):
                for i in (0, len(S.sizes) - 1):
                    (S.dev_view(i) if side == "dev" else S.host_view(i))[:] = 0x11
            back.switch()                      # B out to host, A back into HBM
            back.verify(h_in, h_out)
            for i, e in zip(ia, exp_a):
                assert np.array_equal(A.dev_view(i).cpu().numpy(), e)
            for i, e in zip(ib, exp_b):
                assert np.array_equal(B.host_view(i), e)
            for S, side in ((A, "host"), (B, "dev")):
                for i in (0, len(S.sizes) - 1):
                    (S.dev_view(i) if side == "dev" else S.host_view(i))[:] = 0x22
            plan.switch()                      # and forth again
            plan.verify(h_out, h_in)
        back.close()
        for i, e in zip(ia, exp_a):
            assert np.array_equal(A.host_view(i), e)
        for i, e in zip(ib, exp_b):
            assert np.array_equal(B.dev_view(i).cpu().numpy(), e)
    plan.close()
    del A, B
    torch.cuda.empty_cache()
    return info, st


def test_config2_llm_full(nx, oracle):
    info, st = full_case(nx, oracle, 2, 256 * MiB)
    assert info["slot_bytes"] == 4 * MiB and info["out_slots"] == 32 and info["in_slots"] == 32
    print(f"\nconfig 2: {st['ns_total'] / 1e6:.1f} ms, out {st['bytes_out'] / st['ns_out_done']:.1f} GB/s, "
          f"in {st['bytes_in'] / st['ns_in_done']:.1f} GB/s")


def test_config3_asymmetric_full(nx, oracle):
    info, st = full_case(nx, oracle, 3, 128 * MiB)
    assert st["ns_in_done"] < st["ns_out_done"]        # 6 GiB in is ready long before 20 GiB are out
    info, st = full_case(nx, oracle, 3, 128 * MiB, opts_kw=dict(flags=nx.SPLIT_BY_BYTES, order=nx.ORDER_LARGE_FIRST))


def test_config4_fragmented_full(nx, oracle):
    info, st = full_case(nx, oracle, 4, 64 * MiB)
    assert info["segments_out"] >= 100_000
    print(f"\nconfig 4: {st['ns_total'] / 1e6:.1f} ms, {info['segments_out']} segments out")


def test_config6_the_metric_taken_literally_full(nx, oracle):
    """Exactly 16 GiB out and 16 GiB in (64 x 256 MiB each) through the 256 MiB ring in 4 MiB slots."""
    info, st = full_case(nx, oracle, 6, 256 * MiB)
    assert info["bytes_out"] == 16 * GiB and info["bytes_in"] == 16 * GiB
    assert info["slot_bytes"] == 4 * MiB and info["pinned_ring_bytes"] == 256 * MiB


@pytest.mark.parametrize("ring_mib", [16, 64, 256, 1024])
def test_config5_pingpong_full(nx, oracle, ring_mib):
    info, st = full_case(nx, oracle, 5, ring_mib * MiB, round_trips=1)
    assert info["pinned_ring_bytes"] <= ring_mib * MiB


def test_config2_in_place_full(nx, oracle):
    """In-place switch at full size: B is restored into the very HBM that A is evicted from (one
    17 GiB arena instead of two), then A comes back the same way."""
    import torch
    from workloads.device import BigSet
    cf = W.config(2)
    A = BigSet(cf["A"], cf["seed_A"], "dev", cf["content"])
    B = BigSet(cf["B"], cf["seed_B"], "host", cf["content"], share_dev=A)
    torch.cuda.empty_cache()
    ia, ib = sample_indices(A.sizes, 1), sample_indices(B.sizes, 2)
    exp_a, hash_a = oracle_expectation(oracle, A, ia, "dev")
    exp_b, hash_b = oracle_expectation(oracle, B, ib, "host")
    opts = nx.Opts(slot_bytes=cf["slot_bytes"], flags=nx.IN_PLACE)
    with pytest.raises(nx.NixieError):
        nx.Plan(A.rows_np(), B.rows_np(), 256 * MiB, nx.Opts(slot_bytes=cf["slot_bytes"]))
    fwd = nx.Plan(A.rows_np(), B.rows_np(), 256 * MiB, opts)
    back = nx.Plan(B.rows_np(), A.rows_np(), 256 * MiB, opts)
    h_a, h_b = fwd.hash_tables()
    assert [int(h_a[i]) for i in ia] == hash_a and [int(h_b[i]) for i in ib] == hash_b
    st = fwd.switch()
    for i, e in zip(ia, exp_a):
        assert np.array_equal(A.host_view(i), e), f"evicted allocation {i} differs from the oracle"
    for i, e in zip(ib, exp_b):
        assert np.array_equal(B.dev_view(i).cpu().numpy(), e), f"restored allocation {i} differs from the oracle"
    assert B.arenas_equal(), "HBM arena differs from B's pageable arena"
    fwd.verify(h_a, h_b)
    print(f"\nin-place config 2: {st['ns_total'] / 1e6:.1f} ms, out {st['bytes_out'] / st['ns_out_done']:.1f} GB/s, "
          f"in {st['bytes_in'] / st['ns_in_done']:.1f} GB/s")
    for i in (0, len(B.sizes) - 1):
        B.host_view(i)[:] = 0x33                      # sources are don't-care
    back.switch()                                     # B out, A back in, same HBM
    back.verify(h_b, h_a)
    for i, e in zip(ia, exp_a):
        assert np.array_equal(A.dev_view(i).cpu().numpy(), e)
    for i, e in zip(ib, exp_b):
        assert np.array_equal(B.host_view(i), e)
    fwd.close(); back.close()


def test_allocation_larger_than_4gib(nx, oracle):
    """One 5 GiB + 3 B allocation each way: offsets beyond 32 bits in the planner, the copy kernels
    and the hash kernel.  The oracle's direct definition runs on the whole thing."""
    import torch
    from workloads.device import BigSet
    n = 5 * GiB + 3
    A = BigSet([("a", n), ("a2", 4097)], 11, "dev", "splitmix")
    B = BigSet([("b", n), ("b2", 17)], 12, "host", "splitmix")
    src_a = [A.dev_view(i).cpu().numpy().copy() for i in range(2)]
    src_b = [B.host_view(i).copy() for i in range(2)]
    exp_a = [np.zeros_like(x) for x in src_a]
    exp_b = [np.zeros_like(x) for x in src_b]
    oracle.switch_direct(list(zip(src_a, exp_a)), list(zip(exp_b, src_b)))
    plan = nx.Plan(A.rows_np(), B.rows_np(), 64 * MiB)
    h_out, h_in = plan.hash_tables()
    assert int(h_out[1]) == oracle.hash64(src_a[1]) and int(h_in[1]) == oracle.hash64(src_b[1])
    plan.switch()
    for i in range(2):
        assert np.array_equal(A.host_view(i), exp_a[i]), f"evicted allocation {i}"
        assert np.array_equal(B.dev_view(i).cpu().numpy(), exp_b[i]), f"restored allocation {i}"
    assert A.arenas_equal() and B.arenas_equal()
    plan.verify(h_out, h_in)
    # the big hashes against an independent evaluation of the same definition on sampled words is
    # not possible (the hash is a sum over all words), so compare GPU hash and host hash of equal bytes
    h_host = nx.hash_buffers([A.host.ctypes.data + A.layout.offsets[0]], [n], on_device=False)
    assert int(h_host[0]) == int(h_out[0])
    plan.close()
    del A, B
    torch.cuda.empty_cache()


def test_largest_slot(nx, oracle):
    """The largest slot the planner accepts (1 GiB), two per direction: a chunk of 2^30 bytes, a team capped
    at 256 workgroups with 4 MiB units, slot offsets up to the 32-bit limit of a segment."""
    import torch
    from workloads.device import BigSet
    A = BigSet([("a", 2 * GiB + GiB // 2 + 5), ("a2", 100)], 21, "dev", "splitmix")
    B = BigSet([("b", GiB + 5), ("b2", 3 * MiB + 1)], 22, "host", "splitmix")
    src_a = [A.dev_view(i).cpu().numpy().copy() for i in range(2)]
    src_b = [B.host_view(i).copy() for i in range(2)]
    exp_a = [np.zeros_like(x) for x in src_a]
    exp_b = [np.zeros_like(x) for x in src_b]
    oracle.switch_direct(list(zip(src_a, exp_a)), list(zip(exp_b, src_b)))
    plan = nx.Plan(A.rows_np(), B.rows_np(), 4 * GiB, nx.Opts(slot_bytes=GiB))
    info = plan.info()
    assert info["slot_bytes"] == GiB and info["out_slots"] == 2 and info["in_slots"] == 2
    assert info["team_out"] == 256 and info["chunks_out"] == 3 and info["chunks_in"] == 2
    h_out, h_in = plan.hash_tables()
    plan.switch()
    for i in range(2):
        assert np.array_equal(A.host_view(i), exp_a[i]), f"evicted allocation {i}"
        assert np.array_equal(B.dev_view(i).cpu().numpy(), exp_b[i]), f"restored allocation {i}"
    assert A.arenas_equal() and B.arenas_equal()
    plan.verify(h_out, h_in)
    with pytest.raises(nx.NixieError) as e:
        nx.Plan(A.rows_np(), B.rows_np(), 8 * GiB, nx.Opts(slot_bytes=2 * GiB))       # beyond the largest slot
    assert e.value.code == nx.EINVAL
    plan.close()
    del A, B
    torch.cuda.empty_cache()


def test_pingpong_stress_small_ring(nx, oracle):
    """Twelve back-to-back switches A<->B of a 2 GiB-class pair through a 16 MiB ring, whole-arena
    compare after every one: the flag / slot protocol is exercised ~400k times."""
    import torch
    from workloads.device import BigSet
    cf = W.config(5, scale=1 / 12)
    A = BigSet(cf["A"], cf["seed_A"], "dev", cf["content"])
    B = BigSet(cf["B"], cf["seed_B"], "host", cf["content"])
    fwd = nx.Plan(A.rows_np(), B.rows_np(), 16 * MiB)
    back = nx.Plan(B.rows_np(), A.rows_np(), 16 * MiB)
    h_a, h_b = fwd.hash_tables()
    ia = sample_indices(A.sizes, 3, cap_bytes=256 * MiB)
    exp_a, hash_a = oracle_expectation(oracle, A, ia, "dev")
    assert [int(h_a[i]) for i in ia] == hash_a
    for t in range(12):
        if t % 2 == 0:
            fwd.switch()
            fwd.verify(h_a, h_b)
            assert A.arenas_equal() and B.arenas_equal()
            A.dev_view(0)[:] = t + 1              # A's device copy is dead now: scribble on it
            A.dev_view(len(A.sizes) - 1)[:] = t + 1
            B.host_view(0)[:] = t + 1
            B.host_view(len(B.sizes) - 1)[:] = t + 1
        else:
            back.switch()
            back.verify(h_b, h_a)
            assert A.arenas_equal() and B.arenas_equal()
            for i, e in zip(ia, exp_a):
                assert np.array_equal(A.dev_view(i).cpu().numpy(), e)
            A.host_view(0)[:] = t + 1
            A.host_view(len(A.sizes) - 1)[:] = t + 1
            B.dev_view(0)[:] = t + 1
            B.dev_view(len(B.sizes) - 1)[:] = t + 1
    fwd.close(); back.close()
    del A, B
    torch.cuda.empty_cache()


def test_scheduler_drives_the_swaps(nx, oracle):
    """The two halves together: the scheduler's decisions (a scripted trace in simulated time:
    one batch application, two interactive ones) select which nixie_switch runs; after every
    switch the new owner's working set must be in HBM and the evicted one in pageable memory,
    checked by the per-allocation hashes taken at the start."""
    import torch
    from workloads.device import BigSet
    SEC, MS = 1_000_000_000, 1_000_000
    sizes = [W.log_uniform_sizes(40 + i, 24, 256 << 10, 8 << 20, 16) for i in range(3)]
    sets = [BigSet(sz, 50 + i, "host", "bf16_normal") for i, sz in enumerate(sizes)]
    ref = [nx.hash_buffers([r[1] for r in s.rows()], s.sizes, on_device=False) for s in sets]   # all start in pageable memory
    for i, s in enumerate(sets):                       # oracle hash on a sample pins the library's host hash
        assert int(ref[i][3]) == oracle.hash64(s.host_view(3))
    sched = nx.Sched()
    apps = [sched.add_app(0) for _ in sets]
    plans = {}

    def do_switch(evict, run):
        key = (evict, run)
        if key not in plans:
            plans[key] = nx.Plan(sets[evict].rows_np() if evict >= 0 else [], sets[run].rows_np(), 32 * MiB)
        plans[key].switch()
        plans[key].verify(ref[evict] if evict >= 0 else None, ref[run])
        if evict >= 0:
            sets[evict].dev[:] = 0xEE                    # its HBM is dead now

    # script: (time, app that is active in the 250 ms before the tick, apps that ask for the GPU)
    t, owner, log = 0, -1, []
    script = ([(0, [0])] + [(0, [])] * 8 + [(0, [1])] + [(1, [])] + [(1, [0])] * 1 + [(-1, [])] * 2 +
              [(0, [2])] + [(2, [])] + [(2, [0, 1])] + [(-1, [])] * 3)
    for active, asking in script:
        t += 250 * MS
        if active >= 0 and active == owner:
            for k in range(1, 26):
                sched.api_return(active, t - 250 * MS + k * 10 * MS)
        for a in asking:
            sched.request(a, t - 5 * MS)
        d = sched.tick(t)
        if d["switched"]:
            do_switch(d["evict"], d["run"])
            log.append((d["evict"], d["run"]))
        owner = d["run"]
    assert len(log) >= 5 and log[0] == (-1, 0)
    assert (0, 1) in log and any(e == 1 and r == 0 for e, r in log)      # the interactive one got in and the batch one came back
    for p in plans.values():
        p.close()
    sched.close()
    del sets
    torch.cuda.empty_cache()


def test_config2_between_two_spaces_full(nx, oracle):
    """Config 2 at full size, A and B each in an address space of their own over ONE 17 GiB pool of
    physical memory: map B, switch in place, unmap A; and the way back."""
    import torch
    from workloads.device import BigSet, device_view
    cf = W.config(2)
    sizes = [s[1] for s in cf["A"]]
    pool = nx.Pool(W.make_layout(sizes, redzone=256).total, 0)
    sp_a, sp_b = nx.Space(pool), nx.Space(pool)
    sp_a.map()
    sp_b.map()
    A = BigSet(cf["A"], cf["seed_A"], "dev", cf["content"], dev_arena=device_view(sp_a.base, pool.bytes))
    B = BigSet(cf["B"], cf["seed_B"], "host", cf["content"], dev_arena=device_view(sp_b.base, pool.bytes))
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    sp_b.unmap()
    ia, ib = sample_indices(A.sizes, 1), sample_indices(B.sizes, 2)
    exp_a, hash_a = oracle_expectation(oracle, A, ia, "dev")
    exp_b, hash_b = oracle_expectation(oracle, B, ib, "host")
    opts = nx.Opts(slot_bytes=cf["slot_bytes"], flags=nx.IN_PLACE)
    fwd = nx.Plan(A.rows_np(), B.rows_np(), 256 * MiB, opts)
    back = nx.Plan(B.rows_np(), A.rows_np(), 256 * MiB, opts)
    h_a, h_b = fwd.hash_tables()
    assert [int(h_a[i]) for i in ia] == hash_a and [int(h_b[i]) for i in ib] == hash_b
    assert fwd.switch(check=False)["rc"] == nx.EUNMAPPED          # B's addresses have no memory yet
    sp_b.map()
    st = fwd.switch()
    sp_a.unmap()
    for i, e in zip(ia, exp_a):
        assert np.array_equal(A.host_view(i), e), f"evicted allocation {i} differs from the oracle"
    for i, e in zip(ib, exp_b):
        assert np.array_equal(B.dev_view(i).cpu().numpy(), e), f"restored allocation {i} differs from the oracle"
    assert B.arenas_equal(), "pool seen through B's space differs from B's pageable arena"
    fwd.verify(h_a, h_b)
    print(f"\nconfig 2 between two spaces: {st['ns_total'] / 1e6:.1f} ms")
    sp_a.map()
    back.switch()
    sp_b.unmap()
    back.verify(h_b, h_a)
    for i, e in zip(ia, exp_a):
        assert np.array_equal(A.dev_view(i).cpu().numpy(), e)
    assert A.arenas_equal()
    fwd.close(); back.close()
    del A, B
    sp_a.close(); sp_b.close(); pool.close()


def test_config2_pinned_tier_full(nx, oracle):
    """Config 2 at full size with the host side of both working sets in the registered pinned tier:
    no ring, no host threads, every chunk direct."""
    import torch
    from workloads.device import BigSet
    cf = W.config(2)
    A = BigSet(cf["A"], cf["seed_A"], "dev", cf["content"], pinned_host=True)
    B = BigSet(cf["B"], cf["seed_B"], "host", cf["content"], pinned_host=True)
    nx.tier_register(A.host.ctypes.data, A.host.size)
    nx.tier_register(B.host.ctypes.data, B.host.size)
    try:
        ia, ib = sample_indices(A.sizes, 1), sample_indices(B.sizes, 2)
        exp_a, hash_a = oracle_expectation(oracle, A, ia, "dev")
        exp_b, hash_b = oracle_expectation(oracle, B, ib, "host")
        plan = nx.Plan(A.rows_np(), B.rows_np(), 0)
        info = plan.info()
        assert info["pinned_ring_bytes"] == 0 and info["drain_threads"] == 0 and info["fill_threads"] == 0
        assert info["direct_bytes_out"] == A.total_bytes and info["direct_bytes_in"] == B.total_bytes
        h_a, h_b = plan.hash_tables()
        assert [int(h_a[i]) for i in ia] == hash_a and [int(h_b[i]) for i in ib] == hash_b
        st = plan.switch()
        for i, e in zip(ia, exp_a):
            assert np.array_equal(A.host_view(i), e), f"evicted allocation {i} differs from the oracle"
        for i, e in zip(ib, exp_b):
            assert np.array_equal(B.dev_view(i).cpu().numpy(), e), f"restored allocation {i} differs from the oracle"
        assert A.arenas_equal() and B.arenas_equal()
        plan.verify(h_a, h_b)
        print(f"\nconfig 2, pinned tier both sides: {st['ns_total'] / 1e6:.1f} ms")
        plan.close()
    finally:
        nx.tier_unregister(A.host.ctypes.data)
        nx.tier_unregister(B.host.ctypes.data)
    del A, B
    torch.cuda.empty_cache()
