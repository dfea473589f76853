"""GPU parity for switches between two applications that keep their own device addresses over one
pool of physical memory (paper, "Maintaining consistent virtual memory addresses").

The oracle's model of shared physical memory is one arena that both tables point into; on the GPU
the two tables point into two different reserved address ranges that map the same pool blocks.
Results must agree bit for bit, and every use of an unmapped range must be refused on the host."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu

KiB, MiB = 1 << 10, 1 << 20
S = 64 * KiB
BLOCK = 2 * MiB

CASES = [
    ([5 * S + 1, 300, 2 * S, 9 * S + 77], [4 * S, 11, 3 * S + 9, 7 * S], 0),
    ([3 * S, 3 * S, 3 * S, 3 * S], [3 * S, 3 * S, 3 * S, 3 * S], 0),
    ([20 * S + 5, 999, 13 * S, 40 * S + 3], [17 * S, 4, 15 * S + 1, 38 * S], 256),
    ([4 * S], [100, 200, 6 * S], 3 * S),
]


@pytest.fixture(scope="module")
def nx():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2601_11743_amd as nx
    nx.lib()
    return nx


@pytest.fixture(scope="module")
def raw(nx):
    from tests.gpu_helpers import RawDevice
    return RawDevice(nx.lib_path())


def rows(base, ldev, host, lhost, sizes):
    return [(base + od, host.ctypes.data + oh, b) for od, oh, b in zip(ldev.offsets, lhost.offsets, sizes)]


def test_two_spaces_share_the_pool(nx, raw):
    pool = nx.Pool(3 * BLOCK + 5, BLOCK)
    assert pool.bytes == 4 * BLOCK and pool.block_bytes == BLOCK
    a, b = nx.Space(pool), nx.Space(pool)
    assert a.base != b.base and not a.mapped() and not b.mapped()
    a.map()
    b.map(BLOCK, 2 * BLOCK)
    assert a.mapped() and not b.mapped() and b.mapped(BLOCK, 2 * BLOCK) and not b.mapped(0, BLOCK)
    img = W.content_bytes(5, 0, 2 * BLOCK)
    raw.upload(a.base + BLOCK, img)
    assert np.array_equal(raw.download(b.base + BLOCK, 2 * BLOCK), img)      # same bytes, other address
    # device hashes see the same content through either address
    h = nx.hash_buffers([a.base + BLOCK, b.base + BLOCK], [2 * BLOCK, 2 * BLOCK], True)
    assert h[0] == h[1]
    a.map()                                      # mapping mapped blocks is not an error
    b.unmap(BLOCK, BLOCK)
    assert not b.mapped(BLOCK, 2 * BLOCK) and b.mapped(2 * BLOCK, BLOCK)
    with pytest.raises(nx.NixieError) as e:
        nx.hash_buffers([b.base + BLOCK], [64], True)            # refused on the host, never launched
    assert e.value.code == nx.EUNMAPPED
    for bad in [(1, BLOCK), (0, BLOCK + 1), (4 * BLOCK, BLOCK)]:
        with pytest.raises(nx.NixieError) as e:
            a.map(*bad)
        assert e.value.code == nx.EINVAL
    with pytest.raises(nx.NixieError) as e:
        pool.close()
    assert e.value.code == nx.EBUSY
    b.close()
    a.close()
    pool.close()


@pytest.mark.parametrize("case", range(len(CASES)))
def test_switch_there_and_back_between_spaces(nx, oracle, raw, case):
    from tests.helpers import AliasedPair
    from tests.gpu_helpers import first_diff
    sa, sb, shift = CASES[case]
    mk = lambda: AliasedPair(sa, sb, 47, shift_b=shift, skew_a=case % 3, skew_b=(case * 5) % 16)
    ref, g = mk(), mk()
    h_a = oracle.hash_table(ref.pairs_a(), "dev")
    h_b = oracle.hash_table(ref.pairs_b(), "host")
    oracle.switch_direct(ref.pairs_a(), ref.pairs_b())           # A out, then B in, in one arena
    ref.check()
    dev_after_b = ref.dev.copy()
    oracle.switch_direct(ref.pairs_b(), ref.pairs_a())           # and back: B out, then A in
    dev_after_a = ref.dev.copy()

    pool = nx.Pool(g.dev.size, BLOCK)
    sp_a, sp_b = nx.Space(pool), nx.Space(pool)
    sp_a.map()
    raw.upload(sp_a.base, g.dev)
    rows_a = rows(sp_a.base, g.la, g.host_a, g.lha, g.sizes_a)
    rows_b = rows(sp_b.base, g.lb, g.host_b, g.lhb, g.sizes_b)
    opts = nx.Opts(slot_bytes=S, flags=nx.IN_PLACE)
    ring = 8 * S

    # B's addresses are reserved but nothing is behind them yet: planning is fine, switching is not
    plan_ab = nx.Plan(rows_a, rows_b, ring, opts)
    assert plan_ab.switch(check=False)["rc"] == nx.EUNMAPPED
    assert np.array_equal(raw.download(sp_a.base, g.dev.size), g.dev)        # nothing was touched
    sp_b.map()
    with pytest.raises(nx.NixieError) as e:
        nx.Plan(rows_a, rows_b, ring, nx.Opts(slot_bytes=S))     # shared blocks without NIXIE_IN_PLACE
    assert e.value.code == nx.EOVERLAP
    lay = nx.Layout(rows_a, rows_b, ring, opts)
    deps = lay.chunks(1)["dep_out"]
    assert deps.max() > 0, "dependencies must be found although the addresses differ"
    lay.close()

    h_out, h_in = plan_ab.hash_tables()
    assert np.array_equal(h_out, h_a) and np.array_equal(h_in, h_b)
    plan_ab.switch_begin()
    for call in (sp_a.unmap, sp_b.map, lambda: sp_b.assign(0, [0])):
        with pytest.raises(nx.NixieError) as e:
            call()                                               # nothing is remapped while a switch is running
        assert e.value.code == nx.EBUSY
    plan_ab.switch_end()
    sp_a.unmap()                                                 # A keeps its addresses, nothing behind them
    got = raw.download(sp_b.base, g.dev.size)
    assert np.array_equal(got, dev_after_b), "pool after A->B: " + first_diff(got, dev_after_b)
    exp_host_a = g.expected_host_a()
    assert np.array_equal(g.host_a, exp_host_a), "evicted A: " + first_diff(g.host_a, exp_host_a)
    plan_ab.verify(h_a, h_b)
    with pytest.raises(nx.NixieError) as e:
        plan_ab.hash_tables()                                    # would read A's unmapped addresses
    assert e.value.code == nx.EUNMAPPED
    assert plan_ab.switch(check=False)["rc"] == nx.EUNMAPPED

    # the way back: A's old pointers become valid again, holding A's old bytes
    plan_ba = nx.Plan(rows_b, rows_a, ring, opts)
    sp_a.map()
    plan_ba.switch()
    sp_b.unmap()
    got = raw.download(sp_a.base, g.dev.size)
    assert np.array_equal(got, dev_after_a), "pool after B->A: " + first_diff(got, dev_after_a)
    assert np.array_equal(g.host_b, ref.host_b), "evicted B: " + first_diff(g.host_b, ref.host_b)
    plan_ba.verify(h_b, h_a)
    for i, (o, b) in enumerate(zip(g.la.offsets, g.sizes_a)):    # A is back where its pointers say
        assert np.array_equal(got[o:o + b], W.content_bytes(47, i, b))

    plan_ab.close()
    plan_ba.close()
    sp_a.close()
    sp_b.close()
    pool.close()


def test_disjoint_blocks_need_no_in_place_flag(nx, oracle, raw):
    """Two spaces over one pool whose tables use different blocks share nothing: an ordinary switch."""
    from tests.helpers import HostSet
    from tests.gpu_helpers import first_diff
    sizes_a, sizes_b = [3 * S + 5, 700, 9 * S], [2 * S, 6 * S + 1, 90]
    rA, rB = HostSet(sizes_a, 3, "dev"), HostSet(sizes_b, 4, "host")
    gA, gB = HostSet(sizes_a, 3, "dev"), HostSet(sizes_b, 4, "host")
    oracle.switch_direct(rA.pairs(), rB.pairs())
    assert max(gA.ldev.total, gB.ldev.total) <= BLOCK
    pool = nx.Pool(2 * BLOCK, BLOCK)
    sp_a, sp_b = nx.Space(pool), nx.Space(pool)
    sp_a.map(0, BLOCK)
    sp_b.map(BLOCK, BLOCK)
    raw.upload(sp_a.base, gA.dev)
    raw.upload(sp_b.base + BLOCK, gB.dev)
    rows_a = rows(sp_a.base, gA.ldev, gA.host, gA.lhost, gA.sizes)
    rows_b = rows(sp_b.base + BLOCK, gB.ldev, gB.host, gB.lhost, gB.sizes)
    plan = nx.Plan(rows_a, rows_b, 8 * S, nx.Opts(slot_bytes=S))
    plan.switch()
    got = raw.download(sp_b.base + BLOCK, gB.dev.size)
    assert np.array_equal(got, rB.dev), "restored set: " + first_diff(got, rB.dev)
    assert np.array_equal(gA.host, rA.host), "evicted set: " + first_diff(gA.host, rA.host)
    plan.close()
    sp_a.close()
    sp_b.close()
    pool.close()


def physical_pairs(phys, offsets, sizes, host, host_offsets, perm):
    """(device piece, host piece) pairs of allocations seen through a space whose block i is pool block
    perm[i]: an allocation that crosses a block boundary is several pieces of the physical arena."""
    pairs = []
    for o, b, oh in zip(offsets, sizes, host_offsets):
        done = 0
        while done < b:
            va = o + done
            take = min(b - done, BLOCK - va % BLOCK)
            p = perm[va // BLOCK] * BLOCK + va % BLOCK
            pairs.append((phys[p:p + take], host[oh + done:oh + done + take]))
            done += take
    return pairs


@pytest.mark.parametrize("perm", [[5, 2, 7, 0, 1, 3, 4, 6], [1, 0, 3, 2, 5, 4, 7, 6], [0, 1, 2, 3, 4, 5, 6, 7]])
def test_switch_with_any_pool_block_behind_any_address(nx, oracle, raw, perm):
    """A sees the pool in order, B sees its blocks permuted: B's allocations are scattered over the
    physical memory and cross block boundaries.  Oracle: one physical arena, B's allocations as the
    pieces they are there; the definition (all of A out, then B in) gives the expected arena."""
    from tests.helpers import HostSet
    from tests.gpu_helpers import first_diff
    sizes_a = [20 * S + 5, 999, 13 * S, 40 * S + 3, 30 * S]          # 6.4 MiB: pool blocks 0..3 through A
    sizes_b = [17 * S, 4, 45 * S + 1, 38 * S, 700]                   # crosses block boundaries of B's space
    n_blocks = len(perm)
    A_ref, B_ref = HostSet(sizes_a, 71, "dev"), HostSet(sizes_b, 72, "host")
    A_gpu, B_gpu = HostSet(sizes_a, 71, "dev"), HostSet(sizes_b, 72, "host")
    assert max(A_ref.ldev.total, B_ref.ldev.total) <= 4 * BLOCK
    ident = list(range(n_blocks))
    phys = np.full(n_blocks * BLOCK, 0xC3, dtype=np.uint8)
    phys[:A_ref.dev.size] = A_ref.dev                                # A is resident, seen in order
    out_pairs = physical_pairs(phys, A_ref.ldev.offsets, sizes_a, A_ref.host, A_ref.lhost.offsets, ident)
    in_pairs = physical_pairs(phys, B_ref.ldev.offsets, sizes_b, B_ref.host, B_ref.lhost.offsets, perm)
    oracle.switch_direct(out_pairs, in_pairs)

    pool = nx.Pool(n_blocks * BLOCK, BLOCK)
    sp_a, sp_b, sp_all = nx.Space(pool), nx.Space(pool), nx.Space(pool)
    sp_b.assign(0, perm)
    sp_a.map(0, 4 * BLOCK)
    sp_all.map()                                                     # an observer that sees the pool in order
    raw.upload(sp_all.base, np.full(n_blocks * BLOCK, 0xC3, dtype=np.uint8))
    raw.upload(sp_a.base, A_gpu.dev)
    rows_a = rows(sp_a.base, A_gpu.ldev, A_gpu.host, A_gpu.lhost, sizes_a)
    rows_b = rows(sp_b.base, B_gpu.ldev, B_gpu.host, B_gpu.lhost, sizes_b)
    opts = nx.Opts(slot_bytes=S, flags=nx.IN_PLACE)
    plan = nx.Plan(rows_a, rows_b, 8 * S, opts)
    assert plan.switch(check=False)["rc"] == nx.EUNMAPPED
    sp_b.map(0, 4 * BLOCK)
    with pytest.raises(nx.NixieError) as e:
        sp_b.assign(0, [perm[1]])                                    # a mapped block keeps what is behind it
    assert e.value.code == nx.EBUSY
    shares = len(set(perm[:4]) & {0, 1, 2, 3})
    if shares:
        with pytest.raises(nx.NixieError) as e:
            nx.Plan(rows_a, rows_b, 8 * S, nx.Opts(slot_bytes=S))
        assert e.value.code == nx.EOVERLAP
    plan.switch()
    got = raw.download(sp_all.base, n_blocks * BLOCK)
    assert np.array_equal(got, phys), "physical memory: " + first_diff(got, phys)
    assert np.array_equal(A_gpu.host, A_ref.host), "evicted A: " + first_diff(A_gpu.host, A_ref.host)
    seen_by_b = raw.download(sp_b.base, B_gpu.ldev.total)            # and B finds its bytes at its own addresses
    for i, (o, b) in enumerate(zip(B_gpu.ldev.offsets, sizes_b)):
        assert np.array_equal(seen_by_b[o:o + b], W.content_bytes(72, i, b)), f"B's allocation {i}"
    # the plan saw one assignment; with another pool block behind a block it needs, it refuses to run
    sp_b.unmap(0, BLOCK)
    spare = next(k for k in range(n_blocks) if k not in perm[:4])
    sp_b.assign(0, [spare])
    sp_b.map(0, BLOCK)
    assert plan.switch(check=False)["rc"] == nx.EUNMAPPED
    plan.close()
    for sp in (sp_a, sp_b, sp_all):
        sp.close()
    pool.close()
