"""The switch in three steps (begin / wait for the incoming application / end): the incoming
application's bytes are complete and visible to other streams at nixie_switch_wait_in, while the
outgoing application is still being evicted.  Parity against the oracle as everywhere."""
import time

import numpy as np
import pytest

from tests.helpers import HostSet, AliasedPair

pytestmark = pytest.mark.gpu

KiB, MiB = 1 << 10, 1 << 20
S = 64 * KiB


@pytest.fixture(scope="module")
def nx():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2601_11743_amd as nx
    nx.lib()
    return nx


def test_incoming_application_is_ready_before_the_eviction_ends(nx, oracle):
    import torch
    from tests.gpu_helpers import GpuSet, first_diff
    sizes_a = [192 * MiB + 5, 128 * MiB, 3 * S + 1, 192 * MiB]        # 512 MiB to evict
    sizes_b = [3 * MiB + 9, 700, 2 * MiB, 11 * S]                    # 6 MiB to restore
    rA, rB = HostSet(sizes_a, 61, "dev"), HostSet(sizes_b, 62, "host")
    oracle.switch_direct(rA.pairs(), rB.pairs())
    gA, gB = GpuSet(sizes_a, 61, "dev"), GpuSet(sizes_b, 62, "host")
    swap_stream, other = torch.cuda.Stream(), torch.cuda.Stream()
    plan = nx.Plan(gA.rows(), gB.rows(), 16 * MiB)
    plan.switch(swap_stream.cuda_stream)                             # warm-up: first-touch, thread start, stream's queue
    for o, b in zip(gA.hs.lhost.offsets, sizes_a):                   # poison again what the warm-up wrote
        gA.hs.host[o:o + b] = 0x5A
    gB.dev_t.copy_(torch.from_numpy(gB.hs.dev))                      # the pre-switch image: B's ranges poisoned
    torch.cuda.synchronize()

    t0 = time.perf_counter()
    plan.switch_begin(swap_stream.cuda_stream)
    with pytest.raises(nx.NixieError) as e:
        plan.switch()                                                # the plan is busy until switch_end
    assert e.value.code == nx.EBUSY
    plan.switch_wait_in()
    t_in = time.perf_counter() - t0
    with torch.cuda.stream(other):                                   # B runs: another stream reads its memory now
        dev_B = gB.dev_t.cpu().numpy()
    st = plan.switch_end()
    t_all = time.perf_counter() - t0
    assert np.array_equal(dev_B, rB.dev), "restored set at wait_in: " + first_diff(dev_B, rB.dev)
    assert np.array_equal(gA.hs.host, rA.host), "evicted set: " + first_diff(gA.hs.host, rA.host)
    assert st["rc"] == 0 and st["bytes_out"] == sum(sizes_a)
    assert 0 < st["ns_in_done"] < st["ns_total"]
    # 6 MiB against 512 MiB: a small fraction of the switch (workgroups that serve either direction must leave
    # the incoming one when its units run out, or this wait lasts until the outgoing units run out too)
    assert t_in < 0.4 * t_all, f"B ready after {t_in * 1e3:.2f} ms of {t_all * 1e3:.2f} ms"
    print(f"B ready after {t_in * 1e3:.2f} ms, switch complete after {t_all * 1e3:.2f} ms")
    # a second time with the same plan, without the early wait
    plan.switch_begin(swap_stream.cuda_stream)
    assert plan.switch_end()["rc"] == 0
    plan.close()


def test_three_step_switch_in_place(nx, oracle):
    import torch
    from tests.gpu_helpers import first_diff
    sa, sb, shift = [20 * S + 5, 999, 13 * S, 40 * S], [17 * S, 4, 15 * S + 1], 256
    ref = AliasedPair(sa, sb, 31, shift_b=shift)
    oracle.switch_direct(ref.pairs_a(), ref.pairs_b())
    g = AliasedPair(sa, sb, 31, shift_b=shift)
    dev_t = torch.from_numpy(g.dev).to("cuda:0")
    base = dev_t.data_ptr()
    rows_a = [(base + od, g.host_a.ctypes.data + oh, b) for od, oh, b in zip(g.la.offsets, g.lha.offsets, g.sizes_a)]
    rows_b = [(base + od, g.host_b.ctypes.data + oh, b) for od, oh, b in zip(g.lb.offsets, g.lhb.offsets, g.sizes_b)]
    swap_stream, other = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    plan = nx.Plan(rows_a, rows_b, 8 * S, nx.Opts(slot_bytes=S, flags=nx.IN_PLACE))
    plan.switch_begin(swap_stream.cuda_stream)
    plan.switch_wait_in()
    with torch.cuda.stream(other):
        dev_now = dev_t.cpu().numpy()
    for i, (o, b) in enumerate(zip(g.lb.offsets, g.sizes_b)):        # B's ranges are final at wait_in
        assert np.array_equal(dev_now[o:o + b], ref.dev[o:o + b]), f"incoming allocation {i} at wait_in"
    plan.switch_end()
    assert np.array_equal(g.host_a, ref.host_a), "evicted set: " + first_diff(g.host_a, ref.host_a)
    assert np.array_equal(dev_t.cpu().numpy(), ref.dev)
    plan.close()


def test_misuse_and_abandoned_switch(nx):
    from tests.gpu_helpers import GpuSet
    gA, gB = GpuSet([40 * S], 1, "dev"), GpuSet([3 * S], 2, "host")
    plan = nx.Plan(gA.rows(), gB.rows(), 4 * S, nx.Opts(slot_bytes=S))
    with pytest.raises(nx.NixieError) as e:
        plan.switch_wait_in()                                        # nothing was begun
    assert e.value.code == nx.EINVAL
    assert plan.switch_end(check=False)["rc"] == nx.EINVAL
    plan.close()
    ser = nx.Plan(gA.rows(), gB.rows(), 4 * S, nx.Opts(slot_bytes=S, flags=nx.SERIALIZE))
    with pytest.raises(nx.NixieError) as e:
        ser.switch_begin()
    assert e.value.code == nx.EINVAL
    ser.close()
    # a switch that is begun and never ended is stopped when its plan is destroyed
    gA2, gB2 = GpuSet([400 * S], 1, "dev"), GpuSet([3 * S], 2, "host")
    plan = nx.Plan(gA2.rows(), gB2.rows(), 4 * S, nx.Opts(slot_bytes=S))
    plan.switch_begin()
    plan.close()
    # and the device is healthy afterwards
    gA3, gB3 = GpuSet([40 * S], 1, "dev"), GpuSet([3 * S], 2, "host")
    plan = nx.Plan(gA3.rows(), gB3.rows(), 4 * S, nx.Opts(slot_bytes=S))
    plan.switch()
    gA3.hs.check_moved()
    plan.close()
