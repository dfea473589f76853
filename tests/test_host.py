"""Host-side logic of libnixie without a GPU: the library loads and exports what the header
declares; the chunk planner's output partitions every allocation exactly; host hashing agrees
with the oracle.  No GPU compute is called here."""
import os
import re

import numpy as np
import pytest

import workloads as W

KiB, MiB, GiB = 1 << 10, 1 << 20, 1 << 30
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def nx():
    import paper_2601_11743_amd as nx
    if not os.path.exists(nx.lib_path()):
        from paper_2601_11743_amd import build
        build.build()
    nx.lib()
    return nx


def test_library_exports_every_declared_symbol(nx):
    header = open(os.path.join(ROOT, "include", "nixie.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(nixie_[a-z0-9_]+)\s*\(", header))
    assert declared == set(nx.DECLARED_SYMBOLS)
    L = nx.lib()
    for name in declared:
        assert getattr(L, name) is not None, name
    assert nx.strerror(0) == "ok" and "overlap" in nx.strerror(nx.EOVERLAP)


def fake_rows(sizes, dev_base=0x7F00_0000_0000, host_base=0x1000_0000_0000, skew_dev=0, skew_host=0, gap=256):
    rows, d, h = [], dev_base, host_base
    for b in sizes:
        d = (d + 255) // 256 * 256 + skew_dev
        h = (h + 255) // 256 * 256 + skew_host
        rows.append((d, h, b))
        d += b + gap
        h += b + gap
    return rows


def check_layout(lay, rows_out, rows_in, ring):
    info = lay.info()
    S = info["slot_bytes"]
    assert (info["out_slots"] + info["in_slots"]) * S == info["pinned_ring_bytes"] <= ring
    for direction, rows in ((0, rows_out), (1, rows_in)):
        ch, sg = lay.chunks(direction), lay.segments(direction)
        total = sum(b for _, _, b in rows)
        assert int(sg["len"].sum()) == total == info["bytes_out" if direction == 0 else "bytes_in"]
        if len(sg) == 0:
            assert len(ch) == 0
            continue
        assert (sg["len"] > 0).all()
        # chunks tile the segment array in order
        assert ch["seg_begin"][0] == 0 and (ch["seg_count"] > 0).all()
        assert np.array_equal(ch["seg_begin"][1:], (ch["seg_begin"] + ch["seg_count"])[:-1])
        assert int(ch["seg_begin"][-1] + ch["seg_count"][-1]) == len(sg)
        # inside a chunk: ascending, non-overlapping slot ranges that fit the slot; alignment congruence
        chunk_of = np.repeat(np.arange(len(ch)), ch["seg_count"])
        end = sg["slot_off"].astype(np.int64) + sg["len"]
        assert (end <= S).all()
        same = chunk_of[1:] == chunk_of[:-1]
        assert (sg["slot_off"][1:][same] >= end[:-1][same]).all()
        assert ((sg["slot_off"].astype(np.uint64) & 15) == (sg["dev_addr"] & 15)).all()
        used = np.zeros(len(ch), dtype=np.int64)
        np.maximum.at(used, chunk_of, end)
        assert np.array_equal(used, ch["used_bytes"].astype(np.int64))
        # segments partition every allocation: sorted by device address they abut exactly
        order = np.argsort(sg["dev_addr"], kind="stable")
        dev, ln, host = sg["dev_addr"][order], sg["len"][order].astype(np.uint64), sg["host_addr"][order]
        ranges = sorted((d, h, b) for d, h, b in rows if b)
        starts = np.array([r[0] for r in ranges], dtype=np.uint64)
        idx = np.searchsorted(starts, dev, side="right") - 1
        a_dev = starts[idx]
        a_host = np.array([r[1] for r in ranges], dtype=np.uint64)[idx]
        a_len = np.array([r[2] for r in ranges], dtype=np.uint64)[idx]
        assert ((dev - a_dev) == (host - a_host)).all()          # same offset on both sides
        assert (dev + ln <= a_dev + a_len).all()
        first = np.r_[True, idx[1:] != idx[:-1]]
        assert (dev[first] == a_dev[first]).all()
        assert (dev[1:][~first[1:]] == (dev + ln)[:-1][~first[1:]]).all()   # pieces abut
        covered = np.zeros(len(ranges), dtype=np.uint64)
        np.add.at(covered, idx, ln)
        assert np.array_equal(covered, np.array([r[2] for r in ranges], dtype=np.uint64))
    return info


@pytest.mark.parametrize("order", [0, 1, 2, 3])
def test_planner_partitions_exactly(nx, order):
    S = 64 * KiB
    sizes_a = [1, 15, 16, 17, 255, 4096, S - 1, S, S + 1, 3 * S + 5, 0, 10 * S + 333, 7]
    sizes_b = [S + 1, 2, 7 * S - 3, 0, 31, 5 * S, 16]
    for skew in ((0, 0), (3, 9), (15, 1)):
        ra = fake_rows(sizes_a, skew_dev=skew[0], skew_host=skew[1])
        rb = fake_rows(sizes_b, dev_base=0x7F80_0000_0000, host_base=0x1800_0000_0000, skew_dev=skew[1], skew_host=skew[0])
        lay = nx.Layout(ra, rb, 8 * S, nx.Opts(slot_bytes=S, order=order))
        info = check_layout(lay, ra, rb, 8 * S)
        assert info["out_slots"] == 4 and info["in_slots"] == 4
        lay.close()


def test_planner_order_modes(nx):
    S = 64 * KiB
    rows = fake_rows([100, 5 * S, 300, 2 * S])
    first_dev = {}
    for order in range(4):
        lay = nx.Layout(rows, [], 8 * S, nx.Opts(slot_bytes=S, order=order))
        first_dev[order] = int(lay.segments(0)["dev_addr"][0])
        lay.close()
    assert first_dev[0] == rows[0][0] and first_dev[3] == rows[3][0]
    assert first_dev[1] == rows[1][0]                 # largest first
    assert first_dev[2] == min(r[0] for r in rows)    # lowest address first


def test_planner_packing_is_dense(nx):
    """Small allocations share slots: 16-byte-aligned pieces waste nothing, so the chunk count is
    ceil(total / slot)."""
    S = 256 * KiB
    sizes = [16 * (1 + (i * 37) % 500) for i in range(4000)]
    rows = fake_rows(sizes, gap=0)
    lay = nx.Layout(rows, [], 16 * S, nx.Opts(slot_bytes=S))
    info = check_layout(lay, rows, [], 16 * S)
    assert info["chunks_out"] == -(-sum(sizes) // S)
    lay.close()


def test_out_slots_must_leave_two_slots_for_the_other_direction(nx):
    """The caller's share for the outgoing direction is an unsigned count: one that exceeds the ring
    must be refused before it is subtracted, or the incoming share wraps round and the pinned
    budget with it (ring 4 MiB in 64 KiB slots = 64 slots)."""
    ra, rb = fake_rows([1 * MiB]), fake_rows([1 * MiB], dev_base=0x7F80_0000_0000, host_base=0x1800_0000_0000)
    for bad in (1, 63, 64, 65, 100, 2**32 - 1):
        with pytest.raises(nx.NixieError) as e:
            nx.Layout(ra, rb, 4 * MiB, nx.Opts(slot_bytes=64 * KiB, out_slots=bad))
        assert e.value.code == nx.EINVAL, bad
    for good in (2, 32, 62):
        lay = nx.Layout(ra, rb, 4 * MiB, nx.Opts(slot_bytes=64 * KiB, out_slots=good))
        i = lay.info()
        assert i["out_slots"] == good and i["in_slots"] == 64 - good
        assert i["pinned_ring_bytes"] == 4 * MiB and i["pinned_ctrl_bytes"] < 64 * KiB
        lay.close()
    # one direction only: the option does not apply, the whole ring serves the staged direction
    lay = nx.Layout(ra, [], 4 * MiB, nx.Opts(slot_bytes=64 * KiB, out_slots=100))
    assert lay.info()["out_slots"] == 64 and lay.info()["in_slots"] == 0
    lay.close()


def test_planner_ring_split_and_defaults(nx):
    ra, rb = fake_rows([20 * MiB]), fake_rows([6 * MiB], dev_base=0x7F80_0000_0000, host_base=0x1800_0000_0000)
    lay = nx.Layout(ra, rb, 512 * MiB)
    i = lay.info()
    assert i["slot_bytes"] == 2 * MiB and i["out_slots"] == 128 and i["in_slots"] == 128
    assert i["team_out"] == 32 and i["gather_wgs"] == 128 and i["scatter_wgs"] == 64   # 64 KiB work units
    lay = nx.Layout(ra, rb, 128 * MiB)                 # about 128 slots per direction
    i = lay.info()
    assert i["slot_bytes"] == 512 * KiB and i["out_slots"] == 128 and i["in_slots"] == 128 and i["team_out"] == 8
    lay = nx.Layout(ra, rb, 128 * MiB, nx.Opts(flags=nx.SPLIT_BY_BYTES))
    i = lay.info()
    assert i["out_slots"] == round(256 * 20 / 26) and i["out_slots"] + i["in_slots"] == 256
    lay = nx.Layout(ra, rb, 128 * MiB, nx.Opts(out_slots=10))
    assert lay.info()["out_slots"] == 10 and lay.info()["in_slots"] == 246
    lay = nx.Layout(ra, [], 128 * MiB)                 # pure evict: the whole ring serves one direction
    i = lay.info()
    assert i["slot_bytes"] == 1 * MiB and i["out_slots"] == 128 and i["in_slots"] == 0 and i["scatter_wgs"] == 0
    lay = nx.Layout(ra, rb, 16 * MiB)                  # small ring: smaller slots and smaller work units
    i = lay.info()
    assert i["slot_bytes"] == 64 * KiB and i["out_slots"] == 128
    assert i["team_out"] == 4                          # 16 KiB units, the floor: one 4 KiB tile per wave
    assert i["gather_wgs"] == 64 and i["scatter_wgs"] == 32   # small ring: one gather workgroup per 128 KiB of a share
    lay = nx.Layout(ra, rb, 4 * MiB)
    assert lay.info()["slot_bytes"] == 64 * KiB and lay.info()["out_slots"] == 32
    lay = nx.Layout(ra, rb, 256 * KiB)
    assert lay.info()["slot_bytes"] == 64 * KiB and lay.info()["out_slots"] == 2
    lay = nx.Layout(ra, rb, 256 * MiB, nx.Opts(slot_bytes=4 * MiB))   # the headline geometry
    i = lay.info()
    assert i["out_slots"] == 32 and i["team_out"] == 64


def test_planner_errors(nx):
    S = 64 * KiB
    rows = fake_rows([5000, 6000])

    def code(fn):
        with pytest.raises(nx.NixieError) as e:
            fn()
        return e.value.code

    assert code(lambda: nx.Layout(rows, [], S, nx.Opts(slot_bytes=S))) == nx.EINVAL          # one slot
    assert code(lambda: nx.Layout(rows, rows, 8 * S, nx.Opts(slot_bytes=S))) == nx.EOVERLAP  # same ranges twice
    assert code(lambda: nx.Layout(rows + [(rows[0][0] + 4999, 0x2000_0000_0000, 2)], [], 8 * S)) == nx.EOVERLAP
    assert code(lambda: nx.Layout(rows + [(0x7F90_0000_0000, rows[1][1] + 5999, 2)], [], 8 * S)) == nx.EOVERLAP
    assert code(lambda: nx.Layout(rows, [], 8 * S, nx.Opts(slot_bytes=1000))) == nx.EINVAL
    assert code(lambda: nx.Layout(rows, [], 8 * S, nx.Opts(order=9))) == nx.EINVAL
    assert code(lambda: nx.Layout([(0, 0x1000, 10)], [], 8 * S)) == nx.EINVAL               # NULL device pointer
    assert code(lambda: nx.Layout(rows, fake_rows([10], dev_base=0x7F80_0000_0000, host_base=0x1800_0000_0000),
                                  3 * S, nx.Opts(slot_bytes=S))) == nx.EINVAL               # < 2 slots per direction
    nx.Layout([(0, 0, 0)], [], 8 * S).close()                                               # empty entries are legal
    # adjacent (touching) ranges are not an overlap
    nx.Layout([(0x7F00_0000_0000, 0x1000_0000_0000, 4096), (0x7F00_0000_1000, 0x1000_0000_1000, 4096)], [], 8 * S).close()


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_planner_on_benchmark_configs(nx, cfg):
    cf = W.config(cfg)
    ra = fake_rows([b for _, b in cf["A"]])
    rb = fake_rows([b for _, b in cf["B"]], dev_base=0x7A00_0000_0000, host_base=0x1A00_0000_0000)
    for ring in cf["ring_bytes"]:
        lay = nx.Layout(ra, rb, ring, nx.Opts(slot_bytes=cf["slot_bytes"] or 0))
        info = check_layout(lay, ra, rb, ring)
        S = info["slot_bytes"]
        # packing keeps slots full: at most one partly filled chunk beyond the dense count per direction
        assert info["chunks_out"] <= -(-info["bytes_out"] // S) + max(1, len(ra) * 15 // S + 1)
        lay.close()


def test_host_hash_matches_oracle(nx, oracle):
    sizes = [0, 1, 7, 8, 9, 4095, 32768, 32769, 100000, 3 * MiB + 5]
    for skew in (0, 3):
        bufs = [np.concatenate([np.zeros(skew, np.uint8), W.content_bytes(5, i, b)])[skew:] for i, b in enumerate(sizes)]
        got = nx.hash_buffers([b.ctypes.data for b in bufs], sizes, on_device=False)
        assert [int(x) for x in got] == [oracle.hash64(b) for b in bufs]


def test_in_place_dependencies(nx):
    """NIXIE_IN_PLACE: every incoming chunk depends on exactly the outgoing chunks whose device
    bytes it overwrites (as a prefix length), and the incoming table is walked in the order its
    GPU memory becomes free."""
    S = 64 * KiB
    rng = np.random.default_rng(4)
    sizes_a = [int(x) for x in rng.integers(1, 5 * S, size=40)]
    sizes_b = [int(x) for x in rng.integers(1, 7 * S, size=25)]
    ra = fake_rows(sizes_a, gap=64)
    rb = fake_rows(sizes_b, host_base=0x1800_0000_0000, gap=192)     # same device base: overlaps A's ranges
    with pytest.raises(nx.NixieError) as e:
        nx.Layout(ra, rb, 16 * S, nx.Opts(slot_bytes=S))
    assert e.value.code == nx.EOVERLAP                                 # aliasing needs the flag
    lay = nx.Layout(ra, rb, 16 * S, nx.Opts(slot_bytes=S, flags=nx.IN_PLACE))
    check_layout(lay, ra, rb, 16 * S)
    co, so, ci, si = lay.chunks(0), lay.segments(0), lay.chunks(1), lay.segments(1)
    assert (co["dep_out"] == 0).all()
    out_chunk_of = np.repeat(np.arange(len(co)), co["seg_count"])
    in_chunk_of = np.repeat(np.arange(len(ci)), ci["seg_count"])
    want = np.zeros(len(ci), dtype=np.int64)
    for q in range(len(si)):                                           # brute force over all segment pairs
        a, b = int(si["dev_addr"][q]), int(si["dev_addr"][q]) + int(si["len"][q])
        hit = (so["dev_addr"].astype(np.int64) < b) & (so["dev_addr"].astype(np.int64) + so["len"] > a)
        if hit.any():
            want[in_chunk_of[q]] = max(want[in_chunk_of[q]], int(out_chunk_of[hit].max()) + 1)
    assert np.array_equal(ci["dep_out"].astype(np.int64), want)
    assert want.max() > 0
    # walked in the order the memory becomes free: dependencies never decrease by more than one allocation's span
    first_dep = [int(want[in_chunk_of[np.flatnonzero(si["dev_addr"] == r[0])[0]]]) for r in rb if r[2]]
    order = np.argsort([int(np.flatnonzero(si["dev_addr"] == r[0])[0]) for r in rb if r[2]])
    alloc_dep = []
    for r in rb:
        a, b = r[0], r[0] + r[2]
        hit = (so["dev_addr"].astype(np.int64) < b) & (so["dev_addr"].astype(np.int64) + so["len"] > a)
        alloc_dep.append(int(out_chunk_of[hit].max()) + 1 if hit.any() else 0)
    walked = [alloc_dep[i] for i in order]
    assert walked == sorted(walked)
    # overlap inside one table is still refused, and so is any host overlap
    with pytest.raises(nx.NixieError):
        nx.Layout(ra + [(ra[0][0] + 1, 0x2000_0000_0000, 2)], rb, 16 * S, nx.Opts(slot_bytes=S, flags=nx.IN_PLACE))
    with pytest.raises(nx.NixieError):
        nx.Layout(ra, [(r[0], ra[0][1], r[2]) for r in rb[:1]], 16 * S, nx.Opts(slot_bytes=S, flags=nx.IN_PLACE))


@pytest.mark.parametrize("order", [0, 1, 2, 3])
def test_in_place_evicts_first_what_the_incoming_table_reuses(nx, order):
    """A large outgoing table, a small incoming one that reuses the GPU memory of the LAST outgoing
    allocations: those are walked first (in the given order among themselves), so the incoming chunks
    depend on a short prefix of the eviction, not on nearly all of it."""
    S = 64 * KiB
    sizes_a = [3 * S + 5] * 40
    ra = fake_rows(sizes_a, gap=64)
    reused = ra[-6:]                                                   # B sits exactly where A's last six allocations are
    rb = [(d, 0x1800_0000_0000 + i * (1 << 24), b - 7) for i, (d, _, b) in enumerate(reused)]
    lay = nx.Layout(ra, rb, 16 * S, nx.Opts(slot_bytes=S, flags=nx.IN_PLACE, order=order))
    check_layout(lay, ra, rb, 16 * S)
    co, so, ci = lay.chunks(0), lay.segments(0), lay.chunks(1)
    n_first = int(np.ceil(6 * (3 * S + 5) / S)) + 1                    # chunks that can hold the six reused allocations
    assert int(ci["dep_out"].max()) <= n_first < len(co) // 4
    first_addrs = {int(a) for a in so["dev_addr"][: int(co["seg_begin"][min(n_first, len(co) - 1)])]}
    assert {d for d, _, _ in reused} <= first_addrs                    # they lead the walk
    # the other allocations keep the order asked for among themselves
    rest = [int(a) for a in so["dev_addr"] if int(a) in {d for d, _, _ in ra[:-6]}]
    want = {0: [d for d, _, _ in ra[:-6]], 1: [d for d, _, _ in ra[:-6]], 2: sorted(d for d, _, _ in ra[:-6]),
            3: [d for d, _, _ in ra[:-6]][::-1]}[order]
    assert rest == want


def test_plan_without_gpu_fails_loudly(nx):
    """No CPU fallback: without a GPU the product path reports a HIP error instead of doing the work."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("this check is for machines without a GPU")
    a, b = np.zeros(4096, np.uint8), np.zeros(4096, np.uint8)
    with pytest.raises(nx.NixieError) as e:
        nx.Plan([(0x7F00_0000_0000, a.ctypes.data, 4096)], [(0x7F00_0001_0000, b.ctypes.data, 4096)], 1 << 20)
    assert e.value.code in (nx.EHIP, nx.ENOMEM)
    with pytest.raises(nx.NixieError):
        nx.hash_buffers([0x7F00_0000_0000], [64], on_device=True)
    with pytest.raises(nx.NixieError):
        nx.link_peak(1 << 20, 1)


@pytest.mark.parametrize("threads", [0, 1, 5])
def test_host_copy_equals_plain_copy(nx, threads):
    """nixie_host_copy (the pinned <-> pageable leg outside a switch) against numpy slicing:
    ragged sizes across the 1 MiB work unit, every source / destination misalignment, canaries."""
    rng = np.random.default_rng(5)
    sizes = [0, 1, 15, 16, 17, 4095, (1 << 20) - 1, 1 << 20, (1 << 20) + 1, 3 * (1 << 20) + 77, 123457]
    src, dst, want = [], [], []
    for i, b in enumerate(sizes):
        s = rng.integers(0, 256, b + 64, dtype=np.uint8)
        d = np.full(b + 96, 0xC3, dtype=np.uint8)
        so, do = i % 16, (i * 7) % 16 + 16
        src.append(s[so:so + b])
        dst.append(d[do:do + b])
        want.append((d, do, s[so:so + b].copy()))
    nx.host_copy([d.ctypes.data for d in dst], [s.ctypes.data for s in src], sizes, threads)
    for (d, do, w), b in zip(want, sizes):
        assert np.array_equal(d[do:do + b], w)
        assert (d[:do] == 0xC3).all() and (d[do + b:] == 0xC3).all()
    with pytest.raises(nx.NixieError) as e:
        nx.host_copy([0], [src[3].ctypes.data], [16])
    assert e.value.code == nx.EINVAL


def test_header_is_plain_c_and_binding_structs_match(tmp_path):
    """include/nixie.h compiles as C99 and as C++, and every struct of the ctypes binding has the
    size the C compiler gives it (a drifted field would shift every one behind it)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    from paper_2601_11743_amd import nixie as binding
    import ctypes
    pairs = {"nixie_alloc_t": binding._Alloc, "nixie_table_t": binding._Table, "nixie_opts_t": binding._Opts,
             "nixie_plan_info_t": binding._Info, "nixie_segment_t": binding._Segment, "nixie_chunk_t": binding._Chunk,
             "nixie_stats_t": binding._Stats, "nixie_verify_report_t": binding._Report,
             "nixie_link_peak_t": binding._LinkPeak, "nixie_sched_params_t": binding._SchedParams,
             "nixie_sched_decision_t": binding._SchedDecision, "nixie_sched_app_t": binding._SchedApp,
             "nixie_chunk_state_t": binding._ChunkState, "nixie_capacity_t": binding._Capacity,
             "nixie_placement_t": binding._Placement}
    src = tmp_path / "sizes.c"
    body = "".join(f'    printf("{name} %zu\\n", sizeof({name}));\n' for name in pairs)
    src.write_text('#include <stdio.h>\n#include "nixie.h"\nint main(void) {\n' + body + "    return 0;\n}\n")
    exe = tmp_path / "sizes"
    inc = "-I" + os.path.join(ROOT, "include")
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", inc, str(src), "-o", str(exe)])
    subprocess.check_call(["g++", "-std=c++17", "-fsyntax-only", "-x", "c++", inc, str(src)])
    out = subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout
    sizes = dict(line.split() for line in out.splitlines())
    for name, ct in pairs.items():
        assert int(sizes[name]) == ctypes.sizeof(ct), f"{name}: C says {sizes[name]}, the binding {ctypes.sizeof(ct)}"


def test_shim_library_exports_what_its_header_declares():
    """libnixie_shim.so (include/nixie_shim.h): the interposed runtime calls under the runtime's own
    names plus the three nixie_shim_* calls.  Loaded privately here, so nothing is interposed."""
    import ctypes
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    path = os.path.join(root, "paper_2601_11743_amd", "libnixie_shim.so")
    assert os.path.exists(path), "build first: python -m paper_2601_11743_amd.build"
    header = open(os.path.join(root, "include", "nixie_shim.h")).read()
    declared = set(re.findall(r"\b(nixie_shim_\w+)\s*\(", header)) - {"nixie_shim_info_t"}
    assert declared == {"nixie_shim_info", "nixie_shim_evict", "nixie_shim_restore"}
    lib = ctypes.CDLL(path, mode=os.RTLD_LOCAL)
    # both ways: every runtime call the library defines is documented, every documented one is defined
    import subprocess
    nm = subprocess.run(["nm", "-D", "--defined-only", path], capture_output=True, text=True, check=True).stdout
    defined = {l.split()[-1] for l in nm.splitlines() if l.split()[-1].startswith("hip")}
    block = header[header.index("Interposed runtime calls"):header.index("Not interposed")]
    documented = set(re.findall(r"\bhip[A-Z]\w+", block)) - {"hipErrorOutOfMemory"}
    assert defined == documented, (sorted(defined - documented), sorted(documented - defined))
    assert {"hipMalloc", "hipFree", "hipMemGetInfo", "hipLaunchKernel", "hipModuleLaunchKernel", "hipMemcpyAsync",
            "hipMemsetAsync", "hipDeviceSynchronize", "hipStreamSynchronize"} <= defined
    for name in sorted(declared | defined):
        assert getattr(lib, name) is not None, name
    info = (ctypes.c_uint64 * 16)()
    assert lib.nixie_shim_info(info) == -1               # NIXIE_EINVAL: no interposed call has been made


def test_planner_properties_on_random_tables(nx):
    """Property test (hypothesis): for random tables, slot sizes, orders, ring splits and skews the
    planner's output partitions every allocation exactly, fits the slots, keeps the 16-byte congruence and
    stays inside the ring; the launch geometry it proposes is self-consistent."""
    from hypothesis import given, settings, strategies as st, HealthCheck

    sizes = st.lists(st.one_of(st.integers(0, 64), st.integers(1, 5000), st.integers(60_000, 300_000),
                               st.sampled_from([4095, 4096, 4097, 65535, 65536, 65537, 1 << 20])), min_size=0, max_size=24)

    @settings(max_examples=120, deadline=None, suppress_health_check=[HealthCheck.too_slow])
    @given(sizes, sizes, st.sampled_from([4096, 8192, 65536, 262144]), st.integers(4, 40), st.integers(0, 3),
           st.integers(0, 15), st.integers(0, 15), st.booleans(), st.integers(0, 200))
    def run(sa, sb, S, slots, order, skew_d, skew_h, by_bytes, flex):
        ra = fake_rows(sa, skew_dev=skew_d, skew_host=skew_h)
        rb = fake_rows(sb, dev_base=0x7F80_0000_0000, host_base=0x1800_0000_0000, skew_dev=skew_h, skew_host=skew_d)
        ring = slots * S
        o = nx.Opts(slot_bytes=S, order=order, flags=nx.SPLIT_BY_BYTES if by_bytes else 0, flex_wgs=flex)
        lay = nx.Layout(ra, rb, ring, o)
        info = check_layout(lay, ra, rb, ring)
        n_out, n_in = sum(sa) > 0, sum(sb) > 0
        assert (info["out_slots"] >= 2) == n_out and (info["in_slots"] >= 2) == n_in
        assert (info["gather_wgs"] > 0) == n_out and (info["scatter_wgs"] > 0) == n_in
        assert (info["flex_wgs"] > 0) == (n_out and n_in)               # only where both directions run
        assert info["flex_wgs"] == (min(flex, 256) if flex else max(4, info["gather_wgs"] // 8)) or not (n_out and n_in)
        for team, key in ((info["team_out"], "gather_wgs"), (info["team_in"], "scatter_wgs")):
            if info[key]:
                assert 1 <= team <= 256 and info[key] <= 1024
        # a chunk count that follows from the sizes alone: never fewer chunks than bytes / slot
        assert info["chunks_out"] >= -(-sum(sa) // S) and info["chunks_in"] >= -(-sum(sb) // S)
        lay.close()

    run()
