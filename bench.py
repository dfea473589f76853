#!/usr/bin/env python3
"""Benchmark of the context-switch swap on one MI355X.

A step is one bidirectional switch of the LLM-shaped working sets (config 2): the chunk planner
runs, then nixie_switch evicts application A (8B bf16 decoder + 2 GiB KV cache, 16.96 GiB in 355
allocations) to pageable memory while bringing application B (same shapes, other seed) into HBM,
through a 256 MiB pinned ring in 4 MiB slots.  Inputs are resident (A in HBM, B in pageable
memory) before the timed region.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def cpu_baseline(cf, sample_bytes: int) -> dict:
    """The CPU oracle as it stands, timed on this machine's host cores on the leading allocations
    of both tables (ordinary arrays stand in for HBM)."""
    import numpy as np
    import oracle
    from workloads.device import pageable_arena

    orc = oracle.Oracle()

    def sample(sizes):
        out, acc = [], 0
        for _, b in sizes:
            if acc + b > sample_bytes and out:
                break
            out.append(b)
            acc += b
        return out

    sa, sb = sample(cf["A"]), sample(cf["B"])

    def arenas(sizes, seed):
        tot = sum(sizes)
        src = pageable_arena(tot, fill=None)
        rng = np.random.default_rng(seed)
        blk = rng.integers(0, 256, size=1 << 24, dtype=np.uint8)
        for a in range(0, tot, blk.size):
            n = min(blk.size, tot - a)
            src[a:a + n] = blk[:n]
        dst = pageable_arena(tot, fill=0)
        offs = np.concatenate([[0], np.cumsum(sizes)])
        return src, dst, [(int(offs[i]), int(sizes[i])) for i in range(len(sizes))]

    a_dev, a_host, la = arenas(sa, 1)
    b_host, b_dev, lb = arenas(sb, 2)
    pa = [(a_dev[o:o + b], a_host[o:o + b]) for o, b in la]
    pb = [(b_dev[o:o + b], b_host[o:o + b]) for o, b in lb]
    nbytes = sum(sa) + sum(sb)
    orc.switch_direct(pa[:1], pb[:1])                      # touch code paths once
    t_direct = min(orc.switch_direct(pa, pb) for _ in range(2))
    cores = os.cpu_count() or 1
    T = max(1, min(8, cores // 2))
    slot = cf["slot_bytes"] or (2 << 20)
    ring = max(cf["ring_bytes"][0], 2 * T * slot)
    t_mt = min(orc.switch_staged_mt(pa, pb, ring, slot, T) for _ in range(2))
    ok = bool(np.array_equal(a_dev, a_host) and np.array_equal(b_dev, b_host))
    return {
        "value": round(nbytes / t_direct / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": f"direct definition (two memcpy loops, 1 thread) on the first {len(sa)}+{len(sb)} allocations "
                  f"of config 2 ({sum(sa) / 2**30:.2f} GiB out + {sum(sb) / 2**30:.2f} GiB in), host arrays stand in for HBM",
        "ms": round(t_direct * 1e3, 2),
        "staged_mt": {"value": round(nbytes / t_mt / 1e9, 3), "unit": "GB/s", "cores": 2 * T,
                      "ms": round(t_mt * 1e3, 2), "ring_bytes": ring, "slot_bytes": slot},
        "result_checked": ok,
    }


def read_traffic(path: str):
    """HBM bytes per launch of the swap kernel from the committed rocprofv3 --pmc summary."""
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=2,
                    help="benchmark config 1..5 (2 = headline); 6 = exactly 16 GiB out / 16 GiB in as 64 x 256 MiB")
    ap.add_argument("--no-serialized", action="store_true",
                    help="skip the serialised self-baseline (evict completely, then restore)")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink all sizes (debug only)")
    ap.add_argument("--ring-mib", type=int, default=0, help="override ring size")
    ap.add_argument("--slot-kib", type=int, default=0)
    ap.add_argument("--gather-wgs", type=int, default=0)
    ap.add_argument("--scatter-wgs", type=int, default=0)
    ap.add_argument("--team", type=int, default=0)
    ap.add_argument("--drain-threads", type=int, default=0)
    ap.add_argument("--fill-threads", type=int, default=0)
    ap.add_argument("--flags", type=int, default=0)
    ap.add_argument("--order", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-link-peak", action="store_true")
    ap.add_argument("--cpu-sample-gib", type=float, default=4.0)
    ap.add_argument("--in-place", action="store_true",
                    help="in-place switch: B is restored into the HBM that A is evicted from (one device arena); "
                         "every step is a switch in the opposite direction of the one before")
    ap.add_argument("--spaces", action="store_true",
                    help="in-place switch between two applications that keep their own device addresses over one "
                         "pool of physical memory: every step maps the incoming application's address space, "
                         "switches, and unmaps the outgoing one's (all inside the timed region)")
    ap.add_argument("--block-mib", type=int, default=0, help="--spaces: pool block size (0 = library default)")
    ap.add_argument("--pinned-tier", choices=["none", "out", "in", "both"], default="none",
                    help="keep the host side of the outgoing / incoming / both working sets in registered pinned "
                         "memory: those allocations move directly, without ring slots or host threads")
    ap.add_argument("--oversub-sweep", action="store_true",
                    help="switch latency against the amount of memory oversubscription: a notional GPU capacity "
                         "of (A + B - oversubscribed size); nixie_place evicts only what the incoming application "
                         "needs; ping-pong A<->B; adds an 'oversubscription_sweep' list to the JSON line")
    ap.add_argument("--ring-sweep", action="store_true",
                    help="config 5 protocol: for every ring size of the config, 10 back-to-back ping-pong "
                         "switches A<->B; adds a 'ring_sweep' list to the JSON line")
    ap.add_argument("--quiet", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the swap has no multi-GPU part: each GPU has "
              "its own host link, ring and tables); re-run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2601_11743_amd as nx
    import workloads as W
    from workloads.device import BigSet

    def log(*a):
        if not args.quiet:
            print(*a, file=sys.stderr, flush=True)

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    nx.lib()
    torch.cuda.set_device(0)
    cf = W.config(args.config, scale=args.scale)
    ring = (args.ring_mib << 20) if args.ring_mib else cf["ring_bytes"][min(2, len(cf["ring_bytes"]) - 1)]
    slot = (args.slot_kib << 10) if args.slot_kib else (cf["slot_bytes"] or 0)
    if args.scale != 1.0 and not args.ring_mib:
        ring = max(16 << 20, int(ring * args.scale) >> 20 << 20)
        slot = 0 if not slot else max(64 << 10, int(slot * args.scale) >> 12 << 12)

    t0 = time.perf_counter()
    pool = space_a = space_b = None
    if args.spaces:
        from workloads.device import device_view
        args.in_place = True
        sizes = lambda t: [s if isinstance(s, int) else s[1] for s in t]
        need = max(W.make_layout(sizes(cf["A"]), redzone=256).total, W.make_layout(sizes(cf["B"]), redzone=256).total)
        pool = nx.Pool(need, args.block_mib << 20)
        space_a, space_b = nx.Space(pool), nx.Space(pool)
        space_a.map()
        space_b.map()
        A = BigSet(cf["A"], cf["seed_A"], "dev", cf["content"], dev_arena=device_view(space_a.base, pool.bytes))
        B = BigSet(cf["B"], cf["seed_B"], "host", cf["content"], dev_arena=device_view(space_b.base, pool.bytes))
        torch.cuda.synchronize()
        space_b.unmap()                 # B waits in pageable memory: its addresses are reserved, nothing behind them
    else:
        pin_a, pin_b = args.pinned_tier in ("out", "both"), args.pinned_tier in ("in", "both")
        A = BigSet(cf["A"], cf["seed_A"], "dev", cf["content"], pinned_host=pin_a)
        B = BigSet(cf["B"], cf["seed_B"], "host", cf["content"], share_dev=A if args.in_place else None,
                   pinned_host=pin_b)
        for s_, pinned in ((A, pin_a), (B, pin_b)):
            if pinned:
                nx.tier_register(s_.host.ctypes.data, s_.host.size)
    if args.in_place:
        args.flags |= nx.IN_PLACE
        torch.cuda.empty_cache()
    log(f"[bench] working sets built in {time.perf_counter() - t0:.1f} s: "
        f"A {A.total_bytes / 2**30:.2f} GiB / {len(A.sizes)} allocations, "
        f"B {B.total_bytes / 2**30:.2f} GiB / {len(B.sizes)} allocations")

    peak = None
    if not args.no_link_peak:
        peak = nx.link_peak(1 << 30, 3)
        log("[bench] link peak GB/s:", {k: round(v, 2) for k, v in peak.items()})

    opts = nx.Opts(slot_bytes=slot, gather_wgs=args.gather_wgs, scatter_wgs=args.scatter_wgs, team=args.team,
                   drain_threads=args.drain_threads, fill_threads=args.fill_threads, flags=args.flags,
                   order=args.order)
    t0 = time.perf_counter()
    rows_a, rows_b = A.rows_np(), B.rows_np()
    plan = nx.Plan(rows_a, rows_b, ring, opts)
    plan_ms = (time.perf_counter() - t0) * 1e3
    info = plan.info()
    log("[bench] plan:", info, f"nixie_plan {plan_ms:.1f} ms")
    h_out, h_in = plan.hash_tables()

    back = nx.Plan(rows_b, rows_a, ring, opts) if args.in_place else None
    n_switches = [0]
    remap_ms = {"map": [], "unmap": []}

    def step():
        fwd_turn = (n_switches[0] % 2 == 0) or back is None
        lay = nx.Layout(rows_a if fwd_turn else rows_b, rows_b if fwd_turn else rows_a, ring, opts)
        lay.close()                                    # the chunk planner is part of every step
        n_switches[0] += 1
        if pool is None:
            return (plan if fwd_turn else back).switch()
        t_a = time.perf_counter()
        (space_b if fwd_turn else space_a).map()       # the incoming application's addresses get memory
        t_b = time.perf_counter()
        st = (plan if fwd_turn else back).switch()
        t_c = time.perf_counter()
        (space_a if fwd_turn else space_b).unmap()     # the outgoing application keeps only its addresses
        remap_ms["map"].append((t_b - t_a) * 1e3)
        remap_ms["unmap"].append((time.perf_counter() - t_c) * 1e3)
        return st

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    stats = []
    cpu_begin = time.process_time()
    t_begin = time.perf_counter()
    for _ in range(args.steps):
        stats.append(step())
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_begin
    host_cpu_s = (time.process_time() - cpu_begin) / args.steps   # all threads of this process

    serialized = None
    if not args.no_serialized and not args.in_place and not (args.flags & nx.SERIALIZE) and info["bytes_out"] and info["bytes_in"]:
        # self-baseline: the same library with the overlap switched off (one link direction at a time)
        so = nx.Opts(slot_bytes=slot, gather_wgs=args.gather_wgs, scatter_wgs=args.scatter_wgs, team=args.team,
                     drain_threads=args.drain_threads, fill_threads=args.fill_threads,
                     flags=args.flags | nx.SERIALIZE, order=args.order)
        sp = nx.Plan(rows_a, rows_b, ring, so)
        sp.switch()
        sms = sorted(sp.switch()["ns_total"] / 1e6 for _ in range(2))
        sp.close()
        serialized = {"ms": round(sms[0], 3), "slowdown_vs_bidirectional": round(sms[0] / (elapsed / args.steps * 1e3), 3)}

    oversub = None
    if args.oversub_sweep and pool is None and not args.in_place:
        # The timed steps left A in pageable memory and B in HBM.  From here on a chunk is an allocation
        # and lives where the placement says; both sets have HBM of their own on this machine, the
        # capacity is the planner's input.
        oversub = []
        shared_ring = nx.Ring(ring)                       # every switch is planned anew; the pinned ring stays
        sets, rws = (A, B), (rows_a, rows_b)
        chunks0 = [(int(b), a, nx.TIER_GPU if a == 1 else nx.TIER_PAGEABLE) for a in (0, 1) for b in sets[a].sizes]
        owner_of = [(a, i) for a in (0, 1) for i in range(len(sets[a].sizes))]
        total = [sets[0].total_bytes, sets[1].total_bytes]
        for frac in (0.125, 0.25, 0.5, 0.75, 1.0):
            capacity = int(total[0] + total[1] - frac * min(total))
            tiers = [t for _, _, t in chunks0]
            lat, moved = [], []
            for turn in range(6):                           # A in, B in, A in, ...
                run = turn % 2
                cur = [(b, a, t) for (b, a, _), t in zip(chunks0, tiers)]
                new, summ, _ = nx.place(capacity, 0, cur, run, [1 - run])
                out_rows = np.array([rws[a][i] for (a, i), t0, t1 in zip(owner_of, tiers, new) if t0 == nx.TIER_GPU and t1 != nx.TIER_GPU], dtype=np.uint64).reshape(-1, 3)
                in_rows = np.array([rws[a][i] for (a, i), t0, t1 in zip(owner_of, tiers, new) if t0 != nx.TIER_GPU and t1 == nx.TIER_GPU], dtype=np.uint64).reshape(-1, 3)
                pl = nx.Plan(out_rows, in_rows, shared_ring, opts)
                st = pl.switch()
                pl.close()
                tiers = new
                if turn >= 2:                               # the first two turns only establish the steady state
                    lat.append(st["ns_total"] / 1e6)
                    moved.append((summ["evicted_bytes"], summ["restored_bytes"]))
            lat.sort()
            oversub.append({"oversubscribed_GiB": round(frac * min(total) / 2**30, 2),
                            "evicted_GiB": round(float(np.mean([m[0] for m in moved])) / 2**30, 2),
                            "restored_GiB": round(float(np.mean([m[1] for m in moved])) / 2**30, 2),
                            "latency_ms": {"min": round(lat[0], 2), "median": round(lat[len(lat) // 2], 2), "max": round(lat[-1], 2)}})
            log("[bench] oversubscription sweep:", oversub[-1])
            # back to the state the sweep started from (B in HBM, A in pageable memory), every chunk moved by a switch
            cur = [(b, a, t) for (b, a, _), t in zip(chunks0, tiers)]
            want = [t for _, _, t in chunks0]
            out_rows = np.array([rws[a][i] for (a, i), t0, t1 in zip(owner_of, tiers, want) if t0 == nx.TIER_GPU and t1 != nx.TIER_GPU], dtype=np.uint64).reshape(-1, 3)
            in_rows = np.array([rws[a][i] for (a, i), t0, t1 in zip(owner_of, tiers, want) if t0 != nx.TIER_GPU and t1 == nx.TIER_GPU], dtype=np.uint64).reshape(-1, 3)
            if len(out_rows) or len(in_rows):
                pl = nx.Plan(out_rows, in_rows, shared_ring, opts)
                pl.switch()
                pl.close()
        shared_ring.close()

    sweep = None
    if args.ring_sweep:
        sweep = []
        for r in cf["ring_bytes"]:
            fwd, rev = nx.Plan(rows_a, rows_b, r, opts), nx.Plan(rows_b, rows_a, r, opts)
            fwd.switch(); rev.switch()                   # warm-up round trip
            sts = []
            for t in range(10):
                sts.append((fwd if t % 2 == 0 else rev).switch())
            rev.verify(h_in, h_out)                      # 10 switches end with A back in HBM, B in pageable memory
            pi = fwd.info()
            msl = sorted(x["ns_total"] / 1e6 for x in sts)
            sweep.append({"ring_mib": r >> 20, "slot_kib": pi["slot_bytes"] >> 10,
                          "pinned_bytes": pi["pinned_ring_bytes"] + pi["pinned_ctrl_bytes"],
                          "latency_ms": {"min": round(msl[0], 2), "median": round(msl[5], 2), "max": round(msl[-1], 2)},
                          "bidir_GBps": round((pi["bytes_out"] + pi["bytes_in"]) / msl[5] / 1e6, 2)})
            fwd.close(); rev.close()
            log("[bench] ring sweep:", sweep[-1])

    diag = bool(args.flags & nx.DIAG_RING_ONLY)
    if back is not None:                # in place: where the sets are depends on the number of switches so far
        b_in_hbm = n_switches[0] % 2 == 1
        rep = (plan.verify(h_out, h_in, check=not diag) if b_in_hbm else back.verify(h_in, h_out, check=not diag))
        here = B if b_in_hbm else A
        if pool is None or A.layout.offsets == B.layout.offsets:
            arenas_ok = None if diag else bool(here.arenas_equal())
        else:                           # the gaps of one layout hold the other application's bytes
            arenas_ok = None if diag or len(here.sizes) > 5000 else bool(here.allocations_equal())
        back.close()
    else:
        rep = plan.verify(h_out, h_in, check=not diag)  # per-allocation hashes on the side that now holds the data
        arenas_ok = None if diag else bool(A.arenas_equal() and B.arenas_equal())
    if arenas_ok is False:
        raise SystemExit("bench.py: full-buffer compare failed after the timed switches")
    plan.close()

    nbytes = info["bytes_out"] + info["bytes_in"]
    ms = elapsed / args.steps * 1e3
    value = nbytes * args.steps / elapsed / 1e9
    lat = sorted(s["ns_total"] / 1e6 for s in stats)
    kern_s = sum(s["ns_kernel"] for s in stats) / len(stats) / 1e9
    out_gbs = sorted(s["bytes_out"] / max(1, s["ns_out_done"]) for s in stats)
    in_gbs = sorted(s["bytes_in"] / max(1, s["ns_in_done"]) for s in stats)
    med = lambda v: v[len(v) // 2]

    roof = {"bound": "host_link", "kernel": "nixie_swap_kernel", "unit": "GB/s",
            "achieved": round(nbytes / kern_s / 1e9, 3), "peak": None, "frac": None,
            "traffic": read_traffic(os.path.join(ROOT, "profiles", "nixie_swap_kernel_llm_pmc.txt")),
            "algorithmic_bytes_per_launch": nbytes, "kernel_ms": round(kern_s * 1e3, 3),
            "traffic_note": "FETCH_SIZE + WRITE_SIZE count every switched byte twice (fetched once, from HBM or over "
                            "the link, and written once, over the link or into HBM): compare with 2 x "
                            "algorithmic_bytes_per_launch",
            "hbm": {"achieved": round(nbytes / kern_s / 1e9, 3), "peak": 8000.0,
                    "frac": round(nbytes / kern_s / 1e9 / 8000.0, 5)}}
    if peak:
        p_uni = peak["sdma_d2h"] + peak["sdma_h2d"]
        roof.update(peak=round(p_uni, 3), frac=round(nbytes / kern_s / 1e9 / p_uni, 4),
                    peak_note="sum of the two one-direction-at-a-time hipMemcpyAsync rates measured in this run",
                    per_direction={
                        "out_GBps": round(med(out_gbs), 3), "in_GBps": round(med(in_gbs), 3),
                        "out_frac_of_unidirectional_peak": round(med(out_gbs) / peak["sdma_d2h"], 4),
                        "in_frac_of_unidirectional_peak": round(med(in_gbs) / peak["sdma_h2d"], 4),
                        "out_frac_of_simultaneous_peak": round(med(out_gbs) / peak["sdma_d2h_both"], 4),
                        "in_frac_of_simultaneous_peak": round(med(in_gbs) / peak["sdma_h2d_both"], 4)},
                    link_peak={k: round(v, 3) for k, v in peak.items()})

    res = {
        "metric": "bidirectional swap GB/s and switch latency (ms), 16 GiB out/in, 256 MiB ring",
        "value": round(value, 3), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"config {args.config} ({W.CONFIG_NAMES[args.config]}): "
                               f"{info['bytes_out'] / 2**30:.2f} GiB out in {len(A.sizes)} allocations / "
                               f"{info['bytes_in'] / 2**30:.2f} GiB in in {len(B.sizes)} allocations, "
                               f"ring {ring >> 20} MiB in {info['slot_bytes'] >> 10} KiB slots",
                   "ring_bytes": ring, "slot_bytes": info["slot_bytes"], "out_slots": info["out_slots"],
                   "in_slots": info["in_slots"], "gather_wgs": info["gather_wgs"], "scatter_wgs": info["scatter_wgs"],
                   "team": info["team_out"], "drain_threads": info["drain_threads"],
                   "fill_threads": info["fill_threads"], "flags": args.flags, "scale": args.scale,
                   "in_place": bool(args.in_place), "pinned_tier": args.pinned_tier,
                   "direct_bytes_out": info["direct_bytes_out"], "direct_bytes_in": info["direct_bytes_in"]},
        "switch_latency_ms": {"min": round(lat[0], 3), "median": round(med(lat), 3), "max": round(lat[-1], 3)},
        "b_ready_ms": round(med(sorted(s["ns_in_done"] / 1e6 for s in stats)), 3),
        "plan_ms": round(plan_ms, 2),
        "host_cpu_s_per_step": round(host_cpu_s, 4),
        "pinned_bytes": {"ring": info["pinned_ring_bytes"], "control": info["pinned_ctrl_bytes"]},
        "verified": {"hash_mismatches": rep["mismatched_out"] + rep["mismatched_in"], "full_buffer_equal": arenas_ok},
        "stalls": {"drain_wait_ms": round(med(sorted(s["drain_wait_ns"] for s in stats)) / 1e6, 2),
                   "fill_wait_ms": round(med(sorted(s["fill_wait_ns"] for s in stats)) / 1e6, 2),
                   "gather_stall_ms_sum": round(med(sorted(s["gather_stall_ticks"] for s in stats)) / 1e5, 2),
                   "scatter_stall_ms_sum": round(med(sorted(s["scatter_stall_ticks"] for s in stats)) / 1e5, 2)},
        "roofline": roof,
    }
    if serialized is not None:
        res["serialized_self_baseline"] = serialized
    if pool is not None:
        k = len(remap_ms["map"]) - args.steps           # timed steps only
        res["config"]["spaces"] = {"pool_bytes": pool.bytes, "block_bytes": pool.block_bytes,
                                   "blocks": pool.bytes // pool.block_bytes}
        res["remap_ms"] = {"map_median": round(med(sorted(remap_ms["map"][k:])), 3),
                           "unmap_median": round(med(sorted(remap_ms["unmap"][k:])), 3),
                           "note": "inside ms_per_step: map the incoming application's space before the switch, "
                                   "unmap the outgoing one's after it"}
    if sweep is not None:
        res["ring_sweep"] = sweep
    if oversub is not None:
        res["oversubscription_sweep"] = oversub
    del A, B
    if pool is not None:
        space_a.close()
        space_b.close()
        pool.close()
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(cf, int(args.cpu_sample_gib * 2**30))
    print(json.dumps(res), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
