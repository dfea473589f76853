#!/usr/bin/env python3
"""Benchmark of the context-switch swap on one MI355X.

A step is one bidirectional switch of the LLM-shaped working sets (config 2): the chunk planner
runs, then nixie_switch evicts application A (8B bf16 decoder + 2 GiB KV cache, 16.96 GiB in 355
allocations) to pageable memory while bringing application B (same shapes, other seed) into HBM,
through a 256 MiB pinned ring in 4 MiB slots.  Inputs are resident (A in HBM, B in pageable
memory) before the timed region.  Prints one JSON line.

Without --config the same line also carries a "configs" list: the metric taken literally (config 6,
64 x 256 MiB each way), the asymmetric (3), fragmented (4) and tiny (1) configs, and config 5's
pinned-budget sweep (rings of 16 / 64 / 256 / 1024 MiB, 10 ping-pong switches each), every one
in the library's default launch configuration, verified by per-allocation hashes and, except for the
sweep, a whole-arena compare; and a "shim" object: an unmodified HIP program (tests/shim_app, 2.7 GiB)
evicted and restored three times under the LD_PRELOAD shim, as the shim itself reports it.
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


# committed rocprofv3 --pmc summaries, by (config, ring MiB): the counters were read on exactly that workload
PMC_SUMMARIES = {(2, 256): "nixie_swap_kernel_llm_pmc.txt",
                 (4, 64): "nixie_swap_kernel_fragmented_pmc.txt",
                 (5, 16): "nixie_swap_kernel_budget16_pmc.txt"}


def read_traffic(config: int, ring_bytes: int, plain: bool):
    """HBM bytes per launch of the swap kernel from the committed rocprofv3 --pmc summary of this
    very workload, or None when no counters were taken on it (or options changed the run)."""
    name = PMC_SUMMARIES.get((config, ring_bytes >> 20))
    if not name or not plain:
        return None
    try:
        for line in open(os.path.join(ROOT, "profiles", name)):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


def summarize(stats, info, peak) -> dict:
    """Latency, rates and stall sums of a list of nixie_stats dicts (one per switch)."""
    med = lambda v: sorted(v)[len(v) // 2]
    lat = sorted(s["ns_total"] / 1e6 for s in stats)
    out_gbs = med([s["bytes_out"] / max(1, s["ns_out_done"]) for s in stats]) if info["bytes_out"] else 0.0
    in_gbs = med([s["bytes_in"] / max(1, s["ns_in_done"]) for s in stats]) if info["bytes_in"] else 0.0
    r = {"latency_ms": {"min": round(lat[0], 3), "median": round(med(lat), 3), "max": round(lat[-1], 3)},
         "bidir_GBps": round((info["bytes_out"] + info["bytes_in"]) / med(lat) / 1e6, 3),
         "out_GBps": round(out_gbs, 3), "in_GBps": round(in_gbs, 3),
         "b_ready_ms": round(med([s["ns_in_done"] / 1e6 for s in stats]), 3),
         "kernel_ms": round(med([s["ns_kernel"] / 1e6 for s in stats]), 3),
         "stalls": {"drain_wait_ms": round(med([s["drain_wait_ns"] for s in stats]) / 1e6, 2),
                    "fill_wait_ms": round(med([s["fill_wait_ns"] for s in stats]) / 1e6, 2),
                    "gather_stall_ms_sum": round(med([s["gather_stall_ticks"] for s in stats]) / 1e5, 2),
                    "scatter_stall_ms_sum": round(med([s["scatter_stall_ticks"] for s in stats]) / 1e5, 2)}}
    if peak:
        r["out_frac_of_unidirectional_peak"] = round(out_gbs / peak["sdma_d2h"], 4)
        r["in_frac_of_unidirectional_peak"] = round(in_gbs / peak["sdma_h2d"], 4)
    return r


def workload_name(W, cfg_id, A, B, info, ring) -> str:
    return (f"config {cfg_id} ({W.CONFIG_NAMES[cfg_id]}): {info['bytes_out'] / 2**30:.2f} GiB out in {len(A.sizes)} "
            f"allocations / {info['bytes_in'] / 2**30:.2f} GiB in in {len(B.sizes)} allocations, "
            f"ring {ring >> 20} MiB in {info['slot_bytes'] >> 10} KiB slots")


def ring_sweep(nx, rows_a, rows_b, rings, opts, h_a, h_b, peak, log, switches: int = 10) -> list:
    """Config 5 protocol: per ring size a warm-up round trip, then `switches` back-to-back ping-pong
    switches A<->B over the same buffers, hashes checked at the end (A is back in HBM, B in
    pageable memory after an even number)."""
    out = []
    for r in rings:
        fwd, rev = nx.Plan(rows_a, rows_b, r, opts), nx.Plan(rows_b, rows_a, r, opts)
        fwd.switch(); rev.switch()
        sts = [(fwd if t % 2 == 0 else rev).switch() for t in range(switches)]
        rep = (rev if switches % 2 == 0 else fwd).verify(*((h_b, h_a) if switches % 2 == 0 else (h_a, h_b)), check=False)
        pi = fwd.info()
        row = {"ring_mib": r >> 20, "slot_kib": pi["slot_bytes"] >> 10,
               "pinned_bytes": pi["pinned_ring_bytes"] + pi["pinned_ctrl_bytes"], "switches": switches,
               **summarize(sts, pi, peak),
               "hash_mismatches": rep["mismatched_out"] + rep["mismatched_in"]}
        fwd.close(); rev.close()
        out.append(row)
        log("[bench] ring sweep:", row)
    return out


def extra_config(nx, W, torch, cfg_id: int, peak, log) -> dict:
    """One of the other benchmark configs, in the library's default launch configuration: built,
    switched (1 warm-up + timed), verified by per-allocation hashes and a whole-arena compare."""
    from workloads.device import BigSet
    cf = W.config(cfg_id)
    t0 = time.perf_counter()
    A = BigSet(cf["A"], cf["seed_A"], "dev", cf["content"])
    B = BigSet(cf["B"], cf["seed_B"], "host", cf["content"])
    rows_a, rows_b = A.rows_np(), B.rows_np()
    opts = nx.Opts(slot_bytes=cf["slot_bytes"] or 0)
    res = {"config": cfg_id, "build_s": round(time.perf_counter() - t0, 1)}
    if cfg_id == 5:
        probe = nx.Plan(rows_a, rows_b, cf["ring_bytes"][0], opts)
        h_a, h_b = probe.hash_tables()
        res["workload"] = workload_name(W, cfg_id, A, B, probe.info(), cf["ring_bytes"][0]) + " (ring swept)"
        probe.close()
        res["ring_sweep"] = ring_sweep(nx, rows_a, rows_b, cf["ring_bytes"], opts, h_a, h_b, peak, log)
        res["verified"] = {"hash_mismatches": sum(r["hash_mismatches"] for r in res["ring_sweep"]),
                           "full_buffer_equal": None,
                           "note": "after each ring size's 10 switches A is back in HBM and B in pageable memory: "
                                   "per-allocation hashes of both against the hashes taken before the first switch"}
    else:
        ring = cf["ring_bytes"][0]
        plan = nx.Plan(rows_a, rows_b, ring, opts)
        info = plan.info()
        h_out, h_in = plan.hash_tables()
        steps = 20 if cfg_id == 1 else 5

        def step():
            nx.Layout(rows_a, rows_b, ring, opts).close()      # the chunk planner is part of every step
            return plan.switch()
        step()
        t1 = time.perf_counter()
        stats = [step() for _ in range(steps)]
        ms = (time.perf_counter() - t1) / steps * 1e3
        wait_in_ms = None
        if cfg_id == 3:
            # the same switch once more in three steps: when does nixie_switch_wait_in let the incoming application run?
            t2 = time.perf_counter()
            plan.switch_begin()
            plan.switch_wait_in()
            wait_in_ms = round((time.perf_counter() - t2) * 1e3, 3)
            plan.switch_end()
        rep = plan.verify(h_out, h_in, check=False)
        equal = bool(A.arenas_equal() and B.arenas_equal())
        plan.close()
        res.update(workload=workload_name(W, cfg_id, A, B, info, ring), steps=steps, ms_per_step=round(ms, 3),
                   **summarize(stats, info, peak),
                   pinned_bytes=info["pinned_ring_bytes"] + info["pinned_ctrl_bytes"],
                   traffic=read_traffic(cfg_id, ring, True),
                   algorithmic_bytes_per_launch=info["bytes_out"] + info["bytes_in"],
                   **({"wait_in_returned_ms": wait_in_ms} if wait_in_ms is not None else {}),
                   verified={"hash_mismatches": rep["mismatched_out"] + rep["mismatched_in"], "full_buffer_equal": equal})
    del A, B
    torch.cuda.empty_cache()
    log(f"[bench] config {cfg_id}:", {k: v for k, v in res.items() if k != "ring_sweep"})
    return res


def shim_leg(log) -> dict | None:
    """The transparent shim at GiB scale: tests/shim_app (an ordinary HIP program) as a child process under
    LD_PRELOAD=libnixie_shim.so with the paper's idleness rule, 2.7 GiB in three buffers, three pauses.  Reports
    what the shim logs about each eviction and restore.  Must run before this process touches the GPU (a
    process that has initialised the GPU may not start another program here)."""
    import re
    import subprocess
    root = os.path.dirname(os.path.abspath(__file__))
    app = os.path.join(root, "tests", "shim_app", "shim_app")
    shim = os.path.join(root, "paper_2601_11743_amd", "libnixie_shim.so")
    if not (os.path.exists(app) and os.path.exists(shim)):
        from paper_2601_11743_amd import build
        build.build()
    env = dict(os.environ)
    have = env.get("LD_PRELOAD", "")
    env.update(LD_PRELOAD=(have + ":" if have else "") + shim, NIXIE_SHIM_LOG="1", NIXIE_SHIM_IDLE_MS="100",
               NIXIE_SHIM_POOL_MIB="4096", NIXIE_SHIM_RING_MIB="64")
    try:
        r = subprocess.run([app, "500", "2048", "3"], env=env, capture_output=True, text=True, timeout=120)
    except (OSError, subprocess.TimeoutExpired) as e:
        log("[bench] shim leg did not run:", e)
        return None
    ev = [(int(b), float(ms)) for b, ms in re.findall(r"evicted \d+ allocations, (\d+) bytes, in ([\d.]+) ms", r.stderr)]
    rs = [(int(b), float(ms)) for b, ms in re.findall(r"restored \d+ allocations, (\d+) bytes, in ([\d.]+) ms", r.stderr)]
    bg = [(int(n), float(ms)) for n, ms in re.findall(r"unmapped (\d+) blocks in the background in ([\d.]+) ms", r.stderr)]
    out = {"workload": "tests/shim_app 500 2048 3 under LD_PRELOAD=libnixie_shim.so, idle eviction after 100 ms, "
                       "2 MiB units in 32 MiB blocks, 64 MiB ring",
           "ok": r.returncode == 0 and "RESULT ok" in r.stdout,
           "bytes": ev[0][0] if ev else 0,
           "evict_ms": [ms for _, ms in ev], "restore_ms": [ms for _, ms in rs],
           "evict_GBps": round(max((b / ms / 1e6 for b, ms in ev), default=0.0), 2),
           "restore_GBps": round(max((b / ms / 1e6 for b, ms in rs), default=0.0), 2),
           "background_unmap": [{"blocks": n, "ms": ms} for n, ms in bg]}
    log("[bench] shim:", out)
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=0,
                    help="run only this benchmark config: 1..5 (2 = headline); 6 = exactly 16 GiB out / 16 GiB in as "
                         "64 x 256 MiB.  Default: the headline config 2 as the timed steps, then configs 6, 3, 4, 1 "
                         "and the ring sweep of config 5 as a 'configs' list in the same JSON line")
    ap.add_argument("--no-extras", action="store_true", help="default run without the 'configs' list")
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
    ap.add_argument("--prefetch", action="store_true",
                    help="after the timed steps: act on a scheduler's prefetch hint for B -- nixie_host_copy moves B from "
                         "pageable memory into a registered pinned tier (timed, off the switch's critical path), then the "
                         "same switch runs with B moving directly; adds a 'prefetch' object to the JSON line")
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

    nx.lib()                      # (builds the library first if nothing is built: before the GPU is touched)
    shim = None
    if args.config == 0 and not args.no_extras:
        shim = shim_leg(log)      # a child process: also before the GPU is touched
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    plain_run = (args.config in (0, 2) and not (args.ring_mib or args.slot_kib or args.gather_wgs or args.scatter_wgs or
                 args.team or args.flags or args.order or args.in_place or args.spaces or args.pinned_tier != "none" or
                 args.scale != 1.0))
    with_extras = args.config == 0 and not args.no_extras and plain_run
    if args.config == 0:
        args.config = 2
    cf = W.config(args.config, scale=args.scale)
    ring = (args.ring_mib << 20) if args.ring_mib else cf["ring_bytes"][min(2, len(cf["ring_bytes"]) - 1)]
    slot = (args.slot_kib << 10) if args.slot_kib else (cf["slot_bytes"] or 0)
    if args.scale != 1.0 and not args.ring_mib:
        ring = max(16 << 20, int(ring * args.scale) >> 20 << 20)
        slot = 0 if not slot else max(64 << 10, int(slot * args.scale) >> 12 << 12)

    peak = None
    if not args.no_link_peak:     # before the working sets exist: the probe pins 2 GiB of its own
        peak = nx.link_peak(1 << 30, 3)
        log("[bench] link peak GB/s:", {k: round(v, 2) for k, v in peak.items()})

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

    # What a scheduler pays that makes a fresh plan for every switch (the tables change) but keeps its
    # pinned ring: descriptors, counters, control block and host threads, without the ring's allocation.
    plan_on_ring_ms = None
    if pool is None and not args.in_place:
        keep = nx.Ring(ring)
        took = []
        for _ in range(3):
            t0 = time.perf_counter()
            nx.Plan(rows_a, rows_b, keep, opts).close()
            took.append((time.perf_counter() - t0) * 1e3)
        keep.close()
        plan_on_ring_ms = round(sorted(took)[1], 2)
        log(f"[bench] nixie_plan_on_ring + destroy: {took} ms")

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

    prefetch = None
    if args.prefetch and pool is None and not args.in_place and args.pinned_tier == "none":
        # B's bytes are still in its pageable arena (a switch leaves its sources alone unless they are reused).
        pin_t = torch.empty(max(B.layout.total, 4096), dtype=torch.uint8, pin_memory=True)
        pin = pin_t.numpy()
        nx.tier_register(pin.ctypes.data, pin.size)
        offs = np.asarray(B.layout.offsets, dtype=np.uint64)
        src = (np.uint64(B.host.ctypes.data) + offs).tolist()
        dst = (np.uint64(pin.ctypes.data) + offs).tolist()
        threads = max(1, min(8, (os.cpu_count() or 2) // 2))
        pin[::4096] = 0                                               # a long-lived tier: its pages are mapped already
        nx.host_copy(dst[:1], src[:1], B.sizes[:1], threads)          # touch the code path
        c0, t0 = time.process_time(), time.perf_counter()
        nx.host_copy(dst, src, B.sizes, threads)
        pf_s, pf_cpu = time.perf_counter() - t0, time.process_time() - c0
        rows_bp = rows_b.copy()
        rows_bp[:, 1] = np.uint64(pin.ctypes.data) + offs
        pp = nx.Plan(rows_a, rows_bp, ring, opts)
        pi = pp.info()
        pp.switch()
        c0 = time.process_time()
        sts = [pp.switch() for _ in range(3)]
        cpu_after = (time.process_time() - c0) / 3
        rep_p = pp.verify(h_out, h_in, check=False)
        pp.close()
        nx.tier_unregister(pin.ctypes.data)
        prefetch = {"prefetch_ms": round(pf_s * 1e3, 2), "prefetch_GBps": round(B.total_bytes / pf_s / 1e9, 2),
                    "prefetch_threads": threads, "prefetch_cpu_s": round(pf_cpu, 3),
                    "direct_bytes_in": pi["direct_bytes_in"], "fill_threads_after": pi["fill_threads"],
                    "switch_after_prefetch": summarize(sts, pi, peak), "host_cpu_s_per_switch_after": round(cpu_after, 4),
                    "hash_mismatches": rep_p["mismatched_out"] + rep_p["mismatched_in"],
                    "note": "the prefetch runs while the outgoing application still owns the GPU; compare "
                            "switch_after_prefetch and host_cpu_s_per_switch_after with the line's own figures"}
        log("[bench] prefetch:", prefetch)
        del pin, pin_t

    sweep = None
    if args.ring_sweep:
        sweep = ring_sweep(nx, rows_a, rows_b, cf["ring_bytes"], opts, h_out, h_in, peak, log)

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
            "traffic": read_traffic(args.config, ring, plain_run or (args.config in (4, 5) and not args.flags)),
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
                   "flex_wgs": info["flex_wgs"],
                   "team": info["team_out"], "drain_threads": info["drain_threads"],
                   "fill_threads": info["fill_threads"], "flags": args.flags, "scale": args.scale,
                   "in_place": bool(args.in_place), "pinned_tier": args.pinned_tier,
                   "repeat": "every timed step runs the chunk planner and then the same switch again (A out, B in; "
                             "a source's bytes are unspecified after a switch and are not restored in between); "
                             "the ping-pong protocol is config 5's ring sweep",
                   "direct_bytes_out": info["direct_bytes_out"], "direct_bytes_in": info["direct_bytes_in"]},
        "switch_latency_ms": {"min": round(lat[0], 3), "median": round(med(lat), 3), "max": round(lat[-1], 3)},
        "b_ready_ms": round(med(sorted(s["ns_in_done"] / 1e6 for s in stats)), 3),
        "plan_ms": round(plan_ms, 2), "plan_on_shared_ring_ms": plan_on_ring_ms,
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
    if prefetch is not None:
        res["prefetch"] = prefetch
    if sweep is not None:
        res["ring_sweep"] = sweep
    if oversub is not None:
        res["oversubscription_sweep"] = oversub
    del A, B
    if pool is not None:
        space_a.close()
        space_b.close()
        pool.close()
    torch.cuda.empty_cache()
    if with_extras:
        res["configs"] = [extra_config(nx, W, torch, c, peak, log) for c in (6, 3, 4, 1, 5)]
    if shim is not None:
        res["shim"] = shim
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(cf, int(args.cpu_sample_gib * 2**30))
    print(json.dumps(res), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
