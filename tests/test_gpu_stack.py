"""All parts together, as the paper's daemon uses them: the scheduler decides who runs, the placement
planner decides which chunks leave the GPU and to which host tier, freed physical blocks are
assigned to the incoming application's addresses, and one in-place switch moves everything.
Three applications, a pool of physical memory that holds about two of them, a pinned tier that
holds part of one.  After every switch every chunk of every application must hold the bytes it was
generated with, wherever it lives (plain definition of the moves, applied step after step)."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu

MiB = 1 << 20
BLOCK = 2 * MiB


@pytest.fixture(scope="module")
def nx():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2601_11743_amd as nx
    nx.lib()
    return nx


class World:
    """Test-side bookkeeping only: who owns which pool block and which pinned unit."""

    def __init__(self, nx, raw, chunk_blocks, pool_blocks, pinned_units):
        import torch
        self.nx, self.raw = nx, raw
        self.pool = nx.Pool(pool_blocks * BLOCK, BLOCK)
        self.free_blocks = list(range(pool_blocks))
        self.pin_t = torch.empty(pinned_units * BLOCK, dtype=torch.uint8, pin_memory=True)
        self.pin = self.pin_t.numpy()
        nx.tier_register(self.pin.ctypes.data, self.pin.size)
        self.free_units = list(range(pinned_units))
        self.pinned_cap = pinned_units * BLOCK
        self.apps = []
        for a, blocks in enumerate(chunk_blocks):
            sizes = [n * BLOCK for n in blocks]
            offs = np.concatenate([[0], np.cumsum(sizes)[:-1]]).astype(int).tolist()
            pageable = np.zeros(sum(sizes), dtype=np.uint8)
            for j, (o, b) in enumerate(zip(offs, sizes)):                # every application starts in pageable memory
                pageable[o:o + b] = W.content_bytes(100 + a, j, b)
            self.apps.append(dict(space=nx.Space(self.pool), sizes=sizes, offs=offs, pageable=pageable,
                                  tier=[nx.TIER_PAGEABLE] * len(sizes), blocks=[None] * len(sizes),
                                  units=[None] * len(sizes)))

    def close(self):
        for ap in self.apps:
            ap["space"].close()
        self.pool.close()
        self.nx.tier_unregister(self.pin.ctypes.data)

    def host_ptr(self, ap, j, tier, units=None):
        if tier == self.nx.TIER_PAGEABLE:
            return ap["pageable"].ctypes.data + ap["offs"][j]
        units = ap["units"][j] if units is None else units
        assert units is not None and units == list(range(units[0], units[0] + len(units))), "pinned chunk must be contiguous"
        return self.pin.ctypes.data + units[0] * BLOCK

    def take_units(self, n):
        """n contiguous free units of the pinned tier, or None."""
        free = sorted(self.free_units)
        for i in range(len(free) - n + 1):
            if free[i + n - 1] - free[i] == n - 1:
                got = free[i:i + n]
                self.free_units = [u for u in self.free_units if u not in got]
                return got
        return None

    def prefetch(self, a):
        """Act on the scheduler's prefetch hint (paper, "MLFQ with Prefetching": the application at the
        head of the queue is the one most likely to run next, so its data is brought up a tier ahead
        of time): chunks of application a that wait in pageable memory move into the pinned tier with
        nixie_host_copy while there is room.  Returns the bytes moved."""
        nx, ap, moved = self.nx, self.apps[a], 0
        for j, b in enumerate(ap["sizes"]):
            if ap["tier"][j] != nx.TIER_PAGEABLE:
                continue
            units = self.take_units(b // BLOCK)
            if units is None:
                continue
            nx.host_copy([self.pin.ctypes.data + units[0] * BLOCK], [ap["pageable"].ctypes.data + ap["offs"][j]], [b])
            ap["pageable"][ap["offs"][j]:ap["offs"][j] + b] = 0xDD          # exactly one copy: the old one is dead
            ap["tier"][j], ap["units"][j] = nx.TIER_PINNED, units
            moved += b
        return moved

    def activate(self, run, victims):
        nx = self.nx
        index, chunks = [], []
        for a, ap in enumerate(self.apps):
            for j, b in enumerate(ap["sizes"]):
                index.append((a, j))
                chunks.append((b, a, ap["tier"][j]))
        tier, summ, order = nx.place(self.pool.bytes, self.pinned_cap, chunks, run, victims)
        out_rows, in_rows, evicted, restored = [], [], [], []
        for k in order:                                                  # migration order: two-tier moves first
            a, j = index[k]
            ap = self.apps[a]
            if chunks[k][2] == nx.TIER_GPU:                              # leaves the GPU
                units = None
                new = tier[k]
                if new == nx.TIER_PINNED:
                    units = self.take_units(ap["sizes"][j] // BLOCK)
                    if units is None:                                    # fragmented pinned tier: go one tier further down
                        new = nx.TIER_PAGEABLE
                out_rows.append((ap["space"].base + ap["offs"][j], self.host_ptr(ap, j, new, units), ap["sizes"][j]))
                evicted.append((a, j, new, units))
            elif tier[k] == nx.TIER_GPU:
                restored.append((a, j))
        # physical blocks for the incoming chunks: free ones first, then the victims' (in eviction order)
        supply = list(self.free_blocks) + [b for a, j, _, _ in evicted for b in self.apps[a]["blocks"][j]]
        used = 0
        for a, j in restored:
            ap = self.apps[a]
            n = ap["sizes"][j] // BLOCK
            mine = supply[used:used + n]
            used += n
            assert len(mine) == n, "placement promised room that is not there"
            ap["space"].assign(ap["offs"][j], mine)
            ap["space"].map(ap["offs"][j], ap["sizes"][j])
            in_rows.append((ap["space"].base + ap["offs"][j], self.host_ptr(ap, j, ap["tier"][j]), ap["sizes"][j]))
            ap["new_blocks"] = ap.get("new_blocks", {})
            ap["new_blocks"][j] = mine
        st = None
        if out_rows or in_rows:
            plan = nx.Plan(out_rows, in_rows, 8 * MiB, nx.Opts(flags=nx.IN_PLACE))
            info = plan.info()
            self.last_info = info
            assert info["bytes_out"] == summ["evicted_bytes"] and info["bytes_in"] == summ["restored_bytes"]
            plan.switch_begin()
            plan.switch_wait_in()                                        # the application could run from here on
            st = plan.switch_end()
            plan.close()
        # bookkeeping after the switch
        taken = set(supply[:used])
        self.free_blocks = [b for b in self.free_blocks if b not in taken]
        for a, j, new, units in evicted:
            ap = self.apps[a]
            ap["space"].unmap(ap["offs"][j], ap["sizes"][j])
            self.free_blocks += [b for b in ap["blocks"][j] if b not in taken]
            ap["blocks"][j], ap["tier"][j], ap["units"][j] = None, new, units
        for a, j in restored:
            ap = self.apps[a]
            if ap["units"][j] is not None:
                self.free_units += ap["units"][j]
            ap["blocks"][j], ap["tier"][j], ap["units"][j] = ap["new_blocks"][j], nx.TIER_GPU, None
        return summ, st

    def check_everything(self):
        nx = self.nx
        owners = {}
        for a, ap in enumerate(self.apps):
            for j, (o, b) in enumerate(zip(ap["offs"], ap["sizes"])):
                want = W.content_bytes(100 + a, j, b)
                if ap["tier"][j] == nx.TIER_GPU:
                    got = self.raw.download(ap["space"].base + o, b)
                    for blk in ap["blocks"][j]:
                        assert blk not in owners, f"pool block {blk} has two owners"
                        owners[blk] = (a, j)
                elif ap["tier"][j] == nx.TIER_PINNED:
                    u = ap["units"][j][0]
                    got = self.pin[u * BLOCK:u * BLOCK + b]
                else:
                    got = ap["pageable"][o:o + b]
                assert np.array_equal(got, want), f"application {a} chunk {j} (tier {ap['tier'][j]}) lost its bytes"
        assert not (set(owners) & set(self.free_blocks))


def test_scheduler_placement_and_switch_together(nx):
    from tests.gpu_helpers import RawDevice
    raw = RawDevice(nx.lib_path())
    SEC, MS = 1_000_000_000, 1_000_000
    # chunks in blocks: 0 = a batch job (14 blocks), 1 and 2 = interactive applications (9 and 11 blocks);
    # the pool has 24 blocks: any two fit, all three do not; the pinned tier holds 6 blocks
    world = World(nx, raw, [[4, 3, 2, 5], [3, 3, 3], [2, 4, 1, 4]], pool_blocks=24, pinned_units=6)
    sched = nx.Sched()
    ids = [sched.add_app(0) for _ in world.apps]
    t, owner, log = 0, -1, []
    last_run = {a: -1 for a in ids}
    script = ([(0, [0])] + [(0, [])] * 4 + [(0, [1])] + [(1, [])] * 2 + [(1, [2])] + [(2, [])] * 2 + [(2, [0])] +
              [(-1, [])] * 2 + [(0, [1, 2])] + [(-1, [])] * 6)
    for step, (active, asking) in enumerate(script):
        t += 250 * MS
        if active >= 0 and active == owner:
            for k in range(1, 26):
                sched.api_return(active, t - 250 * MS + k * 10 * MS)
        for a in asking:
            sched.request(a, t - 5 * MS)
        d = sched.tick(t)
        if d["switched"]:
            run = d["run"]
            victims = sorted((a for a in ids if a != run), key=lambda a: last_run[a])   # least recently run goes first
            summ, st = world.activate(run, victims)
            world.check_everything()
            assert all(x == nx.TIER_GPU for x in world.apps[run]["tier"])
            log.append((run, summ["evicted_bytes"] // BLOCK, summ["kept_pinned_bytes"] // BLOCK,
                        summ["restored_bytes"] // BLOCK))
        if d["run"] >= 0:
            last_run[d["run"]] = step
        owner = d["run"]
    print("\n(run, evicted, kept in pinned tier, restored) in blocks:", log)
    assert len(log) >= 5
    assert log[0][1] == 0 and log[1][1] == 0            # the first two fit side by side: nothing is evicted
    assert any(e > 0 and k > 0 for _, e, k, _ in log)   # later someone has to go, partly into the pinned tier
    assert any(0 < e < 14 for _, e, _, _ in log)        # and only as far as needed (the batch job has 14 blocks)
    sched.close()
    world.close()


def test_prefetch_hint_is_acted_on_before_the_switch(nx):
    """Two applications of level 1, a pool that holds one of them.  While application 0 computes,
    application 1 asks for the GPU and has to wait for the end of the turn (S_1 = 4 s): every tick
    names it as the prefetch candidate, and the harness moves its chunks from pageable memory into
    the pinned tier as far as that has room.  The switch that follows then moves exactly those
    chunks directly (no ring slot, no host thread) and the rest through the ring, and every chunk of
    both applications holds its bytes before and after."""
    from tests.gpu_helpers import RawDevice
    raw = RawDevice(nx.lib_path())
    SEC, MS = 1_000_000_000, 1_000_000
    world = World(nx, raw, [[4, 3, 2], [3, 3, 3]], pool_blocks=10, pinned_units=6)
    sched = nx.Sched()
    a0, a1 = sched.add_app(0), sched.add_app(0)
    sched.request(a0, 0)
    d = sched.tick(0)
    assert d["run"] == a0 and d["switched"]
    world.activate(a0, [a1])
    world.check_everything()
    t, prefetched, hints, switched_at = 0, 0, 0, None
    while t < 6 * SEC and switched_at is None:
        t += 250 * MS
        for k in range(1, 26):                                   # application 0 computes without a pause
            sched.api_return(a0, t - 250 * MS + k * 10 * MS)
        if t == 1 * SEC:
            sched.request(a1, t - 5 * MS)
        d = sched.tick(t)
        if d["switched"]:
            assert d["run"] == a1 and d["evict"] == a0
            switched_at = t
            break
        if d["prefetch"] >= 0:
            assert d["prefetch"] == a1 and d["run"] == a0
            hints += 1
            prefetched += world.prefetch(d["prefetch"])          # idempotent once the tier is full
            world.check_everything()
    assert switched_at == 4 * SEC                                 # the turn of application 0 began at 0
    assert hints >= 10 and prefetched == 6 * BLOCK               # two of its three chunks fit the six units
    assert [x == nx.TIER_PINNED for x in world.apps[a1]["tier"]] == [True, True, False]
    summ, st = world.activate(a1, [a0])
    info = world.last_info
    assert info["direct_bytes_in"] == prefetched and info["bytes_in"] == 9 * BLOCK
    assert info["direct_bytes_out"] == 0                          # the pinned tier was full when the eviction was planned
    assert summ["restored_from_pageable_bytes"] == 3 * BLOCK
    world.check_everything()
    assert all(x == nx.TIER_GPU for x in world.apps[a1]["tier"]) and sorted(world.free_units) == list(range(6))
    sched.close()
    world.close()
