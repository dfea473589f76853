"""Scheduler parity: the library's scheduler (through its C ABI) against the oracle, decision by
decision, on seeded synthetic application traces.

The paper's workloads (interactive chat / code completion next to long batch jobs, "Case
Studies") are not here; the traces stand in for them: interactive applications work in short
bursts separated by think time, batch applications compute for minutes, some calls block.
Both implementations see the same events; since every decision feeds back into what the
applications do next, they must agree at every single tick."""
import numpy as np
import pytest

from oracle import SchedOracle

SEC, MS = 1_000_000_000, 1_000_000


def simulate(seed, n_inter, n_batch, levels, allot, preempt, horizon_s, tick_ms=250):
    import paper_2601_11743_amd as nx
    rng = np.random.default_rng(seed)
    orc = SchedOracle(levels, allot, preempt)
    lib = nx.Sched(levels=levels, allot_ns=allot, preempt_ns=preempt)
    kinds = ["i"] * n_inter + ["b"] * n_batch
    apps = []
    for k in kinds:
        a, b = orc.add_app(0), lib.add_app(0)
        assert a == b
        apps.append(dict(kind=k, work=0, wake=int(rng.integers(0, 3 * SEC)), block_until=0))
    owner, decisions, switches = -1, 0, 0
    step = 10 * MS
    last_return_owner = 0
    for t in range(step, horizon_s * SEC + 1, step):
        for a, st in enumerate(apps):
            if st["work"] <= 0 and t >= st["wake"]:
                st["work"] = int(rng.integers(50, 3000)) * MS if st["kind"] == "i" else int(rng.integers(20, 120)) * SEC
            if st["work"] > 0:
                if a == owner:
                    if st["block_until"]:
                        if t >= st["block_until"]:            # a blocking call returns
                            orc.api_return(a, t); lib.api_return(a, t)
                            st["block_until"] = 0
                    elif rng.random() < 0.01:                 # a synchronisation that blocks for a while
                        orc.api_enter(a, t, True); lib.api_enter(a, t, True)
                        st["block_until"] = t + int(rng.integers(20, 400)) * MS
                    else:
                        orc.api_enter(a, t, False); lib.api_enter(a, t, False)
                        orc.api_return(a, t); lib.api_return(a, t)
                    st["work"] -= step
                    last_return_owner = t
                    if st["work"] <= 0:
                        st["block_until"] = 0
                        orc.api_return(a, t); lib.api_return(a, t)
                        think = int(rng.integers(1, 30)) * SEC if st["kind"] == "i" else int(rng.integers(1, 5)) * SEC
                        st["wake"] = t + think
                else:
                    orc.request(a, t); lib.request(a, t)
        idle_note = owner >= 0 and t - last_return_owner == 100 * MS + step   # idleness notification
        if t % (tick_ms * MS) == 0 or idle_note:
            d1, d2 = orc.tick(t), lib.tick(t)
            assert d1 == d2, f"seed {seed} t={t / SEC:.2f}s: oracle {d1} library {d2}"
            for a in range(len(apps)):
                assert orc.info(a, t) == lib.info(a, t), f"seed {seed} t={t / SEC:.2f}s app {a}"
            decisions += 1
            switches += d1["switched"]
            owner = d1["run"]
    levels_seen = {orc.info(a, horizon_s * SEC)["priority"] for a in range(len(apps))}
    lib.close()
    return decisions, switches, levels_seen


@pytest.mark.parametrize("seed,n_inter,n_batch,levels,allot_s,preempt_s", [
    (1, 2, 1, 4, 8, 4),        # the paper's constants
    (2, 1, 3, 4, 8, 4),
    (3, 3, 3, 4, 8, 4),
    (4, 2, 2, 3, 2, 1),        # short allotments: many level changes
    (5, 4, 2, 5, 1, 1),
    (6, 0, 4, 2, 4, 2),
    (7, 5, 0, 4, 8, 4),
    (8, 1, 1, 16, 1, 1),
])
def test_decisions_match_the_oracle(seed, n_inter, n_batch, levels, allot_s, preempt_s):
    decisions, switches, levels_seen = simulate(seed, n_inter, n_batch, levels, allot_s * SEC, preempt_s * SEC, 240)
    assert decisions >= 900
    if n_inter + n_batch > 1:
        assert switches > 5
    if n_batch:
        assert max(levels_seen) > 1            # somebody was demoted: the inference ran for real


def test_scheduler_abi_errors():
    import paper_2601_11743_amd as nx
    with pytest.raises(nx.NixieError):
        nx.Sched(levels=17)
    s = nx.Sched()
    a = s.add_app(0)
    with pytest.raises(nx.NixieError):
        s.request(a + 1, 0)
    with pytest.raises(nx.NixieError):
        s.info(-1, 0)
    assert s.tick(0) == {"run": -1, "evict": -1, "prefetch": -1, "switched": False}
    s.close()
