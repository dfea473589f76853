"""Pins for the scheduler oracle: traces whose outcome follows by hand from the constants the
paper states (100 ms idle threshold; T = 8 s, S = 4 s at the top level, doubling per level) and
from the inequalities of Algorithm 1."""
import pytest

from oracle import SchedOracle

SEC, MS = 1_000_000_000, 1_000_000


class _Product:
    """The library's scheduler behind the oracle's method names (so every pin runs on both)."""

    def __init__(self, levels=4, **kw):
        import paper_2601_11743_amd as nx
        self._s = nx.Sched(levels=levels, **kw)
        self.running = -1
        for name in ("add_app", "api_enter", "api_return", "request", "info"):
            setattr(self, name, getattr(self._s, name))

    def is_idle(self, a, now):
        return self._s.info(a, now)["idle"]

    def tick(self, now):
        d = self._s.tick(now)
        self.running = d["run"]
        return d


@pytest.fixture(params=["oracle", "library"])
def SchedImpl(request):
    return SchedOracle if request.param == "oracle" else _Product


def active(o, a, t0, t1, step=10 * MS):
    """Application a returns from an API call every `step` in (t0, t1]."""
    t = t0 + step
    while t <= t1:
        o.api_return(a, t)
        t += step


def test_idleness_threshold_and_blocking_calls(SchedImpl):
    o = SchedImpl()
    a = o.add_app(0)
    o.api_return(a, 1 * SEC)
    assert not o.is_idle(a, 1 * SEC + 100 * MS)        # exactly the threshold: not yet idle
    assert o.is_idle(a, 1 * SEC + 100 * MS + 1)
    o.api_enter(a, 2 * SEC, blocking=True)             # blocked inside the runtime is not idle
    assert not o.is_idle(a, 10 * SEC)
    o.api_return(a, 10 * SEC)
    assert not o.is_idle(a, 10 * SEC + 50 * MS) and o.is_idle(a, 10 * SEC + 101 * MS)
    o.api_enter(a, 11 * SEC, blocking=False)           # a launch does not hold idleness off
    assert o.is_idle(a, 11 * SEC + 200 * MS)


def test_demotion_times_follow_the_doubling_allotments(SchedImpl):
    """One application computing without pause, ticks every second: t_a first exceeds 8 s at the
    9th accrued second, then 16 s after 17 more, then 32 s after 33 more: 9 s, 26 s, 59 s."""
    o = SchedImpl(levels=4)
    a = o.add_app(0)
    o.request(a, 0)
    d = o.tick(0)
    assert d == {"run": a, "evict": -1, "prefetch": -1, "switched": True}
    changes = []
    level = 1
    for s in range(1, 200):
        active(o, a, (s - 1) * SEC, s * SEC)
        o.tick(s * SEC)
        if o.info(a, s * SEC)["priority"] != level:
            level = o.info(a, s * SEC)["priority"]
            changes.append((s, level))
    assert changes == [(9, 2), (26, 3), (59, 4)]       # and it stays in the lowest queue
    assert o.info(a, 199 * SEC)["priority"] == 4


def test_round_robin_at_the_preemption_threshold(SchedImpl):
    """Two applications that never pause, same level: turns of S_1 = 4 s, the longer waiter first."""
    o = SchedImpl()
    a, b = o.add_app(0), o.add_app(0)
    o.request(a, 0); o.request(b, 1)                   # a waits longer
    owner, switches, prefetch = [], [], {}
    for s in range(0, 17):
        t = s * SEC
        if s:
            r = o.running
            active(o, r, t - SEC, t)
            other = b if r == a else a
            o.request(other, t - SEC + 1)              # the one without the GPU keeps asking
        d = o.tick(t)
        if d["switched"]:
            switches.append((s, d["run"], d["evict"]))
        owner.append(d["run"])
        prefetch[s] = d["prefetch"]
    assert switches[:4] == [(0, a, -1), (4, b, a), (8, a, b), (12, b, a)]
    # while one computes, the other is the head of the queue: that is the prefetch candidate
    assert prefetch[1] == b and prefetch[5] == a and prefetch[13] == a
    assert prefetch[4] == -1                              # right after the swap nobody waits yet


def test_higher_level_preempts_at_once_and_idle_owner_yields(SchedImpl):
    o = SchedImpl()
    batch, inter = o.add_app(0), o.add_app(0)
    o.request(batch, 0)
    o.tick(0)
    for s in range(1, 12):                              # batch computes 11 s: demoted at 9 s
        active(o, batch, (s - 1) * SEC, s * SEC)
        o.tick(s * SEC)
    assert o.info(batch, 11 * SEC)["priority"] == 2
    o.request(inter, 11 * SEC + 5 * MS)                 # interactive application in Q_1 asks
    active(o, batch, 11 * SEC, 11 * SEC + 10 * MS)
    d = o.tick(11 * SEC + 10 * MS)                      # next decision point: preempted although its turn is young
    assert d["run"] == inter and d["evict"] == batch and d["switched"]
    # the interactive one works 300 ms, then falls silent; batch asks again and gets the GPU back
    # as soon as the owner is idle (> 100 ms after its last API return), whatever the levels
    active(o, inter, 11 * SEC + 10 * MS, 11 * SEC + 310 * MS)
    o.request(batch, 11 * SEC + 20 * MS)
    assert o.tick(11 * SEC + 400 * MS)["run"] == inter  # 90 ms of silence: not idle yet
    d = o.tick(11 * SEC + 411 * MS)
    assert d["run"] == batch and d["evict"] == inter
    assert d["prefetch"] == -1


def demote(o, a, upto_level):
    """Run a alone until it sits at upto_level; returns the time."""
    o.request(a, 0)
    s = 0
    o.tick(0)
    while o.info(a, s * SEC)["priority"] < upto_level:
        s += 1
        active(o, a, (s - 1) * SEC, s * SEC)
        o.tick(s * SEC)
    return s * SEC


def test_soft_promotion_needs_long_idleness_and_no_jitter(SchedImpl):
    """Level 3, t_a = 5 s there, then idle and not waiting: promoted when p_a > T_3 = 32 s and
    i_a > T_2 + t_a = 16 s + 5 s.  The first bound is the later one here."""
    o = SchedImpl()
    a = o.add_app(0)
    t0 = demote(o, a, 3)                                # reaches level 3 at 26 s
    assert t0 == 26 * SEC
    for s in range(1, 6):                               # 5 more seconds of execution at level 3
        active(o, a, t0 + (s - 1) * SEC, t0 + s * SEC)
        o.tick(t0 + s * SEC)
    assert o.info(a, t0 + 5 * SEC)["t_a"] == 5 * SEC
    last_exec = t0 + 5 * SEC
    hist = {}
    for s in range(1, 40):
        t = last_exec + s * SEC
        o.tick(t)
        hist[s] = o.info(a, t)["priority"]
    # i_a > 21 s holds from s = 22, p_a > 32 s (since 26 s) only from t > 58 s, i.e. s = 28
    assert hist[27] == 3 and hist[28] == 2
    # from level 2 the next step up needs p_a > T_2 = 16 s again and i_a > T_1 + 0 = 8 s: 17 s later
    t = last_exec + 28 * SEC
    for s in range(1, 18):
        o.tick(t + s * SEC)
    assert o.info(a, t + 16 * SEC)["priority"] in (1, 2)
    assert o.info(a, t + 17 * SEC)["priority"] == 1     # and never above the top level
    o.tick(t + 100 * SEC)
    assert o.info(a, t + 100 * SEC)["priority"] == 1


def test_pending_time_is_discounted_with_R_below_one_over_N(SchedImpl):
    """Same as above but the application is waiting in the queue behind a busy owner: with N
    applications at its level the condition is (N+1) i_a - q_a > (N+1)(T_{p-1} + t_a)."""
    o = SchedImpl(levels=3)
    a, hog = o.add_app(0), o.add_app(0)
    t0 = demote(o, a, 3)                                # a alone at level 3 at 26 s, t_a = 0
    o.request(hog, t0)                                  # hog (level 1) takes the GPU and keeps it busy
    active(o, a, t0, t0 + 10 * MS)
    o.tick(t0 + 10 * MS)
    assert o.running == hog
    last_exec = t0                                      # a last executed at the 26 s tick
    o.request(a, t0 + 1 * SEC)                          # a asks again and waits: q_a runs from 27 s
    promoted_at = None
    s = 1
    while promoted_at is None and s < 200:
        t = t0 + s * SEC
        active(o, hog, t - SEC, t)
        o.tick(t)
        if o.info(a, t)["priority"] == 2:
            promoted_at = s
        s += 1
    # N = 1 at level 3 (hog is demoted on its own clock but never shares level 3 before this):
    # 2 i_a - q_a > 2 * 16 s with i_a = s and q_a = s - 1  ->  s + 1 > 32  ->  s = 32, and p_a = s > 32 s -> s = 33
    assert promoted_at == 33


def test_bottom_queue_allotment_restarts_so_soft_promotion_stays_reachable(SchedImpl):
    """Algorithm 1's demotion branch ends with t_a <- 0 also where there is no lower queue to move to.
    K = 2 (T_1 = 8 s, T_2 = 16 s), one application computing without pause: level 2 at 9 s; at 26 s
    t_a = 17 s > T_2, it stays in Q_2 and its allotment restarts; 4 more seconds of work (t_a = 4 s at
    30 s), then silence.  p_a counts from 9 s (no priority change at 26 s), so p_a > T_2 already
    holds, and the promotion waits for i_a > T_1 + t_a = 12 s: the tick at 43 s."""
    o = SchedImpl(levels=2)
    a = o.add_app(0)
    o.request(a, 0)
    o.tick(0)
    level_at = {}
    for s in range(1, 31):
        active(o, a, (s - 1) * SEC, s * SEC)
        o.tick(s * SEC)
        level_at[s] = o.info(a, s * SEC)["priority"]
        if s == 25:
            assert o.info(a, s * SEC)["t_a"] == 16 * SEC       # not yet above T_2
        if s == 26:
            assert o.info(a, s * SEC)["t_a"] == 0              # restarted in place
    assert level_at[8] == 1 and level_at[9] == 2 and level_at[30] == 2
    assert o.info(a, 30 * SEC)["t_a"] == 4 * SEC
    promoted_at = None
    for s in range(31, 80):
        o.tick(s * SEC)
        if promoted_at is None and o.info(a, s * SEC)["priority"] == 1:
            promoted_at = s
    assert promoted_at == 43
