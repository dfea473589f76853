"""CPU oracle of the scheduler (idleness detection, priority inference, MLFQ).  TEST INFRASTRUCTURE.

Plain Python, integer nanoseconds, written in the paper's order and notation; it shares nothing
with the library's scheduler and never imports it.

What it follows
  * "Idleness Detection": an application is idle iff the time since its most recent API return
    exceeds a fixed threshold (100 ms) and it is not inside a blocking call.
  * "Priority Inference", Algorithm 1: demotion when the execution time t_a accumulated at the
    current priority exceeds the allotment T_p; otherwise, for an idle application, soft
    promotion when p_a > T_p and i_a - R*q_a > T_{p-1} + t_a, with R < 1/N.
  * "MLFQ with Prefetching": K queues, Q_1 the highest; higher levels first, round-robin inside
    a level starting with the longest waiter; a running application is preempted after S_p if
    another one waits at its level; T = 8 s and S = 4 s at the top, doubling per level; the head
    of the queue is the prefetch candidate.  The scheduler runs these steps periodically and on
    an idleness notification.

Readings where the paper is silent (also listed in the design notes): R = 1/(N+1); an
application whose level changes starts with t_a = 0 there; new applications start in Q_1; a
running application that is idle yields to any waiting application; execution time accrues, tick
to tick, while the application owns the GPU and is not idle; "time since last execution" counts
from the last tick at which it was executing (or from its creation); in the lowest queue Q_K the
demotion branch has no queue to move to but still ends with t_a <- 0 as the algorithm prints it
(the priority, and so p_a, is unchanged), which keeps the idle branch reachable for an
application that once outran T_K.
"""
from __future__ import annotations

from dataclasses import dataclass

SEC = 1_000_000_000
MS = 1_000_000


@dataclass
class App:
    created: int
    p: int = 1                 # priority level, 1 = highest
    t_a: int = 0               # execution time accumulated at the current priority
    last_api_return: int = 0
    in_blocking: bool = False
    last_exec: int = 0         # last tick at which it was executing
    last_prio_change: int = 0
    pending: bool = False
    enqueued: int = 0
    running: bool = False
    turn_start: int = 0


class SchedOracle:
    def __init__(self, levels: int = 4, allot_ns: int = 8 * SEC, preempt_ns: int = 4 * SEC, idle_ns: int = 100 * MS):
        self.K, self.T1, self.S1, self.idle_ns = levels, allot_ns, preempt_ns, idle_ns
        self.apps: list[App] = []
        self.running: int = -1
        self.last_account = 0

    def T(self, p: int) -> int:
        return self.T1 * 2 ** (p - 1)

    def S(self, p: int) -> int:
        return self.S1 * 2 ** (p - 1)

    # ---- events -----------------------------------------------------------------------
    def add_app(self, now: int) -> int:
        self.apps.append(App(created=now, last_api_return=now, last_exec=now, last_prio_change=now))
        return len(self.apps) - 1

    def api_enter(self, a: int, now: int, blocking: bool) -> None:
        if blocking:
            self.apps[a].in_blocking = True

    def api_return(self, a: int, now: int) -> None:
        self.apps[a].last_api_return = now
        self.apps[a].in_blocking = False

    def request(self, a: int, now: int) -> None:
        app = self.apps[a]
        if not app.running and not app.pending:
            app.pending, app.enqueued = True, now

    def is_idle(self, a: int, now: int) -> bool:
        app = self.apps[a]
        return (not app.in_blocking) and now - app.last_api_return > self.idle_ns

    # ---- the periodic step ------------------------------------------------------------------
    def tick(self, now: int) -> dict:
        # execution time of the running application since the previous tick
        if self.running >= 0:
            r = self.apps[self.running]
            if not self.is_idle(self.running, now):
                r.t_a += now - self.last_account
                r.last_exec = now
        self.last_account = now

        # Algorithm 1 for every application
        for a, app in enumerate(self.apps):
            p = app.p
            if app.t_a > self.T(p):                               # standard MLFQ demotion
                if p < self.K:
                    app.p, app.last_prio_change = p + 1, now
                app.t_a = 0                                       # also in Q_K, where there is no lower queue
            elif self.is_idle(a, now):
                i_a = now - app.last_exec                          # time since last execution
                p_a = now - app.last_prio_change                   # time since last priority change
                q_a = now - app.enqueued if app.pending else 0     # time since enqueued (0 if no request)
                if p_a > self.T(p) and p > 1:                      # prevent priority jitter
                    N = sum(1 for o in self.apps if o.p == p)
                    # i_a - R*q_a > T_{p-1} + t_a with R = 1/(N+1), in integers
                    if (N + 1) * i_a - q_a > (N + 1) * (self.T(p - 1) + app.t_a):
                        app.p, app.t_a, app.last_prio_change = p - 1, 0, now

        # who runs: highest level first, inside a level the longest waiter
        waiting = sorted((app.p, app.enqueued, a) for a, app in enumerate(self.apps) if app.pending)
        evict, switched = -1, False
        if waiting:
            bp, _, b = waiting[0]
            take = False
            if self.running < 0 or self.is_idle(self.running, now):
                take = True
            else:
                r = self.apps[self.running]
                take = bp < r.p or (bp == r.p and now - r.turn_start >= self.S(r.p))
            if take:
                if self.running >= 0:
                    evict = self.running
                    self.apps[evict].running = False
                nb = self.apps[b]
                nb.running, nb.pending, nb.turn_start = True, False, now
                self.running, switched = b, True
                waiting = waiting[1:]
        prefetch = waiting[0][2] if waiting else -1
        return {"run": self.running, "evict": evict, "prefetch": prefetch, "switched": switched}

    def info(self, a: int, now: int) -> dict:
        app = self.apps[a]
        return {"priority": app.p, "t_a": app.t_a, "idle": self.is_idle(a, now), "pending": app.pending,
                "running": app.running}
