// Scheduler: who owns the GPU next, and therefore which context-switch swap to run.
//
// Paper, "Scheduling".  Idleness Detection: an application is idle once the time since its most
// recent API return exceeds a threshold (100 ms) unless it sits inside a blocking call.
// Priority Inference (Algorithm 1): an application that has used more than its level's
// allotment T_p is moved one queue down; an idle one is moved one queue up when its level has
// not changed for more than T_p and its idle time, less a share R < 1/N of the time it has been
// waiting in the queue, exceeds T_{p-1} plus the execution time it has accumulated.  MLFQ with
// Prefetching: K queues, the highest non-empty one is served, inside a queue the longest
// waiter first; the owner is preempted after S_p when someone waits at its level; T and S
// double from queue to queue; the head of the queue is the application worth prefetching.
//
// Pure host code, integer nanoseconds supplied by the caller (so a trace replays exactly).
// Choices the paper leaves open: R = 1/(N+1); a level change starts a fresh allotment; new
// applications enter the top queue; an idle owner yields to any waiter; execution time accrues
// from tick to tick while the owner is not idle.
#include <cstdint>
#include <new>
#include <vector>

#include "nixie.h"

namespace {

struct AppState {
    uint64_t last_return = 0;    // most recent API return
    uint64_t last_exec = 0;      // last tick at which it was executing
    uint64_t last_change = 0;    // last change of level
    uint64_t enqueued = 0;       // when its pending request was made
    uint64_t turn_start = 0;     // when it last got the GPU
    uint64_t exec_ns = 0;        // t_a: execution time accumulated at this level
    uint32_t level = 1;          // 1 = highest
    bool blocking = false, pending = false, running = false;
};

}  // namespace

struct nixie_sched {
    uint32_t levels = 4;
    uint64_t allot = 8000000000ull, preempt = 4000000000ull, idle = 100000000ull;
    std::vector<AppState> apps;
    std::vector<uint32_t> population;   // applications per level, index 1..levels
    int owner = -1;
    uint64_t accounted = 0;

    uint64_t T(uint32_t level) const { return allot << (level - 1); }
    uint64_t S(uint32_t level) const { return preempt << (level - 1); }
    bool is_idle(const AppState &a, uint64_t now) const { return !a.blocking && now - a.last_return > idle; }
    void move(AppState &a, uint32_t to, uint64_t now) {
        population[a.level]--;
        population[to]++;
        a.level = to;
        a.exec_ns = 0;
        a.last_change = now;
    }
};

extern "C" {

int nixie_sched_create(const nixie_sched_params_t *params, nixie_sched_t **sched) {
    if (!sched) return NIXIE_EINVAL;
    nixie_sched *s = new (std::nothrow) nixie_sched();
    if (!s) return NIXIE_ENOMEM;
    if (params) {
        if (params->levels) s->levels = params->levels;
        if (params->allot_ns) s->allot = params->allot_ns;
        if (params->preempt_ns) s->preempt = params->preempt_ns;
        if (params->idle_ns) s->idle = params->idle_ns;
    }
    if (s->levels > 16 || (s->allot >> 40) || (s->preempt >> 40)) {   // keeps T << (levels - 1) far from overflow
        delete s;
        return NIXIE_EINVAL;
    }
    s->population.assign(s->levels + 1, 0);
    *sched = s;
    return NIXIE_OK;
}

void nixie_sched_destroy(nixie_sched_t *sched) { delete sched; }

int nixie_sched_add_app(nixie_sched_t *s, uint64_t now_ns) {
    if (!s || s->apps.size() >= (1u << 20)) return NIXIE_EINVAL;
    AppState a;
    a.last_return = a.last_exec = a.last_change = now_ns;
    try {
        s->apps.push_back(a);
    } catch (const std::bad_alloc &) {
        return NIXIE_ENOMEM;
    }
    s->population[1]++;
    return (int)s->apps.size() - 1;
}

static AppState *app_of(nixie_sched_t *s, int app) {
    return (s && app >= 0 && (size_t)app < s->apps.size()) ? &s->apps[(size_t)app] : nullptr;
}

int nixie_sched_api_enter(nixie_sched_t *s, int app, uint64_t now_ns, int blocking) {
    AppState *a = app_of(s, app);
    if (!a) return NIXIE_EINVAL;
    (void)now_ns;
    if (blocking) a->blocking = true;
    return NIXIE_OK;
}

int nixie_sched_api_return(nixie_sched_t *s, int app, uint64_t now_ns) {
    AppState *a = app_of(s, app);
    if (!a) return NIXIE_EINVAL;
    a->last_return = now_ns;
    a->blocking = false;
    return NIXIE_OK;
}

int nixie_sched_request(nixie_sched_t *s, int app, uint64_t now_ns) {
    AppState *a = app_of(s, app);
    if (!a) return NIXIE_EINVAL;
    if (!a->running && !a->pending) {
        a->pending = true;
        a->enqueued = now_ns;
    }
    return NIXIE_OK;
}

int nixie_sched_tick(nixie_sched_t *s, uint64_t now, nixie_sched_decision_t *out) {
    if (!s || !out) return NIXIE_EINVAL;
    // execution time of the owner since the previous tick
    if (s->owner >= 0) {
        AppState &r = s->apps[(size_t)s->owner];
        if (!s->is_idle(r, now)) {
            r.exec_ns += now - s->accounted;
            r.last_exec = now;
        }
    }
    s->accounted = now;

    // priority inference, application by application (a move changes N for the ones after it)
    for (AppState &a : s->apps) {
        const uint32_t p = a.level;
        if (a.exec_ns > s->T(p)) {
            // The demotion branch ends with t_a <- 0 also in the lowest queue, where there is nowhere
            // to move to: the allotment restarts, level and time of the last change stay, and a later
            // long idle period can still lift the application again.
            if (p < s->levels) s->move(a, p + 1, now);
            else a.exec_ns = 0;
        } else if (p > 1 && s->is_idle(a, now) && now - a.last_change > s->T(p)) {
            const __int128 n1 = (__int128)s->population[p] + 1;                 // 1 / R
            const __int128 idle_for = (__int128)(now - a.last_exec);
            const __int128 queued_for = a.pending ? (__int128)(now - a.enqueued) : 0;
            if (n1 * idle_for - queued_for > n1 * ((__int128)s->T(p - 1) + (__int128)a.exec_ns)) s->move(a, p - 1, now);
        }
    }

    // the two best waiters: (level, waiting since, id) ascending
    int best = -1, second = -1;
    auto before = [&](int x, int y) {   // x is served before y
        const AppState &a = s->apps[(size_t)x], &b = s->apps[(size_t)y];
        if (a.level != b.level) return a.level < b.level;
        if (a.enqueued != b.enqueued) return a.enqueued < b.enqueued;
        return x < y;
    };
    for (int i = 0; i < (int)s->apps.size(); i++) {
        if (!s->apps[(size_t)i].pending) continue;
        if (best < 0 || before(i, best)) { second = best; best = i; }
        else if (second < 0 || before(i, second)) second = i;
    }

    out->run = s->owner;
    out->evict = -1;
    out->prefetch = best;
    out->switched = 0;
    if (best >= 0) {
        bool take;
        if (s->owner < 0 || s->is_idle(s->apps[(size_t)s->owner], now)) {
            take = true;
        } else {
            const AppState &r = s->apps[(size_t)s->owner], &b = s->apps[(size_t)best];
            take = b.level < r.level || (b.level == r.level && now - r.turn_start >= s->S(r.level));
        }
        if (take) {
            if (s->owner >= 0) {
                out->evict = s->owner;
                s->apps[(size_t)s->owner].running = false;
            }
            AppState &b = s->apps[(size_t)best];
            b.running = true;
            b.pending = false;
            b.turn_start = now;
            s->owner = best;
            out->run = best;
            out->switched = 1;
            out->prefetch = second;
        }
    }
    return NIXIE_OK;
}

int nixie_sched_app_info(const nixie_sched_t *s, int app, uint64_t now_ns, nixie_sched_app_t *out) {
    if (!s || !out || app < 0 || (size_t)app >= s->apps.size()) return NIXIE_EINVAL;
    const AppState &a = s->apps[(size_t)app];
    out->priority = a.level;
    out->exec_ns = a.exec_ns;
    out->idle = s->is_idle(a, now_ns) ? 1u : 0u;
    out->pending = a.pending ? 1u : 0u;
    out->running = a.running ? 1u : 0u;
    return NIXIE_OK;
}

}  // extern "C"
