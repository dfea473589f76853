// libnixie_shim.so: the transparent shim for unmodified HIP applications (LD_PRELOAD).
//
// Paper, "Supporting Unmodified CUDA Applications": the shim interposes allocation and free,
// kernel launches and the memory report.  Large allocations become ranges of one reserved
// address space over a pool of physical blocks ("Maintaining consistent virtual memory
// addresses"), so the application keeps its pointers while its bytes are in host memory; before a
// migration new launches are held back and the device is synchronized ("Valid memory access during
// migration"); the memory report is the process's own sum ("GPU Memory information"); a launch
// checks the execution flag first and brings the application back when it is off ("Overview",
// steps 1, 2, 5, 6 of the architecture figure).  The migration itself is the library's
// context-switch swap (nixie_plan / nixie_switch).  One process, no daemon: the scheduler's side is
// nixie_shim_evict / nixie_shim_restore, or the shim's own idleness rule ("Idleness Detection").
#include <hip/hip_runtime_api.h>
#include <hip/hip_ext.h>

#include <dlfcn.h>
#include <sys/mman.h>
#include <time.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <shared_mutex>
#include <thread>
#include <unordered_map>
#include <vector>

#include "nixie.h"
#include "nixie_shim.h"
#include "blockruns.hpp"

namespace {

// ---- the runtime's own entry points -----------------------------------------------------------
template <typename F>
F next_symbol(const char *name) {
    void *p = dlsym(RTLD_NEXT, name);
    if (!p) {
        std::fprintf(stderr, "nixie-shim: the HIP runtime does not export %s\n", name);
        std::abort();   // nothing sensible can be returned for a call that cannot be forwarded
    }
    return reinterpret_cast<F>(p);
}
// (spelled out rather than taken from the declarations: the runtime's header overloads some of these names)
using fn_hipMalloc = hipError_t (*)(void **, size_t);
using fn_hipFree = hipError_t (*)(void *);
using fn_hipMemGetInfo = hipError_t (*)(size_t *, size_t *);
using fn_hipMemset = hipError_t (*)(void *, int, size_t);
using fn_hipDeviceSynchronize = hipError_t (*)(void);
using fn_hipStreamSynchronize = hipError_t (*)(hipStream_t);
#define REAL(name) ([]() { static fn_##name f = next_symbol<fn_##name>(#name); return f; }())

// Calls made by the shim itself (and by libnixie underneath it) pass straight through.
thread_local int t_inside = 0;
struct Inside {
    Inside() { t_inside++; }
    ~Inside() { t_inside--; }
};

uint64_t now_ns() {
    timespec ts;
    clock_gettime(CLOCK_MONOTONIC, &ts);
    return (uint64_t)ts.tv_sec * 1000000000ull + (uint64_t)ts.tv_nsec;
}

uint64_t env_u64(const char *name, uint64_t dflt) {
    const char *v = std::getenv(name);
    if (!v || !*v) return dflt;
    char *end = nullptr;
    const unsigned long long x = std::strtoull(v, &end, 10);
    return end && *end == 0 ? (uint64_t)x : dflt;
}

struct Alloc {
    uint64_t bytes = 0;      // as the application asked
    uint64_t units = 0;      // what it occupies, in allocation units
    void *host = nullptr;    // the pageable copy while evicted (exactly one live copy of the bytes at any time), else null
    // The mapping behind `host` is kept from one eviction to the next: after a restore its pages are
    // handed back lazily (MADV_FREE: the kernel may take them when it needs memory), so the next
    // eviction usually finds them still there and pays neither page faults nor zeroing -- with fresh
    // memory every time those cost three times what the transfer itself does.
    void *backing = nullptr;
};

struct Shim {
    bool ok = false;
    // Two granularities.  `unit` is what allocations are rounded to and the smallest managed allocation
    // (the paper's 2 MB block).  `block` is what the driver maps and unmaps at a time: it costs 0.03 - 0.05 ms
    // to map and 0.25 ms to unmap whatever its size, so it is larger (the paper, too, backs its 2 MB blocks
    // with physical chunks of up to 128 MB), and neighbouring allocations share one.
    uint64_t capacity = 0, unit = 0, block = 0, min_bytes = 0, ring = 0, idle_ns = 0;
    bool scribble = false, log = false;
    nixie_pool_t *pool = nullptr;
    nixie_space_t *space = nullptr;
    nixie_ring_t *staging = nullptr;   // the pinned ring, made at the first migration and kept: every later one reuses it
    uint64_t base = 0;

    // Launches hold `gate` shared; eviction and restore hold it exclusively, which is what holds
    // new launches back during a migration.  `mu` guards the tables.
    std::shared_mutex gate;
    std::mutex mu;
    std::map<uint64_t, Alloc> table;          // by device address
    nixie::BlockRuns free_runs;               // units of the space that no allocation holds
    // Which blocks of the space have physical memory mapped behind them.  A block is mapped when an
    // allocation first covers it and stays mapped when that allocation is freed (every block of the space
    // has its own physical block, so nothing is gained by taking it away, and the next allocation there
    // costs no driver call); only an eviction unmaps, everything, in the background, from block 0 up.
    std::vector<uint8_t> mapped;
    uint64_t reap_cursor = 0;                 // blocks below it have been dealt with since the last eviction
    uint64_t managed_bytes = 0;
    // Allocations below the threshold are the runtime's own, but they count in the process's memory
    // report like the others (paper, "GPU Memory information": the sum of the process's own allocations).
    std::unordered_map<const void *, uint64_t> small;
    uint64_t small_bytes = 0;
    std::atomic<bool> resident{true};
    std::atomic<uint32_t> evictions{0}, restores{0};
    std::atomic<uint64_t> last_switch_ns{0}, launches_held{0};

    // idleness: time of the last return from a runtime call; calls that may block are bracketed
    std::atomic<uint64_t> last_return{0};
    std::atomic<int> blocking{0};
    // stream captures in progress: until the last one ends the shim makes no runtime call of its own
    // (a synchronize or a copy from another thread would break the application's capture)
    std::atomic<int> captures{0};
    std::thread watcher;
    std::atomic<bool> quit{false};

    // Unmapping costs a driver call per block (0.25 ms each on MI355X) and nobody waits for it: the
    // evicted application cannot run, and whoever gets the physical blocks maps them at addresses of
    // its own.  It is done by this thread after the eviction, a few blocks at a time; an application
    // that comes back first simply keeps what is still mapped.
    int host_release = 0;   // what a restore does with the host copies' pages: 0 lazy release, 1 keep them, 2 return them at once
    bool sync_unmap = false;
    std::atomic<int> wanted_back{0};   // threads waiting to bring the application back: the background work gives way to them
    std::thread reaper;
    std::mutex reap_mu;
    std::condition_variable reap_cv;
    bool reap_pending = false;
};

Shim *g = nullptr;
std::once_flag g_once;

void say(const char *fmt, ...) __attribute__((format(printf, 1, 2)));
void say(const char *fmt, ...) {
    if (!g || !g->log) return;
    char line[512];   // one write per line: several threads log
    va_list ap;
    va_start(ap, fmt);
    const int n = std::vsnprintf(line, sizeof(line) - 1, fmt, ap);
    va_end(ap);
    if (n < 0) return;
    std::fprintf(stderr, "nixie-shim: %s\n", line);
}

int evict_locked(Shim &s);
int restore_locked(Shim &s);

void watch_idleness(Shim *s) {
    const timespec nap{0, (long)std::min<uint64_t>(s->idle_ns / 4 + 1, 20000000)};
    while (!s->quit.load()) {
        nanosleep(&nap, nullptr);
        if (!s->resident.load() || s->blocking.load() > 0 || s->captures.load() > 0) continue;
        const uint64_t last = s->last_return.load();
        if (last == 0 || now_ns() - last <= s->idle_ns) continue;
        std::unique_lock<std::shared_mutex> hold(s->gate);
        if (s->blocking.load() > 0 || now_ns() - s->last_return.load() <= s->idle_ns) continue;   // woke up meanwhile
        Inside in;
        (void)evict_locked(*s);
    }
}

// Unmap the next run of mapped blocks, `budget` at most; returns how many (0: none left).  Gate held
// exclusively, mu held.
uint64_t unmap_some(Shim &s, uint64_t budget) {
    const uint64_t n_blocks = s.mapped.size();
    while (s.reap_cursor < n_blocks && !s.mapped[s.reap_cursor]) s.reap_cursor++;
    uint64_t n = 0;
    while (s.reap_cursor + n < n_blocks && n < budget && s.mapped[s.reap_cursor + n]) n++;
    if (n == 0) return 0;
    const int u = nixie_space_unmap(s.space, s.reap_cursor * s.block, n * s.block);
    if (u == NIXIE_EBUSY) return 0;   // a switch of somebody else's is running: the next eviction starts over
    if (u)   // a block the driver refuses to unmap stays reserved until a restore maps over whatever state it finds
        std::fprintf(stderr, "nixie-shim: some blocks could not be unmapped (%s)\n", nixie_strerror(u));
    for (uint64_t b = 0; b < n; b++) s.mapped[s.reap_cursor + b] = 0;
    s.reap_cursor += n;
    return n;
}

// Map the blocks under units [first_unit, first_unit + n_units) that are not mapped yet.  mu held.
int map_range(Shim &s, uint64_t first_unit, uint64_t n_units) {
    const uint64_t first = first_unit * s.unit / s.block;
    const uint64_t count = ((first_unit + n_units) * s.unit + s.block - 1) / s.block - first;
    bool all = true;
    for (uint64_t b = first; b < first + count; b++) all = all && s.mapped[b];
    if (all) return NIXIE_OK;
    const int rc = nixie_space_map(s.space, first * s.block, count * s.block);   // skips what is mapped already
    if (rc == NIXIE_OK)
        for (uint64_t b = first; b < first + count; b++) s.mapped[b] = 1;
    return rc;
}

void reap_unmapped(Shim *s) {
    for (;;) {
        {
            std::unique_lock<std::mutex> lk(s->reap_mu);
            s->reap_cv.wait(lk, [&] { return s->quit.load() || s->reap_pending; });
            if (s->quit.load()) return;
            s->reap_pending = false;
        }
        const uint64_t t0 = now_ns();
        uint64_t total = 0;
        bool came_back = false;
        for (;;) {
            // (the lock has no queue: without this the loop could take it again and again ahead of a waiting restore)
            while (s->wanted_back.load() > 0 && !s->quit.load()) std::this_thread::sleep_for(std::chrono::microseconds(50));
            std::unique_lock<std::shared_mutex> hold(s->gate);   // short slices: a launch that wants the application back waits 4 ms at most
            if (s->quit.load()) return;
            if (s->resident.load()) { came_back = true; break; }
            Inside in;
            std::lock_guard<std::mutex> lk(s->mu);
            const uint64_t n = unmap_some(*s, 16);
            total += n;
            if (n == 0) break;
        }
        if (total || came_back)
            say("unmapped %llu blocks in the background in %.3f ms%s", (unsigned long long)total, (now_ns() - t0) / 1e6,
                came_back ? "; the application came back first and keeps the rest" : "");
    }
}

void init_once() {
    // Never destroyed: the application's own static destructors may still free memory through the
    // wrappers after this library's have run.
    static Shim &shim = *new Shim;
    Inside in;
    Shim &s = shim;
    s.capacity = env_u64("NIXIE_SHIM_POOL_MIB", 1024) << 20;
    s.unit = env_u64("NIXIE_SHIM_UNIT_MIB", 2) << 20;
    s.block = env_u64("NIXIE_SHIM_BLOCK_MIB", 32) << 20;
    if (s.unit == 0 || s.block % s.unit) {
        std::fprintf(stderr, "nixie-shim: the block size must be a multiple of the unit; allocations pass through\n");
        g = &s;
        return;
    }
    s.ring = env_u64("NIXIE_SHIM_RING_MIB", 64) << 20;
    s.idle_ns = env_u64("NIXIE_SHIM_IDLE_MS", 0) * 1000000ull;
    s.scribble = env_u64("NIXIE_SHIM_SCRIBBLE", 0) != 0;
    s.log = env_u64("NIXIE_SHIM_LOG", 0) != 0;
    s.sync_unmap = env_u64("NIXIE_SHIM_SYNC_UNMAP", 0) != 0;
    s.host_release = (int)std::min<uint64_t>(2, env_u64("NIXIE_SHIM_HOST_RELEASE", 0));
    g = &s;
    if (nixie_abi_check(sizeof(nixie_opts_t), sizeof(nixie_plan_info_t), sizeof(nixie_stats_t)) != NIXIE_OK) {
        std::fprintf(stderr, "nixie-shim: libnixie.so is of another version than this shim; allocations pass through\n");
        return;
    }
    int rc = nixie_pool_create(s.capacity, s.block, &s.pool);
    if (rc == NIXIE_EINVAL) {   // the device wants coarser blocks: take the library's default
        say("block of %llu MiB does not suit this device, using the default", (unsigned long long)(s.block >> 20));
        rc = nixie_pool_create(s.capacity, 0, &s.pool);
    }
    void *base = nullptr;
    if (!rc) rc = nixie_pool_info(s.pool, &s.capacity, &s.block);
    if (!rc && s.block % s.unit) rc = NIXIE_EINVAL;
    if (!rc) rc = nixie_space_create(s.pool, &s.space, &base);
    if (rc) {
        std::fprintf(stderr, "nixie-shim: cannot set up %llu MiB of managed GPU memory (%s); allocations pass through\n",
                     (unsigned long long)(s.capacity >> 20), nixie_strerror(rc));
        return;
    }
    s.base = (uint64_t)(uintptr_t)base;
    s.min_bytes = env_u64("NIXIE_SHIM_MIN_BYTES", s.unit);
    s.free_runs = nixie::BlockRuns(s.capacity / s.unit);
    s.mapped.assign(s.capacity / s.block, 0);
    s.last_return.store(now_ns());
    s.ok = true;
    say("managing %llu MiB in units of %llu MiB, mapped in blocks of %llu MiB, at %p, allocations from %llu bytes",
        (unsigned long long)(s.capacity >> 20), (unsigned long long)(s.unit >> 20), (unsigned long long)(s.block >> 20), base,
        (unsigned long long)s.min_bytes);
    if (s.idle_ns) s.watcher = std::thread(watch_idleness, &s);
    if (!s.sync_unmap) s.reaper = std::thread(reap_unmapped, &s);
    std::atexit([] {
        if (!g) return;
        {
            std::lock_guard<std::mutex> lk(g->reap_mu);
            g->quit.store(true);
        }
        g->reap_cv.notify_all();
        if (g->watcher.joinable()) g->watcher.join();
        if (g->reaper.joinable()) g->reaper.join();
    });
}

Shim *shim() {
    std::call_once(g_once, init_once);
    return g && g->ok ? g : nullptr;
}

// ---- the application's allocation table as a swap table -------------------------------------------
std::vector<nixie_alloc_t> rows_with_host_copy(Shim &s) {
    std::vector<nixie_alloc_t> rows;
    for (auto &kv : s.table)
        if (kv.second.host) rows.push_back(nixie_alloc_t{(void *)(uintptr_t)kv.first, kv.second.host, kv.second.bytes});
    return rows;
}

int run_switch(Shim &s, const std::vector<nixie_alloc_t> &out, const std::vector<nixie_alloc_t> &in) {
    nixie_table_t to{out.data(), out.size()}, ti{in.data(), in.size()};
    uint64_t moved = 0;
    for (auto &r : out) moved += r.bytes;
    for (auto &r : in) moved += r.bytes;
    if (moved == 0) return NIXIE_OK;
    nixie_plan_t *plan = nullptr;
    if (!s.staging && nixie_ring_create(s.ring, &s.staging) != NIXIE_OK) s.staging = nullptr;
    // (without a ring of its own the plan allocates one for this migration only)
    int rc = s.staging ? nixie_plan_on_ring(&to, &ti, s.staging, nullptr, &plan) : nixie_plan(&to, &ti, s.ring, nullptr, &plan);
    if (rc) return rc;
    nixie_stats_t st{};
    rc = nixie_switch(plan, nullptr, &st);
    nixie_plan_destroy(plan);
    return rc;
}

// gate held exclusively, t_inside set
int evict_locked(Shim &s) {
    if (!s.resident.load()) return NIXIE_OK;
    if (s.captures.load() > 0) return NIXIE_EBUSY;   // paper, "CUDA graph compatibility": hands off until the capture ends
    std::lock_guard<std::mutex> lk(s.mu);
    if (s.table.empty()) return NIXIE_OK;   // nothing of the application's is managed: nothing to take away
    const uint64_t t_begin = now_ns();
    if (REAL(hipDeviceSynchronize)() != hipSuccess) return NIXIE_EHIP;   // nothing of the application's is running any more
    const uint64_t t_quiet = now_ns();
    uint64_t bytes = 0;
    auto give_up = [&]() {   // the application stays resident, its bytes are still in HBM
        for (auto &u : s.table) u.second.host = nullptr;
    };
    for (auto &kv : s.table) {
        Alloc &a = kv.second;
        if (!a.backing) {
            void *m = mmap(nullptr, a.bytes, PROT_READ | PROT_WRITE, MAP_PRIVATE | MAP_ANONYMOUS, -1, 0);
            if (m == MAP_FAILED) { give_up(); return NIXIE_ENOMEM; }
            (void)madvise(m, a.bytes, MADV_HUGEPAGE);   // fewer, larger faults the first time, where the kernel offers them
            a.backing = m;
        }
        a.host = a.backing;
        bytes += a.bytes;
    }
    int rc = run_switch(s, rows_with_host_copy(s), {});
    if (rc) { give_up(); return rc; }
    const uint64_t t_moved = now_ns();
    // From here on the host copies are the application's memory; its blocks are unmapped behind its back.
    s.reap_cursor = 0;
    if (s.sync_unmap)
        while (unmap_some(s, ~0ull)) {}
    const uint64_t t_end = now_ns();
    if (s.scribble) {
        // what another application would do with the physical memory meanwhile
        nixie_space_t *other = nullptr;
        void *ob = nullptr;
        if (nixie_space_create(s.pool, &other, &ob) == NIXIE_OK) {
            if (nixie_space_map(other, 0, s.capacity) == NIXIE_OK) {
                (void)REAL(hipMemset)(ob, 0xEE, s.capacity);
                (void)REAL(hipDeviceSynchronize)();
            }
            (void)nixie_space_destroy(other);
        }
    }
    s.resident.store(false);
    s.evictions++;
    s.last_switch_ns.store(t_end - t_begin);
    say("evicted %zu allocations, %llu bytes, in %.3f ms (waiting for the device %.3f, swap %.3f, unmapping %.3f%s)", s.table.size(),
        (unsigned long long)bytes, (t_end - t_begin) / 1e6, (t_quiet - t_begin) / 1e6, (t_moved - t_quiet) / 1e6,
        (t_end - t_moved) / 1e6, s.sync_unmap ? "" : ": left to the background");
    if (!s.sync_unmap) {
        {
            std::lock_guard<std::mutex> lk(s.reap_mu);
            s.reap_pending = true;
        }
        s.reap_cv.notify_one();
    }
    return NIXIE_OK;
}

int restore_locked(Shim &s) {
    if (s.resident.load()) return NIXIE_OK;
    std::lock_guard<std::mutex> lk(s.mu);
    int rc = NIXIE_OK;
    const uint64_t t_begin = now_ns();
    for (auto &kv : s.table)
        if ((rc = map_range(s, (kv.first - s.base) / s.unit, kv.second.units)) != 0) return rc;
    const uint64_t t_mapped = now_ns();
    const std::vector<nixie_alloc_t> rows = rows_with_host_copy(s);   // allocations made while evicted have nothing to bring back
    rc = run_switch(s, {}, rows);
    if (rc) return rc;
    uint64_t bytes = 0;
    for (auto &kv : s.table) {
        Alloc &a = kv.second;
        if (!a.host) continue;
        a.host = nullptr;                                        // one copy: the bytes are in HBM again
        if (s.host_release == 1) {
            // kept as they are: the memory stays this process's
        } else if (s.host_release == 2 || madvise(a.backing, a.bytes, MADV_FREE) != 0) {   // (or no lazy release on this kernel)
            munmap(a.backing, a.bytes);
            a.backing = nullptr;
        }
        bytes += a.bytes;
    }
    s.resident.store(true);
    s.restores++;
    const uint64_t t_end = now_ns();
    s.last_switch_ns.store(t_end - t_begin);
    say("restored %zu allocations, %llu bytes, in %.3f ms (mapping %.3f, swap and release of the host copies %.3f)", rows.size(),
        (unsigned long long)bytes, (t_end - t_begin) / 1e6, (t_mapped - t_begin) / 1e6, (t_end - t_mapped) / 1e6);
    return NIXIE_OK;
}

// Around every interposed call of the application that uses device memory: the execution flag.
// Holds the gate shared for the duration of the call, so a migration cannot start underneath it.
struct Running {
    Shim *s;
    std::shared_lock<std::shared_mutex> hold;
    explicit Running(Shim *sh) : s(sh) {
        if (!s) return;
        s->blocking++;   // inside a runtime call the application is not idle, however long the call takes
        hold = std::shared_lock<std::shared_mutex>(s->gate);
        while (!s->resident.load()) {          // step 2: not runnable -> ask for the GPU, wait for the memory
            hold.unlock();
            s->launches_held++;
            {
                s->wanted_back++;
                std::unique_lock<std::shared_mutex> x(s->gate);
                s->wanted_back--;
                Inside in;
                const int rc = restore_locked(*s);
                if (rc) {
                    std::fprintf(stderr, "nixie-shim: cannot bring the application back (%s)\n", nixie_strerror(rc));
                    std::abort();   // its pointers have nothing behind them: no call can go ahead
                }
            }
            hold.lock();
        }
    }
    ~Running() {
        if (!s) return;
        s->last_return.store(now_ns());
        s->blocking--;
    }
};

}  // namespace

extern "C" {

hipError_t hipMalloc(void **ptr, size_t size) {
    if (t_inside) return REAL(hipMalloc)(ptr, size);
    Shim *s = shim();
    if (!s || !ptr || size < s->min_bytes) {
        const hipError_t e = REAL(hipMalloc)(ptr, size);
        if (s && e == hipSuccess && ptr && *ptr) {
            std::lock_guard<std::mutex> lk(s->mu);
            s->small[*ptr] = size;
            s->small_bytes += size;
        }
        if (s) s->last_return.store(now_ns());
        return e;
    }
    std::shared_lock<std::shared_mutex> hold(s->gate);   // not in the middle of a migration
    Inside in;
    std::lock_guard<std::mutex> lk(s->mu);
    const uint64_t need = (size + s->unit - 1) / s->unit;
    const uint64_t first = s->free_runs.find(need);
    // an evicted application's new memory gets its physical blocks when the application comes back
    if (first != nixie::BlockRuns::kNone && (!s->resident.load() || map_range(*s, first, need) == NIXIE_OK)) {
        s->free_runs.take(first, need);
        const uint64_t addr = s->base + first * s->unit;
        Alloc fresh;
        fresh.bytes = size;
        fresh.units = need;
        s->table[addr] = fresh;
        s->managed_bytes += need * s->unit;
        *ptr = (void *)(uintptr_t)addr;
        s->last_return.store(now_ns());
        return hipSuccess;
    }
    s->last_return.store(now_ns());
    return hipErrorOutOfMemory;
}

hipError_t hipFree(void *ptr) {
    if (t_inside) return REAL(hipFree)(ptr);
    Shim *s = shim();
    if (s && ptr) {
        std::shared_lock<std::shared_mutex> hold(s->gate);
        Inside in;
        std::unique_lock<std::mutex> lk(s->mu);
        auto it = s->table.find((uint64_t)(uintptr_t)ptr);
        if (it != s->table.end()) {
            const Alloc a = it->second;
            if (s->resident.load()) {
                lk.unlock();
                (void)REAL(hipDeviceSynchronize)();   // as the runtime's hipFree does: nothing may still use it
                lk.lock();
            }
            // (its blocks stay mapped for whoever is given these addresses next; an eviction takes them away)
            if (a.backing) munmap(a.backing, a.bytes);
            const uint64_t first = (it->first - s->base) / s->unit;
            s->table.erase(it);
            s->managed_bytes -= a.units * s->unit;
            s->free_runs.give(first, a.units);
            s->last_return.store(now_ns());
            return hipSuccess;
        }
        auto sm = s->small.find(ptr);
        if (sm != s->small.end()) {
            s->small_bytes -= sm->second;
            s->small.erase(sm);
        }
    }
    const hipError_t e = REAL(hipFree)(ptr);
    if (s) s->last_return.store(now_ns());
    return e;
}

hipError_t hipMemGetInfo(size_t *free_bytes, size_t *total_bytes) {
    if (t_inside) return REAL(hipMemGetInfo)(free_bytes, total_bytes);
    Shim *s = shim();
    if (!s) return REAL(hipMemGetInfo)(free_bytes, total_bytes);
    if (!free_bytes || !total_bytes) return hipErrorInvalidValue;
    std::lock_guard<std::mutex> lk(s->mu);
    *total_bytes = s->capacity;
    const uint64_t used = s->managed_bytes + s->small_bytes;
    *free_bytes = used < s->capacity ? s->capacity - used : 0;
    s->last_return.store(now_ns());
    return hipSuccess;
}

// Everything that launches work or touches device memory checks the execution flag first (and brings
// the application back if it is off), and holds the gate shared while the runtime call is in
// progress.  Same prototypes as the runtime's; the compiler checks them against its header.
#define NIXIE_GUARDED(name, params, args)                   \
    hipError_t name params {                                \
        using fn = hipError_t(*) params;                    \
        static const fn real = next_symbol<fn>(#name);      \
        if (t_inside) return real args;                     \
        Running r(shim());                                  \
        return real args;                                   \
    }

NIXIE_GUARDED(hipLaunchKernel,
              (const void *function_address, dim3 numBlocks, dim3 dimBlocks, void **args, size_t sharedMemBytes, hipStream_t stream),
              (function_address, numBlocks, dimBlocks, args, sharedMemBytes, stream))
NIXIE_GUARDED(hipLaunchCooperativeKernel,
              (const void *f, dim3 gridDim, dim3 blockDimX, void **kernelParams, unsigned int sharedMemBytes, hipStream_t stream),
              (f, gridDim, blockDimX, kernelParams, sharedMemBytes, stream))
NIXIE_GUARDED(hipLaunchKernelExC, (const hipLaunchConfig_t *config, const void *fPtr, void **args), (config, fPtr, args))
NIXIE_GUARDED(hipModuleLaunchKernel,
              (hipFunction_t f, unsigned int gridDimX, unsigned int gridDimY, unsigned int gridDimZ, unsigned int blockDimX,
               unsigned int blockDimY, unsigned int blockDimZ, unsigned int sharedMemBytes, hipStream_t stream,
               void **kernelParams, void **extra),
              (f, gridDimX, gridDimY, gridDimZ, blockDimX, blockDimY, blockDimZ, sharedMemBytes, stream, kernelParams, extra))
NIXIE_GUARDED(hipModuleLaunchCooperativeKernel,
              (hipFunction_t f, unsigned int gridDimX, unsigned int gridDimY, unsigned int gridDimZ, unsigned int blockDimX,
               unsigned int blockDimY, unsigned int blockDimZ, unsigned int sharedMemBytes, hipStream_t stream,
               void **kernelParams),
              (f, gridDimX, gridDimY, gridDimZ, blockDimX, blockDimY, blockDimZ, sharedMemBytes, stream, kernelParams))
NIXIE_GUARDED(hipExtModuleLaunchKernel,
              (hipFunction_t f, uint32_t globalWorkSizeX, uint32_t globalWorkSizeY, uint32_t globalWorkSizeZ,
               uint32_t localWorkSizeX, uint32_t localWorkSizeY, uint32_t localWorkSizeZ, size_t sharedMemBytes,
               hipStream_t hStream, void **kernelParams, void **extra, hipEvent_t startEvent, hipEvent_t stopEvent,
               uint32_t flags),
              (f, globalWorkSizeX, globalWorkSizeY, globalWorkSizeZ, localWorkSizeX, localWorkSizeY, localWorkSizeZ,
               sharedMemBytes, hStream, kernelParams, extra, startEvent, stopEvent, flags))

NIXIE_GUARDED(hipMemcpy, (void *dst, const void *src, size_t sizeBytes, hipMemcpyKind kind), (dst, src, sizeBytes, kind))
NIXIE_GUARDED(hipMemcpyAsync, (void *dst, const void *src, size_t sizeBytes, hipMemcpyKind kind, hipStream_t stream),
              (dst, src, sizeBytes, kind, stream))
NIXIE_GUARDED(hipMemcpyWithStream, (void *dst, const void *src, size_t sizeBytes, hipMemcpyKind kind, hipStream_t stream),
              (dst, src, sizeBytes, kind, stream))
NIXIE_GUARDED(hipMemcpyHtoD, (hipDeviceptr_t dst, const void *src, size_t sizeBytes), (dst, src, sizeBytes))
NIXIE_GUARDED(hipMemcpyDtoH, (void *dst, hipDeviceptr_t src, size_t sizeBytes), (dst, src, sizeBytes))
NIXIE_GUARDED(hipMemcpyDtoD, (hipDeviceptr_t dst, hipDeviceptr_t src, size_t sizeBytes), (dst, src, sizeBytes))
NIXIE_GUARDED(hipMemcpyHtoDAsync, (hipDeviceptr_t dst, const void *src, size_t sizeBytes, hipStream_t stream),
              (dst, src, sizeBytes, stream))
NIXIE_GUARDED(hipMemcpyDtoHAsync, (void *dst, hipDeviceptr_t src, size_t sizeBytes, hipStream_t stream),
              (dst, src, sizeBytes, stream))
NIXIE_GUARDED(hipMemcpyDtoDAsync, (hipDeviceptr_t dst, hipDeviceptr_t src, size_t sizeBytes, hipStream_t stream),
              (dst, src, sizeBytes, stream))
NIXIE_GUARDED(hipMemset, (void *dst, int value, size_t sizeBytes), (dst, value, sizeBytes))
NIXIE_GUARDED(hipMemsetAsync, (void *dst, int value, size_t sizeBytes, hipStream_t stream), (dst, value, sizeBytes, stream))
NIXIE_GUARDED(hipMemsetD8, (hipDeviceptr_t dest, unsigned char value, size_t count), (dest, value, count))
NIXIE_GUARDED(hipMemsetD8Async, (hipDeviceptr_t dest, unsigned char value, size_t count, hipStream_t stream),
              (dest, value, count, stream))
NIXIE_GUARDED(hipMemsetD32, (hipDeviceptr_t dest, int value, size_t count), (dest, value, count))
NIXIE_GUARDED(hipMemsetD32Async, (hipDeviceptr_t dst, int value, size_t count, hipStream_t stream), (dst, value, count, stream))

// A launched graph runs kernels that hold the application's pointers: the addresses stay valid across
// a migration, so the graph needs no patching, only the same flag check as a launch.
NIXIE_GUARDED(hipGraphLaunch, (hipGraphExec_t graphExec, hipStream_t stream), (graphExec, stream))

// Paper, "CUDA graph compatibility": the start and the end of a stream capture are interposed so that
// no migration (which synchronizes the device and launches work of its own) falls into a capture.
// The capture starts with the application resident, and evictions are refused until it has ended.
hipError_t hipStreamBeginCapture(hipStream_t stream, hipStreamCaptureMode mode) {
    using fn = hipError_t (*)(hipStream_t, hipStreamCaptureMode);
    static const fn real = next_symbol<fn>("hipStreamBeginCapture");
    if (t_inside) return real(stream, mode);
    Shim *s = shim();
    Running r(s);
    const hipError_t e = real(stream, mode);
    if (s && e == hipSuccess) s->captures++;
    return e;
}

hipError_t hipStreamBeginCaptureToGraph(hipStream_t stream, hipGraph_t graph, const hipGraphNode_t *dependencies,
                                        const hipGraphEdgeData *dependencyData, size_t numDependencies,
                                        hipStreamCaptureMode mode) {
    using fn = hipError_t (*)(hipStream_t, hipGraph_t, const hipGraphNode_t *, const hipGraphEdgeData *, size_t,
                              hipStreamCaptureMode);
    static const fn real = next_symbol<fn>("hipStreamBeginCaptureToGraph");
    if (t_inside) return real(stream, graph, dependencies, dependencyData, numDependencies, mode);
    Shim *s = shim();
    Running r(s);
    const hipError_t e = real(stream, graph, dependencies, dependencyData, numDependencies, mode);
    if (s && e == hipSuccess) s->captures++;
    return e;
}

hipError_t hipStreamEndCapture(hipStream_t stream, hipGraph_t *pGraph) {
    using fn = hipError_t (*)(hipStream_t, hipGraph_t *);
    static const fn real = next_symbol<fn>("hipStreamEndCapture");
    if (t_inside) return real(stream, pGraph);
    Shim *s = shim();
    const hipError_t e = real(stream, pGraph);
    if (s) {
        // the capture is over whether it produced a graph or not (an invalidated one ends here too)
        int have = s->captures.load();
        while (have > 0 && !s->captures.compare_exchange_weak(have, have - 1)) {}
        s->last_return.store(now_ns());
    }
    return e;
}

// Creating and destroying streams changes runtime state that a migration's own calls walk through
// (the paper's shim intercepts stream creation as well, as a call that allocates implicitly): such a
// call never overlaps a migration, but it needs no memory behind the application's pointers.
#define NIXIE_NOT_DURING_MIGRATION(name, params, args)      \
    hipError_t name params {                                \
        using fn = hipError_t(*) params;                    \
        static const fn real = next_symbol<fn>(#name);      \
        Shim *s = t_inside ? nullptr : shim();              \
        if (!s) return real args;                           \
        std::shared_lock<std::shared_mutex> hold(s->gate);  \
        const hipError_t e = real args;                     \
        s->last_return.store(now_ns());                     \
        return e;                                           \
    }
NIXIE_NOT_DURING_MIGRATION(hipStreamCreate, (hipStream_t * stream), (stream))
NIXIE_NOT_DURING_MIGRATION(hipStreamCreateWithFlags, (hipStream_t * stream, unsigned int flags), (stream, flags))
NIXIE_NOT_DURING_MIGRATION(hipStreamDestroy, (hipStream_t stream), (stream))

// Calls that neither block nor touch device memory, but with which an application polls or keeps a
// stream busy: their return counts as a sign of life (paper, "Idleness Detection": idle = no runtime
// call has returned for longer than the threshold), or a program that waits by polling would be evicted
// in the middle of its work.
#define NIXIE_SEEN(name, params, args)                          \
    hipError_t name params {                                    \
        using fn = hipError_t(*) params;                        \
        static const fn real = next_symbol<fn>(#name);          \
        const hipError_t e = real args;                         \
        if (!t_inside)                                          \
            if (Shim *s = shim()) s->last_return.store(now_ns()); \
        return e;                                               \
    }
NIXIE_SEEN(hipEventQuery, (hipEvent_t event), (event))
NIXIE_SEEN(hipStreamQuery, (hipStream_t stream), (stream))
NIXIE_SEEN(hipEventRecord, (hipEvent_t event, hipStream_t stream), (event, stream))
NIXIE_SEEN(hipStreamWaitEvent, (hipStream_t stream, hipEvent_t event, unsigned int flags), (stream, event, flags))

// Blocking calls are bracketed so that an application waiting inside the runtime is not taken for idle.
hipError_t hipDeviceSynchronize(void) {
    if (t_inside) return REAL(hipDeviceSynchronize)();
    Shim *s = shim();
    if (s) s->blocking++;
    const hipError_t e = REAL(hipDeviceSynchronize)();
    if (s) { s->blocking--; s->last_return.store(now_ns()); }
    return e;
}

hipError_t hipStreamSynchronize(hipStream_t stream) {
    if (t_inside) return REAL(hipStreamSynchronize)(stream);
    Shim *s = shim();
    if (s) s->blocking++;
    const hipError_t e = REAL(hipStreamSynchronize)(stream);
    if (s) { s->blocking--; s->last_return.store(now_ns()); }
    return e;
}

hipError_t hipEventSynchronize(hipEvent_t event) {
    using fn = hipError_t (*)(hipEvent_t);
    static const fn real = next_symbol<fn>("hipEventSynchronize");
    if (t_inside) return real(event);
    Shim *s = shim();
    if (s) s->blocking++;
    const hipError_t e = real(event);
    if (s) { s->blocking--; s->last_return.store(now_ns()); }
    return e;
}

int nixie_shim_info(nixie_shim_info_t *info) {
    if (!info || !g || !g->ok) return NIXIE_EINVAL;
    Shim &s = *g;
    std::lock_guard<std::mutex> lk(s.mu);
    info->capacity_bytes = s.capacity;
    info->block_bytes = s.block;
    info->unit_bytes = s.unit;
    info->managed_bytes = s.managed_bytes;
    info->managed_allocs = s.table.size();
    info->passthrough_allocs = s.small.size();
    info->passthrough_bytes = s.small_bytes;
    info->resident = s.resident.load() ? 1u : 0u;
    info->evictions = s.evictions.load();
    info->restores = s.restores.load();
    info->last_switch_ns = s.last_switch_ns.load();
    info->launches_held = s.launches_held.load();
    info->mapped_blocks = 0;
    for (uint8_t m : s.mapped) info->mapped_blocks += m;
    info->host_backing_bytes = 0;
    for (auto &kv : s.table)
        if (kv.second.backing) info->host_backing_bytes += kv.second.bytes;
    return NIXIE_OK;
}

int nixie_shim_evict(void) {
    Shim *s = shim();
    if (!s) return NIXIE_EINVAL;
    std::unique_lock<std::shared_mutex> hold(s->gate);
    Inside in;
    return evict_locked(*s);
}

int nixie_shim_restore(void) {
    Shim *s = shim();
    if (!s) return NIXIE_EINVAL;
    s->wanted_back++;
    std::unique_lock<std::shared_mutex> hold(s->gate);
    s->wanted_back--;
    Inside in;
    return restore_locked(*s);
}

}  // extern "C"
