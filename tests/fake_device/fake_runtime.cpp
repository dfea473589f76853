// A CPU stand-in for everything the transparent shim calls: the few HIP runtime entry points it
// forwards to and the libnixie calls it makes.  Built as a shared library and linked BEHIND a test
// program that contains the shim's own source, so that the shim's wrappers come first in symbol
// order and find these through dlsym(RTLD_NEXT), exactly as under LD_PRELOAD.  The point is the
// shim's own logic -- execution flag, gate, idleness rule, allocation table -- under
// ThreadSanitizer, with several application threads; nothing here is shared with the library.
//
// Model: "device memory" is host memory.  Launches are asynchronous: one executor thread runs them
// in order, and only the synchronizing calls wait for it.  A "kernel" is a plain function taking
// three 64-bit arguments.  A space is a reserved address range; map makes blocks accessible (with
// arbitrary contents, as fresh physical memory has), unmap discards their contents and makes them
// inaccessible again, so that a launch that slips past the execution flag while the application is
// evicted dies on the spot, and a migration that starts before outstanding kernels have finished is
// a data race ThreadSanitizer reports.
#include <hip/hip_runtime_api.h>
#include <sys/mman.h>

#include <atomic>
#include <condition_variable>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <functional>
#include <mutex>
#include <thread>
#include <vector>

#include "nixie.h"

namespace {

struct Executor {
    std::mutex mu;
    std::condition_variable cv_work, cv_done;
    std::deque<std::function<void()>> queue;
    uint64_t submitted = 0, completed = 0;
    bool quit = false;
    std::thread th;
    Executor() : th([this] { run(); }) {}
    ~Executor() {
        {
            std::lock_guard<std::mutex> g(mu);
            quit = true;
        }
        cv_work.notify_all();
        th.join();
    }
    void run() {
        for (;;) {
            std::function<void()> job;
            {
                std::unique_lock<std::mutex> lk(mu);
                cv_work.wait(lk, [&] { return quit || !queue.empty(); });
                if (queue.empty()) return;
                job = std::move(queue.front());
                queue.pop_front();
            }
            job();
            {
                std::lock_guard<std::mutex> g(mu);
                completed++;
            }
            cv_done.notify_all();
        }
    }
    void submit(std::function<void()> job) {
        {
            std::lock_guard<std::mutex> g(mu);
            queue.push_back(std::move(job));
            submitted++;
        }
        cv_work.notify_one();
    }
    void drain() {   // everything submitted before this call has run
        std::unique_lock<std::mutex> lk(mu);
        const uint64_t upto = submitted;
        cv_done.wait(lk, [&] { return completed >= upto; });
    }
};

Executor &executor() {
    static Executor e;
    return e;
}

std::atomic<int> g_captures{0};

}  // namespace

struct nixie_pool { uint64_t bytes, block; int spaces; };
struct nixie_space { nixie_pool *pool; uint8_t *base; std::vector<uint8_t> mapped; };
struct nixie_ring { int unused; };
struct nixie_plan { std::vector<nixie_alloc_t> out, in; };

extern "C" {

// ---- HIP ------------------------------------------------------------------------------------------
hipError_t hipMalloc(void **p, size_t n) {
    return posix_memalign(p, 256, n ? n : 1) == 0 ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipFree(void *p) {
    executor().drain();
    std::free(p);
    return hipSuccess;
}
hipError_t hipMemGetInfo(size_t *f, size_t *t) { *f = 1ull << 36; *t = 1ull << 38; return hipSuccess; }
hipError_t hipDeviceSynchronize(void) { executor().drain(); return hipSuccess; }
hipError_t hipStreamSynchronize(hipStream_t) { executor().drain(); return hipSuccess; }
hipError_t hipGetLastError(void) { return hipSuccess; }
hipError_t hipStreamCreate(hipStream_t *s) { *s = (hipStream_t) new int(0); return hipSuccess; }
hipError_t hipStreamCreateWithFlags(hipStream_t *s, unsigned int) { return hipStreamCreate(s); }
hipError_t hipEventSynchronize(hipEvent_t) { executor().drain(); return hipSuccess; }
hipError_t hipStreamDestroy(hipStream_t s) { executor().drain(); delete (int *)s; return hipSuccess; }
hipError_t hipMemset(void *d, int v, size_t n) {
    executor().drain();
    std::memset(d, v, n);
    return hipSuccess;
}
hipError_t hipMemcpy(void *d, const void *s, size_t n, hipMemcpyKind) {
    executor().drain();
    std::memcpy(d, s, n);
    return hipSuccess;
}
hipError_t hipMemsetAsync(void *d, int v, size_t n, hipStream_t) {
    executor().submit([=] { std::memset(d, v, n); });
    return hipSuccess;
}
// function_address: void (*)(uint64_t, uint64_t, uint64_t); args: three pointers to 64-bit values
hipError_t hipLaunchKernel(const void *function_address, dim3, dim3, void **args, size_t, hipStream_t) {
    auto fn = (void (*)(uint64_t, uint64_t, uint64_t))function_address;
    const uint64_t a = *(uint64_t *)args[0], b = *(uint64_t *)args[1], c = *(uint64_t *)args[2];
    executor().submit([=] { fn(a, b, c); });
    return hipSuccess;
}
hipError_t hipStreamBeginCapture(hipStream_t, hipStreamCaptureMode) { g_captures++; return hipSuccess; }
hipError_t hipStreamEndCapture(hipStream_t, hipGraph_t *g) {
    g_captures--;
    if (g) *g = nullptr;
    return hipSuccess;
}

// ---- libnixie ---------------------------------------------------------------------------------------
int nixie_abi_check(uint64_t, uint64_t, uint64_t) { return NIXIE_OK; }
const char *nixie_strerror(int) { return "(fake runtime)"; }

int nixie_pool_create(uint64_t bytes, uint64_t block, nixie_pool_t **pool) {
    if (!pool || bytes == 0) return NIXIE_EINVAL;
    if (block == 0) block = 2u << 20;
    if (block % 4096) return NIXIE_EINVAL;
    *pool = new nixie_pool{(bytes + block - 1) / block * block, block, 0};
    return NIXIE_OK;
}
int nixie_pool_info(const nixie_pool_t *p, uint64_t *bytes, uint64_t *block) {
    if (bytes) *bytes = p->bytes;
    if (block) *block = p->block;
    return NIXIE_OK;
}
int nixie_pool_destroy(nixie_pool_t *p) { delete p; return NIXIE_OK; }

int nixie_space_create(nixie_pool_t *pool, nixie_space_t **space, void **base) {
    void *m = mmap(nullptr, pool->bytes, PROT_NONE, MAP_PRIVATE | MAP_ANONYMOUS | MAP_NORESERVE, -1, 0);
    if (m == MAP_FAILED) return NIXIE_ENOMEM;
    *space = new nixie_space{pool, (uint8_t *)m, std::vector<uint8_t>(pool->bytes / pool->block, 0)};
    *base = m;
    pool->spaces++;
    return NIXIE_OK;
}
int nixie_space_map(nixie_space_t *s, uint64_t off, uint64_t bytes) {
    const uint64_t B = s->pool->block;
    if (off % B || bytes % B || off + bytes > s->pool->bytes) return NIXIE_EINVAL;
    for (uint64_t b = off / B; b < (off + bytes) / B; b++) {
        if (s->mapped[b]) continue;
        if (mprotect(s->base + b * B, B, PROT_READ | PROT_WRITE)) return NIXIE_EHIP;
        std::memset(s->base + b * B, 0xEE, B);   // whatever the last user of the physical block left there
        s->mapped[b] = 1;
    }
    return NIXIE_OK;
}
int nixie_space_unmap(nixie_space_t *s, uint64_t off, uint64_t bytes) {
    const uint64_t B = s->pool->block;
    if (off % B || bytes % B || off + bytes > s->pool->bytes) return NIXIE_EINVAL;
    // (waits for nothing, like the driver's unmap: a kernel still using the block dies)
    for (uint64_t b = off / B; b < (off + bytes) / B; b++) {
        if (!s->mapped[b]) continue;
        madvise(s->base + b * B, B, MADV_DONTNEED);
        if (mprotect(s->base + b * B, B, PROT_NONE)) return NIXIE_EHIP;
        s->mapped[b] = 0;
    }
    return NIXIE_OK;
}
int nixie_space_destroy(nixie_space_t *s) {
    munmap(s->base, s->pool->bytes);
    s->pool->spaces--;
    delete s;
    return NIXIE_OK;
}

int nixie_ring_create(uint64_t, nixie_ring_t **ring) { *ring = new nixie_ring{0}; return NIXIE_OK; }
int nixie_ring_destroy(nixie_ring_t *r) { delete r; return NIXIE_OK; }

static int make_plan(const nixie_table_t *o, const nixie_table_t *i, nixie_plan_t **plan) {
    auto *p = new struct nixie_plan;
    if (o && o->count) p->out.assign(o->allocs, o->allocs + o->count);
    if (i && i->count) p->in.assign(i->allocs, i->allocs + i->count);
    *plan = p;
    return NIXIE_OK;
}
int nixie_plan(const nixie_table_t *o, const nixie_table_t *i, uint64_t, const nixie_opts_t *, nixie_plan_t **plan) {
    return make_plan(o, i, plan);
}
int nixie_plan_on_ring(const nixie_table_t *o, const nixie_table_t *i, nixie_ring_t *, const nixie_opts_t *,
                       nixie_plan_t **plan) {
    return make_plan(o, i, plan);
}
// Not ordered after anything: like the real one on a stream of its own, it relies on the caller having
// waited for the application's kernels.  If the caller has not, these copies race with the executor.
int nixie_switch(nixie_plan_t *p, void *, nixie_stats_t *st) {
    if (g_captures.load() > 0) std::abort();   // a migration inside a stream capture
    for (auto &a : p->out) std::memcpy(a.host_ptr, a.dev_ptr, a.bytes);
    for (auto &a : p->in) std::memcpy(a.dev_ptr, a.host_ptr, a.bytes);
    if (st) {
        std::memset(st, 0, sizeof(*st));
        st->ns_total = 1000;
    }
    return NIXIE_OK;
}
void nixie_plan_destroy(nixie_plan_t *p) { delete p; }

}  // extern "C"
