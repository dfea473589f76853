// A small, ordinary HIP program that knows nothing of nixie: it allocates, fills its buffers with
// kernels, falls silent for a while (an interactive application waiting for its user), then
// checks every buffer with kernels through the pointers it got at the start.  The shim's GPU test
// runs it unchanged, once alone and once under LD_PRELOAD=libnixie_shim.so with idle eviction on:
// there it loses its GPU memory while it is silent and must find the same bytes at the same
// addresses when it wakes up.
//
// With mode "explicit" it plays an application that a scheduler in the same process takes off the
// GPU at a moment of its choosing: if the process exports nixie_shim_evict (it does only under the
// shim) that call is made in every pause, and the next runtime call has to bring the memory back.
//
// With mode "graph" (implies the explicit evictions, where available) the per-round update of the
// buffers is a graph captured once from a stream and launched after every pause: the graph holds
// the buffers' addresses, and its launch is the call that finds the application evicted.  An
// eviction asked for in the middle of the capture must be refused.
//
// With mode "threads" three host threads, each with a stream and a buffer of its own, update their
// buffers `rounds` x 50 times while the main thread asks for an eviction every pause_ms: launches
// and waits of several threads meet migrations at arbitrary points.
//
// With mode "overhead" it measures what the paper's "Runtime Overheads" and "Memory Overheads" measure:
// the time of a small kernel launch (asynchronous, and with a wait after each) and of an allocation
// followed by a fill and a free, by size.  Run once alone and once under the shim.
//
// With mode "poll" it queues `rounds` x 100 ms of kernels and waits for them by polling hipStreamQuery:
// busy all the time, but never inside a blocking call.
//
// usage: shim_app <pause_ms> <big_mib> [rounds] [idle|explicit|graph|threads|overhead|poll]
#include <hip/hip_runtime.h>
#include <dlfcn.h>
#include <execinfo.h>
#include <signal.h>
#include <unistd.h>

#include <chrono>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <algorithm>
#include <atomic>
#include <cstring>
#include <thread>
#include <vector>

#define CHECK(call)                                                                           \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess) {                                                               \
            std::printf("FAIL %s: %s\n", #call, hipGetErrorString(e_));                       \
            return 1;                                                                         \
        }                                                                                     \
    } while (0)

__device__ __host__ inline uint32_t pattern(uint32_t seed, uint64_t i) {
    uint64_t z = (i + 1) * 0x9E3779B97F4A7C15ull + seed;
    z = (z ^ (z >> 29)) * 0xBF58476D1CE4E5B9ull;
    return (uint32_t)(z >> 32);
}

__global__ void fill(uint32_t *p, uint64_t n, uint32_t seed) {
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x)
        p[i] = pattern(seed, i);
}

__global__ void bump(uint32_t *p, uint64_t n) {
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x)
        p[i] += 1;
}

__global__ void check(const uint32_t *p, uint64_t n, uint32_t seed, uint32_t bumps, unsigned long long *bad) {
    unsigned long long mine = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x)
        mine += p[i] != pattern(seed, i) + bumps;
    if (mine) atomicAdd(bad, mine);
}

__global__ void tiny(uint32_t *p) {
    if (threadIdx.x == 0 && blockIdx.x == 0) p[0] += 1;
}

__global__ void spin(uint32_t *p, uint64_t ticks) {   // ticks of the 100 MHz wall clock; bounded by construction
    const uint64_t t0 = wall_clock64();
    while (wall_clock64() - t0 < ticks) __builtin_amdgcn_s_sleep(32);
    if (threadIdx.x == 0) p[0] += 1;
}

// mode "poll"
int run_poll(uint64_t big, int rounds) {
    uint32_t *buf = nullptr;
    CHECK(hipMalloc((void **)&buf, big));
    CHECK(hipMemset(buf, 0, 4096));
    const int n = rounds * 50;
    for (int i = 0; i < n; i++) spin<<<1, 64>>>(buf, 200000);   // 2 ms each
    CHECK(hipGetLastError());
    uint64_t polls = 0;
    hipError_t q;
    while ((q = hipStreamQuery(nullptr)) == hipErrorNotReady) polls++;
    CHECK(q);
    uint32_t count = 0;
    CHECK(hipMemcpy(&count, buf, 4, hipMemcpyDeviceToHost));
    CHECK(hipFree(buf));
    std::printf("polled %llu times, %u kernels done\n", (unsigned long long)polls, count);
    std::printf(count == (uint32_t)n ? "RESULT ok 0\n" : "RESULT wrong 1\n");
    return count == (uint32_t)n ? 0 : 1;
}

// mode "overhead"
int run_overhead(uint64_t big) {
    using clk = std::chrono::steady_clock;
    auto us = [](clk::time_point a, clk::time_point b) { return std::chrono::duration<double, std::micro>(b - a).count(); };
    uint32_t *buf = nullptr;
    CHECK(hipMalloc((void **)&buf, big));            // a managed allocation for the kernels to touch
    CHECK(hipMemset(buf, 0, 4096));
    for (int i = 0; i < 2000; i++) tiny<<<1, 64>>>(buf);
    CHECK(hipDeviceSynchronize());
    const int n = 20000;
    auto t0 = clk::now();
    for (int i = 0; i < n; i++) tiny<<<1, 64>>>(buf);
    auto t1 = clk::now();
    CHECK(hipDeviceSynchronize());
    auto t2 = clk::now();
    std::printf("launch: %.3f us per asynchronous launch, %.3f us per kernel with the queue draining\n", us(t0, t1) / n, us(t0, t2) / n);
    t0 = clk::now();
    for (int i = 0; i < n / 4; i++) { tiny<<<1, 64>>>(buf); CHECK(hipDeviceSynchronize()); }
    t1 = clk::now();
    std::printf("launch+wait: %.3f us\n", us(t0, t1) / (n / 4));
    uint32_t count = 0;
    CHECK(hipMemcpy(&count, buf, 4, hipMemcpyDeviceToHost));
    const uint64_t sizes[] = {64ull << 10, 1ull << 20, 2ull << 20, 16ull << 20, 128ull << 20, 512ull << 20};
    for (uint64_t sz : sizes) {
        double best_alloc = 1e30, best_free = 1e30, first_alloc = 0, first_free = 0;
        for (int rep = 0; rep < 5; rep++) {
            void *p = nullptr;
            t0 = clk::now();
            CHECK(hipMalloc(&p, sz));
            CHECK(hipMemset(p, 1, sz));              // as the paper does: takes lazy initialisation out of the comparison
            CHECK(hipDeviceSynchronize());
            t1 = clk::now();
            CHECK(hipFree(p));
            t2 = clk::now();
            best_alloc = std::min(best_alloc, us(t0, t1));
            best_free = std::min(best_free, us(t1, t2));
            if (rep == 0) { first_alloc = us(t0, t1); first_free = us(t1, t2); }
        }
        std::printf("malloc+fill %llu KiB: first %.1f us, best of 5 %.1f us; free: first %.1f us, best %.1f us\n",
                    (unsigned long long)(sz >> 10), first_alloc, best_alloc, first_free, best_free);
    }
    CHECK(hipFree(buf));
    const bool good = count == 2000u + n + n / 4;
    std::printf(good ? "RESULT ok 0\n" : "RESULT wrong 1\n");
    return good ? 0 : 1;
}

// mode "threads"; returns the process's exit code
int run_threads(int pause_ms, uint64_t big, int iters, int (*evict)(void)) {
    constexpr int kWorkers = 3;
    uint32_t *buf[kWorkers];
    const uint64_t n = big / kWorkers / 4;
    for (int w = 0; w < kWorkers; w++) CHECK(hipMalloc((void **)&buf[w], n * 4));
    unsigned long long *bad = nullptr;
    CHECK(hipMalloc((void **)&bad, sizeof(*bad)));
    CHECK(hipMemset(bad, 0, sizeof(*bad)));
    for (int w = 0; w < kWorkers; w++) fill<<<256, 256>>>(buf[w], n, 200 + w);
    CHECK(hipDeviceSynchronize());
    std::atomic<int> running{kWorkers}, failed{0};
    std::vector<std::thread> workers;
    for (int w = 0; w < kWorkers; w++)
        workers.emplace_back([&, w] {
            hipStream_t st = nullptr;
            bool ok = hipStreamCreate(&st) == hipSuccess;
            for (int it = 0; ok && it < iters; it++) {
                bump<<<64, 256, 0, st>>>(buf[w], n);
                ok = hipGetLastError() == hipSuccess;
                if (ok && it % 8 == 7) ok = hipStreamSynchronize(st) == hipSuccess;
                if (ok && it % 16 == 15) std::this_thread::sleep_for(std::chrono::microseconds(300 * (w + 1)));
            }
            ok = ok && hipStreamSynchronize(st) == hipSuccess;
            if (st) (void)hipStreamDestroy(st);
            if (!ok) failed++;
            running--;
        });
    int asked = 0, refused = 0;
    while (running.load() > 0) {
        std::this_thread::sleep_for(std::chrono::milliseconds(pause_ms));
        if (evict && running.load() > 0) {
            asked++;
            if (evict() != 0) refused++;
        }
    }
    for (auto &t : workers) t.join();
    std::printf("threads: %d evictions asked for, %d refused, %d workers failed\n", asked, refused, failed.load());
    for (int w = 0; w < kWorkers; w++) check<<<256, 256>>>(buf[w], n, 200 + w, (uint32_t)iters, bad);
    unsigned long long h = 0;
    CHECK(hipMemcpy(&h, bad, sizeof(h), hipMemcpyDeviceToHost));
    for (int w = 0; w < kWorkers; w++) CHECK(hipFree(buf[w]));
    CHECK(hipFree(bad));
    const bool good = h == 0 && failed.load() == 0 && refused == 0;
    std::printf(good ? "RESULT ok %llu\n" : "RESULT wrong %llu\n", h);
    return good ? 0 : 1;
}

// Should the program ever die on a signal, say where: the test harness only sees the exit status.
void say_where(int sig) {
    void *frames[64];
    const int n = backtrace(frames, 64);
    const char msg[] = "shim_app: fatal signal, backtrace follows\n";
    (void)!write(2, msg, sizeof(msg) - 1);
    backtrace_symbols_fd(frames, n, 2);
    signal(sig, SIG_DFL);
    raise(sig);
}

int main(int argc, char **argv) {
    for (int sig : {SIGSEGV, SIGBUS, SIGABRT, SIGFPE}) signal(sig, say_where);
    const int pause_ms = argc > 1 ? std::atoi(argv[1]) : 500;
    const uint64_t big = (argc > 2 ? std::strtoull(argv[2], nullptr, 10) : 48) << 20;
    const int rounds = argc > 3 ? std::atoi(argv[3]) : 2;
    const bool graph_mode = argc > 4 && std::strcmp(argv[4], "graph") == 0;
    const bool threads_mode = argc > 4 && std::strcmp(argv[4], "threads") == 0;
    const bool explicit_mode = graph_mode || threads_mode || (argc > 4 && std::strcmp(argv[4], "explicit") == 0);
    using evict_fn = int (*)(void);
    const evict_fn evict = explicit_mode ? (evict_fn)dlsym(RTLD_DEFAULT, "nixie_shim_evict") : nullptr;
    if (threads_mode) return run_threads(pause_ms, big, rounds * 50, evict);
    if (argc > 4 && std::strcmp(argv[4], "overhead") == 0) return run_overhead(big);
    if (argc > 4 && std::strcmp(argv[4], "poll") == 0) return run_poll(big, rounds);
    size_t free0 = 0, total0 = 0;
    CHECK(hipMemGetInfo(&free0, &total0));
    // a few buffers of mixed sizes: three large ones and two small ones
    const uint64_t sizes[5] = {big, big / 3 + 4096, 5u << 20, 64u << 10, 1000};
    uint32_t *buf[5];
    for (int b = 0; b < 5; b++) CHECK(hipMalloc((void **)&buf[b], sizes[b]));
    size_t free1 = 0, total1 = 0;
    CHECK(hipMemGetInfo(&free1, &total1));
    std::printf("meminfo total %zu free_before %zu free_after %zu\n", total1, free0, free1);
    for (int b = 0; b < 5; b++) std::printf("buffer %d at %p, %llu bytes\n", b, (void *)buf[b], (unsigned long long)sizes[b]);
    unsigned long long *bad = nullptr;
    CHECK(hipMalloc((void **)&bad, sizeof(*bad)));
    CHECK(hipMemset(bad, 0, sizeof(*bad)));
    uint32_t *scratch = nullptr;                       // 1 MiB: below the shim's threshold, the runtime's own memory
    CHECK(hipMalloc((void **)&scratch, 1 << 20));
    for (int b = 0; b < 5; b++) fill<<<256, 256>>>(buf[b], sizes[b] / 4, 100 + b);
    CHECK(hipGetLastError());
    CHECK(hipDeviceSynchronize());
    std::fflush(stdout);
    hipStream_t stream = nullptr;
    hipGraphExec_t update = nullptr;
    if (graph_mode) {
        hipGraph_t graph = nullptr;
        CHECK(hipStreamCreate(&stream));
        CHECK(hipStreamBeginCapture(stream, hipStreamCaptureModeGlobal));
        for (int b = 0; b < 3; b++) bump<<<256, 256, 0, stream>>>(buf[b], sizes[b] / 4);
        if (evict) std::printf("eviction asked for during the capture: rc %d\n", evict());
        for (int b = 3; b < 5; b++) bump<<<256, 256, 0, stream>>>(buf[b], sizes[b] / 4);
        CHECK(hipStreamEndCapture(stream, &graph));
        CHECK(hipGraphInstantiate(&update, graph, nullptr, nullptr, 0));
        CHECK(hipGraphDestroy(graph));
    }
    unsigned long long total_bad = 0;
    for (int r = 0; r < rounds && graph_mode; r++) {
        std::this_thread::sleep_for(std::chrono::milliseconds(pause_ms));
        if (evict) {
            const int rc = evict();
            std::printf("round %d: scheduler took the GPU away, rc %d\n", r, rc);
            if (rc) return 1;
        }
        CHECK(hipGraphLaunch(update, stream));                                                  // wakes up with the graph
        CHECK(hipStreamSynchronize(stream));
        for (int b = 0; b < 5; b++) check<<<256, 256>>>(buf[b], sizes[b] / 4, 100 + b, (uint32_t)r + 1, bad);
        CHECK(hipGetLastError());
        unsigned long long h = 0;
        CHECK(hipMemcpy(&h, bad, sizeof(h), hipMemcpyDeviceToHost));
        std::printf("round %d: %llu wrong words\n", r, h);
        std::fflush(stdout);
        total_bad = h;
    }
    for (int r = 0; r < rounds && !graph_mode; r++) {
        std::this_thread::sleep_for(std::chrono::milliseconds(pause_ms));   // silence: no runtime call at all
        if (evict) {
            const int rc = evict();
            std::printf("round %d: scheduler took the GPU away, rc %d\n", r, rc);
            if (rc) return 1;
        }
        if (r % 2 == 1) {
            // this round wakes up with a copy engine call instead of a launch: the scratch buffer gets the
            // head of buffer 0 device to device, and the check below reads buffer 0 itself as always
            CHECK(hipMemcpyDtoDAsync((hipDeviceptr_t)scratch, (hipDeviceptr_t)buf[0], 1 << 20, nullptr));
        }
        for (int b = 0; b < 5; b++) check<<<256, 256>>>(buf[b], sizes[b] / 4, 100 + b, (uint32_t)r, bad);
        if (r % 2 == 1) check<<<256, 256>>>(scratch, (1 << 20) / 4, 100, (uint32_t)r, bad);
        for (int b = 0; b < 5; b++) bump<<<256, 256>>>(buf[b], sizes[b] / 4);                  // the state moves on
        CHECK(hipGetLastError());
        unsigned long long h = 0;
        CHECK(hipMemcpy(&h, bad, sizeof(h), hipMemcpyDeviceToHost));
        std::printf("round %d: %llu wrong words\n", r, h);
        std::fflush(stdout);
        total_bad = h;
    }
    // a host-side look at one large buffer through the runtime's copy, as an application would read results back
    std::vector<uint32_t> head(1024);
    CHECK(hipMemcpy(head.data(), buf[0], head.size() * 4, hipMemcpyDeviceToHost));
    for (size_t i = 0; i < head.size(); i++) total_bad += head[i] != pattern(100, i) + (uint32_t)rounds;
    // and with the driver-style calls: the tail of the second large buffer, then a 32-bit fill read back
    if (evict && evict()) return 1;
    const uint64_t n1 = sizes[1] / 4;
    CHECK(hipMemcpyDtoH(head.data(), (hipDeviceptr_t)(buf[1] + n1 - head.size()), head.size() * 4));
    for (size_t i = 0; i < head.size(); i++) total_bad += head[i] != pattern(101, n1 - head.size() + i) + (uint32_t)rounds;
    if (evict && evict()) return 1;
    CHECK(hipMemsetD32((hipDeviceptr_t)buf[2], 0x5EED5EED, 4096));
    CHECK(hipMemcpyDtoH(head.data(), (hipDeviceptr_t)buf[2], head.size() * 4));
    for (size_t i = 0; i < head.size(); i++) total_bad += head[i] != 0x5EED5EEDu;
    CHECK(hipMemcpyDtoH(head.data(), (hipDeviceptr_t)(buf[2] + 4096), head.size() * 4));
    for (size_t i = 0; i < head.size(); i++) total_bad += head[i] != pattern(102, 4096 + i) + (uint32_t)rounds;
    CHECK(hipFree(buf[1]));
    size_t free2 = 0, total2 = 0;
    CHECK(hipMemGetInfo(&free2, &total2));
    std::printf("meminfo free_after_one_free %zu\n", free2);
    for (int b = 0; b < 5; b++)
        if (b != 1) CHECK(hipFree(buf[b]));
    CHECK(hipFree(bad));
    CHECK(hipFree(scratch));
    if (update) CHECK(hipGraphExecDestroy(update));
    if (stream) CHECK(hipStreamDestroy(stream));
    std::printf(total_bad ? "RESULT wrong %llu\n" : "RESULT ok %llu\n", total_bad);
    return total_bad ? 1 : 0;
}
