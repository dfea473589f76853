// The transparent shim's own logic on the CPU, under ThreadSanitizer.  This program is compiled
// together with paper_2601_11743_amd/csrc/shim.cpp and linked in front of libfake_runtime.so
// (fake_runtime.cpp): its runtime calls hit the shim's wrappers first, as an application's do under
// LD_PRELOAD, and the wrappers forward to the fake.  It plays a multi-threaded application against
// evictions that come at arbitrary moments.
//
//   threads   three threads launch, wait, copy and allocate while the main thread evicts all the time
//   idle      the same threads with pauses, evicted by the shim's own idleness rule
//   capture   an eviction asked for between the start and the end of a stream capture is refused
//
// usage: shim_model_test <scenario> <seed>
#include <hip/hip_runtime_api.h>

#include <atomic>
#include <chrono>
#include <condition_variable>
#include <mutex>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <thread>
#include <vector>

#include "nixie.h"
#include "nixie_shim.h"

namespace {

constexpr uint64_t kWords = (4u << 20) / 4;   // a managed buffer: 4 MiB, two units

// "kernels": three 64-bit arguments each
void k_fill(uint64_t p, uint64_t n, uint64_t v) {
    uint32_t *w = (uint32_t *)(uintptr_t)p;
    for (uint64_t i = 0; i < n; i++) w[i] = (uint32_t)(v + i);
}
void k_bump(uint64_t p, uint64_t n, uint64_t) {
    uint32_t *w = (uint32_t *)(uintptr_t)p;
    for (uint64_t i = 0; i < n; i += 512) w[i] += 1;   // a sample of the words: enough to notice lost or doubled updates
}

hipError_t launch(void (*fn)(uint64_t, uint64_t, uint64_t), uint64_t a, uint64_t b, uint64_t c, hipStream_t st) {
    void *args[3] = {&a, &b, &c};
    return hipLaunchKernel((const void *)fn, dim3(1), dim3(1), args, 0, st);
}

// all application threads fall silent together (an application between two requests)
struct Meet {
    std::mutex mu;
    std::condition_variable cv;
    int waiting = 0, round = 0;
    void arrive(int parties) {
        std::unique_lock<std::mutex> lk(mu);
        const int mine = round;
        if (++waiting == parties) { waiting = 0; round++; cv.notify_all(); }
        else cv.wait(lk, [&] { return round != mine; });
    }
};

#define MUST(call)                                                            \
    do {                                                                      \
        if ((call) != hipSuccess) {                                           \
            std::printf("FAIL %s (line %d)\n", #call, __LINE__);              \
            std::exit(1);                                                     \
        }                                                                     \
    } while (0)

int run_threads(int seed, bool by_idleness) {
    constexpr int kWorkers = 3;
    const int iters = by_idleness ? 120 : 400;
    uint32_t *buf[kWorkers];
    for (int w = 0; w < kWorkers; w++) {
        MUST(hipMalloc((void **)&buf[w], kWords * 4));
        MUST(launch(k_fill, (uint64_t)(uintptr_t)buf[w], kWords, 1000 * (w + 1), nullptr));
    }
    MUST(hipDeviceSynchronize());
    std::atomic<int> running{kWorkers};
    std::atomic<bool> bad{false};
    Meet meet;
    std::vector<std::thread> workers;
    for (int w = 0; w < kWorkers; w++)
        workers.emplace_back([&, w] {
            std::mt19937 rng(seed * 10 + w);
            hipStream_t st = nullptr;
            MUST(hipStreamCreate(&st));
            for (int it = 0; it < iters; it++) {
                MUST(launch(k_bump, (uint64_t)(uintptr_t)buf[w], kWords, 0, st));
                switch (rng() % 8) {
                case 0: MUST(hipStreamSynchronize(st)); break;
                case 1: {   // read one word back, as an application looks at a result
                    uint32_t v = 0;
                    MUST(hipMemcpy(&v, buf[w], 4, hipMemcpyDeviceToHost));
                    if (v != 1000u * (w + 1) + (uint32_t)(it + 1)) bad.store(true);
                    break;
                }
                case 2: {   // a short-lived managed allocation of its own (the table and the free runs move)
                    void *tmp = nullptr;
                    MUST(hipMalloc(&tmp, 2u << 20));
                    MUST(hipMemsetAsync(tmp, 7, 4096, st));
                    MUST(hipFree(tmp));
                    break;
                }
                case 3: {
                    size_t f = 0, t = 0;
                    MUST(hipMemGetInfo(&f, &t));
                    if (f > t) bad.store(true);
                    break;
                }
                default: break;
                }
                if (by_idleness && it % 20 == 19) {
                    MUST(hipStreamSynchronize(st));
                    meet.arrive(kWorkers);
                    std::this_thread::sleep_for(std::chrono::milliseconds(6));
                }
            }
            MUST(hipStreamSynchronize(st));
            MUST(hipStreamDestroy(st));
            running--;
        });
    int asked = 0, failed = 0;
    while (running.load() > 0) {
        std::this_thread::sleep_for(std::chrono::microseconds(by_idleness ? 1000 : 150));
        if (!by_idleness && running.load() > 0) {
            asked++;
            if (nixie_shim_evict() != 0) failed++;
        }
    }
    for (auto &t : workers) t.join();
    nixie_shim_info_t info{};
    if (nixie_shim_info(&info) != 0) { std::printf("FAIL no shim info\n"); return 1; }
    std::vector<uint32_t> back(kWords);
    uint64_t wrong = 0;
    for (int w = 0; w < kWorkers; w++) {
        MUST(hipMemcpy(back.data(), buf[w], kWords * 4, hipMemcpyDeviceToHost));
        for (uint64_t i = 0; i < kWords; i++)
            wrong += back[i] != (uint32_t)(1000 * (w + 1) + i) + (i % 512 == 0 ? (uint32_t)iters : 0u);
        MUST(hipFree(buf[w]));
    }
    std::printf("evictions %u restores %u held %llu asked %d failed %d wrong %llu bad %d, %llu blocks mapped, %llu bytes of host backing\n",
                info.evictions, info.restores, (unsigned long long)info.launches_held, asked, failed, (unsigned long long)wrong,
                (int)bad.load(), (unsigned long long)info.mapped_blocks, (unsigned long long)info.host_backing_bytes);
    const bool ok = wrong == 0 && !bad.load() && failed == 0 && info.evictions >= (by_idleness ? 2u : 3u) &&
                    info.restores >= info.evictions - 1 && info.host_backing_bytes == kWorkers * kWords * 4 &&
                    info.mapped_blocks <= info.capacity_bytes / info.block_bytes;
    std::printf(ok ? "ok\n" : "FAIL\n");
    return ok ? 0 : 1;
}

int run_capture() {
    uint32_t *buf = nullptr;
    MUST(hipMalloc((void **)&buf, kWords * 4));
    MUST(launch(k_fill, (uint64_t)(uintptr_t)buf, kWords, 5, nullptr));
    MUST(hipDeviceSynchronize());
    if (nixie_shim_evict() != 0) { std::printf("FAIL evict\n"); return 1; }
    hipStream_t st = nullptr;
    MUST(hipStreamCreate(&st));
    MUST(hipStreamBeginCapture(st, hipStreamCaptureModeGlobal));   // brings the application back first
    nixie_shim_info_t info{};
    nixie_shim_info(&info);
    const int rc = nixie_shim_evict();                             // must be refused; the fake aborts on a migration inside a capture
    hipGraph_t g = nullptr;
    MUST(hipStreamEndCapture(st, &g));
    const int after = nixie_shim_evict();
    uint32_t v = 0;
    MUST(hipMemcpy(&v, buf + 9, 4, hipMemcpyDeviceToHost));
    std::printf("resident at capture %u, evict during capture %d, after %d, word %u\n", info.resident, rc, after, v);
    const bool ok = info.resident == 1 && rc == NIXIE_EBUSY && after == 0 && v == 14;
    std::printf(ok ? "ok\n" : "FAIL\n");
    return ok ? 0 : 1;
}

}  // namespace

int main(int argc, char **argv) {
    const char *scenario = argc > 1 ? argv[1] : "threads";
    const int seed = argc > 2 ? std::atoi(argv[2]) : 1;
    setenv("NIXIE_SHIM_POOL_MIB", "32", 1);
    setenv("NIXIE_SHIM_UNIT_MIB", "2", 1);
    setenv("NIXIE_SHIM_BLOCK_MIB", "6", 1);    // three units to a block: allocations share blocks and straddle them
    setenv("NIXIE_SHIM_RING_MIB", "1", 1);
    setenv("NIXIE_SHIM_SCRIBBLE", "1", 1);
    if (!std::strcmp(scenario, "idle")) setenv("NIXIE_SHIM_IDLE_MS", "1", 1);
    if (!std::strcmp(scenario, "threads")) return run_threads(seed, false);
    if (!std::strcmp(scenario, "idle")) return run_threads(seed, true);
    if (!std::strcmp(scenario, "capture")) return run_capture();
    std::printf("unknown scenario %s\n", scenario);
    return 2;
}
