// nixie_linkprobe -- the measurements behind the swap kernel's design, as one reproducible
// program for one MI355X.  Not part of the library; built by build.py next to it.
//
// Every variant is one fused kernel that copies 2 GiB HBM -> pinned host memory (gather role)
// and 2 GiB pinned host memory -> HBM (scatter role) at the same time, through 128 MiB host
// windows that are reused like a ring, 256 threads per workgroup, each wave moving 8 KiB per
// pass with eight 16-byte accesses in flight per lane.  What varies is how payload is stored
// into / loaded from host memory and what is done between work pieces to order payload against
// a flag.  Output: GB/s per direction (time until both directions are done).
//
// usage: nixie_linkprobe [ordering] [loads] [stores] [pieces] [xcd] [sdma] [slots]      (no argument = all)
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <atomic>
#include <string>
#include <thread>
#include <vector>

#define CK(x)                                                                                  \
    do {                                                                                       \
        hipError_t e_ = (x);                                                                   \
        if (e_ != hipSuccess) {                                                                \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);         \
            std::exit(2);                                                                      \
        }                                                                                      \
    } while (0)

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

enum Store { kStorePlain, kStoreWriteThrough };
enum Load { kLoadPlain, kLoadSystemScope, kLoadAtomic8 };
enum Sync { kSyncNone, kSyncWaitBarrierRelaxedFlag, kSyncReleaseFence, kSyncOneThreadReleaseStore,
            kSyncWaitBarrierPlusAcquireFence };

struct Params {
    const u32x4 *dev_src;   // 2 GiB in HBM
    u32x4 *dev_dst;         // 2 GiB in HBM
    u32x4 *host_out;        // window in pinned memory, gather target
    const u32x4 *host_in;   // window in pinned memory, scatter source
    uint64_t n16, win16;    // vectors to move per direction; vectors per host window
    uint32_t gather_wgs, scatter_wgs, piece16;
    int store, load, sync;
    uint32_t *flags;        // pinned, one word per workgroup slot
    uint64_t *stats;        // pinned, per workgroup: ticks, XCC id
};

static double now_s() {
    return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

template <int DIR>
__device__ void role(const Params &p, uint32_t wg, uint32_t nwg) {
    const uint64_t pieces = (p.n16 + p.piece16 - 1) / p.piece16;
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    for (uint64_t t = wg; t < pieces; t += nwg) {
        const uint64_t base = t * p.piece16, end = base + p.piece16 < p.n16 ? base + p.piece16 : p.n16;
        for (uint64_t i = base + wave * 512ull; i < end; i += 4 * 512ull) {
            u32x4 v[8];
#pragma unroll
            for (uint32_t u = 0; u < 8; u++) {
                const uint64_t j = i + lane + 64ull * u;
                if (j >= end) continue;
                if (DIR == 0) {
                    v[u] = p.dev_src[j];
                } else {
                    const u32x4 *q = p.host_in + j % p.win16;
                    if (p.load == kLoadSystemScope) {
                        asm volatile("global_load_dwordx4 %0, %1, off sc0 sc1\n s_waitcnt vmcnt(0)" : "=&v"(v[u]) : "v"(q) : "memory");
                    } else if (p.load == kLoadAtomic8) {
                        const uint64_t a = __hip_atomic_load((const uint64_t *)q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                        const uint64_t b = __hip_atomic_load((const uint64_t *)q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                        v[u] = u32x4{(uint32_t)a, (uint32_t)(a >> 32), (uint32_t)b, (uint32_t)(b >> 32)};
                    } else {
                        v[u] = *q;
                    }
                }
            }
#pragma unroll
            for (uint32_t u = 0; u < 8; u++) {
                const uint64_t j = i + lane + 64ull * u;
                if (j >= end) continue;
                if (DIR == 0) {
                    u32x4 *q = p.host_out + j % p.win16;
                    if (p.store == kStoreWriteThrough) asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(q), "v"(v[u]) : "memory");
                    else *q = v[u];
                } else {
                    p.dev_dst[j] = v[u];
                }
            }
        }
        // between work pieces: what a real protocol would do before publishing "piece done"
        if (p.sync == kSyncReleaseFence && DIR == 0) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "");
        if (p.sync == kSyncWaitBarrierRelaxedFlag || p.sync == kSyncOneThreadReleaseStore ||
            p.sync == kSyncWaitBarrierPlusAcquireFence)
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (p.sync != kSyncNone) __syncthreads();
        if (DIR == 0 && threadIdx.x == 0) {
            if (p.sync == kSyncWaitBarrierRelaxedFlag || p.sync == kSyncWaitBarrierPlusAcquireFence)
                __hip_atomic_store(p.flags + 16 * (wg & 255u), (uint32_t)t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            if (p.sync == kSyncOneThreadReleaseStore)
                __hip_atomic_store(p.flags + 16 * (wg & 255u), (uint32_t)t, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
        }
        if (DIR == 1 && p.sync == kSyncWaitBarrierPlusAcquireFence) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "");
    }
}

// The system-scope load variant above waits after every load, which would serialise the eight
// loads; the library issues them in one asm block with a single wait.  Same here.
__device__ void scatter_system_scope(const Params &p, uint32_t wg, uint32_t nwg) {
    const uint64_t pieces = (p.n16 + p.piece16 - 1) / p.piece16;
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    for (uint64_t t = wg; t < pieces; t += nwg) {
        const uint64_t base = t * p.piece16, end = base + p.piece16 < p.n16 ? base + p.piece16 : p.n16;
        for (uint64_t i = base + wave * 512ull; i < end; i += 4 * 512ull) {
            u32x4 v[8];
            const u32x4 *a[8];
#pragma unroll
            for (uint32_t u = 0; u < 8; u++) {
                const uint64_t j = i + lane + 64ull * u;
                a[u] = p.host_in + (j < end ? j : end - 1) % p.win16;
            }
            asm volatile(
                "global_load_dwordx4 %0, %8, off sc0 sc1\n"
                "global_load_dwordx4 %1, %9, off sc0 sc1\n"
                "global_load_dwordx4 %2, %10, off sc0 sc1\n"
                "global_load_dwordx4 %3, %11, off sc0 sc1\n"
                "global_load_dwordx4 %4, %12, off sc0 sc1\n"
                "global_load_dwordx4 %5, %13, off sc0 sc1\n"
                "global_load_dwordx4 %6, %14, off sc0 sc1\n"
                "global_load_dwordx4 %7, %15, off sc0 sc1\n"
                "s_waitcnt vmcnt(0)"
                : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7])
                : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7])
                : "memory");
#pragma unroll
            for (uint32_t u = 0; u < 8; u++) {
                const uint64_t j = i + lane + 64ull * u;
                if (j < end) p.dev_dst[j] = v[u];
            }
        }
        if (p.sync != kSyncNone) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); __syncthreads(); }
    }
}

__global__ void __launch_bounds__(256) probe_kernel(Params p) {
    const uint64_t t0 = wall_clock64();
    if (blockIdx.x < p.gather_wgs) role<0>(p, blockIdx.x, p.gather_wgs);
    else if (p.load == kLoadSystemScope) scatter_system_scope(p, blockIdx.x - p.gather_wgs, p.scatter_wgs);
    else role<1>(p, blockIdx.x - p.gather_wgs, p.scatter_wgs);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0 && p.stats) {
        p.stats[2 * blockIdx.x] = wall_clock64() - t0;                                   // 100 MHz ticks
        p.stats[2 * blockIdx.x + 1] = __builtin_amdgcn_s_getreg((3 << 11) | 20) & 15u;   // XCC_ID
    }
}

struct Bench {
    size_t bytes = (size_t)2 << 30;
    char *d_src = nullptr, *d_dst = nullptr, *h_out = nullptr, *h_in = nullptr;
    uint32_t *flags = nullptr;
    uint64_t *stats = nullptr;
    hipStream_t s = nullptr, s2 = nullptr;

    void init() {
        CK(hipMalloc(&d_src, bytes));
        CK(hipMalloc(&d_dst, bytes));
        CK(hipMemset(d_src, 1, bytes));
        CK(hipMemset(d_dst, 2, bytes));
        CK(hipHostMalloc(&h_out, bytes, hipHostMallocMapped | hipHostMallocCoherent));
        CK(hipHostMalloc(&h_in, bytes, hipHostMallocMapped | hipHostMallocCoherent));
        std::memset(h_out, 3, bytes);
        std::memset(h_in, 4, bytes);
        CK(hipHostMalloc(&flags, 1 << 16, hipHostMallocMapped | hipHostMallocCoherent));
        CK(hipHostMalloc(&stats, 1 << 16, hipHostMallocMapped | hipHostMallocCoherent));
        std::memset(flags, 0, 1 << 16);
        CK(hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
        CK(hipStreamCreateWithFlags(&s2, hipStreamNonBlocking));
    }
    Params params(uint32_t g, uint32_t sc, int store, int load, int sync) const {
        Params p{};
        p.dev_src = (const u32x4 *)d_src; p.dev_dst = (u32x4 *)d_dst;
        p.host_out = (u32x4 *)h_out; p.host_in = (const u32x4 *)h_in;
        p.n16 = bytes / 16; p.win16 = (128ull << 20) / 16;
        p.gather_wgs = g; p.scatter_wgs = sc; p.piece16 = 32768;   // 512 KiB work pieces
        p.store = store; p.load = load; p.sync = sync;
        p.flags = flags; p.stats = stats;
        return p;
    }
    double run(const Params &p) {   // GB/s per direction, best of 3 after a warm-up
        double best = 1e30;
        for (int it = 0; it < 4; it++) {
            CK(hipDeviceSynchronize());
            const double t0 = now_s();
            probe_kernel<<<p.gather_wgs + p.scatter_wgs, 256, 0, s>>>(p);
            CK(hipGetLastError());
            CK(hipDeviceSynchronize());
            const double dt = now_s() - t0;
            if (it && dt < best) best = dt;
        }
        return (double)bytes / best / 1e9;
    }
};

int main(int argc, char **argv) {
    auto want = [&](const char *name) {
        if (argc < 2) return true;
        for (int i = 1; i < argc; i++) if (std::string(argv[i]) == name) return true;
        return false;
    };
    Bench b;
    b.init();
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    std::printf("device: %s, %d CUs\n", prop.gcnArchName, prop.multiProcessorCount);

    if (want("sdma")) {
        const char *names[] = {"", "GPU->host alone", "host->GPU alone", "both at once"};
        for (int mode = 1; mode <= 3; mode++) {
            double best = 1e30;
            for (int it = 0; it < 4; it++) {
                CK(hipDeviceSynchronize());
                const double t0 = now_s();
                if (mode & 1) CK(hipMemcpyAsync(b.h_out, b.d_src, b.bytes, hipMemcpyDeviceToHost, b.s));
                if (mode & 2) CK(hipMemcpyAsync(b.d_dst, b.h_in, b.bytes, hipMemcpyHostToDevice, b.s2));
                CK(hipDeviceSynchronize());
                const double dt = now_s() - t0;
                if (it && dt < best) best = dt;
            }
            std::printf("sdma      hipMemcpyAsync %-18s %6.2f GB/s per direction\n", names[mode], (double)b.bytes / best / 1e9);
        }
    }
    if (want("slots")) {
        // The alternative to a copy kernel on the link: the copy engines moving one ring slot per call
        // (the kernels would then only gather / scatter inside HBM).  Host threads issue
        // hipMemcpyAsync calls of one slot each, both directions at once, one copy in flight per thread.
        for (size_t slot : {(size_t)1 << 20, (size_t)4 << 20, (size_t)16 << 20}) {
            for (int threads : {1, 2}) {
                std::atomic<size_t> next[2];
                next[0].store(0); next[1].store(0);
                const size_t n = b.bytes / slot, window = (size_t)128 << 20;
                auto worker = [&](int dir) {
                    CK(hipSetDevice(0));
                    hipStream_t st;
                    CK(hipStreamCreateWithFlags(&st, hipStreamNonBlocking));
                    for (;;) {
                        const size_t i = next[dir].fetch_add(1);
                        if (i >= n) break;
                        if (dir) CK(hipMemcpyAsync(b.d_dst + i * slot, b.h_in + (i * slot) % window, slot, hipMemcpyHostToDevice, st));
                        else CK(hipMemcpyAsync(b.h_out + (i * slot) % window, b.d_src + i * slot, slot, hipMemcpyDeviceToHost, st));
                        CK(hipStreamSynchronize(st));
                    }
                    CK(hipStreamDestroy(st));
                };
                CK(hipDeviceSynchronize());
                const double t0 = now_s();
                std::vector<std::thread> pool;
                for (int t = 0; t < threads; t++) { pool.emplace_back(worker, 0); pool.emplace_back(worker, 1); }
                for (auto &th : pool) th.join();
                const double dt = now_s() - t0;
                std::printf("slots     hipMemcpyAsync of %2zu MiB per call, %d thread(s) per direction, both at once   %6.2f GB/s per direction\n",
                            slot >> 20, threads, (double)b.bytes / dt / 1e9);
            }
        }
    }
    if (want("ordering")) {
        struct { const char *name; int store, sync; } v[] = {
            {"plain stores, nothing between pieces (not a protocol: upper bound)", kStorePlain, kSyncNone},
            {"plain stores, system-scope release fence per piece", kStorePlain, kSyncReleaseFence},
            {"plain stores, wait+barrier, ONE thread does a release store", kStorePlain, kSyncOneThreadReleaseStore},
            {"write-through stores, wait+barrier, relaxed flag store", kStoreWriteThrough, kSyncWaitBarrierRelaxedFlag},
        };
        for (auto &x : v)
            std::printf("ordering  128+64 wgs  %-68s %6.2f GB/s per direction\n", x.name,
                        b.run(b.params(128, 64, x.store, kLoadSystemScope, x.sync)));
    }
    if (want("loads")) {
        struct { const char *name; int load, sync; } v[] = {
            {"16 B loads with system-scope bits, no fence", kLoadSystemScope, kSyncWaitBarrierRelaxedFlag},
            {"plain 16 B loads + system-scope acquire fence per piece", kLoadPlain, kSyncWaitBarrierPlusAcquireFence},
            {"two 8 B system-scope atomic loads, no fence", kLoadAtomic8, kSyncWaitBarrierRelaxedFlag},
        };
        for (auto &x : v)
            std::printf("loads     128+64 wgs  %-68s %6.2f GB/s per direction\n", x.name,
                        b.run(b.params(128, 64, kStoreWriteThrough, x.load, x.sync)));
        std::printf("loads     0+64 wgs    %-68s %6.2f GB/s\n", "scatter alone, system-scope loads",
                    b.run(b.params(0, 64, kStoreWriteThrough, kLoadSystemScope, kSyncNone)));
        std::printf("loads     0+64 wgs    %-68s %6.2f GB/s\n", "scatter alone, 8 B atomic loads",
                    b.run(b.params(0, 64, kStoreWriteThrough, kLoadAtomic8, kSyncNone)));
    }
    if (want("stores")) {
        const uint32_t shapes[][2] = {{64, 0}, {64, 64}, {128, 64}, {128, 128}, {256, 128}};
        for (auto &s : shapes)
            for (int st = 0; st < 2; st++)
                std::printf("stores    %3u+%-3u wgs  %-68s %6.2f GB/s per direction\n", s[0], s[1],
                            st ? "write-through stores" : "plain (cached) stores, no ordering at all",
                            b.run(b.params(s[0], s[1], st, kLoadSystemScope, st ? kSyncWaitBarrierRelaxedFlag : kSyncNone)));
    }
    if (want("pieces")) {
        // how often the store drain + barrier + flag happens: work piece size, write-through protocol
        for (uint32_t kib : {32u, 64u, 128u, 256u, 512u, 2048u}) {
            Params p = b.params(128, 64, kStoreWriteThrough, kLoadSystemScope, kSyncWaitBarrierRelaxedFlag);
            p.piece16 = kib * 1024 / 16;
            std::printf("pieces    128+64 wgs  write-through, drain + barrier + flag every %4u KiB %*s %6.2f GB/s per direction\n", kib, 19, "", b.run(p));
        }
    }
    if (want("xcd")) {
        // equal static work per workgroup, both directions active: how long does a workgroup on each XCD take?
        Params p = b.params(128, 64, kStoreWriteThrough, kLoadSystemScope, kSyncNone);
        p.piece16 = 4096;
        const double gbs = b.run(p);
        double sum[2][8] = {{0}};
        int cnt[2][8] = {{0}};
        for (uint32_t w = 0; w < 192; w++) {
            const int d = w >= 128, x = (int)(b.stats[2 * w + 1] & 7);
            sum[d][x] += (double)b.stats[2 * w] / 1e5;
            cnt[d][x]++;
        }
        std::printf("xcd       128+64 wgs, static partition: %.2f GB/s per direction; mean workgroup time in ms by XCD:\n", gbs);
        for (int d = 0; d < 2; d++) {
            std::printf("xcd         %-8s", d ? "scatter" : "gather");
            for (int x = 0; x < 8; x++) std::printf("  XCD%d(%2d wgs) %5.1f", x, cnt[d][x], cnt[d][x] ? sum[d][x] / cnt[d][x] : 0.0);
            std::printf("\n");
        }
    }
    return 0;
}
