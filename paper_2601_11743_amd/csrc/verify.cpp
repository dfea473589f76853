// Verification (per-allocation 64-bit hashes on the side that holds the data) and the
// host-link probe.
//
// Paper, "Hierarchical Memory": a working set has exactly one copy, so after a switch the only
// place to check A is pageable memory and the only place to check B is HBM.  "Microbenchmarks":
// copy throughput is judged against the link's measured maximum, which nixie_link_peak supplies
// for this machine.
#include <hip/hip_runtime.h>
#include <time.h>

#include <algorithm>
#include <cstring>
#include <thread>
#include <shared_mutex>
#include <vector>

#include "internal.hpp"

struct nixie_plan;
namespace nixie {
void set_last_hip_error(int e);
const Layout &plan_layout(const nixie_plan_t *p);
HashDesc *plan_hash_descs(const nixie_plan_t *p, int x);
uint64_t plan_hash_tiles(const nixie_plan_t *p, int x);
uint64_t *plan_hash_buffer(const nixie_plan_t *p);
int plan_device(const nixie_plan_t *p);
}  // namespace nixie

using namespace nixie;

namespace {

#define NIXIE_HIP(call)                                  \
    do {                                                 \
        hipError_t e_ = (call);                          \
        if (e_ != hipSuccess) {                          \
            set_last_hip_error((int)e_);                 \
            return NIXIE_EHIP;                           \
        }                                                \
    } while (0)

double now_s() {
    timespec ts;
    clock_gettime(CLOCK_MONOTONIC, &ts);
    return (double)ts.tv_sec + 1e-9 * (double)ts.tv_nsec;
}

unsigned host_threads() {
    unsigned hc = std::thread::hardware_concurrency();
    return std::max(1u, std::min(hc ? hc : 4u, 16u));
}

int hash_device(const HashDesc *descs_d, uint64_t n, uint64_t tiles, uint64_t *hashes_d, hipStream_t stream,
                uint64_t *out) {
    if (n == 0) return NIXIE_OK;
    int e = nixie_launch_zero32((uint32_t *)hashes_d, 2 * n, stream);
    if (e) { set_last_hip_error(e); return NIXIE_EHIP; }
    e = nixie_launch_hash(descs_d, n, tiles, hashes_d, stream);
    if (e) { set_last_hip_error(e); return NIXIE_EHIP; }
    NIXIE_HIP(hipMemcpyAsync(out, hashes_d, n * sizeof(uint64_t), hipMemcpyDeviceToHost, stream));
    NIXIE_HIP(hipStreamSynchronize(stream));
    return NIXIE_OK;
}

int hash_table_host(const std::vector<nixie_alloc_t> &T, uint64_t *out) {
    std::vector<const void *> ptrs(T.size());
    std::vector<uint64_t> bytes(T.size());
    for (size_t i = 0; i < T.size(); i++) { ptrs[i] = T[i].host_ptr; bytes[i] = T[i].bytes; }
    return hash_host_buffers(ptrs.data(), bytes.data(), T.size(), out, host_threads());
}

}  // namespace

extern "C" {

int nixie_hash_tables(const nixie_plan_t *plan, void *hip_stream, uint64_t *out_hash, uint64_t *in_hash) {
    if (!plan) return NIXIE_EINVAL;
    const Layout &L = plan_layout(plan);
    if ((!L.table[0].empty() && !out_hash) || (!L.table[1].empty() && !in_hash)) return NIXIE_EINVAL;
    std::shared_lock<std::shared_mutex> maps(switch_lock());
    if (!space_uses_valid(L.uses[0])) return NIXIE_EUNMAPPED;
    int rc = hash_device(plan_hash_descs(plan, 0), L.table[0].size(), plan_hash_tiles(plan, 0),
                         plan_hash_buffer(plan), (hipStream_t)hip_stream, out_hash);
    if (rc) return rc;
    if (!L.table[1].empty()) rc = hash_table_host(L.table[1], in_hash);
    return rc;
}

int nixie_verify(const nixie_plan_t *plan, void *hip_stream, const uint64_t *expect_out_hash,
                 const uint64_t *expect_in_hash, nixie_verify_report_t *report) {
    if (!plan) return NIXIE_EINVAL;
    const Layout &L = plan_layout(plan);
    nixie_verify_report_t r{};
    r.first_bad_out = r.first_bad_in = -1;
    int rc = NIXIE_OK;
    if (expect_out_hash && !L.table[0].empty()) {   // the evicted set now lives in pageable memory
        std::vector<uint64_t> h(L.table[0].size());
        rc = hash_table_host(L.table[0], h.data());
        if (rc) return rc;
        for (size_t i = 0; i < h.size(); i++) {
            r.checked_out++;
            if (h[i] != expect_out_hash[i]) { if (r.first_bad_out < 0) r.first_bad_out = (int64_t)i; r.mismatched_out++; }
        }
    }
    if (expect_in_hash && !L.table[1].empty()) {    // the restored set now lives in HBM
        std::shared_lock<std::shared_mutex> maps(switch_lock());
        if (!space_uses_valid(L.uses[1])) return NIXIE_EUNMAPPED;
        std::vector<uint64_t> h(L.table[1].size());
        rc = hash_device(plan_hash_descs(plan, 1), h.size(), plan_hash_tiles(plan, 1), plan_hash_buffer(plan),
                         (hipStream_t)hip_stream, h.data());
        if (rc) return rc;
        for (size_t i = 0; i < h.size(); i++) {
            r.checked_in++;
            if (h[i] != expect_in_hash[i]) { if (r.first_bad_in < 0) r.first_bad_in = (int64_t)i; r.mismatched_in++; }
        }
    }
    if (report) *report = r;
    return (r.mismatched_out || r.mismatched_in) ? NIXIE_EMISMATCH : NIXIE_OK;
}

int nixie_hash_buffers(const void *const *ptrs, const uint64_t *bytes, uint64_t n, int on_device, void *hip_stream,
                       uint64_t *hashes) {
    if (n == 0) return NIXIE_OK;
    if (!ptrs || !bytes || !hashes) return NIXIE_EINVAL;
    if (!on_device) return hash_host_buffers(ptrs, bytes, n, hashes, host_threads());
    std::vector<HashDesc> hd(n);
    std::vector<SpaceUse> uses;
    uint64_t tiles = 0;
    for (uint64_t i = 0; i < n; i++) {
        if (bytes[i] && !ptrs[i]) return NIXIE_EINVAL;
        if (!space_translate((uint64_t)(uintptr_t)ptrs[i], bytes[i], nullptr, &uses)) return NIXIE_EINVAL;
        hd[i] = HashDesc{(uint64_t)(uintptr_t)ptrs[i], bytes[i], tiles};
        tiles += ((bytes[i] + 7) / 8 + kHashTileWords - 1) / kHashTileWords;
    }
    std::shared_lock<std::shared_mutex> maps(switch_lock());
    if (!space_uses_valid(uses)) return NIXIE_EUNMAPPED;
    HashDesc *hd_d = nullptr;
    uint64_t *h_d = nullptr;
    NIXIE_HIP(hipMalloc((void **)&hd_d, n * sizeof(HashDesc)));
    hipError_t e = hipMalloc((void **)&h_d, n * sizeof(uint64_t));
    if (e != hipSuccess) { (void)hipFree(hd_d); set_last_hip_error((int)e); return NIXIE_EHIP; }
    int rc = NIXIE_OK;
    e = hipMemcpy(hd_d, hd.data(), n * sizeof(HashDesc), hipMemcpyHostToDevice);
    if (e != hipSuccess) { set_last_hip_error((int)e); rc = NIXIE_EHIP; }
    if (!rc) rc = hash_device(hd_d, n, tiles, h_d, (hipStream_t)hip_stream, hashes);
    (void)hipFree(hd_d);
    (void)hipFree(h_d);
    return rc;
}

int nixie_hash_buffers_noalloc(const void *const *ptrs, const uint64_t *bytes, uint64_t n, void *hip_stream,
                               uint64_t *hashes_dev) {
    if (n == 0) return NIXIE_OK;
    if (!ptrs || !bytes || !hashes_dev) return NIXIE_EINVAL;
    if (n > kNoAllocMaxBuffers) return NIXIE_EINVAL;   // beyond the static scratch memory: use nixie_hash_buffers
    std::shared_lock<std::shared_mutex> maps(switch_lock());
    for (uint64_t i = 0; i < n; i++) {   // everything is checked before anything is enqueued
        if (bytes[i] && !ptrs[i]) return NIXIE_EINVAL;
        const int where = space_range_state((uint64_t)(uintptr_t)ptrs[i], bytes[i]);
        if (where) return where == 1 ? NIXIE_EUNMAPPED : NIXIE_EINVAL;
    }
    HashDesc batch[kNoAllocBatch];   // on the stack: no heap, and no thread-local block for the loader to allocate
    uint64_t tiles = 0;
    int e = 0;
    for (uint64_t first = 0; first < n && !e; first += kNoAllocBatch) {
        const uint32_t count = (uint32_t)std::min<uint64_t>(kNoAllocBatch, n - first);
        for (uint32_t i = 0; i < count; i++) {
            batch[i] = HashDesc{(uint64_t)(uintptr_t)ptrs[first + i], bytes[first + i], tiles};
            tiles += ((bytes[first + i] + 7) / 8 + kHashTileWords - 1) / kHashTileWords;
        }
        e = nixie_noalloc_put_descs(batch, count, (uint32_t)first, hip_stream);
    }
    if (!e) e = nixie_noalloc_hash((uint32_t)n, tiles, hashes_dev, hip_stream);
    if (e) { set_last_hip_error(e); return NIXIE_EHIP; }
    return NIXIE_OK;
}

int nixie_host_copy(void *const *dst, const void *const *src, const uint64_t *bytes, uint64_t n, uint32_t threads) {
    if (n == 0) return NIXIE_OK;
    if (!dst || !src || !bytes) return NIXIE_EINVAL;
    return copy_host_buffers(dst, src, bytes, n, threads ? threads : host_threads() / 2);
}

int nixie_link_peak(uint64_t bytes, int reps, nixie_link_peak_t *out) {
    if (!out || bytes < (1u << 20) || bytes % 16 || reps < 1) return NIXIE_EINVAL;
    std::memset(out, 0, sizeof(*out));
    void *d0 = nullptr, *d1 = nullptr, *h0 = nullptr, *h1 = nullptr;
    // The HIP runtime maps streams onto a few hardware queues; two copies that land on the same
    // queue run one after the other.  Several streams are created and the "both at once" case
    // is timed on every pair (first stream with each of the others), keeping the best.
    constexpr int kStreams = 4;
    hipStream_t st[kStreams] = {nullptr, nullptr, nullptr, nullptr};
    int rc = NIXIE_OK;
    auto cleanup = [&]() {
        for (auto &x : st) if (x) (void)hipStreamDestroy(x);
        if (d0) (void)hipFree(d0);
        if (d1) (void)hipFree(d1);
        if (h0) (void)hipHostFree(h0);
        if (h1) (void)hipHostFree(h1);
    };
#define LP(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { set_last_hip_error((int)e_); cleanup(); return NIXIE_EHIP; } } while (0)
    LP(hipMalloc(&d0, bytes));
    LP(hipMalloc(&d1, bytes));
    LP(hipHostMalloc(&h0, bytes, hipHostMallocMapped | hipHostMallocCoherent));
    LP(hipHostMalloc(&h1, bytes, hipHostMallocMapped | hipHostMallocCoherent));
    LP(hipMemset(d0, 1, bytes));
    LP(hipMemset(d1, 2, bytes));
    std::memset(h0, 3, bytes);
    std::memset(h1, 4, bytes);
    for (auto &x : st) LP(hipStreamCreateWithFlags(&x, hipStreamNonBlocking));
    LP(hipDeviceSynchronize());
    const uint32_t wgs = 128;
    // mode: bit0 = d2h active, bit1 = h2d active; engine 0 = SDMA, 1 = kernel
    for (int engine = 0; engine < 2; engine++)
        for (int mode = 1; mode <= 3; mode++) {
            double best = 1e30;
            for (int pair = 1; pair < (mode == 3 ? kStreams : 2); pair++)
                for (int r = 0; r < reps + 1; r++) {   // first repetition is a warm-up
                    hipStream_t s0 = st[0], s1 = st[pair];
                    LP(hipDeviceSynchronize());
                    const double t0 = now_s();
                    if (mode & 1) {
                        if (engine == 0) LP(hipMemcpyAsync(h0, d0, bytes, hipMemcpyDeviceToHost, s0));
                        else { int e = nixie_launch_copy16(d0, h0, bytes, wgs, s0); if (e) { set_last_hip_error(e); cleanup(); return NIXIE_EHIP; } }
                    }
                    if (mode & 2) {
                        if (engine == 0) LP(hipMemcpyAsync(d1, h1, bytes, hipMemcpyHostToDevice, s1));
                        else { int e = nixie_launch_copy16(h1, d1, bytes, wgs, s1); if (e) { set_last_hip_error(e); cleanup(); return NIXIE_EHIP; } }
                    }
                    LP(hipStreamSynchronize(s0));
                    LP(hipStreamSynchronize(s1));
                    const double dt = now_s() - t0;
                    if (r > 0 && dt < best) best = dt;
                }
            const double gbs = (double)bytes / best / 1e9;
            if (engine == 0) {
                if (mode == 1) out->sdma_d2h = gbs;
                else if (mode == 2) out->sdma_h2d = gbs;
                else out->sdma_d2h_both = out->sdma_h2d_both = gbs;
            } else {
                if (mode == 1) out->kernel_d2h = gbs;
                else if (mode == 2) out->kernel_h2d = gbs;
                else out->kernel_d2h_both = out->kernel_h2d_both = gbs;
            }
        }
#undef LP
    cleanup();
    return rc;
}

}  // extern "C"
