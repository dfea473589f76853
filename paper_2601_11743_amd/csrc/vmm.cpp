// Memory the library is told about rather than given per call: the pinned tier (paper,
// "Hierarchical Memory"), and pools and spaces -- physical device memory in equal blocks, and
// reserved address ranges that map those blocks (paper, "Maintaining consistent virtual memory
// addresses"; "Granularity of Memory Management").  All driver calls here run outside a switch:
// they need the switch lock exclusively and return NIXIE_EBUSY while a switch holds it shared.
#include <hip/hip_runtime.h>

#include <mutex>
#include <new>
#include <shared_mutex>
#include <vector>

#include "internal.hpp"
#include "spaces.hpp"

namespace nixie {
void set_last_hip_error(int e);
}  // namespace nixie

using namespace nixie;

struct nixie_pool {
    int device = 0;
    uint64_t bytes = 0, block_bytes = 0, key_base = 0;
    std::vector<hipMemGenericAllocationHandle_t> blocks;
    uint32_t spaces = 0;
    std::mutex mu;
};

struct nixie_space {
    nixie_pool *pool = nullptr;
    void *base = nullptr;
    std::vector<uint64_t> assigned;   // pool block behind each block of the space (block i by default)
    std::vector<uint8_t> mapped;
};

namespace {

// An unmap call takes about 0.25 ms on MI355X whatever the block size (a map call 0.03 ms), so
// the block size sets the cost of a remap: 17 GiB in 64 MiB blocks unmaps in 71 ms, in 256 MiB
// blocks in 17 ms, in 1 GiB blocks in 4 ms.
constexpr uint64_t kDefaultBlock = 256ull << 20;

int fail(hipError_t e) {
    set_last_hip_error((int)e);
    return e == hipErrorOutOfMemory ? NIXIE_ENOMEM : NIXIE_EHIP;
}

hipMemAllocationProp device_prop(int device) {
    hipMemAllocationProp prop{};
    prop.type = hipMemAllocationTypePinned;          // ordinary, non-migratable device memory
    prop.location.type = hipMemLocationTypeDevice;
    prop.location.id = device;
    return prop;
}

// s->mapped[b]: 0 = not mapped, 1 = mapped and in the registry, kUnmapPending = taken out of the
// registry by an unmap that the driver refused (see unmap_blocks)
constexpr uint8_t kUnmapPending = 2;

int block_range(const nixie_space *s, uint64_t offset, uint64_t bytes, uint64_t *first, uint64_t *count) {
    const uint64_t B = s->pool->block_bytes;
    if (offset % B || bytes % B || offset > s->pool->bytes || bytes > s->pool->bytes - offset) return NIXIE_EINVAL;
    *first = offset / B;
    *count = bytes / B;
    return NIXIE_OK;
}

// caller holds the switch lock exclusively
int unmap_blocks(nixie_space *s, uint64_t first, uint64_t count) {
    const uint64_t B = s->pool->block_bytes;
    for (uint64_t b = first; b < first + count; b++) {
        if (!s->mapped[b]) continue;
        // out of the registry first: from here on no switch may count on this block
        space_set_mapped((uint64_t)(uintptr_t)s->base, b, 1, false);
        hipError_t e = hipMemUnmap((char *)s->base + b * B, B);
        if (e != hipSuccess) {
            // The registry says "not mapped" (no switch will touch the block), the driver may still
            // have it mapped: remember that, so that the next map or unmap of the block first
            // finishes this unmap instead of mapping over it.
            s->mapped[b] = kUnmapPending;
            return fail(e);
        }
        s->mapped[b] = 0;
    }
    return NIXIE_OK;
}

}  // namespace

extern "C" {

// ---- pinned tier: announce GPU-addressable pinned host memory to the planner -----------------
int nixie_tier_register(void *host_base, uint64_t bytes) {
    if (!host_base || bytes == 0) return NIXIE_EINVAL;
    hipPointerAttribute_t attr{};
    hipError_t e = hipPointerGetAttributes(&attr, host_base);
    if (e != hipSuccess) {
        (void)hipGetLastError();                 // unknown to the runtime: ordinary pageable memory
        return NIXIE_EINVAL;
    }
    if (attr.type != hipMemoryTypeHost) return NIXIE_EINVAL;
    void *seen_by_gpu = nullptr;
    e = hipHostGetDevicePointer(&seen_by_gpu, host_base, 0);
    if (e != hipSuccess) return fail(e);
    if (!seen_by_gpu) return NIXIE_EINVAL;
    // the whole range must belong to the same pinned allocation
    hipPointerAttribute_t last{};
    e = hipPointerGetAttributes(&last, (char *)host_base + bytes - 1);
    if (e != hipSuccess) { (void)hipGetLastError(); return NIXIE_EINVAL; }
    if (last.type != hipMemoryTypeHost) return NIXIE_EINVAL;
    void *last_seen = nullptr;
    e = hipHostGetDevicePointer(&last_seen, (char *)host_base + bytes - 1, 0);
    if (e != hipSuccess) return fail(e);
    if ((char *)last_seen - (char *)seen_by_gpu != (ptrdiff_t)(bytes - 1)) return NIXIE_EINVAL;
    TierSpan t{(uint64_t)(uintptr_t)host_base, bytes, (uint64_t)(uintptr_t)seen_by_gpu};
    return tier_register(t) ? NIXIE_OK : NIXIE_EINVAL;
}

int nixie_tier_unregister(void *host_base) {
    if (!host_base) return NIXIE_EINVAL;
    switch (tier_unregister((uint64_t)(uintptr_t)host_base)) {
    case kTierDropped: return NIXIE_OK;
    case kTierInUse: return NIXIE_EBUSY;   // a live plan moves chunks straight to or from this memory
    default: return NIXIE_EINVAL;
    }
}

// ---- pools and spaces ---------------------------------------------------------------------------
int nixie_pool_create(uint64_t bytes, uint64_t block_bytes, nixie_pool_t **pool) {
    if (!pool || bytes == 0) return NIXIE_EINVAL;
    *pool = nullptr;
    int device = 0, supported = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return fail(e);
    e = hipDeviceGetAttribute(&supported, hipDeviceAttributeVirtualMemoryManagementSupported, device);
    if (e != hipSuccess) return fail(e);
    if (!supported) { set_last_hip_error((int)hipErrorNotSupported); return NIXIE_EHIP; }
    hipMemAllocationProp prop = device_prop(device);
    size_t gran = 0;
    e = hipMemGetAllocationGranularity(&gran, &prop, hipMemAllocationGranularityRecommended);
    if (e != hipSuccess) return fail(e);
    if (block_bytes == 0) block_bytes = kDefaultBlock;
    if (gran == 0 || block_bytes % gran || block_bytes % 4096 || block_bytes > (1ull << 36)) return NIXIE_EINVAL;
    const uint64_t n = (bytes + block_bytes - 1) / block_bytes;
    if (n > (1ull << 22) || n * block_bytes > kKeyStride) return NIXIE_EINVAL;
    nixie_pool *p = new (std::nothrow) nixie_pool;
    if (!p) return NIXIE_ENOMEM;
    p->device = device;
    p->block_bytes = block_bytes;
    p->bytes = n * block_bytes;
    p->key_base = next_pool_key();
    p->blocks.reserve(n);
    for (uint64_t i = 0; i < n; i++) {
        hipMemGenericAllocationHandle_t h;
        e = hipMemCreate(&h, block_bytes, &prop, 0);
        if (e != hipSuccess) {
            for (auto &b : p->blocks) (void)hipMemRelease(b);
            delete p;
            return fail(e);
        }
        p->blocks.push_back(h);
    }
    *pool = p;
    return NIXIE_OK;
}

int nixie_pool_info(const nixie_pool_t *pool, uint64_t *bytes, uint64_t *block_bytes) {
    if (!pool) return NIXIE_EINVAL;
    if (bytes) *bytes = pool->bytes;
    if (block_bytes) *block_bytes = pool->block_bytes;
    return NIXIE_OK;
}

int nixie_pool_destroy(nixie_pool_t *pool) {
    if (!pool) return NIXIE_OK;
    {
        std::lock_guard<std::mutex> g(pool->mu);
        if (pool->spaces) return NIXIE_EBUSY;
    }
    int rc = NIXIE_OK;
    for (auto &b : pool->blocks) {
        hipError_t e = hipMemRelease(b);
        if (e != hipSuccess) rc = fail(e);
    }
    delete pool;
    return rc;
}

int nixie_space_create(nixie_pool_t *pool, nixie_space_t **space, void **base) {
    if (!pool || !space || !base) return NIXIE_EINVAL;
    *space = nullptr;
    *base = nullptr;
    nixie_space *s = new (std::nothrow) nixie_space;
    if (!s) return NIXIE_ENOMEM;
    // aligned to the block size (a power of two is not required: alignment 0 = the driver's own)
    hipError_t e = hipMemAddressReserve(&s->base, pool->bytes, 0, nullptr, 0);
    if (e != hipSuccess || !s->base) {
        delete s;
        return e == hipSuccess ? NIXIE_ENOMEM : fail(e);
    }
    s->pool = pool;
    s->mapped.assign(pool->blocks.size(), 0);
    s->assigned.resize(pool->blocks.size());
    for (size_t i = 0; i < s->assigned.size(); i++) s->assigned[i] = i;
    SpaceSpan span;
    span.base = (uint64_t)(uintptr_t)s->base;
    span.bytes = pool->bytes;
    span.key_base = pool->key_base;
    span.block_bytes = pool->block_bytes;
    span.mapped.assign(pool->blocks.size(), 0);
    span.assigned = s->assigned;
    space_register(span);
    {
        std::lock_guard<std::mutex> g(pool->mu);
        pool->spaces++;
    }
    *space = s;
    *base = s->base;
    return NIXIE_OK;
}

int nixie_space_map(nixie_space_t *s, uint64_t offset, uint64_t bytes) {
    if (!s) return NIXIE_EINVAL;
    uint64_t first = 0, count = 0;
    int rc = block_range(s, offset, bytes, &first, &count);
    if (rc) return rc;
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return fail(e);
    if (device != s->pool->device) return NIXIE_EINVAL;
    std::unique_lock<std::shared_mutex> lk(switch_lock(), std::try_to_lock);
    if (!lk.owns_lock()) return NIXIE_EBUSY;   // a switch is running: never wait for it here (it may be the caller's own)
    const uint64_t B = s->pool->block_bytes;
    hipMemAccessDesc acc{};
    acc.location.type = hipMemLocationTypeDevice;
    acc.location.id = device;
    acc.flags = hipMemAccessFlagsProtReadWrite;
    // map, then open access for each run of newly mapped blocks with one call
    for (uint64_t q = first; q < first + count; q++)     // finish what an earlier unmap left behind
        if (s->mapped[q] == kUnmapPending) {
            e = hipMemUnmap((char *)s->base + q * B, B);
            if (e != hipSuccess) return fail(e);
            s->mapped[q] = 0;
        }
    uint64_t b = first;
    while (b < first + count) {
        if (s->mapped[b]) { b++; continue; }
        uint64_t run = b;
        while (run < first + count && !s->mapped[run]) {
            e = hipMemMap((char *)s->base + run * B, B, 0, s->pool->blocks[s->assigned[run]], 0);
            if (e != hipSuccess) break;
            run++;
        }
        hipError_t e2 = hipSuccess;
        if (run > b) e2 = hipMemSetAccess((char *)s->base + b * B, (run - b) * B, &acc, 1);
        if (e2 != hipSuccess) {              // mapped but not accessible: take the run back out
            for (uint64_t q = b; q < run; q++) (void)hipMemUnmap((char *)s->base + q * B, B);
            return fail(e2);
        }
        for (uint64_t q = b; q < run; q++) s->mapped[q] = 1;
        space_set_mapped((uint64_t)(uintptr_t)s->base, b, run - b, true);
        if (e != hipSuccess) return fail(e);
        b = run;
    }
    return NIXIE_OK;
}

int nixie_space_assign(nixie_space_t *s, uint64_t offset, const uint64_t *pool_blocks, uint64_t n_blocks) {
    if (!s || (n_blocks && !pool_blocks)) return NIXIE_EINVAL;
    uint64_t first = 0, count = 0;
    const uint64_t B = s->pool->block_bytes;
    if (n_blocks > s->assigned.size()) return NIXIE_EINVAL;
    int rc = block_range(s, offset, n_blocks * B, &first, &count);
    if (rc) return rc;
    std::unique_lock<std::shared_mutex> lk(switch_lock(), std::try_to_lock);
    if (!lk.owns_lock()) return NIXIE_EBUSY;   // a switch is running: never wait for it here (it may be the caller's own)
    for (uint64_t i = 0; i < count; i++) {
        if (pool_blocks[i] >= s->assigned.size()) return NIXIE_EINVAL;
        if (s->mapped[first + i] && s->assigned[first + i] != pool_blocks[i]) return NIXIE_EBUSY;   // unmap it first
    }
    if (!space_assign((uint64_t)(uintptr_t)s->base, first, pool_blocks, count)) return NIXIE_EINVAL;
    for (uint64_t i = 0; i < count; i++) s->assigned[first + i] = pool_blocks[i];
    return NIXIE_OK;
}

int nixie_space_unmap(nixie_space_t *s, uint64_t offset, uint64_t bytes) {
    if (!s) return NIXIE_EINVAL;
    uint64_t first = 0, count = 0;
    int rc = block_range(s, offset, bytes, &first, &count);
    if (rc) return rc;
    std::unique_lock<std::shared_mutex> lk(switch_lock(), std::try_to_lock);
    if (!lk.owns_lock()) return NIXIE_EBUSY;   // a switch is running: never wait for it here (it may be the caller's own)
    // work queued on any stream may still use these addresses
    hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) return fail(e);
    return unmap_blocks(s, first, count);
}

int nixie_space_mapped(const nixie_space_t *s, uint64_t offset, uint64_t bytes) {
    if (!s) return NIXIE_EINVAL;
    uint64_t first = 0, count = 0;
    int rc = block_range(s, offset, bytes, &first, &count);
    if (rc) return rc;
    for (uint64_t b = first; b < first + count; b++)   // (changed only by the owner's own map / unmap calls)
        if (s->mapped[b] != 1) return 0;
    return 1;
}

int nixie_space_destroy(nixie_space_t *s) {
    if (!s) return NIXIE_OK;
    int rc;
    {
        std::unique_lock<std::shared_mutex> lk(switch_lock(), std::try_to_lock);
        if (!lk.owns_lock()) return NIXIE_EBUSY;   // a switch is running: never wait for it here (it may be the caller's own)
        hipError_t e = hipDeviceSynchronize();
        if (e != hipSuccess) return fail(e);
        rc = unmap_blocks(s, 0, s->mapped.size());
        if (rc) return rc;
        space_unregister((uint64_t)(uintptr_t)s->base);
    }
    hipError_t e = hipMemAddressFree(s->base, s->pool->bytes);
    if (e != hipSuccess) rc = fail(e);
    {
        std::lock_guard<std::mutex> g(s->pool->mu);
        s->pool->spaces--;
    }
    delete s;
    return rc;
}

}  // extern "C"
