// Plan object, slot-credit runtime (host drain / fill threads) and nixie_switch.
//
// Paper, "Speeding Up Context Switches": the evicted application's data and the incoming
// application's data cross the host link at the same time; the pinned tier between GPU memory
// and pageable memory is small, so it is run as a stream: a slot is refilled as soon as the
// stage below has emptied it (back-pressure), a window of it is reserved for the evicted
// application so the two directions cannot block each other, and the pageable<->pinned leg is
// copied by several threads.  "Hierarchical Memory": after the switch each working set has
// exactly one copy -- A in pageable memory, B in HBM -- and the pinned ring holds nothing.
#include <hip/hip_runtime.h>
#include <time.h>

#include <algorithm>
#include <atomic>
#include <condition_variable>
#include <cstring>
#include <mutex>
#include <new>
#include <shared_mutex>
#include <thread>

#include "internal.hpp"
#include "hostside.hpp"

using namespace nixie;

namespace {

thread_local int t_last_hip_error = 0;

inline uint64_t now_ns() {
    timespec ts;
    clock_gettime(CLOCK_MONOTONIC, &ts);
    return (uint64_t)ts.tv_sec * 1000000000ull + (uint64_t)ts.tv_nsec;
}

#define NIXIE_HIP(call)                                  \
    do {                                                 \
        hipError_t e_ = (call);                          \
        if (e_ != hipSuccess) {                          \
            t_last_hip_error = (int)e_;                  \
            return NIXIE_EHIP;                           \
        }                                                \
    } while (0)


}  // namespace

struct nixie_layout {
    Layout L;
};

// Pinned payload memory that several plans use in turn.
struct nixie_ring {
    uint8_t *h = nullptr, *d = nullptr;
    uint64_t bytes = 0;
    int device = -1;
    std::mutex busy;                 // one switch at a time on this memory
    std::atomic<uint32_t> users{0};  // plans made on it and not yet destroyed
};

struct nixie_plan {
    Layout L;
    nixie_plan_info_t info{};
    int device = -1;

    // pinned, mapped, coherent
    uint8_t *ring_h = nullptr, *ring_d = nullptr;
    nixie_ring *shared = nullptr;    // non-null: ring_h / ring_d belong to it
    uint64_t *ctrl_h = nullptr, *ctrl_d = nullptr;
    size_t ctrl_bytes = 0;

    // device memory (descriptors and counters only, never payload)
    DevSeg *segs_d[2] = {nullptr, nullptr};
    DevChunk *chunks_d[2] = {nullptr, nullptr};
    uint64_t *direct_d[2] = {nullptr, nullptr};
    uint32_t *counters_d = nullptr;
    uint64_t n_counters = 0, seen_off[2] = {0, 0}, stamp_off[2] = {0, 0}, cslot_off[2] = {0, 0}, arrive_off[2] = {0, 0};
    HashDesc *hdesc_d[2] = {nullptr, nullptr};
    uint64_t htiles[2] = {0, 0};
    uint64_t *hashes_d = nullptr;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;

    bool tier_held = false;  // L.tier_ids are counted as in use by this plan

    HostSide hs;           // flags, ring and counters as the host threads see them
    HostCrew crew;         // the parked drain / fill threads
    std::mutex switch_mu;  // one switch at a time

    // a switch begun with nixie_switch_begin and not yet ended
    struct Flight {
        bool on = false;
        hipStream_t stream = nullptr;
        uint64_t t_entry = 0;
        uint32_t mask = 0;
        nixie_stats_t st{};
        std::unique_lock<std::mutex> plan_lock, ring_lock;
        std::shared_lock<std::shared_mutex> maps;
    } flight;
};

namespace {

void destroy_plan(nixie_plan_t *p) {
    if (!p) return;
    p->crew.stop();
    int prev = -1;
    if (hipGetDevice(&prev) == hipSuccess && p->device >= 0 && prev != p->device) (void)hipSetDevice(p->device);
    if (p->ev0) (void)hipEventDestroy(p->ev0);
    if (p->ev1) (void)hipEventDestroy(p->ev1);
    for (int x = 0; x < 2; x++) {
        if (p->segs_d[x]) (void)hipFree(p->segs_d[x]);
        if (p->chunks_d[x]) (void)hipFree(p->chunks_d[x]);
        if (p->direct_d[x]) (void)hipFree(p->direct_d[x]);
        if (p->hdesc_d[x]) (void)hipFree(p->hdesc_d[x]);
    }
    if (p->counters_d) (void)hipFree(p->counters_d);
    if (p->hashes_d) (void)hipFree(p->hashes_d);
    if (p->tier_held) tier_release(p->L.tier_ids);
    if (p->shared) p->shared->users.fetch_sub(1);
    else if (p->ring_h) (void)hipHostFree(p->ring_h);
    if (p->ctrl_h) (void)hipHostFree(p->ctrl_h);
    if (prev >= 0 && prev != p->device) (void)hipSetDevice(prev);
    delete p;
}

// Fresh pinned memory is mapped into the process lazily: the host threads' first pass over a new
// ring would take a page fault per 4 KiB inside the switch (about 15 ms for 256 MiB).  Touch every
// page here, where nobody is waiting.
int warm_ring(uint8_t *ring_h, uint64_t bytes) {
    const unsigned T = (unsigned)std::min<uint64_t>(std::max(1u, std::min(8u, std::thread::hardware_concurrency() / 2)),
                                                     bytes / (8u << 20) + 1);
    auto touch = [&](unsigned t) {
        volatile uint8_t *p = ring_h;
        const uint64_t per = (bytes / T + 4095) / 4096 * 4096;
        for (uint64_t off = t * per; off < std::min(bytes, (t + 1) * per); off += 4096) p[off] = 0;
    };
    std::vector<std::thread> pool;
    for (unsigned t = 1; t < T; t++) pool.emplace_back(touch, t);
    touch(0);
    for (auto &th : pool) th.join();
    return NIXIE_OK;
}

int upload(const void *src, size_t bytes, void **dst) {
    *dst = nullptr;
    if (bytes == 0) return NIXIE_OK;
    hipError_t e = hipMalloc(dst, bytes);
    if (e != hipSuccess) { t_last_hip_error = (int)e; return e == hipErrorOutOfMemory ? NIXIE_ENOMEM : NIXIE_EHIP; }
    NIXIE_HIP(hipMemcpy(*dst, src, bytes, hipMemcpyHostToDevice));
    return NIXIE_OK;
}

int create_plan(nixie_plan_t *p) {
    const Layout &L = p->L;
    NIXIE_HIP(hipGetDevice(&p->device));
    // The direct chunks carry raw GPU addresses of pinned-tier memory: from here until the plan is
    // destroyed its registrations cannot be dropped (nixie_tier_unregister returns NIXIE_EBUSY).
    if (!tier_acquire(L.tier_ids)) return NIXIE_EINVAL;   // unregistered while the layout was being made
    p->tier_held = true;

    // payload ring: exactly (out_slots + in_slots) * slot_bytes, never more than the budget
    if (p->info.pinned_ring_bytes > L.ring_bytes) return NIXIE_EINVAL;
    if (p->shared) {
        if (p->shared->device != p->device || p->info.pinned_ring_bytes > p->shared->bytes) return NIXIE_EINVAL;
        p->ring_h = p->shared->h;
        p->ring_d = p->shared->d;
    } else if (p->info.pinned_ring_bytes) {
        hipError_t e = hipHostMalloc((void **)&p->ring_h, p->info.pinned_ring_bytes,
                                     hipHostMallocMapped | hipHostMallocCoherent);
        if (e != hipSuccess) { t_last_hip_error = (int)e; return NIXIE_ENOMEM; }
        NIXIE_HIP(hipHostGetDevicePointer((void **)&p->ring_d, p->ring_h, 0));
        int rc = warm_ring(p->ring_h, p->info.pinned_ring_bytes);
        if (rc) return rc;
    }
    // control block: [host-written flags out | in (8 B each, padded to lines)] [GPU-written flags out | in
    // (one 64 B line each)] [abort word] [status word] [direction-done words]
    p->ctrl_bytes = p->info.pinned_ctrl_bytes;
    {
        hipError_t e = hipHostMalloc((void **)&p->ctrl_h, p->ctrl_bytes, hipHostMallocMapped | hipHostMallocCoherent);
        if (e != hipSuccess) { t_last_hip_error = (int)e; return NIXIE_ENOMEM; }
        NIXIE_HIP(hipHostGetDevicePointer((void **)&p->ctrl_d, p->ctrl_h, 0));
        std::memset(p->ctrl_h, 0, p->ctrl_bytes);
    }
    uint64_t *c = p->ctrl_h;
    p->hs.wait[0] = c;                                   c += wait_flag_words(L.dir[0].slots);
    p->hs.wait[1] = c;                                   c += wait_flag_words(L.dir[1].slots);
    p->hs.post[0] = c;                                   c += (size_t)L.dir[0].slots * kFlagStride;
    p->hs.post[1] = c;                                   c += (size_t)L.dir[1].slots * kFlagStride;
    p->hs.abort_word = (uint32_t *)c;                         c += kFlagStride;
    p->hs.status_word = (uint32_t *)c;                        c += kFlagStride;
    p->hs.done_word = (uint32_t *)c;                          c += kFlagStride;
    if ((size_t)(c - p->ctrl_h) * 8 != p->ctrl_bytes) return NIXIE_EINVAL;

    // descriptors
    for (int x = 0; x < 2; x++) {
        const DirLayout &D = L.dir[x];
        std::vector<DevSeg> segs(D.segs.size());
        for (size_t i = 0; i < segs.size(); i++) segs[i] = DevSeg{D.segs[i].dev_addr, D.segs[i].slot_off, D.segs[i].len};
        std::vector<DevChunk> chunks(D.chunks.size());
        for (size_t i = 0; i < chunks.size(); i++)
            chunks[i] = DevChunk{(uint32_t)D.chunks[i].seg_begin, D.chunks[i].seg_count, D.chunks[i].used_bytes,
                                 (uint32_t)D.chunks[i].dep_out};
        int rc = upload(segs.data(), segs.size() * sizeof(DevSeg), (void **)&p->segs_d[x]);
        if (rc) return rc;
        rc = upload(chunks.data(), chunks.size() * sizeof(DevChunk), (void **)&p->chunks_d[x]);
        if (rc) return rc;
        rc = upload(D.direct_base.data(), D.direct_base.size() * sizeof(uint64_t), (void **)&p->direct_d[x]);
        if (rc) return rc;

        // hash descriptors of the table (table order)
        const auto &T = L.table[x];
        std::vector<HashDesc> hd(T.size());
        uint64_t tiles = 0;
        for (size_t i = 0; i < T.size(); i++) {
            hd[i] = HashDesc{(uint64_t)(uintptr_t)T[i].dev_ptr, T[i].bytes, tiles};
            uint64_t words = (T[i].bytes + 7) / 8;
            tiles += (words + kHashTileWords - 1) / kHashTileWords;
        }
        p->htiles[x] = tiles;
        rc = upload(hd.data(), hd.size() * sizeof(HashDesc), (void **)&p->hdesc_d[x]);
        if (rc) return rc;
    }
    // counters (u32 units): [0] ticket out, [1] ticket in, [2] abort, [3] pad, [4,5] stall out, [6,7] stall in,
    // [8] exited out, [9] exited in, [10] gathered prefix, [11] workgroups that have left, [12..15] pad, then per
    // direction: seen[] and stamp[] (u64 per slot), chunk_slot[] and arrive[] (u32 per chunk).  All zero between switches:
    // cleared here once, and by the last workgroup to leave every kernel.
    uint64_t off = 16;
    for (int x = 0; x < 2; x++) { p->seen_off[x] = off; off += 2 * wait_flag_words(L.dir[x].slots); }
    for (int x = 0; x < 2; x++) { p->stamp_off[x] = off; off += 2 * wait_flag_words(L.dir[x].slots); }
    for (int x = 0; x < 2; x++) { p->cslot_off[x] = off; off += L.dir[x].chunks.size(); }
    for (int x = 0; x < 2; x++) { p->arrive_off[x] = off; off += L.dir[x].chunks.size(); }
    p->n_counters = off;
    {
        hipError_t e = hipMalloc((void **)&p->counters_d, p->n_counters * sizeof(uint32_t));
        if (e != hipSuccess) { t_last_hip_error = (int)e; return NIXIE_ENOMEM; }
        NIXIE_HIP(hipMemset(p->counters_d, 0, p->n_counters * sizeof(uint32_t)));
        NIXIE_HIP(hipDeviceSynchronize());
    }
    const size_t n_hash = std::max<size_t>(1, std::max(L.table[0].size(), L.table[1].size()));
    {
        hipError_t e = hipMalloc((void **)&p->hashes_d, n_hash * sizeof(uint64_t));
        if (e != hipSuccess) { t_last_hip_error = (int)e; return NIXIE_ENOMEM; }
    }
    NIXIE_HIP(hipEventCreate(&p->ev0));
    NIXIE_HIP(hipEventCreate(&p->ev1));

    p->hs.L = &p->L;
    p->hs.ring = p->ring_h;
    p->hs.threads[0] = p->info.drain_threads;
    p->hs.threads[1] = p->info.fill_threads;
    // +1: the thread that calls nixie_switch also needs a core while it launches the kernel
    p->hs.yield_when_idle = p->info.drain_threads + p->info.fill_threads + 1 > std::max(1u, std::thread::hardware_concurrency());
    if (!(L.opts.flags & NIXIE_HOST_SPIN)) {
        // One sixteenth of the time the smaller direction's share of the ring lasts at link rate
        // (50 GB/s = 50 B/ns), at most 50 us; below 4 us a system call is not worth it.
        uint64_t share = 0;
        for (int x = 0; x < 2; x++) {
            const uint64_t b = (uint64_t)L.dir[x].slots * L.slot_bytes;
            if (b && (share == 0 || b < share)) share = b;
        }
        const uint64_t nap = std::min<uint64_t>(50000, share / 50 / 16);
        p->hs.idle_sleep_ns = nap < 4000 ? 0 : nap;
    }
    p->crew.start(&p->hs);
    return NIXIE_OK;
}

// One pass: the directions in mask run together.  pass_begin launches and returns; pass_end waits
// for the host threads and the kernel and collects the figures.
int pass_begin(nixie_plan_t *p, uint32_t mask, hipStream_t stream, nixie_stats_t *st, uint64_t t_entry) {
    const Layout &L = p->L;
    std::memset(p->ctrl_h, 0, p->ctrl_bytes);
    p->hs.begin_pass();   // counters to zero, every outgoing slot marked released

    SwapArgs a{};
    for (int x = 0; x < 2; x++) {
        const DirLayout &D = L.dir[x];
        DevDir &d = a.d[x];
        const bool on = (mask & (1u << x)) && !D.chunks.empty();
        d.segs = p->segs_d[x];
        d.chunks = p->chunks_d[x];
        d.ring = p->ring_d + (x ? (uint64_t)L.dir[0].slots * L.slot_bytes : 0);
        const size_t wait_off = (size_t)(p->hs.wait[x] - p->ctrl_h), post_off = (size_t)(p->hs.post[x] - p->ctrl_h);
        d.host_flags = p->ctrl_d + wait_off;
        d.post_flags = p->ctrl_d + post_off;
        d.ticket = p->counters_d + x;
        d.exited = p->counters_d + 8 + x;
        d.seen = (uint64_t *)(p->counters_d + p->seen_off[x]);
        d.stamp = (uint64_t *)(p->counters_d + p->stamp_off[x]);
        d.chunk_slot = p->counters_d + p->cslot_off[x];
        d.arrive = p->counters_d + p->arrive_off[x];
        d.stall_ticks = (uint64_t *)(p->counters_d + 4 + 2 * x);
        d.n_chunks = on ? (uint32_t)D.chunks.size() : 0;
        d.n_staged = on ? (uint32_t)D.staged : 0;
        d.direct_base = p->direct_d[x];
        d.n_slots = D.slots;
        d.team = x ? p->info.team_in : p->info.team_out;
        if (d.team == 0) d.team = 1;
        a.fixed_wgs[x] = on ? (x ? p->info.scatter_wgs : p->info.gather_wgs) : 0;
    }
    a.flex_wgs = (a.fixed_wgs[0] && a.fixed_wgs[1]) ? p->info.flex_wgs : 0;
    for (int x = 0; x < 2; x++) a.d[x].wgs = a.fixed_wgs[x] ? a.fixed_wgs[x] + a.flex_wgs : 0;
    a.slot_bytes = L.slot_bytes;
    a.host_abort = (const uint32_t *)(p->ctrl_d + (size_t)((uint64_t *)p->hs.abort_word - p->ctrl_h));
    a.gpu_status = (uint32_t *)(p->ctrl_d + (size_t)((uint64_t *)p->hs.status_word - p->ctrl_h));
    a.dir_done = (uint32_t *)(p->ctrl_d + (size_t)((uint64_t *)p->hs.done_word - p->ctrl_h));
    a.dev_abort = p->counters_d + 2;
    a.timeout_ticks = p->hs.timeout_ns / 10;   // wall clock runs at 100 MHz
    a.gathered_prefix = p->counters_d + 10;
    a.all_left = p->counters_d + 11;
    a.counters = p->counters_d;
    a.n_counters = p->n_counters;
    a.stall_out = (uint64_t *)(a.dir_done + kStallWord);
    a.xcd_mask = L.opts.xcd_mask & 0xFFu;
    // when the directions run one after the other, everything has left HBM before the restore starts
    a.track_prefix = ((L.opts.flags & NIXIE_IN_PLACE) && a.d[0].wgs && a.d[1].wgs) ? 1u : 0u;
    // a direction that does not run in this pass has nothing to wait for
    for (int x = 0; x < 2; x++)
        if (a.d[x].wgs == 0) ((uint32_t *)p->hs.done_word)[x] = 1;

    // The host threads start first: while the launches below are in flight they are already waking
    // up and loading the first incoming slots.
    p->crew.wake(mask);
    int e = (int)hipEventRecord(p->ev0, stream);
    if (!e) e = nixie_launch_swap(a, stream);
    if (!e) e = (int)hipEventRecord(p->ev1, stream);
    if (e) {
        // Something on the launch path failed.  The kernel may or may not be running: tell both
        // halves to stop (the pump relays the abort word to every workgroup), let the threads
        // finish, and drain the stream before returning, so that the caller can never destroy
        // the plan (ring, flags, descriptors) underneath a live kernel.
        t_last_hip_error = e;
        p->hs.raise_abort(NIXIE_EHIP);
        p->crew.wait();
        (void)hipStreamSynchronize(stream);
        return NIXIE_EHIP;
    }
    if (st && st->ns_launch == 0) st->ns_launch = now_ns() - t_entry;
    return NIXIE_OK;
}

int pass_end(nixie_plan_t *p, uint32_t mask, hipStream_t stream, nixie_stats_t *st) {
    const Layout &L = p->L;
    p->crew.wait();   // drain / fill threads done (finished, aborted or timed out)
    // A long switch whose chunks move without host threads would leave the caller spinning in the
    // stream synchronize for its whole length: sleep in short naps until the kernel's pump waves
    // report both directions complete (or the switch fails), then synchronize.
    if (L.dir[0].bytes + L.dir[1].bytes >= (256ull << 20) && !(L.opts.flags & NIXIE_HOST_SPIN))
        for (int x = 0; x < 2; x++)
            if ((mask & (1u << x)) && p->hs.wait_direction(x, 50000) != NIXIE_OK) break;
    hipError_t se = hipStreamSynchronize(stream);
    if (se != hipSuccess) { t_last_hip_error = (int)se; return NIXIE_EHIP; }
    // directly moved chunks are complete when the kernel is: no host thread saw them go by
    for (int x = 0; x < 2; x++)
        if ((mask & (1u << x)) && L.dir[x].staged < L.dir[x].chunks.size() && p->hs.end_ns[x].load() == 0)
            p->hs.end_ns[x].store(now_ns());

    if (st) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, p->ev0, p->ev1) == hipSuccess) st->ns_kernel += (uint64_t)((double)ms * 1e6);
        // written by the last workgroup to leave; the kernel is complete, so they are final
        const uint64_t *stall = (const uint64_t *)(p->hs.done_word + kStallWord);
        st->gather_stall_ticks += __atomic_load_n(stall + 0, __ATOMIC_ACQUIRE);
        st->scatter_stall_ticks += __atomic_load_n(stall + 1, __ATOMIC_ACQUIRE);
        st->pump_rounds_out += __atomic_load_n(p->hs.done_word + kRoundsWord + 0, __ATOMIC_ACQUIRE);
        st->pump_rounds_in += __atomic_load_n(p->hs.done_word + kRoundsWord + 1, __ATOMIC_ACQUIRE);
        st->credit_rtt_ticks_out = __atomic_load_n(p->hs.done_word + kRttWord + 0, __ATOMIC_ACQUIRE);
        st->credit_rtt_ticks_in = __atomic_load_n(p->hs.done_word + kRttWord + 1, __ATOMIC_ACQUIRE);
        st->drain_wait_ns += p->hs.wait_ns[0].load();
        st->fill_wait_ns += p->hs.wait_ns[1].load();
        st->kernels++;
        const uint32_t gs = __atomic_load_n(p->hs.status_word, __ATOMIC_ACQUIRE);
        if (gs) st->gpu_status = gs;
    }
    int err = p->hs.error.load();
    if (!err && __atomic_load_n(p->hs.status_word, __ATOMIC_ACQUIRE) != kGpuOk) err = NIXIE_ETIMEOUT;
    return err;
}

int run_pass(nixie_plan_t *p, uint32_t mask, hipStream_t stream, nixie_stats_t *st, uint64_t t_entry) {
    int rc = pass_begin(p, mask, stream, st, t_entry);
    return rc ? rc : pass_end(p, mask, stream, st);
}

void finish_stats(nixie_plan_t *p, nixie_stats_t &st, uint64_t t_entry) {
    st.ns_total = now_ns() - t_entry;
    st.ns_out_done = p->hs.end_ns[0].load() > t_entry ? p->hs.end_ns[0].load() - t_entry : 0;
    st.ns_in_done = p->hs.end_ns[1].load() > t_entry ? p->hs.end_ns[1].load() - t_entry : 0;
}

void reset_for_switch(nixie_plan_t *p, nixie_stats_t &st) {
    st = nixie_stats_t{};
    st.bytes_out = p->L.dir[0].bytes;
    st.bytes_in = p->L.dir[1].bytes;
    p->hs.timeout_ns = (uint64_t)(p->L.opts.timeout_ms ? p->L.opts.timeout_ms : 30000u) * 1000000ull;
    p->hs.error.store(0);
    p->hs.end_ns[0].store(0);
    p->hs.end_ns[1].store(0);
}

}  // namespace

extern "C" {

int nixie_layout_create(const nixie_table_t *out_table, const nixie_table_t *in_table, uint64_t ring_bytes,
                        const nixie_opts_t *opts, nixie_layout_t **layout) {
    if (!layout) return NIXIE_EINVAL;
    nixie_layout *l = new (std::nothrow) nixie_layout();
    if (!l) return NIXIE_ENOMEM;
    int rc;
    try {
        rc = build_layout(out_table, in_table, ring_bytes, opts, l->L);
    } catch (const std::bad_alloc &) {
        rc = NIXIE_ENOMEM;
    }
    if (rc) { delete l; return rc; }
    *layout = l;
    return NIXIE_OK;
}

int nixie_layout_info(const nixie_layout_t *layout, nixie_plan_info_t *info) {
    if (!layout || !info) return NIXIE_EINVAL;
    fill_info(layout->L, info);
    return NIXIE_OK;
}

int64_t nixie_layout_chunks(const nixie_layout_t *layout, int dir, nixie_chunk_t *chunks, uint64_t cap) {
    if (!layout || dir < 0 || dir > 1 || (cap && !chunks)) return NIXIE_EINVAL;
    const auto &v = layout->L.dir[dir].chunks;
    const uint64_t n = std::min<uint64_t>(cap, v.size());
    if (n) std::memcpy(chunks, v.data(), n * sizeof(nixie_chunk_t));
    return (int64_t)v.size();
}

int64_t nixie_layout_segments(const nixie_layout_t *layout, int dir, nixie_segment_t *segs, uint64_t cap) {
    if (!layout || dir < 0 || dir > 1 || (cap && !segs)) return NIXIE_EINVAL;
    const auto &v = layout->L.dir[dir].segs;
    const uint64_t n = std::min<uint64_t>(cap, v.size());
    if (n) std::memcpy(segs, v.data(), n * sizeof(nixie_segment_t));
    return (int64_t)v.size();
}

void nixie_layout_destroy(nixie_layout_t *layout) { delete layout; }

int nixie_plan(const nixie_table_t *out_table, const nixie_table_t *in_table, uint64_t ring_bytes,
               const nixie_opts_t *opts, nixie_plan_t **plan) {
    if (!plan) return NIXIE_EINVAL;
    nixie_plan_t *p = new (std::nothrow) nixie_plan_t();
    if (!p) return NIXIE_ENOMEM;
    int rc;
    try {
        rc = build_layout(out_table, in_table, ring_bytes, opts, p->L);
        if (!rc) {
            fill_info(p->L, &p->info);
            rc = create_plan(p);
        }
    } catch (const std::bad_alloc &) {
        rc = NIXIE_ENOMEM;
    } catch (const std::system_error &) {
        rc = NIXIE_ENOMEM;
    }
    if (rc) { destroy_plan(p); return rc; }
    *plan = p;
    return NIXIE_OK;
}

int nixie_ring_create(uint64_t bytes, nixie_ring_t **ring) {
    if (!ring || bytes == 0 || bytes % 4096) return NIXIE_EINVAL;
    *ring = nullptr;
    nixie_ring *r = new (std::nothrow) nixie_ring;
    if (!r) return NIXIE_ENOMEM;
    hipError_t e = hipGetDevice(&r->device);
    if (e == hipSuccess) e = hipHostMalloc((void **)&r->h, bytes, hipHostMallocMapped | hipHostMallocCoherent);
    if (e != hipSuccess) { t_last_hip_error = (int)e; delete r; return e == hipErrorOutOfMemory ? NIXIE_ENOMEM : NIXIE_EHIP; }
    e = hipHostGetDevicePointer((void **)&r->d, r->h, 0);
    if (e != hipSuccess) { t_last_hip_error = (int)e; (void)hipHostFree(r->h); delete r; return NIXIE_EHIP; }
    r->bytes = bytes;
    const int rc = warm_ring(r->h, bytes);
    if (rc) { (void)hipHostFree(r->h); delete r; return rc; }
    *ring = r;
    return NIXIE_OK;
}

int nixie_ring_destroy(nixie_ring_t *ring) {
    if (!ring) return NIXIE_OK;
    if (ring->users.load()) return NIXIE_EBUSY;
    (void)hipHostFree(ring->h);
    delete ring;
    return NIXIE_OK;
}

int nixie_plan_on_ring(const nixie_table_t *out_table, const nixie_table_t *in_table, nixie_ring_t *ring,
                       const nixie_opts_t *opts, nixie_plan_t **plan) {
    if (!plan || !ring) return NIXIE_EINVAL;
    nixie_plan_t *p = new (std::nothrow) nixie_plan_t();
    if (!p) return NIXIE_ENOMEM;
    int rc;
    try {
        rc = build_layout(out_table, in_table, ring->bytes, opts, p->L);
        if (!rc) {
            fill_info(p->L, &p->info);
            p->shared = ring;
            ring->users.fetch_add(1);
            rc = create_plan(p);
        }
    } catch (const std::bad_alloc &) {
        rc = NIXIE_ENOMEM;
    } catch (const std::system_error &) {
        rc = NIXIE_ENOMEM;
    }
    if (rc) { destroy_plan(p); return rc; }
    *plan = p;
    return NIXIE_OK;
}

int nixie_plan_info(const nixie_plan_t *plan, nixie_plan_info_t *info) {
    if (!plan || !info) return NIXIE_EINVAL;
    *info = plan->info;
    return NIXIE_OK;
}

void nixie_plan_destroy(nixie_plan_t *plan) {
    if (plan && plan->flight.on) {           // a switch was begun and never ended: stop it first
        plan->hs.raise_abort(NIXIE_EBUSY);
        (void)nixie_switch_end(plan, nullptr);
    }
    destroy_plan(plan);
}

int nixie_switch(nixie_plan_t *p, void *hip_stream, nixie_stats_t *stats) {
    if (!p) return NIXIE_EINVAL;
    std::unique_lock<std::mutex> lk(p->switch_mu, std::try_to_lock);
    if (!lk.owns_lock()) return NIXIE_EBUSY;
    std::unique_lock<std::mutex> ring_lk;
    if (p->shared) {
        ring_lk = std::unique_lock<std::mutex>(p->shared->busy, std::try_to_lock);
        if (!ring_lk.owns_lock()) return NIXIE_EBUSY;   // another plan is switching through the same ring
    }
    // no block of a registered space is mapped or unmapped while the kernel runs
    std::shared_lock<std::shared_mutex> maps(switch_lock());
    if (!space_uses_valid(p->L.uses[0]) || !space_uses_valid(p->L.uses[1])) return NIXIE_EUNMAPPED;
    const uint64_t t_entry = now_ns();
    int dev = -1;
    NIXIE_HIP(hipGetDevice(&dev));
    if (dev != p->device) return NIXIE_EINVAL;
    nixie_stats_t st;
    reset_for_switch(p, st);

    int rc = NIXIE_OK;
    const bool both = !p->L.dir[0].chunks.empty() && !p->L.dir[1].chunks.empty();
    if ((p->L.opts.flags & NIXIE_SERIALIZE) && both) {
        rc = run_pass(p, 1u, (hipStream_t)hip_stream, &st, t_entry);
        if (!rc) rc = run_pass(p, 2u, (hipStream_t)hip_stream, &st, t_entry);
    } else {
        rc = run_pass(p, 3u, (hipStream_t)hip_stream, &st, t_entry);
    }
    finish_stats(p, st, t_entry);
    if (stats) *stats = st;
    return rc;
}

int nixie_switch_begin(nixie_plan_t *p, void *hip_stream) {
    if (!p) return NIXIE_EINVAL;
    if (p->L.opts.flags & NIXIE_SERIALIZE) return NIXIE_EINVAL;   // two passes cannot be left running
    std::unique_lock<std::mutex> lk(p->switch_mu, std::try_to_lock);
    if (!lk.owns_lock()) return NIXIE_EBUSY;
    std::unique_lock<std::mutex> ring_lk;
    if (p->shared) {
        ring_lk = std::unique_lock<std::mutex>(p->shared->busy, std::try_to_lock);
        if (!ring_lk.owns_lock()) return NIXIE_EBUSY;
    }
    std::shared_lock<std::shared_mutex> maps(switch_lock());
    if (!space_uses_valid(p->L.uses[0]) || !space_uses_valid(p->L.uses[1])) return NIXIE_EUNMAPPED;
    const uint64_t t_entry = now_ns();
    int dev = -1;
    NIXIE_HIP(hipGetDevice(&dev));
    if (dev != p->device) return NIXIE_EINVAL;
    nixie_plan::Flight &f = p->flight;
    reset_for_switch(p, f.st);
    int rc = pass_begin(p, 3u, (hipStream_t)hip_stream, &f.st, t_entry);
    if (rc) return rc;                                           // nothing is left running
    f.on = true;
    f.stream = (hipStream_t)hip_stream;
    f.t_entry = t_entry;
    f.mask = 3u;
    f.plan_lock = std::move(lk);                                 // held until nixie_switch_end
    f.ring_lock = std::move(ring_lk);
    f.maps = std::move(maps);
    return NIXIE_OK;
}

int nixie_switch_wait_in(nixie_plan_t *p) {
    if (!p || !p->flight.on) return NIXIE_EINVAL;
    const int rc = p->hs.wait_direction(1);
    if (!rc && p->hs.end_ns[1].load() == 0) p->hs.end_ns[1].store(now_ns());
    return rc;
}

int nixie_switch_end(nixie_plan_t *p, nixie_stats_t *stats) {
    if (!p || !p->flight.on) return NIXIE_EINVAL;
    nixie_plan::Flight &f = p->flight;
    const int rc = pass_end(p, f.mask, f.stream, &f.st);
    finish_stats(p, f.st, f.t_entry);
    if (stats) *stats = f.st;
    f.on = false;
    f.maps.unlock();
    if (f.ring_lock.owns_lock()) f.ring_lock.unlock();
    f.plan_lock.unlock();
    return rc;
}

int nixie_abi_check(uint64_t sizeof_opts, uint64_t sizeof_plan_info, uint64_t sizeof_stats) {
    return sizeof_opts == sizeof(nixie_opts_t) && sizeof_plan_info == sizeof(nixie_plan_info_t) &&
                   sizeof_stats == sizeof(nixie_stats_t)
               ? NIXIE_OK
               : NIXIE_EINVAL;
}

const char *nixie_strerror(int err) {
    switch (err) {
    case NIXIE_OK: return "ok";
    case NIXIE_EINVAL: return "invalid argument";
    case NIXIE_EOVERLAP: return "allocation ranges overlap";
    case NIXIE_ENOMEM: return "out of memory (pinned or descriptor allocation failed)";
    case NIXIE_EHIP: return "HIP runtime error";
    case NIXIE_ETIMEOUT: return "credit wait timed out; switch aborted";
    case NIXIE_EMISMATCH: return "hash mismatch";
    case NIXIE_EBUSY: return "busy: the plan is running a switch, or the pool still has spaces";
    case NIXIE_EUNMAPPED: return "a listed device range lies in unmapped blocks of a space";
    default: return "unknown error";
    }
}

int nixie_last_hip_error(void) { return t_last_hip_error; }

}  // extern "C"

// shared with verify.cpp
namespace nixie {
void set_last_hip_error(int e) { t_last_hip_error = e; }
const Layout &plan_layout(const nixie_plan_t *p) { return p->L; }
HashDesc *plan_hash_descs(const nixie_plan_t *p, int x) { return p->hdesc_d[x]; }
uint64_t plan_hash_tiles(const nixie_plan_t *p, int x) { return p->htiles[x]; }
uint64_t *plan_hash_buffer(const nixie_plan_t *p) { return p->hashes_d; }
int plan_device(const nixie_plan_t *p) { return p->device; }
}  // namespace nixie
