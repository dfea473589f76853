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
#include <immintrin.h>
#include <time.h>

#include <atomic>
#include <condition_variable>
#include <cstring>
#include <mutex>
#include <new>
#include <thread>

#include "internal.hpp"

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

inline uint64_t load_acq(const uint64_t *p) { return __atomic_load_n(p, __ATOMIC_ACQUIRE); }
inline void store_rel(uint64_t *p, uint64_t v) { __atomic_store_n(p, v, __ATOMIC_RELEASE); }

}  // namespace

struct nixie_layout {
    Layout L;
};

struct nixie_plan {
    Layout L;
    nixie_plan_info_t info{};
    int device = -1;

    // pinned, mapped, coherent
    uint8_t *ring_h = nullptr, *ring_d = nullptr;
    uint64_t *ctrl_h = nullptr, *ctrl_d = nullptr;
    size_t ctrl_bytes = 0;
    uint64_t *wait_h[2] = {nullptr, nullptr}, *post_h[2] = {nullptr, nullptr};  // host views of the flag arrays
    uint32_t *abort_h = nullptr, *status_h = nullptr;

    // device memory (descriptors and counters only, never payload)
    DevSeg *segs_d[2] = {nullptr, nullptr};
    DevChunk *chunks_d[2] = {nullptr, nullptr};
    uint32_t *counters_d = nullptr;
    uint64_t n_counters = 0, seen_off[2] = {0, 0}, cslot_off[2] = {0, 0}, arrive_off[2] = {0, 0};
    HashDesc *hdesc_d[2] = {nullptr, nullptr};
    uint64_t htiles[2] = {0, 0};
    uint64_t *hashes_d = nullptr;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;

    // workers
    std::vector<std::thread> threads;
    std::mutex mu;
    std::condition_variable cv_go, cv_done;
    uint64_t epoch = 0;
    bool quit = false;
    uint32_t running = 0;

    // state of the switch in flight
    std::mutex switch_mu;
    uint32_t pass_mask = 0;
    uint64_t timeout_ns = 0;
    std::atomic<uint64_t> next_chunk[2];
    std::atomic<uint64_t> done_chunks[2];
    std::atomic<int> error{0};
    std::atomic<uint32_t> abort_local{0};
    std::atomic<uint64_t> wait_ns[2];
    std::atomic<uint64_t> end_ns[2];   // latest completion time seen per direction
};

namespace {

void raise_abort(nixie_plan_t *p, int err) {
    int expected = 0;
    p->error.compare_exchange_strong(expected, err);
    p->abort_local.store(1, std::memory_order_release);
    __atomic_store_n(p->abort_h, 1u, __ATOMIC_RELEASE);   // the kernel polls this word
}

// Idle bookkeeping of a host thread that scans its slots: aborts the switch when nothing has
// moved for longer than the bound, or when the kernel reported that it gave up.
struct IdleWatch {
    nixie_plan_t *p;
    int dir;
    uint64_t idle_since = 0;
    uint32_t spins = 0;
    // call after a scan that made no progress; false = stop
    bool idle() {
        _mm_pause();
        if (idle_since == 0) idle_since = now_ns();
        if ((++spins & 63u) != 0) return true;
        if (p->abort_local.load(std::memory_order_acquire)) return false;
        if (__atomic_load_n(p->status_h, __ATOMIC_ACQUIRE) != kGpuOk || now_ns() - idle_since > p->timeout_ns) {
            raise_abort(p, NIXIE_ETIMEOUT);
            return false;
        }
        return true;
    }
    void progressed() {
        if (idle_since) p->wait_ns[dir].fetch_add(now_ns() - idle_since, std::memory_order_relaxed);
        idle_since = 0;
    }
};

void note_end(nixie_plan_t *p, int dir) {
    uint64_t t = now_ns(), cur = p->end_ns[dir].load(std::memory_order_relaxed);
    while (cur < t && !p->end_ns[dir].compare_exchange_weak(cur, t, std::memory_order_relaxed)) {}
}

// ring -> pageable.  Consumer of the outgoing direction.  Thread idx owns slots idx, idx + T, ...
// and drains whichever of them the GPU has marked ready (ready[s] = chunk id + 1), in any order.
void run_drain(nixie_plan_t *p, uint32_t idx, uint32_t T) {
    const DirLayout &D = p->L.dir[0];
    const uint32_t flags = p->L.opts.flags;
    const uint64_t n = D.chunks.size(), S = p->L.slot_bytes;
    const bool plain = flags & NIXIE_HOST_PLAIN_MEMCPY;
    std::vector<uint64_t> last(D.slots, 0);
    IdleWatch watch{p, 0};
    while (p->done_chunks[0].load(std::memory_order_acquire) < n) {
        bool moved = false;
        for (uint64_t slot = idx; slot < D.slots; slot += T) {
            const uint64_t v = load_acq(p->post_h[0] + slot * kFlagStride);
            if (v == last[slot]) continue;
            last[slot] = v;
            const uint64_t k = v - 1;
            if (k >= n) { raise_abort(p, NIXIE_EINVAL); return; }
            if (!(flags & NIXIE_DIAG_RING_ONLY)) {
                const nixie_chunk_t &c = D.chunks[k];
                const uint8_t *src = p->ring_h + slot * S;
                for (uint64_t q = c.seg_begin; q < c.seg_begin + c.seg_count; q++) {
                    const nixie_segment_t &sg = D.segs[q];
                    if (plain) std::memcpy((void *)(uintptr_t)sg.host_addr, src + sg.slot_off, sg.len);
                    else copy_stream((void *)(uintptr_t)sg.host_addr, src + sg.slot_off, sg.len);
                }
                _mm_sfence();
            }
            if (!(flags & NIXIE_DIAG_STALL_DRAIN)) store_rel(p->wait_h[0] + slot, k + 2);   // released
            p->done_chunks[0].fetch_add(1, std::memory_order_acq_rel);
            moved = true;
        }
        if (moved) watch.progressed();
        else if (!watch.idle()) return;
    }
    watch.progressed();
    note_end(p, 0);
}

// pageable -> ring.  Producer of the incoming direction.  Thread idx owns slots idx, idx + T, ...;
// whenever one of them is free it claims the next chunk, loads it and publishes filled[s] = id + 1.
// A slot is free again when the GPU has written freed[s] = id + 1 for the chunk it held.
void run_fill(nixie_plan_t *p, uint32_t idx, uint32_t T) {
    const DirLayout &D = p->L.dir[1];
    const uint32_t flags = p->L.opts.flags;
    const uint64_t n = D.chunks.size(), S = p->L.slot_bytes;
    const bool plain = flags & NIXIE_HOST_PLAIN_MEMCPY;
    std::vector<uint64_t> pending(D.slots, 0);
    uint64_t outstanding = 0;
    bool claiming = true;
    IdleWatch watch{p, 1};
    for (;;) {
        bool moved = false;
        for (uint64_t slot = idx; slot < D.slots; slot += T) {
            if (pending[slot]) {
                if (load_acq(p->post_h[1] + slot * kFlagStride) != pending[slot]) continue;
                pending[slot] = 0;
                outstanding--;
                moved = true;
            }
            if (!claiming) continue;
            const uint64_t k = p->next_chunk[1].fetch_add(1, std::memory_order_relaxed);
            if (k >= n) { claiming = false; continue; }
            if (!(flags & NIXIE_DIAG_RING_ONLY)) {
                const nixie_chunk_t &c = D.chunks[k];
                uint8_t *dst = p->ring_h + ((uint64_t)p->L.dir[0].slots + slot) * S;
                for (uint64_t q = c.seg_begin; q < c.seg_begin + c.seg_count; q++) {
                    const nixie_segment_t &sg = D.segs[q];
                    if (plain) std::memcpy(dst + sg.slot_off, (const void *)(uintptr_t)sg.host_addr, sg.len);
                    else copy_stream(dst + sg.slot_off, (const void *)(uintptr_t)sg.host_addr, sg.len);
                }
                _mm_sfence();
            }
            store_rel(p->wait_h[1] + slot, k + 1);   // filled
            pending[slot] = k + 1;
            outstanding++;
            moved = true;
        }
        if (!claiming && outstanding == 0) break;
        if (moved) watch.progressed();
        else if (!watch.idle()) return;
    }
    watch.progressed();
    note_end(p, 1);   // this thread's last chunk has reached HBM; the latest such time is "B ready"
}

void worker_main(nixie_plan_t *p, int dir, uint32_t idx) {
    uint64_t seen = 0;
    for (;;) {
        {
            std::unique_lock<std::mutex> lk(p->mu);
            p->cv_go.wait(lk, [&] { return p->quit || p->epoch != seen; });
            if (p->quit) return;
            seen = p->epoch;
        }
        if (p->pass_mask & (1u << dir)) {
            if (dir == 0) run_drain(p, idx, p->info.drain_threads);
            else run_fill(p, idx, p->info.fill_threads);
        }
        {
            std::lock_guard<std::mutex> lk(p->mu);
            if (--p->running == 0) p->cv_done.notify_all();
        }
    }
}

void destroy_plan(nixie_plan_t *p) {
    if (!p) return;
    {
        std::lock_guard<std::mutex> lk(p->mu);
        p->quit = true;
    }
    p->cv_go.notify_all();
    for (auto &t : p->threads) t.join();
    int prev = -1;
    if (hipGetDevice(&prev) == hipSuccess && p->device >= 0 && prev != p->device) (void)hipSetDevice(p->device);
    if (p->ev0) (void)hipEventDestroy(p->ev0);
    if (p->ev1) (void)hipEventDestroy(p->ev1);
    for (int x = 0; x < 2; x++) {
        if (p->segs_d[x]) (void)hipFree(p->segs_d[x]);
        if (p->chunks_d[x]) (void)hipFree(p->chunks_d[x]);
        if (p->hdesc_d[x]) (void)hipFree(p->hdesc_d[x]);
    }
    if (p->counters_d) (void)hipFree(p->counters_d);
    if (p->hashes_d) (void)hipFree(p->hashes_d);
    if (p->ring_h) (void)hipHostFree(p->ring_h);
    if (p->ctrl_h) (void)hipHostFree(p->ctrl_h);
    if (prev >= 0 && prev != p->device) (void)hipSetDevice(prev);
    delete p;
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
    const uint32_t n_slots = L.dir[0].slots + L.dir[1].slots;

    // payload ring: exactly n_slots * slot_bytes, never more than the budget
    if (p->info.pinned_ring_bytes > L.ring_bytes) return NIXIE_EINVAL;
    if (p->info.pinned_ring_bytes) {
        hipError_t e = hipHostMalloc((void **)&p->ring_h, p->info.pinned_ring_bytes,
                                     hipHostMallocMapped | hipHostMallocCoherent);
        if (e != hipSuccess) { t_last_hip_error = (int)e; return NIXIE_ENOMEM; }
        NIXIE_HIP(hipHostGetDevicePointer((void **)&p->ring_d, p->ring_h, 0));
    }
    // control block: one 64 B line per flag; [out wait | out post | in wait | in post | abort | status]
    p->ctrl_bytes = p->info.pinned_ctrl_bytes;
    {
        hipError_t e = hipHostMalloc((void **)&p->ctrl_h, p->ctrl_bytes, hipHostMallocMapped | hipHostMallocCoherent);
        if (e != hipSuccess) { t_last_hip_error = (int)e; return NIXIE_ENOMEM; }
        NIXIE_HIP(hipHostGetDevicePointer((void **)&p->ctrl_d, p->ctrl_h, 0));
        std::memset(p->ctrl_h, 0, p->ctrl_bytes);
    }
    uint64_t *c = p->ctrl_h;
    p->wait_h[0] = c;                                   c += wait_flag_words(L.dir[0].slots);
    p->wait_h[1] = c;                                   c += wait_flag_words(L.dir[1].slots);
    p->post_h[0] = c;                                   c += (size_t)L.dir[0].slots * kFlagStride;
    p->post_h[1] = c;                                   c += (size_t)L.dir[1].slots * kFlagStride;
    p->abort_h = (uint32_t *)c;                         c += kFlagStride;
    p->status_h = (uint32_t *)c;                        c += kFlagStride;
    if ((size_t)(c - p->ctrl_h) * 8 != p->ctrl_bytes) return NIXIE_EINVAL;
    (void)n_slots;

    // descriptors
    uint64_t n_arrive = 0;
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
        n_arrive += D.chunks.size();

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
    // [8] exited out, [9] exited in, [10] gathered prefix, [11..15] pad, then per direction: seen[] (u64 per slot),
    // chunk_slot[] and arrive[] (u32 per chunk).  All of it is cleared before every launch.
    uint64_t off = 16;
    for (int x = 0; x < 2; x++) { p->seen_off[x] = off; off += 2 * wait_flag_words(L.dir[x].slots); }
    for (int x = 0; x < 2; x++) { p->cslot_off[x] = off; off += L.dir[x].chunks.size(); }
    for (int x = 0; x < 2; x++) { p->arrive_off[x] = off; off += L.dir[x].chunks.size(); }
    p->n_counters = off;
    (void)n_arrive;
    {
        hipError_t e = hipMalloc((void **)&p->counters_d, p->n_counters * sizeof(uint32_t));
        if (e != hipSuccess) { t_last_hip_error = (int)e; return NIXIE_ENOMEM; }
    }
    const size_t n_hash = std::max<size_t>(1, std::max(L.table[0].size(), L.table[1].size()));
    {
        hipError_t e = hipMalloc((void **)&p->hashes_d, n_hash * sizeof(uint64_t));
        if (e != hipSuccess) { t_last_hip_error = (int)e; return NIXIE_ENOMEM; }
    }
    NIXIE_HIP(hipEventCreate(&p->ev0));
    NIXIE_HIP(hipEventCreate(&p->ev1));

    for (uint32_t t = 0; t < p->info.drain_threads; t++) p->threads.emplace_back(worker_main, p, 0, t);
    for (uint32_t t = 0; t < p->info.fill_threads; t++) p->threads.emplace_back(worker_main, p, 1, t);
    return NIXIE_OK;
}

// One pass: the directions in mask run together.
int run_pass(nixie_plan_t *p, uint32_t mask, hipStream_t stream, nixie_stats_t *st, uint64_t t_entry) {
    const Layout &L = p->L;
    std::memset(p->ctrl_h, 0, p->ctrl_bytes);
    p->abort_local.store(0);
    for (int x = 0; x < 2; x++) {
        p->next_chunk[x].store(0);
        p->done_chunks[x].store(0);
        p->wait_ns[x].store(0);
    }
    for (uint32_t sl = 0; sl < L.dir[0].slots; sl++) p->wait_h[0][sl] = 1;   // every outgoing slot starts released
    std::atomic_thread_fence(std::memory_order_seq_cst);

    SwapArgs a{};
    for (int x = 0; x < 2; x++) {
        const DirLayout &D = L.dir[x];
        DevDir &d = a.d[x];
        const bool on = (mask & (1u << x)) && !D.chunks.empty();
        d.segs = p->segs_d[x];
        d.chunks = p->chunks_d[x];
        d.ring = p->ring_d + (x ? (uint64_t)L.dir[0].slots * L.slot_bytes : 0);
        const size_t wait_off = (size_t)(p->wait_h[x] - p->ctrl_h), post_off = (size_t)(p->post_h[x] - p->ctrl_h);
        d.host_flags = p->ctrl_d + wait_off;
        d.post_flags = p->ctrl_d + post_off;
        d.ticket = p->counters_d + x;
        d.exited = p->counters_d + 8 + x;
        d.seen = (uint64_t *)(p->counters_d + p->seen_off[x]);
        d.chunk_slot = p->counters_d + p->cslot_off[x];
        d.arrive = p->counters_d + p->arrive_off[x];
        d.stall_ticks = (uint64_t *)(p->counters_d + 4 + 2 * x);
        d.n_chunks = on ? (uint32_t)D.chunks.size() : 0;
        d.n_slots = D.slots ? D.slots : 1;
        d.team = x ? p->info.team_in : p->info.team_out;
        if (d.team == 0) d.team = 1;
        d.wgs = on ? (x ? p->info.scatter_wgs : p->info.gather_wgs) : 0;
    }
    a.slot_bytes = L.slot_bytes;
    a.host_abort = (const uint32_t *)(p->ctrl_d + (size_t)((uint64_t *)p->abort_h - p->ctrl_h));
    a.gpu_status = (uint32_t *)(p->ctrl_d + (size_t)((uint64_t *)p->status_h - p->ctrl_h));
    a.dev_abort = p->counters_d + 2;
    a.timeout_ticks = p->timeout_ns / 10;   // wall clock runs at 100 MHz
    a.gathered_prefix = p->counters_d + 10;
    // when the directions run one after the other, everything has left HBM before the restore starts
    a.track_prefix = ((L.opts.flags & NIXIE_IN_PLACE) && a.d[0].wgs && a.d[1].wgs) ? 1u : 0u;

    int e = nixie_launch_zero32(p->counters_d, p->n_counters, stream);
    if (e) { t_last_hip_error = e; return NIXIE_EHIP; }
    NIXIE_HIP(hipEventRecord(p->ev0, stream));
    e = nixie_launch_swap(a, stream);
    if (e) { t_last_hip_error = e; return NIXIE_EHIP; }
    NIXIE_HIP(hipEventRecord(p->ev1, stream));
    if (st && st->ns_launch == 0) st->ns_launch = now_ns() - t_entry;

    {
        std::lock_guard<std::mutex> lk(p->mu);
        p->pass_mask = mask;
        p->running = (uint32_t)p->threads.size();
        p->epoch++;
    }
    p->cv_go.notify_all();
    {
        std::unique_lock<std::mutex> lk(p->mu);
        p->cv_done.wait(lk, [&] { return p->running == 0; });
    }
    hipError_t se = hipStreamSynchronize(stream);
    if (se != hipSuccess) { t_last_hip_error = (int)se; return NIXIE_EHIP; }

    if (st) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, p->ev0, p->ev1) == hipSuccess) st->ns_kernel += (uint64_t)((double)ms * 1e6);
        uint64_t stall[2] = {0, 0};
        NIXIE_HIP(hipMemcpy(stall, p->counters_d + 4, sizeof(stall), hipMemcpyDeviceToHost));
        st->gather_stall_ticks += stall[0];
        st->scatter_stall_ticks += stall[1];
        st->drain_wait_ns += p->wait_ns[0].load();
        st->fill_wait_ns += p->wait_ns[1].load();
        st->kernels++;
        const uint32_t gs = __atomic_load_n(p->status_h, __ATOMIC_ACQUIRE);
        if (gs) st->gpu_status = gs;
    }
    int err = p->error.load();
    if (!err && __atomic_load_n(p->status_h, __ATOMIC_ACQUIRE) != kGpuOk) err = NIXIE_ETIMEOUT;
    return err;
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

int nixie_plan_info(const nixie_plan_t *plan, nixie_plan_info_t *info) {
    if (!plan || !info) return NIXIE_EINVAL;
    *info = plan->info;
    return NIXIE_OK;
}

void nixie_plan_destroy(nixie_plan_t *plan) { destroy_plan(plan); }

int nixie_switch(nixie_plan_t *p, void *hip_stream, nixie_stats_t *stats) {
    if (!p) return NIXIE_EINVAL;
    std::unique_lock<std::mutex> lk(p->switch_mu, std::try_to_lock);
    if (!lk.owns_lock()) return NIXIE_EBUSY;
    const uint64_t t_entry = now_ns();
    int dev = -1;
    NIXIE_HIP(hipGetDevice(&dev));
    if (dev != p->device) return NIXIE_EINVAL;
    nixie_stats_t st{};
    st.bytes_out = p->L.dir[0].bytes;
    st.bytes_in = p->L.dir[1].bytes;
    p->timeout_ns = (uint64_t)(p->L.opts.timeout_ms ? p->L.opts.timeout_ms : 30000u) * 1000000ull;
    p->error.store(0);
    p->end_ns[0].store(0);
    p->end_ns[1].store(0);

    int rc = NIXIE_OK;
    const bool both = !p->L.dir[0].chunks.empty() && !p->L.dir[1].chunks.empty();
    if ((p->L.opts.flags & NIXIE_SERIALIZE) && both) {
        rc = run_pass(p, 1u, (hipStream_t)hip_stream, &st, t_entry);
        if (!rc) rc = run_pass(p, 2u, (hipStream_t)hip_stream, &st, t_entry);
    } else {
        rc = run_pass(p, 3u, (hipStream_t)hip_stream, &st, t_entry);
    }
    const uint64_t t_end = now_ns();
    st.ns_total = t_end - t_entry;
    st.ns_out_done = p->end_ns[0].load() > t_entry ? p->end_ns[0].load() - t_entry : 0;
    st.ns_in_done = p->end_ns[1].load() > t_entry ? p->end_ns[1].load() - t_entry : 0;
    if (stats) *stats = st;
    return rc;
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
    case NIXIE_EBUSY: return "plan is busy";
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
