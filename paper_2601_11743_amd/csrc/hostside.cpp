// Host half of the slot protocol: drain and fill threads, their watchdog, and the crew that
// parks them between switches.
//
// Paper, "Speeding Up Context Switches": the pinned tier is run as a stream with back-pressure
// -- a slot is refilled as soon as the stage below has emptied it -- and the pageable<->pinned
// leg is copied by several threads.  Each thread owns a fixed subset of the slots and serves
// whichever of them has work, so a slot that is slow to come back delays nothing else.
#include "hostside.hpp"

#include <immintrin.h>
#include <sched.h>
#include <sys/prctl.h>
#include <time.h>

#include <cstring>

namespace nixie {

namespace {

inline uint64_t now_ns() {
    timespec ts;
    clock_gettime(CLOCK_MONOTONIC, &ts);
    return (uint64_t)ts.tv_sec * 1000000000ull + (uint64_t)ts.tv_nsec;
}
inline uint64_t load_acq(const uint64_t *p) { return __atomic_load_n(p, __ATOMIC_ACQUIRE); }
inline void store_rel(uint64_t *p, uint64_t v) { __atomic_store_n(p, v, __ATOMIC_RELEASE); }

}  // namespace

void HostSide::begin_pass() {
    abort_local.store(0);
    for (int x = 0; x < 2; x++) {
        next_chunk[x].store(0);
        done_chunks[x].store(0);
        wait_ns[x].store(0);
    }
    for (uint32_t s = 0; s < L->dir[0].slots; s++) wait[0][s] = 1;   // every outgoing slot starts released
    std::atomic_thread_fence(std::memory_order_seq_cst);
}

void HostSide::raise_abort(int err) {
    int expected = 0;
    error.compare_exchange_strong(expected, err);
    abort_local.store(1, std::memory_order_release);
    __atomic_store_n(abort_word, 1u, __ATOMIC_RELEASE);   // the kernel's pump polls this word
}

namespace {

// Idle bookkeeping of a host thread that scans its slots: aborts the switch when nothing has
// moved for longer than the bound, or when the kernel reported that it gave up.
struct IdleWatch {
    HostSide *p;
    int dir;
    uint64_t idle_since = 0;
    uint32_t spins = 0;
    bool force_yield = false;   // for a waiter that is not one of the crew's threads
    uint64_t nap_ns = ~0ull;    // ~0: the plan's setting
    bool account = true;        // idle time counts towards the direction's wait_ns
    bool started = false;       // the kernel has been seen running
    // call after a scan that made no progress; false = stop
    bool idle() {
        // Spin: a slot usually turns around in microseconds.  Only where the threads outnumber
        // the cores does a long-idle thread give its core away between looks, so that a waiting
        // thread cannot keep the one it waits for off the processor; with a core each, yielding
        // costs a small ring one to two percent and buys nothing.
        const uint64_t nap_for = nap_ns != ~0ull ? nap_ns : (force_yield ? 0 : p->idle_sleep_ns);
        if (nap_for && spins >= 64) {
            // Nothing for a few microseconds: the ring holds far more than a nap's worth of
            // transfer, so give the core to whoever needs it (the applications do).
            timespec nap{0, (long)nap_for};
            nanosleep(&nap, nullptr);
        } else if ((p->yield_when_idle || force_yield) && spins >= 4096) sched_yield();
        else _mm_pause();
        if (idle_since == 0) idle_since = now_ns();
        if ((++spins & 63u) != 0) return true;
        if (p->abort_local.load(std::memory_order_acquire)) return false;
        // The bound is on a credit wait.  While the kernel has not been seen running (it may be queued
        // behind the caller's earlier work on the stream) the thread waits longer, and the clock of
        // the credit wait starts when the kernel does.
        if (!started && __atomic_load_n(p->done_word + kStartedWord, __ATOMIC_ACQUIRE)) {
            started = true;
            idle_since = now_ns();
        }
        const uint64_t bound = started ? p->timeout_ns : kStartGrace * p->timeout_ns;
        if (__atomic_load_n(p->status_word, __ATOMIC_ACQUIRE) != kGpuOk || now_ns() - idle_since > bound) {
            p->raise_abort(NIXIE_ETIMEOUT);
            return false;
        }
        return true;
    }
    void progressed() {
        if (idle_since && account) p->wait_ns[dir].fetch_add(now_ns() - idle_since, std::memory_order_relaxed);
        idle_since = 0;
        spins = 0;
    }
};

void note_end(HostSide *p, int dir) {
    uint64_t t = now_ns(), cur = p->end_ns[dir].load(std::memory_order_relaxed);
    while (cur < t && !p->end_ns[dir].compare_exchange_weak(cur, t, std::memory_order_relaxed)) {}
}

}  // namespace

// ring -> pageable.  Consumer of the outgoing direction.  Thread idx owns slots idx, idx + T, ...
// and drains whichever of them the GPU has marked ready (ready[s] = chunk id + 1), in any order.
void HostSide::run_drain(uint32_t idx) {
    HostSide *p = this;
    const uint32_t T = threads[0];
    const DirLayout &D = L->dir[0];
    const uint32_t flags = L->opts.flags;
    const uint64_t n = D.staged, S = L->slot_bytes;   // direct chunks never come through the ring
    const bool plain = flags & NIXIE_HOST_PLAIN_MEMCPY;
    std::vector<uint64_t> last(D.slots, 0);
    IdleWatch watch{p, 0};
    while (p->done_chunks[0].load(std::memory_order_acquire) < n) {
        bool moved = false;
        for (uint64_t slot = idx; slot < D.slots; slot += T) {
            const uint64_t v = load_acq(p->post[0] + slot * kFlagStride);
            if (v == last[slot]) continue;
            last[slot] = v;
            const uint64_t k = v - 1;
            if (k >= n) { p->raise_abort(NIXIE_EINVAL); return; }
            if (!(flags & NIXIE_DIAG_RING_ONLY)) {
                const nixie_chunk_t &c = D.chunks[k];
                const uint8_t *src = p->ring + slot * S;
                for (uint64_t q = c.seg_begin; q < c.seg_begin + c.seg_count; q++) {
                    const nixie_segment_t &sg = D.segs[q];
                    if (plain) std::memcpy((void *)(uintptr_t)sg.host_addr, src + sg.slot_off, sg.len);
                    else copy_stream((void *)(uintptr_t)sg.host_addr, src + sg.slot_off, sg.len);
                }
                _mm_sfence();
            }
            if (!(flags & NIXIE_DIAG_STALL_DRAIN)) store_rel(p->wait[0] + slot, k + 2);   // released
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
void HostSide::run_fill(uint32_t idx) {
    HostSide *p = this;
    const uint32_t T = threads[1];
    const DirLayout &D = L->dir[1];
    const uint32_t flags = L->opts.flags;
    const uint64_t n = D.staged, S = L->slot_bytes;   // direct chunks never come through the ring
    const bool plain = flags & NIXIE_HOST_PLAIN_MEMCPY;
    std::vector<uint64_t> pending(D.slots, 0);
    uint64_t outstanding = 0;
    bool claiming = true;
    IdleWatch watch{p, 1};
    for (;;) {
        bool moved = false;
        for (uint64_t slot = idx; slot < D.slots; slot += T) {
            if (pending[slot]) {
                if (load_acq(p->post[1] + slot * kFlagStride) != pending[slot]) continue;
                pending[slot] = 0;
                outstanding--;
                moved = true;
            }
            if (!claiming) continue;
            const uint64_t k = p->next_chunk[1].fetch_add(1, std::memory_order_relaxed);
            if (k >= n) { claiming = false; continue; }
            if (!(flags & NIXIE_DIAG_RING_ONLY)) {
                const nixie_chunk_t &c = D.chunks[k];
                uint8_t *dst = p->ring + ((uint64_t)p->L->dir[0].slots + slot) * S;
                for (uint64_t q = c.seg_begin; q < c.seg_begin + c.seg_count; q++) {
                    const nixie_segment_t &sg = D.segs[q];
                    if (plain) std::memcpy(dst + sg.slot_off, (const void *)(uintptr_t)sg.host_addr, sg.len);
                    else copy_stream(dst + sg.slot_off, (const void *)(uintptr_t)sg.host_addr, sg.len);
                }
                _mm_sfence();
            }
            store_rel(p->wait[1] + slot, k + 1);   // filled
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

int HostSide::wait_direction(int x, uint64_t nap_ns) {
    IdleWatch watch{this, x};
    watch.force_yield = true;
    watch.nap_ns = nap_ns;
    watch.account = false;
    int rc = NIXIE_OK;
    // The bound is on the time without any sign of progress, not on the length of the direction:
    // chunks claimed or delivered by the host threads, or work units handed out on the GPU.
    uint64_t seen = 0;
    while (__atomic_load_n(done_word + x, __ATOMIC_ACQUIRE) == 0) {
        const uint64_t sign = done_chunks[x].load(std::memory_order_relaxed) + next_chunk[x].load(std::memory_order_relaxed) +
                              __atomic_load_n(done_word + kProgressWord + x, __ATOMIC_RELAXED);
        if (sign != seen) {
            seen = sign;
            watch.progressed();
        } else if (!watch.idle()) break;
    }
    if (__atomic_load_n(done_word + x, __ATOMIC_ACQUIRE) == 0 || error.load() ||
        __atomic_load_n(status_word, __ATOMIC_ACQUIRE) != kGpuOk)
        rc = error.load() ? error.load() : NIXIE_ETIMEOUT;
    return rc;
}

void HostCrew::worker(int dir, uint32_t idx) {
    prctl(PR_SET_TIMERSLACK, 1000UL, 0UL, 0UL, 0UL);   // naps of tens of microseconds, not the default 50 us slack on top
    uint64_t seen = 0;
    for (;;) {
        uint32_t mask;
        {
            std::unique_lock<std::mutex> lk(mu_);
            cv_go_.wait(lk, [&] { return quit_ || epoch_ != seen; });
            if (quit_) return;
            seen = epoch_;
            mask = mask_;
        }
        if (mask & (1u << dir)) {
            if (dir == 0) hs_->run_drain(idx);
            else hs_->run_fill(idx);
        }
        {
            std::lock_guard<std::mutex> lk(mu_);
            if (--running_ == 0) cv_done_.notify_all();
        }
    }
}

void HostCrew::start(HostSide *hs) {
    hs_ = hs;
    for (uint32_t t = 0; t < hs->threads[0]; t++) threads_.emplace_back(&HostCrew::worker, this, 0, t);
    for (uint32_t t = 0; t < hs->threads[1]; t++) threads_.emplace_back(&HostCrew::worker, this, 1, t);
}

void HostCrew::wake(uint32_t mask) {
    {
        std::lock_guard<std::mutex> lk(mu_);
        mask_ = mask;
        running_ = (uint32_t)threads_.size();
        epoch_++;
    }
    cv_go_.notify_all();
}

void HostCrew::wait() {
    std::unique_lock<std::mutex> lk(mu_);
    cv_done_.wait(lk, [&] { return running_ == 0; });
}

void HostCrew::stop() {
    {
        std::lock_guard<std::mutex> lk(mu_);
        quit_ = true;
    }
    cv_go_.notify_all();
    for (auto &t : threads_) t.join();
    threads_.clear();
}

}  // namespace nixie
