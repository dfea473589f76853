// Host half of the slot protocol: what the drain / fill threads see and do.  No HIP types here,
// so this half can be built and run (and raced under a thread sanitizer) without a GPU.
#pragma once
#include <atomic>
#include <condition_variable>
#include <cstdint>
#include <mutex>
#include <thread>
#include <vector>

#include "internal.hpp"

namespace nixie {

struct HostSide {
    const Layout *L = nullptr;
    uint8_t *ring = nullptr;                          // host view of the pinned ring, outgoing sub-ring first
    uint64_t *wait[2] = {nullptr, nullptr};           // host-written, packed: out released[s], in filled[s]
    const uint64_t *post[2] = {nullptr, nullptr};     // GPU-written, kFlagStride apart: out ready[s], in freed[s]
    uint32_t *abort_word = nullptr;                   // host-written, the kernel's pump relays it
    const uint32_t *status_word = nullptr;            // GPU-written: kGpuOk or why the kernel gave up
    const uint32_t *done_word = nullptr;              // GPU-written: [x] = 1 once direction x has left the GPU
    uint64_t timeout_ns = 0;
    uint32_t threads[2] = {0, 0};                     // drain, fill
    bool yield_when_idle = false;                     // set when the threads outnumber the usable cores
    uint64_t idle_sleep_ns = 0;                       // > 0: a thread with nothing to do sleeps this long between looks

    std::atomic<uint64_t> next_chunk[2];              // incoming: next chunk to claim
    std::atomic<uint64_t> done_chunks[2];             // outgoing: chunks that reached pageable memory
    std::atomic<uint64_t> wait_ns[2];                 // summed idle time per direction
    std::atomic<uint64_t> end_ns[2];                  // latest completion time seen per direction
    std::atomic<int> error{0};
    std::atomic<uint32_t> abort_local{0};

    void begin_pass();                                // flags must already be cleared
    void raise_abort(int err);
    void run_drain(uint32_t idx);                     // ring -> pageable, thread idx of threads[0]
    void run_fill(uint32_t idx);                      // pageable -> ring, thread idx of threads[1]
    // Blocks until the kernel reports that every workgroup of direction x has left (for x = 1:
    // every incoming byte is in HBM), or the switch fails.  NIXIE_OK or the switch's error.
    // nap_ns > 0: sleep that long between looks instead of spinning.
    int wait_direction(int x, uint64_t nap_ns = 0);
};

// The parked threads.  wake() starts them on the directions in mask; wait() returns when all of
// them are done (finished, aborted or timed out).  run_pass() is the two in a row.
class HostCrew {
public:
    void start(HostSide *hs);
    void wake(uint32_t mask);
    void wait();
    void run_pass(uint32_t mask) { wake(mask); wait(); }
    void stop();
    ~HostCrew() { stop(); }

private:
    void worker(int dir, uint32_t idx);
    HostSide *hs_ = nullptr;
    std::vector<std::thread> threads_;
    std::mutex mu_;
    std::condition_variable cv_go_, cv_done_;
    uint64_t epoch_ = 0;
    uint32_t running_ = 0, mask_ = 0;
    bool quit_ = false;
};

}  // namespace nixie
