// CPU stand-in for the device half of the slot protocol, for tests only.
//
// Builds the library's planner, streaming copies and host half (drain / fill threads, watchdog,
// crew) for the CPU, and drives them against a model of what the swap kernel does: one pump
// thread per direction that turns host-written flags into chunk -> slot assignments, and worker
// threads that take tickets, wait for their chunk's slot, copy, meet on the arrive counter and
// publish the GPU-written flag.  "Device memory" is ordinary memory.  Meant to run under a
// thread sanitizer: every hand-over that the real hardware orders physically is an
// acquire/release pair here, so a missing hand-over in the host half shows up as a data race.
//
// usage: fake_gpu <scenario> [seed]
//   swap        bidirectional switch, mixed sizes, small ring; result must equal memcpy
//   in_place    incoming ranges reuse the outgoing "device" memory; evict-before-overwrite
//   spaces      the same, but the two applications see that memory at different addresses (one
//               file mapped twice, registered as two spaces of one pool): the planner must find
//               the dependencies through the pool coordinate
//   tier        A's host side and half of B's lie in a registered pinned tier: those allocations move
//               directly, without slots or host threads, next to staged ones in the same switch
//   tier_in_place  the same with B reusing A's "device" memory
//   stall       the host withholds credits (NIXIE_DIAG_STALL_DRAIN): must end with NIXIE_ETIMEOUT
//   gpu_quits   the device reports that it gave up: the host must stop with NIXIE_ETIMEOUT
//   dead_gpu    the device never starts: the host watchdog must fire
#include <atomic>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <thread>
#include <vector>

#include <sys/mman.h>
#include <unistd.h>

#include "hostside.hpp"
#include "spaces.hpp"

using namespace nixie;

namespace {

uint64_t rng_state = 1;
uint64_t rnd() {
    rng_state += 0x9E3779B97F4A7C15ull;
    uint64_t z = rng_state;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

struct FakeGpu {
    const Layout *L;
    uint8_t *ring;
    const uint64_t *host_flags[2];   // host-written (packed)
    uint64_t *post[2];               // "GPU"-written (kFlagStride apart)
    const uint32_t *host_abort;
    uint32_t *status;
    uint32_t *done = nullptr;        // [dir] = 1 once every worker of the direction has left
    uint32_t team[2], wgs[2];
    bool in_place = false;
    bool never_start = false, quit_early = false;

    std::vector<std::atomic<uint32_t>> chunk_slot[2], arrive[2];
    std::atomic<uint32_t> ticket[2], exited[2], dev_abort{0}, gathered_prefix{0};
    std::vector<std::thread> threads;

    void copy_unit(int dir, uint32_t k, uint32_t part, uint32_t slot) {
        const DirLayout &D = L->dir[dir];
        const nixie_chunk_t &c = D.chunks[k];
        uint8_t *base = k >= D.staged ? (uint8_t *)(uintptr_t)D.direct_base[k - D.staged]      // pinned tier: no slot
                                      : ring + ((dir ? L->dir[0].slots : 0) + (uint64_t)slot) * L->slot_bytes;
        const uint32_t n_tiles = (c.used_bytes + kTileBytes - 1) / kTileBytes;
        for (uint32_t t = part; t < n_tiles; t += team[dir]) {
            const uint32_t t0 = t * kTileBytes, t1 = std::min(t0 + kTileBytes, c.used_bytes);
            for (uint64_t q = c.seg_begin; q < c.seg_begin + c.seg_count; q++) {
                const nixie_segment_t &s = D.segs[q];
                const uint32_t x0 = std::max(s.slot_off, t0), x1 = std::min(s.slot_off + s.len, t1);
                if (x0 >= x1) continue;
                uint8_t *dev = (uint8_t *)(uintptr_t)(s.dev_addr + (x0 - s.slot_off));
                if (dir == 0) std::memcpy(base + x0, dev, x1 - x0);
                else std::memcpy(dev, base + x0, x1 - x0);
            }
        }
    }

    void worker(int dir) {
        const DirLayout &D = L->dir[dir];
        const uint32_t total = (uint32_t)D.chunks.size() * team[dir];
        for (;;) {
            const uint32_t u = ticket[dir].fetch_add(1, std::memory_order_relaxed);
            if (u >= total || dev_abort.load(std::memory_order_acquire)) break;
            const uint32_t k = u / team[dir], part = u % team[dir];
            const bool direct = k >= D.staged;
            uint32_t cs = direct ? 0xFFFFFFFFu : 0;
            while (!direct && (cs = chunk_slot[dir][k].load(std::memory_order_acquire)) == 0) {
                if (dev_abort.load(std::memory_order_acquire)) break;
                std::this_thread::yield();
            }
            if (cs == 0) break;
            if (dir == 1 && in_place) {
                bool stop = false;
                while (gathered_prefix.load(std::memory_order_acquire) < D.chunks[k].dep_out) {
                    if (dev_abort.load(std::memory_order_acquire)) { stop = true; break; }
                    std::this_thread::yield();
                }
                if (stop) break;
            }
            copy_unit(dir, k, part, cs - 1);
            const uint32_t old = arrive[dir][k].fetch_add(1, std::memory_order_acq_rel);
            if (old == team[dir] - 1 && !direct)
                __atomic_store_n(post[dir] + (size_t)(cs - 1) * kFlagStride, (uint64_t)k + 1, __ATOMIC_RELEASE);
        }
        exited[dir].fetch_add(1, std::memory_order_release);
    }

    void pump(int dir) {
        const DirLayout &D = L->dir[dir];
        if (wgs[dir] == 0) return;
        std::vector<uint64_t> seen(D.slots, 0);
        uint32_t next = 0, prefix = 0;
        for (;;) {
            for (uint32_t s = 0; s < D.slots; s++) {
                const uint64_t v = __atomic_load_n(host_flags[dir] + s, __ATOMIC_ACQUIRE);
                if (v == seen[s]) continue;
                seen[s] = v;
                const uint64_t k = dir == 0 ? next++ : v - 1;
                if (k < D.staged) chunk_slot[dir][k].store(s + 1, std::memory_order_release);
            }
            if (dir == 0 && in_place) {
                while (prefix < D.chunks.size() && arrive[0][prefix].load(std::memory_order_acquire) >= team[0]) prefix++;
                gathered_prefix.store(prefix, std::memory_order_release);
            }
            if (__atomic_load_n(host_abort, __ATOMIC_ACQUIRE) && !dev_abort.load()) {
                dev_abort.store(1, std::memory_order_release);
                __atomic_store_n(status, (uint32_t)kGpuSawAbort, __ATOMIC_RELEASE);
            }
            __atomic_store_n(done + kProgressWord + dir, ticket[dir].load(std::memory_order_relaxed), __ATOMIC_RELAXED);
            if (exited[dir].load(std::memory_order_acquire) >= wgs[dir]) {
                __atomic_store_n(done + dir, 1u, __ATOMIC_RELEASE);
                break;
            }
            std::this_thread::yield();
        }
    }

    void launch() {
        for (int x = 0; x < 2; x++) {
            const size_t n = L->dir[x].chunks.size();
            chunk_slot[x] = std::vector<std::atomic<uint32_t>>(n);
            arrive[x] = std::vector<std::atomic<uint32_t>>(n);
            for (size_t i = 0; i < n; i++) { chunk_slot[x][i].store(0); arrive[x][i].store(0); }
            ticket[x].store(0);
            exited[x].store(0);
            if (n == 0) wgs[x] = 0;
        }
        if (never_start) return;
        __atomic_store_n(done + kStartedWord, 1u, __ATOMIC_RELEASE);
        if (quit_early) {   // the kernel hit its own wait bound
            __atomic_store_n(status, (uint32_t)kGpuTimeout, __ATOMIC_RELEASE);
            return;
        }
        for (int x = 0; x < 2; x++) {
            if (wgs[x]) threads.emplace_back(&FakeGpu::pump, this, x);
            for (uint32_t w = 0; w < wgs[x]; w++) threads.emplace_back(&FakeGpu::worker, this, x);
        }
    }
    void join() { for (auto &t : threads) t.join(); threads.clear(); }
};

struct Arena {
    std::vector<uint8_t> host;
    std::vector<nixie_alloc_t> rows;
};

uint64_t arena_bytes(const std::vector<uint64_t> &sizes) {
    uint64_t total = 256;
    for (uint64_t b : sizes) total += b + 64;
    return total;
}

// Allocations of the given sizes inside the "device" arena dev, 64 B gaps, bases skewed by `skew`
// bytes; the resident side gets content f(seed, byte index, size).
void build(Arena &a, const std::vector<uint64_t> &sizes, uint64_t seed, bool resident_dev, uint8_t *dev, uint64_t skew) {
    a.host.assign(arena_bytes(sizes), 0xC3);
    uint64_t off = 64 + skew;
    for (uint64_t b : sizes) {
        a.rows.push_back(nixie_alloc_t{dev + off, a.host.data() + off, b});
        uint8_t *src = resident_dev ? dev + off : a.host.data() + off;
        for (uint64_t i = 0; i < b; i++) src[i] = (uint8_t)((seed * 131 + i * 7 + (i >> 8) + b) & 0xFF);
        off += b + 64;
    }
}

int run(const std::string &scenario, uint64_t seed) {
    rng_state = seed * 7919 + 1;
    const uint64_t S = 64 << 10;
    std::vector<uint64_t> sa, sb;
    for (int i = 0; i < 14; i++) sa.push_back(1 + rnd() % (3 * S));
    for (int i = 0; i < 11; i++) sb.push_back(1 + rnd() % (4 * S));
    sa.push_back(0); sa.push_back(S); sa.push_back(5 * S + 1);
    sb.push_back(S - 1); sb.push_back(15);
    const bool spaces = scenario == "spaces";
    const bool tier = scenario == "tier" || scenario == "tier_in_place";
    const bool in_place = scenario == "in_place" || spaces || scenario == "tier_in_place";

    // in place: B's device ranges lie in the same "device" arena as A's
    std::vector<uint8_t> dev_a(std::max(arena_bytes(sa), in_place ? arena_bytes(sb) : 0) + 64, 0xC3);
    std::vector<uint8_t> dev_b(in_place ? 0 : arena_bytes(sb) + 64, 0xC3);
    uint8_t *base_a = dev_a.data(), *base_b = in_place ? dev_a.data() : dev_b.data();
    uint64_t span_bytes = 0;
    if (spaces) {   // one "pool" seen through two address ranges
        const uint64_t blk = 64 << 10;
        span_bytes = (dev_a.size() + blk - 1) / blk * blk;
        const int fd = memfd_create("fake_pool", 0);
        if (fd < 0 || ftruncate(fd, (off_t)span_bytes) != 0) { std::printf("memfd failed\n"); return 2; }
        base_a = (uint8_t *)mmap(nullptr, span_bytes, PROT_READ | PROT_WRITE, MAP_SHARED, fd, 0);
        base_b = (uint8_t *)mmap(nullptr, span_bytes, PROT_READ | PROT_WRITE, MAP_SHARED, fd, 0);
        if (base_a == MAP_FAILED || base_b == MAP_FAILED || base_a == base_b) { std::printf("mmap failed\n"); return 2; }
        std::memset(base_a, 0xC3, span_bytes);
        // B sees the pool's blocks in another order (odd seeds): block i of B's range is pool block perm[i]
        const uint64_t nblk = span_bytes / blk;
        std::vector<uint64_t> perm(nblk);
        for (uint64_t i = 0; i < nblk; i++) perm[i] = seed % 2 ? (i * 5 + 3) % nblk : i;
        if (seed % 2 && nblk % 5 == 0) for (uint64_t i = 0; i < nblk; i++) perm[i] = nblk - 1 - i;   // keep it a permutation
        for (uint64_t i = 0; i < nblk; i++)
            if (mmap(base_b + i * blk, blk, PROT_READ | PROT_WRITE, MAP_SHARED | MAP_FIXED, fd, (off_t)(perm[i] * blk)) == MAP_FAILED) {
                std::printf("mmap of block %llu failed\n", (unsigned long long)i);
                return 2;
            }
        close(fd);
        const uint64_t key = next_pool_key();
        for (uint8_t *b : {base_a, base_b}) {
            SpaceSpan sp;
            sp.base = (uint64_t)(uintptr_t)b; sp.bytes = span_bytes; sp.key_base = key; sp.block_bytes = blk;
            sp.mapped.assign(nblk, 1);
            sp.assigned.resize(nblk);
            for (uint64_t i = 0; i < nblk; i++) sp.assigned[i] = b == base_b ? perm[i] : i;
            space_register(sp);
        }
        // a mapped block keeps its pool block; naming the one it has is fine
        const uint64_t other = (perm[0] + 1) % nblk;
        if (space_assign((uint64_t)(uintptr_t)base_b, 0, &other, 1) || !space_assign((uint64_t)(uintptr_t)base_b, 0, &perm[0], 1)) {
            std::printf("space_assign on a mapped block\n");
            return 1;
        }
    }
    Arena A, B;
    build(A, sa, seed, true, base_a, seed % 16);
    build(B, sb, seed + 1, false, base_b, (seed * 5) % 16);
    // expectation by plain memcpy, in definition order: all of A out, then B in
    std::vector<std::vector<uint8_t>> want_a, want_b;
    for (auto &r : A.rows) want_a.emplace_back((uint8_t *)r.dev_ptr, (uint8_t *)r.dev_ptr + r.bytes);
    for (auto &r : B.rows) want_b.emplace_back((uint8_t *)r.host_ptr, (uint8_t *)r.host_ptr + r.bytes);

    if (tier) {   // on the CPU the "GPU's address" of pinned memory is the address itself
        const uint64_t ha = (uint64_t)(uintptr_t)A.host.data(), hb = (uint64_t)(uintptr_t)B.host.data();
        if (!tier_register(TierSpan{ha, A.host.size(), ha}) || !tier_register(TierSpan{hb, B.host.size() / 2, hb}) ||
            tier_register(TierSpan{hb + 100, 50, hb + 100})) { std::printf("tier registration\n"); return 1; }
    }
    nixie_opts_t o{};
    o.slot_bytes = S;
    o.drain_threads = 3;
    o.fill_threads = 2;
    const bool must_succeed = scenario == "swap" || in_place || tier;
    o.timeout_ms = must_succeed ? 20000 : 300;
    if (in_place) o.flags |= NIXIE_IN_PLACE;
    if (scenario == "stall") o.flags |= NIXIE_DIAG_STALL_DRAIN;
    nixie_table_t ta{A.rows.data(), A.rows.size()}, tb{B.rows.data(), B.rows.size()};
    Layout L;
    const uint64_t ring_bytes = 12 * S;
    if (spaces) {
        // the two address ranges share their bytes, and the planner must know it
        nixie_opts_t plain = o;
        plain.flags &= ~(uint32_t)NIXIE_IN_PLACE;
        int e = build_layout(&ta, &tb, ring_bytes, &plain, L);
        if (e != NIXIE_EOVERLAP) { std::printf("expected NIXIE_EOVERLAP without NIXIE_IN_PLACE, got %d\n", e); return 1; }
        // a range that runs over the end of a space belongs to no one
        std::vector<uint8_t> h(256);
        nixie_alloc_t over{base_b + span_bytes - 100, h.data(), 200};
        nixie_table_t tover{&over, 1};
        e = build_layout(nullptr, &tover, ring_bytes, &o, L);
        if (e != NIXIE_EINVAL) { std::printf("expected NIXIE_EINVAL for a range across the edge of a space, got %d\n", e); return 1; }
        if (L.uses[0].size() != 0) { std::printf("stale uses\n"); return 1; }
        // the planner sees the pool through the assignment: a piece of B's range that shares a pool
        // block and offset with A's first allocation overlaps it, one in another block does not
        std::vector<KeyPiece> pa, pb;
        space_translate((uint64_t)(uintptr_t)A.rows[0].dev_ptr, 16, &pa, nullptr);
        const uint64_t blk_sz = 64 << 10, off_a = (uint64_t)((uint8_t *)A.rows[0].dev_ptr - base_a);
        uint64_t where = 0;
        for (uint64_t i = 0; i < span_bytes / blk_sz; i++) {
            std::vector<KeyPiece> t;
            space_translate((uint64_t)(uintptr_t)(base_b + i * blk_sz + off_a % blk_sz), 16, &t, nullptr);
            if (t.size() == 1 && t[0].key == pa[0].key) where++;
        }
        if (pa.size() != 1 || where != 1) { std::printf("translation: %zu pieces, %llu aliases\n", pa.size(), (unsigned long long)where); return 1; }
    }
    int rc = build_layout(&ta, &tb, ring_bytes, &o, L);
    if (rc) { std::printf("build_layout failed %d\n", rc); return 2; }
    if (spaces) {
        if (L.uses[0].empty() || L.uses[1].empty() || !space_uses_valid(L.uses[0]) || !space_uses_valid(L.uses[1])) {
            std::printf("uses: %zu out, %zu in\n", L.uses[0].size(), L.uses[1].size());
            return 1;
        }
        uint64_t deps = 0;
        for (const auto &c : L.dir[1].chunks) deps += c.dep_out != 0;
        if (deps == 0) { std::printf("no dependencies found through the pool coordinate\n"); return 1; }
        space_set_mapped((uint64_t)(uintptr_t)base_a, 0, 1, false);
        if (space_uses_valid(L.uses[0])) { std::printf("unmapped block not noticed\n"); return 1; }
        // ... and a block that comes back with other memory behind it is not the block the plan saw
        const uint64_t one = 1, zero = 0;
        if (!space_assign((uint64_t)(uintptr_t)base_a, 0, &one, 1)) { std::printf("reassignment of an unmapped block refused\n"); return 1; }
        space_set_mapped((uint64_t)(uintptr_t)base_a, 0, 1, true);
        if (space_uses_valid(L.uses[0])) { std::printf("reassigned block not noticed\n"); return 1; }
        space_set_mapped((uint64_t)(uintptr_t)base_a, 0, 1, false);
        space_assign((uint64_t)(uintptr_t)base_a, 0, &zero, 1);
        space_set_mapped((uint64_t)(uintptr_t)base_a, 0, 1, true);
        if (!space_uses_valid(L.uses[0])) { std::printf("restored block not accepted\n"); return 1; }
    }
    nixie_plan_info_t info;
    fill_info(L, &info);
    if (tier) {
        uint64_t direct_b = 0, staged_b = 0;
        for (const auto &r : B.rows) {
            const bool inside = (uint8_t *)r.host_ptr + r.bytes <= B.host.data() + B.host.size() / 2;
            const bool congruent = (((uintptr_t)r.host_ptr ^ (uintptr_t)r.dev_ptr) & 15) == 0;
            (inside && congruent ? direct_b : staged_b) += r.bytes;
        }
        const bool a_congruent = (((uintptr_t)A.rows[0].host_ptr ^ (uintptr_t)A.rows[0].dev_ptr) & 15) == 0;
        if (info.direct_bytes_in != direct_b || info.bytes_in != direct_b + staged_b || direct_b == 0 || staged_b == 0 ||
            (a_congruent && (info.direct_bytes_out != info.bytes_out || L.dir[0].staged != 0 || info.drain_threads != 0 ||
                             L.dir[0].slots != 0))) {
            std::printf("tier split: direct in %llu (want %llu), direct out %llu of %llu, drain threads %u, out slots %u\n",
                        (unsigned long long)info.direct_bytes_in, (unsigned long long)direct_b,
                        (unsigned long long)info.direct_bytes_out, (unsigned long long)info.bytes_out, info.drain_threads,
                        L.dir[0].slots);
            return 1;
        }
        // a plan made from this layout would hold both registrations: no unregistering under it
        const uint64_t ha = (uint64_t)(uintptr_t)A.host.data(), hb = (uint64_t)(uintptr_t)B.host.data();
        if (L.tier_ids.size() != (a_congruent ? 2u : 1u) || !tier_acquire(L.tier_ids) || tier_unregister(hb) != kTierInUse ||
            (a_congruent && tier_unregister(ha) != kTierInUse) || tier_unregister(hb + 8) != kTierUnknown) {
            std::printf("tier lifetime: a registration in use was dropped\n");
            return 1;
        }
        tier_release(L.tier_ids);
        if (tier_unregister(hb) != kTierDropped || tier_acquire(L.tier_ids) ||                 // gone: all or nothing
            !tier_register(TierSpan{hb, B.host.size() / 2, hb}) || tier_acquire(L.tier_ids)) {  // a new registration is a new id
            std::printf("tier lifetime: stale registration acquired\n");
            return 1;
        }
        nixie_opts_t off = o;   // the same tables with the tier ignored: everything is staged
        off.flags |= NIXIE_NO_DIRECT;
        Layout L2;
        if (build_layout(&ta, &tb, ring_bytes, &off, L2) || L2.dir[0].staged != L2.dir[0].chunks.size() || L2.dir[0].direct_bytes) {
            std::printf("NIXIE_NO_DIRECT ignored\n");
            return 1;
        }
    }

    std::vector<uint8_t> ring(info.pinned_ring_bytes + 64);
    std::vector<uint64_t> ctrl(info.pinned_ctrl_bytes / 8 + 8, 0);
    HostSide hs;
    uint64_t *c = ctrl.data();
    hs.wait[0] = c; c += wait_flag_words(L.dir[0].slots);
    hs.wait[1] = c; c += wait_flag_words(L.dir[1].slots);
    uint64_t *post0 = c; c += (size_t)L.dir[0].slots * kFlagStride;
    uint64_t *post1 = c; c += (size_t)L.dir[1].slots * kFlagStride;
    hs.post[0] = post0; hs.post[1] = post1;
    hs.abort_word = (uint32_t *)c; c += kFlagStride;
    uint32_t *status = (uint32_t *)c; c += kFlagStride;
    hs.status_word = status;
    uint32_t *done = (uint32_t *)c;
    hs.done_word = done;
    hs.L = &L;
    hs.ring = ring.data();
    hs.threads[0] = info.drain_threads;
    hs.threads[1] = info.fill_threads;
    hs.yield_when_idle = seed % 2 == 0;                // both idle policies get raced
    hs.timeout_ns = (uint64_t)o.timeout_ms * 1000000ull;
    hs.error.store(0);
    hs.end_ns[0].store(0); hs.end_ns[1].store(0);
    HostCrew crew;
    crew.start(&hs);

    FakeGpu gpu;
    gpu.L = &L; gpu.ring = ring.data();
    gpu.host_flags[0] = hs.wait[0]; gpu.host_flags[1] = hs.wait[1];
    gpu.post[0] = post0; gpu.post[1] = post1;
    gpu.host_abort = hs.abort_word; gpu.status = status; gpu.done = done;
    gpu.team[0] = info.team_out ? info.team_out : 1; gpu.team[1] = info.team_in ? info.team_in : 1;
    gpu.wgs[0] = 5; gpu.wgs[1] = 3;
    gpu.in_place = in_place;
    gpu.never_start = scenario == "dead_gpu";
    gpu.quit_early = scenario == "gpu_quits";

    int fails = 0;
    for (int round = 0; round < (scenario == "swap" ? 2 : 1); round++) {   // a plan is reusable: two passes
        std::fill(ctrl.begin(), ctrl.end(), 0);
        hs.begin_pass();
        gpu.dev_abort.store(0); gpu.gathered_prefix.store(0);
        const auto t0 = std::chrono::steady_clock::now();
        for (int x = 0; x < 2; x++)
            if (L.dir[x].chunks.empty()) done[x] = 1;
        gpu.launch();
        crew.wake(3u);
        // the caller's early exit: every incoming byte is in "HBM" when this returns 0
        const int in_rc = hs.wait_direction(1);
        int early_fails = 0;
        if (must_succeed || scenario == "stall") {   // withheld outgoing credits do not hold the incoming side up
            if (in_rc) { std::printf("wait_direction(1) failed: %d\n", in_rc); early_fails++; }
            for (size_t i = 0; i < B.rows.size() && !in_rc; i++)
                if (std::memcmp(B.rows[i].dev_ptr, want_b[i].data(), B.rows[i].bytes)) { std::printf("incoming allocation %zu not complete at wait_direction\n", i); early_fails++; }
        } else if (in_rc != NIXIE_ETIMEOUT) {
            std::printf("wait_direction(1) on a dead device returned %d\n", in_rc);
            early_fails++;
        }
        crew.wait();
        gpu.join();
        fails += early_fails;
        const double ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
        const int err = hs.error.load();
        if (must_succeed) {
            if (err) { std::printf("switch failed: %d\n", err); fails++; }
            for (size_t i = 0; i < A.rows.size(); i++)
                if (std::memcmp(A.rows[i].host_ptr, want_a[i].data(), A.rows[i].bytes)) { std::printf("evicted allocation %zu differs\n", i); fails++; }
            for (size_t i = 0; i < B.rows.size(); i++)
                if (std::memcmp(B.rows[i].dev_ptr, want_b[i].data(), B.rows[i].bytes)) { std::printf("restored allocation %zu differs\n", i); fails++; }
            if (hs.done_chunks[0].load() != L.dir[0].staged) { std::printf("drained %llu of %llu chunks\n", (unsigned long long)hs.done_chunks[0].load(), (unsigned long long)L.dir[0].staged); fails++; }
        } else {
            if (err != NIXIE_ETIMEOUT) { std::printf("expected NIXIE_ETIMEOUT, got %d\n", err); fails++; }
            if (ms > 5000) { std::printf("took %.0f ms to give up\n", ms); fails++; }
        }
        std::printf("%s seed %llu pass %d: %zu + %zu chunks, %.1f ms, error %d\n", scenario.c_str(), (unsigned long long)seed, round,
                    L.dir[0].chunks.size(), L.dir[1].chunks.size(), ms, err);
    }
    crew.stop();
    if (tier) {
        tier_unregister((uint64_t)(uintptr_t)A.host.data());
        tier_unregister((uint64_t)(uintptr_t)B.host.data());
    }
    if (spaces) {
        space_unregister((uint64_t)(uintptr_t)base_a);
        space_unregister((uint64_t)(uintptr_t)base_b);
        munmap(base_a, span_bytes);
        munmap(base_b, span_bytes);
    }
    return fails ? 1 : 0;
}

}  // namespace

int main(int argc, char **argv) {
    if (argc < 2) { std::printf("usage: fake_gpu <swap|in_place|spaces|tier|tier_in_place|stall|gpu_quits|dead_gpu> [seed]\n"); return 2; }
    return run(argv[1], argc > 2 ? std::strtoull(argv[2], nullptr, 10) : 1);
}
