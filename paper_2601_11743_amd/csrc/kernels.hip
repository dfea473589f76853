// HIP kernels of libnixie for gfx950: the persistent gather/scatter swap kernel, the
// per-allocation hash kernel, a counter-clearing kernel and the plain copy kernel used by the
// link probe.
//
// Paper, "Speeding Up Context Switches": while application B's data moves into GPU memory,
// application A's data moves out, so both directions of the full-duplex host link carry
// payload at once ("Existing Approach #3" explains why one direction at a time wastes half the
// link).  The paper issues the device leg as asynchronous 2 MB block copies; here one kernel
// drives both directions itself: gather workgroups copy outgoing chunks from HBM into pinned
// ring slots, scatter workgroups copy incoming chunks from ring slots into HBM, 16 bytes per
// lane, each wave instruction moving 1 KiB of contiguous bytes.
//
// Slots and flags.  A direction's slots are a free pool.  Every flag carries a chunk id, so a
// change of value is the event:
//   outgoing: GPU  ready[s]    = k + 1  "slot s holds chunk k"        -> a host drain thread copies it out
//             host released[s] = k + 2  "chunk k has left slot s"     -> the pump gives s to the next chunk
//   incoming: host filled[s]   = k + 1  "slot s holds chunk k"        -> the pump tells the scatter workers
//             GPU  freed[s]    = k + 1  "chunk k has left slot s"     -> a host fill thread refills it
// In-place switch (incoming ranges reuse GPU memory of outgoing ones): the outgoing pump also
// publishes how many leading outgoing chunks have left HBM, and a scatter unit waits until that
// count reaches its chunk's dependency before it overwrites anything.
// Workgroups sharing a chunk meet on a device-scope counter and the last one stores the
// host-visible flag.  All flag traffic is relaxed system-scope atomics; the ordering of payload
// against flags is built by hand (see the comments at the places that do it), because
// cache-maintaining fences at device or system scope cost 5-15 % of the link rate here: payload
// goes into the ring with write-through system-scope stores and comes out of it with
// system-scope loads.
//
// Workers never poll host memory: one pump wave per direction reads the host-written flags and
// publishes chunk -> slot assignments in device memory, and relays the host's abort word.
//
// Forward progress: work units are handed out in order by an atomic ticket and slots are given
// to chunks in order, so the oldest unfinished chunk always has a slot and workgroups that are
// already running.  Every worker wait is bounded (abort word in device memory, 100 MHz
// wall-clock limit) and the pump leaves once all workers have, so the grid always drains.
#include <hip/hip_runtime.h>

#include <mutex>

#include "internal.hpp"

using namespace nixie;

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kDirect = 0xFFFFFFFFu;             // "slot + 1" of a chunk that uses no slot
// loads in flight per lane before the stores, per direction: 16 B x 64 lanes x N = one tile per wave pass
constexpr uint32_t kUnrollOut = NIXIE_UNROLL_OUT, kUnrollIn = NIXIE_UNROLL_IN;
static_assert(kUnrollOut == 8 || kUnrollOut == 4 || kUnrollOut == 2 || kUnrollOut == 1, "gather unroll");
static_assert(kUnrollIn == 8 || kUnrollIn == 4 || kUnrollIn == 2, "load_from_host is written out for these");

__device__ __forceinline__ uint64_t mix64_dev(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// kUnrollIn 16-byte loads from the pinned ring, then one wait for all of them.  The loads carry
// the system-scope bits (sc0 sc1), so they are served from host memory itself and never from
// a cache line left over from an earlier use of the slot; no cache invalidation is needed
// between the host's "slot ready" flag and these loads.  One asm block, because the compiler
// does not track loads issued from inline asm: the values are only valid after the wait.
__device__ __forceinline__ void load_from_host(u32x4 (&v)[kUnrollIn], const u32x4 *const (&a)[kUnrollIn]) {
#if NIXIE_UNROLL_IN == 8
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
#elif NIXIE_UNROLL_IN == 4
    asm volatile(
        "global_load_dwordx4 %0, %4, off sc0 sc1\n"
        "global_load_dwordx4 %1, %5, off sc0 sc1\n"
        "global_load_dwordx4 %2, %6, off sc0 sc1\n"
        "global_load_dwordx4 %3, %7, off sc0 sc1\n"
        "s_waitcnt vmcnt(0)"
        : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3])
        : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3])
        : "memory");
#else
    asm volatile(
        "global_load_dwordx4 %0, %2, off sc0 sc1\n"
        "global_load_dwordx4 %1, %3, off sc0 sc1\n"
        "s_waitcnt vmcnt(0)"
        : "=&v"(v[0]), "=&v"(v[1])
        : "v"(a[0]), "v"(a[1])
        : "memory");
#endif
}

// One 16-byte store into the pinned ring with the system-scope bits set: written through to
// host memory instead of being held in the L2 (the driver maps pinned host memory cacheable
// for the GPU), so that "all my stores are acknowledged" means "the payload is in host memory".
__device__ __forceinline__ void store_to_host(u32x4 *p, u32x4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(p), "v"(v) : "memory");
}

// Copy n bytes between a device range and its image in a ring slot.  The two addresses are
// congruent modulo 16 (the planner guarantees it), so one head/tail peel serves both sides.
// Both sides are addressed as global memory (address space 1): the addresses arrive as integers in
// the descriptors, and through a generic pointer every access would be a flat instruction that
// also has to be checked against the LDS and scratch apertures.
typedef __attribute__((address_space(1))) u32x4 GVec;
typedef __attribute__((address_space(1))) uint8_t GByte;
template <bool TO_RING>
__device__ __forceinline__ void copy_span(uint8_t *dev, uint8_t *ring, uint32_t n, uint32_t lane) {
    GByte *gdev = (GByte *)(uintptr_t)dev, *gring = (GByte *)(uintptr_t)ring;
    uint32_t head = (16u - ((uint32_t)(uintptr_t)ring & 15u)) & 15u;
    if (head > n) head = n;
    if (lane < head) {   // byte accesses to the ring are system-scope atomics: same write-through / no-cache rule
        if (TO_RING) __hip_atomic_store(gring + lane, gdev[lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        else gdev[lane] = __hip_atomic_load(gring + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    const uint32_t nvec = (n - head) >> 4;
    GVec *dev4 = (GVec *)(gdev + head);
    const u32x4 *ring4_in = (const u32x4 *)(ring + head);   // the ring side goes through the asm loads and stores
    u32x4 *ring4_out = (u32x4 *)(ring + head);
    constexpr uint32_t kU = TO_RING ? kUnrollOut : kUnrollIn;
    for (uint32_t j = lane; j - lane < nvec; j += 64 * kU) {   // wave-uniform trip count
        u32x4 v[kU];
        if constexpr (TO_RING) {
#pragma unroll
            for (uint32_t u = 0; u < kU; u++)
                if (j + 64 * u < nvec) v[u] = dev4[j + 64 * u];
        } else {
            // out-of-range lanes re-read the last vector of the span (one extra line) and drop it
            const u32x4 *a[kU];
#pragma unroll
            for (uint32_t u = 0; u < kU; u++) a[u] = ring4_in + (j + 64 * u < nvec ? j + 64 * u : nvec - 1);
            load_from_host(v, a);
        }
#pragma unroll
        for (uint32_t u = 0; u < kU; u++)
            if (j + 64 * u < nvec) {
                if (TO_RING) store_to_host(ring4_out + j + 64 * u, v[u]);
                else dev4[j + 64 * u] = v[u];
            }
    }
    const uint32_t done = head + (nvec << 4);
    if (lane < n - done) {
        if (TO_RING) __hip_atomic_store(gring + done + lane, gdev[done + lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        else gdev[done + lane] = __hip_atomic_load(gring + done + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

// One wave copies the part of the slot image [t0, t1) that the chunk's segments cover.
template <bool TO_RING>
__device__ __forceinline__ void copy_tile(const DevSeg *segs, uint32_t nseg, uint8_t *slot, uint32_t t0,
                                          uint32_t t1, uint32_t lane) {
    uint32_t lo = 0, hi = nseg;   // first segment that ends after t0
    while (lo < hi) {
        uint32_t mid = (lo + hi) >> 1;
        DevSeg s = segs[mid];
        if (s.slot_off + s.len <= t0) lo = mid + 1; else hi = mid;
    }
    for (uint32_t i = lo; i < nseg; i++) {
        DevSeg s = segs[i];
        if (s.slot_off >= t1) break;
        uint32_t x0 = s.slot_off > t0 ? s.slot_off : t0;
        uint32_t x1 = s.slot_off + s.len < t1 ? s.slot_off + s.len : t1;
        if (x0 >= x1) continue;
        copy_span<TO_RING>((uint8_t *)(uintptr_t)(s.dev + (x0 - s.slot_off)), slot + x0, x1 - x0, lane);
    }
}

// One work unit of direction DIR: take a ticket, wait for the chunk's slot (and, in place, for the
// GPU bytes it overwrites to have left), copy, arrive.  Returns false when the direction has no
// unit left for this workgroup (tickets used up, abort, or a wait ran out).  Workgroup-uniform.
template <int DIR>
__device__ bool do_unit(const SwapArgs &a, uint64_t &stall) {
    const DevDir &D = a.d[DIR];
    __shared__ uint32_t s_unit;
    __shared__ uint32_t s_slot;   // slot + 1 of the unit's chunk, 0 = stop
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t waves_per_wg = kWgThreads / 64;
    const uint32_t total_units = D.n_chunks * D.team;
    if (tid == 0) {
        uint32_t cs = 0;
        const uint32_t u = __hip_atomic_fetch_add(D.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (u < total_units && !__hip_atomic_load(a.dev_abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
            // The pump wave writes chunk_slot[k] once chunk k has a slot: outgoing, a slot the
            // host has released; incoming, the slot the host has filled with chunk k.  Workers
            // only ever poll device memory: a poll over the link queues behind the bulk reads.
            // A direct chunk (pinned tier) needs no slot: its image already has a place.
            const uint32_t *where = D.chunk_slot + u / D.team;
            cs = u / D.team >= D.n_staged ? kDirect
                                          : __hip_atomic_load(where, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (cs == 0) {
                const uint64_t t0 = wall_clock64();
                uint32_t it = 0;
                while ((cs = __hip_atomic_load(where, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) == 0) {
                    if ((++it & 7u) == 0) {
                        if (__hip_atomic_load(a.dev_abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) break;
                        if (wall_clock64() - t0 > a.timeout_ticks) {
                            __hip_atomic_store(a.dev_abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            __hip_atomic_store(a.gpu_status, (uint32_t)kGpuTimeout, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                            break;
                        }
                    }
                    __builtin_amdgcn_s_sleep(4);
                }
                stall += wall_clock64() - t0;
            }
            // In-place switch: the GPU bytes this chunk overwrites must have been gathered.
            if (DIR == 1 && cs != 0 && a.track_prefix) {
                const uint32_t dep = D.chunks[u / D.team].dep;
                if (__hip_atomic_load(a.gathered_prefix, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < dep) {
                    const uint64_t t0 = wall_clock64();
                    uint32_t it = 0;
                    while (__hip_atomic_load(a.gathered_prefix, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < dep) {
                        if ((++it & 7u) == 0) {
                            if (__hip_atomic_load(a.dev_abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) { cs = 0; break; }
                            if (wall_clock64() - t0 > a.timeout_ticks) {
                                __hip_atomic_store(a.dev_abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                                __hip_atomic_store(a.gpu_status, (uint32_t)kGpuTimeout, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                                cs = 0;
                                break;
                            }
                        }
                        __builtin_amdgcn_s_sleep(4);
                    }
                    stall += wall_clock64() - t0;
                }
            }
        }
        s_unit = u;
        s_slot = cs;
    }
    __syncthreads();
    const uint32_t u = s_unit, cs = s_slot;
    __syncthreads();   // everybody has read the two words before thread 0 can write them again
    if (u >= total_units || cs == 0) return false;
    const uint32_t k = u / D.team, part = u % D.team;
    const uint32_t slot = cs - 1;
    const bool direct = cs == kDirect;
    const DevChunk ch = D.chunks[k];
    uint8_t *slot_base = direct ? (uint8_t *)(uintptr_t)D.direct_base[k - D.n_staged]
                                : D.ring + (size_t)slot * a.slot_bytes;

    constexpr uint32_t kTile = kTileBytesDir[DIR];
    const uint32_t n_tiles = (ch.used + kTile - 1) / kTile;
    for (uint32_t t = part * waves_per_wg + wave; t < n_tiles; t += D.team * waves_per_wg) {
        const uint32_t t0 = t * kTile;
        const uint32_t t1 = t0 + kTile < ch.used ? t0 + kTile : ch.used;
        copy_tile<DIR == 0>(D.segs + ch.seg_begin, ch.seg_count, slot_base, t0, t1, lane);
    }
    // Payload before flag, without a release fence.  A system- or device-scope release would
    // write back the whole L2 (which holds the scatter side's dirty HBM lines) for every work
    // unit, and measurably slows both directions.  Every store into the ring is a write-through
    // system-scope store, so it is enough that every wave waits until all of its stores are
    // acknowledged (vmcnt = 0), that the workgroup then meets at the barrier, and that
    // thread 0 only afterwards bumps the arrive counter and stores the flag.  The flag is a
    // later posted write on the same link and cannot pass the payload.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) {
        // (for the outgoing direction the counter also tells the pump that the chunk has left HBM:
        //  every load of this unit completed before the barrier above)
        const uint32_t old = __hip_atomic_fetch_add(D.arrive + k, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool last = (old == D.team - 1) && !direct;   // nobody waits for a direct chunk's slot
        if (last) {   // outgoing: "slot holds chunk k"; incoming: "chunk k has left the slot"
            __hip_atomic_store(D.post_flags + (size_t)slot * kFlagStride, (uint64_t)k + 1u, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_SYSTEM);
            __hip_atomic_store(D.stamp + slot, wall_clock64(), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    return true;
}

// This workgroup will take no more units of direction DIR.  The pump reports "direction complete"
// to the host once every workgroup that could work on the direction has said so, and the host may
// then let the incoming application run while this kernel is still evicting.  What this workgroup
// scattered into HBM must therefore be out of this XCD's L2 before it counts as gone: all waves wait
// for their stores, and one device-scope release (an L2 write-back, once per workgroup, not per work
// unit) precedes the increment.  The gather side wrote only write-through stores and needs none.
template <int DIR>
__device__ void leave_direction(const SwapArgs &a, uint64_t &stall) {
    const DevDir &D = a.d[DIR];
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        if (stall) __hip_atomic_fetch_add(D.stall_ticks, stall, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (DIR == 1) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        __hip_atomic_fetch_add(D.exited, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // on every exit path
    }
    stall = 0;
}

// XCC_ID hardware register, bits 3:0 = the XCD this workgroup runs on
__device__ __forceinline__ bool sits_out(const SwapArgs &a) {
    return a.xcd_mask && !((a.xcd_mask >> (__builtin_amdgcn_s_getreg((3 << 11) | 20) & 7u)) & 1u);
}

// A workgroup with a fixed role: units of one direction until there are none left.
template <int DIR>
__device__ void run_direction(const SwapArgs &a) {
    uint64_t stall = 0;
    if (!sits_out(a))
        while (do_unit<DIR>(a, stall)) {}
    leave_direction<DIR>(a, stall);
}

// A workgroup without a fixed role: before every unit it looks at how many chunks either direction
// still has to hand out and takes a unit of the one with more left (the outgoing one on a tie:
// its stores need more workgroups than the loads of the other).  Two equal working sets therefore
// finish together whatever the rates of the two directions turn out to be on this machine, and once
// one direction is done its share of these workgroups goes to the other.
__device__ void run_either(const SwapArgs &a) {
    __shared__ int s_dir;
    __shared__ uint32_t s_none_left;   // bit x: direction x has handed out its last unit
    uint64_t stall[2] = {0, 0};
    bool live[2] = {a.d[0].wgs != 0, a.d[1].wgs != 0};
    if (sits_out(a)) {
        if (live[0]) leave_direction<0>(a, stall[0]);
        if (live[1]) leave_direction<1>(a, stall[1]);
        return;
    }
    while (live[0] || live[1]) {
        if (threadIdx.x == 0) {
            uint32_t left[2];
            for (int x = 0; x < 2; x++) {
                const uint32_t total = a.d[x].n_chunks * a.d[x].team;
                const uint32_t t = live[x] ? __hip_atomic_load(a.d[x].ticket, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : total;
                left[x] = t < total ? (total - t + a.d[x].team - 1) / a.d[x].team : 0;
            }
            // In place the incoming direction can never be ahead (a chunk is written only where the old
            // bytes have left), so "more left" would always point at it, and the help would stand waiting
            // for the outgoing side: there the help goes to the outgoing direction while it has units.
            s_dir = !left[0] ? 1 : !left[1] ? 0 : a.track_prefix ? 0 : left[1] > left[0] ? 1 : 0;
            s_none_left = (left[0] ? 0u : 1u) | (left[1] ? 0u : 2u);
        }
        __syncthreads();
        const int dir = s_dir;
        const uint32_t none_left = s_none_left;
        __syncthreads();
        // A direction without units left is left at once, not when the other one runs dry too: the pump
        // reports "direction complete" only after every workgroup that could have worked on it has said
        // goodbye, and the host may be waiting for exactly that to let the incoming application run.
        if (live[0] && (none_left & 1u)) { live[0] = false; leave_direction<0>(a, stall[0]); }
        if (live[1] && (none_left & 2u)) { live[1] = false; leave_direction<1>(a, stall[1]); }
        if (!live[dir]) continue;   // (then the other one has units, or the loop ends)
        if (dir == 0) {
            if (!do_unit<0>(a, stall[0])) { live[0] = false; leave_direction<0>(a, stall[0]); }
        } else {
            if (!do_unit<1>(a, stall[1])) { live[1] = false; leave_direction<1>(a, stall[1]); }
        }
    }
}

// Slot pump: one wave per direction reads that direction's host-written flags from pinned
// memory, over and over, and turns every change into a chunk -> slot assignment in device memory.
//   outgoing: released[s] changed  -> slot s is free again -> it goes to the next chunk, in order
//   incoming: filled[s] = k + 1    -> chunk k sits in slot s
// Slots are therefore a free pool, not a fixed k mod n rotation: a chunk whose workgroups run on
// a slow XCD (they differ by 2x on the way to the host link) holds only its own slot instead of
// stalling every chunk behind it.  The pump also relays the host's abort word.  It leaves when
// every worker workgroup of its direction has left; workers always leave (bounded waits).
__device__ void run_pump(const SwapArgs &a, int dir) {
    const DevDir &D = a.d[dir];
    if (D.wgs == 0) return;
    const uint32_t lane = threadIdx.x & 63u;
    uint32_t next = 0;     // outgoing: next chunk without a slot (wave-uniform)
    uint32_t prefix = 0;   // outgoing, in-place switch: leading chunks that have left HBM (wave-uniform)
    const bool track = dir == 0 && a.track_prefix;
    uint32_t rounds = 0, told = 0;   // sign of life for the host: units handed out, every 32nd round if it moved
    auto advance_prefix = [&]() {   // up to 64 chunks per call; true if it moved
        const uint32_t k = prefix + lane;
        const bool done = k < D.n_chunks &&
                          __hip_atomic_load(D.arrive + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= D.team;
        const uint64_t pending = ~__ballot(done);                         // first zero bit = first unfinished chunk
        const uint32_t step = pending ? (uint32_t)__builtin_ctzll(pending) : 64u;
        if (step == 0) return false;
        prefix += step;
        if (lane == 0) __hip_atomic_store(a.gathered_prefix, prefix, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return true;
    };
    // One round: read every host-written flag once, act on the changes.  The first 256 slots (four
    // per lane) are read with all loads in flight at once -- a round then costs one trip over the link
    // instead of one per 64 slots -- and their last-seen values stay in registers; slots beyond that
    // go 64 at a time through seen[] in device memory.
    constexpr uint32_t kRegGroups = 4;
    uint64_t seen_r[kRegGroups] = {0, 0, 0, 0};
    uint64_t rtt_sum = 0;   // per lane: credit round trips of this lane's slots
    uint32_t rtt_n = 0;
    auto act = [&](uint32_t s, uint64_t v, bool changed) {   // wave-uniform call, per-lane arguments
        if (changed) {
            const uint64_t posted = __hip_atomic_load(D.stamp + s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (posted) { rtt_sum += wall_clock64() - posted; rtt_n++; }
        }
        if (dir == 0) {
            const uint64_t mask = __ballot(changed);
            const uint32_t rank = __popcll(mask & ((1ull << lane) - 1ull));
            if (changed) {
                const uint32_t k = next + rank;
                if (k < D.n_staged)
                    __hip_atomic_store(D.chunk_slot + k, s + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            next += (uint32_t)__popcll(mask);
        } else if (changed) {
            const uint64_t k = v - 1;
            if (k < D.n_staged)
                __hip_atomic_store(D.chunk_slot + k, s + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    };
    for (;;) {
        uint64_t v_r[kRegGroups];
#pragma unroll
        for (uint32_t j = 0; j < kRegGroups; j++) {   // unconditional (a lane without a slot re-reads slot 0): no branch, no wait between them
            const uint32_t s = lane + 64 * j;
            v_r[j] = __hip_atomic_load(D.host_flags + (s < D.n_slots ? s : 0), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
        const uint32_t gone = __hip_atomic_load(D.exited, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (uint32_t j = 0; j < kRegGroups; j++) {
            if (64 * j >= D.n_slots) break;
            const bool mine = lane + 64 * j < D.n_slots;
            const bool changed = mine && v_r[j] != seen_r[j];
            act(lane + 64 * j, v_r[j], changed);
            if (mine) seen_r[j] = v_r[j];
        }
        for (uint32_t base = 64 * kRegGroups; base < D.n_slots; base += 64) {
            const uint32_t s = base + lane;
            uint64_t v = 0, old = 0;
            if (s < D.n_slots) {
                v = __hip_atomic_load(D.host_flags + s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                old = __hip_atomic_load(D.seen + s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            const bool changed = v != old;
            act(s, v, changed);
            if (changed) __hip_atomic_store(D.seen + s, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        // the host's abort word: every eighth round is soon enough (every wait is bounded anyway)
        if ((rounds & 7u) == 0 && __hip_atomic_load(a.host_abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) &&
            !__hip_atomic_load(a.dev_abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) && lane == 0) {
            __hip_atomic_store(a.dev_abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(a.gpu_status, (uint32_t)kGpuSawAbort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
        if (track) advance_prefix();
        if ((++rounds & 31u) == 0) {
            const uint32_t t = __hip_atomic_load(D.ticket, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (t != told && lane == 0)
                __hip_atomic_store(a.dir_done + kProgressWord + dir, t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            told = t;
        }
        if (gone >= D.wgs) {   // (read at the start of this round: everything those workgroups did came before)
            // every gather workgroup has left, so every arrive counter is final: publish the rest
            // (bounded: at most n_chunks / 64 + 1 rounds)
            if (track) while (prefix < D.n_chunks && advance_prefix()) {}
            for (int off = 32; off > 0; off >>= 1) {
                rtt_sum += __shfl_down((unsigned long long)rtt_sum, off, 64);
                rtt_n += __shfl_down(rtt_n, off, 64);
            }
            if (lane == 0) {
                __hip_atomic_store(a.dir_done + kRttWord + dir, rtt_n ? (uint32_t)(rtt_sum / rtt_n) : 0u, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_SYSTEM);
                __hip_atomic_store(a.dir_done + kRoundsWord + dir, rounds, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                __hip_atomic_store(a.dir_done + dir, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            }
            break;
        }
        __builtin_amdgcn_s_sleep(2);
    }
}

// The last workgroup to leave the kernel hands the stall sums to the host and clears every counter,
// so the next switch needs no clearing launch of its own.  Every access to the counters, the
// clearing included, is an agent-scope atomic: the XCDs' L2s are not coherent with each other for
// plain accesses, and a stale dirty line written back at the end of the kernel must not undo the
// clearing.  A workgroup only counts as gone once its own counter traffic has been acknowledged.
__device__ void leave_kernel(const SwapArgs &a) {
    __shared__ uint32_t s_last;
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0)
        s_last = __hip_atomic_fetch_add(a.all_left, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == gridDim.x - 1;
    __syncthreads();
    if (!s_last) return;
    if (threadIdx.x < 2) {
        const uint64_t t = __hip_atomic_load(a.d[threadIdx.x].stall_ticks, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(a.stall_out + threadIdx.x, t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    for (uint64_t i = threadIdx.x; i < a.n_counters; i += kWgThreads)
        __hip_atomic_store(a.counters + i, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Block 0 is the pump (first to be dispatched, so it is resident before any worker can wait on
// it); then the gather workers, the scatter workers, and the workgroups that serve either direction.
__global__ void __launch_bounds__(kWgThreads) nixie_swap_kernel(SwapArgs a) {
    if (blockIdx.x == 0) {
        const uint32_t wave = threadIdx.x >> 6;
        if (threadIdx.x == 0)   // from here on a host thread's wait is a credit wait, not queue delay
            __hip_atomic_store(a.dir_done + kStartedWord, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        if (wave < 2) run_pump(a, (int)wave);
    } else if (blockIdx.x - 1 < a.fixed_wgs[0]) {
        run_direction<0>(a);
    } else if (blockIdx.x - 1 < a.fixed_wgs[0] + a.fixed_wgs[1]) {
        run_direction<1>(a);
    } else {
        run_either(a);
    }
    leave_kernel(a);
}

__global__ void __launch_bounds__(256) nixie_zero32_kernel(uint32_t *p, uint64_t n) {
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x)
        p[i] = 0;
}

// H = mix64(bytes) + sum_k mix64(w_k + G (k+1)).  A tile is up to 4096 words (32 KiB) of one
// allocation; each workgroup takes a contiguous run of tiles, so it finds its first allocation
// by binary search once and then only steps forward.  Every thread keeps one running sum for the
// allocation it is in and hands it over only when the run moves on to another allocation (or ends):
// a wave-shuffle reduction and one 64-bit atomic add per wave into the allocation's slot (hashes
// must be zero on entry).  No barrier anywhere, so a wave's loads of the next tile are not held up
// by the slowest wave of the last one.  16 B loads, eight in flight per lane.  HBM-read bound: 1 B
// read per byte hashed.
__global__ void __launch_bounds__(256) nixie_hash_kernel(const HashDesc *descs, uint64_t n, uint64_t total_tiles,
                                                         uint64_t *hashes) {
    constexpr uint64_t G = 0x9E3779B97F4A7C15ull;
    typedef uint64_t u64x2 __attribute__((ext_vector_type(2)));
    typedef __attribute__((address_space(1))) u64x2 GlobalU64x2;
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint64_t per = (total_tiles + gridDim.x - 1) / gridDim.x;
    const uint64_t t_begin = (uint64_t)blockIdx.x * per;
    const uint64_t t_end = t_begin + per < total_tiles ? t_begin + per : total_tiles;
    if (t_begin >= t_end) return;
    uint64_t lo = 0, hi = n;   // last descriptor whose first tile is <= t_begin
    while (lo < hi) {
        uint64_t mid = (lo + hi) >> 1;
        if (descs[mid].first_tile <= t_begin) lo = mid + 1; else hi = mid;
    }
    uint64_t i = lo - 1;
    HashDesc d = descs[i];
    uint64_t acc = 0;
    auto hand_over = [&](uint64_t owner) {   // wave-uniform call
        for (int off = 32; off > 0; off >>= 1) acc += __shfl_down((unsigned long long)acc, off, 64);
        if (lane == 0 && acc) atomicAdd((unsigned long long *)&hashes[owner], (unsigned long long)acc);
        acc = 0;
    };
    for (uint64_t t = t_begin; t < t_end; t++) {
        // step to the allocation that owns tile t (allocations of zero bytes own no tile)
        if (i + 1 < n && descs[i + 1].first_tile <= t) {
            hand_over(i);
            while (i + 1 < n && descs[i + 1].first_tile <= t) d = descs[++i];
        }
        const uint64_t words = (d.bytes + 7) / 8, full = d.bytes / 8;
        const uint64_t w0 = (t - d.first_tile) * kHashTileWords;
        const uint64_t w1 = w0 + kHashTileWords < words ? w0 + kHashTileWords : words;
        const uint8_t *p = (const uint8_t *)(uintptr_t)d.ptr;
        if ((d.ptr & 15u) == 0 && w1 - w0 == kHashTileWords && w1 <= full) {   // whole aligned tile
            const GlobalU64x2 *v = (const GlobalU64x2 *)(d.ptr + 8 * w0);   // a device address: global, not generic, loads
            u64x2 r[8];
#pragma unroll
            for (uint32_t u = 0; u < 8; u++) r[u] = __builtin_nontemporal_load(v + tid + 256 * u);
#pragma unroll
            for (uint32_t u = 0; u < 8; u++) {
                const uint64_t k = w0 + 2 * (uint64_t)(tid + 256 * u);
                acc += mix64_dev(r[u].x + G * (k + 1)) + mix64_dev(r[u].y + G * (k + 2));
            }
        } else {
            const bool aligned = (d.ptr & 7u) == 0;
            for (uint64_t k = w0 + tid; k < w1; k += 256) {
                uint64_t w = 0;
                if (k < full && aligned) {
                    w = *(const uint64_t *)(p + 8 * k);
                } else {
                    const uint32_t nb = k < full ? 8u : (uint32_t)(d.bytes - 8 * k);
                    for (uint32_t b = 0; b < nb; b++) w |= (uint64_t)p[8 * k + b] << (8 * b);
                }
                acc += mix64_dev(w + G * (k + 1));
            }
        }
        if (w0 == 0 && tid == 0) acc += mix64_dev(d.bytes);
    }
    hand_over(i);
}

// Plain copy for the link probe: each workgroup moves contiguous 64 KiB tiles, 16 B per lane.
__global__ void __launch_bounds__(256) nixie_copy16_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst,
                                                           uint64_t n16) {
    constexpr uint64_t kTile = 4096;
    const uint64_t ntiles = (n16 + kTile - 1) / kTile;
    for (uint64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const uint64_t base = t * kTile, end = base + kTile < n16 ? base + kTile : n16;
        for (uint64_t i = base + threadIdx.x; i < end; i += 256 * 4) {
            u32x4 v[4];
#pragma unroll
            for (int u = 0; u < 4; u++) if (i + 256ull * u < end) v[u] = src[i + 256ull * u];
#pragma unroll
            for (int u = 0; u < 4; u++) if (i + 256ull * u < end) dst[i + 256ull * u] = v[u];
        }
    }
}

// ---- hashing without allocation -------------------------------------------------------------
// The descriptor table and the per-buffer sums of nixie_hash_buffers live in device memory that
// the call allocates and frees.  The variant below keeps them in this array instead, so that it
// can be called where nothing may be allocated.  One copy of the array exists on every GPU the
// library runs on, from the moment the code object is loaded until the process ends.
struct HashScratch {
    HashDesc descs[kNoAllocMaxBuffers];
    uint64_t sums[kNoAllocMaxBuffers];
};
static __device__ __align__(256) unsigned char scratch[sizeof(HashScratch)];

// Descriptors travel as kernel arguments (by value), kNoAllocBatch at a time: no staging copy, nothing for
// the runtime to allocate.  Each launch writes its batch and clears the matching sums.
struct DescBatch { HashDesc d[kNoAllocBatch]; };
static_assert(sizeof(DescBatch) + 32 <= 4096, "a batch must fit the kernel argument buffer");

__global__ void __launch_bounds__(kNoAllocBatch) nixie_put_descs_kernel(DescBatch b, uint32_t count, HashScratch *hs,
                                                                      uint32_t first) {
    const uint32_t i = threadIdx.x;
    if (i < count) {
        hs->descs[first + i] = b.d[i];
        hs->sums[first + i] = 0;
    }
}

__global__ void __launch_bounds__(256) nixie_copy64_kernel(const uint64_t *src, uint64_t *dst, uint32_t n) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

}  // namespace

// The array's name is only a handle on the host; its address differs from GPU to GPU and is asked
// for once per device, with that device current.
int nixie_noalloc_scratch(void **out) {
    constexpr int kMaxDevices = 64;
    static void *addr[kMaxDevices];
    static std::mutex mu;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> g(mu);
    if (!addr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return (int)e;
        if (!ptr) return (int)hipErrorInvalidSymbol;
        addr[dev] = ptr;
    }
    *out = addr[dev];
    return (int)hipSuccess;
}

// The no-allocation hash in two steps, both only enqueueing on stream.  First the table, a batch at a
// time: batch = HOST array of count <= kNoAllocBatch descriptors (first_tile filled in) that become
// entries first .. first + count - 1; the matching sums are cleared.
int nixie_noalloc_put_descs(const HashDesc *batch, uint32_t count, uint32_t first, void *stream) {
    if (count == 0) return (int)hipSuccess;
    if (count > kNoAllocBatch || first + count > kNoAllocMaxBuffers) return (int)hipErrorInvalidValue;
    void *base = nullptr;
    const int e = nixie_noalloc_scratch(&base);
    if (e) return e;
    DescBatch b;
    for (uint32_t i = 0; i < count; i++) b.d[i] = batch[i];
    for (uint32_t i = count; i < kNoAllocBatch; i++) b.d[i] = HashDesc{0, 0, 0};
    nixie_put_descs_kernel<<<1, kNoAllocBatch, 0, (hipStream_t)stream>>>(b, count, (HashScratch *)base, first);
    return (int)hipGetLastError();
}

// Then the hashes of entries 0 .. n - 1 into out_d (DEVICE array of n).
int nixie_noalloc_hash(uint32_t n, uint64_t total_tiles, uint64_t *out_d, void *stream) {
    if (n == 0) return (int)hipSuccess;
    if (n > kNoAllocMaxBuffers) return (int)hipErrorInvalidValue;
    void *base = nullptr;
    int e = nixie_noalloc_scratch(&base);
    if (e) return e;
    HashScratch *hs = (HashScratch *)base;
    hipStream_t st = (hipStream_t)stream;
    if (total_tiles) {
        const uint32_t grid = (uint32_t)(total_tiles < 4096 ? total_tiles : 4096);
        nixie_hash_kernel<<<grid, 256, 0, st>>>(hs->descs, n, total_tiles, hs->sums);
        e = (int)hipGetLastError();
        if (e) return e;
    }
    nixie_copy64_kernel<<<(n + 255) / 256, 256, 0, st>>>(hs->sums, out_d, n);
    return (int)hipGetLastError();
}

int nixie_launch_swap(const SwapArgs &a, void *stream) {
    if (a.d[0].wgs + a.d[1].wgs == 0) return (int)hipSuccess;
    const uint32_t grid = a.fixed_wgs[0] + a.fixed_wgs[1] + a.flex_wgs + 1;   // + the pump
    nixie_swap_kernel<<<grid, kWgThreads, 0, (hipStream_t)stream>>>(a);
    return (int)hipGetLastError();
}

int nixie_launch_zero32(uint32_t *p, uint64_t n, void *stream) {
    if (n == 0) return (int)hipSuccess;
    uint32_t grid = (uint32_t)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
    nixie_zero32_kernel<<<grid, 256, 0, (hipStream_t)stream>>>(p, n);
    return (int)hipGetLastError();
}

int nixie_launch_hash(const HashDesc *descs, uint64_t n, uint64_t total_tiles, uint64_t *hashes, void *stream) {
    if (total_tiles == 0) return (int)hipSuccess;
    uint32_t grid = (uint32_t)(total_tiles < 4096 ? total_tiles : 4096);   // 16 workgroups per CU
    nixie_hash_kernel<<<grid, 256, 0, (hipStream_t)stream>>>(descs, n, total_tiles, hashes);
    return (int)hipGetLastError();
}

int nixie_launch_copy16(const void *src, void *dst, uint64_t bytes, uint32_t wgs, void *stream) {
    if (bytes < 16) return (int)hipSuccess;
    nixie_copy16_kernel<<<wgs, 256, 0, (hipStream_t)stream>>>((const u32x4 *)src, (u32x4 *)dst, bytes / 16);
    return (int)hipGetLastError();
}
