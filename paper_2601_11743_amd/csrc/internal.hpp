// Internal declarations of libnixie: planner output, device descriptor ABI, launchers.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

#include "nixie.h"
#include "spaces.hpp"

namespace nixie {

// ---- planner output (host) ---------------------------------------------------------------
struct DirLayout {
    std::vector<nixie_segment_t> segs;   // sorted by slot_off inside each chunk
    std::vector<nixie_chunk_t> chunks;   // in execution order: [0, staged) through the ring, then direct ones
    uint64_t bytes = 0;
    uint32_t slots = 0;
    uint64_t staged = 0;                 // number of chunks that use ring slots
    uint64_t direct_bytes = 0;
    // per direct chunk: GPU address of the pinned-tier image of slot offset 0 (16-byte aligned), so
    // that "base + slot_off" addresses a direct segment exactly as it addresses one in a ring slot
    std::vector<uint64_t> direct_base;
};

struct Layout {
    uint64_t ring_bytes = 0, slot_bytes = 0;
    nixie_opts_t opts{};
    DirLayout dir[2];                     // 0 = outgoing (GPU -> host), 1 = incoming
    std::vector<nixie_alloc_t> table[2];  // copies of the caller's tables, table order
    std::vector<SpaceUse> uses[2];        // blocks of registered spaces that each table touches
    std::vector<uint64_t> tier_ids;       // registrations of the pinned tier that direct chunks point into
};

int build_layout(const nixie_table_t *out_table, const nixie_table_t *in_table, uint64_t ring_bytes,
                 const nixie_opts_t *opts, Layout &L);
void fill_info(const Layout &L, nixie_plan_info_t *info);

// ---- host copies and hashing ---------------------------------------------------------------
void copy_stream(void *dst, const void *src, size_t n);   // non-temporal stores, any alignment
uint64_t mix64(uint64_t z);
uint64_t hash_host_range(const uint8_t *base, uint64_t n, uint64_t word_begin, uint64_t word_end);
int copy_host_buffers(void *const *dst, const void *const *src, const uint64_t *bytes, uint64_t n, unsigned threads);
int hash_host_buffers(const void *const *ptrs, const uint64_t *bytes, uint64_t n, uint64_t *hashes,
                      unsigned threads);

// ---- device descriptor ABI (shared by runtime.cpp and kernels.hip) ------------------------
struct DevSeg { uint64_t dev; uint32_t slot_off; uint32_t len; };
struct DevChunk { uint32_t seg_begin, seg_count, used, dep; };   // dep: see nixie_chunk_t::dep_out

constexpr uint32_t kFlagStride = 8;        // GPU-written flags: one 64 B line (8 x u64) per flag
// Host-written flags are packed (one u64 each, a direction's array padded to whole 64 B lines):
// a single wave of the kernel reads a direction's credits with a few line-sized link reads.
inline uint64_t wait_flag_words(uint32_t slots) { return ((uint64_t)slots + 7) / 8 * 8; }
constexpr uint32_t kWgThreads = 256;
// One wave pass ("tile"): 16 B per lane, 64 lanes, N loads in flight per lane before the stores.  N is
// chosen per direction: the bytes a wave has in flight set how deep the queues towards the link run,
// and posted writes (outgoing) want shallower queues than reads (incoming).
#ifndef NIXIE_UNROLL_OUT
#define NIXIE_UNROLL_OUT 4
#endif
#ifndef NIXIE_UNROLL_IN
#define NIXIE_UNROLL_IN 4
#endif
constexpr uint32_t kTileBytesDir[2] = {16 * 64 * NIXIE_UNROLL_OUT, 16 * 64 * NIXIE_UNROLL_IN};
constexpr uint32_t kTileBytes = 16 * 64 * 8;   // nominal tile of the host-side device model used in tests

// Words of the GPU-written "done" line (u32 each): [0], [1] = 1 once every workgroup of direction
// 0 / 1 has left; [kStartedWord] = 1 once the kernel runs (until then a waiting host thread is
// looking at queue delay, not at a stalled credit); [kProgressWord + x] = work units of direction
// x handed out so far, refreshed by the pump now and then (a sign of life for a waiter that sees
// no slot traffic, e.g. when every chunk moves directly).
constexpr uint32_t kStartedWord = 2, kProgressWord = 4;
constexpr uint32_t kRoundsWord = 6;  // [kRoundsWord + x]: rounds the pump of direction x made over the host's flags
constexpr uint32_t kRttWord = 12;    // [kRttWord + x]: mean time, in 100 MHz ticks, between the GPU's flag for a slot of direction x
                                     // and the pump seeing the host's answer for that slot (the credit round trip)
constexpr uint32_t kStallWord = 8;   // u32 index of two u64: summed stall ticks per direction, written as the kernel ends
// a host thread that has not yet seen the kernel start waits this many times the credit bound
constexpr uint64_t kStartGrace = 4;

// gpu_status values (host-visible word written by the kernel when it stops early)
enum : uint32_t { kGpuOk = 0, kGpuSawAbort = 1, kGpuTimeout = 2 };

struct DevDir {
    const DevSeg *segs;
    const DevChunk *chunks;
    uint8_t *ring;               // device-visible address of this direction's first slot
    const uint64_t *host_flags;  // host-written, pinned, packed: out: released[s]  in: filled[s]
    uint64_t *post_flags;        // GPU-written,  pinned, one line each: out: ready[s]  in: freed[s]
    uint64_t *seen;              // device memory, pump only: last value of host_flags[s] acted on (slots beyond 256)
    uint64_t *stamp;             // device memory, per slot: wall clock when the GPU last posted a flag for it
    uint32_t *chunk_slot;        // device memory, per chunk: 0 = no slot yet, else slot + 1
    uint32_t *ticket;            // device memory, one counter
    uint32_t *exited;            // device memory, workgroups of this direction that have left
    uint32_t *arrive;            // device memory, one counter per chunk
    uint64_t *stall_ticks;       // device memory, summed wait time
    uint32_t n_chunks, n_slots, team;
    uint32_t wgs;                // workgroups that may take units of this direction (fixed + either); 0 = the direction does not run
    uint32_t n_staged;           // chunks [0, n_staged) take ring slots; the rest are direct
    const uint64_t *direct_base; // device memory, per direct chunk
};

struct SwapArgs {
    DevDir d[2];
    uint64_t slot_bytes;
    const uint32_t *host_abort;  // pinned, host-written
    uint32_t *gpu_status;        // pinned, GPU-written
    uint32_t *dev_abort;         // device memory
    uint64_t timeout_ticks;      // 100 MHz wall clock
    uint32_t *gathered_prefix;   // device memory: number of leading outgoing chunks that have left HBM
    uint32_t track_prefix;       // 1: in-place switch with both directions running in this launch
    uint32_t xcd_mask;           // 0 = every XCD takes part
    uint32_t *dir_done;          // pinned, GPU-written "done" line: see kStartedWord / kProgressWord
    uint32_t fixed_wgs[2];       // workgroups that only gather / only scatter
    uint32_t flex_wgs;           // workgroups that take units of whichever direction has more left
    uint32_t *counters;          // device memory: the whole counter block, cleared by the last workgroup to leave
    uint64_t n_counters;
    uint32_t *all_left;          // device memory: workgroups (pump included) that have left the kernel
    uint64_t *stall_out;         // pinned, GPU-written at the end: [x] = summed stall ticks of direction x
};

struct HashDesc { uint64_t ptr; uint64_t bytes; uint64_t first_tile; };
constexpr uint32_t kHashTileWords = 4096;   // 32 KiB per tile
constexpr uint32_t kNoAllocMaxBuffers = 4096;   // nixie_hash_buffers_noalloc: 128 KiB of static device memory
constexpr uint32_t kNoAllocBatch = 128;         // descriptors handed to the device per launch, as kernel arguments

}  // namespace nixie

// launchers implemented in kernels.hip (hipStream_t passed as void* to keep this header HIP-free)
extern "C++" {
int nixie_launch_swap(const nixie::SwapArgs &a, void *stream);
int nixie_launch_zero32(uint32_t *p, uint64_t n, void *stream);
int nixie_launch_hash(const nixie::HashDesc *descs, uint64_t n, uint64_t total_tiles, uint64_t *hashes,
                      void *stream);
int nixie_launch_copy16(const void *src, void *dst, uint64_t bytes, uint32_t wgs, void *stream);
int nixie_noalloc_scratch(void **out);   // this device's address of the static scratch array
int nixie_noalloc_put_descs(const nixie::HashDesc *batch, uint32_t count, uint32_t first, void *stream);
int nixie_noalloc_hash(uint32_t n, uint64_t total_tiles, uint64_t *out_d, void *stream);
}
