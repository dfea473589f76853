// Registry of reserved device address ranges ("spaces") that share physical memory ("pools").
// HIP-free, so the planner can be built and tested without a GPU.
//
// Paper, "Maintaining consistent virtual memory addresses": an application keeps its device
// addresses while the physical memory behind them changes hands.  Every block of a space is
// ASSIGNED one block of the pool (which physical block backs it whenever it is mapped; block i
// by default) and is MAPPED or not.  "Do these two device ranges share memory?" is answered by
// translating both into the pool's own coordinate (a key: pool, pool block, offset in the
// block) and comparing there; a range that spans several blocks becomes several pieces.
#pragma once
#include <cstdint>
#include <shared_mutex>
#include <vector>

namespace nixie {

// Keys of pool memory lie above every user-space address, 2^44 bytes apart per pool.
constexpr uint64_t kKeyOrigin = 1ull << 62;
constexpr uint64_t kKeyStride = 1ull << 44;

struct SpaceSpan {
    uint64_t base = 0, bytes = 0;     // the reserved device address range
    uint64_t key_base = 0;            // pool coordinate of the pool's first byte
    uint64_t block_bytes = 0;
    std::vector<uint64_t> assigned;   // per block: the pool block that backs it
    std::vector<uint8_t> mapped;      // per block: 1 while that pool block is mapped there
};

// One block of a space as a plan saw it: a switch needs it mapped, and backed by the same pool
// block as when the dependencies were computed.
struct SpaceUse {
    uint64_t base, index, pool_block;
    bool operator<(const SpaceUse &o) const { return base != o.base ? base < o.base : index < o.index; }
    bool operator==(const SpaceUse &o) const { return base == o.base && index == o.index && pool_block == o.pool_block; }
};

// A run of bytes in pool coordinates (or plain addresses, outside every space).
struct KeyPiece { uint64_t key, len; };

uint64_t next_pool_key();                                      // a fresh key_base
void space_register(const SpaceSpan &s);
void space_unregister(uint64_t base);
void space_set_mapped(uint64_t base, uint64_t first, uint64_t count, bool on);
// false if the space is unknown, a block is out of range, or a block to be reassigned is mapped
bool space_assign(uint64_t base, uint64_t first, const uint64_t *pool_blocks, uint64_t count);

// Pool coordinates of [addr, addr + bytes), appended to pieces (pieces with adjacent keys are
// merged; one piece {addr, bytes} when the range touches no space).  Returns false when the
// range straddles the edge of a space.  uses, when given, receives the blocks the range occupies.
bool space_translate(uint64_t addr, uint64_t bytes, std::vector<KeyPiece> *pieces, std::vector<SpaceUse> *uses);
// The same question without building anything (no heap use): 0 = the range touches no space or lies
// in mapped blocks of one, 1 = it touches an unmapped block, 2 = it straddles the edge of a space.
int space_range_state(uint64_t addr, uint64_t bytes);
// True when every block is mapped right now and backed by the pool block recorded in its use.
bool space_uses_valid(const std::vector<SpaceUse> &uses);


// ---- pinned tier ------------------------------------------------------------------------------
// Paper, "Hierarchical Memory": a chunk lives in exactly one of GPU memory, CPU pinned memory,
// CPU pageable memory (or disk).  Host ranges registered here are pinned memory that the GPU can
// address; an allocation whose host side lies in one moves between HBM and that range directly,
// with no ring slot and no host copy.
struct TierSpan { uint64_t host_base, bytes, dev_base; };   // dev_base: the GPU's address of host_base
bool tier_register(const TierSpan &t);                       // false: overlaps a registered range
// A plan with direct chunks holds raw GPU addresses of the span, so a span stays registered (and
// the caller keeps its memory allocated) while such a plan lives.  Every registration has an id
// of its own; a plan acquires the ids its layout recorded and releases them when it is destroyed.
enum TierDrop { kTierDropped = 0, kTierUnknown = 1, kTierInUse = 2 };
TierDrop tier_unregister(uint64_t host_base);
// GPU address of [host_addr, host_addr + bytes) when the range lies wholly inside one registered
// span; span_id, when given, receives the id of that registration
bool tier_translate(uint64_t host_addr, uint64_t bytes, uint64_t *dev_addr, uint64_t *span_id = nullptr);
// all or nothing: false (and nothing counted) when one of the registrations is gone
bool tier_acquire(const std::vector<uint64_t> &span_ids);
void tier_release(const std::vector<uint64_t> &span_ids);

// Number of registered spaces and of registered tier spans right now (one look under the lock, so a
// planner facing large tables can skip the per-allocation lookups when both are zero).
void registry_counts(uint64_t *spaces, uint64_t *tier_spans);

// Held shared by a running switch (and by the hash kernels), exclusively by map / unmap.
std::shared_mutex &switch_lock();

}  // namespace nixie
