// Registry of reserved device address ranges ("spaces") that share physical memory ("pools").
// HIP-free, so the planner can be built and tested without a GPU.
//
// Paper, "Maintaining consistent virtual memory addresses": an application keeps its device
// addresses while the physical memory behind them changes hands.  Two spaces of one pool map
// block i of the pool at the same offset, so "do these two device ranges share memory?" is
// answered by translating both into the pool's own coordinate (a key) and comparing there.
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
    uint64_t key_base = 0;            // pool coordinate of its first byte
    uint64_t block_bytes = 0;
    std::vector<uint8_t> mapped;      // per block: 1 while physical memory is mapped there
};

// One use of a space by a plan: blocks [first, first + count) must be mapped during a switch.
struct SpaceUse { uint64_t base, first, count; };

uint64_t next_pool_key();                                      // a fresh key_base
void space_register(const SpaceSpan &s);
void space_unregister(uint64_t base);
void space_set_mapped(uint64_t base, uint64_t first, uint64_t count, bool on);

// Pool coordinate of [addr, addr + bytes): `key` = addr itself when the range touches no space.
// Returns false when the range straddles the edge of a space.  `use`, when given, receives the
// blocks the range occupies (count 0 outside spaces).
bool space_translate(uint64_t addr, uint64_t bytes, uint64_t *key, SpaceUse *use);
// True when every block of every use is mapped right now.
bool space_uses_mapped(const std::vector<SpaceUse> &uses);


// ---- pinned tier ------------------------------------------------------------------------------
// Paper, "Hierarchical Memory": a chunk lives in exactly one of GPU memory, CPU pinned memory,
// CPU pageable memory (or disk).  Host ranges registered here are pinned memory that the GPU can
// address; an allocation whose host side lies in one moves between HBM and that range directly,
// with no ring slot and no host copy.
struct TierSpan { uint64_t host_base, bytes, dev_base; };   // dev_base: the GPU's address of host_base
bool tier_register(const TierSpan &t);                       // false: overlaps a registered range
bool tier_unregister(uint64_t host_base);
// GPU address of [host_addr, host_addr + bytes) when the range lies wholly inside one registered span
bool tier_translate(uint64_t host_addr, uint64_t bytes, uint64_t *dev_addr);

// Held shared by a running switch (and by the hash kernels), exclusively by map / unmap.
std::shared_mutex &switch_lock();

}  // namespace nixie
