// Chunk planner: split, pack, order, divide the ring.  Pure host code.
//
// Paper, "Speeding Up Context Switches": a global plan decides what moves where before any
// transfer starts, and an orchestrator fixes the order under limited staging space; a window
// of the pinned tier is reserved for the evicted application so neither direction can starve
// the other.  "Granularity of Memory Management": large allocations are subdivided and moved
// in fixed-size units so that mixed tensor sizes do not fragment the staging tier.
// Here the fixed unit is the ring slot: an allocation larger than a slot becomes several
// chunks, allocations smaller than a slot share one.
#include <algorithm>
#include <cstring>
#include <numeric>
#include <thread>

#include "internal.hpp"
#include "spaces.hpp"

namespace nixie {

namespace {

// Device ranges are compared where they really live: a range inside a registered space is
// translated into the coordinate of the physical pool behind it (one piece per run of pool
// blocks), so two spaces that map the same pool are seen to share memory although their
// addresses differ.  Ranges were validated when the table was copied.
const std::vector<KeyPiece> &dev_pieces(uint64_t addr, uint64_t len, std::vector<KeyPiece> &scratch) {
    scratch.clear();
    space_translate(addr, len, &scratch, nullptr);
    return scratch;
}

constexpr uint64_t kDefaultSlot = 2ull << 20;
constexpr uint64_t kMinAutoSlot = 64ull << 10;
constexpr uint64_t kMaxSlot = 1ull << 30;

struct Range { uint64_t lo, hi; };

// r holds the ranges of the outgoing table in [0, mid) and of the incoming table in [mid, end).
// Allocation tables usually come in address order, so try a linear merge before a full sort.
bool any_overlap(std::vector<Range> &r, size_t mid) {
    auto less = [](const Range &a, const Range &b) { return a.lo < b.lo; };
    if (std::is_sorted(r.begin(), r.begin() + (ptrdiff_t)mid, less) && std::is_sorted(r.begin() + (ptrdiff_t)mid, r.end(), less))
        std::inplace_merge(r.begin(), r.begin() + (ptrdiff_t)mid, r.end(), less);
    else
        std::sort(r.begin(), r.end(), less);
    for (size_t i = 1; i < r.size(); i++)
        if (r[i].lo < r[i - 1].hi) return true;
    return false;
}

int copy_table(const nixie_table_t *t, std::vector<nixie_alloc_t> &dst) {
    dst.clear();
    if (!t || t->count == 0) return NIXIE_OK;
    if (!t->allocs) return NIXIE_EINVAL;
    dst.assign(t->allocs, t->allocs + t->count);
    for (const auto &a : dst) {
        if (a.bytes == 0) continue;
        if (!a.dev_ptr || !a.host_ptr) return NIXIE_EINVAL;
        uint64_t d = (uint64_t)(uintptr_t)a.dev_ptr, h = (uint64_t)(uintptr_t)a.host_ptr;
        if (d + a.bytes < d || h + a.bytes < h) return NIXIE_EINVAL;  // wraps the address space
    }
    return NIXIE_OK;
}

// In-place switch.  osegs: outgoing segments sorted by device address (they are disjoint), with the
// chunk each belongs to.  Returns 1 + the highest outgoing chunk index that covers a byte of
// [a, b), or 0: that many leading outgoing chunks must have left HBM before [a, b) is written.
struct OutSpan { uint64_t lo, hi, chunk; };
uint64_t dep_of_range(const std::vector<OutSpan> &osegs, uint64_t a, uint64_t b) {
    if (a >= b) return 0;
    auto it = std::upper_bound(osegs.begin(), osegs.end(), a, [](uint64_t v, const OutSpan &s) { return v < s.hi; });
    uint64_t dep = 0;
    for (; it != osegs.end() && it->lo < b; ++it) dep = std::max(dep, it->chunk + 1);
    return dep;
}

uint64_t dep_of_pieces(const std::vector<OutSpan> &osegs, const std::vector<KeyPiece> &pieces) {
    uint64_t dep = 0;
    for (const KeyPiece &p : pieces) dep = std::max(dep, dep_of_range(osegs, p.key, p.key + p.len));
    return dep;
}

std::vector<uint64_t> walk_order(const std::vector<nixie_alloc_t> &t, uint32_t order) {
    std::vector<uint64_t> idx(t.size());
    std::iota(idx.begin(), idx.end(), 0);
    switch (order) {
    case NIXIE_ORDER_LARGE_FIRST:
        std::stable_sort(idx.begin(), idx.end(), [&](uint64_t a, uint64_t b) { return t[a].bytes > t[b].bytes; });
        break;
    case NIXIE_ORDER_ADDRESS:
        std::stable_sort(idx.begin(), idx.end(), [&](uint64_t a, uint64_t b) {
            return (uintptr_t)t[a].dev_ptr < (uintptr_t)t[b].dev_ptr;
        });
        break;
    case NIXIE_ORDER_REVERSE:
        std::reverse(idx.begin(), idx.end());
        break;
    default:
        break;
    }
    return idx;
}

// Greedy sequential packing.  A segment's slot offset is congruent to its device address
// modulo 16, so the 16-byte lanes of the copy kernels are aligned on both sides at once.
// direct[i] != 0: allocation i lives in the pinned tier on the host side and is cut by cut_direct.
void cut(const std::vector<nixie_alloc_t> &t, const std::vector<uint64_t> &walk, const std::vector<uint64_t> &direct,
         uint64_t S, DirLayout &D) {
    D.segs.clear();
    D.chunks.clear();
    D.direct_base.clear();
    D.bytes = D.direct_bytes = 0;
    uint64_t total = 0;
    for (const auto &a : t) total += a.bytes;
    D.segs.reserve(t.size() + total / S + 8);     // every allocation once, plus one cut per slot boundary
    D.chunks.reserve(total / (S - 16) + 8);       // at most 15 padding bytes per segment start
    uint64_t fill = 0;
    bool open = false;
    for (uint64_t i : walk) {
        if (direct[i]) continue;
        const nixie_alloc_t &a = t[i];
        uint64_t off = 0;
        while (off < a.bytes) {
            uint64_t dev = (uint64_t)(uintptr_t)a.dev_ptr + off;
            uint64_t pos = open ? fill + ((dev - fill) & 15) : S;
            if (!open || pos >= S) {
                D.chunks.push_back(nixie_chunk_t{(uint64_t)D.segs.size(), 0, 0, 0});
                open = true;
                pos = dev & 15;
            }
            uint64_t take = std::min(S - pos, a.bytes - off);
            D.segs.push_back(nixie_segment_t{dev, (uint64_t)(uintptr_t)a.host_ptr + off, (uint32_t)pos, (uint32_t)take});
            nixie_chunk_t &c = D.chunks.back();
            c.seg_count++;
            c.used_bytes = (uint32_t)(pos + take);
            fill = pos + take;
            off += take;
            D.bytes += take;
        }
    }
    D.staged = D.chunks.size();
    // Pinned tier: nothing to pack, the bytes go where they already have a place.  One chunk per
    // slot-sized piece, one segment each; the piece's image starts at the same offset modulo 16
    // as on the device, like a segment in a ring slot.
    for (uint64_t i : walk) {
        if (!direct[i]) continue;
        const nixie_alloc_t &a = t[i];
        uint64_t off = 0;
        while (off < a.bytes) {
            const uint64_t dev = (uint64_t)(uintptr_t)a.dev_ptr + off, pos = dev & 15;
            const uint64_t take = std::min(S - pos, a.bytes - off);
            D.chunks.push_back(nixie_chunk_t{(uint64_t)D.segs.size(), 1, (uint32_t)(pos + take), 0});
            D.segs.push_back(nixie_segment_t{dev, (uint64_t)(uintptr_t)a.host_ptr + off, (uint32_t)pos, (uint32_t)take});
            D.direct_base.push_back(direct[i] + off - pos);
            off += take;
            D.bytes += take;
            D.direct_bytes += take;
        }
    }
}

}  // namespace

int build_layout(const nixie_table_t *out_table, const nixie_table_t *in_table, uint64_t ring_bytes,
                 const nixie_opts_t *opts, Layout &L) {
    L = Layout{};
    if (opts) L.opts = *opts;
    if (L.opts.order > NIXIE_ORDER_REVERSE) return NIXIE_EINVAL;
    int rc = copy_table(out_table, L.table[0]);
    if (rc) return rc;
    rc = copy_table(in_table, L.table[1]);
    if (rc) return rc;

    // no aliasing: device ranges pairwise disjoint across both tables, host ranges likewise
    std::vector<Range> dev, host;
    std::vector<uint64_t> direct[2];      // per allocation: its GPU-visible pinned-tier address, or 0
    uint64_t tot[2] = {0, 0}, staged_tot[2] = {0, 0};
    const bool use_tier = !(L.opts.flags & NIXIE_NO_DIRECT);
    size_t mid = 0, mid_host = 0;
    std::vector<KeyPiece> pieces;
    dev.reserve(L.table[0].size() + L.table[1].size());
    host.reserve(L.table[0].size() + L.table[1].size());
    uint64_t n_spaces = 0, n_tier_spans = 0;   // with neither, an address is just an address: no lookups
    registry_counts(&n_spaces, &n_tier_spans);
    for (int x = 0; x < 2; x++) {
        if (x == 1) { mid = dev.size(); mid_host = host.size(); }
        direct[x].assign(L.table[x].size(), 0);
        for (size_t i = 0; i < L.table[x].size(); i++) {
            const nixie_alloc_t &a = L.table[x][i];
            if (a.bytes == 0) continue;
            uint64_t d = (uint64_t)(uintptr_t)a.dev_ptr, h = (uint64_t)(uintptr_t)a.host_ptr;
            if (n_spaces) {
                pieces.clear();
                if (!space_translate(d, a.bytes, &pieces, &L.uses[x])) return NIXIE_EINVAL;   // straddles the edge of a space
                for (const KeyPiece &p : pieces) dev.push_back({p.key, p.key + p.len});
            } else {
                dev.push_back({d, d + a.bytes});
            }
            host.push_back({h, h + a.bytes});
            tot[x] += a.bytes;
            uint64_t seen_by_gpu = 0, span_id = 0;
            if (use_tier && n_tier_spans && tier_translate(h, a.bytes, &seen_by_gpu, &span_id) && ((seen_by_gpu ^ d) & 15) == 0) {
                direct[x][i] = seen_by_gpu;
                if (L.tier_ids.empty() || L.tier_ids.back() != span_id) L.tier_ids.push_back(span_id);
            } else staged_tot[x] += a.bytes;
        }
    }
    const bool in_place = (L.opts.flags & NIXIE_IN_PLACE) != 0;
    if (in_place) {   // device ranges may overlap across the tables, not inside one
        std::vector<Range> d0(dev.begin(), dev.begin() + (ptrdiff_t)mid), d1(dev.begin() + (ptrdiff_t)mid, dev.end());
        if (any_overlap(d0, d0.size()) || any_overlap(d1, d1.size())) return NIXIE_EOVERLAP;
    } else if (any_overlap(dev, mid)) {
        return NIXIE_EOVERLAP;
    }
    if (any_overlap(host, mid_host)) return NIXIE_EOVERLAP;
    std::sort(L.tier_ids.begin(), L.tier_ids.end());
    L.tier_ids.erase(std::unique(L.tier_ids.begin(), L.tier_ids.end()), L.tier_ids.end());
    for (int x = 0; x < 2; x++) {   // one entry per block of a space that the table touches
        std::sort(L.uses[x].begin(), L.uses[x].end());
        L.uses[x].erase(std::unique(L.uses[x].begin(), L.uses[x].end()), L.uses[x].end());
    }

    // only what goes through the ring counts for the ring's geometry
    const int active = (staged_tot[0] > 0) + (staged_tot[1] > 0);
    uint64_t S = L.opts.slot_bytes;
    if (S == 0 && active == 0) {
        S = kDefaultSlot;        // no ring: the slot size only sets the size of a direct chunk
    } else if (S == 0) {
        // About 128 slots per active direction, between 64 KiB and 2 MiB.  Slots are a free pool,
        // so what counts is how finely the ring is recycled: on a 64 MiB ring 2 MiB slots lose
        // 15 % against 256 KiB slots, on a 16 MiB ring 256 KiB slots lose 20 % against 64 KiB ones,
        // while beyond ~128 slots per direction nothing more is gained.
        S = kDefaultSlot;
        while (S > kMinAutoSlot && ring_bytes / S < 128ull * (uint64_t)std::max(active, 1)) S >>= 1;
    } else if (S % 4096 != 0 || S > kMaxSlot) {
        return NIXIE_EINVAL;
    }
    const uint64_t n_slots = ring_bytes / S;
    if (n_slots < 2ull * (uint64_t)active || n_slots > (1ull << 20)) return NIXIE_EINVAL;   // no ring needed when nothing is staged

    uint64_t n_out;
    if (staged_tot[0] == 0) n_out = 0;
    else if (staged_tot[1] == 0) n_out = n_slots;
    else if (L.opts.out_slots) {
        // both directions are staged: each needs two slots, and the caller's share for the outgoing
        // one must leave them (checked before any subtraction: these are unsigned counts)
        if ((uint64_t)L.opts.out_slots < 2 || (uint64_t)L.opts.out_slots + 2 > n_slots) return NIXIE_EINVAL;
        n_out = L.opts.out_slots;
    }
    else if (L.opts.flags & NIXIE_SPLIT_BY_BYTES) {
        long double f = (long double)staged_tot[0] / (long double)(staged_tot[0] + staged_tot[1]);
        n_out = (uint64_t)(f * (long double)n_slots + 0.5L);
        n_out = std::min(std::max<uint64_t>(n_out, 2), n_slots - 2);
    } else n_out = n_slots / 2;
    if (staged_tot[0] && staged_tot[1] && (n_out < 2 || n_slots - n_out < 2)) return NIXIE_EINVAL;

    L.ring_bytes = ring_bytes;
    L.slot_bytes = S;
    L.dir[0].slots = (uint32_t)n_out;
    L.dir[1].slots = (uint32_t)(staged_tot[1] ? n_slots - n_out : 0);
    std::vector<uint64_t> walk0 = walk_order(L.table[0], L.opts.order);
    std::vector<uint64_t> walk1 = walk_order(L.table[1], L.opts.order);
    if (in_place && tot[0] && tot[1]) {
        // The incoming application is ready when its last chunk is in HBM, and a chunk can only be written
        // where the old bytes have left: the outgoing allocations whose GPU memory the incoming table reuses
        // are walked first (in the given order among themselves), so that what the incoming side waits for
        // is a short prefix of the eviction and not, at worst, all of it.
        {
            std::vector<Range> in_pieces;
            for (const nixie_alloc_t &a : L.table[1])
                for (const KeyPiece &q : dev_pieces((uint64_t)(uintptr_t)a.dev_ptr, a.bytes, pieces))
                    in_pieces.push_back({q.key, q.key + q.len});
            std::sort(in_pieces.begin(), in_pieces.end(), [](const Range &a, const Range &b) { return a.lo < b.lo; });
            // (incoming ranges are pairwise disjoint, so sorted by lo they are sorted by hi as well)
            auto reused = [&](uint64_t i) {
                const nixie_alloc_t &a = L.table[0][i];
                for (const KeyPiece &q : dev_pieces((uint64_t)(uintptr_t)a.dev_ptr, a.bytes, pieces)) {
                    auto it = std::upper_bound(in_pieces.begin(), in_pieces.end(), q.key,
                                               [](uint64_t v, const Range &r) { return v < r.hi; });
                    if (it != in_pieces.end() && it->lo < q.key + q.len) return true;
                }
                return false;
            };
            std::stable_partition(walk0.begin(), walk0.end(), reused);
        }
        cut(L.table[0], walk0, direct[0], S, L.dir[0]);
        std::vector<OutSpan> osegs;
        osegs.reserve(L.dir[0].segs.size());
        for (uint64_t k = 0; k < L.dir[0].chunks.size(); k++) {
            const nixie_chunk_t &c = L.dir[0].chunks[k];
            for (uint64_t q = c.seg_begin; q < c.seg_begin + c.seg_count; q++)
                for (const KeyPiece &p : dev_pieces(L.dir[0].segs[q].dev_addr, L.dir[0].segs[q].len, pieces))
                    osegs.push_back({p.key, p.key + p.len, k});
        }
        std::sort(osegs.begin(), osegs.end(), [](const OutSpan &a, const OutSpan &b) { return a.lo < b.lo; });
        // Walk the incoming table in the order in which its GPU memory becomes free, so that the
        // scatter side follows right behind the gather side instead of waiting for its end.
        std::vector<uint64_t> adep(L.table[1].size());
        for (size_t i = 0; i < adep.size(); i++) {
            adep[i] = dep_of_pieces(osegs, dev_pieces((uint64_t)(uintptr_t)L.table[1][i].dev_ptr, L.table[1][i].bytes, pieces));
        }
        std::stable_sort(walk1.begin(), walk1.end(), [&](uint64_t a, uint64_t b) { return adep[a] < adep[b]; });
        cut(L.table[1], walk1, direct[1], S, L.dir[1]);
        for (nixie_chunk_t &c : L.dir[1].chunks)
            for (uint64_t q = c.seg_begin; q < c.seg_begin + c.seg_count; q++) {
                const nixie_segment_t &sg = L.dir[1].segs[q];
                c.dep_out = std::max(c.dep_out, dep_of_pieces(osegs, dev_pieces(sg.dev_addr, sg.len, pieces)));
            }
    } else if (L.table[0].size() + L.table[1].size() > 20000 || (tot[0] + tot[1]) / S > 50000) {
        // many allocations or many chunks: one direction per thread
        std::thread other([&] { cut(L.table[1], walk1, direct[1], S, L.dir[1]); });
        cut(L.table[0], walk0, direct[0], S, L.dir[0]);
        other.join();
    } else {
        cut(L.table[0], walk0, direct[0], S, L.dir[0]);
        cut(L.table[1], walk1, direct[1], S, L.dir[1]);
    }
    if (L.dir[0].chunks.size() > 0xFFFFFFF0ull / 256 || L.dir[1].chunks.size() > 0xFFFFFFF0ull / 256 ||
        L.dir[0].segs.size() > 0xFFFFFFF0ull || L.dir[1].segs.size() > 0xFFFFFFF0ull)
        return NIXIE_EINVAL;
    return NIXIE_OK;
}

}  // namespace nixie

namespace nixie {

// Launch shape and thread counts the runtime will use for this layout (options override).
void fill_info(const Layout &L, nixie_plan_info_t *info) {
    std::memset(info, 0, sizeof(*info));
    info->ring_bytes = L.ring_bytes;
    info->slot_bytes = L.slot_bytes;
    info->out_slots = L.dir[0].slots;
    info->in_slots = L.dir[1].slots;
    info->chunks_out = L.dir[0].chunks.size();
    info->chunks_in = L.dir[1].chunks.size();
    info->segments_out = L.dir[0].segs.size();
    info->segments_in = L.dir[1].segs.size();
    info->bytes_out = L.dir[0].bytes;
    info->bytes_in = L.dir[1].bytes;
    info->direct_chunks_out = L.dir[0].chunks.size() - L.dir[0].staged;
    info->direct_chunks_in = L.dir[1].chunks.size() - L.dir[1].staged;
    info->direct_bytes_out = L.dir[0].direct_bytes;
    info->direct_bytes_in = L.dir[1].direct_bytes;
    const uint64_t all_slots = (uint64_t)L.dir[0].slots + (uint64_t)L.dir[1].slots;   // 64-bit: no wrap
    info->pinned_ring_bytes = all_slots * L.slot_bytes;
    info->pinned_ctrl_bytes = (wait_flag_words(L.dir[0].slots) + wait_flag_words(L.dir[1].slots) +
                               (all_slots + 3) * kFlagStride) * 8;
    // Measured on MI355X with both directions active: write-through stores into the ring need
    // about twice the workgroups that the reads out of it need; 128 + 64 balance the two directions for
    // slots up to 512 KiB, and larger slots are within 2 % of their best (144 + 64).
    uint32_t wgs[2] = {L.opts.gather_wgs ? L.opts.gather_wgs : 128u, L.opts.scatter_wgs ? L.opts.scatter_wgs : 64u};
    // Work unit: at most 64 KiB of a slot -- per unit a workgroup pays a ticket, a slot lookup, a
    // store drain and a barrier, while with large units a chunk waits too long for its slowest one
    // (config 2, ms per switch by unit size: 512 KiB 467, 256 KiB 418, 128 KiB 381, 64 KiB 380,
    // 32 KiB 398) -- and small enough that the units in flight (one per
    // workgroup) occupy no more than a quarter of the direction's share of the ring (where the unit floor allows): the rest is
    // what the host threads drain or fill meanwhile.
    // (a team of more than 256 could not be counted by the chunk limits checked in build_layout)
    uint32_t team[2];
    for (int x = 0; x < 2; x++) {
        team[x] = L.opts.team;
        if (team[x] == 0) {
            // Never below one tile per wave: a smaller unit would leave waves, or whole units, without a
            // tile while still paying for the unit.
            const uint64_t floor_unit = (uint64_t)(kWgThreads / 64) * kTileBytesDir[x];
            uint64_t unit = 64u << 10;
            while (L.dir[x].slots && unit > floor_unit && unit * 4 * wgs[x] > (uint64_t)L.dir[x].slots * L.slot_bytes) unit >>= 1;
            team[x] = (uint32_t)std::max<uint64_t>(1, L.slot_bytes / std::max(unit, floor_unit));
        }
        team[x] = std::min(team[x], 256u);
    }
    // Small rings: every workgroup holds one unit's worth of a slot while the link works it off, and the
    // flag that hands a finished chunk to the host queues behind whatever the other workgroups have in
    // flight.  Measured with a 16 MiB ring (8 MiB per direction), 128 + 64 workgroups wait for slots
    // (570 ms for 24 + 24 GiB) where 48 + 24 to 80 + 40 do not (554 - 560 ms); with a 4 MiB ring 32 + 16
    // are best and 16 + 8 starve the incoming direction; from 16 MiB per direction on, 128 + 64 are best.
    // Default: one gather workgroup per 128 KiB of the outgoing share, between 32 and 128; half as many
    // scatter workgroups.
    if (L.opts.gather_wgs == 0 && L.opts.scatter_wgs == 0 && L.dir[0].slots && L.dir[1].slots) {
        const uint64_t share = (uint64_t)std::min(L.dir[0].slots, L.dir[1].slots) * L.slot_bytes;
        wgs[0] = (uint32_t)std::min<uint64_t>(128, std::max<uint64_t>(32, share >> 17));
        wgs[1] = wgs[0] / 2;
    }
    // Host threads busy-poll their slots, so the default never takes more than half the cores for
    // the two directions together (4 + 4 on the 16-core boxes measured; 3 + 3 already saturate the link).
    const uint32_t cores = std::max(1u, std::thread::hardware_concurrency());
    const uint32_t dflt = std::max(1u, std::min(4u, cores / 4));
    uint32_t thr[2] = {L.opts.drain_threads ? L.opts.drain_threads : dflt, L.opts.fill_threads ? L.opts.fill_threads : dflt};
    for (int x = 0; x < 2; x++) {
        if (L.dir[x].chunks.empty()) { wgs[x] = 0; thr[x] = 0; continue; }
        // more workgroups than slots * team could only spin on credits (direct chunks need none)
        uint64_t cap = L.dir[x].staged == L.dir[x].chunks.size() ? (uint64_t)L.dir[x].slots * team[x] : ~0ull;
        wgs[x] = (uint32_t)std::max<uint64_t>(1, std::min<uint64_t>(wgs[x], cap));
        wgs[x] = std::min(wgs[x], 1024u);
        // no host thread where nothing goes through the ring
        thr[x] = L.dir[x].staged ? std::min(std::min(thr[x], 64u), std::max(1u, L.dir[x].slots)) : 0;
    }
    info->gather_wgs = wgs[0];
    info->scatter_wgs = wgs[1];
    // Workgroups that serve either direction only make sense where both directions run in one launch.
    // Measured: with 128 + 64 fixed workgroups the incoming direction of two equal sets finishes 5 % ahead of
    // the outgoing one (more with large slots, less or the other way round with small ones); 16 workgroups
    // that go where more is left make both finish together and shorten the switch by 1.5 - 2.5 % on every
    // configuration; beyond 32 they only wait for slots.  Default: an eighth of the gather workgroups.
    uint32_t flex = (L.opts.flags & (NIXIE_NO_FLEX_WGS | NIXIE_SERIALIZE)) ? 0
                    : L.opts.flex_wgs ? L.opts.flex_wgs : std::max(4u, wgs[0] / 8);
    if (wgs[0] == 0 || wgs[1] == 0) flex = 0;
    info->flex_wgs = std::min(flex, 256u);
    info->team_out = L.dir[0].chunks.empty() ? 0 : team[0];
    info->team_in = L.dir[1].chunks.empty() ? 0 : team[1];
    info->drain_threads = thr[0];
    info->fill_threads = thr[1];
}

}  // namespace nixie
