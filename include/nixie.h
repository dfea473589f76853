/*
 * nixie.h -- C ABI of the MI355X context-switch swap library (libnixie.so).
 *
 * One operation: when application A yields the GPU and application B is
 * scheduled, A's working set (a table of device allocations) is evicted to
 * pageable host memory while B's working set is brought back into HBM at the
 * same time, both directions of the host link busy, through a pinned staging
 * ring of bounded size.  (Paper: "Overview" step 4 of the architecture figure;
 * "Hierarchical Memory" -- every chunk has exactly one copy and GPU-resident
 * data needs no pinned backing; "Speeding Up Context Switches" -- bidirectional
 * migration, global plan, orchestrated order, reserved window for the evicted
 * application, multi-threaded pageable<->pinned copies.)
 *
 * Conventions
 *  - Plain C types only.  Every pointer is labelled HOST or DEVICE below.
 *  - All functions return 0 (NIXIE_OK) or a negative nixie_err code; nothing
 *    throws or aborts across this boundary; outputs are untouched on failure
 *    unless stated.
 *  - The library never allocates device memory for payload.  It owns the pinned
 *    ring, a small pinned control block, descriptor arrays and its host threads.
 *  - A plan is bound to the HIP device that is current when it is created.
 */
#ifndef NIXIE_H
#define NIXIE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum nixie_err {
    NIXIE_OK = 0,
    NIXIE_EINVAL = -1,    /* NULL where data is required, bad ring / slot geometry, bad option */
    NIXIE_EOVERLAP = -2,  /* two listed ranges intersect (device side or host side)           */
    NIXIE_ENOMEM = -3,    /* pinned / descriptor allocation failed; the budget is never exceeded silently */
    NIXIE_EHIP = -4,      /* a HIP runtime call failed; see nixie_last_hip_error()             */
    NIXIE_ETIMEOUT = -5,  /* a credit wait exceeded its bound; the kernel was told to stop     */
    NIXIE_EMISMATCH = -6, /* nixie_verify found a hash that differs                            */
    NIXIE_EBUSY = -7,     /* the plan is already running a switch; the pool still has spaces   */
    NIXIE_EUNMAPPED = -8  /* a listed device range lies in a space whose blocks are not mapped */
};

/* One allocation of a working set.  Memory is caller-owned on both sides.
 * dev_ptr:  DEVICE address of the allocation (any alignment).
 * host_ptr: HOST address of its pageable backing (any alignment, >= bytes long).  For an outgoing
 *           allocation the range is written by the host threads inside the switch: memory that has
 *           never been touched costs a page fault and a zeroed page per 4 KiB there (measured: three
 *           times the transfer itself), so keep backing memory from one eviction to the next, or
 *           touch it beforehand.
 * bytes:    length; 0 is legal and the entry is skipped. */
typedef struct {
    void *dev_ptr;
    void *host_ptr;
    uint64_t bytes;
} nixie_alloc_t;

/* HOST array of count entries, borrowed for the duration of the call and copied. */
typedef struct {
    const nixie_alloc_t *allocs;
    uint64_t count;
} nixie_table_t;

/* Order in which the planner walks a table (paper, "Speeding Up Context
 * Switches": the orchestrator manages migration order).  The result of a switch
 * does not depend on it. */
enum nixie_order {
    NIXIE_ORDER_TABLE = 0,       /* as listed                           */
    NIXIE_ORDER_LARGE_FIRST = 1, /* by size, descending                 */
    NIXIE_ORDER_ADDRESS = 2,     /* by device address, ascending        */
    NIXIE_ORDER_REVERSE = 3      /* as listed, backwards                */
};

enum nixie_flags {
    NIXIE_SPLIT_BY_BYTES = 1u << 0,   /* divide the ring's slots between the directions by byte ratio, not 50/50 */
    NIXIE_SERIALIZE = 1u << 1,        /* self-baseline: evict completely, then restore (one link direction at a time) */
    NIXIE_DIAG_RING_ONLY = 1u << 2,   /* measurement only: host threads recycle credits without touching pageable
                                         memory, so destinations on the host side are NOT written */
    NIXIE_DIAG_STALL_DRAIN = 1u << 3, /* failure-path test: drain threads never return credits, so the switch must
                                         end with NIXIE_ETIMEOUT after timeout_ms */
    NIXIE_HOST_PLAIN_MEMCPY = 1u << 4,/* host threads use libc memcpy instead of streaming stores */
    NIXIE_IN_PLACE = 1u << 5,         /* in-place switch: device ranges of the incoming table may overlap device ranges
                                         of the outgoing table (the incoming application reuses the GPU memory the
                                         outgoing one gives up; paper, "Maintaining consistent virtual memory
                                         addresses").  A chunk is scattered only after every outgoing chunk that
                                         covers GPU bytes it overwrites has left HBM.  Ranges inside one table must
                                         still be disjoint, and so must all host ranges.  The outgoing allocations
                                         whose GPU memory the incoming table reuses are evicted first (among
                                         themselves, and the others after them, in the order asked for), so that the
                                         incoming application is ready as early as its own size allows. */
    NIXIE_HOST_SPIN = 1u << 7,        /* host threads with nothing to do spin.  By default they sleep for 1/16 of the time
                                         their direction's share of the ring lasts at link rate (at most 50 us, never
                                         when that is under 4 us): same latency, less than half the CPU time */
    NIXIE_NO_DIRECT = 1u << 6,        /* measurement: allocations whose host side lies in the registered pinned tier
                                         go through the ring and the host threads like all others */
    NIXIE_NO_FLEX_WGS = 1u << 8       /* every workgroup has a fixed direction (flex_wgs = 0 means "default") */
};

/* Every field 0 = library default. */
typedef struct {
    uint64_t slot_bytes;     /* ring slot size; multiple of 4096, <= 1 GiB.  Default 2 MiB, halved until each
                                active direction has about 128 slots (never below 64 KiB)                  */
    uint32_t out_slots;      /* slots reserved for the outgoing direction (the evicted application's
                                streaming window); default half, or all when the other table is empty      */
    uint32_t order;          /* enum nixie_order                                                            */
    uint32_t gather_wgs;     /* workgroups copying HBM -> ring                                              */
    uint32_t scatter_wgs;    /* workgroups copying ring -> HBM                                              */
    uint32_t team;           /* workgroups that share one chunk; default one per 16-64 KiB of slot, at most 256  */
    uint32_t drain_threads;  /* host threads moving ring -> pageable; default min(4, cores / 4), at least 1   */
    uint32_t fill_threads;   /* host threads moving pageable -> ring; same default                           */
    uint32_t timeout_ms;     /* bound on any single credit wait, host or GPU side; default 30000.  It is a
                                bound on time without progress, not on the length of a switch: a caller waiting
                                for a whole direction gives up only after this long with no chunk claimed,
                                delivered or handed out.  Until the kernel is seen running (it may be queued
                                behind earlier work on the stream) host threads allow four times as long     */
    uint32_t flags;          /* enum nixie_flags                                                            */
    uint32_t xcd_mask;       /* tuning: bit i set = workgroups that land on XCD i take part, the others leave at
                                once (workgroups are dealt round-robin over the 8 XCDs, so raise gather_wgs /
                                scatter_wgs accordingly); 0 = all XCDs                                       */
    uint32_t flex_wgs;       /* workgroups on top of gather_wgs + scatter_wgs that serve either direction: before
                                every work unit they take the direction with more chunks left, so that two
                                working sets of equal size finish together; NIXIE_NO_FLEX_WGS in flags = none */
} nixie_opts_t;

typedef struct nixie_plan nixie_plan_t;     /* opaque; owns ring, flags, descriptors, host threads */
typedef struct nixie_layout nixie_layout_t; /* opaque; the planner's output alone, host memory only */

/* What the planner decided; also the pinned-memory account. */
typedef struct {
    uint64_t ring_bytes;        /* as requested                                    */
    uint64_t slot_bytes;
    uint32_t out_slots, in_slots;
    uint64_t chunks_out, chunks_in;
    uint64_t segments_out, segments_in;
    uint64_t bytes_out, bytes_in;
    uint64_t pinned_ring_bytes; /* payload slots actually allocated, <= ring_bytes  */
    uint64_t pinned_ctrl_bytes; /* flag block, reported separately                  */
    uint32_t gather_wgs, scatter_wgs, team_out, team_in;
    uint32_t drain_threads, fill_threads;
    uint64_t direct_chunks_out, direct_chunks_in; /* chunks that move between HBM and the pinned tier  */
    uint64_t direct_bytes_out, direct_bytes_in;   /* directly: the last of chunks_* / part of bytes_*  */
    uint32_t flex_wgs;                            /* workgroups that serve either direction            */
} nixie_plan_info_t;

/* One contiguous piece of one allocation inside one chunk. */
typedef struct {
    uint64_t dev_addr;   /* DEVICE address of the piece                     */
    uint64_t host_addr;  /* HOST address of the piece                       */
    uint32_t slot_off;   /* offset inside the ring slot; == dev_addr mod 16 */
    uint32_t len;
} nixie_segment_t;

/* One ring-slot's worth of work: segments [seg_begin, seg_begin + seg_count).  The chunks of a
 * direction that go through the ring come first; direct chunks (pinned tier) follow, one segment
 * each, and use no slot. */
typedef struct {
    uint64_t seg_begin;
    uint32_t seg_count;
    uint32_t used_bytes; /* extent of the slot image, <= slot_bytes */
    uint64_t dep_out;    /* incoming chunks of an in-place switch: number of leading outgoing chunks that must
                            have left HBM before this chunk may be written there; otherwise 0 */
} nixie_chunk_t;

/* Timers and counters of one switch.  Times are nanoseconds since nixie_switch was entered. */
typedef struct {
    uint64_t bytes_out, bytes_in;
    uint64_t ns_total;        /* entry -> return: kernel done and last drain in pageable memory */
    uint64_t ns_out_done;     /* entry -> last outgoing byte written to pageable memory         */
    uint64_t ns_in_done;      /* entry -> last incoming byte written to HBM ("B ready")         */
    uint64_t ns_kernel;       /* duration of the swap kernel(s) by HIP events                   */
    uint64_t ns_launch;       /* entry -> kernel launch call returned                           */
    uint64_t drain_wait_ns;   /* summed over drain threads: time waiting for ready flags        */
    uint64_t fill_wait_ns;    /* summed over fill threads: time waiting for free flags          */
    uint64_t gather_stall_ticks;  /* summed over gather workgroups, 100 MHz ticks waiting for credits */
    uint64_t scatter_stall_ticks; /* summed over scatter workgroups, ticks waiting for filled slots   */
    uint32_t kernels;         /* swap kernels launched (2 when serialised)                      */
    uint32_t gpu_status;      /* 0, or the reason the kernel stopped early                      */
    uint32_t pump_rounds_out, pump_rounds_in; /* times the kernel read the host's flags of a direction: kernel
                                 time / rounds = how stale a credit can be when the GPU sees it  */
    uint32_t credit_rtt_ticks_out, credit_rtt_ticks_in; /* mean credit round trip of the last kernel, 100 MHz ticks:
                                 from the GPU's flag for a slot (outgoing: "slot holds a chunk", incoming: "slot
                                 is free") to the kernel seeing the host's answer for that slot                 */
} nixie_stats_t;

typedef struct {
    uint64_t checked_out, checked_in;
    uint64_t mismatched_out, mismatched_in;
    int64_t first_bad_out, first_bad_in; /* table index, -1 if none */
} nixie_verify_report_t;

/* Host-link rates measured on this machine, GB/s (1e9 B/s) per direction.  d2h = GPU to host. */
typedef struct {
    double sdma_d2h, sdma_h2d;             /* hipMemcpyAsync, one direction at a time  */
    double sdma_d2h_both, sdma_h2d_both;   /* hipMemcpyAsync, both at once             */
    double kernel_d2h, kernel_h2d;         /* plain 16 B/lane copy kernel, one at a time */
    double kernel_d2h_both, kernel_h2d_both;
} nixie_link_peak_t;

/* ---- planner (paper, "Speeding Up Context Switches": global plan + orchestrated order;
 *      "Granularity of Memory Management": large allocations are subdivided into
 *      fixed-size units, which avoids fragmentation of the staging tier) ------------------
 * Pure host work, no GPU needed.  Splits allocations larger than a slot, packs smaller ones
 * into shared slots (each segment's slot offset is congruent to its device address mod 16),
 * orders the chunks, and divides the ring's slots between the two directions.
 * out_table: allocations that hold data at dev_ptr and must end up at host_ptr.
 * in_table:  allocations that hold data at host_ptr and must end up at dev_ptr.
 * Either table may be NULL or empty.  All device ranges must be pairwise disjoint, and all
 * host ranges too (no aliasing), else NIXIE_EOVERLAP; NIXIE_IN_PLACE lifts this for device
 * ranges of different tables and makes the planner walk the incoming table in the order in
 * which its GPU memory becomes free.
 * ring_bytes must hold at least 2 slots per active direction, else NIXIE_EINVAL.
 * *layout is library-owned; release with nixie_layout_destroy. */
int nixie_layout_create(const nixie_table_t *out_table, const nixie_table_t *in_table,
                        uint64_t ring_bytes, const nixie_opts_t *opts /* NULL = defaults */,
                        nixie_layout_t **layout);
int nixie_layout_info(const nixie_layout_t *layout, nixie_plan_info_t *info);
/* dir: 0 = outgoing, 1 = incoming.  Copies up to cap entries into a HOST array; returns the
 * total number of entries (>= 0) or a negative error. */
int64_t nixie_layout_chunks(const nixie_layout_t *layout, int dir, nixie_chunk_t *chunks, uint64_t cap);
int64_t nixie_layout_segments(const nixie_layout_t *layout, int dir, nixie_segment_t *segs, uint64_t cap);
void nixie_layout_destroy(nixie_layout_t *layout);

/* ---- plan: layout + pinned ring + flags + device descriptors + parked host threads --------
 * Same arguments and checks as nixie_layout_create.  Allocates exactly
 * (out_slots + in_slots) * slot_bytes <= ring_bytes of mapped pinned memory for payload and a
 * separately reported control block for the slot flags (paper, "Hierarchical Memory": the
 * pinned tier is the scarce one; "Speeding Up Context Switches": a window of it is reserved
 * for the evicted application).  A plan may be switched any number of times; a second plan
 * with the tables exchanged gives the way back. */
int nixie_plan(const nixie_table_t *out_table, const nixie_table_t *in_table,
               uint64_t ring_bytes, const nixie_opts_t *opts /* NULL = defaults */,
               nixie_plan_t **plan);
int nixie_plan_info(const nixie_plan_t *plan, nixie_plan_info_t *info);
void nixie_plan_destroy(nixie_plan_t *plan);

/* One ring for many plans.  Allocation tables change while applications run, so a caller
 * typically plans anew for every switch; a ring object keeps the pinned payload memory across
 * plans (allocating and pre-faulting 256 MiB takes about 20 ms, a plan on an existing ring
 * about 1 ms), and keeps the pinned budget exact when several plans exist at once.
 * nixie_plan_on_ring is nixie_plan with ring_bytes = the ring's size; the plan borrows the
 * memory.  Plans of one ring switch one at a time (NIXIE_EBUSY otherwise).  A ring is
 * destroyed after its plans (NIXIE_EBUSY before).  bytes: multiple of 4096. */
typedef struct nixie_ring nixie_ring_t;
int nixie_ring_create(uint64_t bytes, nixie_ring_t **ring);
int nixie_ring_destroy(nixie_ring_t *ring);
int nixie_plan_on_ring(const nixie_table_t *out_table, const nixie_table_t *in_table, nixie_ring_t *ring,
                       const nixie_opts_t *opts /* NULL = defaults */, nixie_plan_t **plan);

/* ---- the switch (paper, "Overview" step 4; "Speeding Up Context Switches") ----------------
 * Stream-ordered after everything already queued on hip_stream (a hipStream_t, NULL = the
 * default stream); this stands in for the paper's quiesce ("Valid memory access during
 * migration").  Launches one persistent kernel whose workgroups gather outgoing chunks from
 * HBM into ring slots and scatter incoming chunks from ring slots into HBM, paced by per-slot
 * credits; host drain threads move filled slots to the outgoing allocations' host_ptr and
 * host fill threads load slots from the incoming allocations' host_ptr.
 * BLOCKS the calling thread until both directions are complete, the last drain included.
 * On return 0: host_ptr[0..bytes) of every outgoing allocation equals its device bytes from
 * before the call, dev_ptr[0..bytes) of every incoming allocation equals its host bytes from
 * before the call, no byte outside a listed range was written, the ring holds nothing live.
 * Sources are unspecified afterwards.  stats may be NULL. */
int nixie_switch(nixie_plan_t *plan, void *hip_stream, nixie_stats_t *stats);

/* The same switch in three steps, for a caller that wants to let the incoming application run
 * as soon as ITS memory is ready (paper, "Overview" step 5: an application is re-enabled when
 * its memory is ready; what the user waits for is the incoming application) while the outgoing
 * one is still being evicted:
 *   nixie_switch_begin    checks, wakes the host threads, launches the kernel, returns at once;
 *   nixie_switch_wait_in  blocks until every byte of the incoming table is in HBM and visible to
 *                         kernels launched afterwards on any stream (each scatter workgroup
 *                         writes its L2 back before it counts as finished); returns the
 *                         switch's error if it failed meanwhile.  Optional, may be called once;
 *   nixie_switch_end      blocks until everything is complete, fills stats, returns the result
 *                         of the switch exactly as nixie_switch does.
 * Between begin and end the plan is busy (NIXIE_EBUSY for another switch), map / unmap calls
 * return NIXIE_EBUSY, and the three calls must come from one thread.  nixie_switch_wait_in / _end without a
 * begun switch: NIXIE_EINVAL.  Not available with NIXIE_SERIALIZE (NIXIE_EINVAL).  With
 * NIXIE_IN_PLACE the incoming bytes are complete at wait_in like otherwise; the outgoing
 * application's device ranges are the incoming one's by then. */
int nixie_switch_begin(nixie_plan_t *plan, void *hip_stream);
int nixie_switch_wait_in(nixie_plan_t *plan);
int nixie_switch_end(nixie_plan_t *plan, nixie_stats_t *stats);

/* ---- verification: per-allocation 64-bit hash ---------------------------------------------
 * H(b[0..n)) = mix64(n) + sum_k mix64(w_k + G*(k+1)) mod 2^64, w_k the k-th little-endian
 * 8-byte word (last one zero padded), G = 0x9E3779B97F4A7C15, mix64 the splitmix64 output
 * function.  Position keyed and additive, so partial sums combine in any order.
 *
 * nixie_hash_tables: BEFORE a switch.  out_hash[i] from DEVICE memory of the outgoing
 * table, in_hash[j] from HOST memory of the incoming table.  HOST output arrays of
 * table length (may be NULL when that table is empty).
 * nixie_verify: AFTER a switch.  Hashes the outgoing table at host_ptr and the incoming
 * table at dev_ptr and compares with the expected arrays; returns NIXIE_EMISMATCH and fills
 * report if any differs.  Either expected array may be NULL to skip that side. */
int nixie_hash_tables(const nixie_plan_t *plan, void *hip_stream, uint64_t *out_hash, uint64_t *in_hash);
int nixie_verify(const nixie_plan_t *plan, void *hip_stream, const uint64_t *expect_out_hash,
                 const uint64_t *expect_in_hash, nixie_verify_report_t *report);
/* Hash n buffers.  ptrs, bytes, hashes: HOST arrays of n.  on_device != 0: ptrs[i] are DEVICE
 * addresses hashed by the GPU kernel; else HOST addresses hashed by host threads. */
int nixie_hash_buffers(const void *const *ptrs, const uint64_t *bytes, uint64_t n, int on_device,
                       void *hip_stream, uint64_t *hashes);

/* nixie_hash_buffers for DEVICE buffers, for callers that cannot allocate: code between the
 * begin and end of a HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * It calls no hipMalloc / hipFree or other allocating routine and copies nothing between host and
 * device: the descriptor table reaches the GPU as kernel arguments, and it and the per-buffer
 * sums live in 128 KiB of static device memory that every GPU the library is used on holds until
 * the process ends.
 * ptrs, bytes: HOST arrays of n (ptrs[i] a DEVICE address).  hashes_dev: DEVICE array of n,
 * caller-owned; hashes_dev[i] = H(buffer i) once the work enqueued on hip_stream has run.
 * The call only enqueues kernels on hip_stream and returns; the buffers, and the mapping of any
 * space they lie in, must stay as they are until that work is complete.
 * n > 4096: NIXIE_EINVAL (use nixie_hash_buffers).  Other errors as nixie_hash_buffers.
 * All calls on one GPU share the static memory: calls on the same stream run one after the
 * other and are fine; calls whose kernels could overlap on one GPU (different streams, no
 * dependency between them) race and give wrong hashes. */
int nixie_hash_buffers_noalloc(const void *const *ptrs, const uint64_t *bytes, uint64_t n, void *hip_stream,
                               uint64_t *hashes_dev);

/* ---- stable device addresses over shared physical memory (paper, "Maintaining consistent
 *      virtual memory addresses": addresses are reserved once and mapped to different
 *      physical allocations before and after a migration; "Granularity of Memory
 *      Management": physical memory is handled in fixed-size blocks) -------------------------
 * A pool is physical device memory of the current device, cut into equal blocks.  A space is
 * a reserved range of device addresses as long as the pool, owned by one application, which
 * keeps its pointers for life.  Every block of a space is ASSIGNED a block of the pool: the
 * physical block that backs it whenever it is mapped (block i for block i unless
 * nixie_space_assign says otherwise; a mapped block cannot be reassigned: NIXIE_EBUSY).
 * nixie_space_map puts the assigned pool blocks behind a range of the space; several spaces
 * (or several blocks of one) may map the same pool block at once, and then they share its
 * bytes.  The planner knows this: device ranges count as overlapping exactly where they
 * share pool blocks and offsets inside them, whatever their addresses, so a switch between
 * two applications that take turns on the same physical blocks is an in-place switch
 * (NIXIE_IN_PLACE), ordered by the same per-chunk dependencies as for equal addresses, and
 * applications assigned different blocks are resident side by side.  A plan remembers the
 * assignment it was made under; nixie_switch returns NIXIE_EUNMAPPED if a block it needs is
 * unmapped or has been reassigned since.  The calls around a switch:
 *     nixie_space_map(B)  ->  nixie_switch(plan(A's table, B's table, NIXIE_IN_PLACE))
 *     ->  nixie_space_unmap(A)           (A's pointers stay reserved, and fault if used)
 * None of these calls runs inside the switch: while any switch is running (between
 * nixie_switch_begin and nixie_switch_end too) assign, map, unmap and destroy return
 * NIXIE_EBUSY and change nothing.  nixie_switch returns NIXIE_EUNMAPPED without touching the
 * GPU when a listed range lies in unmapped blocks.
 * block_bytes: multiple of the device's allocation granularity, 0 = 256 MiB (a map or unmap
 * call costs the same for any block size, so small blocks make the remap slow).  bytes is
 * rounded up to whole blocks.  offset and bytes of map / unmap must be multiples of the
 * block size; mapping a mapped block or unmapping an unmapped one is not an error.
 * Errors: NIXIE_EINVAL, NIXIE_ENOMEM (no physical memory or address range left),
 * NIXIE_EHIP, NIXIE_EBUSY (pool destroyed while spaces exist).  Spaces are destroyed before
 * their pool; destroying a space unmaps it. */
typedef struct nixie_pool nixie_pool_t;
typedef struct nixie_space nixie_space_t;
int nixie_pool_create(uint64_t bytes, uint64_t block_bytes, nixie_pool_t **pool);
int nixie_pool_info(const nixie_pool_t *pool, uint64_t *bytes, uint64_t *block_bytes);
int nixie_pool_destroy(nixie_pool_t *pool);
int nixie_space_create(nixie_pool_t *pool, nixie_space_t **space, void **base /* device address */);
/* pool_blocks[i] (an index into the pool) backs block offset / block_bytes + i from now on */
int nixie_space_assign(nixie_space_t *space, uint64_t offset, const uint64_t *pool_blocks, uint64_t n_blocks);
int nixie_space_map(nixie_space_t *space, uint64_t offset, uint64_t bytes);
int nixie_space_unmap(nixie_space_t *space, uint64_t offset, uint64_t bytes);
/* 1 = every block of [offset, offset + bytes) is mapped, 0 = not, negative = error */
int nixie_space_mapped(const nixie_space_t *space, uint64_t offset, uint64_t bytes);
int nixie_space_destroy(nixie_space_t *space);

/* ---- pinned tier (paper, "Hierarchical Memory": a chunk lives in exactly one of GPU memory,
 *      CPU pinned memory, CPU pageable memory or disk, and migrates between tiers as a whole) ---
 * nixie_tier_register announces a range of pinned host memory that the GPU can address (from
 * hipHostMalloc; the caller keeps it allocated while registered).  From then on, an allocation
 * of a table whose [host_ptr, host_ptr + bytes) lies inside a registered range, with
 * host_ptr == dev_ptr modulo 16, is moved by the kernel straight between HBM and host_ptr: it
 * takes no ring slot, no host thread touches it, and it costs host DRAM one access per byte
 * instead of three.  Allocations elsewhere (pageable memory) go through the ring as before,
 * in the same switch; a plan whose tables are entirely in the pinned tier needs no ring
 * (ring_bytes may be 0) and starts no host threads.  Semantics of nixie_switch are unchanged.
 * Plans pick the registry up when they are made, and a plan that moves chunks directly holds the
 * GPU's addresses of the registered memory: until every such plan is destroyed
 * nixie_tier_unregister returns NIXIE_EBUSY and changes nothing, and the caller must not free the
 * memory (unregister first, free after it returned 0).  Plans whose chunks all go through the
 * ring hold nothing.  Errors: NIXIE_EINVAL (NULL, 0 bytes, not pinned host memory, overlaps a
 * registered range, unknown base), NIXIE_EBUSY, NIXIE_EHIP. */
int nixie_tier_register(void *host_base, uint64_t bytes);
int nixie_tier_unregister(void *host_base);
/* The leg between the pinned and the pageable tier outside a switch (paper, "Speeding Up Context
 * Switches": the incoming application's data is brought into pinned memory by several threads,
 * to use the DRAM bandwidth; "Scheduling": the head of the queue is the prefetch candidate):
 * dst[i][0..bytes[i]) = src[i][0..bytes[i]) for i < n, HOST pointers on both sides, any
 * alignment, ranges must not overlap; streaming stores, work split in 1 MiB units over
 * `threads` threads (0 = half the cores, at most 8).  Blocks until done.  No GPU involved. */
int nixie_host_copy(void *const *dst, const void *const *src, const uint64_t *bytes, uint64_t n, uint32_t threads);

/* ---- placement (paper, "Speeding Up Context Switches": a global plan decides which chunks must
 *      be migrated, their source and their destination; evicted data stays in the highest tier
 *      that can hold it; transfers that cross several tiers come first) ----------------------
 * Host only, no GPU needed.  chunks[i] says where chunk i is now.  On return new_tier[i] says
 * where it should be once incoming_app owns the GPU:
 *   - every chunk of incoming_app is in GPU memory;
 *   - chunks of the applications in victim_apps (in that order, e.g. lowest priority first;
 *     inside an application in table order) leave GPU memory, but only until incoming_app fits;
 *   - an evicted chunk stays in the pinned tier if it fits the room that is free there now
 *     (both directions of a switch run at once, so incoming_app's pinned chunks still hold
 *     their space while evicted data arrives), else it goes to pageable memory;
 *   - everything else stays.
 * order (nullable, room for n entries) receives the indices of the chunks that move, in
 * migration order: moves between GPU and pageable memory first; *n_moved their number.
 * The outgoing table of the switch is the set of chunks with tier GPU -> not GPU, the incoming
 * table the set with not GPU -> GPU; a chunk's host_ptr is chosen by its host tier.
 * Errors: NIXIE_EINVAL (NULL, unknown tier, a capacity already exceeded, incoming_app listed
 * as a victim), NIXIE_ENOMEM (incoming_app does not fit even with every victim evicted);
 * outputs are unspecified on error. */
enum nixie_tier { NIXIE_TIER_GPU = 0, NIXIE_TIER_PINNED = 1, NIXIE_TIER_PAGEABLE = 2 };
typedef struct {
    uint64_t bytes;
    uint32_t app;
    uint32_t tier; /* enum nixie_tier */
} nixie_chunk_state_t;
typedef struct {
    uint64_t gpu_bytes;    /* GPU memory available to applications        */
    uint64_t pinned_bytes; /* size of the pinned tier (the ring not included) */
} nixie_capacity_t;
typedef struct {
    uint64_t restored_bytes, restored_from_pageable_bytes;
    uint64_t evicted_bytes, kept_pinned_bytes, to_pageable_bytes;
    uint64_t gpu_used_after, pinned_used_after;
} nixie_placement_t;
int nixie_place(const nixie_capacity_t *cap, const nixie_chunk_state_t *chunks, uint64_t n,
                uint32_t incoming_app, const uint32_t *victim_apps, uint32_t n_victims,
                uint32_t *new_tier, uint64_t *order, uint64_t *n_moved, nixie_placement_t *summary);

/* ---- host-link probe (paper, "Microbenchmarks": throughput is judged against the link's
 *      measured maximum) ---------------------------------------------------------------------
 * Allocates 2 device + 2 pinned buffers of `bytes` each for the duration of the call, times
 * best-of-reps transfers, frees them.  out: HOST. */
int nixie_link_peak(uint64_t bytes, int reps, nixie_link_peak_t *out);

/* ---- scheduler (paper, "Scheduling": Idleness Detection, Priority Inference / Algorithm 1,
 *      MLFQ with Prefetching) ------------------------------------------------------------------
 * Pure host logic: decides which application owns the GPU; the caller then runs the matching
 * nixie_switch.  All times are nanoseconds on a clock of the caller's choice, non-decreasing
 * over the calls on one scheduler, so a recorded trace replays exactly.  Not thread safe.
 * Applications are numbered 0, 1, ... in the order they are added; levels are 1 (highest
 * priority) .. levels.  Level p has allotment T_p = allot_ns * 2^(p-1) and preemption
 * threshold S_p = preempt_ns * 2^(p-1). */
typedef struct nixie_sched nixie_sched_t;

typedef struct {          /* every field 0 = default */
    uint32_t levels;      /* K, default 4, at most 16              */
    uint64_t allot_ns;    /* T of the top level, default 8 s       */
    uint64_t preempt_ns;  /* S of the top level, default 4 s       */
    uint64_t idle_ns;     /* idleness threshold, default 100 ms    */
} nixie_sched_params_t;

typedef struct {
    int32_t run;          /* application that owns the GPU after this tick, -1 = none           */
    int32_t evict;        /* application that lost it in this tick, -1 = none                   */
    int32_t prefetch;     /* head of the queue after the decision: worth prefetching, -1 = none */
    uint32_t switched;    /* 1 if run changed in this tick: the caller switches evict -> run    */
} nixie_sched_decision_t;

typedef struct {
    uint32_t priority;    /* current level                                           */
    uint32_t idle, pending, running;
    uint64_t exec_ns;     /* t_a: execution time accumulated at the current level    */
} nixie_sched_app_t;

int nixie_sched_create(const nixie_sched_params_t *params /* NULL = defaults */, nixie_sched_t **sched);
void nixie_sched_destroy(nixie_sched_t *sched);
/* Returns the new application's id (>= 0) or a negative error.  It starts at level 1. */
int nixie_sched_add_app(nixie_sched_t *sched, uint64_t now_ns);
/* The application entered / returned from a runtime API call.  blocking != 0: it may sit inside
 * the call for long (a synchronisation) and is not idle meanwhile. */
int nixie_sched_api_enter(nixie_sched_t *sched, int app, uint64_t now_ns, int blocking);
int nixie_sched_api_return(nixie_sched_t *sched, int app, uint64_t now_ns);
/* The application tried to launch work while it does not own the GPU: it joins the queue of its
 * level (no effect if it already waits or owns the GPU). */
int nixie_sched_request(nixie_sched_t *sched, int app, uint64_t now_ns);
/* The periodic step, also to be called on an idleness notification: accounts the owner's
 * execution time, applies the priority inference to every application, then decides. */
int nixie_sched_tick(nixie_sched_t *sched, uint64_t now_ns, nixie_sched_decision_t *decision);
int nixie_sched_app_info(const nixie_sched_t *sched, int app, uint64_t now_ns, nixie_sched_app_t *info);

/* A caller compiled against another version of this header would hand the library structures of the
 * wrong size.  Pass sizeof(nixie_opts_t), sizeof(nixie_plan_info_t), sizeof(nixie_stats_t): 0 if
 * they are the library's own, NIXIE_EINVAL otherwise.  The shim and the Python binding check this
 * once when they start. */
int nixie_abi_check(uint64_t sizeof_opts, uint64_t sizeof_plan_info, uint64_t sizeof_stats);

const char *nixie_strerror(int err);
int nixie_last_hip_error(void); /* hipError_t of the last NIXIE_EHIP on this thread */

#ifdef __cplusplus
}
#endif
#endif /* NIXIE_H */
