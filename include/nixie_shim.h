/*
 * nixie_shim.h -- the transparent shim (libnixie_shim.so), for unmodified HIP applications.
 *
 * Paper, "Supporting Unmodified CUDA Applications": a library loaded with LD_PRELOAD interposes
 * the runtime's memory allocation and free, its kernel launches and its memory-usage report, so
 * that an application that knows nothing of the system can lose the GPU and get it back:
 *   - "Maintaining consistent virtual memory addresses": device addresses are reserved once and
 *     the physical memory behind them changes across a migration -- here every large allocation
 *     is a range of one nixie_space over one nixie_pool, so the application's pointers stay
 *     valid for life;
 *   - "Valid memory access during migration": before a migration new launches are held back and
 *     the device is synchronized;
 *   - "GPU Memory information": the memory report is the sum of the process's own allocations;
 *   - "Overview", steps 1, 2, 5, 6 of the architecture figure: a launch first checks the
 *     execution flag; if the application's memory is not resident it is brought back (the
 *     context-switch swap of nixie.h) before the launch goes ahead.
 * Single process: there is no daemon and no IPC here.  The scheduler's side is either a thread in
 * the same process calling nixie_shim_evict / nixie_shim_restore, or the shim's own idleness
 * rule (paper, "Idleness Detection": idle = no runtime call has returned for longer than a
 * threshold), after which the application is evicted as if another one had been scheduled.
 *
 * Application threads: the shim's own state is safe against calls from several threads (checked on a
 * CPU model under ThreadSanitizer), but on the GPU only applications that make their runtime calls
 * from one thread at a time are validated; with several launching threads a migration's own runtime
 * calls overlap those of the other threads, and that combination is not supported yet.
 *
 * Use:  LD_PRELOAD=/path/to/libnixie_shim.so  ./application      (set before the process starts)
 *
 * Interposed runtime calls (same prototypes as the HIP runtime's; everything else passes through):
 *   hipMalloc        size >= NIXIE_SHIM_MIN_BYTES: whole units of the shim's address space
 *                    (first fit), entered in the application's allocation table; smaller ones go
 *                    to the runtime unchanged (the paper leaves allocations under one block to the
 *                    plain allocator).  hipErrorOutOfMemory when the space is full.
 *   hipFree          releases such a range (and its host copy, if the application is evicted).  The
 *                    range's blocks stay mapped for the next allocation at these addresses (an
 *                    eviction unmaps them): a use after free is not caught by a fault.
 *   hipMemGetInfo    total = the capacity the shim was given, free = total - the application's
 *                    own allocations: the managed ones in whole units, the small ones as asked for.
 *   hipLaunchKernel, hipLaunchKernelExC, hipLaunchCooperativeKernel, hipModuleLaunchKernel,
 *   hipModuleLaunchCooperativeKernel, hipExtModuleLaunchKernel, hipGraphLaunch
 *                    check the execution flag; restore the application first if it is evicted.
 *                    Launches made by the shim's own library calls pass straight through.
 *   hipMemcpy, hipMemcpyAsync, hipMemcpyWithStream, hipMemcpyHtoD, hipMemcpyDtoH, hipMemcpyDtoD,
 *   hipMemcpyHtoDAsync, hipMemcpyDtoHAsync, hipMemcpyDtoDAsync, hipMemset, hipMemsetAsync,
 *   hipMemsetD8, hipMemsetD8Async, hipMemsetD32, hipMemsetD32Async
 *                    address device memory as well: the same flag check before they go ahead.
 *   hipStreamBeginCapture, hipStreamBeginCaptureToGraph, hipStreamEndCapture
 *                    paper, "CUDA graph compatibility": between the start and the end of a stream
 *                    capture the shim makes no runtime call of its own -- the capture starts with
 *                    the application resident, the idleness rule is suspended and
 *                    nixie_shim_evict returns NIXIE_EBUSY.  A graph instantiated from the capture
 *                    holds the application's pointers, which stay valid across migrations, so it
 *                    is launched unchanged afterwards.
 *   hipStreamCreate, hipStreamCreateWithFlags, hipStreamDestroy
 *                    never overlap a migration (the paper's shim intercepts stream creation too, as
 *                    a call that allocates implicitly); they do not bring an evicted application back.
 * Interposed only to time the application's activity (idleness), bracketed as calls that may
 * block: hipDeviceSynchronize, hipStreamSynchronize, hipEventSynchronize (the calls above count as
 * activity too, for as long as they take); and as plain signs of life the calls a program polls
 * with or feeds a stream with: hipEventQuery, hipStreamQuery, hipEventRecord, hipStreamWaitEvent.  They are not held back during a migration: a thread
 * waiting for work that another thread has yet to submit must not block the migration that holds
 * that other thread back.
 * Not interposed: graphs built node by node are launched like any other (hipGraphLaunch) but their
 * construction is not watched; stream-ordered allocators (hipMallocAsync), 2-D/3-D
 * and array copies, peer copies, managed memory.  A program that reaches its managed allocations
 * only through those must not be run with idle eviction on.
 *
 * Environment (read once, at the first interposed call):
 *   NIXIE_SHIM_POOL_MIB     capacity of the managed GPU memory, MiB (default 1024)
 *   NIXIE_SHIM_UNIT_MIB     allocation granularity, MiB (default 2: the paper's block)
 *   NIXIE_SHIM_BLOCK_MIB    what the driver maps and unmaps at a time, MiB: a multiple of the unit that
 *                           suits the device's allocation granularity (default 32; a driver call per
 *                           block is on the way of an application that comes back, 0.03-0.05 ms each)
 *   NIXIE_SHIM_MIN_BYTES    smallest managed allocation (default: one unit)
 *   NIXIE_SHIM_RING_MIB     pinned staging ring of the swap, MiB (default 64)
 *   NIXIE_SHIM_IDLE_MS      > 0: a watcher thread evicts the application once it has been idle
 *                           this long (default 0 = never; the paper's threshold is 100)
 *   NIXIE_SHIM_SCRIBBLE     1: after an eviction the freed physical memory is overwritten through
 *                           a second address space, as another application would (test aid)
 *   NIXIE_SHIM_SYNC_UNMAP   1: an eviction unmaps the application's blocks before it returns.  By default
 *                           that is left to a background thread (a driver call per block, 0.25 ms each on
 *                           MI355X, that nobody has to wait for: the evicted application cannot run, and
 *                           an application that comes back first keeps what is still mapped)
 *   NIXIE_SHIM_HOST_RELEASE what a restore does with the pages of the host copies: 0 (default) releases them
 *                           lazily, 1 keeps them (the memory stays the process's), 2 returns the range at once
 *   NIXIE_SHIM_LOG          1: one line per eviction / restore on stderr
 * Host memory: the pageable copy of an allocation keeps its address range from one eviction to the
 * next; after a restore its pages are released lazily (MADV_FREE), so a later eviction usually pays
 * no page faults for them.  hipFree gives the range back.
 */
#ifndef NIXIE_SHIM_H
#define NIXIE_SHIM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    uint64_t capacity_bytes;    /* managed GPU memory                                     */
    uint64_t block_bytes;       /* what is mapped and unmapped at a time                  */
    uint64_t unit_bytes;        /* what allocations are rounded to                        */
    uint64_t managed_bytes;     /* live managed allocations, in whole units               */
    uint64_t managed_allocs;
    uint64_t passthrough_allocs;/* live allocations below the threshold                   */
    uint32_t resident;          /* the execution flag: 1 = the application's memory is in HBM */
    uint32_t evictions, restores;
    uint64_t last_switch_ns;    /* duration of the last eviction (device wait, swap, unmapping) or restore */
    uint64_t launches_held;     /* launches that found the flag off and waited for a restore */
    uint64_t mapped_blocks;     /* blocks of the space with physical memory behind them right now */
    uint64_t passthrough_bytes; /* their sum, as asked for                                */
    uint64_t host_backing_bytes;/* pageable address ranges kept for this application's copies (their pages are the
                                   kernel's to reclaim while the application is resident)  */
} nixie_shim_info_t;

/* HOST out.  Returns 0, or NIXIE_EINVAL when the shim has not been initialised yet (no interposed
 * call so far) or info is NULL. */
int nixie_shim_info(nixie_shim_info_t *info);

/* The scheduler's two actions, for a caller inside the process.  nixie_shim_evict holds back new
 * launches, waits for the device, moves every managed allocation to pageable host memory with
 * nixie_switch, and has the physical memory unmapped; the application keeps its pointers.
 * nixie_shim_restore maps it again and brings the bytes back; any launch does the same on its own.
 * Both return 0 (also when there is nothing to do) or a negative nixie_err code; nixie_shim_evict
 * returns NIXIE_EBUSY while the application is capturing a stream. */
int nixie_shim_evict(void);
int nixie_shim_restore(void);

#ifdef __cplusplus
}
#endif
#endif /* NIXIE_SHIM_H */
