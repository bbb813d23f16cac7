/*
 * fdy_arena.h - deterministic device-memory layout for MI355X (gfx950), C ABI.
 *
 * Section 4.1.1 ("Deterministic Memory Layout") and Section 5.1 of the paper: allocations
 * are placed one after another inside one reserved virtual address range, so that a run
 * that repeats the same sequence of allocations gets the same addresses relative to the
 * range's base, and the record of the allocations is a sorted, non-overlapping table.  An
 * arena is that: a virtual address reservation (at a requested address when the driver
 * grants it), backed by physical memory mapped in one shot (the paper's replay mode
 * preallocates the recorded total), and a bump pointer.  Its table is the allocation table
 * that fdy_scan_pointers takes (fdy.h); the bases of a second arena that replayed the same
 * sequence are the base map that fdy_materialize / fdy_scan_rebase take.
 *
 * Unlike the calls of fdy.h these own device memory, hold state (the arena) and synchronize
 * nothing: they are host-side set-up calls, not part of the per-graph hot path.  Not
 * thread-safe per arena.  Return codes are those of fdy.h.
 */
#ifndef FDY_ARENA_H
#define FDY_ARENA_H

#include <stddef.h>
#include <stdint.h>

#include "fdy.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fdy_arena fdy_arena; /* opaque */

/* Reserves `capacity_bytes` (rounded up to the device's mapping granularity) of virtual
 * address space on the current device, at `va_hint` if the driver grants that address
 * (0: anywhere; if the driver refuses the address, or access to it, the arena is placed
 * anywhere: check fdy_arena_base), maps physical memory behind all of it and enables read/write access.
 * FDY_ERR_INVALID_ARG: null out pointer or zero capacity; FDY_ERR_HIP: a driver call failed
 * (nothing stays reserved). */
int fdy_arena_create(fdy_arena** out, uint64_t va_hint, size_t capacity_bytes);

/* The driver call that failed last on this thread, with the driver's text ("" if none). */
const char* fdy_arena_last_failure(void);

/* Base address and capacity of the reservation (0 for a null arena). */
uint64_t fdy_arena_base(const fdy_arena* a);
size_t fdy_arena_capacity(const fdy_arena* a);

/* Places the next allocation: `bytes` >= 1 at the bump pointer rounded up to `alignment`
 * (a power of two >= 8; 0 means 512), records {base, bytes} in the table.
 * FDY_ERR_CAPACITY: it does not fit (nothing changes). */
int fdy_arena_alloc(fdy_arena* a, size_t bytes, size_t alignment, void** d_ptr);

/* Number of allocations recorded so far, and a copy of the table (ascending by base,
 * non-overlapping by construction; valid per fdy_table_validate).  Copies
 * min(n, capacity) records to h_table. */
uint32_t fdy_arena_count(const fdy_arena* a);
int fdy_arena_table(const fdy_arena* a, fdy_alloc* h_table, uint32_t capacity);

/* Forgets all allocations (the memory stays mapped): the next sequence starts at the base
 * again.  Capture-window replay: the same sequence gives the same addresses. */
int fdy_arena_reset(fdy_arena* a);

/* Capture-window replay from a recording (Section 4.1.1, Section 5.1): h_recorded[n] is the
 * table of an earlier arena whose base was recorded_base (fdy_arena_table and fdy_arena_base
 * of the recording run, e.g. out of an archive).  Every recorded allocation is placed in `a`
 * at the same distance from a's base, appended to a's table, and the bump pointer moves behind
 * the last one; h_new_base[i] receives the new address of recorded allocation i (the base map
 * for fdy_materialize / fdy_scan_rebase).  Placement and errors are those of
 * fdy_layout_replay (fdy.h) with a's base, capacity and bump pointer; on any error nothing
 * changes.  FDY_ERR_INVALID_ARG also for a null arena. */
int fdy_arena_replay(fdy_arena* a, const fdy_alloc* h_recorded, uint32_t n, uint64_t recorded_base,
                     uint64_t* h_new_base);

/* Unmaps and releases everything.  Null is allowed. */
int fdy_arena_destroy(fdy_arena* a);

#ifdef __cplusplus
}
#endif
#endif /* FDY_ARENA_H */
