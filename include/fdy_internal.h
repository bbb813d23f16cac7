/* fdy_internal.h - INTERNAL exports of libfdy: tuning knobs (launch shapes, LDS budget, spin
 * limit) and per-kernel event timing.  They exist for measurement sweeps, for the bench, and
 * for tests that force the bounded-wait error path from the host; they are not part of the
 * public interface (fdy.h) and may change without notice.
 *
 * This is the only state the library keeps between calls: a process-wide array of integers
 * (the knobs) and the timing records.  Every entry point reads the knobs it needs once, at
 * the start of the call.  Neither is thread-safe: set knobs, and enable or read timing, only
 * while no other thread is inside a library call.  A knob that changes the layout of the
 * search hierarchy (FDY_TUNE_SCAN_TOP_LOG2) invalidates prepared tables made before the
 * change; the scan detects that on the device (FDY_ST_BAD_PREPARED). */
#ifndef FDY_INTERNAL_H
#define FDY_INTERNAL_H
#ifdef __cplusplus
extern "C" {
#endif

enum {
  FDY_TUNE_SCAN_TOP_LOG2 = 0,   /* log2 of the most sampled bases staged in LDS           */
  FDY_TUNE_SCAN_WG_PER_CU = 1,  /* persistent scan workgroups launched per compute unit    */
  FDY_TUNE_SCAN_SPIN_LIMIT = 2, /* polls of a predecessor tile before giving up            */
  FDY_TUNE_MAT_MAP_GROUP = 3,     /* base maps per materialize workgroup, 0 = automatic      */
  FDY_TUNE_SCAN_SMALL_LOG2 = 4, /* inputs below 2^this sub-tiles use the small-chunk scan   */
  FDY_TUNE_MAT_SELF_WGS = 5,    /* materialize launches of up to this many workgroups       *
                                 * resolve their tiles themselves (no prep launch); 0: none */
  FDY_TUNE_MAT_ONCE_TILES = 6,  /* a materialization of one map group over at least this many   *
                                 * tiles streams templates and relocation lists past the L2s  */
  FDY_TUNE_COUNT = 8
};

int fdy__tune_get(int knob);
/* returns the previous value, or -1 for an unknown knob / value out of range */
int fdy__tune_set(int knob, int value);

/* Per-kernel timing for the bench: when enabled with a record count n > 0, each launch of an
 * instrumented kernel carries a hipEvent pair (hipExtLaunchKernelGGL) that receives the kernel's
 * begin and end on the caller's stream (at most n launches per slot are recorded, later ones are
 * not; a group of launches that shares a slot is bracketed by two event records instead).
 * fdy__prof_read synchronizes the recorded events and returns, per slot, the number of records
 * and their total elapsed milliseconds; fdy__prof_enable(0) destroys the events.  Not
 * thread-safe; off by default. */
enum {
  FDY_PROF_SCAN_MAIN = 0,
  FDY_PROF_SCAN_INIT = 1,
  FDY_PROF_SEGMENT = 2,
  FDY_PROF_FP_KEYS = 3,
  FDY_PROF_FP_GROUP = 4,
  FDY_PROF_MAT_PREP_GRAPHS = 5,
  FDY_PROF_MAT_PREP_TILES = 6,
  FDY_PROF_MAT_MAIN = 7,
  FDY_PROF_SCAN_OUT = 8,
  FDY_PROF_SCAN_REBASE = 9,
  FDY_PROF_SCAN_RECORDS = 10, /* the launch ahead of the scan with output (scan_leafmap_kernel) */
  FDY_PROF_SLOTS = 11
};
int fdy__prof_enable(int n_records);
void fdy__prof_mask(unsigned slot_mask); /* which slots record; default all */
int fdy__prof_read(int slot, int* n_records, float* total_ms, float* min_ms, float* max_ms);
const char* fdy__prof_name(int slot);

#ifdef __cplusplus
}

namespace fdy {
/* internal: bracket a group of launches with two event records; no-ops unless profiling is
 * enabled */
void prof_begin(int slot, void* stream);
void prof_end(int slot, void* stream);
/* internal: the next pair of events of a slot for ONE launch that carries them itself (the
 * events then hold the kernel's own begin and end on the device, as a kernel trace reports
 * them; two records around a launch add the dispatch on either side, 2-6 us).  False: this
 * launch is not timed. */
bool prof_take(int slot, void** start_event, void** stop_event);
}  // namespace fdy
#endif
#endif
