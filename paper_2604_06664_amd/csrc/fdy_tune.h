/* Internal tuning knobs of libfdy (launch shapes, LDS budget, spin limit).  They exist for
 * measurement sweeps and for tests that force the bounded-wait error path from the host;
 * they are not part of the public interface and may change without notice.  Values are
 * process-wide and read at call time. */
#ifndef FDY_TUNE_H
#define FDY_TUNE_H
#ifdef __cplusplus
extern "C" {
#endif

enum {
  FDY_TUNE_SCAN_TOP_LOG2 = 0,   /* log2 of the most sampled bases staged in LDS           */
  FDY_TUNE_SCAN_WG_PER_CU = 1,  /* persistent scan workgroups launched per compute unit    */
  FDY_TUNE_SCAN_SPIN_LIMIT = 2, /* polls of a predecessor tile before giving up            */
  FDY_TUNE_MAT_VARIANT = 3,     /* materialize kernel variant                              */
  FDY_TUNE_COUNT = 8
};

int fdy__tune_get(int knob);
/* returns the previous value, or -1 for an unknown knob / value out of range */
int fdy__tune_set(int knob, int value);

#ifdef __cplusplus
}
#endif
#endif
