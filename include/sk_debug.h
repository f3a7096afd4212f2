/*
 * libsk -- testing, tuning and measurement aids.  NOT part of the layer's definition and
 * not needed to use the library (include/sk.h is the interface of the layer); everything
 * here is process- or thread-wide state that the tests and the benchmark harness use.
 */
#ifndef SK_DEBUG_H
#define SK_DEBUG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Plan parameters that the per-shape planner normally chooses by itself.  Forcing one lets
 * a test reach the large-shape code paths (big tiles, tall token tiles, many splits) on a
 * shape small enough for a full pass of the CPU oracle, and lets a sweep measure the
 * alternatives.  Process-wide; value < 0 restores the automatic choice.  Out-of-range
 * values are clamped or ignored exactly as the planner documents for each knob.
 * sk_linear_workspace_bytes follows the knobs, so size the workspace after setting them.
 */
typedef enum {
  SK_TUNE_TILE = 0,     /* tile of the general GEMMs (0..7: 256x256/4 waves, 128x128, 128x64, 64x128,
                           64x64, 256x128, 128x256, 256x256/8 waves) */
  SK_TUNE_WTILE = 1,    /* tile of the token contraction of sk_linear_bwd_weight (same numbering) */
  SK_TUNE_WSPLITS = 2,  /* number of token splits of that contraction */
  SK_TUNE_BM = 3,       /* rows of a token tile in the on-chip (chain) kernels: 64 or 128 */
  SK_TUNE_SLICES = 4,   /* output slices per token tile in the chain kernels */
  SK_TUNE_STILE = 5,    /* tile of the split first contraction of the split+expand plan */
  SK_TUNE_SSPLITS = 6,  /* number of splits of that contraction */
  SK_TUNE_NARROW_BWD = 7, /* sk_linear_bwd's one-pass schedule for narrow sketches: 0 = never, 1 = wherever
                           the kernel can serve the shape, 32 or 64 = the same with that many tokens per
                           work-group */
  SK_TUNE_COUNT = 8
} sk_tune_knob;

/* Returns the previous value (negative = automatic), or INT32_MIN for an unknown knob. */
int32_t sk_set_tuning(sk_tune_knob knob, int32_t value);

/*
 * Launch trace (host only, works on a machine without a GPU).  Between sk_trace_begin()
 * and sk_trace_end() the calling thread's libsk calls plan exactly as usual but launch
 * nothing: every kernel they would have launched records the byte ranges it reads and
 * writes instead.  Pointers are never dereferenced, so made-up addresses serve.  A test
 * uses this to check, for any shape and plan, that every access stays inside the caller's
 * buffers and the workspace size sk_linear_workspace_bytes reports.
 */
typedef struct {
  uint64_t address;  /* first byte */
  uint64_t bytes;    /* length of the range (the rows of a strided matrix are covered from the
                        first byte of the first row to the last byte of the last one) */
  int32_t write;     /* 1 = written, 0 = read */
  int32_t launch;    /* index of the kernel launch within the trace, from 0 */
} sk_trace_access;

void sk_trace_begin(void);
/* Ends the trace; copies up to `max` records to `out` (may be NULL when max is 0) and
 * returns how many were recorded in all.  `launches`, if not NULL, receives the number of
 * kernel launches the traced calls would have made. */
int64_t sk_trace_end(sk_trace_access* out, int64_t max, int32_t* launches);

/*
 * Per-kernel timing.  Between sk_profile_begin() and sk_profile_end() every kernel the
 * calling thread's libsk calls launch is bracketed by a pair of HIP events on the launch
 * stream (this is the one place where the library creates HIP objects: up to max_kernels
 * pairs, created in sk_profile_begin and destroyed in sk_profile_end).  sk_profile_end
 * synchronises on the last event and reports, per launch in launch order, the kernel's
 * name as a profiler prints it and the time between its two events.  The events sit
 * between back-to-back kernels, so for kernels of a few microseconds the figure includes
 * their cost; for the millisecond kernels of the large configurations it does not matter.
 */
typedef struct {
  char name[120];
  float ms;
  int32_t groups;    /* work-groups in the launch */
  double flops;      /* flops of the products the launch forms (2 M N K per contraction) */
  double bytes;      /* bytes it must move: each operand read once, each result written once
                        (re-reads across tiles and cache traffic not counted) */
} sk_kernel_time;

/* Returns 0, or a negative value if the events could not be created (nothing is then recorded). */
int32_t sk_profile_begin(int32_t max_kernels);
/* Returns the number of launches recorded (at most max_kernels of sk_profile_begin), having
 * written min(that, max) records to `out`; negative on a HIP error. */
int32_t sk_profile_end(sk_kernel_time* out, int32_t max);

#ifdef __cplusplus
}
#endif
#endif /* SK_DEBUG_H */
