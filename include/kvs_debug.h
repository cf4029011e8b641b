/*
 * kvs_debug.h - testing aids of libkvs.  Nothing here is part of the merge step's interface (include/kvs.h):
 * the switches below only choose between kernels that compute the same thing, so that a test can reach
 * every code path on any input shape, and so that a tuning run can compare them.
 *
 * The switches are process-global integers.  They are read (one relaxed atomic load each, no environment
 * lookup) by the calls of kvs.h; kvs_debug_set() while another thread is inside such a call gives that call
 * either value.  Initial values come from the environment variables named below, read ONCE when the library
 * is loaded; 0 always means "the library decides".
 */
#ifndef KVS_DEBUG_H
#define KVS_DEBUG_H

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  KVS_DEBUG_SCORE_PATH = 0,   /* KVS_SCORE_PATH=valu   1: vector-ALU score kernels also where the MFMA kernels apply   */
  KVS_DEBUG_SCORE_WIDE = 1,   /* KVS_SCORE_WIDE=0      1: more than 128 query rows take the kernel for 64 rows per
                                                          wavefront in several passes                                   */
  KVS_DEBUG_FUSE_OBAR = 2,    /* KVS_FUSE_OBAR=0|1     1: the pass over V never rides along in score sweep 1,
                                                       2: always (where the kernel can carry it)                        */
  KVS_DEBUG_DECODE_PATH = 3,  /* KVS_DECODE_PATH=valu|mfma   1: vector-ALU decode kernel, 2: MFMA decode kernel         */
  KVS_DEBUG_SCORE_CHUNK = 4,  /* KVS_SCORE_CHUNK=<n>   tokens per score workgroup (clamped to the supported range)      */
  KVS_DEBUG_VERBOSE = 5,      /* KVS_VERBOSE=1         1: the HIP error string of a failed launch goes to stderr        */
  KVS_DEBUG_SCORE_FUSED = 6,  /* KVS_SCORE_FUSED=1     2: the one-pass score kernel (K kept in LDS between the statistics
                                                          and the alpha_bar phase) wherever it applies; it is off
                                                          otherwise (measured slower than the two sweeps)              */
  KVS_DEBUG_SELECT_SPLIT = 7, /* KVS_SELECT_SPLIT=<n>  how a unit's edge selection is spread over workgroups.  1: always one
                                                       workgroup per unit, 2: as many parts as a unit can have (down to
                                                       64 edges each), whatever the launch, 3: the same with a wait limit
                                                       of zero, so that the parts give up at their first wait and the
                                                       unit's first part selects alone (a test of that way out)         */
  KVS_DEBUG_FUSED_WAIT_US = 8,/* KVS_FUSED_WAIT_US=<n> n + 1: a workgroup of the one-pass score kernel waits at most n
                                                       microseconds for its unit's normalisers before it hands its
                                                       item to the second kernel (1: it never waits)                   */
  KVS_DEBUG_FUSED_STAGGER = 9,/* KVS_FUSED_STAGGER=<n> n + 1: the four cohorts of workgroups of the one-pass score kernel start
                                                       n tenths of a microsecond apart                                 */
  KVS_DEBUG_GROUP_UNITS = 10, /* KVS_GROUP_UNITS=<n>   most units of one launch (the library puts up to 1024 short units, or 2 M
                                                       tokens, into one; groups of more than 64 keep their descriptors in
                                                       the workspace)                                                   */
  KVS_DEBUG_N_SWITCHES = 11
} kvs_debug_switch;

/* Sets a switch (a kvs_debug_switch, passed as an int) and returns its previous value; -1 (nothing changed) for an
 * unknown switch or a negative value. */
int kvs_debug_set(int which, int value);
/* Current value of a switch (-1 for an unknown one). */
int kvs_debug_get(int which);

#ifdef __cplusplus
}
#endif
#endif /* KVS_DEBUG_H */
