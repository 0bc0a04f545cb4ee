/*
 * lohan_adam_tuning.h -- BENCH-ONLY additions to the C ABI of lohan_adam.h: a launch-shape
 * override for tuning sweeps and the bandwidth probes that measure what the machine sustains for
 * the step's access pattern.  Nothing here is part of the product interface; a framework that
 * runs the block step of Sec. IV-C never includes this file.
 */
#ifndef LOHAN_ADAM_TUNING_H
#define LOHAN_ADAM_TUNING_H

#include "lohan_adam.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Launch-shape override for the calls made afterwards BY THE CALLING THREAD (thread-local: other
 * threads, and work they have in flight, keep the built-in shape).
 *   adam_variant            bits [1:0] workgroup size (64, 128, 256 lanes), bits [3:2]
 *                           vectors per lane per tile (1, 2), bits [5:4] cache policy (0 default,
 *                           1 nontemporal, 2 nontemporal loads + write-through streaming stores);
 *                           negative = automatic (64 lanes, 1 vector; default policy for blocks
 *                           that fit the 256 MiB memory-side cache, policy 2 above that; reported
 *                           as -1 by the getter); other values -> LOHAN_ERR_ARG
 *   adam_workgroups_per_cu  0 = one tile per workgroup (grid = number of tiles); > 0 caps the
 *                           grid at that many workgroups per compute unit; negative = default
 *   adam_waves_per_cu       occupancy throttle: at most this many wavefronts of the Adam kernel
 *                           resident per compute unit (0 or 32 = no throttle); negative = default
 *   reduce_workgroups_per_cu  grid of the gradient reduction per compute unit (<= 16);
 *                           <= 0 = default
 *   reduce_policy           loads of the gradient reduction: 0 default cache policy,
 *                           1 nontemporal, negative = automatic (by block size, as above)
 */
lohan_status_t lohan_tuning_set_launch_config(int adam_variant, int adam_workgroups_per_cu,
                                              int adam_waves_per_cu, int reduce_workgroups_per_cu,
                                              int reduce_policy);
void lohan_tuning_get_launch_config(int *adam_variant, int *adam_workgroups_per_cu,
                                    int *adam_waves_per_cu, int *reduce_workgroups_per_cu,
                                    int *reduce_policy);

/*
 * Bound of the grid-wide wait inside lohan_adam_small_block_step, in polls (one poll is a trip to
 * memory and a short sleep, a third of a microsecond), for the calls made afterwards by the
 * calling thread; negative = the built-in bound (2^20).  With 0 every workgroup but the one that
 * arrives last gives up at once, which is how the tests reach the LOHAN_OVERFLOW_INCOMPLETE
 * report without anything going wrong on the device.  LOHAN_ERR_ARG above 2^32 - 1.
 */
lohan_status_t lohan_tuning_set_wait_limit(int64_t polls);

/* What the library read from the current device's attributes: compute units and bytes of LDS
 * per compute unit (the occupancy throttle is sized from the latter).  LOHAN_ERR_HIP if the
 * attributes cannot be read. */
lohan_status_t lohan_tuning_device_info(int *compute_units, size_t *lds_bytes_per_cu);

/*
 * Bandwidth probes: the access patterns of the step with trivial arithmetic, to measure the
 * ceiling the machine sustains for each (64-lane workgroups handed out in address order, 128-bit
 * accesses per lane, nontemporal loads and write-through streaming stores; the five-stream probe
 * has the update kernel's exact launch shape, one 256-element tile per workgroup, the
 * single-stream probes take eight such rows per workgroup).  Each call enqueues ONE kernel on
 * `stream` (LOHAN_PROBE_MEMCPY: one hipMemcpyAsync device-to-device) and returns.
 *   LOHAN_PROBE_READ         reads n floats from a                       4 n bytes
 *   LOHAN_PROBE_WRITE        writes n floats to b                        4 n bytes
 *   LOHAN_PROBE_COPY         b[i] = a[i]                                 8 n bytes
 *   LOHAN_PROBE_FIVE_STREAM  the update kernel's pattern in place: reads g16 (n halves), a, b, c
 *                            (n floats each), writes a, b, c and h16 (n 16-bit values), with a
 *                            few multiply-adds in between                28 n bytes
 *   LOHAN_PROBE_MEMCPY       hipMemcpyAsync(b, a, 4 n, DeviceToDevice)   8 n bytes
 * a, b, c, g16, h16: device, 16-byte aligned, n elements each, not overlapping; pointers a
 * pattern does not use may be NULL.  Only whole tiles are touched: n is rounded down to a
 * multiple of 256 elements (five-stream, memcpy) or of 2048 elements (read, write, copy).
 * waves_per_cu: occupancy throttle as above (0 = none).  The contents of written arrays are
 * unspecified afterwards.  Errors: LOHAN_ERR_NULL / _ALIGN / _ARG, LOHAN_ERR_HIP.
 */
enum {
    LOHAN_PROBE_READ = 0,
    LOHAN_PROBE_WRITE = 1,
    LOHAN_PROBE_COPY = 2,
    LOHAN_PROBE_FIVE_STREAM = 3,
    LOHAN_PROBE_MEMCPY = 4
};
lohan_status_t lohan_tuning_probe(int pattern, float *a, float *b, float *c, const void *g16,
                                  void *h16, uint64_t n, int waves_per_cu, hipStream_t stream);

/*
 * Fault injection for tests of the offload pipeline's error path: the (after_calls + 1)-th HIP
 * runtime call that later lohan_offload_submit calls on this handle would make is not issued and
 * reports failure instead.  Nothing faults on the device: the submit returns LOHAN_ERR_HIP and
 * the handle is poisoned exactly as after a real runtime failure.  LOHAN_ERR_NULL / _ARG.
 */
lohan_status_t lohan_tuning_offload_inject_failure(lohan_offload_t *handle, int after_calls);

/*
 * Durations of the three stages of the block that last went through staging slot `slot` of an
 * offload pipeline: its host-to-device copies, its flag/norm pass + step, its device-to-host
 * copies, each from event to event on the stream that ran it (milliseconds; outputs may be
 * NULL).  Waits for that block's copy-out to finish.  LOHAN_ERR_ARG for a slot that has not been
 * used, LOHAN_ERR_HIP if the events cannot be read.
 */
lohan_status_t lohan_tuning_offload_slot_times(lohan_offload_t *handle, int slot, float *h2d_ms,
                                               float *step_ms, float *d2h_ms);

#ifdef __cplusplus
}
#endif

#endif /* LOHAN_ADAM_TUNING_H */
