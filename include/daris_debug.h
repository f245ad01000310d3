/*
 * daris_debug.h -- instrumentation of the MI355X DARIS library: launch plans, per-layer outputs and timings, kernel
 * timing by sampling, the driver's wall-time breakdown and the CU-mask probe.  None of this is on the hot path; the
 * product calls are in daris.h, whose general rules (status codes, host / device pointers, one API thread) apply here too.
 */
#ifndef DARIS_DEBUG_H
#define DARIS_DEBUG_H

#include "daris.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Launch plan of one layer, for inspection and for host-side checks of what the kernels assume (no device needed).
 * Writes 27 values into out (host int64[cap >= 27]) and returns 27: [0] kernel id (daris_kernel_name), [1] 1 = dense
 * convolution (the rest is meaningful only then), [2] pixels per wave tile (32, or 16: then channel blocks are 16 wide too), [3] M = output
 * pixels, [4] N = output channels incl. padding, [5] K, [6] K padded, [7] channel blocks per wave tile, [8] waves
 * per workgroup, [9] K steps in total, [10] per workgroup slice, [11] per wave, [12] split-K factor, [13] pixel tiles,
 * [14] channel tiles, [15] weight groups, [16] workgroup order mode, [17..19] grid x y z, [20] threads per workgroup,
 * [21] split-K workspace bytes, [22] layer it shares a launch with or -1, [23] 1 = the joint launch is issued at this
 * layer, [24] activation slot of the layer's output (-1: the caller's logits), [25] slot of its input, [26] slot of its
 * residual operand or -1.  A slot is a device buffer shared by tensors whose lifetimes do not overlap. */
int32_t daris_get_launch_plan(daris_task t, int layer, int64_t* out, int32_t cap);
/* After daris_forward with DARIS_KEEP_ACTIVATIONS: copy layer l's output to host float[c][h][w]. */
daris_status daris_read_layer(daris_task t, int layer, float* host_out, int64_t cap_elems);
/* Time each layer of task t on stream 0 of partition p: `reps` runs back to back, from the start time stamp of the
 * first dispatch to the end time stamp of the last, divided by reps (the earlier layer of a launch pair reports 0).
 * ms_per_layer = host float[n_layers]; kernel_id = host int32[n_layers] (which kernel variant ran, see
 * daris_kernel_name); flops = host double[n_layers] algorithmic FLOPs (2*MACs) of the layer. */
daris_status daris_profile_layers(daris_task t, daris_part p, int reps, float* ms_per_layer, int32_t* kernel_id,
                                  double* flops);
const char* daris_kernel_name(int32_t kernel_id);
/* Kernel timing by sampling, for roofline figures measured inside a scheduled run: from now on every `every`-th job
 * of each task (0 = off) has every launch complete a signal of its own, into which the command processor of the
 * queue the kernel runs on writes the start and end time stamp of that dispatch (the figures a kernel trace shows);
 * for at most about max_samples launches.  Sampled jobs run slightly slower (one signal per launch). */
daris_status daris_kernel_timing_start(int every, int max_samples);
/* Waits until idle, stops the sampling and sums the samples per kernel id: launches[id], total_ms[id], total_flops[id]
 * (algorithmic FLOPs, 2*MACs) for id < the returned count; the arrays (host) must hold `cap` >= 64 entries.
 * *empty_pair_ms (may be NULL) receives the fixed cost contained in every sample: 0 for dispatch time stamps. */
int32_t daris_kernel_timing_read(int32_t cap, int64_t* launches, double* total_ms, double* total_flops, double* empty_pair_ms);
/* Where the wall time of a stage goes in real-time mode (the price of the synchronisation point at each stage
 * boundary, Sec. III-B1).  Waits until idle, copies the totals gathered since the last call to out (host int64[8], may
 * be NULL), clears them, and switches the gathering on (enable != 0) or off.  While it is on, the first launch of each
 * stage completes a signal too.  out[0] stages executed; [1] host ns enqueueing the stage's kernels;
 * [2] host ns from the last enqueue until the completion signal was seen; [3] host ns from then until the scheduler lock
 * was held; [4] host ns in the decision core and the hand-over of the next stages; [5] GPU ns from the start time stamp
 * of the stage's first dispatch to the end time stamp of its last; [6] host ns between a dispatch pass handing a stage to a stream's
 * worker and the worker starting to enqueue it; [7] reserved. */
daris_status daris_driver_profile(int enable, int64_t* out);
/* Mask probing: launch n_groups (<= 65536) short workgroups on stream 0 of partition p; out = host
 * uint32[2 * n_groups] receives, per workgroup, the XCC (die) id and the hardware id register of the compute unit
 * it ran on.  `spin` (0..100000) bounds a sleep loop that keeps workgroups resident so that they spread over
 * every CU the mask allows. */
daris_status daris_probe_cus(daris_part p, int n_groups, int spin, uint32_t* out);

#ifdef __cplusplus
}
#endif
#endif /* DARIS_DEBUG_H */
