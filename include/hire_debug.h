/*
 * hire_debug.h -- testing and measurement aids of libhire, next to the product interface in hire.h.
 *
 * Nothing here is needed to run a HiRE step (arXiv 2402.09360, Algorithm 1).  The calls below let the tests
 * force the general kernel sequence, read how often an equally exact but slower selection route was taken,
 * undo the int4 packing of Sec. 3.2's Zapprox for checking, and let the benchmark time single stages and
 * calibrate a profiler's HBM counters.  The general rules of hire.h apply (device pointers unless stated,
 * work enqueued on `stream`); the per-thread switches affect only steps issued by the calling thread.
 */
#ifndef HIRE_DEBUG_H
#define HIRE_DEBUG_H

#include "hire.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Stage timing hook for profiling.  events: HOST array of HIRE_NUM_STAGE_EVENTS hipEvent_t created by the
 * caller, or NULL to switch the hook off (the default).  While set (per calling thread), each step records
 * event i on its stream in front of stage i and one after the last stage.  Stages of the FFN step:
 * 0 token quantise / low-rank projection, 1 scorer, 2 top-k' select (rows beyond 32768: counting and marking),
 * 3 resolving the threshold bin (rows beyond 32768) and union compaction where the gather does not do it itself
 * (bitmaps beyond 8192 words), 4 exact scores on the candidates (with the union compaction in its prologue),
 * 5 exact top-k, 6 second layer; event 7 closes the step.  The softmax step ends with
 * event 6 after its stage 5 (top-k + softmax).  The batch-1 FFN step with the int4 scorer runs four kernels
 * and records five events: 0 scorer (with token quantisation), 1 k'-selection + exact scores on the candidates,
 * 2 k-selection + second-layer partial sums, 3 final reduction; event 4 closes the step.
 * Do not use while the stream is being captured. */
#define HIRE_NUM_STAGE_EVENTS 8
void hire_set_stage_events(void** events);

/* Testing aid; synchronises the stream.  host_out2 (HOST memory, two uint32) receives how many batch-1 FFN
 * steps on this workspace, since it took its steady state, had to find the k'-th scorer key (first counter)
 * or the k-th activation (second) without the key histogram: a slower, equally exact route taken for unusual
 * value distributions. */
int hire_debug_fast_fallbacks(const void* workspace, uint32_t* host_out2, void* stream);

/* Testing aid; synchronises the stream.  State that batch-1 FFN steps keep at the head of their workspace between
 * steps, read back to host_out3 (HOST memory, three uint32): [0] 1 if the marker is set that says "the histogram of
 * the scorer keys is all zero" (set by every completed step), else 0; [1] the number of counters of that histogram
 * that are not zero (0 after any completed step); [2] the sum of the counters of the histogram of the exact
 * activations, which the next step clears: after a step, the number of its candidates with a positive activation
 * that lie inside the histogram's window.  Allocates a host buffer for the copy. */
int hire_debug_fast_state(const void* workspace, uint32_t* host_out3, void* stream);

/* Testing aid; synchronises the stream.  host_out3 (HOST memory, three uint32) receives, for steps on the general
 * kernel sequence (softmax steps, FFN steps at batch > 1 or with the low-rank scorer), since this workspace took
 * its steady state for the current shapes: [0] how many tokens of long-row steps (rows beyond 32768, selected by
 * many workgroups through key histograms in the workspace) had their k'-th scorer key found by the streaming
 * selection instead; [1] how many single-workgroup selections (k' on shorter rows, k on the activations) found
 * their window histogram unable to answer and narrowed the range instead; [2] how many times since
 * hire_workspace_init the key histograms were found unstamped and had to be cleared: once on a fresh workspace
 * and again after every change of shapes (such steps select by streaming and are not counted in [0]). */
int hire_debug_general_fallbacks(const void* workspace, uint32_t* host_out3, void* stream);

/* Measurement aid (per calling thread).  device_buf: DEVICE buffer of at least 16 KiB, or NULL to switch off.
 * While set, every workgroup g of the batch-1 FFN scorer kernel stores the 100 MHz wall clock at its start and
 * at its end into device_buf[2g] and device_buf[2g+1] (uint64); the span from the smallest start to the largest
 * end over the hire_ffn_scorer_workgroups(d_ff) workgroups is the kernel's execution time without launch cost. */
int hire_set_scorer_clocks(void* device_buf, size_t bytes);
int hire_ffn_scorer_workgroups(int d_ff);

/* Measurement aid: a plain copy kernel (kernel name k_plain_copy) moving `bytes` (multiple of 16) from src to dst.
 * Profilers' HBM traffic counters are calibrated against a launch of known size of this kernel. */
int hire_debug_plain_copy(const void* src, void* dst, size_t bytes, void* stream);

/* Testing aid: the filter stage of the batched exact pre-activations (Algorithm 1, the exact computation over the
 * candidates) on its own, over rows 0 .. *rows_dev - 1 of W (bf16 [rows, d], DEVICE) and the B tokens x (bf16
 * [B, d], DEVICE).  stored (DEVICE float [B, rows]) receives what the stage keeps per (token, row): a value
 * within err_c |u| |x| of <u, x> where that is positive, the smallest positive float where it lies in
 * (-2 err_c |u| |x|, 0], exactly 0 below.  xnorm (DEVICE float [B]) receives upper bounds of the tokens' norms,
 * *wnorm_max (DEVICE, float bits, the caller clears it) of the largest row norm, *err_c (HOST) the constant. */
int hire_debug_filter_stage(const void* W, const void* x, int B, int d, int rows, const int32_t* rows_dev, float* stored,
                            float* xnorm, uint32_t* wnorm_max, float* err_c, void* stream);

/* Testing aid (per calling thread): with on != 0 every step takes the general kernel sequence, also where the
 * batch-1 fast sequence would apply.  Both produce the same outputs. */
void hire_force_generic_path(int on);

/* Testing aid (per calling thread): with on != 0 the FFN step at batch > 1 computes the exact pre-activation of
 * every candidate in fp64, instead of filtering in fp32 and recomputing in fp64 only around the selection
 * threshold.  The selected sets are the same; the float outputs agree within their tolerance. */
void hire_force_exact_stage(int on);

/* Inverse layout transform, for checking: codes_out int8 [rows, cols]. */
int hire_unpack_int4(const void* q4, int rows, int cols, int8_t* codes_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HIRE_DEBUG_H */
