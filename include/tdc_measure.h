/* Measurement aids of libtdc.so: entry points a benchmark harness uses and a product does not.  Kept apart from tdc.h. */
#ifndef TDC_MEASURE_H
#define TDC_MEASURE_H

#ifdef __cplusplus
extern "C" {
#endif

/* Enqueue one empty kernel (a single wavefront that does nothing) on the stream (a hipStream_t; device work only,
 * nothing is allocated or waited for), so that a harness can report the launch floor next to per-layer latencies,
 * which at batch 1 are of the same order (the paper, section 6, also notes that launch time of the extra 1x1 kernels
 * can outweigh the saved FLOPs).  Returns TDC_OK or TDC_ERR_HIP. */
int tdc_launch_null(void *hip_stream);

/* Testing aids for TDC_VARIANT_MERGED_XCD plans (TDC_ERR_BAD_TUNING for plans of other variants).
 * tdc_plan_set_wait_limit: the number of times a workgroup polls for the others of its XCD before it stops waiting and
 * computes all of stage 1 itself (default 512, some hundred microseconds).  0 makes every workgroup that is not the
 * last to arrive take that path at once -- the way the tests exercise it.
 * tdc_plan_waits_given_up: how many workgroups have taken it since the plan was made (copies one word from the
 * device: synchronises). */
struct tdc_plan;
int tdc_plan_set_wait_limit(struct tdc_plan *plan, unsigned polls);
int tdc_plan_waits_given_up(struct tdc_plan *plan, unsigned *count);

#ifdef __cplusplus
}
#endif
#endif /* TDC_MEASURE_H */
