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

/* Testing aid for TDC_VARIANT_MERGED_XCD plans: the number of times a workgroup polls for the others before it
 * gives up (default 1 << 17, tens of milliseconds).  0 makes every workgroup that is not the last to arrive give
 * up at once -- the way the tests reach the TDC_ERR_WAIT path with kernels that still end normally.  Also clears
 * the plan's sticky status.  TDC_ERR_BAD_TUNING for plans of other variants. */
struct tdc_plan;
int tdc_plan_set_wait_limit(struct tdc_plan *plan, unsigned polls);

#ifdef __cplusplus
}
#endif
#endif /* TDC_MEASURE_H */
