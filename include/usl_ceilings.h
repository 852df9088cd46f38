/*
 * usl_ceilings -- small measurement kernels for the rates that bound the uniformly-sparse layer's
 * products on gfx950: HBM streams, the LDS gather (ds_read_b32 at random and at conflict-free
 * addresses, and the wider reads), the copy of an activation row from L2 into LDS by every compute
 * unit at once, and the gather of 128-byte pieces from a region that one XCD's L2 holds; and a timing
 * prototype (synthetic lists, real data movement) of the input gradient in its feature-stationary LDS form,
 * with one row buffer and with two (copy of the next row in flight during the gathers), which is how the
 * design notes know what that form would cost and that copies and gathers of one compute unit do not overlap.
 * They are not part of the training path; the benchmark runs them to put its timings next to what
 * the chip delivers on the same box.  For callers that measure (they allocate and wait).
 */
#ifndef USL_CEILINGS_H
#define USL_CEILINGS_H

#ifdef __cplusplus
extern "C" {
#endif

/* Number of figures usl_ceilings_run produces. */
int usl_ceilings_count(void);
/* Name and unit of figure i ("hbm_read_GBps", "lds_gather_b32_random_lanes_per_clk_cu", ...), or NULL. */
const char* usl_ceilings_name(int i);
/* Runs every measurement on the current HIP device (null stream; allocates 2 GiB of device memory,
 * frees it again, waits for each kernel) and writes figure i to values[i], i < n.  values: host memory.
 * Returns 0, or the hipError_t of the first failing call (values already measured stay). */
int usl_ceilings_run(double* values, int n);

#ifdef __cplusplus
}
#endif
#endif /* USL_CEILINGS_H */
