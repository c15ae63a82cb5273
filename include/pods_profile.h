/* pods_profile.h - per-launch timing of the PODS library's kernels, for benchmarks.
 *
 * Not part of the method and kept apart from its boundary (pods.h).  This is the one piece of state the
 * library keeps: per calling thread, a switch and a list of HIP event pairs.
 *
 * pods_profile_enable(1) makes every later library call on this thread bracket each of its kernel
 * launches with a pair of HIP events on the call's stream, and discards earlier records.
 * pods_profile_enable(0) stops recording and destroys the events (the device must have finished with
 * them: read the records first).  pods_profile_count() is the number of launches recorded so far;
 * pods_profile_get(i, ...) waits for launch i to finish (the only call here that synchronises with the
 * device) and returns the kernel's name (a static host string) and its duration in milliseconds.
 * While disabled, launches are not touched.
 */
#ifndef PODS_PROFILE_H_
#define PODS_PROFILE_H_

#include "pods.h"

#ifdef __cplusplus
extern "C" {
#endif

pods_status pods_profile_enable(int32_t enable);
int32_t pods_profile_count(void);
pods_status pods_profile_get(int32_t i, const char** name, float* ms);

/* Context for the token loss's matrix-core roofline: one launch of `workgroups` workgroups (4 wavefronts
 * each, one workgroup per compute unit at a time) that issue nothing but v_mfma_f32_32x32x16_bf16 on
 * register operands, `iters` x 32 per wavefront.  What this sustains is the ceiling the chip's clock and
 * power management leave to ANY kernel, beside the published peak.  Timed like every other launch (enable
 * the hooks, then read the record named "mfma only").
 *   sink   [1] float32 device, practically never written;  flops: HOST, out, floating-point operations of the launch */
pods_status pods_profile_mfma_only(int32_t workgroups, int32_t iters, float* sink, double* flops /* host */,
                                   void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PODS_PROFILE_H_ */
