/*
 * ssm_measure.h -- measurement aids of libssmscan (no operation of the paper): the forward and the
 * gradient pass with a HIP event recorded on the caller's stream around every kernel, so that a
 * benchmark can time the kernels of the path on the stream they are launched on.
 */
#ifndef SSM_MEASURE_H_
#define SSM_MEASURE_H_

#include "ssm.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Number of per-stage timings written by the *_profiled calls. */
#define SSM_FWD_STAGES 4
#define SSM_BWD_STAGES 6

/* The same code path as ssm_scan_fwd / ssm_scan_bwd.  They wait for the stream before returning and
 * write the milliseconds of each stage to the HOST array stage_ms:
 *   forward : [0] discretise+pack, [1] input projection, [2] scan, [3] output projection
 *   backward: [0] discretise+pack and dD partials, [1] gx = C^H dy (with the reverse scan in its tiles
 *             where the shape allows), [2] reverse scan kernel, [3] du with the dBbar and dC partials
 *             (one launch), [4] empty (the sum of the two halves of du shares the next launch),
 *             [5] parameter epilogue
 * A stage that holds no kernel on this call (a scan that runs inside its projection, a product that
 * is not run as two halves) reads as the few microseconds between two events.                   */
ssm_status ssm_scan_fwd_profiled(const ssm_c64 *Lambda, const ssm_c64 *B, const ssm_c64 *C,
                                 const float *D, const float *log_delta, const float *u,
                                 const uint8_t *is_first, const ssm_c64 *x0,
                                 int64_t Bt, int64_t L, int64_t H, int64_t P,
                                 float *y, ssm_c64 *x, ssm_c64 *x_last,
                                 void *workspace, size_t ws_bytes, void *stream,
                                 float *stage_ms /* host, [SSM_FWD_STAGES] */);
ssm_status ssm_scan_bwd_profiled(const ssm_c64 *Lambda, const ssm_c64 *B, const ssm_c64 *C,
                                 const float *D, const float *log_delta, const float *u,
                                 const uint8_t *is_first, const ssm_c64 *x0,
                                 int64_t Bt, int64_t L, int64_t H, int64_t P,
                                 const ssm_c64 *x, const float *dy,
                                 float *du, ssm_c64 *dLambda, ssm_c64 *dB, ssm_c64 *dC, float *dD,
                                 float *dlog_delta, ssm_c64 *dx0,
                                 void *workspace, size_t ws_bytes, void *stream,
                                 float *stage_ms /* host, [SSM_BWD_STAGES] */);

/* What ssm_scan_fwd / ssm_scan_bwd would launch for a shape: host logic only, no GPU call.  Writes
 * SSM_PLAN_FIELDS int32 values to the HOST array out:
 *   [0] 1 when the input projection and C^H dy scan their own output tiles (no scan kernel)
 *   [1] planes per operand of the layer's products: 2 (scaled fp16) or 3 (bf16)
 *   [2] K slabs of dC, [3] K slabs of dBbar
 *   [4] gradient pass: 3 = du, dBbar slabs and dC slabs in one launch; 2 = two launches of two products
 *   [5] 1 when the slab work items take the first slots of the launch of [4] == 3
 *   [6], [7] the same for the launches of C^H dy with dC and of du with dBbar when [4] == 2
 *   [8] 1 when du runs as two K halves that the parameter epilogue's launch adds
 *   [9] tile tier of the input projection, [10] of the output projection (0: 128x128x32, 1: 64x128x32, 2: 64x64x64)
 *   [11] workgroups along time of the scan kernels (1: no look-back; unused when [0] == 1)
 * Returns SSM_ERR_INVALID_ARG / SSM_ERR_UNSUPPORTED for shapes the library does not take.           */
#define SSM_PLAN_FIELDS 12
ssm_status ssm_plan_describe(int64_t Bt, int64_t L, int64_t H, int64_t P, int32_t *out /* host */);

#ifdef __cplusplus
}
#endif
#endif /* SSM_MEASURE_H_ */
