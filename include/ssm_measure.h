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

#ifdef __cplusplus
}
#endif
#endif /* SSM_MEASURE_H_ */
