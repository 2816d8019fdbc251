/*
 * ssm.h -- C ABI of libssmscan: the sequence-parallel training pass of the S5-style diagonal
 * state-space layer with episode resets, for one AMD MI355X (gfx950).
 *
 * Paper: "Accelerating Model-Based Reinforcement Learning with State-Space World Models".
 * The layer is the discrete linear system of the Preliminaries ("State-Space Models", Eq. 3)
 *        x_t = Abar x_{t-1} + Bbar u_t,        y_t = Cbar x_t + Dbar u_t
 * with a diagonal complex Abar, evaluated over the whole sequence by the associative scan of
 * Eq. 4-7, with the resettable elements and operator of the Methodology ("State-Space World
 * Model", Eq. 9-10) so that an episode boundary cuts the state.
 *
 * Conventions for every entry point
 *   - All array pointers are DEVICE pointers owned by the caller.  The library never allocates,
 *     frees or keeps them.  The only exception is marked "host".
 *   - complex64 = interleaved {float re, im} (bit-compatible with std::complex<float>).
 *     Arrays are dense, row-major, innermost index last.  Complex arrays must be 8-byte aligned,
 *     float arrays 4-byte aligned, the workspace 256-byte aligned.
 *   - Bt sequences, L steps, H = width of u and y (real), P = number of complex diagonal states.
 *   - is_first[b,t] != 0 marks a step whose incoming state is dropped (the flag element
 *     1 - c_k of Eq. 9): x_t = Bbar u_t there.  is_first[b,0] != 0 makes x0[b] irrelevant.
 *   - Calls validate their arguments on the host first and return an error code before any
 *     launch; otherwise they enqueue kernels on `stream` (a hipStream_t, NULL = default stream)
 *     and return without waiting.  No exceptions, no abort; concurrent calls are safe as long
 *     as they use distinct workspaces.
 *   - Outputs are overwritten, never accumulated into.  Outputs must not alias inputs.
 *   - The workspace must hold at least ssm_workspace_bytes(...) bytes; its contents are scratch
 *     and need not be initialised or preserved between calls.
 *   - Gradient of the real loss l w.r.t. a complex quantity q is returned as
 *     dl/dRe(q) + i dl/dIm(q).
 *   - The library reads no environment variable and keeps no state between calls other than the
 *     poll bound of ssm_set_spin_limit below.
 *   - The device pointers and the stream must belong to the copy of the HIP runtime the library is
 *     bound to.  A process that takes its memory from a framework which ships its own copy (PyTorch
 *     does) loads that framework before this library, so that both use one copy; bound to another,
 *     every launch fails with SSM_ERR_HIP.
 *   - Arithmetic of the projections: inputs, outputs and accumulation are fp32; the products run on
 *     the 16-bit matrix cores with both operands split while they are staged.  Where the largest
 *     magnitude of every operand is measured on the device as part of the call (ssm_scan_fwd /
 *     ssm_scan_bwd at shapes where every sequence is a whole number of 128-step tiles, L % 128 == 0
 *     and L <= 4096, or every 128 tokens are whole sequences, L = 16, 32, 64 with Bt * L a multiple of
 *     128, and the batch gives at least 64 tiles of 128 tokens x 64 states) an operand is staged as two
 *     fp16 planes of the operand scaled by a power of two (three partial products, errors at the level
 *     of fp32 products): u, x, dy and chi get a scale per token where tokens are the rows of the
 *     product, the weights and the operands of the sums over tokens one per matrix.  Under one scale
 *     with largest magnitude m an element a is held with an absolute error of at most
 *     max(2^-22 |a|, 2^-39 m): elements more than 2^17 below m are fixed-point, not floating-point.
 *     The same staging is used at other sequence lengths when H >= 512, P >= 512 and Bt * L is large
 *     enough that every product has more than 64 tiles of 128 x 128 (the scan kernels then record the
 *     largest magnitudes of x and chi), and by ssm_half_glu_* / ssm_block_* for the gate's products at
 *     widths that are multiples of 64 from 512 on with at least 200 tiles of 64 tokens x 128 columns.
 *     Everywhere else every operand is split exactly into three bf16 planes (six partial products).
 *     At the shapes named first the input projection and C^H dy also scan their own output tiles
 *     (no scan kernel, no round trip of Bbar u and C^H dy through memory).  Infinite inputs give NaN.
 */
#ifndef SSM_H_
#define SSM_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct { float re, im; } ssm_c64;

typedef enum {
    SSM_OK = 0,
    SSM_ERR_INVALID_ARG = 1,  /* NULL required pointer, non-positive dimension, misalignment */
    SSM_ERR_WORKSPACE = 2,    /* workspace NULL or smaller than ssm_workspace_bytes()        */
    SSM_ERR_UNSUPPORTED = 3,  /* dimension beyond SSM_MAX_*                                   */
    SSM_ERR_HIP = 4,          /* a HIP runtime call or kernel launch failed                   */
    SSM_ERR_SCAN_TIMEOUT = 5, /* reported by ssm_workspace_status(): a cross-block wait gave up */
    SSM_ERR_SCRATCH_LIMIT = 6 /* ssm_scan_states_noalloc: the shape needs more than the built-in scratch */
} ssm_status;

#define SSM_MAX_WIDTH 65536          /* largest H and largest P                        */
#define SSM_MAX_TOKENS 2147483647LL  /* largest Bt * L                                 */
#define SSM_MAX_ELEMS (1LL << 40)    /* largest Bt * L * max(H, 2P)                    */

/* Static description of an error code. Never NULL. */
const char *ssm_strerror(int status);

/* Library version, major * 100 + minor. */
int ssm_version(void);

/* Bound on the polls of one cross-workgroup wait (default 2^20, each poll sleeps about 128 clocks);
 * returns the previous value.  Process-wide and meant for tests: a bound of 0 makes every wait whose
 * predecessor is not ready yet give up at once, so the give-up path can be exercised while every
 * kernel still terminates.                                                                      */
uint32_t ssm_set_spin_limit(uint32_t polls);

/* Scratch bytes the forward (want_bwd = 0) or the gradient pass (want_bwd != 0) needs for the
 * given shape.  Returns 0 for an invalid or unsupported shape.  Pure host function.           */
size_t ssm_workspace_bytes(int64_t Bt, int64_t L, int64_t H, int64_t P, int want_bwd);

/* Zero-order-hold discretisation of the diagonal continuous system (Eq. 2 -> Eq. 3; the paper
 * only says the discrete matrices are functions of the continuous ones and the step, ZOH is the
 * reading used here):  Delta_p = exp(log_delta_p),  A_bar_p = exp(Lambda_p Delta_p),
 * B_bar[p,:] = (A_bar_p - 1)/Lambda_p * B[p,:]  (limit Delta_p * B[p,:] as Lambda_p -> 0).
 *   in : Lambda [P] c64, B [P,H] c64 (may be NULL iff B_bar is NULL), log_delta [P] f32
 *   out: A_bar [P] c64, B_bar [P,H] c64 (may be NULL)                                        */
ssm_status ssm_discretize(const ssm_c64 *Lambda, const ssm_c64 *B, const float *log_delta,
                          int64_t P, int64_t H, ssm_c64 *A_bar, ssm_c64 *B_bar, void *stream);

/* Forward pass of the layer over Bt sequences (Eq. 3 computed by the scan of Eq. 4-7 with the
 * reset operator of Eq. 10; the scan elements carry Bbar u_k, Eq. 6):
 *   x[b,t,:] = (is_first[b,t] ? 0 : A_bar (.) x[b,t-1,:]) + B_bar u[b,t,:],   x[b,-1,:] = x0[b,:]
 *   y[b,t,:] = Re(C x[b,t,:]) + D (.) u[b,t,:]
 *   in : Lambda [P] c64, B [P,H] c64, C [H,P] c64, D [H] f32, log_delta [P] f32,
 *        u [Bt,L,H] f32, is_first [Bt,L] u8 (NULL = no resets), x0 [Bt,P] c64 (NULL = zeros)
 *   out: y [Bt,L,H] f32; x [Bt,L,P] c64, the states, needed by ssm_scan_bwd (NULL allowed when
 *        no gradient pass follows); x_last [Bt,P] c64 = x[:,L-1,:] (NULL allowed), usable as the
 *        x0 of a call that continues the same sequences.                                        */
ssm_status ssm_scan_fwd(const ssm_c64 *Lambda, const ssm_c64 *B, const ssm_c64 *C, const float *D,
                        const float *log_delta, const float *u, const uint8_t *is_first,
                        const ssm_c64 *x0, int64_t Bt, int64_t L, int64_t H, int64_t P,
                        float *y, ssm_c64 *x, ssm_c64 *x_last,
                        void *workspace, size_t ws_bytes, void *stream);

/* Gradient pass matching ssm_scan_fwd for the loss l = sum(dy * y): a reverse-time scan of the
 * adjoint state chi_t = C^H dy_t + [not is_first_{t+1}] conj(A_bar) (.) chi_{t+1} with the same
 * reset operator (Eq. 10) run backwards, then the adjoints of the two projections and of the
 * discretisation.  The paper trains the layer with Adam and back-propagates first-order gradients
 * through the dynamics (Methodology, world-model loss and actor loss) without spelling this out.
 *   in : the eight inputs of the forward call with the same shapes, x [Bt,L,P] c64 as saved by
 *        the forward call, dy [Bt,L,H] f32
 *   out: du [Bt,L,H] f32, dLambda [P] c64, dB [P,H] c64, dC [H,P] c64, dD [H] f32,
 *        dlog_delta [P] f32, dx0 [Bt,P] c64 (NULL allowed)                                      */
ssm_status ssm_scan_bwd(const ssm_c64 *Lambda, const ssm_c64 *B, const ssm_c64 *C, const float *D,
                        const float *log_delta, const float *u, const uint8_t *is_first,
                        const ssm_c64 *x0, int64_t Bt, int64_t L, int64_t H, int64_t P,
                        const ssm_c64 *x, const float *dy,
                        float *du, ssm_c64 *dLambda, ssm_c64 *dB, ssm_c64 *dC, float *dD,
                        float *dlog_delta, ssm_c64 *dx0,
                        void *workspace, size_t ws_bytes, void *stream);

/* The resettable scan alone (Eq. 4 with the elements of Eq. 9 and the operator of Eq. 10) on
 * already projected elements, in place:  on entry v[b,t,p] holds the second component of the
 * scan element (Bbar u_t)_p, on return the state x[b,t,p].
 *   in : A_bar [P] c64 (any value, including 0), is_first [Bt,L] u8 or NULL, x0 [Bt,P] or NULL
 *   io : v [Bt,L,P] c64
 *   out: x_last [Bt,P] c64 (NULL allowed)
 * Workspace: ssm_workspace_bytes(Bt, L, 1, P, 0) suffices.                                     */
ssm_status ssm_scan_states(const ssm_c64 *A_bar, ssm_c64 *v, const uint8_t *is_first,
                           const ssm_c64 *x0, int64_t Bt, int64_t L, int64_t P, ssm_c64 *x_last,
                           void *workspace, size_t ws_bytes, void *stream);

/* The reverse-time scan of the gradient pass alone, in place: on entry gx[b,t,p] = (C^H dy_t)_p,
 * on return chi[b,t,p].  Also reduces dA_bar[p] = sum_{b,t} [not is_first[b,t]] conj(x[b,t-1,p])
 * chi[b,t,p] (x[b,-1] = x0[b]) and dx0[b,p] = [not is_first[b,0]] conj(A_bar_p) chi[b,0,p].
 *   in : A_bar [P], x [Bt,L,P], is_first or NULL, x0 or NULL
 *   io : gx [Bt,L,P]
 *   out: dA_bar [P] c64, dx0 [Bt,P] c64 (NULL allowed)
 * Workspace: ssm_workspace_bytes(Bt, L, 1, P, 1) suffices.                                     */
ssm_status ssm_scan_states_reverse(const ssm_c64 *A_bar, ssm_c64 *gx, const ssm_c64 *x,
                                   const uint8_t *is_first, const ssm_c64 *x0,
                                   int64_t Bt, int64_t L, int64_t P, ssm_c64 *dA_bar, ssm_c64 *dx0,
                                   void *workspace, size_t ws_bytes, void *stream);

/* ssm_scan_states for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels
 * and bit-identical results; the scratch (status header, ticket counters and look-back descriptors of
 * sequences longer than 256 steps) lives in a device array that is part of the library image, one
 * copy per GPU, SSM_NOALLOC_SCRATCH_BYTES long.  The call allocates nothing and frees nothing.
 * A shape whose scratch (ssm_workspace_bytes(Bt, L, 1, P, 0), about Bt * L * P / 8 bytes for L > 256,
 * 256 bytes otherwise) exceeds that size is refused with SSM_ERR_SCRATCH_LIMIT before any launch.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams,
 * two host threads) race on it and must be serialised by the caller; consecutive calls on one stream
 * are fine (what must start at zero is cleared by the call itself, with a kernel).
 * ssm_scan_states_noalloc_status is ssm_workspace_status for that array on the current device.    */
#define SSM_NOALLOC_SCRATCH_BYTES (8u << 20)
ssm_status ssm_scan_states_noalloc(const ssm_c64 *A_bar, ssm_c64 *v, const uint8_t *is_first,
                                   const ssm_c64 *x0, int64_t Bt, int64_t L, int64_t P, ssm_c64 *x_last,
                                   void *stream);
ssm_status ssm_scan_states_noalloc_status(void *stream);

/* Step (recurrent) mode: one transition of the sequence model, x_t, y_t = SSM(u_t, is_first_t,
 * x_{t-1}) (the sequence-model line of Eq. 8), as the imagination roll-out of the actor-critic
 * stage needs it: there the next input depends on the previous output, so the H roll-out steps
 * cannot be scanned (Methodology, "Actor-Critic Learning", Eq. 13).
 *   x[b,:] = (is_first[b] ? 0 : A_bar (.) x_prev[b,:]) + B_bar u[b,:],   y[b,:] = Re(C x[b,:]) + D (.) u[b,:]
 * The discretised, packed parameters are prepared once per roll-out into a caller-owned plan
 * buffer of ssm_step_plan_bytes(H, P) bytes (256-byte aligned) and reused by every step.
 *   ssm_step_prepare  in : Lambda [P] c64, B [P,H] c64, C [H,P] c64, log_delta [P] f32;  out: plan
 *   ssm_step          in : plan, D [H] f32, u [Bt,H] f32, x_prev [Bt,P] c64 (NULL = zeros),
 *                          is_first [Bt] u8 (NULL = none)
 *                     out: x [Bt,P] c64 (must not alias x_prev), y [Bt,H] f32                     */
size_t ssm_step_plan_bytes(int64_t H, int64_t P);
ssm_status ssm_step_prepare(const ssm_c64 *Lambda, const ssm_c64 *B, const ssm_c64 *C,
                            const float *log_delta, int64_t H, int64_t P,
                            void *plan, size_t plan_bytes, void *stream);
ssm_status ssm_step(const void *plan, size_t plan_bytes, const float *D, const float *u,
                    const ssm_c64 *x_prev, const uint8_t *is_first, int64_t Bt, int64_t H, int64_t P,
                    ssm_c64 *x, float *y, void *stream);

/* Adjoint of one ssm_step with respect to its input and its incoming state: the first-order
 * gradients that the actor's loss sends back through the imagined trajectory ("Actor-Critic
 * Training": gradients are backpropagated through the dynamics model).  The world model's
 * parameters are fixed in that stage, so no parameter gradients are formed.
 *   gx[b,:]      = C^H dy[b,:] + dx[b,:]               (total gradient with respect to x_t)
 *   dx_prev[b,:] = [not is_first[b]] conj(A_bar) (.) gx[b,:]
 *   du[b,:]      = Re(B_bar^H gx[b,:]) + D (.) dy[b,:]
 *   in : plan (from ssm_step_prepare), D [H], dy [Bt,H] f32, dx [Bt,P] c64 (gradient arriving from
 *        step t+1, NULL = zeros), is_first [Bt] u8 (the flags of THIS step, NULL = none)
 *   out: gx [Bt,P] c64, du [Bt,H] f32, dx_prev [Bt,P] c64 (NULL allowed); gx, dx, dx_prev distinct */
ssm_status ssm_step_bwd(const void *plan, size_t plan_bytes, const float *D, const float *dy,
                        const ssm_c64 *dx, const uint8_t *is_first, int64_t Bt, int64_t H, int64_t P,
                        ssm_c64 *gx, float *du, ssm_c64 *dx_prev, void *stream);

/* Bootstrapped lambda-return, the critic's target of the actor-critic stage ("Actor-Critic
 * Training", Eq. 14):
 *   V_t = r_t + gamma c_t ((1 - lambda) v_t + lambda V_{t+1}),   V_T = v_T
 * a reverse-time linear recurrence with a coefficient that changes every step.  Arrays are
 * TIME-MAJOR [T, N] f32 (row t = step t of N imagined trajectories, as a roll-out produces them);
 * row T-1 is the paper's last step, whose return is the value itself.  The value that enters step
 * t is v_t as printed (a caller who bootstraps with v_{t+1} passes the shifted array).
 *   ssm_lambda_return      in : reward, cont, value [T,N];                    out: ret [T,N]
 *   ssm_lambda_return_bwd  in : cont, value, ret (from the forward call), dret [T,N]
 *                          out: dreward, dcont, dvalue [T,N] = gradients of sum(dret (.) ret)
 *                               (first-order gradients through the imagined trajectory)
 * No workspace.  Outputs must not alias inputs.                                                 */
ssm_status ssm_lambda_return(const float *reward, const float *cont, const float *value,
                             float gamma, float lambda, int64_t T, int64_t N, float *ret, void *stream);
ssm_status ssm_lambda_return_bwd(const float *cont, const float *value, const float *ret,
                                 const float *dret, float gamma, float lambda, int64_t T, int64_t N,
                                 float *dreward, float *dcont, float *dvalue, void *stream);

/* half-GLU gate of the S5 sequence layer (appendix "S5 Sequence Layer"):
 *   x1 = GELU(u),   y = u (.) sigmoid(W^T x1)       i.e. y[t,j] = u[t,j] sigmoid(sum_i W[i,j] x1[t,i])
 * with the exact Gaussian GELU x Phi(x).  u, y [T,H] f32 row-major (T = Bt*L tokens), W [H,H] f32.
 *   ssm_half_glu_fwd  in : u (16-byte aligned), W;   out: y, gate [T,H] = sigmoid(W^T x1) (NULL
 *                          allowed when no gradient pass follows)
 *   ssm_half_glu_bwd  in : u, W, gate (from the forward call), dy [T,H] (16-byte aligned)
 *                     out: du [T,H], dW [H,H] = gradients of sum(dy (.) y)
 * Workspace: ssm_half_glu_workspace_bytes(T, H, want_bwd) bytes, 256-byte aligned (0 = invalid
 * or unsupported shape).  Outputs must not alias inputs or the workspace.                        */
size_t ssm_half_glu_workspace_bytes(int64_t T, int64_t H, int want_bwd);
ssm_status ssm_half_glu_fwd(const float *u, const float *W, int64_t T, int64_t H,
                            float *y, float *gate, void *workspace, size_t ws_bytes, void *stream);
ssm_status ssm_half_glu_bwd(const float *u, const float *W, const float *gate, const float *dy,
                            int64_t T, int64_t H, float *du, float *dW,
                            void *workspace, size_t ws_bytes, void *stream);

/* The S5 sequence layer as the appendix draws it from the parts the text defines: the resettable SSM
 * layer followed by the half-GLU gate, out = y (.) sigmoid(W^T GELU(y)) with y the layer's output.
 * The output projection stores GELU(y) next to y, so the gate costs one more product and no
 * separate element-wise pass.  Arguments as in ssm_scan_fwd / ssm_scan_bwd and ssm_half_glu_*.
 *   ssm_block_fwd  out: y [Bt,L,H] (the layer's output, needed by the gradient pass), out [Bt,L,H],
 *                       gate [Bt,L,H] (NULL allowed when no gradient pass follows), x, x_last
 *   ssm_block_bwd  in : x, y, gate (from the forward call), dout [Bt,L,H] (16-byte aligned, as y and gate)
 *                  out: the gradients of ssm_scan_bwd and dW [H,H]
 * Workspace: ssm_block_workspace_bytes(Bt, L, H, P, want_bwd).  ssm_workspace_status applies.   */
size_t ssm_block_workspace_bytes(int64_t Bt, int64_t L, int64_t H, int64_t P, int want_bwd);
ssm_status ssm_block_fwd(const ssm_c64 *Lambda, const ssm_c64 *B, const ssm_c64 *C, const float *D,
                         const float *log_delta, const float *W, const float *u, const uint8_t *is_first,
                         const ssm_c64 *x0, int64_t Bt, int64_t L, int64_t H, int64_t P,
                         float *y, float *out, float *gate, ssm_c64 *x, ssm_c64 *x_last,
                         void *workspace, size_t ws_bytes, void *stream);
ssm_status ssm_block_bwd(const ssm_c64 *Lambda, const ssm_c64 *B, const ssm_c64 *C, const float *D,
                         const float *log_delta, const float *W, const float *u, const uint8_t *is_first,
                         const ssm_c64 *x0, int64_t Bt, int64_t L, int64_t H, int64_t P,
                         const ssm_c64 *x, const float *y, const float *gate, const float *dout,
                         float *du, ssm_c64 *dLambda, ssm_c64 *dB, ssm_c64 *dC, float *dD, float *dlog_delta,
                         ssm_c64 *dx0, float *dW, void *workspace, size_t ws_bytes, void *stream);

/* Waits for `stream` and reports whether any scan launched with this workspace since its last
 * use gave up a bounded cross-block wait (SSM_ERR_SCAN_TIMEOUT) or SSM_OK.  Long sequences are
 * split over several workgroups that hand their running state forward; every such wait is bounded
 * so that a kernel always terminates.  A wait that gives up hands on NaN: the states that depend on
 * it, and everything computed from them, are NaN, so the failure cannot pass as data even for a
 * caller who never asks here.                                                                   */
ssm_status ssm_workspace_status(const void *workspace, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SSM_H_ */
