/*
 * CPU oracle for the resettable S5-style diagonal SSM layer (forward + gradient pass).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the slow, plain float64 statement of what the layer
 * computes, used only by the test-suite, the smoke check and the benchmark's CPU-baseline
 * leg.  It shares no code, header, table or helper with the HIP library and neither side
 * includes or links the other.
 *
 * What it follows (paper: "Accelerating Model-Based Reinforcement Learning with State-Space
 * World Models"):
 *   - Preliminaries, "State-Space Models": the continuous system (Eq. 2) and its discrete
 *     recurrence x_t = Abar x_{t-1} + Bbar u_t,  y_t = Cbar x_t + Dbar u_t  (Eq. 3).
 *   - The scan elements e_k = (Abar, Bbar u_k) (Eq. 6) and the worked unrolling (Eq. 7): the
 *     parallel scan reaches exactly the states of this sequential loop, so the oracle IS the
 *     sequential loop.
 *   - Methodology, "State-Space World Model": the resettable elements (Eq. 9) and operator
 *     (Eq. 10): an element whose reset flag is set discards everything to its left, i.e. the
 *     incoming state is dropped and the step's own input Bbar u_k still enters.
 *   - The sequence model line of Eq. 8: SSM(..., c_{t-1}, x_{t-1}) takes a previous state, hence
 *     the optional initial state x0.
 *
 * Readings where the paper is silent (all listed in the repository's design notes):
 *   - Discretisation is zero-order hold with a learnable per-state step: Delta = exp(log_delta),
 *     Abar = exp(Lambda Delta) (diagonal), Bbar = Lambda^{-1}(Abar - I) B, Cbar = C, Dbar = D.
 *   - u, y are real of width H; the state is complex of size P; y = Re(C x) + D (.) u with a
 *     diagonal real feed-through D.
 *   - is_first[b,t] != 0 marks the step whose incoming state is dropped; is_first[b,0] != 0
 *     makes x0 irrelevant.
 *   - Gradients of a real loss l w.r.t. a complex quantity q are returned as
 *     dl/dRe(q) + i dl/dIm(q).
 *
 * Complex arrays are interleaved (re, im) doubles, row-major, innermost index last.
 * All gradient formulas are the adjoint of the forward loop, written in reverse time; they are
 * only trusted because the test-suite checks them against central finite differences of the
 * forward function (see ssm_oracle.py: fd_gradients).
 *
 * Build: gcc -O2 -fopenmp -fcx-limited-range -shared -fPIC ssm_oracle.c -o libssm_oracle.so -lm
 */
#include <complex.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef double complex zc;

/* exp(z) - 1 without cancellation for small |z|:
 * e^a cos b - 1 = expm1(a) cos b - 2 sin^2(b/2),  Im = e^a sin b.                        */
static zc expm1_complex(zc z)
{
    double a = creal(z), b = cimag(z);
    double s = sin(0.5 * b);
    return (expm1(a) * cos(b) - 2.0 * s * s) + I * (exp(a) * sin(b));
}

/* psi(z) = (e^z - 1)/z, psi(0) = 1. */
static zc psi0(zc z)
{
    if (creal(z) == 0.0 && cimag(z) == 0.0) return 1.0;
    return expm1_complex(z) / z;
}

/* psi'(z) = (z e^z - e^z + 1)/z^2 = sum_{k>=0} z^k (k+1)/(k+2)!.
 * The closed form cancels badly for small |z|, so the series is used there.            */
static zc psi1(zc z)
{
    if (cabs(z) < 0.5) {
        zc term = 0.5, sum = 0.5;          /* k = 0: 1/2! */
        for (int k = 1; k < 40; ++k) {
            /* ratio of consecutive coefficients: ((k+1)/(k+2)!) / (k/(k+1)!) = (k+1)/(k(k+2)) */
            term *= z * ((double)(k + 1) / ((double)k * (double)(k + 2)));
            sum += term;
        }
        return sum;
    }
    return (cexp(z) - psi0(z)) / z;
}

/* Zero-order-hold discretisation of the diagonal system (Eq. 3 with the ZOH reading).
 * Abar_p = exp(Lambda_p Delta_p);  g_p = (Abar_p - 1)/Lambda_p = Delta_p psi(Lambda_p Delta_p)
 * so that Bbar[p,:] = g_p B[p,:].                                                        */
void ssm_oracle_discretize(const double *Lambda_, const double *log_delta, long P,
                           double *Abar_, double *g_)
{
    const zc *Lambda = (const zc *)Lambda_;
    zc *Abar = (zc *)Abar_, *g = (zc *)g_;
    for (long p = 0; p < P; ++p) {
        double delta = exp(log_delta[p]);
        zc z = Lambda[p] * delta;
        Abar[p] = cexp(z);
        g[p] = delta * psi0(z);
    }
}

/* The resettable diagonal recurrence alone (Eq. 3 first line + Eq. 9-10), on already
 * projected inputs v = Bbar u:   x_t = (is_first_t ? 0 : Abar x_{t-1}) + v_t.
 * v, x: [Bt, L, P] complex; Abar: [P]; is_first: [Bt, L] or NULL; x0: [Bt, P] or NULL.   */
void ssm_oracle_scan(const double *Abar_, const double *v_, const uint8_t *is_first,
                     const double *x0_, long Bt, long L, long P, double *x_)
{
    const zc *Abar = (const zc *)Abar_, *v = (const zc *)v_, *x0 = (const zc *)x0_;
    zc *x = (zc *)x_;
    for (long b = 0; b < Bt; ++b)
        for (long t = 0; t < L; ++t) {
            int first = is_first ? (is_first[b * L + t] != 0) : 0;
            for (long p = 0; p < P; ++p) {
                zc prev = (t == 0) ? (x0 ? x0[b * P + p] : 0.0) : x[(b * L + t - 1) * P + p];
                zc carried = first ? 0.0 : Abar[p] * prev;
                x[(b * L + t) * P + p] = carried + v[(b * L + t) * P + p];
            }
        }
}

/* Forward pass of the whole layer.
 *   Lambda [P] c, B [P,H] c, C [H,P] c, D [H], log_delta [P], u [Bt,L,H],
 *   is_first [Bt,L] or NULL, x0 [Bt,P] c or NULL
 *   -> y [Bt,L,H], x [Bt,L,P] c (required), x_last [Bt,P] c (may be NULL).
 * Sequences are independent; `nthreads` > 1 only distributes them over cores.            */
int ssm_oracle_fwd(const double *Lambda_, const double *B_, const double *C_, const double *D,
                   const double *log_delta, const double *u, const uint8_t *is_first,
                   const double *x0_, long Bt, long L, long H, long P,
                   double *y, double *x_, double *x_last_, int nthreads)
{
    const zc *B = (const zc *)B_, *C = (const zc *)C_, *x0 = (const zc *)x0_;
    zc *x = (zc *)x_, *x_last = (zc *)x_last_;
    zc *Abar = malloc(sizeof(zc) * P), *g = malloc(sizeof(zc) * P);
    if (!Abar || !g) { free(Abar); free(g); return 1; }
    ssm_oracle_discretize(Lambda_, log_delta, P, (double *)Abar, (double *)g);
    if (nthreads < 1) nthreads = 1;

#pragma omp parallel for num_threads(nthreads) schedule(static)
    for (long b = 0; b < Bt; ++b) {
        for (long t = 0; t < L; ++t) {
            const double *ut = u + (b * L + t) * H;
            zc *xt = x + (b * L + t) * P;
            int first = is_first ? (is_first[b * L + t] != 0) : 0;
            for (long p = 0; p < P; ++p) {
                zc Bu = 0.0;                                   /* (B u_t)_p */
                for (long h = 0; h < H; ++h) Bu += B[p * H + h] * ut[h];
                zc prev = (t == 0) ? (x0 ? x0[b * P + p] : 0.0) : x[(b * L + t - 1) * P + p];
                zc carried = first ? 0.0 : Abar[p] * prev;
                xt[p] = carried + g[p] * Bu;                   /* Abar x_{t-1} + Bbar u_t */
            }
            double *yt = y + (b * L + t) * H;
            for (long h = 0; h < H; ++h) {
                zc Cx = 0.0;
                for (long p = 0; p < P; ++p) Cx += C[h * P + p] * xt[p];
                yt[h] = creal(Cx) + D[h] * ut[h];              /* Re(C x_t) + D u_t */
            }
        }
        if (x_last)
            for (long p = 0; p < P; ++p) x_last[b * P + p] = x[(b * L + L - 1) * P + p];
    }
    free(Abar); free(g);
    return 0;
}

/* Gradient pass for the real loss l = sum(dy * y) (dy is the upstream gradient of y).
 * Inputs as in the forward, plus the saved states x [Bt,L,P] and dy [Bt,L,H].
 * Outputs (all required except dx0): du [Bt,L,H], dLambda [P] c, dB [P,H] c, dC [H,P] c,
 * dD [H], dlog_delta [P], dx0 [Bt,P] c (NULL allowed).
 *
 * Reverse of the forward loop.  With chi_t = dl/dx_t (the adjoint state):
 *   gx_t  = C^H dy_t                               (adjoint of y_t = Re(C x_t) + ...)
 *   chi_t = gx_t + [t+1 < L and not is_first_{t+1}] conj(Abar) chi_{t+1}
 *   dAbar += [not is_first_t] conj(x_{t-1}) chi_t   (x_{-1} = x0)
 *   dBbar += chi_t u_t^T,  du_t = D dy_t + Re(Bbar^H chi_t),  dC += dy_t x_t^H,  dD += dy_t u_t
 * then through Bbar = g B, g = Delta psi(Lambda Delta), Abar = exp(Lambda Delta):
 *   dB = conj(g) dBbar,  dg_p = sum_h conj(B[p,h]) dBbar[p,h]
 *   dLambda = conj(Delta Abar) dAbar + conj(Delta^2 psi'(z)) dg
 *   dDelta  = Re(conj(Lambda Abar) dAbar + conj(Abar) dg)       (d g / d Delta = Abar)
 *   dlog_delta = Delta dDelta
 */
int ssm_oracle_bwd(const double *Lambda_, const double *B_, const double *C_, const double *D,
                   const double *log_delta, const double *u, const uint8_t *is_first,
                   const double *x0_, long Bt, long L, long H, long P,
                   const double *x_, const double *dy,
                   double *du, double *dLambda_, double *dB_, double *dC_, double *dD,
                   double *dlog_delta, double *dx0_, int nthreads)
{
    const zc *Lambda = (const zc *)Lambda_, *B = (const zc *)B_, *C = (const zc *)C_;
    const zc *x0 = (const zc *)x0_, *x = (const zc *)x_;
    zc *dLambda = (zc *)dLambda_, *dB = (zc *)dB_, *dC = (zc *)dC_, *dx0 = (zc *)dx0_;
    if (nthreads < 1) nthreads = 1;
    if (nthreads > Bt) nthreads = (int)Bt;

    zc *Abar = malloc(sizeof(zc) * P), *g = malloc(sizeof(zc) * P);
    /* one private accumulator set per worker, summed in worker order afterwards */
    size_t per = (size_t)P * H + (size_t)H * P + P;          /* dBbar, dC, dAbar */
    zc *accz = calloc((size_t)nthreads * per, sizeof(zc));
    double *accD = calloc((size_t)nthreads * H, sizeof(double));
    zc *chi_buf = malloc(sizeof(zc) * 2 * P * nthreads);
    if (!Abar || !g || !accz || !accD || !chi_buf) {
        free(Abar); free(g); free(accz); free(accD); free(chi_buf); return 1;
    }
    ssm_oracle_discretize(Lambda_, log_delta, P, (double *)Abar, (double *)g);

#pragma omp parallel num_threads(nthreads)
    {
#ifdef _OPENMP
        int w = omp_get_thread_num();
#else
        int w = 0;
#endif
        zc *dBbar = accz + (size_t)w * per, *dCw = dBbar + (size_t)P * H, *dAbar = dCw + (size_t)H * P;
        double *dDw = accD + (size_t)w * H;
        zc *chi = chi_buf + (size_t)w * 2 * P, *chi_next = chi + P;

#pragma omp for schedule(static)
        for (long b = 0; b < Bt; ++b) {
            for (long p = 0; p < P; ++p) chi_next[p] = 0.0;
            for (long t = L - 1; t >= 0; --t) {
                const double *dyt = dy + (b * L + t) * H, *ut = u + (b * L + t) * H;
                const zc *xt = x + (b * L + t) * P;
                double *dut = du + (b * L + t) * H;
                int first = is_first ? (is_first[b * L + t] != 0) : 0;
                int next_first = (t + 1 < L && is_first) ? (is_first[b * L + t + 1] != 0) : 0;

                for (long h = 0; h < H; ++h) {
                    dut[h] = D[h] * dyt[h];
                    dDw[h] += dyt[h] * ut[h];
                }
                for (long p = 0; p < P; ++p) {
                    zc gx = 0.0;                                   /* (C^H dy_t)_p */
                    for (long h = 0; h < H; ++h) gx += conj(C[h * P + p]) * dyt[h];
                    zc carried = (t + 1 < L && !next_first) ? conj(Abar[p]) * chi_next[p] : 0.0;
                    chi[p] = gx + carried;
                    zc prev = (t == 0) ? (x0 ? x0[b * P + p] : 0.0) : x[(b * L + t - 1) * P + p];
                    if (!first) dAbar[p] += conj(prev) * chi[p];
                    for (long h = 0; h < H; ++h) {
                        dCw[h * P + p] += dyt[h] * conj(xt[p]);
                        dBbar[p * H + h] += chi[p] * ut[h];
                        dut[h] += creal(conj(g[p] * B[p * H + h]) * chi[p]);
                    }
                }
                if (t == 0 && dx0)
                    for (long p = 0; p < P; ++p)
                        dx0[b * P + p] = first ? 0.0 : conj(Abar[p]) * chi[p];
                zc *tmp = chi; chi = chi_next; chi_next = tmp;
            }
        }
    }

    /* reduce the workers' accumulators in a fixed order */
    for (int w = 1; w < nthreads; ++w) {
        for (size_t i = 0; i < per; ++i) accz[i] += accz[(size_t)w * per + i];
        for (long h = 0; h < H; ++h) accD[h] += accD[(size_t)w * H + h];
    }
    const zc *dBbar = accz, *dCsum = accz + (size_t)P * H, *dAbar = dCsum + (size_t)H * P;
    for (long h = 0; h < H; ++h) dD[h] = accD[h];
    for (size_t i = 0; i < (size_t)H * P; ++i) dC[i] = dCsum[i];
    for (long p = 0; p < P; ++p) {
        double delta = exp(log_delta[p]);
        zc z = Lambda[p] * delta;
        zc dg = 0.0;
        for (long h = 0; h < H; ++h) {
            dB[p * H + h] = conj(g[p]) * dBbar[p * H + h];
            dg += conj(B[p * H + h]) * dBbar[p * H + h];
        }
        dLambda[p] = conj(delta * Abar[p]) * dAbar[p] + conj(delta * delta * psi1(z)) * dg;
        double dDelta = creal(conj(Lambda[p] * Abar[p]) * dAbar[p] + conj(Abar[p]) * dg);
        dlog_delta[p] = delta * dDelta;
    }
    free(Abar); free(g); free(accz); free(accD); free(chi_buf);
    return 0;
}

int ssm_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
