// Device-side description of one projection problem and the store functions (epilogues) of the
// projection GEMM (gfx950):
//
//   C[m,n] = f( sum_k A(m,k) * B(n,k) )
//
// The hardware deals workgroup ids round-robin to the 8 XCDs; the kernel remaps them so that each
// XCD works on a contiguous band of tiles (or on whole K slabs) and re-reads its operands from its
// own L2 (see gemm_place in gemm_kernel.h).
#pragma once

#include "ssm_internal.h"

namespace ssm {

typedef float v16f __attribute__((ext_vector_type(16)));

struct GemmDev {
    const float *A; long lda;
    const float *B; long ldb;
    float *C; long ldc;
    const float *diag; const float *E; long lde;
    const float *E2; float *C2;                     // gate epilogues (pitch lde / ldc)
    const uint8_t *rowflag;
    int M, N, K, kper;      // kper: K range per split (multiple of the K tile)
    int ntm, ntn, per_xcd;
    // placement of the (tile, split) work items on the 8 XCDs: slots per XCD, mapping mode and its
    // parameter, first slot of this problem in a launch that carries several
    int splits, nx, mode, mpar, slot0;
    // epilogue 7 (scan over the tile's rows): tiles per sequence, column tiles per unit, column
    // groups per sequence, number of units (a unit = the chains of one sequence and column group)
    ScanEpilogue scan;
    int sc_nt, sc_cpu, sc_ncg, sc_units, sc_rev;
    AbsMax amaxA, amaxB;    // two-plane fp16 staging only
    unsigned *c2_rowmax;    // epilogue 6 on tiles whose wavefronts own 64 columns: [ceil(N/64)][M] largest magnitudes of C2, or null
};

// Value stored for an output element whose accumulated product is v.
//   EPI 0: v
//   EPI 1: v + diag[col] * E[row, col]                   (D (.) u and D (.) dy)
//   EPI 2: columns are interleaved (re, im) pairs of complex states; diag holds Abar as
//          interleaved complex; adds [not rowflag[row]] * (Abar_p * E_p)[re or im]: the carried
//          state Abar x_{t-1} of one recurrence step (Eq. 3, first line)
//   EPI 3: half-GLU gate (S5 sequence layer appendix): s = sigmoid(v) is kept in C2 when asked
//          and the stored value is E[row, col] * s        (E = the gated input u)
//   EPI 4: adjoint of the gate with respect to its input: E + v * E2
//          (E = dy (.) s and E2 = GELU'(u), both formed by the element-wise pass before the product; v = dz W^T)
//   EPI 6: v + diag[col] * E[row, col] as EPI 1, and GELU of that value into C2 (the output
//          projection feeding the half-GLU gate of the S5 block)
//   EPI 5 (bf16x3 kernel only, handled where the tile is stored because it needs the partner
//          column): adjoint of one recurrence step.  Columns are (re, im) pairs; the stored value is
//          g = v + E (E = the gradient that arrives from the next step, may be null) and C2 gets
//          [not rowflag[row]] conj(Abar) g, the gradient handed to the previous step (diag = Abar)
__device__ __forceinline__ float gelu_derivative(float x)
{
    // d/dx [x Phi(x)] = Phi(x) + x phi(x)
    const float cdf = 0.5f * erfcf(-0.70710678118654752f * x);
    const float pdf = 0.39894228040143268f * __expf(-0.5f * x * x);
    return fmaf(x, pdf, cdf);
}
__device__ __forceinline__ float gelu_value(float x)
{
    // x Phi(x) with Phi(x) = erfc(-x / sqrt 2) / 2 (no cancellation in the lower tail)
    return 0.5f * x * erfcf(-0.70710678118654752f * x);
}
__device__ __forceinline__ float sigmoidf(float z)
{
    // e^-|z| never overflows; both branches are exact rewrites of 1 / (1 + e^-z)
    const float e = __expf(-fabsf(z));
    const float r = 1.f / (1.f + e);
    return z >= 0.f ? r : e * r;
}
template <int EPI>
__device__ __forceinline__ float gemm_epilogue_apply(const GemmDev &g, long row, int col, float v)
{
    // (explicitly fused: v may itself be a product that the compiler could fuse with this sum instead,
    // and every instantiation must round the same way)
    if (EPI == 1) return fmaf(g.diag[col], g.E[row * g.lde + col], v);
    if (EPI == 2) {
        if (g.rowflag && g.rowflag[row]) return v;
        const float lr = g.diag[col & ~1], li = g.diag[col | 1];
        const float own = g.E[row * g.lde + col], other = g.E[row * g.lde + (col ^ 1)];
        return v + ((col & 1) ? fmaf(lr, own, li * other) : fmaf(lr, own, -li * other));
    }
    if (EPI == 3) {
        const float s = sigmoidf(v);
        if (g.C2) g.C2[row * g.ldc + col] = s;
        return g.E[row * g.lde + col] * s;
    }
    if (EPI == 4) {
        const long i = row * g.lde + col;
        return fmaf(v, g.E2[i], g.E[i]);
    }
    if (EPI == 6) {
        const float y = fmaf(g.diag[col], g.E[row * g.lde + col], v);
        g.C2[row * g.ldc + col] = gelu_value(y);
        return y;
    }
    return v;
}
// second output of EPI 5: (conj(Abar_p) g_p)[re or im] given the element's own part and its partner's
__device__ __forceinline__ float gemm_carry_adjoint(const GemmDev &g, long row, int col, float own, float other)
{
    if (g.rowflag && g.rowflag[row]) return 0.f;
    const float lr = g.diag[col & ~1], li = g.diag[col | 1];
    return (col & 1) ? fmaf(lr, own, -li * other) : fmaf(lr, own, li * other);
}

}  // namespace ssm
