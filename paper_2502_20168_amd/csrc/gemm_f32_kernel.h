// fp32 MFMA GEMM kernel template for the dense projections of the S5 layer (gfx950).
//
//   C[m,n] = sum_k A(m,k) * B(n,k)  (+ diag[n] * E[m,n])
//
// A workgroup of WGM x WGN wavefronts owns a BM x BN tile of C; each wavefront accumulates
// (BM/WGM) x (BN/WGN) outputs in v_mfma_f32_32x32x2_f32 tiles.  Operand tiles are staged
// global -> registers -> LDS, with the global loads of the next K tile in flight while the
// current one feeds the matrix cores.  Both operands sit in LDS as [k][row]: the 32 lanes that
// share a k index read 32 consecutive words, which is conflict-free whatever the global layout.
// Tiles are sized so that several workgroups share a CU: the fp32 MFMA is slow enough (64 cycles
// for 4096 flops) that operand traffic is cheap, and a second wavefront per SIMD fills the
// bubbles the first one leaves at its barriers.
// The hardware deals workgroup ids round-robin to the 8 XCDs; ids are remapped so that each
// XCD works on a contiguous band of tiles and re-reads its band of A from its own L2.
#pragma once

#include "ssm_internal.h"

namespace ssm {

typedef float v16f __attribute__((ext_vector_type(16)));

struct GemmDev {
    const float *A; long lda;
    const float *B; long ldb;
    float *C; long ldc;
    const float *diag; const float *E; long lde;
    const float *E2; const float *E3; float *C2;    // gate epilogues (pitch lde / ldc)
    const uint8_t *rowflag;
    int M, N, K, kper;      // kper: K range per split (multiple of the K tile)
    int ntm, ntn, per_xcd;
    // placement of the (tile, split) work items on the 8 XCDs (bf16x3 kernel): slots per XCD,
    // mapping mode and its parameter, first slot of this problem in a shared launch
    int splits, nx, mode, mpar, slot0, second_first;
    // epilogue 7 (scan over the tile's rows): tiles per sequence, column tiles per unit, column
    // groups per sequence, number of units (a unit = the chains of one sequence and column group)
    ScanEpilogue scan;
    int sc_nt, sc_cpu, sc_ncg, sc_units, sc_rev;
    AbsMax amaxA, amaxB;    // two-plane fp16 staging only
};

// Value stored for an output element whose accumulated product is v.
//   EPI 0: v
//   EPI 1: v + diag[col] * E[row, col]                   (D (.) u and D (.) dy)
//   EPI 2: columns are interleaved (re, im) pairs of complex states; diag holds Abar as
//          interleaved complex; adds [not rowflag[row]] * (Abar_p * E_p)[re or im]: the carried
//          state Abar x_{t-1} of one recurrence step (Eq. 3, first line)
//   EPI 3: half-GLU gate (S5 sequence layer appendix): s = sigmoid(v) is kept in C2 when asked
//          and the stored value is E[row, col] * s        (E = the gated input u)
//   EPI 4: adjoint of the gate with respect to its input: E * E2 + v * GELU'(E3)
//          (E = dy, E2 = the saved gate s, E3 = u; v = the product dz W^T)
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
        return fmaf(v, gelu_derivative(g.E3[i]), g.E[i] * g.E2[i]);
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

// Stages one R x BK operand tile through registers.
// KC = true : global X[row*ld + k]  (k contiguous)   -> float4 along k, transposed into LDS
// KC = false: global X[k*ld + row]  (row contiguous) -> float4 along row, copied into LDS
template <int R, int BK, bool KC, int NT>
struct TileLoader {
    static constexpr int NV = R * BK / 4 / NT;
    static_assert(NV >= 1 && NV * NT * 4 == R * BK, "tile must be a multiple of the workgroup's float4 loads");
    float4 r[NV];

    template <bool FAST>
    __device__ __forceinline__ void load(const float *__restrict__ X, long ld, int row0, int rows, int k0,
                                         int kend, int tid)
    {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int idx = tid + i * NT;
            if (KC) {
                const int row = idx / (BK / 4), kq = idx % (BK / 4);
                const long gr = row0 + row;
                const int k = k0 + 4 * kq;
                if (FAST) {
                    r[i] = *reinterpret_cast<const float4 *>(X + gr * ld + k);
                } else {
                    float t[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) t[j] = (gr < rows && k + j < kend) ? X[gr * ld + k + j] : 0.f;
                    r[i] = make_float4(t[0], t[1], t[2], t[3]);
                }
            } else {
                const int kk = idx / (R / 4), rq = idx % (R / 4);
                const long gr = row0 + 4 * rq;
                const long k = k0 + kk;
                if (FAST) {
                    r[i] = *reinterpret_cast<const float4 *>(X + k * ld + gr);
                } else {
                    float t[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) t[j] = (gr + j < rows && k < kend) ? X[k * ld + gr + j] : 0.f;
                    r[i] = make_float4(t[0], t[1], t[2], t[3]);
                }
            }
        }
    }

    // LDS layout [k][row] with row stride S
    template <int S>
    __device__ __forceinline__ void store(float *lds, int tid) const
    {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int idx = tid + i * NT;
            if (KC) {
                const int row = idx / (BK / 4), kq = idx % (BK / 4);
                lds[(4 * kq + 0) * S + row] = r[i].x;
                lds[(4 * kq + 1) * S + row] = r[i].y;
                lds[(4 * kq + 2) * S + row] = r[i].z;
                lds[(4 * kq + 3) * S + row] = r[i].w;
            } else {
                const int kk = idx / (R / 4), rq = idx % (R / 4);
                *reinterpret_cast<float4 *>(lds + kk * S + 4 * rq) = r[i];
            }
        }
    }
};

// Row stride of an operand tile in LDS: odd for the transposing (k-contiguous) loader so that
// its scattered 4-byte writes spread over the banks, a multiple of 4 for the 16-byte writes.
template <int R, bool KC> struct LdsStride { static constexpr int value = KC ? R + 1 : R + 4; };

template <int BM, int BN, int BK, int WGM, int WGN, bool AKC, bool BKC, int EPI, bool FAST>
__device__ __forceinline__ void gemm_tile(const GemmDev &g, float *As, float *Bs, int m0, int n0, int z,
                                          int kbeg, int kend)
{
    constexpr int NT = 64 * WGM * WGN;
    constexpr int SA = LdsStride<BM, AKC>::value, SB = LdsStride<BN, BKC>::value;
    constexpr int WM = BM / WGM, WN = BN / WGN;      // wavefront tile
    constexpr int MI = WM / 32, NI = WN / 32;        // 32x32 MFMA tiles per wavefront
    static_assert(MI >= 1 && NI >= 1 && WM % 32 == 0 && WN % 32 == 0, "wavefront tile must be 32-aligned");

    const int tid = threadIdx.x;
    const int wave = tid >> 6, l = tid & 63;
    const int wm = wave / WGN, wn = wave % WGN;
    const int li = l & 31, hh = l >> 5;

    TileLoader<BM, BK, AKC, NT> la;
    TileLoader<BN, BK, BKC, NT> lb;

    v16f acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nk = (kend > kbeg) ? (kend - kbeg + BK - 1) / BK : 0;
    if (nk > 0) {
        la.template load<FAST>(g.A, g.lda, m0, g.M, kbeg, kend, tid);
        lb.template load<FAST>(g.B, g.ldb, n0, g.N, kbeg, kend, tid);
        la.template store<SA>(As, tid);
        lb.template store<SB>(Bs, tid);
    }
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) {
            la.template load<FAST>(g.A, g.lda, m0, g.M, kbeg + (kt + 1) * BK, kend, tid);
            lb.template load<FAST>(g.B, g.ldb, n0, g.N, kbeg + (kt + 1) * BK, kend, tid);
        }
        const float *as = As + cur * (BK * SA) + wm * WM + li;
        const float *bs = Bs + cur * (BK * SB) + wn * WN + li;
#pragma unroll
        for (int kk = 0; kk < BK / 2; ++kk) {
            float a[MI], b[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i) a[i] = as[(2 * kk + hh) * SA + i * 32];
#pragma unroll
            for (int j = 0; j < NI; ++j) b[j] = bs[(2 * kk + hh) * SB + j * 32];
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) {
            la.template store<SA>(As + (cur ^ 1) * (BK * SA), tid);
            lb.template store<SB>(Bs + (cur ^ 1) * (BK * SB), tid);
        }
        __syncthreads();
    }

    // Accumulator layout of the 32x32 tile: register r of lane l holds
    // row 8*(r/4) + 4*(l/32) + r%4, column l%32.
    float *Cz = g.C + (long)z * g.M * g.ldc;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int col = n0 + wn * WN + j * 32 + li;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const long row = m0 + wm * WM + i * 32 + 8 * (r / 4) + 4 * hh + (r % 4);
                if (FAST || (row < g.M && col < g.N)) {
                    Cz[row * g.ldc + col] = gemm_epilogue_apply<EPI>(g, row, col, acc[i][j][r]);
                }
            }
        }
}

template <int BM, int BN, int BK, int WGM, int WGN, bool AKC, bool BKC, int EPI>
__global__ void __launch_bounds__(64 * WGM * WGN) gemm_f32_kernel(GemmDev g)
{
    constexpr int SA = LdsStride<BM, AKC>::value, SB = LdsStride<BN, BKC>::value;
    __shared__ __attribute__((aligned(16))) float As[2 * BK * SA];
    __shared__ __attribute__((aligned(16))) float Bs[2 * BK * SB];

    // XCD-aware tile assignment: workgroup id i runs on XCD i % 8; XCD x gets the tiles
    // [x*per_xcd, (x+1)*per_xcd).
    const int id = blockIdx.x;
    const int tile = (id % 8) * g.per_xcd + id / 8;
    if (tile >= g.ntm * g.ntn) return;
    const int tm = tile / g.ntn, tn = tile % g.ntn;
    const int m0 = tm * BM, n0 = tn * BN;
    const int z = blockIdx.y;
    const int kbeg = z * g.kper;
    const int kend = min(g.K, kbeg + g.kper);

    // interior tile with 16-byte aligned rows and whole K tiles: no guards anywhere
    const bool fast = (g.lda % 4 == 0) && ((reinterpret_cast<uintptr_t>(g.A) & 15) == 0) &&
                      (g.ldb % 4 == 0) && ((reinterpret_cast<uintptr_t>(g.B) & 15) == 0) &&
                      (m0 + BM <= g.M) && (n0 + BN <= g.N) && ((kend - kbeg) % BK == 0);
    if (fast)
        gemm_tile<BM, BN, BK, WGM, WGN, AKC, BKC, EPI, true>(g, As, Bs, m0, n0, z, kbeg, kend);
    else
        gemm_tile<BM, BN, BK, WGM, WGN, AKC, BKC, EPI, false>(g, As, Bs, m0, n0, z, kbeg, kend);
}

template <int BM, int BN, int BK, int WGM, int WGN, bool AKC, bool BKC, int EPI>
hipError_t launch_gemm_variant(const GemmArgs &a, hipStream_t s)
{
    GemmDev g;
    g.A = a.A; g.lda = a.lda; g.B = a.B; g.ldb = a.ldb; g.C = a.C; g.ldc = a.ldc;
    g.diag = a.diag; g.E = a.E; g.lde = a.lde; g.rowflag = a.rowflag;
    g.E2 = a.E2; g.E3 = a.E3; g.C2 = a.C2;
    g.M = a.M; g.N = a.N; g.K = a.K;
    const int splits = a.splits < 1 ? 1 : a.splits;
    int kper = (a.K + splits - 1) / splits;
    kper = (kper + BK - 1) / BK * BK;
    g.kper = kper;
    g.ntm = (a.M + BM - 1) / BM;
    g.ntn = (a.N + BN - 1) / BN;
    const long ntiles = (long)g.ntm * g.ntn;
    g.per_xcd = (int)((ntiles + 7) / 8);
    dim3 grid((unsigned)(g.per_xcd * 8), (unsigned)splits, 1);
    hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, BK, WGM, WGN, AKC, BKC, EPI>), grid, dim3(64 * WGM * WGN), 0, s, g);
    return hipGetLastError();
}

}  // namespace ssm
