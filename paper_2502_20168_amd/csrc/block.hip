// Operations around the SSM layer (gfx950): the bootstrapped lambda-return of the actor-critic
// section and the half-GLU gate of the S5 sequence layer (appendix), with their adjoints.
#include "../../include/ssm.h"
#include "ssm_internal.h"
#include "gemm_common.h"

namespace ssm {
namespace {

constexpr size_t ALIGN = 256;
inline size_t up(size_t n) { return (n + ALIGN - 1) / ALIGN * ALIGN; }
inline bool misaligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }
#define HIP_TRY(expr) do { if ((expr) != hipSuccess) return SSM_ERR_HIP; } while (0)

// ---------------------------------------------------------------------------------------------
// lambda-return:  V_t = r_t + gamma c_t ((1 - lambda) v_t + lambda V_{t+1}),  V_T = v_T.
// Time-major arrays [T, N]; one thread per trajectory walks time backwards.  Neighbouring
// threads read neighbouring trajectories of the same step, so every access is one coalesced
// row segment; the only serial dependency is one fused multiply-add per step.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) lambda_return_kernel(const float *__restrict__ r, const float *__restrict__ c,
                                                            const float *__restrict__ v, float gamma, float lam,
                                                            long T, long N, float *__restrict__ ret)
{
    const long n = (long)blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    float V = v[(T - 1) * N + n];
    ret[(T - 1) * N + n] = V;
    const float gl = gamma * lam, g1 = gamma * (1.f - lam);
    long t = T - 2;
    for (; t >= 3; t -= 4) {
        // the loads of four steps do not depend on V: issue them together
        float rr[4], cc[4], vv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const long i = (t - j) * N + n;
            rr[j] = r[i]; cc[j] = c[i]; vv[j] = v[i];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // r + c (g1 v) + (c gl) V
            V = fmaf(cc[j] * gl, V, fmaf(cc[j], g1 * vv[j], rr[j]));
            ret[(t - j) * N + n] = V;
        }
    }
    for (; t >= 0; --t) {
        const long i = t * N + n;
        const float cv = c[i];
        V = fmaf(cv * gl, V, fmaf(cv, g1 * v[i], r[i]));
        ret[i] = V;
    }
}

// Adjoint: G_t = dret_t + gamma lambda c_{t-1} G_{t-1} walks time forwards;
// dr_t = G_t, dc_t = G_t gamma ((1-lambda) v_t + lambda V_{t+1}), dv_t = G_t gamma c_t (1-lambda) for t < T-1;
// the last step has dv = G and no reward / continue gradient.
__global__ void __launch_bounds__(256) lambda_return_bwd_kernel(const float *__restrict__ c, const float *__restrict__ v,
                                                                const float *__restrict__ ret, const float *__restrict__ dret,
                                                                float gamma, float lam, long T, long N,
                                                                float *__restrict__ dr, float *__restrict__ dc,
                                                                float *__restrict__ dv)
{
    const long n = (long)blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    const float gl = gamma * lam, g1 = gamma * (1.f - lam);
    float G = 0.f, cprev = 0.f;
    for (long t = 0; t < T - 1; ++t) {
        const long i = t * N + n;
        const float cv = c[i];
        G = fmaf(gl * cprev, G, dret[i]);
        dr[i] = G;
        dc[i] = G * fmaf(gl, ret[i + N], g1 * v[i]);
        dv[i] = G * (g1 * cv);
        cprev = cv;
    }
    const long i = (T - 1) * N + n;
    G = fmaf(gl * cprev, G, dret[i]);
    dr[i] = 0.f;
    dc[i] = 0.f;
    dv[i] = G;
}

// ---------------------------------------------------------------------------------------------
// half-GLU:  x1 = GELU(u),  y = u (.) sigmoid(x1 W).
// The element-wise halves run as small streaming kernels (float4 per thread); the products run
// on the projection GEMM with the gate fused into its store (epilogues 3 and 4).
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float gelu_exact(float x) { return gelu_value(x); }

__global__ void __launch_bounds__(256) gelu_kernel(const float4 *__restrict__ u, float4 *__restrict__ x1, long n4,
                                                   const float *__restrict__ ut, float *__restrict__ x1t, long n)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) {
        const float4 a = u[i];
        x1[i] = make_float4(gelu_exact(a.x), gelu_exact(a.y), gelu_exact(a.z), gelu_exact(a.w));
    }
    const long j = 4 * n4 + i;                           // the up to three elements past the last float4
    if (i < 4 && j < n) x1t[j] = gelu_exact(ut[j]);
}

// One pass over the inputs of the gate's adjoint (s = the gate saved by the forward call): x1 = GELU(u) and
// dz = dy u s (1 - s), the operands of the two products, and the two terms that the store of dz W^T needs,
// ds = dy s and gd = GELU'(u) (du = ds + (dz W^T) gd): formed here, where u, s and dy pass anyway, they cost
// that store two loads per value and no error function.
__global__ void __launch_bounds__(256) gate_bwd_prep_kernel(const float *__restrict__ u, const float *__restrict__ s,
                                                            const float *__restrict__ dy, float *__restrict__ x1,
                                                            float *__restrict__ dz, float *__restrict__ ds,
                                                            float *__restrict__ gd, long n)
{
    const long i0 = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i0 + 4 <= n) {
        const float4 a = *reinterpret_cast<const float4 *>(u + i0);
        const float4 g = *reinterpret_cast<const float4 *>(s + i0);
        const float4 d = *reinterpret_cast<const float4 *>(dy + i0);
        *reinterpret_cast<float4 *>(x1 + i0) =
            make_float4(gelu_exact(a.x), gelu_exact(a.y), gelu_exact(a.z), gelu_exact(a.w));
        *reinterpret_cast<float4 *>(dz + i0) =
            make_float4(d.x * a.x * (g.x * (1.f - g.x)), d.y * a.y * (g.y * (1.f - g.y)),
                        d.z * a.z * (g.z * (1.f - g.z)), d.w * a.w * (g.w * (1.f - g.w)));
        *reinterpret_cast<float4 *>(ds + i0) = make_float4(d.x * g.x, d.y * g.y, d.z * g.z, d.w * g.w);
        *reinterpret_cast<float4 *>(gd + i0) =
            make_float4(gelu_derivative(a.x), gelu_derivative(a.y), gelu_derivative(a.z), gelu_derivative(a.w));
    } else {
        for (long i = i0; i < n; ++i) {
            x1[i] = gelu_exact(u[i]);
            dz[i] = dy[i] * u[i] * (s[i] * (1.f - s[i]));
            ds[i] = dy[i] * s[i];
            gd[i] = gelu_derivative(u[i]);
        }
    }
}

// The same two passes for widths that are multiples of 64, where the products behind them stage their
// operands as two scaled fp16 planes (three matrix instructions per k block instead of six): they also
// measure the largest magnitudes that scale those planes -- of every token row of the product's first
// operand in pieces of 64 columns (rowmax[piece][row]; 16 neighbouring lanes hold one piece), of a whole
// operand per workgroup (slots[workgroup]), and of W by the extra workgroups behind the first main_blocks.
__device__ __forceinline__ unsigned abs_bits4(float4 v)
{
    return __float_as_uint(fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
}
__device__ __forceinline__ unsigned max16(unsigned v)
{
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) v = max(v, (unsigned)__shfl_xor((int)v, o));
    return v;
}
// maximum over the 256 threads of the workgroup, valid in thread 0 (red: 4 words of LDS)
__device__ __forceinline__ unsigned block_max(unsigned v, unsigned *red)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = max(v, (unsigned)__shfl_xor((int)v, o));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return max(max(red[0], red[1]), max(red[2], red[3]));
}
__device__ __forceinline__ void weight_max_block(const float *__restrict__ W, long nW, unsigned *__restrict__ wslots,
                                                 int b, int nb, unsigned *red)
{
    unsigned m = 0;
    if ((reinterpret_cast<uintptr_t>(W) & 15) == 0 && nW % 4 == 0) {
        const float4 *W4 = reinterpret_cast<const float4 *>(W);
        for (long j = (long)b * 256 + threadIdx.x; j < nW / 4; j += (long)nb * 256) m = max(m, abs_bits4(W4[j]));
    } else {
        for (long j = (long)b * 256 + threadIdx.x; j < nW; j += (long)nb * 256) m = max(m, __float_as_uint(fabsf(W[j])));
    }
    m = block_max(m, red);
    if (threadIdx.x == 0) wslots[b] = m;
}

__global__ void __launch_bounds__(256) gelu_max_kernel(const float4 *__restrict__ u, float4 *__restrict__ x1, long n4,
                                                       int H, long T, unsigned *__restrict__ rowmax,
                                                       const float *__restrict__ W, long nW,
                                                       unsigned *__restrict__ wslots, int w_blocks)
{
    __shared__ unsigned red[4];
    if ((int)blockIdx.x < w_blocks) {                    // (first in the grid: their short chains of loads start at once)
        weight_max_block(W, nW, wslots, (int)blockIdx.x, w_blocks, red);
        return;
    }
    const long i = (long)(blockIdx.x - w_blocks) * 256 + threadIdx.x;
    unsigned m = 0;
    if (i < n4) {                                        // (n4 is a multiple of 16: a row piece is in or out as a whole)
        const float4 a = u[i];
        const float4 g = make_float4(gelu_exact(a.x), gelu_exact(a.y), gelu_exact(a.z), gelu_exact(a.w));
        x1[i] = g;
        m = abs_bits4(g);
    }
    m = max16(m);
    if ((threadIdx.x & 15) == 0 && i < n4) {
        const long e0 = i * 4, row = e0 / H;
        rowmax[(size_t)((e0 - row * H) / 64) * T + row] = m;
    }
}

__global__ void __launch_bounds__(256) gate_bwd_prep_max_kernel(const float *__restrict__ u, const float *__restrict__ s,
                                                                const float *__restrict__ dy, float *__restrict__ x1,
                                                                float *__restrict__ dz, float *__restrict__ ds,
                                                                float *__restrict__ gd, long n, int H, long T,
                                                                unsigned *__restrict__ dz_rowmax,
                                                                unsigned *__restrict__ x1_slots, unsigned *__restrict__ dz_slots,
                                                                const float *__restrict__ W, long nW,
                                                                unsigned *__restrict__ wslots, int w_blocks)
{
    __shared__ unsigned red[4];
    if ((int)blockIdx.x < w_blocks) {
        weight_max_block(W, nW, wslots, (int)blockIdx.x, w_blocks, red);
        return;
    }
    const int b = (int)blockIdx.x - w_blocks, main_blocks = (int)gridDim.x - w_blocks;
    const long stride = (long)main_blocks * 1024;
    unsigned mx = 0, mz = 0;
    for (long base = ((long)b * 256 + threadIdx.x) * 4; base < n; base += 4 * stride) {
        // the inputs of four pieces first, so that their loads are in flight together
        float4 a[4], g[4], d[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const long i0 = base + k * stride;
            if (i0 < n) {
                a[k] = *reinterpret_cast<const float4 *>(u + i0);
                g[k] = *reinterpret_cast<const float4 *>(s + i0);
                d[k] = *reinterpret_cast<const float4 *>(dy + i0);
            }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const long i0 = base + k * stride;
            if (i0 < n) {                                // (n is a multiple of 64: the 16 lanes of a piece stay together)
                const float4 xo = make_float4(gelu_exact(a[k].x), gelu_exact(a[k].y), gelu_exact(a[k].z), gelu_exact(a[k].w));
                const float4 zo = make_float4(d[k].x * a[k].x * (g[k].x * (1.f - g[k].x)), d[k].y * a[k].y * (g[k].y * (1.f - g[k].y)),
                                              d[k].z * a[k].z * (g[k].z * (1.f - g[k].z)), d[k].w * a[k].w * (g[k].w * (1.f - g[k].w)));
                *reinterpret_cast<float4 *>(x1 + i0) = xo;
                *reinterpret_cast<float4 *>(dz + i0) = zo;
                *reinterpret_cast<float4 *>(ds + i0) = make_float4(d[k].x * g[k].x, d[k].y * g[k].y, d[k].z * g[k].z, d[k].w * g[k].w);
                *reinterpret_cast<float4 *>(gd + i0) =
                    make_float4(gelu_derivative(a[k].x), gelu_derivative(a[k].y), gelu_derivative(a[k].z), gelu_derivative(a[k].w));
                const unsigned bz = abs_bits4(zo);
                mx = max(mx, abs_bits4(xo)); mz = max(mz, bz);
                const unsigned piece = max16(bz);
                if ((threadIdx.x & 15) == 0) {
                    const long row = i0 / H;
                    dz_rowmax[(size_t)((i0 - row * H) / 64) * T + row] = piece;
                }
            }
        }
    }
    mx = block_max(mx, red);
    __syncthreads();
    mz = block_max(mz, red);
    if (threadIdx.x == 0) { x1_slots[b] = mx; dz_slots[b] = mz; }
}

// fixed-order sum of the K-split slabs of a product
__global__ void __launch_bounds__(256) sum_slabs_kernel(const float *__restrict__ part, long n, int nslab,
                                                        float *__restrict__ out)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    float acc = 0.f;
    for (int z = 0; z < nslab; ++z) acc += part[(long)z * n + i];
    out[i] = acc;
}

constexpr int GLU_MAX_SLOTS = 512;      // workgroups of the element-wise pass that report a maximum each
constexpr int GLU_W_BLOCKS = 256;       // workgroups that measure W
struct GluLayout {
    size_t x1, dz, ds, gd, dWpart, total; int splits;
    // widths that are multiples of 64: two scaled fp16 planes per operand, with their largest magnitudes
    bool two_planes; size_t rowmax, slots; int row_parts, main_blocks;
    bool paired, dw_first;     // gradient pass: dz W^T and the slabs of x1^T dz in one launch (dW's work items first)
};

bool make_glu_layout(int64_t T, int64_t H, bool bwd, GluLayout &o)
{
    if (T <= 0 || H <= 0 || H > SSM_MAX_WIDTH || T > SSM_MAX_TOKENS || T > SSM_MAX_ELEMS / H) return false;
    size_t off = 0;
    o.x1 = off; off += up((size_t)T * H * 4);
    o.dz = o.ds = o.gd = o.dWpart = 0; o.splits = 1;
    o.two_planes = gate_two_planes_shape(T, H);
    // gradient pass on two planes: both products wait for the same element-wise pass and share one launch, the
    // K splits of the reduction from the schedule model of that launch (no K halves of du then: the slabs
    // fill the chip beside it)
    o.paired = bwd && o.two_planes; o.dw_first = false;
    if (bwd) {
        o.dz = off; off += up((size_t)T * H * 4);
        o.ds = off; off += up((size_t)T * H * 4);
        o.gd = off; off += up((size_t)T * H * 4);
        o.splits = o.paired ? gemm_pick_splits_balanced(H, H, T, ((T + 127) / 128) * ((H + 127) / 128), H, o.dw_first)
                            : gemm_pick_splits(H, H, T, 0);
    }
    if (bwd) { o.dWpart = off; off += up((size_t)o.splits * H * H * 4); }
    o.rowmax = o.slots = 0; o.row_parts = o.main_blocks = 0;
    if (o.two_planes) {
        o.row_parts = (int)(H / 64);
        const int64_t blocks = (T * H / 4 + 255) / 256;
        o.main_blocks = (int)(bwd ? (blocks < GLU_MAX_SLOTS ? blocks : GLU_MAX_SLOTS) : blocks);
        o.rowmax = off; off += up((size_t)o.row_parts * T * 4);
        o.slots = off; off += up((size_t)(2 * GLU_MAX_SLOTS + GLU_W_BLOCKS) * 4);     // x1, dz, W
    }
    o.total = off;
    return true;
}

}  // namespace
}  // namespace ssm

using namespace ssm;

extern "C" {

ssm_status ssm_lambda_return(const float *reward, const float *cont, const float *value, float gamma,
                             float lambda, int64_t T, int64_t N, float *ret, void *stream)
{
    if (!reward || !cont || !value || !ret) return SSM_ERR_INVALID_ARG;
    if (T <= 0 || N <= 0) return SSM_ERR_INVALID_ARG;
    if (T > SSM_MAX_TOKENS || N > SSM_MAX_TOKENS || T > SSM_MAX_ELEMS / N) return SSM_ERR_UNSUPPORTED;
    if (misaligned(reward, 4) || misaligned(cont, 4) || misaligned(value, 4) || misaligned(ret, 4))
        return SSM_ERR_INVALID_ARG;
    const unsigned blocks = (unsigned)((N + 255) / 256);
    hipLaunchKernelGGL(lambda_return_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       reward, cont, value, gamma, lambda, (long)T, (long)N, ret);
    HIP_TRY(hipGetLastError());
    return SSM_OK;
}

ssm_status ssm_lambda_return_bwd(const float *cont, const float *value, const float *ret, const float *dret,
                                 float gamma, float lambda, int64_t T, int64_t N,
                                 float *dreward, float *dcont, float *dvalue, void *stream)
{
    if (!cont || !value || !ret || !dret || !dreward || !dcont || !dvalue) return SSM_ERR_INVALID_ARG;
    if (T <= 0 || N <= 0) return SSM_ERR_INVALID_ARG;
    if (T > SSM_MAX_TOKENS || N > SSM_MAX_TOKENS || T > SSM_MAX_ELEMS / N) return SSM_ERR_UNSUPPORTED;
    if (misaligned(cont, 4) || misaligned(value, 4) || misaligned(ret, 4) || misaligned(dret, 4) ||
        misaligned(dreward, 4) || misaligned(dcont, 4) || misaligned(dvalue, 4))
        return SSM_ERR_INVALID_ARG;
    const unsigned blocks = (unsigned)((N + 255) / 256);
    hipLaunchKernelGGL(lambda_return_bwd_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       cont, value, ret, dret, gamma, lambda, (long)T, (long)N, dreward, dcont, dvalue);
    HIP_TRY(hipGetLastError());
    return SSM_OK;
}

size_t ssm_half_glu_workspace_bytes(int64_t T, int64_t H, int want_bwd)
{
    GluLayout lo;
    return make_glu_layout(T, H, want_bwd != 0, lo) ? lo.total : 0;
}

ssm_status ssm_half_glu_fwd(const float *u, const float *W, int64_t T, int64_t H, float *y, float *gate,
                            void *workspace, size_t ws_bytes, void *stream)
{
    if (!u || !W || !y) return SSM_ERR_INVALID_ARG;
    if (T <= 0 || H <= 0) return SSM_ERR_INVALID_ARG;
    GluLayout lo;
    if (!make_glu_layout(T, H, false, lo)) return SSM_ERR_UNSUPPORTED;
    if (misaligned(u, 16) || misaligned(W, 4) || misaligned(y, 4) || misaligned(gate, 4)) return SSM_ERR_INVALID_ARG;
    if (!workspace || misaligned(workspace, ALIGN) || ws_bytes < lo.total) return SSM_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *x1 = reinterpret_cast<float *>(static_cast<char *>(workspace) + lo.x1);
    const long n = (long)T * H, n4 = n / 4;
    unsigned *rowmax = reinterpret_cast<unsigned *>(static_cast<char *>(workspace) + lo.rowmax);
    unsigned *wslots = reinterpret_cast<unsigned *>(static_cast<char *>(workspace) + lo.slots) + 2 * GLU_MAX_SLOTS;
    if (lo.two_planes) {
        hipLaunchKernelGGL(gelu_max_kernel, dim3((unsigned)(lo.main_blocks + GLU_W_BLOCKS)), dim3(256), 0, s,
                           reinterpret_cast<const float4 *>(u), reinterpret_cast<float4 *>(x1), n4, (int)H, (long)T, rowmax,
                           W, (long)H * H, wslots, GLU_W_BLOCKS);
    } else {
        const long threads = n4 > 4 ? n4 : 4;
        hipLaunchKernelGGL(gelu_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s,
                           reinterpret_cast<const float4 *>(u), reinterpret_cast<float4 *>(x1), n4, u, x1, n);
    }
    HIP_TRY(hipGetLastError());
    // y[t, j] = u[t, j] sigmoid(sum_i x1[t, i] W[i, j])
    GemmArgs g{};
    g.A = x1; g.lda = H; g.a_kcontig = 1;
    g.B = W; g.ldb = H; g.b_kcontig = 0;
    g.C = y; g.ldc = H; g.E = u; g.lde = H; g.C2 = gate; g.epilogue = 3;
    g.M = (int)T; g.N = (int)H; g.K = (int)H; g.splits = 1;
    if (lo.two_planes) { g.amaxA = AbsMax{nullptr, 0, rowmax, lo.row_parts, (long)T}; g.amaxB = AbsMax{wslots, GLU_W_BLOCKS, nullptr, 0, 0}; }
    HIP_TRY(launch_gemm(g, s));
    return SSM_OK;
}

ssm_status ssm_half_glu_bwd(const float *u, const float *W, const float *gate, const float *dy,
                            int64_t T, int64_t H, float *du, float *dW,
                            void *workspace, size_t ws_bytes, void *stream)
{
    if (!u || !W || !gate || !dy || !du || !dW) return SSM_ERR_INVALID_ARG;
    if (T <= 0 || H <= 0) return SSM_ERR_INVALID_ARG;
    GluLayout lo;
    if (!make_glu_layout(T, H, true, lo)) return SSM_ERR_UNSUPPORTED;
    if (misaligned(u, 16) || misaligned(W, 4) || misaligned(gate, 16) || misaligned(dy, 16) || misaligned(du, 4) ||
        misaligned(dW, 4))
        return SSM_ERR_INVALID_ARG;
    if (!workspace || misaligned(workspace, ALIGN) || ws_bytes < lo.total) return SSM_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    float *x1 = reinterpret_cast<float *>(ws + lo.x1);
    float *dz = reinterpret_cast<float *>(ws + lo.dz);
    float *ds = reinterpret_cast<float *>(ws + lo.ds), *gd = reinterpret_cast<float *>(ws + lo.gd);
    float *dWpart = reinterpret_cast<float *>(ws + lo.dWpart);
    const long n = (long)T * H;
    unsigned *rowmax = reinterpret_cast<unsigned *>(ws + lo.rowmax);
    unsigned *x1_slots = reinterpret_cast<unsigned *>(ws + lo.slots), *dz_slots = x1_slots + GLU_MAX_SLOTS, *wslots = dz_slots + GLU_MAX_SLOTS;
    if (lo.two_planes) {
        hipLaunchKernelGGL(gate_bwd_prep_max_kernel, dim3((unsigned)(lo.main_blocks + GLU_W_BLOCKS)), dim3(256), 0, s, u, gate, dy,
                           x1, dz, ds, gd, n, (int)H, (long)T, rowmax, x1_slots, dz_slots, W, (long)H * H, wslots, GLU_W_BLOCKS);
    } else {
        hipLaunchKernelGGL(gate_bwd_prep_kernel, dim3((unsigned)(((n + 3) / 4 + 255) / 256)), dim3(256), 0, s, u, gate, dy, x1,
                           dz, ds, gd, n);
    }
    HIP_TRY(hipGetLastError());
    // du[t, i] = ds[t, i] + gd[t, i] sum_j dz[t, j] W[i, j]
    GemmArgs g{};
    g.A = dz; g.lda = H; g.a_kcontig = 1;
    g.B = W; g.ldb = H; g.b_kcontig = 1;
    g.C = du; g.ldc = H; g.E = ds; g.E2 = gd; g.lde = H; g.epilogue = 4;
    g.M = (int)T; g.N = (int)H; g.K = (int)H; g.splits = 1;
    if (lo.two_planes) { g.amaxA = AbsMax{nullptr, 0, rowmax, lo.row_parts, (long)T}; g.amaxB = AbsMax{wslots, GLU_W_BLOCKS, nullptr, 0, 0}; }
    if (!lo.paired) HIP_TRY(launch_gemm(g, s));
    // dW[i, j] = sum_t x1[t, i] dz[t, j]: reduction over tokens in K slabs, then a fixed-order sum
    GemmArgs h{};
    h.A = x1; h.lda = H; h.a_kcontig = 0;
    h.B = dz; h.ldb = H; h.b_kcontig = 0;
    h.C = dWpart; h.ldc = H;
    h.M = (int)H; h.N = (int)H; h.K = (int)T; h.splits = lo.splits;
    if (lo.two_planes) { h.amaxA = AbsMax{x1_slots, lo.main_blocks, nullptr, 0, 0}; h.amaxB = AbsMax{dz_slots, lo.main_blocks, nullptr, 0, 0}; }
    if (lo.paired) HIP_TRY(launch_gemm_pair(g, h, s, lo.dw_first));
    else HIP_TRY(launch_gemm(h, s));
    const long nw = (long)H * H;
    hipLaunchKernelGGL(sum_slabs_kernel, dim3((unsigned)((nw + 255) / 256)), dim3(256), 0, s, dWpart, nw, lo.splits, dW);
    HIP_TRY(hipGetLastError());
    return SSM_OK;
}

}  // extern "C"
