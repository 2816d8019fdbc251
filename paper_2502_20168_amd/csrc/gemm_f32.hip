// fp32 MFMA GEMM for the dense projections of the S5 layer (input projection Bbar u of Eq. 6,
// output projection C x of Eq. 3, and their four adjoints in the gradient pass).
//
// gfx950 design: a 256-thread workgroup (4 wavefronts, 2 x 2) owns a BM x BN tile of C; each
// wavefront accumulates (BM/2) x (BN/2) outputs in v_mfma_f32_32x32x2_f32 tiles.  Operand tiles
// are staged global -> registers -> LDS with the next K tile in flight while the current one
// feeds the matrix cores.  Both operands sit in LDS as [k][row], so that the 32 lanes that
// share k read 32 consecutive words (no bank conflicts) whatever the global layout was.
// Workgroup ids are dealt round-robin to the 8 XCDs by the hardware; ids are remapped so that
// each XCD works on a contiguous band of tiles and re-reads only its band of A from its own L2.
#include "ssm_internal.h"

namespace ssm {

typedef float v16f __attribute__((ext_vector_type(16)));

struct GemmDev {
    const float *A; long lda;
    const float *B; long ldb;
    float *C; long ldc;
    const float *diag; const float *E; long lde;
    int M, N, K, kper;      // kper: K range per split (multiple of the K tile)
    int ntm, ntn, per_xcd;
};

// Loads one R x BK operand tile into registers as float4s.
// KC = true : global X[row*ld + k]  -> float4 along k
// KC = false: global X[k*ld + row]  -> float4 along row
template <int R, int BK, bool KC>
struct TileLoader {
    static constexpr int NV = R * BK / 4 / 256;
    static_assert(NV >= 1, "tile too small for 256 threads");
    float4 r[NV];

    __device__ __forceinline__ void load(const float *X, long ld, int row0, int rows, int k0,
                                         int kend, bool fast, int tid)
    {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int idx = tid + i * 256;
            if (KC) {
                const int row = idx / (BK / 4), kq = idx % (BK / 4);
                const long gr = row0 + row;
                const int k = k0 + 4 * kq;
                if (fast && k0 + BK <= kend) {
                    r[i] = *reinterpret_cast<const float4 *>(X + gr * ld + k);
                } else {
                    float t[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        t[j] = (gr < rows && k + j < kend) ? X[gr * ld + k + j] : 0.f;
                    r[i] = make_float4(t[0], t[1], t[2], t[3]);
                }
            } else {
                const int kk = idx / (R / 4), rq = idx % (R / 4);
                const long gr = row0 + 4 * rq;
                const long k = k0 + kk;
                if (fast && k0 + BK <= kend) {
                    r[i] = *reinterpret_cast<const float4 *>(X + k * ld + gr);
                } else {
                    float t[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        t[j] = (gr + j < rows && k < kend) ? X[k * ld + gr + j] : 0.f;
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
            const int idx = tid + i * 256;
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

// Row stride of an operand tile in LDS: odd for the transposing (k-contiguous) loader so its
// scattered 4-byte writes spread over the banks, a multiple of 4 for the 16-byte writes.
template <int R, bool KC> struct LdsStride { static constexpr int value = KC ? R + 1 : R + 4; };

template <int BM, int BN, int BK, bool AKC, bool BKC, bool EPI>
__global__ void __launch_bounds__(256) gemm_f32_kernel(GemmDev g)
{
    constexpr int SA = LdsStride<BM, AKC>::value, SB = LdsStride<BN, BKC>::value;
    constexpr int WM = BM / 2, WN = BN / 2;          // wavefront tile
    constexpr int MI = WM / 32, NI = WN / 32;        // 32x32 MFMA tiles per wavefront
    __shared__ __attribute__((aligned(16))) float As[2][BK * SA];
    __shared__ __attribute__((aligned(16))) float Bs[2][BK * SB];

    // XCD-aware tile assignment: workgroup id i runs on XCD i % 8; give XCD x the tiles
    // [x*per_xcd, (x+1)*per_xcd).
    const int id = blockIdx.x;
    const int tile = (id % 8) * g.per_xcd + id / 8;
    if (tile >= g.ntm * g.ntn) return;
    const int tm = tile / g.ntn, tn = tile % g.ntn;
    const int m0 = tm * BM, n0 = tn * BN;
    const int z = blockIdx.y;
    const int kbeg = z * g.kper;
    const int kend = min(g.K, kbeg + g.kper);

    const int tid = threadIdx.x;
    const int wave = tid >> 6, l = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = l & 31, hh = l >> 5;

    const bool fastA = (g.lda % 4 == 0) && ((reinterpret_cast<uintptr_t>(g.A) & 15) == 0) &&
                       (m0 + BM <= g.M) && (kbeg % 4 == 0);
    const bool fastB = (g.ldb % 4 == 0) && ((reinterpret_cast<uintptr_t>(g.B) & 15) == 0) &&
                       (n0 + BN <= g.N) && (kbeg % 4 == 0);

    TileLoader<BM, BK, AKC> la;
    TileLoader<BN, BK, BKC> lb;

    v16f acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nk = (kend > kbeg) ? (kend - kbeg + BK - 1) / BK : 0;
    if (nk > 0) {
        la.load(g.A, g.lda, m0, g.M, kbeg, kend, fastA, tid);
        lb.load(g.B, g.ldb, n0, g.N, kbeg, kend, fastB, tid);
        la.template store<SA>(As[0], tid);
        lb.template store<SB>(Bs[0], tid);
    }
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) {
            la.load(g.A, g.lda, m0, g.M, kbeg + (kt + 1) * BK, kend, fastA, tid);
            lb.load(g.B, g.ldb, n0, g.N, kbeg + (kt + 1) * BK, kend, fastB, tid);
        }
        const float *as = As[cur] + wm * WM + li;
        const float *bs = Bs[cur] + wn * WN + li;
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
            la.template store<SA>(As[cur ^ 1], tid);
            lb.template store<SB>(Bs[cur ^ 1], tid);
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
                if (row < g.M && col < g.N) {
                    float v = acc[i][j][r];
                    if (EPI) v += g.diag[col] * g.E[row * g.lde + col];
                    Cz[row * g.ldc + col] = v;
                }
            }
        }
}

int gemm_pick_splits(int64_t M, int64_t N, int64_t K)
{
    // long reductions with a small result: use enough K splits to give every CU a workgroup,
    // keeping at least 256 rows of K per split
    const int64_t tiles = ((M + 127) / 128) * ((N + 127) / 128);
    int64_t s = (256 + tiles - 1) / tiles;
    const int64_t maxs = (K + 255) / 256;
    if (s > maxs) s = maxs;
    if (s > 64) s = 64;
    if (s < 1) s = 1;
    return (int)s;
}

template <int BM, int BN, int BK, bool AKC, bool BKC, bool EPI>
static hipError_t launch_one(const GemmArgs &a, hipStream_t s)
{
    GemmDev g;
    g.A = a.A; g.lda = a.lda; g.B = a.B; g.ldb = a.ldb; g.C = a.C; g.ldc = a.ldc;
    g.diag = a.diag; g.E = a.E; g.lde = a.lde;
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
    hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, BK, AKC, BKC, EPI>), grid, dim3(256), 0, s, g);
    return hipGetLastError();
}

template <int BM, int BN, int BK>
static hipError_t dispatch_layout(const GemmArgs &a, hipStream_t s)
{
    const bool epi = a.diag != nullptr;
    if (a.a_kcontig && a.b_kcontig)
        return epi ? launch_one<BM, BN, BK, true, true, true>(a, s)
                   : launch_one<BM, BN, BK, true, true, false>(a, s);
    if (a.a_kcontig && !a.b_kcontig)
        return epi ? launch_one<BM, BN, BK, true, false, true>(a, s)
                   : launch_one<BM, BN, BK, true, false, false>(a, s);
    if (!a.a_kcontig && !a.b_kcontig) return launch_one<BM, BN, BK, false, false, false>(a, s);
    return hipErrorInvalidValue;
}

hipError_t launch_gemm(const GemmArgs &a, hipStream_t s)
{
    if (a.M <= 0 || a.N <= 0 || a.K <= 0) return hipErrorInvalidValue;
    if (a.splits > 1 && a.diag) return hipErrorInvalidValue;
    // small problems: 64x64 tiles give the chip more workgroups to spread over
    const long tiles128 = (long)((a.M + 127) / 128) * ((a.N + 127) / 128) * (a.splits < 1 ? 1 : a.splits);
    if (tiles128 < 192) return dispatch_layout<64, 64, 16>(a, s);
    return dispatch_layout<128, 128, 16>(a, s);
}

}  // namespace ssm
