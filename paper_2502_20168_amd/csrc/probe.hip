// Measurement aid: the matrix-instruction stream of the projection kernel's consumer wavefronts
// with nothing around it (no LDS, no global memory in the loop, no producers), on operands whose
// bits change like real data.  What it reaches is the rate the matrix cores sustain on this
// device at the clock they hold under that load: the ceiling of the projection kernel.
#include "ssm_internal.h"
#include "../../include/ssm.h"

namespace ssm {

typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 probe_f16x8 __attribute__((ext_vector_type(8)));
typedef float probe_v16f __attribute__((ext_vector_type(16)));

__device__ __forceinline__ unsigned probe_hash(unsigned x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

// 256 threads = four wavefronts, one per SIMD; every wavefront issues, per iteration, the 24
// instructions of one 16-wide k step of a 64x64 output block with three bf16 planes (six plane
// products, four accumulators), or of two such steps with two fp16 planes (three products each).
template <bool F16>
__global__ void __launch_bounds__(256) mfma_probe_kernel(float *out, int iters)
{
    union Frag { unsigned u[4]; probe_bf16x8 v; probe_f16x8 h; };
    // sign and mantissa bits change, the exponent field stays at that of one
    constexpr unsigned KEEP = F16 ? 0x83ff83ffu : 0x807f807fu, ONE = F16 ? 0x3c003c00u : 0x3f003f00u;
    Frag a[2][3], b[2][3];
    const unsigned id = blockIdx.x * 256u + threadIdx.x;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int s = 0; s < 3; ++s)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                // exponent fields kept near one so that nothing overflows: random sign and mantissa bits
                a[i][s].u[w] = (probe_hash(id * 97u + i * 31u + s * 7u + w) & KEEP) | ONE;
                b[i][s].u[w] = (probe_hash(id * 89u + i * 29u + s * 5u + w + 1000u) & KEEP) | ONE;
            }
    probe_v16f acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    constexpr int PA[6] = {2, 1, 0, 1, 0, 0}, PB[6] = {0, 1, 2, 0, 1, 0};
    constexpr int PA2[6] = {1, 0, 0, 2, 0, 0}, PB2[6] = {0, 1, 0, 0, 2, 0};      // (second step: plane 2 stands in for plane 1)
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int p = 0; p < 6; ++p)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    if (F16) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i][PA2[p]].h, b[j][PB2[p]].h, acc[i][j], 0, 0, 0);
                    else acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i][PA[p]].v, b[j][PB[p]].v, acc[i][j], 0, 0, 0);
                }
        // new mantissa and sign bits for the next step (a dozen integer operations per 24 matrix instructions)
        const unsigned m = probe_hash(it * 2654435761u + id) & KEEP;
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            a[s & 1][s].u[s] ^= m;
            b[(s + 1) & 1][s].u[3 - s] ^= (m >> 1) & KEEP;
        }
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) sum += acc[i][j][r];
    out[id] = sum;
}

}  // namespace ssm

extern "C" ssm_status ssm_mfma_probe(int64_t workgroups, int64_t iters, int fp16, float *out, void *stream)
{
    if (!out || workgroups <= 0 || iters <= 0) return SSM_ERR_INVALID_ARG;
    if (workgroups > 65536 || iters > (1 << 24)) return SSM_ERR_UNSUPPORTED;
    if (fp16)
        hipLaunchKernelGGL(ssm::mfma_probe_kernel<true>, dim3((unsigned)workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                           out, (int)iters);
    else
        hipLaunchKernelGGL(ssm::mfma_probe_kernel<false>, dim3((unsigned)workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                           out, (int)iters);
    return hipGetLastError() == hipSuccess ? SSM_OK : SSM_ERR_HIP;
}
