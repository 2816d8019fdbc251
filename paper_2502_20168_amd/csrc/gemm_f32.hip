// Tile selection and launch of the fp32 MFMA GEMM (kernel template in gemm_f32_kernel.h).
#include "gemm_f32_kernel.h"

namespace ssm {

int gemm_pick_splits(int64_t M, int64_t N, int64_t K)
{
    // long reductions with a small result: enough K splits to give every CU a workgroup, keeping
    // at least 256 rows of K per split
    const int64_t tiles = ((M + 127) / 128) * ((N + 127) / 128);
    int64_t s = (256 + tiles - 1) / tiles;
    const int64_t maxs = (K + 255) / 256;
    if (s > maxs) s = maxs;
    if (s > 64) s = 64;
    if (s < 1) s = 1;
    return (int)s;
}

template <int BM, int BN, int BK, int WGM, int WGN>
static hipError_t dispatch_layout(const GemmArgs &a, hipStream_t s)
{
    const bool epi = a.diag != nullptr;
    if (a.a_kcontig && a.b_kcontig)
        return epi ? launch_gemm_variant<BM, BN, BK, WGM, WGN, true, true, true>(a, s)
                   : launch_gemm_variant<BM, BN, BK, WGM, WGN, true, true, false>(a, s);
    if (a.a_kcontig && !a.b_kcontig)
        return epi ? launch_gemm_variant<BM, BN, BK, WGM, WGN, true, false, true>(a, s)
                   : launch_gemm_variant<BM, BN, BK, WGM, WGN, true, false, false>(a, s);
    if (!a.a_kcontig && !a.b_kcontig && !epi)
        return launch_gemm_variant<BM, BN, BK, WGM, WGN, false, false, false>(a, s);
    return hipErrorInvalidValue;
}

hipError_t launch_gemm(const GemmArgs &a, hipStream_t s)
{
    if (a.M <= 0 || a.N <= 0 || a.K <= 0) return hipErrorInvalidValue;
    if (a.splits > 1 && a.diag) return hipErrorInvalidValue;
    // Measured on MI355X at the benchmark shapes: 128x128 tiles with 8 wavefronts are best when
    // they give at least one workgroup per CU; otherwise 64x64 tiles (several workgroups per CU).
    const long splits = a.splits < 1 ? 1 : a.splits;
    const long tiles128 = (long)((a.M + 127) / 128) * ((a.N + 127) / 128) * splits;
    if (tiles128 >= 256) {
        if (a.a_kcontig && a.b_kcontig) return dispatch_layout<128, 128, 32, 4, 2>(a, s);
        return dispatch_layout<128, 128, 16, 4, 2>(a, s);
    }
    if (a.a_kcontig && a.b_kcontig) return dispatch_layout<64, 64, 32, 2, 2>(a, s);
    return dispatch_layout<64, 64, 16, 2, 2>(a, s);
}

}  // namespace ssm
