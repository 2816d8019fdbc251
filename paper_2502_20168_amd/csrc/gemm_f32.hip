// Tile selection and launch of the projection GEMMs.
//
// Two kernels compute the same fp32-in / fp32-out product:
//   * gemm_bf16x3_ws_kernel (default): exact three-way bf16 split of both operands, six bf16
//     MFMAs per k block accumulated in fp32 -- fp32-class accuracy at 2.7x the fp32 matrix rate;
//   * gemm_f32_kernel: plain fp32 MFMA, selected with the environment variable SSM_GEMM_F32=1
//     (kept as the reference point for the measurement of the default kernel).
#include "gemm_bf16x3_kernel.h"

#include <cstdlib>

namespace ssm {

int gemm_pick_splits(int64_t M, int64_t N, int64_t K)
{
    // long reductions with a small result: enough K splits to give half of the CUs a workgroup
    // (the two reductions of the gradient pass share one launch), keeping at least 256 rows of
    // K per split
    const int64_t tiles = ((M + 127) / 128) * ((N + 127) / 128);
    int64_t s = (128 + tiles - 1) / tiles;
    const int64_t maxs = (K + 255) / 256;
    if (s > maxs) s = maxs;
    if (s > 64) s = 64;
    if (s < 1) s = 1;
    return (int)s;
}

template <int BM, int BN, int BK, int WGM, int WGN>
static hipError_t dispatch_f32(const GemmArgs &a, hipStream_t s)
{
    const bool epi = a.epilogue == 1;
    if (a.epilogue == 2) {
        if (a.a_kcontig && a.b_kcontig) return launch_gemm_variant<BM, BN, BK, WGM, WGN, true, true, 2>(a, s);
        return hipErrorInvalidValue;
    }
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

template <int BM, int BN, int BK, int WGM, int WGN, int NP, int NS>
static hipError_t dispatch_bf16x3(const GemmArgs &a, hipStream_t s, const GemmArgs *b = nullptr)
{
    if (b) {
        if (a.a_kcontig || a.b_kcontig || b->a_kcontig || b->b_kcontig || a.epilogue || b->epilogue)
            return hipErrorInvalidValue;
        return launch_gemm_bf16x3_ws_variant<BM, BN, BK, WGM, WGN, NP, NS, false, false, false>(a, s, b);
    }
    const bool epi = a.epilogue == 1;
    if (a.epilogue == 2) {
        if (a.a_kcontig && a.b_kcontig)
            return launch_gemm_bf16x3_ws_variant<BM, BN, BK, WGM, WGN, NP, NS, true, true, 2>(a, s);
        return hipErrorInvalidValue;
    }
    if (a.a_kcontig && a.b_kcontig)
        return epi ? launch_gemm_bf16x3_ws_variant<BM, BN, BK, WGM, WGN, NP, NS, true, true, true>(a, s)
                   : launch_gemm_bf16x3_ws_variant<BM, BN, BK, WGM, WGN, NP, NS, true, true, false>(a, s);
    if (a.a_kcontig && !a.b_kcontig)
        return epi ? launch_gemm_bf16x3_ws_variant<BM, BN, BK, WGM, WGN, NP, NS, true, false, true>(a, s)
                   : launch_gemm_bf16x3_ws_variant<BM, BN, BK, WGM, WGN, NP, NS, true, false, false>(a, s);
    if (!a.a_kcontig && !a.b_kcontig && !epi)
        return launch_gemm_bf16x3_ws_variant<BM, BN, BK, WGM, WGN, NP, NS, false, false, false>(a, s);
    return hipErrorInvalidValue;
}

static bool use_f32_mfma()
{
    const char *e = std::getenv("SSM_GEMM_F32");
    return e && e[0] == '1';
}

hipError_t launch_gemm(const GemmArgs &a, hipStream_t s)
{
    if (a.M <= 0 || a.N <= 0 || a.K <= 0) return hipErrorInvalidValue;
    if (a.splits > 1 && a.epilogue) return hipErrorInvalidValue;
    if (a.epilogue < 0 || a.epilogue > 2 || (a.epilogue && (!a.diag || !a.E))) return hipErrorInvalidValue;
    const long splits = a.splits < 1 ? 1 : a.splits;
    const long tiles128 = (long)((a.M + 127) / 128) * ((a.N + 127) / 128) * splits;
    if (use_f32_mfma()) {
        // measured on MI355X: 128x128 tiles with 8 wavefronts when they give every CU a workgroup,
        // 64x64 tiles otherwise
        if (tiles128 >= 256) {
            if (a.a_kcontig && a.b_kcontig) return dispatch_f32<128, 128, 32, 4, 2>(a, s);
            return dispatch_f32<128, 128, 16, 4, 2>(a, s);
        }
        if (a.a_kcontig && a.b_kcontig) return dispatch_f32<64, 64, 32, 2, 2>(a, s);
        return dispatch_f32<64, 64, 16, 2, 2>(a, s);
    }
    // measured on MI355X at the benchmark shapes: 128x128x32 tiles, 4 consumer + 4 producer
    // wavefronts; 64x128 tiles with 8 producer wavefronts (staging per multiply-add is 1.5x there)
    // when the wide tile would leave CUs without work
    if (tiles128 >= 200) return dispatch_bf16x3<128, 128, 32, 2, 2, 4, 2>(a, s);
    return dispatch_bf16x3<64, 128, 32, 2, 2, 8, 2>(a, s);
}

// Two K = T reductions (both operands row-contiguous, no epilogue) in one launch.
hipError_t launch_gemm_pair(const GemmArgs &a, const GemmArgs &b, hipStream_t s)
{
    if (a.M <= 0 || a.N <= 0 || a.K <= 0 || b.M <= 0 || b.N <= 0 || b.K <= 0) return hipErrorInvalidValue;
    if (use_f32_mfma()) {
        hipError_t e = launch_gemm(a, s);
        return e != hipSuccess ? e : launch_gemm(b, s);
    }
    return dispatch_bf16x3<128, 128, 32, 2, 2, 4, 2>(a, s, &b);
}

}  // namespace ssm
