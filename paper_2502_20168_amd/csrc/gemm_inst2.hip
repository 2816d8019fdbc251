// Instantiations of the projection kernel with two scaled fp16 planes per operand, one problem per
// launch: every operand layout and store function the library uses, on the three tile tiers.
#include "gemm_kernel.h"

namespace ssm {

template <int BM, int BN, int BK>
static hipError_t dispatch_tile(const GemmArgs &a, hipStream_t s)
{
    constexpr int NPL = 2;
    switch (gemm_layout_of(a)) {
#define SSM_CASE(akc, bkc, epi) \
    case gemm_layout(akc, bkc, epi): \
        return launch_gemm_ws_variant<BM, BN, BK, 2, 2, 8, 2, NPL, gemm_layout(akc, bkc, epi)>(a, s);
        SSM_CASE(true, true, 0) SSM_CASE(true, true, 1) SSM_CASE(true, true, 2)
        SSM_CASE(true, false, 0) SSM_CASE(true, false, 1) SSM_CASE(false, false, 0)
        SSM_CASE(true, false, 3) SSM_CASE(true, true, 4) SSM_CASE(true, false, 5) SSM_CASE(true, true, 6)
#undef SSM_CASE
    default: return hipErrorInvalidValue;
    }
}

// tier 0: 128x128x32 tiles, 1: 64x128x32, 2: 64x64x64; the scanning epilogues exist on tier 0 only
hipError_t gemm_dispatch_two_planes(const GemmArgs &a, int tier, hipStream_t s)
{
    constexpr int NPL = 2;
    if (a.epilogue == 7 || a.epilogue == 8) {
        // More tiles than CUs: four producer wavefronts and at most 128 registers, so that two workgroups
        // share a CU and the scan, the stores and the first loads of one overlap the K loop of the other
        // (4 x 4096 tokens, H = P = 256: input projection 37.7 instead of 44.7 us, C^H dy 45.4 instead of 49.7;
        // 1024 x 16 tokens, H = P = 512: C^H dy 99 instead of 107 us).  One round of tiles or less: eight
        // producers, one workgroup per CU.
        const long tiles = (long)((a.M + 127) / 128) * ((a.N + 127) / 128);
        if (tiles > 256 && a.epilogue == 7)
            return launch_gemm_ws_variant<128, 128, 32, 2, 2, 4, 2, NPL, gemm_layout(true, true, 7), -1, 4>(a, s);
        if (tiles > 256 && a.epilogue == 8)
            return launch_gemm_ws_variant<128, 128, 32, 2, 2, 4, 2, NPL, gemm_layout(true, false, 8), -1, 4>(a, s);
        if (a.epilogue == 7) return launch_gemm_ws_variant<128, 128, 32, 2, 2, 8, 2, NPL, gemm_layout(true, true, 7)>(a, s);
        return launch_gemm_ws_variant<128, 128, 32, 2, 2, 8, 2, NPL, gemm_layout(true, false, 8)>(a, s);
    }
    // (a plain product with several rounds of long work items gains nothing from two workgroups per CU: measured)
    // The output projection (both operands k-contiguous, D u added in the store; K = 2P is its longest
    // contraction) walks K in steps of 64 on 64x128 tiles where K allows: half the workgroup barriers per
    // product (16 x 256 tokens, H = P = 512: -2 to -3 us per step; the other layouts of this tier gain nothing)
    const int lay = gemm_layout_of(a);
    const bool out_like = lay == gemm_layout(true, true, 1) || lay == gemm_layout(true, true, 6);
    if (tier == 1 && out_like && a.K % 64 == 0 && a.splits <= 1) {
        if (lay == gemm_layout(true, true, 1)) return launch_gemm_ws_variant<64, 128, 64, 2, 2, 8, 2, NPL, gemm_layout(true, true, 1)>(a, s);
        return launch_gemm_ws_variant<64, 128, 64, 2, 2, 8, 2, NPL, gemm_layout(true, true, 6)>(a, s);
    }
    // (the same on 128x128 tiles: no change, measured)
    if (tier == 0) return dispatch_tile<128, 128, 32>(a, s);
    if (tier == 1) return dispatch_tile<64, 128, 32>(a, s);
    return dispatch_tile<64, 64, 64>(a, s);
}

}  // namespace ssm
