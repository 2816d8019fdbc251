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
    if (a.epilogue == 7) return launch_gemm_ws_variant<128, 128, 32, 2, 2, 8, 2, NPL, gemm_layout(true, true, 7)>(a, s);
    if (a.epilogue == 8) return launch_gemm_ws_variant<128, 128, 32, 2, 2, 8, 2, NPL, gemm_layout(true, false, 8)>(a, s);
    if (tier == 0) return dispatch_tile<128, 128, 32>(a, s);
    if (tier == 1) return dispatch_tile<64, 128, 32>(a, s);
    return dispatch_tile<64, 64, 64>(a, s);
}

}  // namespace ssm
