// Instantiations of the projection kernel that carry several independent problems in one launch
// (128x128x32 tiles).  The launches of the gradient pass:
//   C^H dy (row-major A, B read along N; plain or running the reverse scan on its output)
//                                                 with  dy^T x  (K = T reduction in slabs)
//   Bbar^H chi + D dy (same layout, epilogue 1)   with  chi^T u (K = T reduction in slabs)
// Pairs of products have the same inputs ready at the same time, and one of them alone would leave
// compute units idle.
#include "gemm_kernel.h"

namespace ssm {

hipError_t launch_gemm_pair(const GemmArgs &a, const GemmArgs &b, hipStream_t s, bool second_first)
{
    if (a.M <= 0 || a.N <= 0 || a.K <= 0 || b.M <= 0 || b.N <= 0 || b.K <= 0) return hipErrorInvalidValue;
    if ((a.splits > 1 && a.epilogue) || (b.splits > 1 && b.epilogue)) return hipErrorInvalidValue;
    constexpr int NN0 = gemm_layout(true, false, 0), NN1 = gemm_layout(true, false, 1),
                  NN8 = gemm_layout(true, false, 8), TN0 = gemm_layout(false, false, 0);
    const int la = gemm_layout_of(a), lb = gemm_layout_of(b);
    if (la == NN8 && !gemm_scan_args_ok(a)) return hipErrorInvalidValue;
    if (gemm_use_two_planes(a) && gemm_use_two_planes(b)) {
        if (la == NN8 && lb == TN0) return launch_gemm_ws_variant<128, 128, 32, 2, 2, 8, 2, 2, NN8, TN0>(a, s, &b, second_first);
        if (la == NN0 && lb == TN0) return launch_gemm_ws_variant<128, 128, 32, 2, 2, 8, 2, 2, NN0, TN0>(a, s, &b, second_first);
        if (la == NN1 && lb == TN0) return launch_gemm_ws_variant<128, 128, 32, 2, 2, 8, 2, 2, NN1, TN0>(a, s, &b, second_first);
    } else if (la != NN8) {
        if (la == NN0 && lb == TN0) return launch_gemm_ws_variant<128, 128, 32, 2, 2, 8, 2, 3, NN0, TN0>(a, s, &b, second_first);
        if (la == NN1 && lb == TN0) return launch_gemm_ws_variant<128, 128, 32, 2, 2, 8, 2, 3, NN1, TN0>(a, s, &b, second_first);
    }
    // no paired instantiation for these layouts: two launches
    hipError_t e = launch_gemm(a, s);
    return e != hipSuccess ? e : launch_gemm(b, s);
}

}  // namespace ssm
