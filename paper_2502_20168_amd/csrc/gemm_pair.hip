// Instantiations of the projection kernel that carry several independent problems in one launch
// (128x128x32 tiles).  The launches of the gradient pass:
//   shapes whose projections scan their own tiles (every operand brings its largest magnitude: two
//   scaled fp16 planes):
//     Re(Bbar^H chi) (+ D dy, or as two K halves)  with  chi^T u  and  dy^T x  (K = T reductions in slabs)
//   other shapes (three bf16 planes):
//     C^H dy                                        with  dy^T x
//     Re(Bbar^H chi) + D dy                         with  chi^T u
// The products of a launch have their inputs ready at the same time, and one of them alone would
// leave compute units idle.
#include "gemm_kernel.h"

namespace ssm {

namespace {
constexpr int NN0 = gemm_layout(true, false, 0), NN1 = gemm_layout(true, false, 1), TN0 = gemm_layout(false, false, 0);
bool plain_problem(const GemmArgs &g)
{
    return g.M > 0 && g.N > 0 && g.K > 0 && !(g.splits > 1 && g.epilogue);
}
}  // namespace

hipError_t launch_gemm_pair(const GemmArgs &a, const GemmArgs &b, hipStream_t s, bool second_first)
{
    if (!plain_problem(a) || !plain_problem(b)) return hipErrorInvalidValue;
    const int la = gemm_layout_of(a), lb = gemm_layout_of(b);
    const int swapped[3] = {1, 0, 2};
    const int *order = second_first ? swapped : nullptr;
    if (!gemm_use_two_planes(a) && !gemm_use_two_planes(b) && lb == TN0) {
        if (la == NN0) return launch_gemm_ws_variant<128, 128, 32, 2, 2, 8, 2, 3, NN0, TN0>(a, s, &b, nullptr, order);
        if (la == NN1) return launch_gemm_ws_variant<128, 128, 32, 2, 2, 8, 2, 3, NN1, TN0>(a, s, &b, nullptr, order);
    }
    // no paired instantiation for these layouts: two launches
    hipError_t e = launch_gemm(a, s);
    return e != hipSuccess ? e : launch_gemm(b, s);
}

// a: Re(Bbar^H chi) (epilogue 0 as K halves, or epilogue 1); b, c: the two K = T reductions.  Work items
// take the slots of every XCD in the order b, c, a: the reductions stream their operands from memory,
// the product with the weights finds chi in the cache behind them.
hipError_t launch_gemm_triple(const GemmArgs &a, const GemmArgs &b, const GemmArgs &c, hipStream_t s)
{
    if (!plain_problem(a) || !plain_problem(b) || !plain_problem(c)) return hipErrorInvalidValue;
    const int la = gemm_layout_of(a), lb = gemm_layout_of(b), lc = gemm_layout_of(c);
    const int order[3] = {1, 2, 0};
    if (gemm_use_two_planes(a) && gemm_use_two_planes(b) && gemm_use_two_planes(c) && lb == TN0 && lc == TN0) {
        if (la == NN0) return launch_gemm_ws_variant<128, 128, 32, 2, 2, 8, 2, 2, NN0, TN0>(a, s, &b, &c, order);
        if (la == NN1) return launch_gemm_ws_variant<128, 128, 32, 2, 2, 8, 2, 2, NN1, TN0>(a, s, &b, &c, order);
    }
    hipError_t e = launch_gemm(a, s);
    if (e == hipSuccess) e = launch_gemm(b, s);
    return e != hipSuccess ? e : launch_gemm(c, s);
}

}  // namespace ssm
