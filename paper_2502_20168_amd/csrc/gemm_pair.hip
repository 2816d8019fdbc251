// Instantiations of the projection kernel that carry several independent problems in one launch
// (128x128x32 tiles).  The launches of the gradient pass:
//   shapes whose projections scan their own tiles (every operand brings its largest magnitude: two
//   scaled fp16 planes), with at least as many scanning tiles as CUs:
//     Re(Bbar^H chi) + D dy                         with  chi^T u  and  dy^T x  (K = T reductions in slabs)
//   the same with fewer scanning tiles (C^H dy alone would leave CUs idle):
//     C^H dy that scans its own tiles               with  dy^T x
//     Re(Bbar^H chi) + D dy                         with  chi^T u
//   other shapes (three bf16 planes):
//     C^H dy                                        with  dy^T x
//     Re(Bbar^H chi) + D dy                         with  chi^T u
// and of the gate's (two scaled fp16 planes):
//     dz W^T with the adjoint of the gate in its store   with  x1^T dz
// The products of a launch have their inputs ready at the same time, and one of them alone would
// leave compute units idle.
#include "gemm_kernel.h"

namespace ssm {

namespace {
constexpr int NN0 = gemm_layout(true, false, 0), NN1 = gemm_layout(true, false, 1), NN8 = gemm_layout(true, false, 8),
              TN0 = gemm_layout(false, false, 0), NT4 = gemm_layout(true, true, 4);
bool plain_problem(const GemmArgs &g)
{
    return g.M > 0 && g.N > 0 && g.K > 0 && !(g.splits > 1 && g.epilogue);
}
long items128(const GemmArgs &g)
{
    return (long)((g.M + 127) / 128) * ((g.N + 127) / 128) * (g.splits < 1 ? 1 : g.splits);
}
}  // namespace

hipError_t launch_gemm_pair(const GemmArgs &a, const GemmArgs &b, hipStream_t s, bool second_first)
{
    if (!plain_problem(a) || !plain_problem(b)) return hipErrorInvalidValue;
    const int la = gemm_layout_of(a), lb = gemm_layout_of(b);
    const int swapped[3] = {1, 0, 2};
    const int *order = second_first ? swapped : nullptr;
    const bool two = gemm_use_two_planes(a) && gemm_use_two_planes(b);
    if (two && lb == TN0) {
        // C^H dy that scans its own tiles, with the dC slabs (shapes with fewer scanning tiles than CUs: the
        // slabs fill the rest of the chip)
        if (la == NN8) {
            if (!gemm_scan_args_ok(a)) return hipErrorInvalidValue;
            return launch_gemm_ws_variant<128, 128, 32, 2, 2, 8, 2, 2, NN8, TN0>(a, s, &b, nullptr, order);
        }
        // Re(Bbar^H chi) + D dy with the dBbar slabs: two workgroups per CU when there is more than one round
        // of work items (see launch_gemm_triple)
        if (la == NN1 && items128(a) + items128(b) > 288)
            return launch_gemm_ws_variant<128, 128, 32, 2, 2, 4, 2, 2, NN1, TN0, 4>(a, s, &b, nullptr, order);
        if (la == NN1) return launch_gemm_ws_variant<128, 128, 32, 2, 2, 8, 2, 2, NN1, TN0>(a, s, &b, nullptr, order);
        // C^H dy with the dC slabs, or two K halves of Re(Bbar^H chi) with the dBbar slabs (separate scan kernels)
        if (la == NN0) return launch_gemm_ws_variant<128, 128, 32, 2, 2, 8, 2, 2, NN0, TN0>(a, s, &b, nullptr, order);
        // the adjoint of the gate: dz W^T with its store function, and the slabs of x1^T dz
        if (la == NT4) return launch_gemm_ws_variant<128, 128, 32, 2, 2, 8, 2, 2, NT4, TN0>(a, s, &b, nullptr, order);
    }
    if (!gemm_use_two_planes(a) && !gemm_use_two_planes(b) && lb == TN0) {
        if (gemm_small_pair(a.M, a.N)) {
            // few tiles: 64x64x64 tiles, so that no workgroup walks a long K loop while most CUs idle
            if (la == NN0) return launch_gemm_ws_variant<64, 64, 64, 2, 2, 8, 2, 3, NN0, TN0>(a, s, &b, nullptr, order);
            if (la == NN1) return launch_gemm_ws_variant<64, 64, 64, 2, 2, 8, 2, 3, NN1, TN0>(a, s, &b, nullptr, order);
        }
        if (la == NN0) return launch_gemm_ws_variant<128, 128, 32, 2, 2, 8, 2, 3, NN0, TN0>(a, s, &b, nullptr, order);
        if (la == NN1) return launch_gemm_ws_variant<128, 128, 32, 2, 2, 8, 2, 3, NN1, TN0>(a, s, &b, nullptr, order);
    }
    // no paired instantiation for these layouts: two launches
    hipError_t e = launch_gemm(a, s);
    return e != hipSuccess ? e : launch_gemm(b, s);
}

// a: Re(Bbar^H chi) + D dy (epilogue 1; or epilogue 0 into K halves); b, c: the two K = T reductions.
hipError_t launch_gemm_triple(const GemmArgs &a, const GemmArgs &b, const GemmArgs &c, hipStream_t s, bool slabs_first)
{
    if (!plain_problem(a) || !plain_problem(b) || !plain_problem(c)) return hipErrorInvalidValue;
    const int la = gemm_layout_of(a), lb = gemm_layout_of(b), lc = gemm_layout_of(c);
    if (gemm_use_two_planes(a) && gemm_use_two_planes(b) && gemm_use_two_planes(c) && lb == TN0 && lc == TN0) {
        // four producer wavefronts and at most 128 registers: two workgroups share a CU (their stages fill
        // its 160 KB of LDS exactly), so that the first loads and the stores of one overlap the K loop of the
        // other -- the launch has several rounds of work items (measured at 16 x 256 tokens, H = P = 512:
        // 54.5 instead of 65.3 us).
        // Re(Bbar^H chi) + D dy stored directly, its long work items (the whole K = 2P) first in every XCD, the
        // slab items fill in behind them (measured against two K halves of it plus a streaming sum: the launch
        // +1 us, the launch that summed the halves -3.8 us, 40 MB less traffic)
        // (where the slab items are the longer kind they go first instead: 1024 x 16 tokens, H = P = 512, four
        // slabs per reduction: 0.469 against 0.482 ms per step)
        const int a_first[3] = {0, 1, 2}, a_last[3] = {1, 2, 0};
        if (la == NN1) return launch_gemm_ws_variant<128, 128, 32, 2, 2, 4, 2, 2, NN1, TN0, 4>(a, s, &b, &c, slabs_first ? a_last : a_first);
    }
    hipError_t e = launch_gemm(a, s);
    if (e == hipSuccess) e = launch_gemm(b, s);
    return e != hipSuccess ? e : launch_gemm(c, s);
}

}  // namespace ssm
