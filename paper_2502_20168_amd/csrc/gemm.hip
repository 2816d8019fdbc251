// Tile selection and launch of the projection GEMMs.
//
// One kernel template (gemm_kernel.h) computes the fp32-in / fp32-out products on the 16-bit matrix
// cores with both operands split while they are staged: exactly into three bf16 planes (six bf16
// MFMAs per k block), or, when the largest magnitude of both operands is known, into two fp16 planes
// of the operand scaled by a power of two (three fp16 MFMAs per k block); fp32 accumulation and
// fp32-class accuracy either way.  The instantiations live in gemm_inst2.hip / gemm_inst3.hip (one
// problem per launch) and gemm_pair.hip (several problems per launch).
#include "gemm_kernel.h"

namespace ssm {

int gemm_pick_splits(int64_t M, int64_t N, int64_t K, int64_t partner_tiles)
{
    // A long reduction with a small result shares its launch with a product of partner_tiles
    // 128x128 tiles: enough K splits that the two together fill the last round of workgroups
    // on the 256 CUs, keeping at least 256 rows of K per split.
    const int64_t tiles = ((M + 127) / 128) * ((N + 127) / 128);
    const int64_t target = 256 - partner_tiles % 256;
    int64_t s = (target + tiles / 2) / tiles;
    const int64_t maxs = (K + 255) / 256;
    if (s > maxs) s = maxs;
    if (s > 64) s = 64;
    if (s < 1) s = 1;
    return (int)s;
}

// A product over T tokens with N columns that has few 128x128 tiles shares its launch with a K = T
// reduction on 64x64x64 tiles: a quarter of the multiply-adds per workgroup, so that the chain of K
// steps a small shape waits for is short.
// (measured: 16 and 32 leave gains on the table, 128 doubles the step at 40 x 100 tokens, H = P = 256)
constexpr int64_t SMALL_PAIR_ITEMS = 64;
bool gemm_small_pair(int64_t T, int64_t N)
{
    return ((T + 127) / 128) * ((N + 127) / 128) <= SMALL_PAIR_ITEMS;
}

// K splits of an M x N reduction over K rows that shares such a launch with a product whose K loop is
// k_main long: work items about as long as that product's, at most two rounds of workgroups in all
int gemm_pick_splits_small(int64_t M, int64_t N, int64_t K, int64_t partner_tiles64, int64_t k_main)
{
    const int64_t tiles = ((M + 63) / 64) * ((N + 63) / 64);
    int64_t s = (K + k_main / 2) / (k_main < 64 ? 64 : k_main);
    const int64_t room = (512 - partner_tiles64) / tiles;
    if (s > room) s = room;
    const int64_t maxs = (K + 63) / 64;
    if (s > maxs) s = maxs;
    if (s > 64) s = 64;
    if (s < 1) s = 1;
    return (int)s;
}

// List scheduling of nl work items of l K tiles and then ns items of s K tiles on the 256 CUs, as the
// dispatcher hands out workgroups in slot order to CUs as they fall free (a CU's two workgroups share its
// throughput, so a CU is one machine): the K tiles the busiest CU ends up with.  Loads are kept as (level, number of CUs) pairs; a batch of items goes to all CUs of
// the lowest level at once.
int64_t lpt_makespan(int64_t nl, int64_t l, int64_t ns, int64_t s)
{
    constexpr int64_t CUS = 256;
    constexpr int MAXLV = 16;
    int64_t lv[MAXLV], cnt[MAXLV];
    int n = 0;
    const int64_t q = nl / CUS, r = nl % CUS;
    lv[n] = q * l; cnt[n] = CUS - r; ++n;                    // ascending levels
    if (r) { lv[n] = (q + 1) * l; cnt[n] = r; ++n; }
    while (ns > 0) {
        const int64_t k = cnt[0] < ns ? cnt[0] : ns;
        const int64_t target = lv[0] + s;
        ns -= k;
        cnt[0] -= k;
        if (cnt[0] == 0) { for (int i = 1; i < n; ++i) { lv[i - 1] = lv[i]; cnt[i - 1] = cnt[i]; } --n; }
        int pos = 0;
        while (pos < n && lv[pos] < target) ++pos;
        if (pos < n && lv[pos] == target) { cnt[pos] += k; continue; }
        if (n == MAXLV) { lv[n - 1] = lv[n - 1] > target ? lv[n - 1] : target; cnt[n - 1] += k; continue; }   // (never with two item lengths)
        for (int i = n; i > pos; --i) { lv[i] = lv[i - 1]; cnt[i] = cnt[i - 1]; }
        lv[pos] = target; cnt[pos] = k; ++n;
    }
    return lv[n - 1];
}

// K splits of the K = T reductions (red_tiles tiles of 128x128 in all, split_bytes of slabs per split in
// all) that share a launch of 128x128x32 tiles with a product of main_tiles tiles whose K loop is k_main
// long: the count that minimises the busiest CU's K tiles plus what every further set of slabs costs (their
// bytes are written by this launch and read by the parameter epilogue's: measured 1.4 us, about 1.4 K
// tiles, per split of two reductions with 2 MiB slabs).  red_first: the reductions' work items belong in the
// first slots of the launch.  One workgroup per CU: whichever order the schedule model finishes earlier,
// the product first on a tie (measured on ten shapes with separate scan kernels: the model's choice was
// the faster order on every one, by up to 5 % of the step).  Two workgroups per CU: the reductions first
// when their items are at least twice as long as the product's (then a CU holds one of each kind for most
// of the launch instead of ending on single long items; 1024 x 16 tokens, H = P = 512: 0.469 against 0.482 ms).
int gemm_pick_splits_model(int64_t T, int64_t main_tiles, int64_t k_main, int64_t red_tiles, size_t split_bytes, bool two_per_cu,
                           bool &red_first)
{
    static const int cand[] = {1, 2, 3, 4, 5, 6, 8, 10, 12, 16, 24, 32, 48, 64};
    const int64_t a = (k_main + 31) / 32;
    const double per_split = 0.2 + 0.6 * (double)split_bytes / (double)(2 << 20);
    int best = 1;
    double best_cost = -1.0;
    red_first = false;
    for (int sp : cand) {
        if (sp > 1 && sp > T / 256) break;
        const int64_t b = (((T + sp - 1) / sp) + 31) / 32;
        const int64_t m_main = lpt_makespan(main_tiles, a, red_tiles * sp, b), m_red = lpt_makespan(red_tiles * sp, b, main_tiles, a);
        const int64_t m = m_red < m_main ? m_red : m_main;
        const double cost = (double)m + per_split * sp;
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = sp; red_first = two_per_cu ? b >= 2 * a : m_red < m_main; }
    }
    return best;
}

// (one reduction of M x N over K rows beside a product of main_tiles tiles, one workgroup per CU)
int gemm_pick_splits_balanced(int64_t M, int64_t N, int64_t K, int64_t main_tiles, int64_t k_main, bool &red_first)
{
    return gemm_pick_splits_model(K, main_tiles, k_main, ((M + 127) / 128) * ((N + 127) / 128), (size_t)M * N * 4, false, red_first);
}

// Layout code of a problem, or -1 when the projection kernel has no instantiation for it.
int gemm_layout_of(const GemmArgs &a)
{
    if (a.epilogue == 2) return (a.a_kcontig && a.b_kcontig) ? gemm_layout(true, true, 2) : -1;
    if (a.epilogue == 3) return (a.a_kcontig && !a.b_kcontig) ? gemm_layout(true, false, 3) : -1;
    if (a.epilogue == 4) return (a.a_kcontig && a.b_kcontig) ? gemm_layout(true, true, 4) : -1;
    if (a.epilogue == 6) return (a.a_kcontig && a.b_kcontig) ? gemm_layout(true, true, 6) : -1;
    if (a.epilogue == 5) return (a.a_kcontig && !a.b_kcontig && a.N % 2 == 0) ? gemm_layout(true, false, 5) : -1;
    if (a.epilogue == 7) return (a.a_kcontig && a.b_kcontig) ? gemm_layout(true, true, 7) : -1;
    if (a.epilogue == 8) return (a.a_kcontig && !a.b_kcontig) ? gemm_layout(true, false, 8) : -1;
    if (a.a_kcontig) return gemm_layout(true, a.b_kcontig != 0, a.epilogue);
    if (!a.b_kcontig && !a.epilogue) return gemm_layout(false, false, 0);
    return -1;
}

bool gemm_use_two_planes(const GemmArgs &a)
{
    // A product whose operands both come with their largest magnitude is staged as two scaled fp16
    // planes per operand (three matrix instructions per k block instead of six, same accuracy class).
    // A: one maximum, or one per row when its rows are contiguous along k; B: one maximum
    const bool a_ok = (a.amaxA.rows && a.amaxA.row_parts > 0 && a.a_kcontig) || (!a.amaxA.rows && a.amaxA.slots && a.amaxA.n > 0);
    return a_ok && a.amaxB.slots && a.amaxB.n > 0;
}

bool gemm_scan_shape_ok(int64_t Bt, int64_t L, int64_t P)
{
    // 128-row tiles that hold a piece of one sequence (a bounded chain of tiles per sequence) or a
    // whole number of sequences made of whole 16-step chunks, and enough tiles
    const bool chain = L % SCAN_TILE == 0 && L / SCAN_TILE <= SCAN_MAX_CHAIN;
    const bool whole = L < SCAN_TILE && SCAN_TILE % L == 0 && L % SCAN_RC == 0 && (Bt * L) % SCAN_TILE == 0;
    if (!chain && !whole) return false;
    // (measured: from 64 tiles on -- a quarter of the CUs -- the scanning tile with its two fp16 planes beats
    // smaller tiles plus a scan kernel: +2 % at 64 tiles, +7..13 % at 96-128; no difference at 32-48)
    constexpr int64_t SCAN_MIN_TILES = 64;
    const int64_t tiles = (Bt * L / SCAN_TILE) * ((2 * P + SCAN_TILE - 1) / SCAN_TILE);
    return tiles >= SCAN_MIN_TILES && tiles * 64 <= 0x7fffffffLL;
}

// argument checks shared by the two scanning epilogues
bool gemm_scan_args_ok(const GemmArgs &a)
{
    if (a.splits > 1 || !a.scan.lam || !a.scan.err || a.scan.L <= 0) return false;
    const int L = a.scan.L;
    const bool chain = L % SCAN_TILE == 0 && L / SCAN_TILE <= SCAN_MAX_CHAIN && a.scan.desc;
    const bool whole = L < SCAN_TILE && SCAN_TILE % L == 0 && L % SCAN_RC == 0 && a.M % SCAN_TILE == 0;
    if (!chain && !whole) return false;
    if (a.M % L != 0 || a.N != 2 * a.scan.P || !a.a_kcontig) return false;
    if (a.epilogue == 7) return a.b_kcontig != 0;
    return !a.b_kcontig && a.scan.xsaved && a.scan.partial;
}

size_t gemm_scan_desc_bytes(int64_t Bt, int64_t L, int64_t P)
{
    if (L < SCAN_TILE) return 0;                     // whole sequences per tile: nothing is handed over
    const int64_t tiles = (Bt * L / SCAN_TILE) * ((2 * P + SCAN_TILE - 1) / SCAN_TILE);
    return (size_t)tiles * 64 * 2 * sizeof(unsigned long long);
}

// du = Re(Bbar^H chi) + D dy has only M/128 * H/128 tiles of 128x128.  Where they would fill less than the
// chip but twice as many would (and the launch is shared with the dBbar slabs on three bf16 planes), it
// runs as two halves of K into two slabs that the parameter epilogue's launch adds.
bool gemm_out_split_shape(int64_t T, int64_t H, int64_t P)
{
    // a half must still be long enough (8 K tiles) to pay for the sum
    const int64_t tiles = ((T + 127) / 128) * ((H + 127) / 128);
    return tiles < 200 && 2 * tiles >= 200 && P >= 256 && (2 * P) % 64 == 0;
}

// Tile tier of an M x N product with `splits` K splits: 0 = 128x128x32 tiles, 1 = 64x128x32, 2 = 64x64x64.
// The launch takes about (rounds of workgroups on the 256 CUs) x (K steps) x (time of a K step); a K step of a
// 64x128x32 tile takes as long as one of a 128x128x32 tile, one of a 64x64x64 tile 1.2 times as long for twice
// the K range (measured), so per unit of K the tiers cost rounds x 1, 1 and 0.6.  The cheapest wins, the
// smaller tile on a tie (more CUs share the work).  (The rule before, "the largest tile that still gives 200
// workgroups", took 64x128 tiles for 192 tiles of 128x128: two rounds instead of one, 40 us instead of 24.)
int gemm_tile_tier(int64_t M, int64_t N, int splits_in)
{
    const int64_t splits = splits_in < 1 ? 1 : splits_in;
    const int64_t r0 = (((M + 127) / 128) * ((N + 127) / 128) * splits + 255) / 256;
    const int64_t r1 = (((M + 63) / 64) * ((N + 127) / 128) * splits + 255) / 256;
    const int64_t r2 = (((M + 63) / 64) * ((N + 63) / 64) * splits + 255) / 256;
    const int64_t c0 = 10 * r0, c1 = 10 * r1, c2 = 6 * r2;
    if (c2 < c0 && c2 < c1) return 2;
    return c1 <= c0 ? 1 : 0;
}

hipError_t launch_gemm(const GemmArgs &a, hipStream_t s)
{
    if (a.M <= 0 || a.N <= 0 || a.K <= 0) return hipErrorInvalidValue;
    const bool two = gemm_use_two_planes(a);
    if (a.epilogue == 7 || a.epilogue == 8) {
        // a projection that scans its own output (forward: the input projection; reverse: C^H dy): 128x128 tiles only
        if (!gemm_scan_args_ok(a) || gemm_layout_of(a) < 0) return hipErrorInvalidValue;
        return two ? gemm_dispatch_two_planes(a, 0, s) : gemm_dispatch_three_planes(a, 0, s);
    }
    if (a.splits > 1 && a.epilogue) return hipErrorInvalidValue;
    if (a.epilogue < 0 || a.epilogue > 6 || (a.epilogue && a.epilogue != 5 && !a.E)) return hipErrorInvalidValue;
    if (a.epilogue == 5 && a.C2 && !a.diag) return hipErrorInvalidValue;
    if ((a.epilogue == 1 || a.epilogue == 2 || a.epilogue == 6) && !a.diag) return hipErrorInvalidValue;
    if (a.epilogue == 6 && !a.C2) return hipErrorInvalidValue;
    if (a.epilogue == 4 && !a.E2) return hipErrorInvalidValue;
    if (gemm_layout_of(a) < 0) return hipErrorInvalidValue;
    const int tier = gemm_tile_tier(a.M, a.N, a.splits);
    return two ? gemm_dispatch_two_planes(a, tier, s) : gemm_dispatch_three_planes(a, tier, s);
}

}  // namespace ssm
