// Host side of libssmscan: argument validation, workspace layout and the kernel sequences of
// the forward and the gradient pass.  See include/ssm.h for the contract of every entry point.
#include "../../include/ssm.h"
#include "../../include/ssm_measure.h"
#include "ssm_internal.h"

#include <atomic>
#include <vector>

using namespace ssm;

namespace ssm {

namespace {
constexpr size_t WS_ALIGN = 256;
inline size_t up256(size_t v) { return (v + WS_ALIGN - 1) / WS_ALIGN * WS_ALIGN; }
inline bool off_align(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }
}  // namespace

int make_scan_layout(int64_t Bt, int64_t L, int64_t P, bool rev, ScanOnlyLayout &o)
{
    if (Bt <= 0 || L <= 0 || P <= 0) return SSM_ERR_INVALID_ARG;
    if (P > SSM_MAX_WIDTH) return SSM_ERR_UNSUPPORTED;
    if (Bt > SSM_MAX_TOKENS || L > SSM_MAX_TOKENS || Bt > SSM_MAX_TOKENS / L) return SSM_ERR_UNSUPPORTED;
    if (Bt * L > SSM_MAX_ELEMS / (2 * P)) return SSM_ERR_UNSUPPORTED;
    o.plan = plan_scan(Bt, L, P);
    if (o.plan.nblocks > 0x7fffffffLL) return SSM_ERR_UNSUPPORTED;
    size_t off = 0;
    o.hdr = off; off += up256(sizeof(WsHeader));
    o.ticket = off; off += up256(o.plan.ticket_bytes);
    o.desc = off; off += up256(o.plan.desc_bytes);
    o.dApart = off; if (rev) off += up256(o.plan.partial_elems * 8);
    o.total = off;
    return SSM_OK;
}

// ssm_scan_states on a caller's workspace, or on the built-in scratch of the no-allocation entry point
int scan_states_forward(const void *A_bar, void *v, const uint8_t *is_first, const void *x0, int64_t Bt, int64_t L,
                        int64_t P, void *x_last, void *workspace, size_t ws_bytes, hipStream_t s)
{
    if (!A_bar || !v) return SSM_ERR_INVALID_ARG;
    ScanOnlyLayout lo;
    const int st = make_scan_layout(Bt, L, P, false, lo);
    if (st != SSM_OK) return st;
    if (off_align(A_bar, 8) || off_align(v, 8) || off_align(x0, 8) || off_align(x_last, 8)) return SSM_ERR_INVALID_ARG;
    if (!workspace || off_align(workspace, WS_ALIGN) || ws_bytes < lo.total) return SSM_ERR_WORKSPACE;
    char *ws = static_cast<char *>(workspace);
    WsHeader *hdr = reinterpret_cast<WsHeader *>(ws + lo.hdr);
    ScanDesc *desc = reinterpret_cast<ScanDesc *>(ws + lo.desc);
    if (lo.plan.nTB > 1 &&
        launch_clear(hdr, ws + lo.ticket, lo.desc + up256(lo.plan.desc_bytes) - lo.ticket, s) != hipSuccess)
        return SSM_ERR_HIP;
    ScanArgs sa{};
    sa.in = static_cast<const float2 *>(v); sa.out = static_cast<float2 *>(v);
    sa.lam = static_cast<const float2 *>(A_bar); sa.is_first = is_first;
    sa.x0 = static_cast<const float2 *>(x0); sa.x_last = static_cast<float2 *>(x_last);
    sa.desc = desc; sa.ticket = reinterpret_cast<uint32_t *>(ws + lo.ticket); sa.err = &hdr->err;
    sa.Bt = (int)Bt; sa.L = (int)L; sa.P = (int)P;
    sa.pxb = lo.plan.pxb; sa.cy = lo.plan.cy; sa.nPX = lo.plan.nPX; sa.nTB = lo.plan.nTB;
    sa.spin_limit = scan_spin_limit();
    return launch_scan(sa, false, s) == hipSuccess ? SSM_OK : SSM_ERR_HIP;
}

// upper bound on the polls of one cross-workgroup wait (each poll sleeps ~128 clocks); the only
// process-wide setting of the library, changed through ssm_set_spin_limit (a test hook)
static std::atomic<uint32_t> g_spin_limit{1u << 20};
uint32_t scan_spin_limit() { return g_spin_limit.load(std::memory_order_relaxed); }
uint32_t scan_set_spin_limit(uint32_t polls) { return g_spin_limit.exchange(polls, std::memory_order_relaxed); }

}  // namespace ssm

namespace {

constexpr size_t ALIGN = 256;
inline size_t up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }

constexpr int64_t SMALL_HALVES_MIN_P = 256;      // a small du as two K halves: each half keeps four K steps of 64
struct Layout {
    ScanPlan plan;
    int splitC, splitB, nslab;
    // scanning shapes with fewer scanning tiles than CUs: the dC slabs share the launch of C^H dy (they need
    // the largest magnitude of the saved states from a pass of the prep launch); otherwise they wait for the
    // launch of Re(Bbar^H chi), and the reverse scan records that magnitude on its way
    bool dc_early;
    // separate scan kernels, products of more than 64 tiles: two scaled fp16 planes there too (the scan kernels
    // record the largest magnitude of every token row of x and chi with atomics, the prep launch measures the rest)
    bool planes2_unfused;
    bool slabs_first;        // launch of three products: the slabs' work items go first
    bool dc_first, db_first; // launches of two products (separate scan kernels): the slab items go first
    size_t hdr, lam, Bri, Cc, xbuf, chi, ticket, desc, dCpart, dBpart, dApart, dDpart, fdesc, fdesc_bytes, yhalves, total;
    // largest magnitudes of the operands of the products (shapes whose projections scan their own tiles):
    // amax_atomic: 2 x ABSMAX_SLOTS words gathered with atomics, directly before fdesc so that one range is
    // cleared; amax_slots: [P] Bbar, [H] Cc, then 2 x PREP_PASS_BLOCKS and 2 x amax_cd words of the passes
    size_t amax_atomic, amax_slots; int amax_cd;
    // per-row maxima of the operands whose rows are tokens: rowmax (u forward: [T]; dy gradient pass: [ceil(H/64), T]) and
    // rowpart [ceil(2P/128), T] (x forward, chi gradient pass: one word per column tile of the scanning projection)
    size_t rowmax, rowpart; int row_parts;
};

// K splits of the two K = T reductions that share the launch of du (shapes whose projections scan their
// own tiles, more scanning tiles than 192), two workgroups per CU; slabs_first: their work items take the
// first slots of the launch.
int pick_triple_splits(int64_t T, int64_t H, int64_t P, bool &slabs_first)
{
    const int64_t n_du = ((T + 127) / 128) * ((H + 127) / 128);
    const int64_t slab_tiles = 2 * ((2 * P + 127) / 128) * ((H + 127) / 128);
    return gemm_pick_splits_model(T, n_du, 2 * P, slab_tiles, (size_t)2 * 2 * P * H * 4, true, slabs_first);
}

ssm_status check_dims(int64_t Bt, int64_t L, int64_t H, int64_t P)
{
    if (Bt <= 0 || L <= 0 || H <= 0 || P <= 0) return SSM_ERR_INVALID_ARG;
    if (H > SSM_MAX_WIDTH || P > SSM_MAX_WIDTH) return SSM_ERR_UNSUPPORTED;
    if (Bt > SSM_MAX_TOKENS || L > SSM_MAX_TOKENS || Bt > SSM_MAX_TOKENS / L) return SSM_ERR_UNSUPPORTED;
    const int64_t w = H > 2 * P ? H : 2 * P;
    if (Bt * L > SSM_MAX_ELEMS / w) return SSM_ERR_UNSUPPORTED;
    return SSM_OK;
}

ssm_status make_layout(int64_t Bt, int64_t L, int64_t H, int64_t P, bool bwd, Layout &o)
{
    ssm_status st = check_dims(Bt, L, H, P);
    if (st != SSM_OK) return st;
    const size_t T = (size_t)Bt * L;
    o.plan = plan_scan(Bt, L, P);
    if (o.plan.nblocks > 0x7fffffffLL) return SSM_ERR_UNSUPPORTED;
    const int64_t rows128 = ((int64_t)T + 127) / 128;
    bool du_small_halves = false;     // a small du on 64x64x64 tiles as two K halves (summed in the parameter epilogue's launch)
    o.slabs_first = o.dc_first = o.db_first = false;
    o.dc_early = gemm_scan_shape_ok(Bt, L, P) && rows128 * ((2 * P + 127) / 128) <= 192;
    if (gemm_scan_shape_ok(Bt, L, P) && !o.dc_early) {
        // dy^T x and chi^T u share the launch of Re(Bbar^H chi)
        o.splitC = o.splitB = pick_triple_splits((int64_t)T, H, P, o.slabs_first);
    } else {
        o.splitC = gemm_pick_splits(H, 2 * P, (int64_t)T, rows128 * ((2 * P + 127) / 128));   // shares C^H dy's launch
        o.splitB = gemm_pick_splits(2 * P, H, (int64_t)T, rows128 * ((H + 127) / 128));       // shares Bbar^H chi's launch
        if (!gemm_scan_shape_ok(Bt, L, P)) {
            // separate scan kernels: a launch of two products with several rounds of work items
            o.splitC = gemm_pick_splits_balanced(H, 2 * P, (int64_t)T, rows128 * ((2 * P + 127) / 128), H, o.dc_first);
            const bool du_halves = gemm_out_split_shape((int64_t)T, H, P);     // du as two K halves (see yhalves below)
            o.splitB = gemm_pick_splits_balanced(2 * P, H, (int64_t)T, rows128 * ((H + 127) / 128) * (du_halves ? 2 : 1),
                                                 du_halves ? P : 2 * P, o.db_first);
        }
        const int64_t rows64 = ((int64_t)T + 63) / 64;
        if (gemm_small_pair((int64_t)T, 2 * P))
            o.splitC = gemm_pick_splits_small(H, 2 * P, (int64_t)T, rows64 * ((2 * P + 63) / 64), H);
        if (gemm_small_pair((int64_t)T, H)) {
            // (measured: a gain when both halves keep four K steps and fit one round of workgroups with room for the slabs)
            du_small_halves = bwd && P >= SMALL_HALVES_MIN_P && 2 * rows64 * ((H + 63) / 64) <= 256;
            o.splitB = du_small_halves ? gemm_pick_splits_small(2 * P, H, (int64_t)T, 2 * rows64 * ((H + 63) / 64), P)
                                       : gemm_pick_splits_small(2 * P, H, (int64_t)T, rows64 * ((H + 63) / 64), 2 * P);
        }
    }
    o.nslab = coldot_slabs((int64_t)T);
    size_t off = 0;
    o.hdr = off; off += up(sizeof(WsHeader));
    o.lam = off; off += up((size_t)P * 8);
    o.Bri = off; off += up((size_t)2 * P * H * 4);
    o.Cc = off; off += up((size_t)2 * P * H * 4);
    o.ticket = off; off += up(o.plan.ticket_bytes);       // tickets and descriptors are contiguous
    o.desc = off; off += up(o.plan.desc_bytes);
    o.xbuf = o.chi = o.dCpart = o.dBpart = o.dApart = o.dDpart = o.fdesc = o.fdesc_bytes = 0;
    size_t dA_elems = o.plan.partial_elems;
    o.amax_atomic = o.amax_slots = o.rowmax = o.rowpart = 0; o.amax_cd = o.row_parts = 0;
    // (measured on eleven shapes: a gain of 6-16 % per step where both contraction lengths are long, H >= 512 and
    // 2P >= 1024; with shorter ones the maxima the scan kernels and the prep launch then record cost more than the
    // third fewer matrix instructions save: 3-9 % slower)
    o.planes2_unfused = !gemm_scan_shape_ok(Bt, L, P) && !gemm_small_pair((int64_t)T, 2 * P) && !gemm_small_pair((int64_t)T, H) &&
                        H >= 512 && P >= 512;
    if (o.planes2_unfused) {
        o.amax_atomic = off; off += 2 * ABSMAX_SLOTS * 4;            // chi / x (atomic slots of the scan kernels)
        o.row_parts = 1;
        o.rowpart = off; off += up(T * 4);                           // rows of x / chi, directly behind: one range is cleared
        o.amax_cd = o.nslab * (int)((H + 63) / 64);
        o.amax_slots = off; off += up((size_t)(P + H + 2 * PREP_PASS_BLOCKS + 2 * o.amax_cd) * 4);
        o.rowmax = off; off += up(T * (size_t)((H + 63) / 64) * 4);
    }
    if (gemm_scan_shape_ok(Bt, L, P)) {              // tagged words of a projection that scans its own output
        static_assert(ABSMAX_SLOTS * 4 % ALIGN == 0, "the atomic slots and the tagged words are cleared as one range");
        o.amax_atomic = off; off += 2 * ABSMAX_SLOTS * 4;            // chi, then the saved states (gradient pass)
        o.fdesc_bytes = gemm_scan_desc_bytes(Bt, L, P);
        o.fdesc = off; off += up(o.fdesc_bytes);
        o.amax_cd = o.nslab * (int)((H + 63) / 64);
        o.amax_slots = off; off += up((size_t)(P + H + 2 * PREP_PASS_BLOCKS + 2 * o.amax_cd) * 4);
        o.row_parts = (int)((2 * P + 127) / 128);
        o.rowmax = off; off += up(T * (size_t)((H + 63) / 64) * 4);
        o.rowpart = off; off += up(T * (size_t)o.row_parts * 4);
        const size_t per_tile = (size_t)(Bt * L / 128) * P;        // one dAbar row per 128-row tile
        if (per_tile > dA_elems) dA_elems = per_tile;
    }
    o.yhalves = 0;
    if (!bwd) {
        o.xbuf = off; off += up(T * P * 8);
    } else {
        o.chi = off; off += up(T * P * 8);
        o.dCpart = off; off += up((size_t)o.splitC * 2 * P * H * 4);
        o.dBpart = off; off += up((size_t)o.splitB * 2 * P * H * 4);
        o.dApart = off; off += up(dA_elems * 8);
        o.dDpart = off; off += up((size_t)o.nslab * H * 4);
        // two K halves of du, where it shares its launch with the dBbar slabs only (at the scanning shapes it
        // runs whole, first in a launch of three problems with two workgroups per CU)
        if (!gemm_scan_shape_ok(Bt, L, P) && (gemm_out_split_shape((int64_t)T, H, P) || du_small_halves)) { o.yhalves = off; off += up(2 * T * H * 4); }
    }
    o.total = off;
    return SSM_OK;
}

// pieces of the pass that measures the largest magnitude of n floats (each workgroup takes whole
// rounds of 256 float4 units)
inline int pass_pieces(size_t n)
{
    const size_t rounds = (n / 4 + 256 * 4 - 1) / (256 * 4);
    return (int)(rounds < 1 ? 1 : (rounds > (size_t)PREP_PASS_BLOCKS ? (size_t)PREP_PASS_BLOCKS : rounds));
}

// workgroups of the pass that measures the largest magnitude of every row: a row per wavefront (four
// wavefronts per workgroup) while that stays within the limit, else four rows per wavefront at a time
inline int row_pass_blocks(size_t rows)
{
    const size_t b = (rows + 3) / 4;
    return (int)(b < 1 ? 1 : (b > (size_t)PREP_ROW_PASS_BLOCKS ? (size_t)PREP_ROW_PASS_BLOCKS : b));
}

inline bool misaligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

inline uint32_t spin_limit() { return scan_spin_limit(); }

// Records an event on the stream around every stage when timing is requested.
struct StageTimer {
    hipStream_t s;
    std::vector<hipEvent_t> ev;
    bool ok = true;
    explicit StageTimer(hipStream_t st) : s(st) {}
    void mark()
    {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) { ok = false; return; }
        if (hipEventRecord(e, s) != hipSuccess) ok = false;
        ev.push_back(e);
    }
    bool finish(float *ms, int n)
    {
        if (hipStreamSynchronize(s) != hipSuccess) ok = false;
        for (int i = 0; i < n; ++i) {
            ms[i] = 0.f;
            if (ok && i + 1 < (int)ev.size() && hipEventElapsedTime(&ms[i], ev[i], ev[i + 1]) != hipSuccess) ok = false;
        }
        for (hipEvent_t e : ev) (void)hipEventDestroy(e);
        ev.clear();
        return ok;
    }
};
#define MARK() do { if (timer) timer->mark(); } while (0)
#define HIP_TRY(expr) do { if ((expr) != hipSuccess) return SSM_ERR_HIP; } while (0)

// The S5 block: the gate's product consumes GELU(y) and W as two scaled fp16 planes, so the layer's forward
// pass measures them on its way: the rows of GELU(y) where the output projection stores it, W in a pass
// of the prep launch.
struct GateMax { unsigned *x1_rowmax; const float *W; size_t nW; unsigned *wslots; int nwslots; };

ssm_status run_fwd(const ssm_c64 *Lambda, const ssm_c64 *B, const ssm_c64 *C, const float *D,
                   const float *log_delta, const float *u, const uint8_t *is_first, const ssm_c64 *x0,
                   int64_t Bt, int64_t L, int64_t H, int64_t P, float *y, ssm_c64 *x, ssm_c64 *x_last,
                   void *workspace, size_t ws_bytes, hipStream_t s, StageTimer *timer, float *gelu_y = nullptr,
                   const GateMax *gate_max = nullptr)
{
    if (!Lambda || !B || !C || !D || !log_delta || !u || !y) return SSM_ERR_INVALID_ARG;
    Layout lo;
    ssm_status st = make_layout(Bt, L, H, P, false, lo);
    if (st != SSM_OK) return st;
    if (misaligned(Lambda, 8) || misaligned(B, 8) || misaligned(C, 8) || misaligned(D, 4) ||
        misaligned(log_delta, 4) || misaligned(u, 4) || misaligned(y, 4) || misaligned(x, 8) ||
        misaligned(x0, 8) || misaligned(x_last, 8))
        return SSM_ERR_INVALID_ARG;
    if (!workspace || misaligned(workspace, ALIGN) || ws_bytes < lo.total) return SSM_ERR_WORKSPACE;

    char *ws = static_cast<char *>(workspace);
    WsHeader *hdr = reinterpret_cast<WsHeader *>(ws + lo.hdr);
    float2 *lam = reinterpret_cast<float2 *>(ws + lo.lam);
    float *Bri = reinterpret_cast<float *>(ws + lo.Bri);
    float *Cc = reinterpret_cast<float *>(ws + lo.Cc);
    ScanDesc *desc = reinterpret_cast<ScanDesc *>(ws + lo.desc);
    float2 *xs = x ? reinterpret_cast<float2 *>(x) : reinterpret_cast<float2 *>(ws + lo.xbuf);
    const int T = (int)(Bt * L);

    // Shapes whose sequences are whole numbers of 128-row tiles: the input projection scans its own
    // output tile and stores the states directly (no scan kernel, Bbar u never goes to memory).
    const bool fused = gemm_scan_shape_ok(Bt, L, P);
    MARK();
    if (!fused && lo.plan.nTB > 1)
        HIP_TRY(launch_clear(hdr, ws + lo.ticket, lo.desc + up(lo.plan.desc_bytes) - lo.ticket, s));
    PrepArgs pa{};
    pa.Lambda = reinterpret_cast<const float2 *>(Lambda); pa.B = reinterpret_cast<const float2 *>(B);
    pa.C = reinterpret_cast<const float2 *>(C); pa.log_delta = log_delta;
    pa.P = (int)P; pa.H = (int)H; pa.lam_bar = lam; pa.Bbar_ri = Bri; pa.Cc = Cc; pa.Bbar_c64 = nullptr;
    pa.hdr = (fused || lo.plan.nTB == 1) ? hdr : nullptr;
    // the atomic slots and the tagged words behind them are cleared in the same launch
    if (fused) { pa.zero16 = reinterpret_cast<uint4 *>(ws + lo.amax_atomic); pa.n16 = (2 * ABSMAX_SLOTS * 4 + lo.fdesc_bytes) / 16; }
    if (lo.planes2_unfused) { pa.zero16 = reinterpret_cast<uint4 *>(ws + lo.amax_atomic); pa.n16 = (2 * ABSMAX_SLOTS * 4 + up((size_t)T * 4)) / 16; }
    // two scaled fp16 planes per operand: every operand of the two products brings its largest magnitude
    const bool two_planes = fused || lo.planes2_unfused;
    unsigned *am_bbar = reinterpret_cast<unsigned *>(ws + lo.amax_slots), *am_cc = am_bbar + P;
    unsigned *rowmax = reinterpret_cast<unsigned *>(ws + lo.rowmax), *rowpart = reinterpret_cast<unsigned *>(ws + lo.rowpart);
    if (two_planes) {
        // u and x enter their products with tokens as rows: every token gets its own scale
        pa.bbar_max = am_bbar; pa.cc_max = am_cc;
        pa.pass[0].x = u; pa.pass[0].n = (size_t)T * H; pa.pass[0].slots = rowmax; pa.pass[0].rowlen = (int)H;
        pa.pass[0].nblocks = row_pass_blocks((size_t)T);
    }
    if (gate_max) {
        pa.pass[1].x = gate_max->W; pa.pass[1].n = gate_max->nW; pa.pass[1].slots = gate_max->wslots;
        pa.pass[1].nblocks = gate_max->nwslots; pa.pass[1].rowlen = 0;
    }
    HIP_TRY(launch_prep(pa, s));
    MARK();

    // v[t, 2p+c] = sum_h u[t,h] * Bbar_ri[2p+c, h]      (second scan-element component, Eq. 6)
    GemmArgs g1{};
    g1.A = u; g1.lda = H; g1.a_kcontig = 1;
    g1.B = Bri; g1.ldb = H; g1.b_kcontig = 1;
    g1.C = reinterpret_cast<float *>(xs); g1.ldc = 2 * P;
    g1.M = T; g1.N = (int)(2 * P); g1.K = (int)H; g1.splits = 1;
    if (fused) {
        g1.epilogue = 7;
        g1.scan.lam = lam; g1.scan.is_first = is_first;
        g1.scan.x0 = reinterpret_cast<const float2 *>(x0); g1.scan.x_last = reinterpret_cast<float2 *>(x_last);
        g1.scan.desc = reinterpret_cast<unsigned long long *>(ws + lo.fdesc); g1.scan.err = &hdr->err;
        g1.scan.L = (int)L; g1.scan.P = (int)P; g1.scan.spin_limit = spin_limit();
        if (two_planes) {
            g1.amaxA = AbsMax{nullptr, 0, rowmax, 1, T}; g1.amaxB = AbsMax{am_bbar, (int)P, nullptr, 0, 0};
            g1.scan.rowmax_out = rowpart;                    // of the states, for the output projection
        }
    } else if (two_planes) {
        g1.amaxA = AbsMax{nullptr, 0, rowmax, 1, T}; g1.amaxB = AbsMax{am_bbar, (int)P, nullptr, 0, 0};
    }
    HIP_TRY(launch_gemm(g1, s));
    MARK();

    if (!fused) {
        ScanArgs sa{};
        sa.in = xs; sa.out = xs; sa.lam = lam; sa.is_first = is_first;
        sa.x0 = reinterpret_cast<const float2 *>(x0); sa.x_last = reinterpret_cast<float2 *>(x_last);
        sa.desc = desc; sa.ticket = reinterpret_cast<uint32_t *>(ws + lo.ticket); sa.err = &hdr->err;
        sa.Bt = (int)Bt; sa.L = (int)L; sa.P = (int)P;
        sa.pxb = lo.plan.pxb; sa.cy = lo.plan.cy; sa.nPX = lo.plan.nPX; sa.nTB = lo.plan.nTB;
        sa.spin_limit = spin_limit();
        if (two_planes) {                                    // rows of the states, for the output projection
            sa.rowmax_out = rowpart;
            sa.amax_out = reinterpret_cast<unsigned *>(ws + lo.amax_atomic) + ABSMAX_SLOTS;
        }
        HIP_TRY(launch_scan(sa, false, s));
    }
    MARK();

    // y[t,h] = sum_p (Re C[h,p] x_re - Im C[h,p] x_im) + D[h] u[t,h]       (Eq. 3, second line)
    GemmArgs g2{};
    g2.A = reinterpret_cast<const float *>(xs); g2.lda = 2 * P; g2.a_kcontig = 1;
    g2.B = Cc; g2.ldb = 2 * P; g2.b_kcontig = 1;
    g2.M = T; g2.N = (int)H; g2.K = (int)(2 * P);
    if (two_planes) { g2.amaxA = AbsMax{nullptr, 0, rowpart, lo.row_parts, T}; g2.amaxB = AbsMax{am_cc, (int)H, nullptr, 0, 0}; }
    g2.C = y; g2.ldc = H; g2.diag = D; g2.E = u; g2.lde = H; g2.epilogue = 1;
    if (gelu_y) { g2.epilogue = 6; g2.C2 = gelu_y; }       // the S5 block: GELU(y) for the gate, same store
    if (gelu_y && gate_max) g2.c2_rowmax = gate_max->x1_rowmax;
    g2.splits = 1;
    HIP_TRY(launch_gemm(g2, s));
    MARK();
    return SSM_OK;
}

ssm_status run_bwd(const ssm_c64 *Lambda, const ssm_c64 *B, const ssm_c64 *C, const float *D,
                   const float *log_delta, const float *u, const uint8_t *is_first, const ssm_c64 *x0,
                   int64_t Bt, int64_t L, int64_t H, int64_t P, const ssm_c64 *x, const float *dy,
                   float *du, ssm_c64 *dLambda, ssm_c64 *dB, ssm_c64 *dC, float *dD, float *dlog_delta,
                   ssm_c64 *dx0, void *workspace, size_t ws_bytes, hipStream_t s, StageTimer *timer)
{
    if (!Lambda || !B || !C || !D || !log_delta || !u || !x || !dy || !du || !dLambda || !dB || !dC ||
        !dD || !dlog_delta)
        return SSM_ERR_INVALID_ARG;
    Layout lo;
    ssm_status st = make_layout(Bt, L, H, P, true, lo);
    if (st != SSM_OK) return st;
    if (misaligned(Lambda, 8) || misaligned(B, 8) || misaligned(C, 8) || misaligned(D, 4) ||
        misaligned(log_delta, 4) || misaligned(u, 4) || misaligned(x, 8) || misaligned(dy, 4) ||
        misaligned(du, 4) || misaligned(dLambda, 8) || misaligned(dB, 8) || misaligned(dC, 8) ||
        misaligned(dD, 4) || misaligned(dlog_delta, 4) || misaligned(dx0, 8) || misaligned(x0, 8))
        return SSM_ERR_INVALID_ARG;
    if (!workspace || misaligned(workspace, ALIGN) || ws_bytes < lo.total) return SSM_ERR_WORKSPACE;

    char *ws = static_cast<char *>(workspace);
    WsHeader *hdr = reinterpret_cast<WsHeader *>(ws + lo.hdr);
    float2 *lam = reinterpret_cast<float2 *>(ws + lo.lam);
    float *Bri = reinterpret_cast<float *>(ws + lo.Bri);
    float *Cc = reinterpret_cast<float *>(ws + lo.Cc);
    ScanDesc *desc = reinterpret_cast<ScanDesc *>(ws + lo.desc);
    float2 *chi = reinterpret_cast<float2 *>(ws + lo.chi);
    float *dCpart = reinterpret_cast<float *>(ws + lo.dCpart);
    float *dBpart = reinterpret_cast<float *>(ws + lo.dBpart);
    float2 *dApart = reinterpret_cast<float2 *>(ws + lo.dApart);
    float *dDpart = reinterpret_cast<float *>(ws + lo.dDpart);
    const int T = (int)(Bt * L);
    const float *xf = reinterpret_cast<const float *>(x);

    // Shapes whose sequences are whole numbers of 128-row tiles: C^H dy runs the reverse scan on its
    // own output tile (chi stored directly, dAbar rows per tile, no scan kernel).
    const bool fused = gemm_scan_shape_ok(Bt, L, P);
    MARK();
    if (!fused && lo.plan.nTB > 1)
        HIP_TRY(launch_clear(hdr, ws + lo.ticket, lo.desc + up(lo.plan.desc_bytes) - lo.ticket, s));
    PrepArgs pa{};
    pa.Lambda = reinterpret_cast<const float2 *>(Lambda); pa.B = reinterpret_cast<const float2 *>(B);
    pa.C = reinterpret_cast<const float2 *>(C); pa.log_delta = log_delta;
    pa.P = (int)P; pa.H = (int)H; pa.lam_bar = lam; pa.Bbar_ri = Bri; pa.Cc = Cc; pa.Bbar_c64 = nullptr;
    pa.hdr = (fused || lo.plan.nTB == 1) ? hdr : nullptr;
    if (fused) { pa.zero16 = reinterpret_cast<uint4 *>(ws + lo.amax_atomic); pa.n16 = (2 * ABSMAX_SLOTS * 4 + lo.fdesc_bytes) / 16; }
    if (lo.planes2_unfused) { pa.zero16 = reinterpret_cast<uint4 *>(ws + lo.amax_atomic); pa.n16 = (2 * ABSMAX_SLOTS * 4 + up((size_t)T * 4)) / 16; }
    // dD slabs: sum_t dy[t,h] u[t,h] over row slabs, in the same launch
    pa.cd.a = dy; pa.cd.b = u; pa.cd.T = T; pa.cd.H = (int)H; pa.cd.nslab = lo.nslab; pa.cd.partial = dDpart;
    // two scaled fp16 planes per operand: dy and u are measured where dD reads them, chi and the saved
    // states where the reverse scan stores / reads them
    const bool two_planes = fused || lo.planes2_unfused;
    const bool x_pass = lo.dc_early || lo.planes2_unfused;       // the largest magnitude of the saved states from a pass of the prep launch
    unsigned *am_atomic = reinterpret_cast<unsigned *>(ws + lo.amax_atomic), *am_xsaved = am_atomic + ABSMAX_SLOTS;
    unsigned *am_bbar = reinterpret_cast<unsigned *>(ws + lo.amax_slots), *am_cc = am_bbar + P, *am_pass = am_cc + H;
    unsigned *am_dy = am_pass + 2 * PREP_PASS_BLOCKS, *am_u = am_dy + lo.amax_cd;
    unsigned *rowmax = reinterpret_cast<unsigned *>(ws + lo.rowmax), *rowpart = reinterpret_cast<unsigned *>(ws + lo.rowpart);
    const int x_pieces = pass_pieces((size_t)T * 2 * P);
    if (two_planes) {
        pa.bbar_max = am_bbar; pa.cc_max = am_cc; pa.cd_amax = am_dy; pa.cd_bmax = am_u;
        pa.cd_arow = rowmax;                 // [ceil(H/64)][T]: rows of dy, measured where the dD column dots read it
        if (x_pass) { pa.pass[0].x = xf; pa.pass[0].n = (size_t)T * 2 * P; pa.pass[0].slots = am_pass; pa.pass[0].nblocks = x_pieces; }
    }
    // dy and chi enter C^H dy and Bbar^H chi with tokens as rows (a scale per token); the sums over tokens
    // (dC, dBbar) take one scale per matrix
    const AbsMax mx_dy{am_dy, lo.amax_cd, nullptr, 0, 0}, mx_u{am_u, lo.amax_cd, nullptr, 0, 0},
                 mx_x{x_pass ? am_pass : am_xsaved, x_pass ? x_pieces : ABSMAX_SLOTS, nullptr, 0, 0},
                 mx_chi{am_atomic, ABSMAX_SLOTS, nullptr, 0, 0},
                 mx_bbar{am_bbar, (int)P, nullptr, 0, 0}, mx_cc{am_cc, (int)H, nullptr, 0, 0},
                 mx_dy_rows{nullptr, 0, rowmax, (int)((H + 63) / 64), T}, mx_chi_rows{nullptr, 0, rowpart, lo.row_parts, T};
    HIP_TRY(launch_prep(pa, s));
    MARK();

    // gx[t, 2p+c] = sum_h dy[t,h] * Cc[h, 2p+c]           (C^H dy_t)
    GemmArgs g3{};
    g3.A = dy; g3.lda = H; g3.a_kcontig = 1;
    g3.B = Cc; g3.ldb = 2 * P; g3.b_kcontig = 0;
    g3.C = reinterpret_cast<float *>(chi); g3.ldc = 2 * P;
    g3.M = T; g3.N = (int)(2 * P); g3.K = (int)H; g3.splits = 1;
    // dC slabs: [h, 2p+c] = sum_t dy[t,h] * x[t, 2p+c]
    GemmArgs g4{};
    g4.A = dy; g4.lda = H; g4.a_kcontig = 0;
    g4.B = xf; g4.ldb = 2 * P; g4.b_kcontig = 0;
    g4.C = dCpart; g4.ldc = 2 * P;
    g4.M = (int)H; g4.N = (int)(2 * P); g4.K = T; g4.splits = lo.splitC;
    if (fused) {
        // the product scans its own tiles; the dC slabs wait for the next launch, where the largest
        // magnitude of the saved states (recorded here, as the scan reads them) is known
        g3.epilogue = 8;
        g3.scan.lam = lam; g3.scan.is_first = is_first;
        g3.scan.x0 = reinterpret_cast<const float2 *>(x0);
        g3.scan.xsaved = reinterpret_cast<const float2 *>(x); g3.scan.partial = dApart;
        g3.scan.dx0 = reinterpret_cast<float2 *>(dx0);
        g3.scan.desc = reinterpret_cast<unsigned long long *>(ws + lo.fdesc); g3.scan.err = &hdr->err;
        g3.scan.L = (int)L; g3.scan.P = (int)P; g3.scan.spin_limit = spin_limit();
        g3.amaxA = mx_dy_rows; g3.amaxB = mx_cc;
        g3.scan.amax_out = am_atomic; g3.scan.xmax_out = lo.dc_early ? nullptr : am_xsaved; g3.scan.rowmax_out = rowpart;
        if (lo.dc_early) { g4.amaxA = mx_dy; g4.amaxB = mx_x; HIP_TRY(launch_gemm_pair(g3, g4, s)); }
        else HIP_TRY(launch_gemm(g3, s));
    } else {
        // dC needs only dy and the saved states: it shares the launch (whichever kind of work item the schedule model puts first)
        if (two_planes) { g3.amaxA = mx_dy_rows; g3.amaxB = mx_cc; g4.amaxA = mx_dy; g4.amaxB = mx_x; }
        HIP_TRY(launch_gemm_pair(g3, g4, s, lo.dc_first));
    }
    MARK();

    if (!fused) {
        ScanArgs sa{};
        sa.in = chi; sa.out = chi; sa.lam = lam; sa.is_first = is_first;
        sa.x0 = reinterpret_cast<const float2 *>(x0);
        sa.xsaved = reinterpret_cast<const float2 *>(x); sa.partial = dApart;
        sa.dx0 = reinterpret_cast<float2 *>(dx0);
        sa.desc = desc; sa.ticket = reinterpret_cast<uint32_t *>(ws + lo.ticket); sa.err = &hdr->err;
        sa.Bt = (int)Bt; sa.L = (int)L; sa.P = (int)P;
        sa.pxb = lo.plan.pxb; sa.cy = lo.plan.cy; sa.nPX = lo.plan.nPX; sa.nTB = lo.plan.nTB;
        sa.spin_limit = spin_limit();
        if (two_planes) { sa.rowmax_out = rowpart; sa.amax_out = am_atomic; }      // rows of chi for du, all of chi for dBbar
        HIP_TRY(launch_scan(sa, true, s));
    }
    MARK();

    // du[t,h] = sum_{p,c} chi[t, 2p+c] * Bbar_ri[2p+c, h] + D[h] dy[t,h]      (Re(Bbar^H chi) + D dy)
    const float *du_halves = nullptr;
    GemmArgs g5{};
    g5.A = reinterpret_cast<const float *>(chi); g5.lda = 2 * P; g5.a_kcontig = 1;
    g5.B = Bri; g5.ldb = H; g5.b_kcontig = 0;
    g5.M = T; g5.N = (int)H; g5.K = (int)(2 * P);
    // dBbar slabs: [2p+c, h] = sum_t chi[t, 2p+c] * u[t,h]   (same launch)
    GemmArgs g6{};
    g6.A = reinterpret_cast<const float *>(chi); g6.lda = 2 * P; g6.a_kcontig = 0;
    g6.B = u; g6.ldb = H; g6.b_kcontig = 0;
    g6.C = dBpart; g6.ldc = H;
    g6.M = (int)(2 * P); g6.N = (int)H; g6.K = T; g6.splits = lo.splitB;
    if (two_planes) { g4.amaxA = mx_dy; g4.amaxB = mx_x; g5.amaxA = mx_chi_rows; g5.amaxB = mx_bbar; g6.amaxA = mx_chi; g6.amaxB = mx_u; }
    if (lo.yhalves) {
        // du has too few 128x128 tiles for half a chip's worth of time: it runs as two K halves (twice
        // the workgroups, half as long); a streaming pass adds the halves and D dy
        float *halves = reinterpret_cast<float *>(ws + lo.yhalves);
        g5.C = halves; g5.ldc = H; g5.splits = 2;
        du_halves = halves;                  // added by extra workgroups of the parameter epilogue's launch
    } else {
        g5.C = du; g5.ldc = H; g5.diag = D; g5.E = dy; g5.lde = H; g5.epilogue = 1; g5.splits = 1;
    }
    if (fused && !lo.dc_early) HIP_TRY(launch_gemm_triple(g5, g6, g4, s, lo.slabs_first));   // three products, two workgroups per CU
    else {
        // (the slabs first when du runs as two K halves, or where the schedule model says so)
        HIP_TRY(launch_gemm_pair(g5, g6, s, lo.yhalves != 0 || (!fused && lo.db_first)));
    }
    MARK();
    MARK();

    EpilogueArgs ea{};
    if (du_halves) {
        ea.sum.s0 = du_halves; ea.sum.s1 = du_halves + (size_t)T * H; ea.sum.D = D; ea.sum.e = dy; ea.sum.out = du;
        ea.sum.n = (long)T * H; ea.sum.H = (int)H;
    }
    ea.Lambda = reinterpret_cast<const float2 *>(Lambda); ea.B = reinterpret_cast<const float2 *>(B);
    ea.log_delta = log_delta; ea.P = (int)P; ea.H = (int)H;
    ea.dBbar_part = dBpart; ea.nsplit_B = lo.splitB;
    ea.dC_part = dCpart; ea.nsplit_C = lo.splitC;
    ea.dAbar_part = dApart; ea.npart = fused ? Bt * L / 128 : (int64_t)Bt * lo.plan.nTB;
    ea.dD_part = dDpart; ea.nslab = lo.nslab;
    ea.dLambda = reinterpret_cast<float2 *>(dLambda); ea.dB = reinterpret_cast<float2 *>(dB);
    ea.dC = reinterpret_cast<float2 *>(dC); ea.dD = dD; ea.dlog_delta = dlog_delta;
    HIP_TRY(launch_epilogue(ea, s));
    MARK();
    return SSM_OK;
}

}  // namespace

extern "C" {

const char *ssm_strerror(int status)
{
    switch (status) {
    case SSM_OK: return "ok";
    case SSM_ERR_INVALID_ARG: return "invalid argument (null required pointer, non-positive dimension or misaligned array)";
    case SSM_ERR_WORKSPACE: return "workspace missing, misaligned or smaller than ssm_workspace_bytes()";
    case SSM_ERR_UNSUPPORTED: return "dimension beyond the supported limits";
    case SSM_ERR_HIP: return "HIP runtime call or kernel launch failed";
    case SSM_ERR_SCAN_TIMEOUT: return "a bounded cross-workgroup wait in the scan gave up; outputs invalid";
    case SSM_ERR_SCRATCH_LIMIT: return "shape needs more than the built-in scratch of the no-allocation entry point";
    default: return "unknown status";
    }
}

int ssm_version(void) { return 200; }

uint32_t ssm_set_spin_limit(uint32_t polls)
{
    return scan_set_spin_limit(polls);
}

size_t ssm_workspace_bytes(int64_t Bt, int64_t L, int64_t H, int64_t P, int want_bwd)
{
    Layout lo;
    if (make_layout(Bt, L, H, P, want_bwd != 0, lo) != SSM_OK) return 0;
    return lo.total;
}

ssm_status ssm_discretize(const ssm_c64 *Lambda, const ssm_c64 *B, const float *log_delta,
                          int64_t P, int64_t H, ssm_c64 *A_bar, ssm_c64 *B_bar, void *stream)
{
    if (!Lambda || !log_delta || !A_bar || (B_bar && !B)) return SSM_ERR_INVALID_ARG;
    if (P <= 0 || H <= 0) return SSM_ERR_INVALID_ARG;
    if (P > SSM_MAX_WIDTH || H > SSM_MAX_WIDTH) return SSM_ERR_UNSUPPORTED;
    if (misaligned(Lambda, 8) || misaligned(B, 8) || misaligned(log_delta, 4) || misaligned(A_bar, 8) ||
        misaligned(B_bar, 8))
        return SSM_ERR_INVALID_ARG;
    PrepArgs pa{};
    pa.Lambda = reinterpret_cast<const float2 *>(Lambda);
    pa.B = B_bar ? reinterpret_cast<const float2 *>(B) : nullptr;
    pa.log_delta = log_delta; pa.P = (int)P; pa.H = (int)H;
    pa.lam_bar = reinterpret_cast<float2 *>(A_bar);
    pa.Bbar_c64 = reinterpret_cast<float2 *>(B_bar);
    HIP_TRY(launch_prep(pa, static_cast<hipStream_t>(stream)));
    return SSM_OK;
}

ssm_status ssm_scan_fwd(const ssm_c64 *Lambda, const ssm_c64 *B, const ssm_c64 *C, const float *D,
                        const float *log_delta, const float *u, const uint8_t *is_first,
                        const ssm_c64 *x0, int64_t Bt, int64_t L, int64_t H, int64_t P,
                        float *y, ssm_c64 *x, ssm_c64 *x_last, void *workspace, size_t ws_bytes, void *stream)
{
    return run_fwd(Lambda, B, C, D, log_delta, u, is_first, x0, Bt, L, H, P, y, x, x_last, workspace,
                   ws_bytes, static_cast<hipStream_t>(stream), nullptr);
}

ssm_status ssm_scan_bwd(const ssm_c64 *Lambda, const ssm_c64 *B, const ssm_c64 *C, const float *D,
                        const float *log_delta, const float *u, const uint8_t *is_first,
                        const ssm_c64 *x0, int64_t Bt, int64_t L, int64_t H, int64_t P,
                        const ssm_c64 *x, const float *dy, float *du, ssm_c64 *dLambda, ssm_c64 *dB,
                        ssm_c64 *dC, float *dD, float *dlog_delta, ssm_c64 *dx0,
                        void *workspace, size_t ws_bytes, void *stream)
{
    return run_bwd(Lambda, B, C, D, log_delta, u, is_first, x0, Bt, L, H, P, x, dy, du, dLambda, dB, dC,
                   dD, dlog_delta, dx0, workspace, ws_bytes, static_cast<hipStream_t>(stream), nullptr);
}

ssm_status ssm_scan_fwd_profiled(const ssm_c64 *Lambda, const ssm_c64 *B, const ssm_c64 *C,
                                 const float *D, const float *log_delta, const float *u,
                                 const uint8_t *is_first, const ssm_c64 *x0,
                                 int64_t Bt, int64_t L, int64_t H, int64_t P,
                                 float *y, ssm_c64 *x, ssm_c64 *x_last,
                                 void *workspace, size_t ws_bytes, void *stream, float *stage_ms)
{
    if (!stage_ms) return SSM_ERR_INVALID_ARG;
    StageTimer timer(static_cast<hipStream_t>(stream));
    ssm_status st = run_fwd(Lambda, B, C, D, log_delta, u, is_first, x0, Bt, L, H, P, y, x, x_last,
                            workspace, ws_bytes, static_cast<hipStream_t>(stream), &timer);
    const bool ok = timer.finish(stage_ms, SSM_FWD_STAGES);
    if (st != SSM_OK) return st;
    return ok ? SSM_OK : SSM_ERR_HIP;
}

ssm_status ssm_scan_bwd_profiled(const ssm_c64 *Lambda, const ssm_c64 *B, const ssm_c64 *C,
                                 const float *D, const float *log_delta, const float *u,
                                 const uint8_t *is_first, const ssm_c64 *x0,
                                 int64_t Bt, int64_t L, int64_t H, int64_t P,
                                 const ssm_c64 *x, const float *dy,
                                 float *du, ssm_c64 *dLambda, ssm_c64 *dB, ssm_c64 *dC, float *dD,
                                 float *dlog_delta, ssm_c64 *dx0,
                                 void *workspace, size_t ws_bytes, void *stream, float *stage_ms)
{
    if (!stage_ms) return SSM_ERR_INVALID_ARG;
    StageTimer timer(static_cast<hipStream_t>(stream));
    ssm_status st = run_bwd(Lambda, B, C, D, log_delta, u, is_first, x0, Bt, L, H, P, x, dy, du, dLambda,
                            dB, dC, dD, dlog_delta, dx0, workspace, ws_bytes,
                            static_cast<hipStream_t>(stream), &timer);
    const bool ok = timer.finish(stage_ms, SSM_BWD_STAGES);
    if (st != SSM_OK) return st;
    return ok ? SSM_OK : SSM_ERR_HIP;
}

ssm_status ssm_plan_describe(int64_t Bt, int64_t L, int64_t H, int64_t P, int32_t *out)
{
    if (!out) return SSM_ERR_INVALID_ARG;
    Layout lo;
    ssm_status st = make_layout(Bt, L, H, P, true, lo);
    if (st != SSM_OK) return st;
    const bool fused = gemm_scan_shape_ok(Bt, L, P);
    const int64_t T = Bt * L;
    out[0] = fused ? 1 : 0;
    out[1] = (fused || lo.planes2_unfused) ? 2 : 3;
    out[2] = lo.splitC; out[3] = lo.splitB;
    out[4] = (fused && !lo.dc_early) ? 3 : 2;
    out[5] = lo.slabs_first ? 1 : 0;
    out[6] = (!fused && lo.dc_first) ? 1 : 0;
    out[7] = (lo.yhalves != 0 || (!fused && lo.db_first)) ? 1 : 0;
    out[8] = lo.yhalves != 0 ? 1 : 0;
    out[9] = fused ? 0 : gemm_tile_tier(T, 2 * P, 1);
    out[10] = gemm_tile_tier(T, H, 1);
    out[11] = lo.plan.nTB;
    return SSM_OK;
}

ssm_status ssm_scan_states(const ssm_c64 *A_bar, ssm_c64 *v, const uint8_t *is_first,
                           const ssm_c64 *x0, int64_t Bt, int64_t L, int64_t P, ssm_c64 *x_last,
                           void *workspace, size_t ws_bytes, void *stream)
{
    return (ssm_status)scan_states_forward(A_bar, v, is_first, x0, Bt, L, P, x_last, workspace, ws_bytes,
                                           static_cast<hipStream_t>(stream));
}

ssm_status ssm_scan_states_reverse(const ssm_c64 *A_bar, ssm_c64 *gx, const ssm_c64 *x,
                                   const uint8_t *is_first, const ssm_c64 *x0,
                                   int64_t Bt, int64_t L, int64_t P, ssm_c64 *dA_bar, ssm_c64 *dx0,
                                   void *workspace, size_t ws_bytes, void *stream)
{
    if (!A_bar || !gx || !x || !dA_bar) return SSM_ERR_INVALID_ARG;
    ScanOnlyLayout lo;
    ssm_status st = (ssm_status)make_scan_layout(Bt, L, P, true, lo);
    if (st != SSM_OK) return st;
    if (misaligned(A_bar, 8) || misaligned(gx, 8) || misaligned(x, 8) || misaligned(x0, 8) ||
        misaligned(dA_bar, 8) || misaligned(dx0, 8))
        return SSM_ERR_INVALID_ARG;
    if (!workspace || misaligned(workspace, ALIGN) || ws_bytes < lo.total) return SSM_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    WsHeader *hdr = reinterpret_cast<WsHeader *>(ws + lo.hdr);
    ScanDesc *desc = reinterpret_cast<ScanDesc *>(ws + lo.desc);
    float2 *dApart = reinterpret_cast<float2 *>(ws + lo.dApart);
    if (lo.plan.nTB > 1)
        HIP_TRY(launch_clear(hdr, ws + lo.ticket, lo.desc + up(lo.plan.desc_bytes) - lo.ticket, s));
    ScanArgs sa{};
    sa.in = reinterpret_cast<const float2 *>(gx); sa.out = reinterpret_cast<float2 *>(gx);
    sa.lam = reinterpret_cast<const float2 *>(A_bar); sa.is_first = is_first;
    sa.x0 = reinterpret_cast<const float2 *>(x0);
    sa.xsaved = reinterpret_cast<const float2 *>(x); sa.partial = dApart;
    sa.dx0 = reinterpret_cast<float2 *>(dx0);
    sa.desc = desc; sa.ticket = reinterpret_cast<uint32_t *>(ws + lo.ticket); sa.err = &hdr->err;
    sa.Bt = (int)Bt; sa.L = (int)L; sa.P = (int)P;
    sa.pxb = lo.plan.pxb; sa.cy = lo.plan.cy; sa.nPX = lo.plan.nPX; sa.nTB = lo.plan.nTB;
    sa.spin_limit = spin_limit();
    HIP_TRY(launch_scan(sa, true, s));
    HIP_TRY(launch_reduce_partials(dApart, (int64_t)Bt * lo.plan.nTB, P,
                                   reinterpret_cast<float2 *>(dA_bar), s));
    return SSM_OK;
}

namespace {
struct StepPlan { size_t lam, Bri, Cc, total; };
bool make_step_plan(int64_t H, int64_t P, StepPlan &o)
{
    if (H <= 0 || P <= 0 || H > SSM_MAX_WIDTH || P > SSM_MAX_WIDTH) return false;
    size_t off = 0;
    o.lam = off; off += up((size_t)P * 8);
    o.Bri = off; off += up((size_t)2 * P * H * 4);
    o.Cc = off; off += up((size_t)2 * P * H * 4);
    o.total = off;
    return true;
}
}  // namespace

size_t ssm_step_plan_bytes(int64_t H, int64_t P)
{
    StepPlan pl;
    return make_step_plan(H, P, pl) ? pl.total : 0;
}

ssm_status ssm_step_prepare(const ssm_c64 *Lambda, const ssm_c64 *B, const ssm_c64 *C,
                            const float *log_delta, int64_t H, int64_t P,
                            void *plan, size_t plan_bytes, void *stream)
{
    if (!Lambda || !B || !C || !log_delta) return SSM_ERR_INVALID_ARG;
    if (H <= 0 || P <= 0) return SSM_ERR_INVALID_ARG;
    StepPlan pl;
    if (!make_step_plan(H, P, pl)) return SSM_ERR_UNSUPPORTED;
    if (misaligned(Lambda, 8) || misaligned(B, 8) || misaligned(C, 8) || misaligned(log_delta, 4))
        return SSM_ERR_INVALID_ARG;
    if (!plan || misaligned(plan, ALIGN) || plan_bytes < pl.total) return SSM_ERR_WORKSPACE;
    char *pb = static_cast<char *>(plan);
    PrepArgs pa{};
    pa.Lambda = reinterpret_cast<const float2 *>(Lambda); pa.B = reinterpret_cast<const float2 *>(B);
    pa.C = reinterpret_cast<const float2 *>(C); pa.log_delta = log_delta;
    pa.P = (int)P; pa.H = (int)H;
    pa.lam_bar = reinterpret_cast<float2 *>(pb + pl.lam);
    pa.Bbar_ri = reinterpret_cast<float *>(pb + pl.Bri);
    pa.Cc = reinterpret_cast<float *>(pb + pl.Cc);
    HIP_TRY(launch_prep(pa, static_cast<hipStream_t>(stream)));
    return SSM_OK;
}

ssm_status ssm_step(const void *plan, size_t plan_bytes, const float *D, const float *u,
                    const ssm_c64 *x_prev, const uint8_t *is_first, int64_t Bt, int64_t H, int64_t P,
                    ssm_c64 *x, float *y, void *stream)
{
    if (!D || !u || !x || !y) return SSM_ERR_INVALID_ARG;
    ssm_status st = check_dims(Bt, 1, H, P);
    if (st != SSM_OK) return st;
    StepPlan pl;
    if (!make_step_plan(H, P, pl)) return SSM_ERR_UNSUPPORTED;
    if (misaligned(D, 4) || misaligned(u, 4) || misaligned(x_prev, 8) || misaligned(x, 8) || misaligned(y, 4) ||
        (x_prev && x_prev == x))
        return SSM_ERR_INVALID_ARG;
    if (!plan || misaligned(plan, ALIGN) || plan_bytes < pl.total) return SSM_ERR_WORKSPACE;
    const char *pb = static_cast<const char *>(plan);
    hipStream_t s = static_cast<hipStream_t>(stream);
    // x = Bbar u (+ Abar (.) x_prev where the sequence continues)          (Eq. 3, first line)
    GemmArgs g1{};
    g1.A = u; g1.lda = H; g1.a_kcontig = 1;
    g1.B = reinterpret_cast<const float *>(pb + pl.Bri); g1.ldb = H; g1.b_kcontig = 1;
    g1.C = reinterpret_cast<float *>(x); g1.ldc = 2 * P;
    g1.M = (int)Bt; g1.N = (int)(2 * P); g1.K = (int)H; g1.splits = 1;
    if (x_prev) {
        g1.epilogue = 2;
        g1.diag = reinterpret_cast<const float *>(pb + pl.lam);
        g1.E = reinterpret_cast<const float *>(x_prev); g1.lde = 2 * P;
        g1.rowflag = is_first;
    }
    HIP_TRY(launch_gemm(g1, s));
    // y = Re(C x) + D (.) u                                                 (Eq. 3, second line)
    GemmArgs g2{};
    g2.A = reinterpret_cast<const float *>(x); g2.lda = 2 * P; g2.a_kcontig = 1;
    g2.B = reinterpret_cast<const float *>(pb + pl.Cc); g2.ldb = 2 * P; g2.b_kcontig = 1;
    g2.C = y; g2.ldc = H; g2.diag = D; g2.E = u; g2.lde = H; g2.epilogue = 1;
    g2.M = (int)Bt; g2.N = (int)H; g2.K = (int)(2 * P); g2.splits = 1;
    HIP_TRY(launch_gemm(g2, s));
    return SSM_OK;
}

ssm_status ssm_step_bwd(const void *plan, size_t plan_bytes, const float *D, const float *dy,
                        const ssm_c64 *dx, const uint8_t *is_first, int64_t Bt, int64_t H, int64_t P,
                        ssm_c64 *gx, float *du, ssm_c64 *dx_prev, void *stream)
{
    if (!D || !dy || !gx || !du) return SSM_ERR_INVALID_ARG;
    ssm_status st = check_dims(Bt, 1, H, P);
    if (st != SSM_OK) return st;
    StepPlan pl;
    if (!make_step_plan(H, P, pl)) return SSM_ERR_UNSUPPORTED;
    if (misaligned(D, 4) || misaligned(dy, 4) || misaligned(dx, 8) || misaligned(gx, 8) || misaligned(du, 4) ||
        misaligned(dx_prev, 8) || (dx && (dx == gx || dx == dx_prev)) || (dx_prev && dx_prev == gx))
        return SSM_ERR_INVALID_ARG;
    if (!plan || misaligned(plan, ALIGN) || plan_bytes < pl.total) return SSM_ERR_WORKSPACE;
    const char *pb = static_cast<const char *>(plan);
    hipStream_t s = static_cast<hipStream_t>(stream);
    // gx = C^H dy + dx;  dx_prev = [not is_first] conj(Abar) (.) gx
    GemmArgs g1{};
    g1.A = dy; g1.lda = H; g1.a_kcontig = 1;
    g1.B = reinterpret_cast<const float *>(pb + pl.Cc); g1.ldb = 2 * P; g1.b_kcontig = 0;
    g1.C = reinterpret_cast<float *>(gx); g1.ldc = 2 * P;
    g1.E = reinterpret_cast<const float *>(dx); g1.lde = 2 * P;
    g1.C2 = reinterpret_cast<float *>(dx_prev);
    g1.diag = reinterpret_cast<const float *>(pb + pl.lam); g1.rowflag = is_first; g1.epilogue = 5;
    g1.M = (int)Bt; g1.N = (int)(2 * P); g1.K = (int)H; g1.splits = 1;
    HIP_TRY(launch_gemm(g1, s));
    // du = Re(Bbar^H gx) + D (.) dy
    GemmArgs g2{};
    g2.A = reinterpret_cast<const float *>(gx); g2.lda = 2 * P; g2.a_kcontig = 1;
    g2.B = reinterpret_cast<const float *>(pb + pl.Bri); g2.ldb = H; g2.b_kcontig = 0;
    g2.C = du; g2.ldc = H; g2.diag = D; g2.E = dy; g2.lde = H; g2.epilogue = 1;
    g2.M = (int)Bt; g2.N = (int)H; g2.K = (int)(2 * P); g2.splits = 1;
    HIP_TRY(launch_gemm(g2, s));
    return SSM_OK;
}

namespace {
struct BlockLayout {
    size_t ssm, x1, glu, dypre, total;
    // forward: the gate's product on two scaled fp16 planes (width a multiple of 64 and an output projection
    // whose wavefronts own 64 columns): rows of GELU(y) in pieces of 64 columns, pieces of W
    bool gate_two_planes; size_t x1_rowmax, wslots; int nwslots;
};
bool make_block_layout(int64_t Bt, int64_t L, int64_t H, int64_t P, bool bwd, BlockLayout &o)
{
    Layout lo;
    if (make_layout(Bt, L, H, P, bwd, lo) != SSM_OK) return false;
    const size_t TH = up((size_t)Bt * L * H * 4);
    size_t off = 0;
    o.ssm = off; off += up(lo.total);
    o.x1 = o.glu = o.dypre = 0;
    o.gate_two_planes = false; o.x1_rowmax = o.wslots = 0; o.nwslots = 0;
    if (!bwd) {
        o.x1 = off; off += TH;
        o.gate_two_planes = gate_two_planes_shape(Bt * L, H) && gemm_tile_tier(Bt * L, H, 1) <= 1;
        if (o.gate_two_planes) {
            o.nwslots = pass_pieces((size_t)H * H);
            o.x1_rowmax = off; off += up((size_t)(H / 64) * Bt * L * 4);
            o.wslots = off; off += up((size_t)o.nwslots * 4);
        }
    } else {
        const size_t g = ssm_half_glu_workspace_bytes(Bt * L, H, 1);
        if (g == 0) return false;
        o.glu = off; off += up(g);
        o.dypre = off; off += TH;
    }
    o.total = off;
    return true;
}
}  // namespace

size_t ssm_block_workspace_bytes(int64_t Bt, int64_t L, int64_t H, int64_t P, int want_bwd)
{
    BlockLayout bl;
    return make_block_layout(Bt, L, H, P, want_bwd != 0, bl) ? bl.total : 0;
}

ssm_status ssm_block_fwd(const ssm_c64 *Lambda, const ssm_c64 *B, const ssm_c64 *C, const float *D,
                         const float *log_delta, const float *W, const float *u, const uint8_t *is_first,
                         const ssm_c64 *x0, int64_t Bt, int64_t L, int64_t H, int64_t P,
                         float *y, float *out, float *gate, ssm_c64 *x, ssm_c64 *x_last,
                         void *workspace, size_t ws_bytes, void *stream)
{
    if (!W || !out || !y) return SSM_ERR_INVALID_ARG;
    ssm_status st = check_dims(Bt, L, H, P);
    if (st != SSM_OK) return st;
    BlockLayout bl;
    if (!make_block_layout(Bt, L, H, P, false, bl)) return SSM_ERR_UNSUPPORTED;
    if (misaligned(W, 4) || misaligned(out, 4) || misaligned(gate, 4)) return SSM_ERR_INVALID_ARG;
    if (!workspace || misaligned(workspace, ALIGN) || ws_bytes < bl.total) return SSM_ERR_WORKSPACE;
    char *ws = static_cast<char *>(workspace);
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *x1 = reinterpret_cast<float *>(ws + bl.x1);
    // the layer; its output projection also stores x1 = GELU(y)
    GateMax gm{reinterpret_cast<unsigned *>(ws + bl.x1_rowmax), W, (size_t)H * H, reinterpret_cast<unsigned *>(ws + bl.wslots), bl.nwslots};
    st = run_fwd(Lambda, B, C, D, log_delta, u, is_first, x0, Bt, L, H, P, y, x, x_last, ws + bl.ssm, bl.x1 - bl.ssm, s,
                 nullptr, x1, bl.gate_two_planes ? &gm : nullptr);
    if (st != SSM_OK) return st;
    // out[t, j] = y[t, j] sigmoid(sum_i x1[t, i] W[i, j])
    GemmArgs g{};
    g.A = x1; g.lda = H; g.a_kcontig = 1;
    g.B = W; g.ldb = H; g.b_kcontig = 0;
    g.C = out; g.ldc = H; g.E = y; g.lde = H; g.C2 = gate; g.epilogue = 3;
    g.M = (int)(Bt * L); g.N = (int)H; g.K = (int)H; g.splits = 1;
    if (bl.gate_two_planes) {
        g.amaxA = AbsMax{nullptr, 0, gm.x1_rowmax, (int)(H / 64), (long)(Bt * L)};
        g.amaxB = AbsMax{gm.wslots, gm.nwslots, nullptr, 0, 0};
    }
    HIP_TRY(launch_gemm(g, s));
    return SSM_OK;
}

ssm_status ssm_block_bwd(const ssm_c64 *Lambda, const ssm_c64 *B, const ssm_c64 *C, const float *D,
                         const float *log_delta, const float *W, const float *u, const uint8_t *is_first,
                         const ssm_c64 *x0, int64_t Bt, int64_t L, int64_t H, int64_t P,
                         const ssm_c64 *x, const float *y, const float *gate, const float *dout,
                         float *du, ssm_c64 *dLambda, ssm_c64 *dB, ssm_c64 *dC, float *dD, float *dlog_delta,
                         ssm_c64 *dx0, float *dW, void *workspace, size_t ws_bytes, void *stream)
{
    if (!W || !y || !gate || !dout || !dW) return SSM_ERR_INVALID_ARG;
    ssm_status st = check_dims(Bt, L, H, P);
    if (st != SSM_OK) return st;
    BlockLayout bl;
    if (!make_block_layout(Bt, L, H, P, true, bl)) return SSM_ERR_UNSUPPORTED;
    if (!workspace || misaligned(workspace, ALIGN) || ws_bytes < bl.total) return SSM_ERR_WORKSPACE;
    char *ws = static_cast<char *>(workspace);
    float *dypre = reinterpret_cast<float *>(ws + bl.dypre);
    // the gate's adjoint turns dout into the gradient of the layer's output, then the layer's own pass
    st = ssm_half_glu_bwd(y, W, gate, dout, Bt * L, H, dypre, dW, ws + bl.glu, bl.dypre - bl.glu, stream);
    if (st != SSM_OK) return st;
    return run_bwd(Lambda, B, C, D, log_delta, u, is_first, x0, Bt, L, H, P, x, dypre, du, dLambda, dB, dC, dD,
                   dlog_delta, dx0, ws + bl.ssm, bl.glu - bl.ssm, static_cast<hipStream_t>(stream), nullptr);
}

ssm_status ssm_workspace_status(const void *workspace, void *stream)
{
    if (!workspace) return SSM_ERR_WORKSPACE;
    HIP_TRY(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
    WsHeader h{};
    HIP_TRY(hipMemcpy(&h, workspace, sizeof(h), hipMemcpyDeviceToHost));
    if (h.magic != 0x53534d31u) return SSM_ERR_INVALID_ARG;   // no call has used this workspace
    return h.err ? SSM_ERR_SCAN_TIMEOUT : SSM_OK;
}

}  // extern "C"
