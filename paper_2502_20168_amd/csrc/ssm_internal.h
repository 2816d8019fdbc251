// Internal declarations shared by the translation units of libssmscan (gfx950 only).
// Nothing here is part of the C ABI; see include/ssm.h for that.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace ssm {

// ---------------------------------------------------------------------------------------------
// Projection GEMM:  C[m,n] = sum_k A(m,k) * B(n,k)  (+ epilogue term)
// epilogue 0: none; 1: + diag[n] * E[m,n]; 2: + [not rowflag[m]] * (Abar (.) E)[m,n] with diag = Abar
// as interleaved complex and the columns of C and E interleaved (re, im) pairs (one recurrence step);
// 3: C = E (.) sigmoid(product), sigmoid kept in C2 when non-null (half-GLU gate);
// 4: C = E + product (.) E2 (adjoint of the gate with respect to its input: E = dy (.) s, E2 = GELU'(u));
// 6: as 1, and C2 = GELU(C) (output projection that feeds the half-GLU gate);
// 7: the resettable scan over the rows of the output tile (see ScanEpilogue): C = states;
// 8: the reverse-time scan of the gradient pass over the rows of the output tile: C = chi;
// 5: C = product + E (E may be null), C2 = [not rowflag[m]] conj(Abar) (.) C with diag = Abar and complex
//    (re, im) column pairs (adjoint of one recurrence step)
// A(m,k) = a_kcontig ? A[m*lda + k] : A[k*lda + m];  B(n,k) = b_kcontig ? B[n*ldb + k] : B[k*ldb + n]
// splits > 1: split z covers a contiguous K range and writes its own slab C + z*M*ldc
// (no epilogue term in that case); the caller reduces the slabs.
// ---------------------------------------------------------------------------------------------
// Epilogue 7 of the projection GEMM: the resettable scan (Eq. 4 with the elements of Eq. 9 and the
// operator of Eq. 10) over the rows of the output tile itself, so that the input projection stores
// the states x directly and Bbar u never goes to memory.  Rows are tokens (Bt sequences of L steps,
// L a multiple of the 128-row tile), columns (re, im) pairs of P states.
// Largest magnitude of a matrix, kept as n bit patterns of non-negative floats whose maximum it is
// (written by the kernel that produced the matrix, or by a pass over it), or, for a matrix whose
// rows are tokens, per row: rows[j * row_stride + r], j < row_parts, are patterns whose maximum is the
// largest magnitude of row r.  A product whose two operands both carry one may stage them as two
// scaled fp16 planes (see gemm_kernel.h); per-row maxima (k-contiguous A operand only) give
// every row its own scale.
constexpr int ABSMAX_SLOTS = 512;            // slots of a maximum that is gathered with atomics
struct AbsMax {
    const unsigned *slots; int n;            // slots == nullptr and rows == nullptr: not known
    const unsigned *rows; int row_parts; long row_stride;
};

struct ScanEpilogue {
    const float2 *lam;            // [P] Abar
    const uint8_t *is_first;      // [Bt*L] or null
    const float2 *x0;             // [Bt, P] or null
    float2 *x_last;               // [Bt, P] or null (forward)
    const float2 *xsaved;         // [Bt, L, P] states of the forward pass (reverse, epilogue 8)
    float2 *partial;              // [Bt * L/128, P] per-tile rows of dAbar (reverse)
    float2 *dx0;                  // [Bt, P] or null (reverse)
    unsigned long long *desc;     // [M/128 * ceil(N/128) * 64][2] tagged aggregate words, zero on entry
    unsigned *err;                // set when a bounded wait gives up
    unsigned *amax_out;           // [ABSMAX_SLOTS] or null: atomic maximum of the magnitudes stored to C, zero on entry
    unsigned *xmax_out;           // [ABSMAX_SLOTS] or null (reverse, with amax_out): atomic maximum of the magnitudes of xsaved
    unsigned *rowmax_out;         // [ceil(N/128), M] or null: per column tile and row, the largest magnitude stored to C
    int L, P;
    unsigned spin_limit;
};

struct GemmArgs {
    const float *A; int64_t lda; int a_kcontig;
    const float *B; int64_t ldb; int b_kcontig;
    float *C; int64_t ldc;
    const float *diag; const float *E; int64_t lde;
    int epilogue; const uint8_t *rowflag;
    const float *E2; float *C2;                      // epilogues 3 and 4 (gate), pitch lde / ldc
    int M, N, K, splits;
    ScanEpilogue scan;                               // epilogues 7 and 8
    AbsMax amaxA, amaxB;                             // largest magnitudes of A and B when known
    unsigned *c2_rowmax;                             // epilogue 6, tile tiers 0 and 1: [ceil(N/64)][M] words, the largest
                                                     // magnitude of every row of C2 per piece of 64 columns; or null
};
// The gate's products stage two scaled fp16 planes per operand (and the passes before them measure the
// largest magnitudes) at widths that are multiples of 64 from 512 on, with enough tokens that a T x H
// product runs on tiles whose wavefronts own 64 columns (measured on 4096 tokens: -13 % at H = 1024, even
// at H = 512; +2 % at 1024 tokens, H = 256, where the passes cost more than the shorter K loops save)
inline bool gate_two_planes_shape(int64_t T, int64_t H) { return H % 64 == 0 && H >= 512 && ((T + 63) / 64) * ((H + 127) / 128) >= 200; }
// tile tier launch_gemm picks for an M x N product with `splits` K splits: 0 = 128x128x32 tiles, 1 = 64x128x32, 2 = 64x64x64
int gemm_tile_tier(int64_t M, int64_t N, int splits);
// the input projection (epilogue 7) and C^H dy (epilogue 8, the reverse scan of the gradient pass) scan
// their own output tiles at this shape
bool gemm_scan_shape_ok(int64_t Bt, int64_t L, int64_t P);
// bytes of tagged words epilogues 7 and 8 need (zeroed before the launch)
size_t gemm_scan_desc_bytes(int64_t Bt, int64_t L, int64_t P);
// a product is staged as two scaled fp16 planes per operand when both operands carry their largest magnitude
bool gemm_use_two_planes(const GemmArgs &g);
// argument checks of the scanning epilogues; layout code of a problem (-1: no instantiation)
bool gemm_scan_args_ok(const GemmArgs &g);
int gemm_layout_of(const GemmArgs &g);
hipError_t launch_gemm(const GemmArgs &g, hipStream_t s);
// the instantiations of the kernel for one problem per launch (tier 0: 128x128x32 tiles, 1: 64x128x32, 2: 64x64x64)
hipError_t gemm_dispatch_two_planes(const GemmArgs &g, int tier, hipStream_t s);
hipError_t gemm_dispatch_three_planes(const GemmArgs &g, int tier, hipStream_t s);
// a T x H product with a K loop of 2P has 100-199 tiles of 128x128 and a K loop long enough to halve (du next to
// the dBbar slabs at shapes with separate scan kernels runs as two K halves then)
bool gemm_out_split_shape(int64_t T, int64_t H, int64_t P);
// two independent problems in one launch (falls back to two launches for layouts without a
// paired instantiation)
hipError_t launch_gemm_pair(const GemmArgs &a, const GemmArgs &b, hipStream_t s, bool second_first = false);
// three independent problems in one launch: a product over the state dimension and two K = T reductions
// (slabs_first: b and c take the first slots of the launch, a the last)
hipError_t launch_gemm_triple(const GemmArgs &a, const GemmArgs &b, const GemmArgs &c, hipStream_t s, bool slabs_first = false);
// number of K splits for a reduction over K rows with an M x N result that shares its launch
// with a product of partner_tiles 128x128 tiles
int gemm_pick_splits(int64_t M, int64_t N, int64_t K, int64_t partner_tiles);
// the same for launches of several rounds of work items (a schedule model of the launch; red_first: the
// reduction's work items belong in the first slots); the model behind it: reductions over T rows with red_tiles
// tiles of 128x128 in all (split_bytes of slabs per split in all) beside a product of main_tiles tiles with a
// K loop of k_main, one or two workgroups per CU
int gemm_pick_splits_balanced(int64_t M, int64_t N, int64_t K, int64_t main_tiles, int64_t k_main, bool &red_first);
int gemm_pick_splits_model(int64_t T, int64_t main_tiles, int64_t k_main, int64_t red_tiles, size_t split_bytes, bool two_per_cu,
                           bool &red_first);
// a product over T tokens with N columns has so few tiles that it and the reduction in its launch run on
// 64x64x64 tiles; the K splits of that reduction (partner_tiles64: the product's 64x64 tiles, k_main: its K)
bool gemm_small_pair(int64_t T, int64_t N);
int gemm_pick_splits_small(int64_t M, int64_t N, int64_t K, int64_t partner_tiles64, int64_t k_main);

// ---------------------------------------------------------------------------------------------
// Resettable scan over the sequence dimension (forward and reverse time).
// One thread owns SCAN_E consecutive steps of one (sequence, state) lane; a workgroup of 256
// threads is laid out as cy chunks x pxb lanes and so covers cy*SCAN_E steps of pxb states;
// longer sequences use several workgroups along time that hand their running state forward
// through descriptors in global memory (decoupled look-back).
// ---------------------------------------------------------------------------------------------
constexpr int SCAN_E = 16;
constexpr int SCAN_THREADS = 256;
constexpr int SCAN_TICKET_STRIDE = 16;   // uint32 slots between the ticket counters of two chains

struct ScanDesc {            // one per (workgroup, lane); 32 bytes; every word = (float << 32) | tag
    unsigned long long agg[2];   // re, im of the state at the end of the workgroup's steps for zero
                                 // incoming state; tag 1 = no reset among the steps, tag 2 = reset
    unsigned long long incl[2];  // re, im of that state with the incoming state included; tag 3
};

struct ScanPlan {
    int pxb, cy;             // lanes and chunks per workgroup (pxb * cy == SCAN_THREADS)
    int nPX, nTB;            // workgroups along the state and the time dimension
    int64_t nblocks;         // nPX * Bt * nTB
    size_t ticket_bytes;     // per-chain ticket counters, 0 when nTB == 1
    size_t desc_bytes;       // 0 when nTB == 1
    size_t partial_elems;    // Bt * nTB * P complex partial sums of the reverse scan
};
ScanPlan plan_scan(int64_t Bt, int64_t L, int64_t P);

struct WsHeader {            // first 256 bytes of every workspace
    uint32_t err, magic;
};

struct ScanArgs {
    const float2 *in;        // v (forward) or gx (reverse), [Bt,L,P]
    float2 *out;             // x (forward) or chi (reverse); may alias `in`
    const float2 *lam;       // A_bar [P]
    const uint8_t *is_first; // [Bt,L] or null
    const float2 *x0;        // [Bt,P] or null
    float2 *x_last;          // forward only, or null
    const float2 *xsaved;    // reverse only: states x [Bt,L,P]
    float2 *partial;         // reverse only: [Bt*nTB, P]
    float2 *dx0;             // reverse only, or null
    ScanDesc *desc;
    uint32_t *ticket;        // per-chain counters, SCAN_TICKET_STRIDE apart (nTB > 1 only)
    uint32_t *err;           // &WsHeader::err (the magic word follows it)
    int Bt, L, P, pxb, cy, nPX, nTB;
    uint32_t spin_limit;
    unsigned *rowmax_out;    // [Bt*L] or null: atomic maximum of the magnitudes of every token row of `out`, zero on entry
    unsigned *amax_out;      // [ABSMAX_SLOTS] (with rowmax_out): atomic maximum of the magnitudes of `out`, zero on entry
};
hipError_t launch_scan(const ScanArgs &a, bool reverse, hipStream_t s);
// workspace layout of the scan-level entry points: header, ticket counters, descriptors, partial rows
struct ScanOnlyLayout { ScanPlan plan; size_t hdr, ticket, desc, dApart, total; };
int make_scan_layout(int64_t Bt, int64_t L, int64_t P, bool rev, ScanOnlyLayout &o);   // returns an ssm_status
// body of ssm_scan_states (returns an ssm_status); workspace may be any 256-byte aligned device memory
int scan_states_forward(const void *A_bar, void *v, const uint8_t *is_first, const void *x0, int64_t Bt, int64_t L,
                        int64_t P, void *x_last, void *workspace, size_t ws_bytes, hipStream_t s);
uint32_t scan_spin_limit();
uint32_t scan_set_spin_limit(uint32_t polls);
// zeroes the header and `scratch_bytes` (a multiple of 16) of ticket counters + descriptors
hipError_t launch_clear(WsHeader *hdr, void *scratch, size_t scratch_bytes, hipStream_t s);
// out[p] = sum_i partial[i*P + p]
hipError_t launch_reduce_partials(const float2 *partial, int64_t n, int64_t P, float2 *out, hipStream_t s);

// ---------------------------------------------------------------------------------------------
// Parameter-sized kernels
// ---------------------------------------------------------------------------------------------
struct ColDotArgs {          // partial[s][h] = sum over the rows of slab s of a[t,h] * b[t,h]
    const float *a; const float *b; int64_t T; int H; int nslab; float *partial;
};
int coldot_slabs(int64_t T);

struct PrepArgs {
    const float2 *Lambda; const float2 *B; const float2 *C; const float *log_delta;
    int P, H;
    float2 *lam_bar;         // [P]
    float *Bbar_ri;          // [2P, H]: row 2p = Re(g_p B[p,:]), row 2p+1 = Im(g_p B[p,:]); may be null
    float *Cc;               // [H, 2P]: (Re C[h,p], -Im C[h,p]) interleaved; may be null
    float2 *Bbar_c64;        // [P, H] interleaved complex, for ssm_discretize; may be null
    WsHeader *hdr;           // cleared when non-null
    ColDotArgs cd;           // cd.partial non-null: the launch also computes the column-dot slabs
    int cd_colblocks;        // set by launch_prep
    uint4 *zero16; size_t n16;   // region to clear in the same launch (tagged words of epilogue 7), may be null
    int zero_block0;         // set by launch_prep: first workgroup of the clearing range
    // largest magnitudes for the two-plane fp16 staging of the products (all may be null):
    unsigned *bbar_max;      // [P]: of the rows 2p, 2p+1 of Bbar_ri
    unsigned *cc_max;        // [H]: of row h of Cc
    unsigned *cd_amax, *cd_bmax;   // [cd.nslab * ceil(cd.H/64)]: of the pieces of cd.a and cd.b
    unsigned *cd_arow;       // [ceil(cd.H/64)][cd.T]: of every row of cd.a within a block of 64 columns
    struct Pass { const float *x; size_t n; unsigned *slots; int nblocks, block0, vec, rowlen; } pass[2];
                             // rowlen == 0: slots[nblocks] of nblocks pieces of x[n]; rowlen > 0: slots[n / rowlen],
                             // one per row of rowlen values; block0 and vec set by launch_prep
};
constexpr int PREP_PASS_BLOCKS = 256;        // pieces of a pass that measures one maximum per piece
constexpr int PREP_ROW_PASS_BLOCKS = 1024;   // workgroups of a pass that measures one maximum per row
hipError_t launch_prep(const PrepArgs &a, hipStream_t s);



// out = s0 + s1 + D (.) e over n = rows * H elements: the two K halves of du and D dy, added by extra
// workgroups of the parameter epilogue's launch (both only wait for the products before them)
struct SumHalvesArgs {
    const float *s0, *s1, *D, *e; float *out; long n; int H;
    int vec, nblocks;                        // set by launch_epilogue
};

struct EpilogueArgs {
    SumHalvesArgs sum;                       // s0 == nullptr: nothing to add
    const float2 *Lambda; const float2 *B; const float *log_delta; int P, H;
    const float *dBbar_part; int nsplit_B;   // [nsplit_B][2P][H]
    const float *dC_part; int nsplit_C;      // [nsplit_C][H][2P]  (sum_t dy x_re, sum_t dy x_im)
    const float2 *dAbar_part; int64_t npart; // [npart][P]
    const float *dD_part; int nslab;         // [nslab][H]
    float2 *dLambda; float2 *dB; float2 *dC; float *dD; float *dlog_delta;
};
hipError_t launch_epilogue(const EpilogueArgs &a, hipStream_t s);

}  // namespace ssm
