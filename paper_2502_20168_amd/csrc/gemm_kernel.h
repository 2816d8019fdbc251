// fp32-accurate GEMM on the 16-bit matrix cores of gfx950: three-way bf16 operand split, or two
// scaled fp16 planes where the largest magnitude of both operands is known (see split2_f16).
//
//   C[m,n] = sum_k A(m,k) * B(n,k)  (+ diag[n] * E[m,n]),   A, B, C fp32
//
// Every fp32 operand value a is split exactly into three bf16 numbers a = a1 + a2 + a3
// (a1 = trunc_bf16(a), a2 = trunc_bf16(a - a1), a3 = a - a1 - a2; 8 + 8 + 8 mantissa bits).  The
// product a*b is then accumulated in fp32 from the six partial products whose weight is at
// least 2^-16 of the leading one (a1b1, a1b2, a2b1, a1b3, a2b2, a3b1); the three dropped ones
// are below 2^-24 |a||b|, i.e. at the level of one fp32 rounding.  Each partial product of two
// bf16 numbers is exact in fp32, so the result has fp32-class accuracy, while the six
// v_mfma_f32_32x32x16_bf16 (32 cycles for 32x32x16 MACs) cost 192 cycles where the fp32 matrix
// instruction needs 512 cycles for the same 32x32x16 block.
//
// The split happens once per staged element, between the global load and the LDS store; LDS
// holds three bf16 planes per operand as [row][k] (k contiguous, row stride BK+8 halves so that
// the 16-byte fragment reads of 16 consecutive rows fall into distinct banks).
#pragma once

#include "gemm_common.h"
#include "lookback.h"

#include <atomic>

namespace ssm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

struct Split4 { bf16x4 p[3]; };

// Exact three-way split of four floats by truncation: a1 = the upper 16 bits of a, a2 = the
// upper 16 bits of a - a1, a3 = a - a1 - a2 (which has at most 8 significant bits left, so its
// upper 16 bits hold it exactly).  Only full-rate integer/float VALU operations are used; two
// bf16 values are packed with one byte permute.
__device__ __forceinline__ Split4 split3(float4 v)
{
    const unsigned x[4] = {__float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z), __float_as_uint(v.w)};
    unsigned h[4], m[4], l[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        h[i] = x[i] & 0xffff0000u;
        const float r1 = __uint_as_float(x[i]) - __uint_as_float(h[i]);
        m[i] = __float_as_uint(r1) & 0xffff0000u;
        const float r2 = r1 - __uint_as_float(m[i]);
        l[i] = __float_as_uint(r2);
    }
    // bytes 2,3 of the first source become the low half, bytes 2,3 of the second the high half
    union { unsigned u[2]; bf16x4 b; } ph, pm, pl;
    ph.u[0] = __builtin_amdgcn_perm(h[1], h[0], 0x07060302u); ph.u[1] = __builtin_amdgcn_perm(h[3], h[2], 0x07060302u);
    pm.u[0] = __builtin_amdgcn_perm(m[1], m[0], 0x07060302u); pm.u[1] = __builtin_amdgcn_perm(m[3], m[2], 0x07060302u);
    pl.u[0] = __builtin_amdgcn_perm(l[1], l[0], 0x07060302u); pl.u[1] = __builtin_amdgcn_perm(l[3], l[2], 0x07060302u);
    Split4 o;
    o.p[0] = ph.b; o.p[1] = pm.b; o.p[2] = pl.b;
    return o;
}

// Two-plane split into fp16: with the operand (the whole matrix, or one row of it) scaled by a power
// of two so that its largest magnitude lies in [2^14, 2^15), a1 = rn_fp16(s a) and a2 = rn_fp16(s a - a1) (the residual is
// formed exactly by one fused multiply-add).  fp16 keeps 11 significant bits, so
// |s a - a1 - a2| <= 2^-22 |s a| as long as a2 is a normal fp16 number, i.e. for |a| down to 2^-17
// of the largest magnitude; below that the planes act as a fixed-point pair with an absolute error
// of at most 2^-25 (half the spacing of the fp16 subnormals) in scaled units, i.e. 2^-39 of the
// largest magnitude.  The three products a1b1, a1b2, a2b1 (each exact in fp32) then leave a
// relative error of about 3 * 2^-22 per product term at worst -- the level of fp32 rounding -- for
// half the matrix instructions of the three-way bf16 split.  The scale is taken off the
// accumulators before anything is stored.
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ Split4 split2_f16(float4 v, float s)
{
    const f32x2 a = {v.x * s, v.y * s}, b = {v.z * s, v.w * s};
    union { f16x2 h; unsigned u; } ha, hb, la, lb;
    ha.h = __builtin_convertvector(a, f16x2);
    hb.h = __builtin_convertvector(b, f16x2);
    const f32x2 ra = {__builtin_fmaf(v.x, s, -(float)ha.h.x), __builtin_fmaf(v.y, s, -(float)ha.h.y)};
    const f32x2 rb = {__builtin_fmaf(v.z, s, -(float)hb.h.x), __builtin_fmaf(v.w, s, -(float)hb.h.y)};
    la.h = __builtin_convertvector(ra, f16x2);
    lb.h = __builtin_convertvector(rb, f16x2);
    union { unsigned u[2]; bf16x4 b; } p0, p1;       // bf16x4 is only the 8-byte container of the LDS store
    p0.u[0] = ha.u; p0.u[1] = hb.u;
    p1.u[0] = la.u; p1.u[1] = lb.u;
    Split4 o;
    o.p[0] = p0.b; o.p[1] = p1.b; o.p[2] = p1.b;
    return o;
}
template <int NPL>
__device__ __forceinline__ Split4 split_planes(float4 v, float s) { return NPL == 3 ? split3(v) : split2_f16(v, s); }

// log2 of the power-of-two scale that brings the largest magnitude of an operand into [2^14, 2^15):
// every lane of the wavefront gets the same value.  The slots hold bit patterns of non-negative
// floats, which order like unsigned integers.  An operand of zeros gets the largest scale (its
// planes are zeros whatever the scale).  Two steps, so that the loads can be issued ahead of other
// memory traffic and waited for behind it: absmax_issue starts eight independent loads per lane (the
// first 512 slots), absmax_log2_scale reduces them (and walks the slots beyond 512, if any).
__device__ __forceinline__ int log2_scale_of(unsigned maxbits);
struct AbsMaxLoads { unsigned w[8]; };
__device__ __forceinline__ AbsMaxLoads absmax_issue(const AbsMax &m, int lane)
{
    AbsMaxLoads r;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int i = lane + 64 * j;
        const unsigned t = m.slots[i < m.n ? i : 0];         // unconditional, so that the loads overlap
        r.w[j] = i < m.n ? t : 0u;
    }
    return r;
}
__device__ __forceinline__ int absmax_log2_scale(const AbsMax &m, const AbsMaxLoads &r, int lane)
{
    unsigned v = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) v = max(v, r.w[j]);
    for (int base = 512; base < m.n; base += 512) {          // more than 512 slots: eight more per lane at a time
        unsigned w[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int i = base + lane + 64 * j;
            const unsigned t = m.slots[i < m.n ? i : 0];
            w[j] = i < m.n ? t : 0u;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) v = max(v, w[j]);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = max(v, (unsigned)__shfl_xor((int)v, o));
    return log2_scale_of(v);     // (defined below) 14 - floor(log2(maximum)), kept inside the exponent range
}
__device__ __forceinline__ float pow2f(int e) { return __uint_as_float((unsigned)(e + 127) << 23); }   // e in [-127, 127]
__device__ __forceinline__ int log2_scale_of(unsigned maxbits)
{
    const int e = (int)((maxbits >> 23) & 0xffu);
    int f = 268 - e;
    f = f < 1 ? 1 : (f > 254 ? 254 : f);
    return f - 127;
}
// The same for one row of an operand with per-row maxima (the first eight parts by independent loads).
__device__ __forceinline__ AbsMaxLoads absmax_row_issue(const AbsMax &m, long row)
{
    AbsMaxLoads r;
    const unsigned *p = m.rows + row;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const unsigned t = p[j < m.row_parts ? (size_t)j * m.row_stride : 0];
        r.w[j] = j < m.row_parts ? t : 0u;
    }
    return r;
}
__device__ __forceinline__ int absmax_row_log2_scale(const AbsMax &m, const AbsMaxLoads &r, long row)
{
    unsigned v = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) v = max(v, r.w[j]);
    for (int j0 = 8; j0 < m.row_parts; j0 += 8) {            // wide states or layers: eight more at a time
        unsigned w[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const unsigned t = m.rows[(j0 + j < m.row_parts ? (size_t)(j0 + j) * m.row_stride : 0) + row];
            w[j] = j0 + j < m.row_parts ? t : 0u;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) v = max(v, w[j]);
    }
    return log2_scale_of(v);
}

// Stages one R x BK fp32 operand tile: global -> registers (fp32) -> split -> NPL LDS planes.
// A thread handles float4 units along the contiguous index of the source and writes the four
// bf16 values of every plane with one 8-byte store, whatever the layout:
//   k-contiguous source (KC):  unit = 1 row x 4 k;   planes are [row][k], row stride BK+8 halves;
//   row-contiguous source:     unit = 1 k x 4 rows;  planes are [k][row], k stride R+16 halves --
//       the same orientation as in memory, so global loads are whole 512-byte lines and nothing is
//       transposed here; the consumers fetch their fragments with the transposing LDS read.
template <int R, int BK, bool KC, int NT, int NPL>
struct SplitLoader {
    static constexpr int NV = R * BK / 4 / NT;
    static_assert(NV >= 1 && NV * NT * 4 == R * BK, "tile must be a multiple of the workgroup's float4 loads");
    static constexpr int S = KC ? BK + 8 : R + 16;        // stride of the slow index in halves
    static constexpr int PLANE = KC ? R * S : BK * S;     // halves per plane
    float4 r[NV];

    // k-contiguous source: row handled by the g-th group of BK/4 lanes.  With BK = 32 a group
    // writes 64 contiguous bytes (16 banks) per plane and the row stride is 80 bytes, so
    // neighbouring groups take rows 4 apart (80*4 = 16 banks mod 32): their writes then tile the 32
    // banks exactly, where consecutive rows would overlap in 4 banks.
    static __device__ __forceinline__ int kc_row(int g)
    {
        return (BK == 32 && R % 4 == 0) ? (g % (R / 4)) * 4 + g / (R / 4) : g;
    }

    // k-contiguous source: the tile row that unit i of this thread belongs to
    static __device__ __forceinline__ int unit_row(int tid, int i) { return kc_row((tid + i * NT) / (BK / 4)); }

    // FAST 0: every element guarded (4-byte loads); 1: 16-byte loads of a tile that lies inside the operand;
    // 2: 16-byte loads of a k-contiguous operand whose tile hangs over the last row (that row is re-read:
    // the values only reach output rows or columns that are never stored)
    template <int FAST>
    __device__ __forceinline__ void load(const float *__restrict__ X, long ld, int row0, int rows, int k0,
                                         int kend, int tid)
    {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int idx = tid + i * NT;
            if (KC) {
                const int row = kc_row(idx / (BK / 4)), kq = idx % (BK / 4);
                const long gr = row0 + row;
                const int k = k0 + 4 * kq;
                if (FAST == 1) {
                    r[i] = *reinterpret_cast<const float4 *>(X + gr * ld + k);
                } else if (FAST == 2) {
                    r[i] = *reinterpret_cast<const float4 *>(X + (gr < rows ? gr : (long)rows - 1) * ld + k);
                } else {
                    float t[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) t[j] = (gr < rows && k + j < kend) ? X[gr * ld + k + j] : 0.f;
                    r[i] = make_float4(t[0], t[1], t[2], t[3]);
                }
            } else {
                const int kk = idx / (R / 4), rq = idx % (R / 4);
                const long k = k0 + kk, gr = row0 + 4 * rq;
                if (FAST != 0) {
                    r[i] = *reinterpret_cast<const float4 *>(X + k * ld + gr);
                } else {
                    float t[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) t[q] = (gr + q < rows && k < kend) ? X[k * ld + gr + q] : 0.f;
                    r[i] = make_float4(t[0], t[1], t[2], t[3]);
                }
            }
        }
    }

    // scale[i]: two-plane staging only (a power of two for the i-th unit of the thread, see split2_f16)
    __device__ __forceinline__ void store(__bf16 *lds, int tid, const float (&scale)[NV]) const
    {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int idx = tid + i * NT;
            const int off = KC ? kc_row(idx / (BK / 4)) * S + 4 * (idx % (BK / 4))
                               : (idx / (R / 4)) * S + 4 * (idx % (R / 4));
            const Split4 sp = split_planes<NPL>(r[i], scale[i]);
#pragma unroll
            for (int s = 0; s < NPL; ++s) *reinterpret_cast<bf16x4 *>(lds + s * PLANE + off) = sp.p[s];
        }
    }

    // Fragment of a 32-row block for one 16-wide k step: lane (li = l % 32, hh = l / 32) gets the
    // 8 values row0 + li, k = kbase + 8 hh .. 8 hh + 7 of a plane.
    //   KC: one 16-byte read.
    //   row-contiguous: two transposing 8-byte reads.  ds_read_b64_tr_b16 works on groups of 16
    //   lanes: lane i of a group receives element i % 4 of the 8-byte chunks addressed by lanes
    //   i / 4, i / 4 + 4, i / 4 + 8, i / 4 + 12 of the group.  With lane sl of a group pointing at
    //   [k0 + sl / 4][m0 + 4 (sl % 4)], lane i receives rows m0 + i at k0 .. k0 + 3.
    static __device__ __forceinline__ bf16x8 fragment(const __bf16 *plane, int row0, int kbase, int l)
    {
        if (KC) {
            return *reinterpret_cast<const bf16x8 *>(plane + (row0 + (l & 31)) * S + kbase + 8 * (l >> 5));
        } else {
            typedef short v4s __attribute__((ext_vector_type(4)));
            const int sl = l & 15, grp = l >> 4;
            const __bf16 *p0 = plane + (kbase + 8 * (grp >> 1) + (sl >> 2)) * S + row0 + 16 * (grp & 1) + 4 * (sl & 3);
            union { v4s h[2]; bf16x8 v; } u;
            u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4s __attribute__((address_space(3))) *)(p0));
            u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4s __attribute__((address_space(3))) *)(p0 + 4 * S));
            return u.v;
        }
    }
};

// ---------------------------------------------------------------------------------------------
// Epilogues 7 and 8: resettable scan (forward, or the reverse one of the gradient pass) over the
// rows of a 128 x 128 output tile: 128 steps of 64 complex states, either a piece of one sequence
// (L a multiple of 128; the pieces form a chain) or 128/L whole sequences (L = 16, 32, 64).
// 512 threads (the consumers and the first four producer wavefronts) are 64 lanes x 8 chunks of
// 16 steps:
//   1. the accumulators go through LDS so that a thread owns 16 consecutive steps of one lane;
//   2. per-thread pass for zero incoming state, chunk aggregates combined through LDS;
//   3. chain of tiles: the tile's aggregate (state for zero incoming state, reset tag) is
//      published as tagged 64-bit words before any wait; the tiles of the same sequence and column
//      block that come earlier in scan order are folded in that order from the sequence start (x0
//      or zero), which is one canonical order whatever the timing, so results are bitwise
//      reproducible;
//   4. second per-thread pass writes the states (forward: x_last at the sequence end; reverse: the
//      per-tile row of dAbar and dx0).
// Every predecessor sits in an earlier slot of the same XCD (placement mode 5), i.e. it was
// dispatched earlier and publishes without waiting for anything, and every wait is bounded.
// ---------------------------------------------------------------------------------------------
constexpr int SCAN_TILE = 128;                       // rows and columns of the tile
constexpr int SCAN_TS = SCAN_TILE + 4;               // LDS row stride of the staged tile (floats)
constexpr int SCAN_MAX_CHAIN = 32;                   // tiles per sequence the fold can take
constexpr int SCAN_WAVES = 8;                        // wavefronts that scan: the consumers and the first producers
constexpr int SCAN_RC = SCAN_TILE / SCAN_WAVES;      // consecutive steps per thread
constexpr size_t SCAN_LDS_BYTES = (size_t)SCAN_TILE * SCAN_TS * 4   // staged tile
                                  + SCAN_WAVES * 64 * 8 + SCAN_WAVES * 64 * 4   // chunk states and reset tags
                                  + SCAN_WAVES * 64 * 8 + SCAN_WAVES * 64 * 4   // predecessors, one batch (a wavefront each)
                                  + 64 * 8;                          // incoming state per lane
static_assert(SCAN_LDS_BYTES <= 80 * 1024, "two scanning workgroups share the 160 KB LDS of a CU");

// v[e], e < 16, per lane -> the maximum over the 64 lanes of v[rows16_index(lane)].  Two halving steps
// inside every quad (lanes that differ in bit 0, then bit 1, swap the half of the remaining values
// the other one keeps; data-parallel-primitive moves, no LDS), then the four values left per lane are
// combined over the lanes with the same two low bits: rotations by 4 and 8 inside a row of 16, then
// the two exchanges across rows (lane swaps).
template <int CTRL>
__device__ __forceinline__ unsigned dpp_move(unsigned v)
{
    return (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xf, 0xf, false);
}
// max(v, v of lane ^ 16) or max(v, v of lane ^ 32) with the lane-swap instructions of gfx950 (given the
// same register twice, v_permlane16_swap / v_permlane32_swap return it and its copy from the partner row
// or half): no LDS involved
template <int X>
__device__ __forceinline__ unsigned lane_xor_max(unsigned v)
{
    static_assert(X == 16 || X == 32, "rows of 16 lanes or halves of 32");
    if constexpr (X == 16) {
        const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
        return max((unsigned)r[0], (unsigned)r[1]);
    } else {
        const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
        return max((unsigned)r[0], (unsigned)r[1]);
    }
}
__device__ __forceinline__ unsigned rows16_wave_max(unsigned (&v)[16], int lane)
{
    {
        const bool up = lane & 1;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const unsigned keep = up ? v[k + 8] : v[k], send = up ? v[k] : v[k + 8];
            v[k] = max(keep, dpp_move<0xb1>(send));                   // quad_perm [1,0,3,2]: lane ^ 1
        }
    }
    {
        const bool up = (lane >> 1) & 1;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const unsigned keep = up ? v[k + 4] : v[k], send = up ? v[k] : v[k + 4];
            v[k] = max(keep, dpp_move<0x4e>(send));                   // quad_perm [2,3,0,1]: lane ^ 2
        }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        v[k] = max(v[k], dpp_move<0x124>(v[k]));                      // row_ror:4
        v[k] = max(v[k], dpp_move<0x128>(v[k]));                      // row_ror:8
        v[k] = lane_xor_max<16>(v[k]);
        v[k] = lane_xor_max<32>(v[k]);
    }
    // lanes 4j .. 4j+3 (j < 4) hand out value j
    const int j = (lane >> 2) & 3;
    return j == 0 ? v[0] : (j == 1 ? v[1] : (j == 2 ? v[2] : v[3]));
}
// the row whose maximum lane `lane` (< 16) holds after rows16_wave_max
__device__ __forceinline__ int rows16_index(int lane) { return ((lane >> 2) & 3) + 4 * ((lane >> 1) & 1) + 8 * (lane & 1); }

// v[e], e < 16, per lane -> the maximum over the 32 lanes that share lane bit 5 of v[rows16_half_index(lane)]
// (the two halves of a wavefront hold different rows of a 32x32 accumulator block): the same halving
// exchanges, then one full exchange between the two rows of 16 lanes.
__device__ __forceinline__ unsigned rows16_half_max(unsigned (&v)[16], int lane)
{
    {
        const bool up = lane & 1;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const unsigned keep = up ? v[k + 8] : v[k], send = up ? v[k] : v[k + 8];
            v[k] = max(keep, dpp_move<0xb1>(send));
        }
    }
    {
        const bool up = (lane >> 1) & 1;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const unsigned keep = up ? v[k + 4] : v[k], send = up ? v[k] : v[k + 4];
            v[k] = max(keep, dpp_move<0x4e>(send));
        }
    }
    {
        const bool up = (lane >> 2) & 1;
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const unsigned keep = up ? v[k + 2] : v[k], send = up ? v[k] : v[k + 2];
            v[k] = max(keep, (unsigned)__shfl_xor((int)send, 4));
        }
    }
    {
        const bool up = (lane >> 3) & 1;
        const unsigned keep = up ? v[1] : v[0], send = up ? v[0] : v[1];
        v[0] = max(keep, (unsigned)__shfl_xor((int)send, 8));
    }
    return max(v[0], (unsigned)__shfl_xor((int)v[0], 16));
}
__device__ __forceinline__ int rows16_half_index(int lane) { return 8 * (lane & 1) + 4 * ((lane >> 1) & 1) + 2 * ((lane >> 2) & 1) + ((lane >> 3) & 1); }

struct ScanLds {
    float *tile; float2 *cS; unsigned *cAny; float2 *pS; unsigned *pAny; float2 *sX;
    __device__ explicit ScanLds(void *base)
    {
        char *p = static_cast<char *>(base);
        tile = reinterpret_cast<float *>(p); p += (size_t)SCAN_TILE * SCAN_TS * 4;
        cS = reinterpret_cast<float2 *>(p); p += SCAN_WAVES * 64 * 8;
        cAny = reinterpret_cast<unsigned *>(p); p += SCAN_WAVES * 64 * 4;
        pS = reinterpret_cast<float2 *>(p); p += SCAN_WAVES * 64 * 8;
        pAny = reinterpret_cast<unsigned *>(p); p += SCAN_WAVES * 64 * 4;
        sX = reinterpret_cast<float2 *>(p);
    }
};

// Reverse scan: the saved states x_{t-1} of a thread's 16 steps (x_{-1} = x0, zero when absent), plus the
// last state of the sequence for the thread that owns its last steps.  They are requested before the K
// loop of the product starts and used in the second pass of the scan, so that their way from memory
// (16 bytes per token and state that nothing else in this launch reads) is hidden behind the matrix work.
struct ScanSaved { float2 xp[SCAN_RC]; float2 xl; };
__device__ __forceinline__ ScanSaved scan_request_saved(const ScanEpilogue &a, int tid, int m0, int n0)
{
    constexpr int RC = SCAN_RC;
    const int c = tid & 63, q = tid >> 6;
    const int p = n0 / 2 + c;
    const bool active = p < a.P;
    const int row0 = m0 + q * RC;
    const int b = row0 / a.L, t0 = row0 % a.L;
    const float2 *xprev = a.xsaved + ((long)row0 - 1) * a.P + p;                     // x_{t0-1}; valid for e >= 1 or t0 > 0
    ScanSaved s;
    s.xl = make_float2(0.f, 0.f);
    if (a.xmax_out && active && t0 + RC == a.L) s.xl = xprev[(long)RC * a.P];
#pragma unroll
    for (int e = 0; e < RC; ++e) {
        s.xp[e] = make_float2(0.f, 0.f);
        if (active) {
            if (t0 + e > 0) s.xp[e] = xprev[(long)e * a.P];
            else if (a.x0) s.xp[e] = a.x0[(long)b * a.P + p];
        }
    }
    return s;
}

// The flags of a thread's 16 steps as bit masks, formed before the K loop of the product so that the
// scan does not start with a trip to memory.  x = fmask: bit e = is_first at time t0 + e.  y = rmask: bit e =
// the state that flows into the step at time t0 + e is dropped -- forward: the step's own flag; reverse:
// the flag of the next time step (nothing flows in at the sequence end).
template <bool REV>
__device__ __forceinline__ uint2 scan_flag_masks(const ScanEpilogue &a, int tid, int m0)
{
    constexpr int RC = SCAN_RC;
    const int row0 = m0 + (tid >> 6) * RC, t0 = row0 % a.L;
    unsigned fmask = 0;
    if (a.is_first) {
        const uint8_t *fp = a.is_first + row0;
        if ((reinterpret_cast<uintptr_t>(fp) & 15) == 0) {
            const uint4 w0 = *reinterpret_cast<const uint4 *>(fp);
            if ((w0.x | w0.y | w0.z | w0.w) != 0) {
                const unsigned ww[4] = {w0.x, w0.y, w0.z, w0.w};
#pragma unroll
                for (int j = 0; j < RC; ++j) fmask |= (unsigned)(((ww[j >> 2] >> (8 * (j & 3))) & 0xffu) != 0) << j;
            }
        } else {
#pragma unroll
            for (int j = 0; j < RC; ++j) fmask |= (unsigned)(fp[j] != 0) << j;
        }
    }
    unsigned rmask = fmask;
    if (REV) {
        unsigned next = 1;
        if (t0 + RC < a.L) next = a.is_first ? (unsigned)(a.is_first[(long)row0 + RC] != 0) : 0u;
        rmask = (fmask >> 1) | (next << (RC - 1));
    }
    return make_uint2(fmask, rmask);
}

// tid: 0 .. 64*SCAN_WAVES-1 (the consumers and the first producer wavefronts: the scan is bound by
// the issue rate of dependent multiply-adds, so eight wavefronts with 16 steps per lane finish a pass
// in about half the time of four with 32); the tile is staged in lds.tile on entry (after the first
// two barriers).
// REV: the scan of the gradient pass, chi_t = gx_t + [not is_first_{t+1}] conj(Abar) chi_{t+1}, which
// walks time backwards (later chunks and later tiles are the predecessors) and also reduces
// dAbar += [not is_first_t] conj(x_{t-1}) chi_t per tile and writes dx0.
// PASSIVE: a wavefront of the workgroup that does not scan (producers beyond the eighth wavefront).  It
// runs through the same function and so meets the others at every workgroup barrier: all barriers stand
// at the top level of this function under conditions that are uniform over the workgroup, all work
// sits in blocks that a passive wavefront skips.
// REREAD (reverse scan): the second pass reads the tile's values from LDS again instead of keeping them in
// registers across the wait for the predecessors (for the register budget of two workgroups per CU).
template <bool REV, bool PASSIVE, bool REREAD = false>
__device__ __forceinline__ void scan_epilogue_body(const GemmDev &g, const ScanLds &lds, int tid, int m0, int n0, int tile,
                                                   const ScanSaved &saved, uint2 masks)
{
    constexpr int RC = SCAN_RC, NCH = SCAN_WAVES;
    constexpr bool ACTIVE = !PASSIVE;
    static_assert(RC == 16, "flag loads and the powers of Abar below assume 16 steps per lane");
    const ScanEpilogue &a = g.scan;
    const int c = tid & 63, q = PASSIVE ? 0 : tid >> 6;
    const int ql = REV ? NCH - 1 - q : q;                    // chunk index in scan order
    const int p = n0 / 2 + c;
    const bool active = ACTIVE && p < a.P;
    // A tile is either one piece of a chain of tiles of one sequence (L a multiple of 128) or holds
    // 128/L whole sequences (L = 16, 32, 64): then there is no chain, a sequence starts at a chunk
    // boundary inside the tile and its incoming state is x0 (forward) or zero (reverse).
    const bool whole_seqs = a.L < SCAN_TILE;
    const int row0 = m0 + q * RC;                            // token index of this thread's first step
    const int b = row0 / a.L, t0 = row0 % a.L;               // its sequence and its lowest time index
    const int tmL = whole_seqs ? 0 : (m0 % a.L) / SCAN_TILE, nt = whole_seqs ? 1 : a.L / SCAN_TILE;
    const int tn = tile % g.ntn;
    const int npred = REV ? nt - 1 - tmL : tmL;              // tiles of the chain that come earlier in scan order (uniform)
    const bool leader = ACTIVE && (ql == NCH - 1) && !whole_seqs;

    // state of a thread that lives across the barriers
    float2 lam = make_float2(0.f, 0.f), val[RC], S = make_float2(0.f, 0.f), lrc, l128;
    float2 Aex = make_float2(1.f, 0.f), Sex = make_float2(0.f, 0.f), X = make_float2(0.f, 0.f);
    float xmax = 0.f, amax = 0.f;                            // largest magnitude of the saved states read / of the values stored
    unsigned fmask = 0, rmask = 0;

    if constexpr (ACTIVE) {
        if (active) lam = a.lam[p];
        if (REV) lam.y = -lam.y;
#pragma unroll
        for (int e = 0; e < RC; ++e) val[e] = *reinterpret_cast<const float2 *>(lds.tile + (q * RC + e) * SCAN_TS + 2 * c);
        // Reverse: the saved states pass through this launch exactly once, so their largest magnitude is
        // recorded on the way: dy^T x, in the next launch, stages x under that scale (x0 is not part of x)
        if constexpr (REV) {
            xmax = fmaxf(fabsf(saved.xl.x), fabsf(saved.xl.y));
#pragma unroll
            for (int e = 0; e < RC; ++e)
                if (t0 + e > 0) xmax = fmaxf(xmax, fmaxf(fabsf(saved.xp[e].x), fabsf(saved.xp[e].y)));
        }
        fmask = masks.x; rmask = masks.y;
        // pass 1: state after the thread's steps for zero incoming state (a reset zeroes the multiplier)
#pragma unroll
        for (int i = 0; i < RC; ++i) {
            const int e = REV ? RC - 1 - i : i;
            const bool r = (rmask >> e) & 1u;
            const float2 le = make_float2(r ? 0.f : lam.x, r ? 0.f : lam.y);
            S = cfma(le, S, val[e]);
        }
        lrc = cmul(lam, lam);                                // Abar^16 by four squarings
        lrc = cmul(lrc, lrc); lrc = cmul(lrc, lrc); lrc = cmul(lrc, lrc);
        l128 = cmul(lrc, lrc);                               // Abar^128 by three more
        l128 = cmul(l128, l128); l128 = cmul(l128, l128);
        lds.cS[ql * 64 + c] = S;
        lds.cAny[ql * 64 + c] = rmask != 0;
    }
    __syncthreads();                                         // the chunk states are in LDS
    if constexpr (ACTIVE) {
        // exclusive combine over the chunks of the same sequence that come earlier in scan order
        const int before = whole_seqs ? (REV ? (a.L - RC - t0) / RC : t0 / RC) : ql;
        const int ql_first = ql - before;
        // (all chunk states are read first, whether this thread folds them or not: left inside the
        // condition below, the reads end up in its branch and a thread waits for LDS once per chunk
        // it folds, the last chunk's wavefront seven times in a row, and the tile's aggregate goes out late)
        float2 Sc[NCH - 1];
        unsigned Rc[NCH - 1];
#pragma unroll
        for (int j = 0; j < NCH - 1; ++j) {
            Sc[j] = lds.cS[j * 64 + c];
            Rc[j] = lds.cAny[j * 64 + c];
            asm volatile("" : "+v"(Sc[j].x), "+v"(Sc[j].y), "+v"(Rc[j]));
        }
#pragma unroll
        for (int j = 0; j < NCH - 1; ++j) {
            const float2 Aj = Rc[j] ? make_float2(0.f, 0.f) : lrc;
            const float2 nS = cfma(Aj, Sex, Sc[j]), nA = cmul(Aj, Aex);
            const bool take = j >= ql_first && j < ql;
            Sex = make_float2(take ? nS.x : Sex.x, take ? nS.y : Sex.y);
            Aex = make_float2(take ? nA.x : Aex.x, take ? nA.y : Aex.y);
        }
        if (leader) {
            // the tile's aggregate goes out before anything is waited for
            const bool has_succ = REV ? (tmL > 0) : (tmL + 1 < nt);
            const float2 Ath = (rmask != 0) ? make_float2(0.f, 0.f) : lrc;
            const float2 Stile = cfma(Ath, Sex, S);
            const bool any_tile = (rmask != 0) || (Aex.x == 0.f && Aex.y == 0.f);
            if (active && has_succ) {
                unsigned long long *mine = a.desc + ((size_t)tile * 64 + c) * 2;
                publish_word(mine, Stile.x, any_tile ? 2u : 1u);
                publish_word(mine + 1, Stile.y, any_tile ? 2u : 1u);
            }
            if (!REV && a.x0 && active) X = a.x0[(long)b * a.P + p];
        }
    }
    // The aggregates of the earlier tiles of the chain, eight at a time in scan order (the k-th predecessor
    // = tile k of the sequence forward, tile nt-1-k in reverse): wavefront q fetches predecessor k0 + q, the
    // leader folds the batch over the incoming state.  One canonical order, whatever the timing.
    for (int k0 = 0; k0 < npred; k0 += NCH) {
        if constexpr (ACTIVE) {
            const int k = k0 + q;
            if (k < npred) {
                float2 Sj = make_float2(0.f, 0.f);
                unsigned tag = 2;
                if (active) {
                    const int j = REV ? nt - 1 - k : k;
                    const size_t ptile = (size_t)(b * nt + j) * g.ntn + tn;
                    if (!wait_pair(a.desc + (ptile * 64 + c) * 2, 1u, a.spin_limit, Sj, tag)) {
                        // gave up: flag it, hand on NaN (every state that depends on the missing aggregate
                        // becomes NaN, so the failure cannot pass as data) and finish anyway
                        atomicOr(a.err, 1u);
                        Sj = make_float2(__builtin_nanf(""), __builtin_nanf("")); tag = 2;
                    }
                }
                lds.pS[q * 64 + c] = Sj;
                lds.pAny[q * 64 + c] = (tag == 2u);
            }
        }
        __syncthreads();                                     // the batch is in LDS
        if constexpr (ACTIVE) {
            if (leader) {
                const int n = min(NCH, npred - k0);
                for (int j = 0; j < n; ++j) {
                    const float2 Aj = lds.pAny[j * 64 + c] ? make_float2(0.f, 0.f) : l128;
                    X = cfma(Aj, X, lds.pS[j * 64 + c]);
                }
            }
        }
        if (k0 + NCH < npred) __syncthreads();               // the next batch may overwrite the slots
    }
    if constexpr (ACTIVE) {
        if (leader) lds.sX[c] = X;
    }
    __syncthreads();                                         // the incoming state of the tile is in LDS
    unsigned rm[RC];                                         // largest magnitude per step (row of the tile), for rowmax_out
    float2 acc = make_float2(0.f, 0.f);
    if constexpr (ACTIVE) {
        // pass 2: the states themselves
        float2 Xin = lds.sX[c];
        if (whole_seqs) Xin = (!REV && a.x0 && active) ? a.x0[(long)b * a.P + p] : make_float2(0.f, 0.f);
        float2 xs = cfma(Aex, Xin, Sex);
        float2 *dst = reinterpret_cast<float2 *>(g.C) + (long)row0 * a.P + p;
        if (!REV) {
#pragma unroll
            for (int e = 0; e < RC; ++e) {
                const bool r = (rmask >> e) & 1u;
                const float2 le = make_float2(r ? 0.f : lam.x, r ? 0.f : lam.y);
                xs = cfma(le, xs, val[e]);
                if (active) dst[(long)e * a.P] = xs;
                const float me = fmaxf(fabsf(xs.x), fabsf(xs.y));
                rm[e] = active ? __float_as_uint(me) : 0u;
                amax = fmaxf(amax, me);
            }
            if (active && a.x_last && t0 + RC == a.L) a.x_last[(long)b * a.P + p] = xs;
        } else {
            if constexpr (REREAD) {
                // (kept in registers across the wait for the predecessors, the values would crowd out the saved
                // states: 193 spilled registers instead of 66 within a budget of 128)
#pragma unroll
                for (int e = 0; e < RC; ++e) {
                    val[e] = *reinterpret_cast<const float2 *>(lds.tile + (q * RC + e) * SCAN_TS + 2 * c);
                    asm volatile("" : "+v"(val[e].x), "+v"(val[e].y));
                }
            }
            // also dAbar += [not is_first_t] conj(x_{t-1}) chi_t
#pragma unroll
            for (int e = RC - 1; e >= 0; --e) {
                const bool r = (rmask >> e) & 1u;
                const float2 le = make_float2(r ? 0.f : lam.x, r ? 0.f : lam.y);
                xs = cfma(le, xs, val[e]);
                if (active) dst[(long)e * a.P] = xs;
                const float me = fmaxf(fabsf(xs.x), fabsf(xs.y));
                rm[e] = active ? __float_as_uint(me) : 0u;
                amax = fmaxf(amax, me);
                const bool m = (fmask >> e) & 1u;
                const float2 qv = make_float2(m ? 0.f : saved.xp[e].x, m ? 0.f : saved.xp[e].y);
                acc.x = fmaf(qv.x, xs.x, fmaf(qv.y, xs.y, acc.x));
                acc.y = fmaf(qv.x, xs.y, fmaf(-qv.y, xs.x, acc.y));
            }
            // lam holds conj(Abar) here: dx0 = [not is_first_0] conj(Abar) chi_0
            if (active && a.dx0 && t0 == 0) a.dx0[(long)b * a.P + p] = (fmask & 1u) ? make_float2(0.f, 0.f) : cmul(lam, xs);
            lds.cS[q * 64 + c] = acc;                      // (every reader of cS is behind the barriers above)
        }
    }
    if (REV) {
        __syncthreads();                                     // the chunks' contributions to dAbar are in LDS
        if constexpr (ACTIVE) {
            if (q == 0 && active) {
                float2 sum = make_float2(0.f, 0.f);
                for (int j = 0; j < NCH; ++j) { sum.x += lds.cS[j * 64 + c].x; sum.y += lds.cS[j * 64 + c].y; }
                a.partial[(size_t)(m0 / SCAN_TILE) * a.P + p] = sum;
            }
        }
    }
    if constexpr (ACTIVE) {
        if (a.rowmax_out) {
            // largest magnitude of every row within this column tile, stored as [column tile][row] (the consumer
            // of C takes the maximum over the column tiles): lane l < 16 ends up with the row rows16_index(l) of
            // the thread's 16
            const unsigned r = rows16_wave_max(rm, c);
            if (c < RC) a.rowmax_out[(size_t)tn * g.M + row0 + rows16_index(c)] = r;
        }
    }
    if (a.amax_out) {
        // one atomic per workgroup, spread over ABSMAX_SLOTS addresses (the bit patterns of non-negative
        // floats order like unsigned integers); cAny is free since the incoming state was published
        unsigned v = active ? __float_as_uint(amax) : 0u, vx = active ? __float_as_uint(xmax) : 0u;
        if constexpr (ACTIVE) {
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                v = max(v, (unsigned)__shfl_xor((int)v, o));
                if (REV) vx = max(vx, (unsigned)__shfl_xor((int)vx, o));
            }
            if (c == 0) { lds.cAny[q] = v; lds.cAny[NCH + q] = vx; }
        }
        __syncthreads();                                     // the wavefronts' maxima are in LDS
        if constexpr (ACTIVE) {
            if (tid == 0) {
                for (int j = 1; j < NCH; ++j) { v = max(v, lds.cAny[j]); vx = max(vx, lds.cAny[NCH + j]); }
                atomicMax(a.amax_out + (unsigned)tile % ABSMAX_SLOTS, v);
                if (REV && a.xmax_out) atomicMax(a.xmax_out + (unsigned)tile % ABSMAX_SLOTS, vx);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Wavefront specialisation: a workgroup has WGM*WGN consumer wavefronts that only read
// operand fragments from LDS and issue MFMAs, and NP producer wavefronts that only stage tiles
// (global load -> three-way split -> LDS).  A producer and a consumer share each SIMD, so the
// VALU work of the split co-executes with the matrix instructions of the other wavefront.
// LDS holds NS stages; in iteration kt the producers fill the stage of tile kt+NS-1 while the
// consumers work on tile kt, with one workgroup barrier per K tile.
// ---------------------------------------------------------------------------------------------
template <int BM, int BN, int BK, int WGM, int WGN, int NP, int NS, int NPL, bool AKC, bool BKC, int EPI, int FAST>
__device__ __forceinline__ void gemm_ws_tile(const GemmDev &g, __bf16 *smem, int m0, int n0, int z,
                                                    int kbeg, int kend, int scan_tile)
{
    constexpr int NC = WGM * WGN;                 // consumer wavefronts
    constexpr bool SAVED_EARLY = NP >= 8;         // one workgroup per CU: registers to spare during the K loop
    constexpr int PF = 2;                         // K tiles of global loads in flight per producer
                                                  // (3, 4 and 6 measured: 1-5 % slower)
    constexpr int PT = 64 * NP;                   // producer threads
    using LA = SplitLoader<BM, BK, AKC, PT, NPL>;
    using LB = SplitLoader<BN, BK, BKC, PT, NPL>;
    static_assert(NPL == 2 || NPL == 3, "three bf16 planes or two scaled fp16 planes per operand");
    constexpr int STAGE_A = NPL * LA::PLANE, STAGE_B = NPL * LB::PLANE, STAGE = STAGE_A + STAGE_B;
    // two-plane staging: log2 of the scale of every row of the A tile (index r < BM) and of B (index BM),
    // written by the producers before the first barrier and read by the consumers after the K loop.
    // They live in the padding of the first A plane of stage 0 (the 16 or 32 bytes behind every row that
    // no staging store and no fragment read touches), so that the stages alone are the LDS footprint
    // (2 x 40 KB for a 128 x 128 x 32 tile with two planes: two workgroups fit the 160 KB of a CU).
    __bf16 *stages = smem;
    auto rowexp = [&](int i) -> int & {
        if constexpr (AKC) return *reinterpret_cast<int *>(stages + (i < BM ? i : 0) * LA::S + BK + (i < BM ? 0 : 2));
        else return *reinterpret_cast<int *>(stages + (i / 8) * LA::S + BM + 2 * (i % 8));
    };
    static_assert(AKC || BM / 8 < BK, "the k rows of a row-contiguous A plane must hold BM + 1 scale words in their padding");
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int MI = WM / 32, NI = WN / 32;
    static_assert(MI >= 1 && NI >= 1 && WM % 32 == 0 && WN % 32 == 0 && BK % 16 == 0 && NS >= 2, "bad tile");

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int nk = (kend > kbeg) ? (kend - kbeg + BK - 1) / BK : 0;
    const bool full = (m0 + BM <= g.M) && (n0 + BN <= g.N);      // no store of this tile needs a bounds check

    if (wave >= NC) {
        // ------------------------------------------------------------------ producers
        // PF register sets: while tile t is split and stored, the loads of tiles t+1 .. t+PF are in
        // flight, which covers the global latency with PF K tiles of matrix work.
        const int ptid = tid - 64 * NC;
        LA la[PF];
        LB lb[PF];
        auto fetch = [&](int set, int t) {
            la[set].template load<FAST>(g.A, g.lda, m0, g.M, kbeg + t * BK, kend, ptid);
            lb[set].template load<FAST>(g.B, g.ldb, n0, g.N, kbeg + t * BK, kend, ptid);
        };
        float sca[LA::NV], scb[LB::NV];
#pragma unroll
        for (int i = 0; i < LA::NV; ++i) sca[i] = 1.f;
#pragma unroll
        for (int i = 0; i < LB::NV; ++i) scb[i] = 1.f;
        // Two-plane staging: log2 of the scales goes through LDS (rowexp(r), r < BM: row r of the A tile;
        // rowexp(BM): B).  The first producer wavefront reduces the one-per-matrix maxima, the first BM
        // producer threads the per-row ones of A; their loads are issued ahead of the tile loads, so they
        // return first and are waited for with tile 0.
        AbsMaxLoads ma, mb, mr;
        const bool arows = NPL == 2 && AKC && g.amaxA.rows != nullptr;      // every row of A has its own scale
        if constexpr (NPL == 2) {
            if (wave == NC) {
                mb = absmax_issue(g.amaxB, tid & 63);
                if (!arows) ma = absmax_issue(g.amaxA, tid & 63);
            }
            if (arows && ptid < BM) mr = absmax_row_issue(g.amaxA, min(m0 + ptid, g.M - 1));
        }
        auto stash = [&](int set, int t) {
            __bf16 *st = stages + (t % NS) * STAGE;
            la[set].store(st, ptid, sca);
            lb[set].store(st + STAGE_A, ptid, scb);
        };
#pragma unroll
        for (int j = 0; j < PF; ++j)
            if (j < nk) fetch(j, j);
        if constexpr (NPL == 2) {
            if (wave == NC) {
                const int e = absmax_log2_scale(g.amaxB, mb, tid & 63);
                if ((tid & 63) == 0) rowexp(BM) = e;
                if (!arows) {
                    const int ea = absmax_log2_scale(g.amaxA, ma, tid & 63);
                    for (int r = tid & 63; r < BM; r += 64) rowexp(r) = ea;
                }
            }
            if (arows && ptid < BM) rowexp(ptid) = absmax_row_log2_scale(g.amaxA, mr, min(m0 + ptid, g.M - 1));
            __syncthreads();                      // (the consumers wait here as well)
            const float sb = pow2f(rowexp(BM));
#pragma unroll
            for (int i = 0; i < LB::NV; ++i) scb[i] = sb;
#pragma unroll
            for (int i = 0; i < LA::NV; ++i) sca[i] = pow2f(rowexp(AKC ? LA::unit_row(ptid, i) : 0));
        }
        // the scanning producers of the reverse scan ask for their saved states behind the first tile loads
        // (with two workgroups per CU the 34 registers are not there: then behind the K loop)
        ScanSaved saved;
        uint2 masks = make_uint2(0u, 0u);
        if constexpr (EPI == 7 || EPI == 8) {
            if (wave < SCAN_WAVES) masks = scan_flag_masks<EPI == 8>(g.scan, tid, m0);
        }
        if constexpr (EPI == 8 && SAVED_EARLY) {
            if (wave < SCAN_WAVES) saved = scan_request_saved(g.scan, tid, m0, n0);
        }
        // prologue: tiles 0 .. NS-2 into their stages
#pragma unroll
        for (int t = 0; t < NS - 1; ++t) {
            if (t < nk) {
                stash(t % PF, t);
                if (t + PF < nk) fetch(t % PF, t + PF);
            }
        }
        __syncthreads();
        // steady state: iteration kt stages tile t = kt + NS - 1 from register set t % PF (kt is a
        // multiple of PF at the top of the unrolled body, so the set index is a constant there)
        for (int kt = 0; kt < nk; kt += PF) {
#pragma unroll
            for (int j = 0; j < PF; ++j) {
                if (kt + j < nk) {
                    const int t = kt + j + NS - 1;
                    if (t < nk) {
                        stash((j + NS - 1) % PF, t);
                        if (t + PF < nk) fetch((j + NS - 1) % PF, t + PF);
                    }
                    __syncthreads();
                }
            }
        }
        if constexpr (EPI == 7 || EPI == 8) {
            static_assert(EPI < 7 || (NC + NP >= SCAN_WAVES && NC <= SCAN_WAVES), "wavefronts of the scan epilogue");
            if constexpr (EPI == 8 && !SAVED_EARLY) {
                if (wave < SCAN_WAVES) saved = scan_request_saved(g.scan, tid, m0, n0);
            }
            if (wave < SCAN_WAVES) {
                // the first producers scan with the consumers: barriers 1 and 2 frame the staging of the tile
                __syncthreads();
                __syncthreads();
                scan_epilogue_body<EPI == 8, false, EPI == 8 && !SAVED_EARLY>(g, ScanLds(smem), tid, m0, n0, scan_tile, saved, masks);
            } else {
                __syncthreads();
                __syncthreads();
                scan_epilogue_body<EPI == 8, true, EPI == 8 && !SAVED_EARLY>(g, ScanLds(smem), tid, m0, n0, scan_tile, saved, masks);
            }
        }
        return;
    }

    // ---------------------------------------------------------------------- consumers
    const int l = tid & 63;
    const int wm = wave / WGN, wn = wave % WGN;
    const int li = l & 31, hh = l >> 5;
    v16f acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // Software pipeline over the 16-wide k steps: the fragments of step s+1 are requested from LDS
    // before the 6*MI*NI matrix instructions of step s are issued, so the LDS latency (there is no
    // second consumer wavefront on the SIMD to hide it) overlaps with matrix work.  At the last
    // step of a K tile the workgroup barrier comes first: it both releases the stage just read
    // (all its reads have completed, they feed the instructions about to be issued) and
    // guarantees that the next stage is filled.
    constexpr int KS = BK / 16;
    bf16x8 fa[2][MI][NPL], fb[2][NI][NPL];
    auto fetch_frags = [&](int set, int kt, int ks) {
        const __bf16 *st = stages + (kt % NS) * STAGE;
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int s = 0; s < NPL; ++s)
                fa[set][i][s] = LA::fragment(st + s * LA::PLANE, wm * WM + i * 32, ks * 16, l);
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int s = 0; s < NPL; ++s)
                fb[set][j][s] = LB::fragment(st + STAGE_A + s * LB::PLANE, wn * WN + j * 32, ks * 16, l);
    };
    // the six products of one accumulator keep their order (smallest first); the MI*NI
    // accumulators alternate so that consecutive matrix instructions are independent
    auto multiply = [&](int set) {
        // three planes: a3b1, a2b2, a1b3, a2b1, a1b2, a1b1;  two planes: a2b1, a1b2, a1b1
        constexpr int NPROD = NPL == 3 ? 6 : 3;
        constexpr int PA3[6] = {2, 1, 0, 1, 0, 0}, PB3[6] = {0, 1, 2, 0, 1, 0};
        constexpr int PA2[3] = {1, 0, 0}, PB2[3] = {0, 1, 0};
#pragma unroll
        for (int p = 0; p < NPROD; ++p)
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    const int pa = NPL == 3 ? PA3[p] : PA2[p % 3], pb = NPL == 3 ? PB3[p] : PB2[p % 3];
                    if constexpr (NPL == 3)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][i][pa], fb[set][j][pb], acc[i][j], 0, 0, 0);
                    else
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, fa[set][i][pa]),
                                                                           __builtin_bit_cast(f16x8, fb[set][j][pb]), acc[i][j], 0, 0, 0);
                }
    };
    static_assert(KS % 2 == 0 || KS == 1, "k steps per tile: 1 or even");
    // issue order of one k step: a fragment read in the shadow of every second matrix
    // instruction (a burst of reads would keep the wavefront from issuing matrix work)
    auto interleave = [&]() {
        constexpr int NREAD = NPL * (MI * (AKC ? 1 : 2) + NI * (BKC ? 1 : 2)), NMFMA = (NPL == 3 ? 6 : 3) * MI * NI;
#pragma unroll
        for (int q = 0; q < NREAD; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x008, NMFMA / NREAD > 0 ? NMFMA / NREAD : 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
    };

    ScanSaved saved;
    uint2 masks = make_uint2(0u, 0u);
    if constexpr (EPI == 7 || EPI == 8) masks = scan_flag_masks<EPI == 8>(g.scan, tid, m0);     // (see the producers)
    if constexpr (EPI == 8 && SAVED_EARLY) saved = scan_request_saved(g.scan, tid, m0, n0);
    if constexpr (NPL == 2) __syncthreads();      // the producers have put log2 of the scales into rowexp
    __syncthreads();
    if (nk > 0) fetch_frags(0, 0, 0);
    if (KS == 1) {
        // one k step per tile: the register set alternates with the tile
        int kt = 0;
        for (; kt + 1 < nk; kt += 2) {
            __syncthreads();
            fetch_frags(1, kt + 1, 0);
            __builtin_amdgcn_sched_barrier(0);
            multiply(0);
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
            if (kt + 2 < nk) fetch_frags(0, kt + 2, 0);
            __builtin_amdgcn_sched_barrier(0);
            multiply(1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (kt < nk) {
            __syncthreads();
            multiply(0);
        }
    } else {
        for (int kt = 0; kt < nk; ++kt) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (ks + 1 < KS) {
                    fetch_frags((ks + 1) & 1, kt, ks + 1);
                } else {
                    __syncthreads();
                    fetch_frags(0, kt + 1, 0);   // past the last tile: a harmless read of a stale stage
                }
                multiply(ks & 1);
                interleave();
            }
        }
    }

    if constexpr (NPL == 2) {
        // the power of two that takes both operand scales off again (their sum can leave the exponent range of
        // a single factor: one exponent adjustment per element, exact like a multiplication by the power)
        const int eb = rowexp(BM);
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int st = rowexp(wm * WM + i * 32 + 8 * (r / 4) + 4 * hh + (r % 4)) + eb;
#pragma unroll
                for (int j = 0; j < NI; ++j) acc[i][j][r] = __builtin_ldexpf(acc[i][j][r], -st);
            }
    }
    if constexpr (EPI == 7 || EPI == 8) {
        static_assert(BM == SCAN_TILE && BN == SCAN_TILE && NC == 4, "scan epilogue: 128x128 tile, 4 consumers");
        const ScanLds lds(smem);
        if constexpr (EPI == 8 && !SAVED_EARLY) saved = scan_request_saved(g.scan, tid, m0, n0);
        __syncthreads();                             // barrier 1: every wavefront has left the K loop, LDS is free
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    lds.tile[(wm * WM + i * 32 + 8 * (r / 4) + 4 * hh + (r % 4)) * SCAN_TS + wn * WN + j * 32 + li] = acc[i][j][r];
        __syncthreads();                             // barrier 2: the tile is staged
        scan_epilogue_body<EPI == 8, false, EPI == 8 && !SAVED_EARLY>(g, lds, tid, m0, n0, scan_tile, saved, masks);
        return;
    }
    float *Cz = g.C + (long)z * g.M * g.ldc;
    if constexpr (EPI == 1 || EPI == 6) {
        // sum + diag (.) E: the 16 values of E that a 32x32 block needs are loaded before its first store
        // (the compiler may not move a load of E above an earlier store to C, so a load-compute-store loop
        // would pay one memory latency per element); the scheduling barrier keeps the loads of the next
        // block from being hoisted as well, which would not fit the register budget
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            unsigned rowmax = 0u;                        // EPI 6: largest |GELU(y)| of row rows16_half_index(l) so far
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                unsigned gmax[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) gmax[r] = 0u;
                const int col = n0 + wn * WN + j * 32 + li;
                const long rbase = m0 + wm * WM + i * 32 + 4 * hh;
                float e[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const long row = rbase + 8 * (r / 4) + (r % 4);
                    e[r] = (full || (row < g.M && col < g.N)) ? g.E[row * g.lde + col] : 0.f;
                }
                const float dcol = (full || col < g.N) ? g.diag[col] : 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const long row = rbase + 8 * (r / 4) + (r % 4);
                    if (full || (row < g.M && col < g.N)) {
                        const float y = fmaf(dcol, e[r], acc[i][j][r]);
                        Cz[row * g.ldc + col] = y;
                        if constexpr (EPI == 6) {
                            const float gy = gelu_value(y);
                            g.C2[row * g.ldc + col] = gy;
                            gmax[r] = __float_as_uint(fabsf(gy));
                        }
                    }
                }
                // (reduced block by block: sixteen values per thread alive for one block only)
                if constexpr (EPI == 6 && WN == 64) {
                    if (g.c2_rowmax) rowmax = max(rowmax, rows16_half_max(gmax, l));
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (EPI == 6 && WN == 64) {
                // the product that consumes C2 stages its rows under a scale each: the largest magnitude of
                // every row within this wavefront's 64 columns, as [piece of 64 columns][row]
                if (g.c2_rowmax) {
                    const unsigned m = rowmax;
                    const int r = rows16_half_index(l);
                    const long row = m0 + wm * WM + i * 32 + 4 * hh + 8 * (r / 4) + (r % 4);
                    // (a wavefront whose 64 columns lie past N entirely has no piece: the last column tile of a
                    // width that is an odd multiple of 64)
                    if ((l & 16) == 0 && row < g.M && n0 + wn * WN < g.N) g.c2_rowmax[(size_t)((n0 + wn * WN) / 64) * g.M + row] = m;
                }
            }
        }
        return;
    }
    if constexpr (EPI == 3) {
        // half-GLU gate: the same order
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int col = n0 + wn * WN + j * 32 + li;
                const long rbase = m0 + wm * WM + i * 32 + 4 * hh;
                float e[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const long row = rbase + 8 * (r / 4) + (r % 4);
                    e[r] = (full || (row < g.M && col < g.N)) ? g.E[row * g.lde + col] : 0.f;
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const long row = rbase + 8 * (r / 4) + (r % 4);
                    if (full || (row < g.M && col < g.N)) {
                        const float sg = sigmoidf(acc[i][j][r]);
                        if (g.C2) g.C2[row * g.ldc + col] = sg;
                        Cz[row * g.ldc + col] = e[r] * sg;
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        return;
    }
    if constexpr (EPI == 4) {
        // adjoint of the gate, E + acc (.) E2: the inputs of a 32x32 block first, as above
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int col = n0 + wn * WN + j * 32 + li;
                const long rbase = m0 + wm * WM + i * 32 + 4 * hh;
                float e[16], e2[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const long row = rbase + 8 * (r / 4) + (r % 4);
                    const bool inb = full || (row < g.M && col < g.N);
                    e[r] = inb ? g.E[row * g.lde + col] : 0.f;
                    e2[r] = inb ? g.E2[row * g.lde + col] : 0.f;
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const long row = rbase + 8 * (r / 4) + (r % 4);
                    if (full || (row < g.M && col < g.N)) Cz[row * g.ldc + col] = fmaf(acc[i][j][r], e2[r], e[r]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        return;
    }
    if constexpr (EPI == 2 || EPI == 5) {
        // one recurrence step and its adjoint (columns are (re, im) pairs, the partner column lives in the
        // neighbouring lane): the same block-wise order, inputs of a block first
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int col = n0 + wn * WN + j * 32 + li;
                const long rbase = m0 + wm * WM + i * 32 + 4 * hh;
                const bool colok = full || col < g.N;
                float e[16];
                bool dropped[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const long row = rbase + 8 * (r / 4) + (r % 4);
                    const bool inb = colok && (full || row < g.M);
                    e[r] = (inb && (EPI == 2 || g.E)) ? g.E[row * g.lde + col] : 0.f;
                    dropped[r] = inb && g.rowflag && g.rowflag[row];
                }
                const bool has_diag = EPI == 2 || g.C2;
                const float lr = (colok && has_diag) ? g.diag[col & ~1] : 0.f, li_ = (colok && has_diag) ? g.diag[col | 1] : 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const long row = rbase + 8 * (r / 4) + (r % 4);
                    const bool inb = colok && (full || row < g.M);
                    if constexpr (EPI == 2) {
                        // the carried state Abar x_{t-1} of the step, unless the step resets
                        const float own = e[r], other = __shfl_xor(own, 1);
                        const float carried = (col & 1) ? fmaf(lr, own, li_ * other) : fmaf(lr, own, -li_ * other);
                        if (inb) Cz[row * g.ldc + col] = dropped[r] ? acc[i][j][r] : acc[i][j][r] + carried;
                    } else {
                        const float v = acc[i][j][r] + e[r];
                        const float other = __shfl_xor(v, 1);
                        if (inb) {
                            Cz[row * g.ldc + col] = v;
                            if (g.C2)
                                g.C2[row * g.ldc + col] = dropped[r] ? 0.f : ((col & 1) ? fmaf(lr, v, -li_ * other) : fmaf(lr, v, li_ * other));
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        return;
    }
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int col = n0 + wn * WN + j * 32 + li;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const long row = m0 + wm * WM + i * 32 + 8 * (r / 4) + 4 * hh + (r % 4);
                const bool inb = full || (row < g.M && col < g.N);
                if constexpr (EPI == 5) {
                    // the partner column (col ^ 1) of a complex pair lives in the neighbouring lane
                    float v = acc[i][j][r];
                    if (inb && g.E) v += g.E[row * g.lde + col];
                    const float other = __shfl_xor(v, 1);
                    if (inb) {
                        Cz[row * g.ldc + col] = v;
                        if (g.C2) g.C2[row * g.ldc + col] = gemm_carry_adjoint(g, row, col, v, other);
                    }
                } else {
                    if (inb) Cz[row * g.ldc + col] = gemm_epilogue_apply<EPI>(g, row, col, acc[i][j][r]);
                }
            }
        }
}

// Operand layouts and epilogue of one problem, packed into one template argument.
constexpr int gemm_layout(bool akc, bool bkc, int epi) { return (akc ? 1 : 0) | (bkc ? 2 : 0) | (epi << 2); }

// Halves of LDS one stage of a problem needs (the planes of both operands; see SplitLoader).
constexpr size_t gemm_stage_halves(int BM, int BN, int BK, int NPL, int lay)
{
    const size_t pa = (lay & 1) ? (size_t)BM * (BK + 8) : (size_t)BK * (BM + 16);
    const size_t pb = (lay & 2) ? (size_t)BN * (BK + 8) : (size_t)BK * (BN + 16);
    return (size_t)NPL * (pa + pb);
}

// Work item (tile, split) of the workgroup in slot q of XCD x.  Workgroup ids are dealt
// round-robin to the 8 XCDs (id % 8), each with its own L2:
//   mode 0 (no K splits): XCD x owns the contiguous band of tiles [x*nx, (x+1)*nx), so it re-reads
//          only its band of A from its own L2;
//   modes 1-3 (K splits): every XCD owns whole K slabs (or, with fewer than 8 splits, one
//          contiguous band of the tiles of one slab), so each operand element is fetched from
//          memory once instead of once per tile band;
//   mode 5: see below.
__device__ __forceinline__ void gemm_place(const GemmDev &g, int x, int q, int &z, int &tile)
{
    if (g.mode == 0) { z = 0; tile = x * g.nx + q; }
    else if (g.mode == 1) { z = x + 8 * (q % g.mpar); tile = q / g.mpar; }        // splits = 8 * mpar
    else if (g.mode == 2) { z = x % g.splits; tile = (x / g.splits) * g.nx + q; } // 8 = splits * mpar: bands of nx tiles
    else if (g.mode == 3) { const int item = x * g.nx + q; z = item / (g.ntm * g.ntn); tile = item % (g.ntm * g.ntn); }
    else {
        // mode 5 (scan epilogue): a unit = the tiles of one sequence and column group, time-major;
        // units are dealt to the XCDs, so a tile only ever waits for tiles in earlier slots of its
        // own XCD, which were dispatched before it
        const int per_unit = g.sc_nt * g.sc_cpu;
        const int uid = x + 8 * (q / per_unit), r = q % per_unit;
        const int b = uid / g.sc_ncg, cg = uid % g.sc_ncg;
        const int tn = cg * g.sc_cpu + r % g.sc_cpu;
        z = 0;
        const int tslot = r / g.sc_cpu;                 // time-ordered slot; the reverse scan starts at the sequence end
        const int tmL = g.sc_rev ? g.sc_nt - 1 - tslot : tslot;
        tile = (uid < g.sc_units && tn < g.ntn) ? (b * g.sc_nt + tmL) * g.ntn + tn : g.ntm * g.ntn;
    }
}

template <int BM, int BN, int BK, int WGM, int WGN, int NP, int NS, int NPL, int LAY>
__device__ __forceinline__ void gemm_ws_problem(const GemmDev &g, __bf16 *smem, int x, int q)
{
    constexpr bool AKC = (LAY & 1) != 0, BKC = (LAY & 2) != 0;
    constexpr int EPI = LAY >> 2;
    int z, tile;
    gemm_place(g, x, q, z, tile);
    if (q >= g.nx || z >= g.splits || tile >= g.ntm * g.ntn) return;
    const int tm = tile / g.ntn, tn = tile % g.ntn;
    const int m0 = tm * BM, n0 = tn * BN;
    const int kbeg = z * g.kper;
    const int kend = min(g.K, kbeg + g.kper);
    // 16-byte loads of both operands: aligned sources, whole K tiles, and whole tiles along the rows of an
    // operand whose rows are contiguous in memory (a k-contiguous operand may hang over its last row)
    const bool fast = (g.lda % 4 == 0) && ((reinterpret_cast<uintptr_t>(g.A) & 15) == 0) &&
                      (g.ldb % 4 == 0) && ((reinterpret_cast<uintptr_t>(g.B) & 15) == 0) &&
                      (AKC || m0 + BM <= g.M) && (BKC || n0 + BN <= g.N) && ((kend - kbeg) % BK == 0);
    const bool inside = (m0 + BM <= g.M) && (n0 + BN <= g.N);
    if (fast && inside)
        gemm_ws_tile<BM, BN, BK, WGM, WGN, NP, NS, NPL, AKC, BKC, EPI, 1>(g, smem, m0, n0, z, kbeg, kend, tile);
    else if (fast && (AKC || BKC))
        gemm_ws_tile<BM, BN, BK, WGM, WGN, NP, NS, NPL, AKC, BKC, EPI, 2>(g, smem, m0, n0, z, kbeg, kend, tile);
    else
        gemm_ws_tile<BM, BN, BK, WGM, WGN, NP, NS, NPL, AKC, BKC, EPI, 0>(g, smem, m0, n0, z, kbeg, kend, tile);
}

// One launch carries one problem (LAY1 < 0), two, or three independent ones (the third has the layout
// of the second; it is absent when its slot count is zero).  Used for the gradient pass, where several
// products have their inputs ready at the same time and one of them alone would leave compute units
// idle.  Every problem owns a contiguous range of the slots of every XCD, [slot0, slot0 + nx); the host
// decides the order (work items that should start first get the lowest slots).
template <int BM, int BN, int BK, int WGM, int WGN, int NP, int NS, int NPL, int LAY0, int LAY1, int WPE>
__global__ void __launch_bounds__(64 * (WGM * WGN + NP), WPE) gemm_ws_kernel(GemmDev g0, GemmDev g1, GemmDev g2)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    __bf16 *smem = reinterpret_cast<__bf16 *>(smem_raw);
    const int x = blockIdx.x % 8, q = blockIdx.x / 8;
    if (LAY1 < 0 || (q >= g0.slot0 && q < g0.slot0 + g0.nx)) {
        gemm_ws_problem<BM, BN, BK, WGM, WGN, NP, NS, NPL, LAY0>(g0, smem, x, q - g0.slot0);
    } else if (q >= g1.slot0 && q < g1.slot0 + g1.nx) {
        gemm_ws_problem<BM, BN, BK, WGM, WGN, NP, NS, NPL, (LAY1 < 0 ? LAY0 : LAY1)>(g1, smem, x, q - g1.slot0);
    } else {
        // (a branch of its own: choosing between the two argument structs at run time would put them on the stack)
        gemm_ws_problem<BM, BN, BK, WGM, WGN, NP, NS, NPL, (LAY1 < 0 ? LAY0 : LAY1)>(g2, smem, x, q - g2.slot0);
    }
}

template <int BM, int BN, int BK>
inline GemmDev make_gemm_dev(const GemmArgs &a)
{
    GemmDev g;
    g.A = a.A; g.lda = a.lda; g.B = a.B; g.ldb = a.ldb; g.C = a.C; g.ldc = a.ldc;
    g.diag = a.diag; g.E = a.E; g.lde = a.lde; g.rowflag = a.rowflag;
    g.E2 = a.E2; g.C2 = a.C2;
    g.M = a.M; g.N = a.N; g.K = a.K;
    const int splits = a.splits < 1 ? 1 : a.splits;
    int kper = (a.K + splits - 1) / splits;
    kper = (kper + BK - 1) / BK * BK;
    g.kper = kper;
    g.ntm = (a.M + BM - 1) / BM;
    g.ntn = (a.N + BN - 1) / BN;
    const long ntiles = (long)g.ntm * g.ntn;
    g.per_xcd = (int)((ntiles + 7) / 8);
    g.splits = splits;
    g.slot0 = 0;
    if (splits == 1) { g.mode = 0; g.mpar = 0; g.nx = g.per_xcd; }
    else if (splits % 8 == 0) { g.mode = 1; g.mpar = splits / 8; g.nx = (int)(ntiles * g.mpar); }
    else if (8 % splits == 0) { g.mode = 2; g.mpar = 8 / splits; g.nx = (int)((ntiles + g.mpar - 1) / g.mpar); }
    else { g.mode = 3; g.mpar = 0; g.nx = (int)((ntiles * splits + 7) / 8); }
    g.scan = a.scan;
    g.amaxA = a.amaxA; g.amaxB = a.amaxB;
    g.c2_rowmax = a.c2_rowmax;
    g.sc_nt = g.sc_cpu = g.sc_ncg = g.sc_units = g.sc_rev = 0;
    if ((a.epilogue == 7 || a.epilogue == 8) && a.scan.L >= BM) {
        g.sc_rev = a.epilogue == 8;
        const int nseq = a.M / a.scan.L;
        g.sc_nt = a.scan.L / BM;
        int ncg = nseq >= 8 ? 1 : (8 + nseq - 1) / nseq;
        if (ncg > g.ntn) ncg = g.ntn;
        g.sc_ncg = ncg;
        g.sc_cpu = (g.ntn + ncg - 1) / ncg;
        g.sc_units = nseq * ncg;
        g.mode = 5; g.mpar = 0;
        g.nx = ((g.sc_units + 7) / 8) * g.sc_nt * g.sc_cpu;
    }
    return g;
}

// b == nullptr: one problem (LAY1 must be -1).  c (optional, only with b): a third problem with the
// layout of b.  order[i] = which problem (0 = a, 1 = b, 2 = c) takes the i-th range of slots in every
// XCD; nullptr = a, b, c.  WPE: wavefronts per SIMD the register allocation must leave room for (with
// 4 consumer + 4 producer wavefronts and WPE = 4, two workgroups share a CU: one's prologue and stores
// overlap the other's K loop).
template <int BM, int BN, int BK, int WGM, int WGN, int NP, int NS, int NPL, int LAY0, int LAY1 = -1, int WPE = 1>
hipError_t launch_gemm_ws_variant(const GemmArgs &a, hipStream_t s, const GemmArgs *b = nullptr,
                                  const GemmArgs *c = nullptr, const int *order = nullptr)
{
    if ((LAY1 >= 0) != (b != nullptr) || (c && !b)) return hipErrorInvalidValue;
    GemmDev g[3];
    g[0] = make_gemm_dev<BM, BN, BK>(a);
    g[1] = b ? make_gemm_dev<BM, BN, BK>(*b) : g[0];
    g[2] = c ? make_gemm_dev<BM, BN, BK>(*c) : g[0];
    const int nprob = c ? 3 : (b ? 2 : 1);
    if (!b) g[1].nx = 0;
    if (!c) g[2].nx = 0;
    static const int natural[3] = {0, 1, 2};
    const int *ord = order ? order : natural;
    long slots = 0;
    int seen = 0;
    for (int i = 0; i < nprob; ++i) {
        const int k = ord[i];
        if (k < 0 || k >= nprob || (seen & (1 << k))) return hipErrorInvalidValue;
        seen |= 1 << k;
        g[k].slot0 = (int)slots;
        slots += g[k].nx;
    }
    for (int k = nprob; k < 3; ++k) g[k].slot0 = (int)slots;
    constexpr size_t stage0 = gemm_stage_halves(BM, BN, BK, NPL, LAY0), stage1 = LAY1 >= 0 ? gemm_stage_halves(BM, BN, BK, NPL, LAY1) : 0;
    constexpr size_t stage_bytes = (size_t)NS * (stage0 > stage1 ? stage0 : stage1) * sizeof(__bf16);
    constexpr bool scans = ((LAY0 >> 2) >= 7) || (LAY1 >= 0 && (LAY1 >> 2) >= 7);
    constexpr size_t smem = (scans && SCAN_LDS_BYTES > stage_bytes) ? SCAN_LDS_BYTES : stage_bytes;
    static_assert(smem <= 160 * 1024, "tile does not fit the 160 KB LDS of a gfx950 CU");
    auto kern = gemm_ws_kernel<BM, BN, BK, WGM, WGN, NP, NS, NPL, LAY0, LAY1, WPE>;
    if (smem > 64 * 1024) {
        // raising the dynamic LDS limit is idempotent; once per instantiation and device is enough
        // (the attribute belongs to the device's copy of the kernel)
        constexpr int MAXDEV = 64;
        static std::atomic<bool> raised[MAXDEV];
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= MAXDEV || !raised[dev].load(std::memory_order_acquire)) {
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)smem);
            if (e != hipSuccess) return e;
            if (dev >= 0 && dev < MAXDEV) raised[dev].store(true, std::memory_order_release);
        }
    }
    if (slots <= 0 || 8 * slots > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)(8 * slots)), dim3(64 * (WGM * WGN + NP)), smem, s, g[0], g[1], g[2]);
    return hipGetLastError();
}

}  // namespace ssm
