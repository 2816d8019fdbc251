// Parameter-sized kernels: zero-order-hold discretisation with operand packing for the
// projection GEMMs, the column dot product behind dD, and the adjoint of the discretisation.
// The handful of transcendental evaluations per state run in double precision: they are
// P-sized (a few hundred values), and the (exp(z) - 1)/z quotient cancels badly in fp32 for the
// small |Lambda Delta| that slowly decaying states have.
#include "ssm_internal.h"

namespace ssm {

struct Zoh {
    double delta;
    double lr, li;   // Abar = exp(Lambda Delta)
    double gr, gi;   // g = (Abar - 1)/Lambda = Delta * expm1(z)/z
    double zr, zi;   // z = Lambda Delta
};

__device__ __forceinline__ void cdiv(double ar, double ai, double br, double bi, double &qr, double &qi)
{
    const double den = br * br + bi * bi;
    qr = (ar * br + ai * bi) / den;
    qi = (ai * br - ar * bi) / den;
}

__device__ Zoh zoh_discretize(float2 Lambda, float log_delta)
{
    Zoh o;
    o.delta = exp((double)log_delta);
    o.zr = (double)Lambda.x * o.delta;
    o.zi = (double)Lambda.y * o.delta;
    const double ea = exp(o.zr), cb = cos(o.zi), sb = sin(o.zi), sh = sin(0.5 * o.zi);
    o.lr = ea * cb;
    o.li = ea * sb;
    // exp(z) - 1 with the cancellation removed: expm1(a) cos b - 2 sin^2(b/2) + i e^a sin b
    const double er = expm1(o.zr) * cb - 2.0 * sh * sh, ei = ea * sb;
    if (o.zr == 0.0 && o.zi == 0.0) {
        o.gr = o.delta; o.gi = 0.0;
    } else {
        double qr, qi;
        cdiv(er, ei, o.zr, o.zi, qr, qi);
        o.gr = o.delta * qr; o.gi = o.delta * qi;
    }
    return o;
}

// ---------------------------------------------------------------------------------------------
// partial[s][h] = sum_{t in slab s} a[t,h] * b[t,h]      (dD = sum_t dy_t (.) u_t)
// workgroup = 64 columns x 4 row phases
// ---------------------------------------------------------------------------------------------
// maximum of v over the wavefront, valid in lane 63 (data-parallel-primitive moves only: inside quads,
// inside rows of 16 lanes, then the last lane of a row broadcast to the following rows)
__device__ __forceinline__ unsigned wave_max_lane63(unsigned v)
{
    v = max(v, (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, 0xb1, 0xf, 0xf, false));    // quad_perm [1,0,3,2]
    v = max(v, (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x4e, 0xf, 0xf, false));    // quad_perm [2,3,0,1]
    v = max(v, (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x124, 0xf, 0xf, false));   // row_ror:4
    v = max(v, (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x128, 0xf, 0xf, false));   // row_ror:8
    v = max(v, (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x142, 0xa, 0xf, false));   // row_bcast:15 into rows 1, 3
    v = max(v, (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x143, 0xc, 0xf, false));   // row_bcast:31 into rows 2, 3
    return v;
}

// Four values per lane -> lane l < 4 gets the maximum over the wavefront of value 2 (l & 1) + (l >> 1):
// two halving steps inside the quads (lanes that differ in bit 0, then bit 1, swap the half the other
// keeps), rotations inside the rows of 16 lanes, lane swaps across rows: seven moves for four reductions.
__device__ __forceinline__ unsigned wave_max4(unsigned v0, unsigned v1, unsigned v2, unsigned v3, int lane)
{
    const bool up0 = lane & 1, up1 = (lane >> 1) & 1;
    const unsigned k0 = up0 ? v2 : v0, s0 = up0 ? v0 : v2, k1 = up0 ? v3 : v1, s1 = up0 ? v1 : v3;
    const unsigned w0 = max(k0, (unsigned)__builtin_amdgcn_update_dpp((int)s0, (int)s0, 0xb1, 0xf, 0xf, false));
    const unsigned w1 = max(k1, (unsigned)__builtin_amdgcn_update_dpp((int)s1, (int)s1, 0xb1, 0xf, 0xf, false));
    const unsigned k = up1 ? w1 : w0, sd = up1 ? w0 : w1;
    unsigned v = max(k, (unsigned)__builtin_amdgcn_update_dpp((int)sd, (int)sd, 0x4e, 0xf, 0xf, false));
    v = max(v, (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x124, 0xf, 0xf, false));   // row_ror:4
    v = max(v, (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x128, 0xf, 0xf, false));   // row_ror:8
    const auto r16 = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    v = max((unsigned)r16[0], (unsigned)r16[1]);
    const auto r32 = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return max((unsigned)r32[0], (unsigned)r32[1]);
}

// largest bit pattern of the non-negative floats v of a 256-thread workgroup, valid in thread 0
__device__ __forceinline__ unsigned block_absmax(float v)
{
    __shared__ unsigned wmax[4];
    unsigned u = __float_as_uint(v);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) u = max(u, (unsigned)__shfl_xor((int)u, o));
    if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = u;
    __syncthreads();
    return max(max(wmax[0], wmax[1]), max(wmax[2], wmax[3]));
}

// arow (may be null): [colblocks][T], the largest magnitude of a[t, 64 columns of the block] per row t
__device__ __forceinline__ void coldot_block(const ColDotArgs &a, int colblock, int slab, unsigned *amax, unsigned *bmax, int slot,
                                             unsigned *arow)
{
    __shared__ float red[256];
    const int tid = threadIdx.x;
    const int col = colblock * 64 + (tid & 63), ph = tid >> 6;
    const long rows_per = (a.T + a.nslab - 1) / a.nslab;
    const long r0 = slab * rows_per, r1 = min((long)a.T, r0 + rows_per);
    float s = 0.f, ma = 0.f, mb = 0.f;
    // every lane walks the rows (a wavefront = 64 columns of the rows r0 + ph, + 4, ...); columns past H read
    // column 0 and count as zero, so that the per-row maxima can be formed across the whole wavefront
    const bool okc = col < a.H;
    const int cc = okc ? col : 0;
    unsigned *arow_cb = arow ? arow + (size_t)colblock * a.T : nullptr;
    long t = r0 + ph;
    for (; t + 60 < r1; t += 64) {           // sixteen independent row pairs in flight (one trip to memory for 64 rows of a slab)
        float av[16], bv[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            av[j] = a.a[(t + 4 * j) * a.H + cc];
            bv[j] = a.b[(t + 4 * j) * a.H + cc];
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) {        // the arithmetic in the order of the loop below
            float a0 = av[4 * g], a1 = av[4 * g + 1], a2 = av[4 * g + 2], a3 = av[4 * g + 3];
            float b0 = bv[4 * g], b1 = bv[4 * g + 1], b2 = bv[4 * g + 2], b3 = bv[4 * g + 3];
            if (!okc) { a0 = a1 = a2 = a3 = 0.f; b0 = b1 = b2 = b3 = 0.f; }
            s = fmaf(a0, b0, s); s = fmaf(a1, b1, s); s = fmaf(a2, b2, s); s = fmaf(a3, b3, s);
            ma = fmaxf(fmaxf(ma, fmaxf(fabsf(a0), fabsf(a1))), fmaxf(fabsf(a2), fabsf(a3)));
            mb = fmaxf(fmaxf(mb, fmaxf(fabsf(b0), fabsf(b1))), fmaxf(fabsf(b2), fabsf(b3)));
            if (arow_cb) {
                const int l = tid & 63;
                const unsigned m = wave_max4(__float_as_uint(fabsf(a0)), __float_as_uint(fabsf(a1)), __float_as_uint(fabsf(a2)),
                                             __float_as_uint(fabsf(a3)), l);
                if (l < 4) arow_cb[t + 16 * g + 4 * (2 * (l & 1) + (l >> 1))] = m;
            }
        }
    }
    for (; t + 12 < r1; t += 16) {           // four independent row pairs in flight
        float a0 = a.a[t * a.H + cc], b0 = a.b[t * a.H + cc];
        float a1 = a.a[(t + 4) * a.H + cc], b1 = a.b[(t + 4) * a.H + cc];
        float a2 = a.a[(t + 8) * a.H + cc], b2 = a.b[(t + 8) * a.H + cc];
        float a3 = a.a[(t + 12) * a.H + cc], b3 = a.b[(t + 12) * a.H + cc];
        if (!okc) { a0 = a1 = a2 = a3 = 0.f; b0 = b1 = b2 = b3 = 0.f; }
        s = fmaf(a0, b0, s); s = fmaf(a1, b1, s); s = fmaf(a2, b2, s); s = fmaf(a3, b3, s);
        ma = fmaxf(fmaxf(ma, fmaxf(fabsf(a0), fabsf(a1))), fmaxf(fabsf(a2), fabsf(a3)));
        mb = fmaxf(fmaxf(mb, fmaxf(fabsf(b0), fabsf(b1))), fmaxf(fabsf(b2), fabsf(b3)));
        if (arow_cb) {
            const int l = tid & 63;
            const unsigned m = wave_max4(__float_as_uint(fabsf(a0)), __float_as_uint(fabsf(a1)), __float_as_uint(fabsf(a2)),
                                         __float_as_uint(fabsf(a3)), l);
            if (l < 4) arow_cb[t + 4 * (2 * (l & 1) + (l >> 1))] = m;
        }
    }
    for (; t < r1; t += 4) {
        float a0 = a.a[t * a.H + cc], b0 = a.b[t * a.H + cc];
        if (!okc) { a0 = 0.f; b0 = 0.f; }
        s = fmaf(a0, b0, s);
        ma = fmaxf(ma, fabsf(a0)); mb = fmaxf(mb, fabsf(b0));
        if (arow_cb) {
            const unsigned u0 = wave_max_lane63(__float_as_uint(fabsf(a0)));
            if ((tid & 63) == 63) arow_cb[t] = u0;
        }
    }
    red[tid] = s;
    __syncthreads();
    if (ph == 0 && col < a.H)
        a.partial[(long)slab * a.H + col] = (red[tid] + red[tid + 64]) + (red[tid + 128] + red[tid + 192]);
    if (amax) {
        const unsigned ua = block_absmax(ma);
        __syncthreads();
        const unsigned ub = block_absmax(mb);
        if (tid == 0) { amax[slot] = ua; bmax[slot] = ub; }
    }
}

// slots[row] = largest magnitude of row `row` of x[n / rowlen][rowlen].  A wavefront takes RW rows at a time
// (all their loads in flight before the first reduction): one row each while there are at least as many
// wavefronts as rows, else four -- measured on 4096 cold rows of 512 values: 2.9 us with one row per
// wavefront in 1024 workgroups, 4.7 us with four rows per wavefront in 256.
template <int RW>
__device__ __forceinline__ void absmax_rows_batch(const PrepArgs::Pass &q, size_t row0, size_t rows, int lane)
{
    float m[RW];
#pragma unroll
    for (int r = 0; r < RW; ++r) m[r] = 0.f;
    if (q.vec && q.rowlen <= 512) {
        // up to two float4 per lane and row: 2 RW independent loads
        float4 a[RW][2];
#pragma unroll
        for (int r = 0; r < RW; ++r)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int i = lane + 64 * h;
                const bool ok = row0 + r < rows && i < q.rowlen / 4;
                const float4 *x4 = reinterpret_cast<const float4 *>(q.x + (ok ? row0 + r : 0) * (size_t)q.rowlen);
                const float4 t = x4[ok ? i : 0];
                a[r][h] = ok ? t : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
        for (int r = 0; r < RW; ++r)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                m[r] = fmaxf(m[r], fmaxf(fmaxf(fabsf(a[r][h].x), fabsf(a[r][h].y)), fmaxf(fabsf(a[r][h].z), fabsf(a[r][h].w))));
    } else {
#pragma unroll
        for (int r = 0; r < RW; ++r) {
            if (row0 + r >= rows) break;
            const float *x = q.x + (row0 + r) * (size_t)q.rowlen;
            if (q.vec) {
                const float4 *x4 = reinterpret_cast<const float4 *>(x);
                for (int i = lane; i < q.rowlen / 4; i += 64) {
                    const float4 t = x4[i];
                    m[r] = fmaxf(m[r], fmaxf(fmaxf(fabsf(t.x), fabsf(t.y)), fmaxf(fabsf(t.z), fabsf(t.w))));
                }
            } else {
                for (int i = lane; i < q.rowlen; i += 64) m[r] = fmaxf(m[r], fabsf(x[i]));
            }
        }
    }
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        const unsigned u = wave_max_lane63(__float_as_uint(m[r]));
        if (lane == 63 && row0 + r < rows) q.slots[row0 + r] = u;
    }
}
__device__ __forceinline__ void absmax_rows_block(const PrepArgs::Pass &q, int piece)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t rows = q.n / (size_t)q.rowlen;
    const size_t wid = (size_t)piece * 4 + wave, nw = (size_t)q.nblocks * 4;
    if (rows <= nw) {
        if (wid < rows) absmax_rows_batch<1>(q, wid, rows, lane);
    } else {
        for (size_t row0 = wid * 4; row0 < rows; row0 += nw * 4) absmax_rows_batch<4>(q, row0, rows, lane);
    }
}

// slots[piece] = largest magnitude of piece `piece` of x[n] (pieces of whole float4 units when vec)
__device__ __forceinline__ void absmax_pass_block(const PrepArgs::Pass &q, int piece)
{
    if (q.rowlen > 0) { absmax_rows_block(q, piece); return; }
    const int tid = threadIdx.x;
    float m = 0.f;
    if (q.vec) {
        const size_t n4 = q.n / 4;
        const float4 *x4 = reinterpret_cast<const float4 *>(q.x);
        size_t i = (size_t)piece * 256 + tid;
        const size_t stride = (size_t)q.nblocks * 256;
        for (; i + 7 * stride < n4; i += 8 * stride) {          // eight loads in flight
            float4 v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = x4[i + j * stride];
#pragma unroll
            for (int j = 0; j < 8; ++j)
                m = fmaxf(m, fmaxf(fmaxf(fabsf(v[j].x), fabsf(v[j].y)), fmaxf(fabsf(v[j].z), fabsf(v[j].w))));
        }
        for (; i + 3 * stride < n4; i += 4 * stride) {          // four loads in flight
            const float4 a = x4[i], b = x4[i + stride], c = x4[i + 2 * stride], d = x4[i + 3 * stride];
            m = fmaxf(m, fmaxf(fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))),
                               fmaxf(fmaxf(fabsf(b.x), fabsf(b.y)), fmaxf(fabsf(b.z), fabsf(b.w)))));
            m = fmaxf(m, fmaxf(fmaxf(fmaxf(fabsf(c.x), fabsf(c.y)), fmaxf(fabsf(c.z), fabsf(c.w))),
                               fmaxf(fmaxf(fabsf(d.x), fabsf(d.y)), fmaxf(fabsf(d.z), fabsf(d.w)))));
        }
        for (; i < n4; i += stride) {
            const float4 a = x4[i];
            m = fmaxf(m, fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))));
        }
    } else {
        for (size_t i = (size_t)piece * 256 + tid; i < q.n; i += (size_t)q.nblocks * 256) m = fmaxf(m, fabsf(q.x[i]));
    }
    const unsigned u = block_absmax(m);
    if (tid == 0) q.slots[piece] = u;
}

// Workgroups [0, P): state p -> Abar_p, packed Bbar rows 2p, 2p+1 (and the interleaved complex
// Bbar when asked).  Workgroups [P, P+H): row h of C -> (Re, -Im) interleaved.  Further workgroups
// (gradient pass only): the column-dot slabs behind dD.
__global__ void __launch_bounds__(256) prep_kernel(PrepArgs a)
{
    const int blk = blockIdx.x, tid = threadIdx.x;
    if (blk == 0 && tid == 0 && a.hdr) {
        a.hdr->err = 0; a.hdr->magic = 0x53534d31u;
    }
    if (a.pass[0].nblocks > 0 && blk >= a.pass[0].block0) {
        // passes over the activations whose largest magnitude no earlier kernel could record
        const int second = (a.pass[1].nblocks > 0 && blk >= a.pass[1].block0) ? 1 : 0;
        absmax_pass_block(a.pass[second], blk - a.pass[second].block0);
    } else if (blk < a.P) {
        const int p = blk;
        const Zoh z = zoh_discretize(a.Lambda[p], a.log_delta[p]);
        const float gr = (float)z.gr, gi = (float)z.gi;
        if (tid == 0 && a.lam_bar) a.lam_bar[p] = make_float2((float)z.lr, (float)z.li);
        float m = 0.f;
        if (a.B) {
            for (int h = tid; h < a.H; h += 256) {
                const float2 bv = a.B[(long)p * a.H + h];
                const float re = gr * bv.x - gi * bv.y, im = gr * bv.y + gi * bv.x;
                if (a.Bbar_ri) {
                    a.Bbar_ri[(long)(2 * p) * a.H + h] = re;
                    a.Bbar_ri[(long)(2 * p + 1) * a.H + h] = im;
                }
                if (a.Bbar_c64) a.Bbar_c64[(long)p * a.H + h] = make_float2(re, im);
                m = fmaxf(m, fmaxf(fabsf(re), fabsf(im)));
            }
        }
        if (a.bbar_max) {
            const unsigned u = block_absmax(m);
            if (tid == 0) a.bbar_max[p] = u;
        }
    } else if (blk < a.P + a.H) {
        const int h = blk - a.P;
        const float2 *src = a.C + (long)h * a.P;
        float2 *dst = reinterpret_cast<float2 *>(a.Cc) + (long)h * a.P;
        float m = 0.f;
        for (int p = tid; p < a.P; p += 256) {
            const float2 c = src[p];
            dst[p] = make_float2(c.x, -c.y);
            m = fmaxf(m, fmaxf(fabsf(c.x), fabsf(c.y)));
        }
        if (a.cc_max) {
            const unsigned u = block_absmax(m);
            if (tid == 0) a.cc_max[h] = u;
        }
    } else if (a.zero16 && blk >= a.zero_block0) {
        // clears the tagged words that the scanning input projection will publish into
        const size_t per = 256 * 8;
        const size_t i0 = (size_t)(blk - a.zero_block0) * per + tid;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const size_t i = i0 + (size_t)j * 256;
            if (i < a.n16) a.zero16[i] = make_uint4(0, 0, 0, 0);
        }
    } else {
        // column-dot slabs of the gradient pass share this launch (they depend on nothing here)
        const int cb = blk - (a.P + a.H);
        coldot_block(a.cd, cb % a.cd_colblocks, cb / a.cd_colblocks, a.cd_amax, a.cd_bmax, cb, a.cd_arow);
    }
}

hipError_t launch_prep(const PrepArgs &a_in, hipStream_t s)
{
    PrepArgs a = a_in;
    a.cd_colblocks = 0;
    unsigned blocks = (unsigned)(a.P + (a.Cc ? a.H : 0));
    if (a.cd.partial) {
        if (!a.Cc) return hipErrorInvalidValue;       // block ranges assume the C rows are present
        a.cd_colblocks = (a.cd.H + 63) / 64;
        blocks += (unsigned)(a.cd_colblocks * a.cd.nslab);
    }
    a.zero_block0 = 0;
    if (a.zero16 && a.n16 > 0) {
        if (!a.Cc) return hipErrorInvalidValue;       // block ranges assume the C rows are present
        a.zero_block0 = (int)blocks;
        blocks += (unsigned)((a.n16 + 256 * 8 - 1) / (256 * 8));
    } else {
        a.zero16 = nullptr;
    }
    // the passes come last; pass[1] without pass[0] moves up
    if (a.pass[0].nblocks <= 0 && a.pass[1].nblocks > 0) { a.pass[0] = a.pass[1]; a.pass[1].nblocks = 0; }
    for (int i = 0; i < 2; ++i) {
        PrepArgs::Pass &q = a.pass[i];
        if (q.nblocks <= 0) { q.nblocks = 0; continue; }
        if (!a.Cc || !q.x || !q.slots) return hipErrorInvalidValue;
        q.vec = (reinterpret_cast<uintptr_t>(q.x) & 15) == 0 && q.n % 4 == 0 && q.rowlen % 4 == 0;
        if (q.rowlen < 0 || (q.rowlen > 0 && q.n % (size_t)q.rowlen != 0)) return hipErrorInvalidValue;
        q.block0 = (int)blocks;
        blocks += (unsigned)q.nblocks;
    }
    hipLaunchKernelGGL(prep_kernel, dim3(blocks), dim3(256), 0, s, a);
    return hipGetLastError();
}

int coldot_slabs(int64_t T)
{
    int64_t n = (T + 63) / 64;
    if (n > 64) n = 64;                     // (128 and 256 slabs at 16384 tokens: within 0.5 % either way)
    if (n < 1) n = 1;
    return (int)n;
}

// ---------------------------------------------------------------------------------------------
// Adjoint of the discretisation and final reduction of the split partial sums.
//   workgroups [0, P): state p.   dBbar[p,h] = sum of the K-split slabs (rows 2p, 2p+1);
//       dB[p,h] = conj(g_p) dBbar[p,h];  dg_p = sum_h conj(B[p,h]) dBbar[p,h];
//       dAbar_p = sum of the reverse scan's partial rows;
//       dLambda_p = conj(Delta Abar) dAbar + conj(Delta^2 psi'(z)) dg,   psi(z) = (e^z - 1)/z
//       dlog_delta_p = Delta * Re(conj(Lambda Abar) dAbar + conj(Abar) dg)
//   workgroups [P, P+H): row h of dC = sum of its slabs with the imaginary part negated
//       (dC[h,p] = sum_t dy[t,h] conj(x[t,p])), and dD[h] = sum of the column-dot slabs.
// ---------------------------------------------------------------------------------------------
__device__ void psi_prime(double zr, double zi, double er, double ei, double &pr, double &pi)
{
    // psi'(z) = (z e^z - e^z + 1)/z^2 = sum_k z^k (k+1)/(k+2)!
    if (zr * zr + zi * zi < 0.25) {
        double tr = 0.5, ti = 0.0;
        pr = 0.5; pi = 0.0;
        for (int k = 1; k < 32; ++k) {
            const double c = (double)(k + 1) / ((double)k * (double)(k + 2));
            const double nr = (tr * zr - ti * zi) * c, ni = (tr * zi + ti * zr) * c;
            tr = nr; ti = ni;
            pr += tr; pi += ti;
        }
    } else {
        // (e^z - psi(z))/z with psi = expm1(z)/z; er, ei = e^z
        const double sh = sin(0.5 * zi);
        const double mr = expm1(zr) * cos(zi) - 2.0 * sh * sh, mi = ei;
        double psr, psi_;
        cdiv(mr, mi, zr, zi, psr, psi_);
        cdiv(er - psr, ei - psi_, zr, zi, pr, pi);
    }
}

// fixed-order sum of n slabs (stride apart) with up to eight loads in flight
__device__ __forceinline__ float sum_slabs(const float *base, long stride, int n, int i = 0, float s = 0.f)
{
    // (i, s: continue behind the first i slabs, whose sum in the same order is s)
    for (; i + 8 <= n; i += 8) {
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = base[(long)(i + j) * stride];
#pragma unroll
        for (int j = 0; j < 8; ++j) s += v[j];
    }
    for (; i + 4 <= n; i += 4) {
        const float v0 = base[(long)i * stride], v1 = base[(long)(i + 1) * stride];
        const float v2 = base[(long)(i + 2) * stride], v3 = base[(long)(i + 3) * stride];
        s = (((s + v0) + v1) + v2) + v3;
    }
    for (; i < n; ++i) s += base[(long)i * stride];
    return s;
}

// deterministic sum of one double pair per thread over the 256 threads of a workgroup; result valid in thread 0.
// Inside a wavefront a fixed butterfly of lane exchanges, then the four wavefront sums in order through LDS
// (two barriers; a tree over all 256 values through LDS took eight and ~0.9 us).
__device__ __forceinline__ double shfl_xor_double(double v, int mask)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __shfl_xor(lo, mask); hi = __shfl_xor(hi, mask);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ void block_sum2(double *red_r, double *red_i, double &r, double &i, int tid)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        r += shfl_xor_double(r, o);
        i += shfl_xor_double(i, o);
    }
    __syncthreads();                                   // (red_r, red_i may still be read from an earlier call)
    if ((tid & 63) == 0) { red_r[tid >> 6] = r; red_i[tid >> 6] = i; }
    __syncthreads();
    r = (red_r[0] + red_r[1]) + (red_r[2] + red_r[3]);
    i = (red_i[0] + red_i[1]) + (red_i[2] + red_i[3]);
}

// 2048 elements per workgroup (eight per thread, as two float4 where alignment allows)
__device__ __forceinline__ void sum_halves_block(const SumHalvesArgs &a, int blk, int tid)
{
    const long base = (long)blk * 2048;
    if (a.vec) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const long i = base + 4L * (tid + 256 * j);
            if (i < a.n) {
                const float4 x = *reinterpret_cast<const float4 *>(a.s0 + i), y = *reinterpret_cast<const float4 *>(a.s1 + i);
                const float4 e = *reinterpret_cast<const float4 *>(a.e + i);
                const float4 d = *reinterpret_cast<const float4 *>(a.D + i % a.H);
                *reinterpret_cast<float4 *>(a.out + i) = make_float4(fmaf(d.x, e.x, x.x + y.x), fmaf(d.y, e.y, x.y + y.y),
                                                                     fmaf(d.z, e.z, x.z + y.z), fmaf(d.w, e.w, x.w + y.w));
            }
        }
    } else {
        for (int j = 0; j < 8; ++j) {
            const long i = base + tid + 256L * j;
            if (i < a.n) a.out[i] = fmaf(a.D[i % a.H], a.e[i], a.s0[i] + a.s1[i]);
        }
    }
}

__global__ void __launch_bounds__(256) epilogue_kernel(EpilogueArgs a)
{
    __shared__ double red_r[256], red_i[256];
    const int tid = threadIdx.x;
    if ((int)blockIdx.x < a.sum.nblocks) {        // the streaming sum of the two halves of du comes first
        sum_halves_block(a.sum, blockIdx.x, tid);
        return;
    }
    const int blk = blockIdx.x - a.sum.nblocks;
    const long PH2 = 2L * a.P * a.H;
    if (blk < a.P) {
        // The workgroups of this launch are all resident at once, so it lasts as long as the chain of dependent
        // steps of one of them.  The loads that need nothing from the discretisation are requested first (the
        // first partial row of dAbar, the slabs of the thread's first column), so that its double-precision
        // transcendentals, and psi' behind them, run while those are under way.
        const int p = blk;
        const float2 apart0 = tid < a.npart ? a.dAbar_part[(long)tid * a.P + p] : make_float2(0.f, 0.f);
        constexpr int EARLY = 8;                      // slabs of the first column requested ahead
        const int hc = tid < a.H ? tid : 0;
        const int nearly = a.nsplit_B < EARLY ? a.nsplit_B : EARLY;
        float vr[EARLY], vi[EARLY];
#pragma unroll
        for (int j = 0; j < EARLY; ++j) {
            const long o = (long)(j < nearly ? j : 0) * PH2;
            vr[j] = a.dBbar_part[o + (long)(2 * p) * a.H + hc];
            vi[j] = a.dBbar_part[o + (long)(2 * p + 1) * a.H + hc];
        }
        const float2 bv0 = a.B[(long)p * a.H + hc];
        const Zoh z = zoh_discretize(a.Lambda[p], a.log_delta[p]);
        double pr, pi;
        psi_prime(z.zr, z.zi, z.lr, z.li, pr, pi);
        // (the barrier keeps the waits for the loads above behind the arithmetic above)
        __builtin_amdgcn_sched_barrier(0);
        float sr0 = 0.f, si0 = 0.f;
#pragma unroll
        for (int j = 0; j < EARLY; ++j)
            if (j < nearly) { sr0 += vr[j]; si0 += vi[j]; }
        sr0 = sum_slabs(a.dBbar_part + (long)(2 * p) * a.H + hc, PH2, a.nsplit_B, nearly, sr0);
        si0 = sum_slabs(a.dBbar_part + (long)(2 * p + 1) * a.H + hc, PH2, a.nsplit_B, nearly, si0);
        const float gr = (float)z.gr, gi = (float)z.gi;
        double dgr = 0.0, dgi = 0.0;
        for (int h = tid; h < a.H; h += 256) {
            const bool first = h == tid;
            const float sr = first ? sr0 : sum_slabs(a.dBbar_part + (long)(2 * p) * a.H + h, PH2, a.nsplit_B);
            const float si = first ? si0 : sum_slabs(a.dBbar_part + (long)(2 * p + 1) * a.H + h, PH2, a.nsplit_B);
            // conj(g) * dBbar
            a.dB[(long)p * a.H + h] = make_float2(gr * sr + gi * si, gr * si - gi * sr);
            const float2 bv = first ? bv0 : a.B[(long)p * a.H + h];
            // conj(B) * dBbar
            dgr += (double)bv.x * sr + (double)bv.y * si;
            dgi += (double)bv.x * si - (double)bv.y * sr;
        }
        block_sum2(red_r, red_i, dgr, dgi, tid);
        double ar = (double)apart0.x, ai = (double)apart0.y;     // dAbar: partial rows of the reverse scan
        for (long i = tid + 256; i < a.npart; i += 256) {
            ar += (double)a.dAbar_part[i * a.P + p].x;
            ai += (double)a.dAbar_part[i * a.P + p].y;
        }
        block_sum2(red_r, red_i, ar, ai, tid);
        if (tid == 0) {
            const double Lr = a.Lambda[p].x, Li = a.Lambda[p].y, d = z.delta;
            // conj(d * Abar) * dAbar + conj(d^2 psi') * dg
            const double c1r = d * z.lr, c1i = d * z.li, c2r = d * d * pr, c2i = d * d * pi;
            const double dLr = (c1r * ar + c1i * ai) + (c2r * dgr + c2i * dgi);
            const double dLi = (c1r * ai - c1i * ar) + (c2r * dgi - c2i * dgr);
            a.dLambda[p] = make_float2((float)dLr, (float)dLi);
            // Re(conj(Lambda Abar) dAbar + conj(Abar) dg)
            const double mr = Lr * z.lr - Li * z.li, mi = Lr * z.li + Li * z.lr;
            const double dDelta = (mr * ar + mi * ai) + (z.lr * dgr + z.li * dgi);
            a.dlog_delta[p] = (float)(d * dDelta);
        }
    } else {
        const int h = blk - a.P;
        for (int j = tid; j < 2 * a.P; j += 256) {
            const float s = sum_slabs(a.dC_part + (long)h * 2 * a.P + j, PH2, a.nsplit_C);
            reinterpret_cast<float *>(a.dC)[(long)h * 2 * a.P + j] = (j & 1) ? -s : s;
        }
        double sd = 0.0, unused = 0.0;
        for (int sl = tid; sl < a.nslab; sl += 256) sd += (double)a.dD_part[(long)sl * a.H + h];
        block_sum2(red_r, red_i, sd, unused, tid);
        if (tid == 0) a.dD[h] = (float)sd;
    }
}

hipError_t launch_epilogue(const EpilogueArgs &a_in, hipStream_t s)
{
    EpilogueArgs a = a_in;
    a.sum.nblocks = 0; a.sum.vec = 0;
    if (a.sum.s0) {
        auto al16 = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
        a.sum.vec = a.sum.H % 4 == 0 && al16(a.sum.s0) && al16(a.sum.s1) && al16(a.sum.D) && al16(a.sum.e) && al16(a.sum.out);
        const long nb = (a.sum.n + 2047) / 2048;
        if (nb > 0x7fff0000L) return hipErrorInvalidValue;
        a.sum.nblocks = (int)nb;
    }
    hipLaunchKernelGGL(epilogue_kernel, dim3((unsigned)(a.sum.nblocks + a.P + a.H)), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace ssm
