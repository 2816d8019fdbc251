// Resettable scan over the sequence dimension, forward and reverse time (gfx950).
//
// What is computed: the inclusive scan of Eq. 4 over the elements (Abar, Bbar u_k, reset flag)
// of Eq. 9 under the operator of Eq. 10.  For a diagonal Abar the products are element-wise, so
// every (sequence, state) pair is an independent lane.  Three nested levels combine partial
// results with that operator:
//   1. a thread walks SCAN_E consecutive steps held in registers (loads are coalesced over the
//      state index: neighbouring threads own neighbouring states of the same step);
//   2. the cy chunks of a workgroup exchange their (product, state) aggregates through LDS;
//   3. workgroups along time exchange aggregates through descriptors in global memory with a
//      decoupled look-back: each publishes its own aggregate before it waits for anything, then
//      fetches the aggregates of the earlier workgroups of its group (one per thread, all in
//      flight at once) plus the inclusive state that closes the previous group.
// Logical time-block ids come from an atomic ticket per chain, so a workgroup only ever waits
// for workgroups that started before it, and every wait is bounded by spin_limit.
// Workgroups whose steps carry no flag at all take a guard-free path (plain recurrence, pointer
// stepping, Abar^16 by squaring): the kernel is issue bound otherwise, not memory bound.
//
// The reverse scan runs the same operator over reversed time with conj(Abar):
//   chi_t = gx_t + [not is_first_{t+1}] conj(Abar) chi_{t+1}
// and additionally reduces dAbar += [not is_first_t] conj(x_{t-1}) chi_t.
#include "ssm_internal.h"
#include "lookback.h"

namespace ssm {

// Abar^(16 * cy) for cy a power of two, in double so that the power itself adds no error
__device__ __forceinline__ float2 pow_block(float2 lam, int cy)
{
    double r = lam.x, i = lam.y;
    for (int n = 1; n < SCAN_E * cy; n *= 2) {
        const double nr = r * r - i * i, ni = 2.0 * r * i;
        r = nr; i = ni;
    }
    return make_float2((float)r, (float)i);
}

// v[e], e < 16, per lane -> the maximum over the 16 lanes of a group (lanes 16g .. 16g+15) of
// v[group16_index(lane)]: halving exchanges between lanes that differ in bit 0, 1, 2, 3.
__device__ __forceinline__ unsigned group16_max(unsigned (&v)[16], int lane)
{
#pragma unroll
    for (int bit = 0; bit < 4; ++bit) {
        const int n = 8 >> bit;
        const bool up = (lane >> bit) & 1;
#pragma unroll
        for (int k = 0; k < n; ++k) {
            const unsigned keep = up ? v[k + n] : v[k], send = up ? v[k] : v[k + n];
            v[k] = max(keep, (unsigned)__shfl_xor((int)send, 1 << bit));
        }
    }
    return v[0];
}
__device__ __forceinline__ int group16_index(int lane) { return 8 * (lane & 1) + 4 * ((lane >> 1) & 1) + 2 * ((lane >> 2) & 1) + ((lane >> 3) & 1); }

// MAXOUT: the kernel also records the largest magnitude of every token row of its output (atomic maxima
// into a.rowmax_out, zero on entry: the product that consumes the output stages every token under its own
// scale) and of the whole output (a.amax_out, ABSMAX_SLOTS slots, zero on entry).
template <bool REV, bool MAXOUT>
__global__ void __launch_bounds__(SCAN_THREADS) scan_kernel(ScanArgs a)
{
    constexpr int E = SCAN_E;
    __shared__ float2 sA[SCAN_THREADS];
    __shared__ float2 sS[SCAN_THREADS];
    __shared__ float2 sX[SCAN_THREADS];
    __shared__ unsigned s_id;

    const int tid = threadIdx.x;
    const int nchains = a.nPX * a.Bt;
    unsigned id;
    if (a.nTB > 1) {
        // One ticket counter per (sequence, state block) chain: the i-th workgroup of a chain to
        // start takes time block i, so its predecessors along time have started before it.
        if (tid == 0) {
            const unsigned chain = blockIdx.x % nchains;
            s_id = atomicAdd(a.ticket + (size_t)chain * SCAN_TICKET_STRIDE, 1u) * nchains + chain;
        }
        __syncthreads();
        id = s_id;
    } else {
        id = blockIdx.x;
        // no cross-workgroup wait can happen: mark the workspace header as clean
        if (id == 0 && tid == 0) { a.err[0] = 0; a.err[1] = 0x53534d31u; }
    }
    // time index slowest: all first-in-time workgroups start before any second-in-time one
    const int px = id % a.nPX;
    const int b = (id / a.nPX) % a.Bt;
    const int tb = id / nchains;
    const int lane = tid % a.pxb, chunk = tid / a.pxb;
    const int p = px * a.pxb + lane;
    const bool active = p < a.P;
    const int L = a.L;
    const int s0 = (tb * a.cy + chunk) * E;          // first logical step of this thread
    const int len = max(0, min(E, L - s0));
    const long rowbase = (long)b * L;
    // every thread of the workgroup owns E steps of a valid state: no guards needed
    const bool full = ((tb + 1) * a.cy * E <= L) && ((px + 1) * a.pxb <= a.P);
    const long stride = REV ? -(long)a.P : (long)a.P;            // elements between consecutive logical steps
    const long first = (rowbase + (REV ? (L - 1 - s0) : s0)) * a.P + p;   // element of logical step s0

    float2 lam = active ? a.lam[p] : make_float2(0.f, 0.f);
    if (REV) lam.y = -lam.y;

    // logical step s <-> time t: forward t = s, reverse t = L-1-s
    float2 val[E];
    float2 xp[REV ? E : 1];
    if (full) {
        const float2 *src = a.in + first;
#pragma unroll
        for (int e = 0; e < E; ++e) val[e] = src[e * stride];
        if constexpr (REV) {
            // state before each step: x[t-1]; only the very last logical step can have t = 0
            const float2 *xs = a.xsaved + first - a.P;
#pragma unroll
            for (int e = 0; e < E - 1; ++e) xp[e] = xs[e * stride];
            if (s0 + E < L) xp[E - 1] = xs[(E - 1) * stride];
            else xp[E - 1] = a.x0 ? a.x0[(long)b * a.P + p] : make_float2(0.f, 0.f);
        }
    } else {
#pragma unroll
        for (int e = 0; e < E; ++e) {
            val[e] = make_float2(0.f, 0.f);
            if constexpr (REV) xp[e] = make_float2(0.f, 0.f);
            if (e < len && active) {
                const int s = s0 + e;
                const int t = REV ? (L - 1 - s) : s;
                val[e] = a.in[(rowbase + t) * a.P + p];
                if constexpr (REV) {
                    if (t > 0) xp[e] = a.xsaved[(rowbase + t - 1) * a.P + p];
                    else if (a.x0) xp[e] = a.x0[(long)b * a.P + p];
                }
            }
        }
    }

    // flags of the thread's steps as a bit mask (bit e = is_first at the time of logical step s0+e)
    unsigned fmask = 0;
    if (a.is_first && len > 0) {
        const int tlo = REV ? (L - s0 - len) : s0;             // lowest time index of the chunk
        const uint8_t *fp = a.is_first + rowbase + tlo;
        if (len == E && (reinterpret_cast<uintptr_t>(fp) & 15) == 0) {
            const uint4 w = *reinterpret_cast<const uint4 *>(fp);
            const unsigned ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const unsigned f = ((ww[j >> 2] >> (8 * (j & 3))) & 0xffu) != 0;
                fmask |= f << (REV ? (E - 1 - j) : j);
            }
        } else {
#pragma unroll
            for (int e = 0; e < E; ++e)
                if (e < len) {
                    const int t = REV ? (L - 1 - (s0 + e)) : (s0 + e);
                    fmask |= (unsigned)(a.is_first[rowbase + t] != 0) << e;
                }
        }
    }
    // rmask bit e: the incoming state of logical step s0+e is dropped.
    // forward: the step's own flag.  reverse: the flag that cuts chi_{t+1} -> chi_t is
    // is_first[t+1], i.e. the flag of the previous logical step.
    unsigned rmask = fmask;
    const unsigned mmask = fmask;                               // reverse only: is_first at the step itself
    if (REV) {
        rmask = fmask << 1;
        if (a.is_first && len > 0 && s0 > 0) rmask |= (unsigned)(a.is_first[rowbase + (L - s0)] != 0);
    }
    // wavefront-uniform: no flag anywhere in the steps of this wavefront -> plain recurrence
    const bool plain = full && (__builtin_amdgcn_ballot_w64((rmask | mmask) != 0) == 0);

    // ---- level 1, first pass: aggregate of the thread's steps for zero incoming state
    float2 A = make_float2(1.f, 0.f), S = make_float2(0.f, 0.f);
    static_assert(E == 16, "Abar^E below is four squarings");
    if (full) {
        if (plain) {
#pragma unroll
            for (int e = 0; e < E; ++e) S = cfma(lam, S, val[e]);
        } else {
            // branch-free: a reset zeroes the multiplier of that step
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const bool r = (rmask >> e) & 1u;
                const float2 le = make_float2(r ? 0.f : lam.x, r ? 0.f : lam.y);
                S = cfma(le, S, val[e]);
            }
        }
        float2 l2 = cmul(lam, lam);
        l2 = cmul(l2, l2); l2 = cmul(l2, l2); l2 = cmul(l2, l2);
        A = (rmask & 0xffffu) ? make_float2(0.f, 0.f) : l2;
    } else {
#pragma unroll
        for (int e = 0; e < E; ++e) {
            if (e < len) {
                if ((rmask >> e) & 1u) { S = val[e]; A = make_float2(0.f, 0.f); }
                else { S = cfma(lam, S, val[e]); A = cmul(A, lam); }
            }
        }
    }
    sA[tid] = A;
    sS[tid] = S;
    __syncthreads();

    // ---- level 2: exclusive combine over the earlier chunks of this workgroup
    float2 Aex = make_float2(1.f, 0.f), Sex = make_float2(0.f, 0.f);
    for (int j = 0; j < chunk; ++j) {
        const float2 Aj = sA[j * a.pxb + lane], Sj = sS[j * a.pxb + lane];
        Sex = cfma(Aj, Sex, Sj);
        Aex = cmul(Aj, Aex);
    }

    // ---- level 3: incoming state of the workgroup.
    // Workgroups along time form groups of G = cy.  The incoming state is always evaluated in
    // one canonical order, whatever the timing: start from the inclusive state of the last
    // workgroup of the previous group (x0 / zero for the first group) and fold the aggregates of
    // the earlier workgroups of the own group over it.  Results are therefore bitwise
    // reproducible.  Every workgroup publishes its aggregate before it waits for anything; the
    // last workgroup of a group also publishes its inclusive state.  Every predecessor covers
    // exactly cy*E steps, so its transition product is Abar^(cy*E) or zero (tag 2).
    const int G = a.cy;
    const int sg0 = (tb / G) * G;
    const bool lastchunk = (chunk == a.cy - 1);
    const size_t desc_stride = (size_t)nchains * a.pxb;          // descriptors per time block
    ScanDesc *mine = a.desc + ((size_t)id * a.pxb + lane);
    float2 Ablk = make_float2(0.f, 0.f), Sblk = make_float2(0.f, 0.f), Xin = make_float2(0.f, 0.f);
    if (lastchunk) {
        Ablk = cmul(A, Aex);
        Sblk = cfma(A, Sex, S);
        if (a.nTB > 1 && tb + 1 < a.nTB) {
            const unsigned tag = (Ablk.x == 0.f && Ablk.y == 0.f) ? 2u : 1u;
            publish_word(&mine->agg[0], Sblk.x, tag);
            publish_word(&mine->agg[1], Sblk.y, tag);
        }
        if (sg0 == 0 && !REV && a.x0 && active) Xin = a.x0[(long)b * a.P + p];
    }
    if (tb > 0) {                                    // uniform over the workgroup
        __syncthreads();                             // level 2 has finished reading sA / sS
        // thread (lane, chunk) fetches the aggregate of workgroup sg0 + chunk of this lane
        float2 Aj = make_float2(1.f, 0.f), Sj = make_float2(0.f, 0.f);
        const int j = sg0 + chunk;
        if (j < tb) {
            const ScanDesc *pred = mine - (size_t)(tb - j) * desc_stride;
            unsigned tag = 0;
            if (!wait_pair(pred->agg, 1u, a.spin_limit, Sj, tag)) {
                // gave up: flag it, hand on NaN (the states that depend on the missing aggregate become
                // NaN, so the failure cannot pass as data) and finish anyway
                atomicOr(a.err, 1u);
                Sj = make_float2(__builtin_nanf(""), __builtin_nanf(""));
                Aj = make_float2(0.f, 0.f);
            } else {
                Aj = (tag == 2u) ? make_float2(0.f, 0.f) : pow_block(lam, a.cy);
            }
        }
        sA[tid] = Aj;
        sS[tid] = Sj;
        if (lastchunk && sg0 > 0) {
            const ScanDesc *pred = mine - (size_t)(tb - sg0 + 1) * desc_stride;
            unsigned tag = 0;
            float2 incl;
            if (!wait_pair(pred->incl, 3u, a.spin_limit, incl, tag)) {
                atomicOr(a.err, 1u);
                Xin = make_float2(__builtin_nanf(""), __builtin_nanf(""));
            } else {
                Xin = incl;
            }
        }
        __syncthreads();
        if (lastchunk) {
            const int n = tb - sg0;
            for (int c = 0; c < n; ++c) Xin = cfma(sA[c * a.pxb + lane], Xin, sS[c * a.pxb + lane]);
        }
    }
    if (lastchunk) {
        if (a.nTB > 1 && tb + 1 < a.nTB && (tb + 1) % G == 0) {
            const float2 incl = cfma(Ablk, Xin, Sblk);
            publish_word(&mine->incl[0], incl.x, 3u);
            publish_word(&mine->incl[1], incl.y, 3u);
        }
        sX[lane] = Xin;
    }
    __syncthreads();

    // ---- level 1, second pass: the states themselves
    float2 xs = cfma(Aex, sX[lane], Sex);
    float2 acc = make_float2(0.f, 0.f);
    unsigned rm[MAXOUT ? E : 1];                     // MAXOUT: magnitude of the value stored at step e
    if constexpr (MAXOUT) {
#pragma unroll
        for (int e = 0; e < E; ++e) rm[e] = 0u;
    }
    if (full) {
        float2 *dst = a.out + first;
        if (plain) {
#pragma unroll
            for (int e = 0; e < E; ++e) {
                xs = cfma(lam, xs, val[e]);
                dst[e * stride] = xs;
                if constexpr (MAXOUT) rm[e] = __float_as_uint(fmaxf(fabsf(xs.x), fabsf(xs.y)));
                if constexpr (REV) {
                    // conj(x_{t-1}) * chi_t
                    acc.x = fmaf(xp[e].x, xs.x, fmaf(xp[e].y, xs.y, acc.x));
                    acc.y = fmaf(xp[e].x, xs.y, fmaf(-xp[e].y, xs.x, acc.y));
                }
            }
        } else {
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const bool r = (rmask >> e) & 1u;
                const float2 le = make_float2(r ? 0.f : lam.x, r ? 0.f : lam.y);
                xs = cfma(le, xs, val[e]);
                dst[e * stride] = xs;
                if constexpr (MAXOUT) rm[e] = __float_as_uint(fmaxf(fabsf(xs.x), fabsf(xs.y)));
                if constexpr (REV) {
                    const bool m = (mmask >> e) & 1u;
                    const float2 q = make_float2(m ? 0.f : xp[e].x, m ? 0.f : xp[e].y);
                    acc.x = fmaf(q.x, xs.x, fmaf(q.y, xs.y, acc.x));
                    acc.y = fmaf(q.x, xs.y, fmaf(-q.y, xs.x, acc.y));
                }
            }
        }
        if constexpr (REV) {
            if (s0 + E == L && a.dx0)
                a.dx0[(long)b * a.P + p] = ((mmask >> (E - 1)) & 1u) ? make_float2(0.f, 0.f) : cmul(lam, xs);
        } else {
            if (s0 + E == L && a.x_last) a.x_last[(long)b * a.P + p] = xs;
        }
    } else {
#pragma unroll
        for (int e = 0; e < E; ++e) {
            if (e < len) {
                const int s = s0 + e;
                const int t = REV ? (L - 1 - s) : s;
                xs = ((rmask >> e) & 1u) ? val[e] : cfma(lam, xs, val[e]);
                if (active) {
                    a.out[(rowbase + t) * a.P + p] = xs;
                    if constexpr (MAXOUT) rm[e] = __float_as_uint(fmaxf(fabsf(xs.x), fabsf(xs.y)));
                    if constexpr (REV) {
                        if (!((mmask >> e) & 1u)) {
                            // conj(x_{t-1}) * chi_t
                            acc.x += xp[e].x * xs.x + xp[e].y * xs.y;
                            acc.y += xp[e].x * xs.y - xp[e].y * xs.x;
                        }
                        if (t == 0 && a.dx0)
                            a.dx0[(long)b * a.P + p] =
                                ((mmask >> e) & 1u) ? make_float2(0.f, 0.f) : cmul(lam, xs);
                    } else {
                        if (t == L - 1 && a.x_last) a.x_last[(long)b * a.P + p] = xs;
                    }
                }
            }
        }
    }

    if constexpr (MAXOUT) {
        // a group of 16 lanes holds 16 neighbouring states of the same 16 steps: one atomic per step and group
        unsigned all = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) all = max(all, rm[e]);
        const unsigned m = group16_max(rm, tid);
        const int e = group16_index(tid);
        if (e < len) {
            const int t = REV ? (L - 1 - (s0 + e)) : (s0 + e);
            atomicMax(a.rowmax_out + rowbase + t, m);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) all = max(all, (unsigned)__shfl_xor((int)all, o));
        if ((tid & 63) == 0) atomicMax(a.amax_out + (blockIdx.x * 4 + (tid >> 6)) % ABSMAX_SLOTS, all);
    }
    if (REV) {
        // sum the chunks' contributions to dAbar; one partial row per (sequence, workgroup in time)
        sA[tid] = acc;
        __syncthreads();
        if (chunk == 0 && active) {
            float2 sum = make_float2(0.f, 0.f);
            for (int j = 0; j < a.cy; ++j) {
                sum.x += sA[j * a.pxb + lane].x;
                sum.y += sA[j * a.pxb + lane].y;
            }
            a.partial[((size_t)b * a.nTB + tb) * a.P + p] = sum;
        }
    }
}

ScanPlan plan_scan(int64_t Bt, int64_t L, int64_t P)
{
    ScanPlan pl;
    // as many chunks per workgroup as the sequence can use, at most 16 (16 lanes = one 128-byte
    // line of complex64 per step)
    int cy = 1;
    while (cy < 16 && (int64_t)cy * SCAN_E < L) cy *= 2;
    pl.cy = cy;
    pl.pxb = SCAN_THREADS / cy;
    pl.nPX = (int)((P + pl.pxb - 1) / pl.pxb);
    pl.nTB = (int)((L + (int64_t)cy * SCAN_E - 1) / ((int64_t)cy * SCAN_E));
    pl.nblocks = (int64_t)pl.nPX * Bt * pl.nTB;
    // look-back scratch: ticket counters (one per chain, 64 bytes apart) followed by descriptors
    pl.ticket_bytes = pl.nTB > 1 ? (size_t)pl.nPX * Bt * SCAN_TICKET_STRIDE * sizeof(uint32_t) : 0;
    pl.desc_bytes = pl.nTB > 1 ? (size_t)pl.nblocks * pl.pxb * sizeof(ScanDesc) : 0;
    pl.partial_elems = (size_t)Bt * pl.nTB * P;
    return pl;
}

hipError_t launch_scan(const ScanArgs &a, bool reverse, hipStream_t s)
{
    const int64_t nblocks = (int64_t)a.nPX * a.Bt * a.nTB;
    if (nblocks <= 0 || nblocks > 0x7fffffffLL || a.pxb * a.cy != SCAN_THREADS) return hipErrorInvalidValue;
    const bool maxout = a.rowmax_out != nullptr;
    if (maxout && !a.amax_out) return hipErrorInvalidValue;
    if (reverse && maxout) hipLaunchKernelGGL((scan_kernel<true, true>), dim3((unsigned)nblocks), dim3(SCAN_THREADS), 0, s, a);
    else if (reverse) hipLaunchKernelGGL((scan_kernel<true, false>), dim3((unsigned)nblocks), dim3(SCAN_THREADS), 0, s, a);
    else if (maxout) hipLaunchKernelGGL((scan_kernel<false, true>), dim3((unsigned)nblocks), dim3(SCAN_THREADS), 0, s, a);
    else hipLaunchKernelGGL((scan_kernel<false, false>), dim3((unsigned)nblocks), dim3(SCAN_THREADS), 0, s, a);
    return hipGetLastError();
}

// zeroes the header and the 16-byte words of the ticket counters + descriptors that follow it
__global__ void __launch_bounds__(256) clear_kernel(WsHeader *hdr, uint4 *desc, size_t n16)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i == 0) {
        hdr->err = 0; hdr->magic = 0x53534d31u;
    }
    for (size_t j = i; j < n16; j += (size_t)gridDim.x * 256) desc[j] = make_uint4(0, 0, 0, 0);
}

hipError_t launch_clear(WsHeader *hdr, void *scratch, size_t scratch_bytes, hipStream_t s)
{
    const size_t n16 = scratch_bytes / 16;
    uint4 *desc = static_cast<uint4 *>(scratch);
    size_t blocks = (n16 + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(clear_kernel, dim3((unsigned)blocks), dim3(256), 0, s, hdr, desc, n16);
    return hipGetLastError();
}

// out[p] = sum_i partial[i * P + p] in one fixed order: a workgroup owns 64 states, its four wavefronts
// take the rows i = w, w + 4, ... (eight loads in flight each), and the four sums are added in order.
__global__ void __launch_bounds__(256) reduce_partials_kernel(const float2 *__restrict__ partial, long n, long P,
                                                              float2 *__restrict__ out)
{
    __shared__ float2 part[4][64];
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    const long p = (long)blockIdx.x * 64 + l;
    float2 s = make_float2(0.f, 0.f);
    if (p < P) {
        long i = w;
        for (; i + 28 < n; i += 32) {
            float2 v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = partial[(i + 4 * k) * P + p];
#pragma unroll
            for (int k = 0; k < 8; ++k) { s.x += v[k].x; s.y += v[k].y; }
        }
        for (; i < n; i += 4) { const float2 v = partial[i * P + p]; s.x += v.x; s.y += v.y; }
    }
    part[w][l] = s;
    __syncthreads();
    if (w == 0 && p < P) {
        float2 t = part[0][l];
#pragma unroll
        for (int k = 1; k < 4; ++k) { t.x += part[k][l].x; t.y += part[k][l].y; }
        out[p] = t;
    }
}

hipError_t launch_reduce_partials(const float2 *partial, int64_t n, int64_t P, float2 *out, hipStream_t s)
{
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((P + 63) / 64)), dim3(256), 0, s,
                       partial, (long)n, (long)P, out);
    return hipGetLastError();
}

}  // namespace ssm
