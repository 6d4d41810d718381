// Backward kernels (Sec. 3.3 "Backward pass", Alg. 2-3 of the AdaSplash-2 paper):
//   dq_kernel   : per 32*QB*NW query rows, over the set bits of their mask rows, in one sweep:
//                 delta_r = sum_j U_rj dP_rj / sum_j U_rj,  U = P^(2-alpha), dP = dO V^T
//                 dQ = [ (U o dP) K - delta (U K) ] / sqrt(d)  ( = dS K / sqrt(d), Alg. 3)
//   dkdv_kernel : per 32*QB*NW keys, over the set bits of their mask columns:
//                 dV += P^T dO,  dK += dS^T Q / sqrt(d)                               (Alg. 2)
// With y = (alpha-1) s - tau on the support:  P = y^r,  U = y^(r-1),  r = 1/(alpha-1).
#pragma once
#include "common.hpp"

namespace ea {

// Two floats -> one register of two fp16 values (round to nearest even).
EA_DEV uint32_t pack_f16x2(float a, float b) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    h2 v;
    v[0] = (_Float16)a; v[1] = (_Float16)b;
    return __builtin_bit_cast(uint32_t, v);
}
// Second-stage operands in two fp16 halves.  A product whose B operand is rounded to fp16 carries a
// relative error of 2^-12 per element; summed over the hundreds or thousands of query rows that
// attend to one key (or over keys that share a large common component) those errors are what is left
// when the exact terms cancel, and they pass 1e-2 (1 + |gradient|).  So the operand is cut in two:
// hi = x with all but its 11 leading significant bits cleared (an fp16 value exactly), lo = x - hi
// (exact in fp32) rounded to fp16; hi + lo carries 21 bits of x, and the product is two MFMAs on the
// same A fragment.  SPLIT_NONE: one fp16 operand; SPLIT_SIGNED: the operands whose terms cancel
// (dS, U (dP - e)) are cut; SPLIT_ALL: P and U as well.
constexpr int SPLIT_NONE = 0, SPLIT_SIGNED = 1, SPLIT_ALL = 2;
#ifndef EA_BWD_SPLIT
#define EA_BWD_SPLIT SPLIT_ALL
#endif
EA_DEV float f16_head(float x) { return __uint_as_float(__float_as_uint(x) & 0xffffe000u); }
// packs of (hi, hi) and (lo, lo) of two floats
EA_DEV void pack_split(float a, float b, uint32_t& hi, uint32_t& lo) {
    const float ha = f16_head(a), hb = f16_head(b);
    hi = pack_f16x2(ha, hb);
    lo = pack_f16x2(a - ha, b - hb);
}
// x -> what fp16 rounding of x leaves behind (the plain tile bodies: stage2 rounds to nearest)
template <int QB> EA_DEV void f16_tail(f32x16 (&Y)[2][QB]) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int v = 0; v < 16; ++v) Y[kb][qb][v] -= (float)(_Float16)Y[kb][qb][v];
}
EA_DEV f16x8 frag_of(const uint32_t (&w)[8], int s2) {
    u32x4 v;
    v[0] = w[4 * s2]; v[1] = w[4 * s2 + 1]; v[2] = w[4 * s2 + 2]; v[3] = w[4 * s2 + 3];
    return __builtin_bit_cast(f16x8, v);
}

// One 64-key tile of the dQ sweep for a wave's 32 rows, 16-bit operands, every statement placed by
// hand.  A wave with 128 accumulator registers runs alone on its SIMD, so nothing but its own
// instruction order lets the vector ALUs work while the matrix pipe is busy.  The tile is cut into
// its two 32-key halves and the work on them is staggered:
//     stage 1, half 0                                    (matrix pipe only)
//     stage 1, half 1    with the score math of half 0   (one or two scores after every MFMA)
//     stage 2, half 0    with the score math of half 1
//     stage 2, half 1                                    (matrix pipe only)
// LDS reads run PF steps ahead of the MFMAs that use them.  An MFMA lasts 32 cycles and a vector
// instruction 4, so up to 7 vector instructions fit behind each MFMA at no cost.
template <class E, class E2, int D, int AM, int SPLIT>
EA_DEV void dq_tile_staggered(const char* kbuf, const char* vbuf, const Owned<E, D, 1>& qf, const Owned<E, D, 1>& gf,
                              f32x16 (&XA)[D / 32][1], f32x16 (&XB)[D / 32][1], float thr, float ctr, float c, float r,
                              float& num, float& den, const Frag1<E, D>& f1, const Frag2<E2, D>& f2) {
    constexpr int NS = D / 16, ND = D / 32;
    constexpr int N1 = 2 * NS;            // stage-1 steps (kb, s): two MFMAs each (scores, dP)
    constexpr int N2 = 4 * ND;            // stage-2 steps (kb, s2, db): two MFMAs each (XA, XB)
    constexpr int PF = 4;                 // steps the LDS reads run ahead
    constexpr int EPM = 8 / NS;           // scores handled after each MFMA of an overlapped phase
    static_assert(8 % NS == 0 && 4 % ND == 0 && EPM == 4 / ND, "halves must divide evenly over the MFMAs");
    using frag = typename E::frag;
    using frag2 = typename E2::frag;
    f32x16 S[2], P[2];
    uint32_t tp[2][8], up[2][8];          // t = u (dP - e) and u as fp16 pairs: the stage-2 B operands
    uint32_t tl[2][8], ul[2][8];          // their low halves (SPLIT)
    frag ak[N1], av[N1];
    frag2 at[N2];
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    auto score_math = [&](int kb, int e) {
        const float y = fmaf(c, S[kb][e], -thr);
        float u;
        if constexpr (AM == ALPHA_15) u = fmaxf(y, 0.f);
        else u = (y > 0.f) ? pow_r1<AM>(y, r) : 0.f;
        const float t = u * (P[kb][e] - ctr);
        num += t;
        den += u;
        S[kb][e] = t;
        P[kb][e] = u;
        if (e & 1) {
            if constexpr (SPLIT >= SPLIT_SIGNED) pack_split(S[kb][e - 1], S[kb][e], tp[kb][e >> 1], tl[kb][e >> 1]);
            else tp[kb][e >> 1] = pack_f16x2(S[kb][e - 1], S[kb][e]);
            if constexpr (SPLIT >= SPLIT_ALL) pack_split(P[kb][e - 1], P[kb][e], up[kb][e >> 1], ul[kb][e >> 1]);
            else up[kb][e >> 1] = pack_f16x2(P[kb][e - 1], P[kb][e]);
        }
    };
    auto read2 = [&](int i2) { at[i2] = f2(kbuf, i2 / (2 * ND), (i2 / ND) & 1, i2 % ND); };

#pragma unroll
    for (int i = 0; i < PF; ++i) { ak[i] = f1(kbuf, i / NS, i % NS); av[i] = f1(vbuf, i / NS, i % NS); }
    sched_fence();
#pragma unroll
    for (int i = 0; i < N1; ++i) {
        const int kb = i / NS, s = i % NS;
        if (i + PF < N1) { ak[i + PF] = f1(kbuf, (i + PF) / NS, (i + PF) % NS); av[i + PF] = f1(vbuf, (i + PF) / NS, (i + PF) % NS); }
        else read2(i + PF - N1);
        S[kb] = E::mma(ak[i], qf.f[0][s], s == 0 ? zero : S[kb]);
        sched_fence();
        if (kb == 1) {
#pragma unroll
            for (int k = 0; k < EPM; ++k) score_math(0, 2 * EPM * s + k);
        }
        sched_fence();
        P[kb] = E::mma(av[i], gf.f[0][s], s == 0 ? zero : P[kb]);
        sched_fence();
        if (kb == 1) {
#pragma unroll
            for (int k = 0; k < EPM; ++k) score_math(0, 2 * EPM * s + EPM + k);
        }
        sched_fence();
    }
#pragma unroll
    for (int i = 0; i < N2; ++i) {
        const int kb = i / (2 * ND), s2 = (i / ND) & 1, db = i % ND, j = i % (2 * ND);
        if (i + PF < N2) read2(i + PF);
        E2::template mma_acc<false>(at[i], frag_of(tp[kb], s2), XA[db][0]);
        sched_fence();
        if (kb == 0) {
#pragma unroll
            for (int k = 0; k < EPM; ++k) score_math(1, 2 * EPM * j + k);
        }
        sched_fence();
        E2::template mma_acc<false>(at[i], frag_of(up[kb], s2), XB[db][0]);
        sched_fence();
        if (kb == 0) {
#pragma unroll
            for (int k = 0; k < EPM; ++k) score_math(1, 2 * EPM * j + EPM + k);
        }
        sched_fence();
        if constexpr (SPLIT >= SPLIT_SIGNED) { E2::template mma_acc<false>(at[i], frag_of(tl[kb], s2), XA[db][0]); sched_fence(); }
        if constexpr (SPLIT >= SPLIT_ALL) { E2::template mma_acc<false>(at[i], frag_of(ul[kb], s2), XB[db][0]); sched_fence(); }
    }
}

template <class E, class E2, int D, int QB, int NW, int NBUF>
struct DqSmem {
    static constexpr int BR = 32 * QB * NW;
    static constexpr int MR = (BR + 63) / 64;
    static constexpr int RBYTES = RowTile<E, D>::BYTES;
    static constexpr int SET = 2 * RBYTES;                   // K, V tiles
};

template <class E, class E2, int D, int QB, int AM, int NW, int NBUF>
__global__ __launch_bounds__(NW * 64) void dq_kernel(Params p) {
    using SM = DqSmem<E, E2, D, QB, NW, NBUF>;
    using elem = typename E::elem;
    constexpr int BR = SM::BR, MR = SM::MR;
    constexpr int THREADS = NW * 64;
    // buffer sets (K tile, V tile) as separate variables (see stream_tiles); all LDS is static
    __shared__ __align__(1024) char set0[SM::SET];
    __shared__ __align__(1024) char set1[NBUF == 2 ? SM::SET : 1024];
    __shared__ uint32_t fm[MR * MAX_W];
    __shared__ int tl[MAX_T];
    __shared__ int tl_count[4];
    __shared__ unsigned long long blk_stats[4];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, h = lane >> 5;
    const int N = p.N, T = p.T, W = p.W;
    int bh, I;
    map_block(blockIdx.x, p.BH, (N + BR - 1) / BR, bh, I);
    const long q0 = (long)I * BR, qw0 = q0 + wave * 32 * QB;
    const bool active = qw0 < N;
    // row groups whose supports were listed get dQ and delta from bwd_rows_kernel
    if (p.gflag && p.gflag[(long)bh * ((N + p.grows - 1) / p.grows) + q0 / p.grows]) return;
    const long hoff = (long)bh * N * D;
    const elem* Kh = (const elem*)p.K + hoff;
    const elem* Vh = (const elem*)p.V + hoff;
    const int myrow = (wave * 32 * QB) / 64;
    const HeadConsts hc = head_consts(p, bh);
    const float c = hc.c, r = hc.r;

    for (int i = tid; i < MR * W; i += THREADS)
        fm[i] = (I * MR + i / W < T) ? (uint32_t)p.mask[((long)bh * T + (long)I * MR + i / W) * W + (i % W)] : 0u;
    build_tile_list(fm, MR, W, tl, tl_count, tid);

    Owned<E, D, QB> qf, gf;
    load_owned<E, D, QB>(qf, (const elem*)p.Q + hoff, active ? qw0 : 0, lane);
    load_owned<E, D, QB>(gf, (const elem*)p.dO + hoff, active ? qw0 : 0, lane);
    float thr[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) thr[qb] = active ? p.tau[(long)bh * N + qw0 + 32 * qb + n] : 0.f;

    // One sweep over the set bits of the mask rows.  With dS = U (dP - delta) and any centre e:
    //     dQ sqrt(d) = sum_j dS_j K_j = sum_j (U (dP - e))_j K_j - (delta - e) sum_j U_j K_j
    //                = XA - (delta - e) XB,     delta - e = sum(U (dP - e)) / sum(U),
    // so delta comes out of the row sums of the same sweep and the scores are computed once.
    // The centre e = <dO_r, O_r> = sum_j P_rj dP_rj is the P-weighted mean of dP over the support
    // (delta is the U-weighted one): it keeps XA - (delta - e) XB free of the cancellation that
    // e = 0 would bring when dP is nearly constant over the support.  Without O, e = 0.
    // With a narrow-range stage-2 type the whole backward runs on dO / max|dO| (amax undoes it at
    // the end): then |dP_rj| = |<dO_r, V_j>| <= sqrt(d) |V_j| and |U (dP - e)| <= 2 sqrt(d) max|V_j|,
    // far inside fp16's range for any V that itself fits fp16 comfortably, and fp16 keeps 11
    // significant bits at any magnitude in its normal range, so no further scaling is needed.
    float amax = 1.f;
    if constexpr (E2::SCALED) {
        amax = __uint_as_float(p.scal[0]);
        if (!(amax > 0.f)) amax = 1.f;
    }
    float ctr[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        float acc = 0.f;
        if (p.O && active) {
            // lane half h takes half of the row; 16-byte loads, all in flight together
            const f32x4* orow = (const f32x4*)(p.O + hoff + (qw0 + 32 * qb + n) * (long)D + h * (D / 2));
            const elem* grow = (const elem*)p.dO + hoff + (qw0 + 32 * qb + n) * (long)D + h * (D / 2);
            f32x4 ov[D / 8];
#pragma unroll
            for (int e = 0; e < D / 8; ++e) ov[e] = orow[e];
            if constexpr (sizeof(elem) == 2) {
                typedef elem ex8 __attribute__((ext_vector_type(8)));
                ex8 gv[D / 16];
#pragma unroll
                for (int e = 0; e < D / 16; ++e) gv[e] = ((const ex8*)grow)[e];
#pragma unroll
                for (int e = 0; e < D / 2; ++e) acc = fmaf(ov[e / 4][e % 4], (float)gv[e / 8][e % 8], acc);
            } else {
#pragma unroll
                for (int e = 0; e < D / 2; ++e) acc = fmaf(ov[e / 4][e % 4], (float)grow[e], acc);
            }
        }
        ctr[qb] = xhalf_sum(acc);
    }

    f32x16 XA[D / 32][QB], XB[D / 32][QB];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int v = 0; v < 16; ++v) { XA[db][qb][v] = 0.f; XB[db][qb][v] = 0.f; }

    f32x16 S[2][QB], dP[2][QB];
    unsigned long long ntile = 0;
    const Frag1<E, D> frag1(lane);
    const Frag2<E2, D> frag2(lane);
    float num[QB], den[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) num[qb] = den[qb] = 0.f;
    auto issue_kv = [&](int it, char* b) {
        const long j = tl[it];
        issue_rows<E, D, NW>(b, Kh, j * 64, wave, lane);
        issue_rows<E, D, NW>(b + SM::RBYTES, Vh, j * 64, wave, lane);
    };
    // any tile, statements left to the compiler's order
    auto tile_plain_order = [&](int it, const char* kbuf) {
        const int j = tl[it];
        if (!mask_bit(fm, W, myrow, j)) return;
        const char* vbuf = kbuf + SM::RBYTES;
        ++ntile;
        stage1<E, D, QB>(S, kbuf, qf, lane);
        if (p.causal && (long)j * 64 + 63 > qw0) causal_hide<QB, true>(S, j * 64, (int)qw0, lane);
        stage1<E, D, QB>(dP, vbuf, gf, lane);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float y = fmaf(c, S[kb][qb][v], -thr[qb]);
                    float u;
                    if constexpr (AM == ALPHA_15) u = fmaxf(y, 0.f);
                    else u = (y > 0.f) ? pow_r1<AM>(y, r) : 0.f;
                    const float t = u * (dP[kb][qb][v] - ctr[qb]);
                    num[qb] += t;
                    den[qb] += u;
                    S[kb][qb][v] = t;
                    dP[kb][qb][v] = u;
                }
        stage2<E2, D, QB, true>(XA, kbuf, S, lane);
        stage2<E2, D, QB, true>(XB, kbuf, dP, lane);
        if constexpr (E2::EPL == 8 && EA_BWD_SPLIT >= SPLIT_SIGNED) { f16_tail<QB>(S); stage2<E2, D, QB, true>(XA, kbuf, S, lane); }
        if constexpr (E2::EPL == 8 && EA_BWD_SPLIT >= SPLIT_ALL) { f16_tail<QB>(dP); stage2<E2, D, QB, true>(XB, kbuf, dP, lane); }
    };
    if constexpr (E::EPL == 8 && QB == 1 && NBUF == 2) {
        // tiles wholly below the diagonal (the head of the ascending list) take the staggered body;
        // the one or two on it, and one more when that makes the head's length even, the plain one
        const int nt = *tl_count;
        int ndiag = 0;
        if (p.causal)
            while (ndiag < nt && (long)tl[nt - 1 - ndiag] * 64 + 63 > q0) ++ndiag;
        stream_tiles_split((nt - ndiag) & ~1, nt, set0, set1, issue_kv,
            [&](int it, const char* kbuf) {
                if (!mask_bit(fm, W, myrow, tl[it])) return;
                ++ntile;
                dq_tile_staggered<E, E2, D, AM, EA_BWD_SPLIT>(kbuf, kbuf + SM::RBYTES, qf, gf, XA, XB, thr[0], ctr[0], c, r, num[0], den[0], frag1, frag2);
            },
            tile_plain_order);
    } else {
        stream_tiles<NBUF>(*tl_count, set0, NBUF == 2 ? set1 : set0, issue_kv, tile_plain_order);
    }
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) { settle_acc(XA[db][qb]); settle_acc(XB[db][qb]); }

    // delta (in units of max|dO|) for the dK/dV kernel, and the combination of the two sums
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float dn = xhalf_sum(den[qb]);
        const float drel = dn > 0.f ? xhalf_sum(num[qb]) / dn : 0.f;      // delta - e
        if (h == 0 && active) {
            // for the dK/dV kernel, as the biases its two stage-1 products start from
            p.delta[(long)bh * N + qw0 + 32 * qb + n] = -(drel + ctr[qb]);
            p.ntau[(long)bh * N + qw0 + 32 * qb + n] = -thr[qb] / hc.rho;
        }
        const float sa = p.inv_sqrt_d * amax, sb = drel * p.inv_sqrt_d * amax;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) XA[db][qb][v] = sa * XA[db][qb][v] - sb * XB[db][qb][v];
    }
    if (active) store_owned_T<D, QB>(p.dQ + hoff, qw0, XA, 1.f, lane);
    {
        const int slot[1] = {3};
        const unsigned long long val[1] = {ntile * QB};
        flush_counters<1>(blk_stats, p.stats, slot, val, tid, lane);
    }
}

// One 64-query tile of the dK/dV walk for a wave's 32 keys, staggered like dq_tile_staggered:
// stage 1 = (Q tile . K_owned^T, dO tile . V_owned^T), score math, stage 2 = (dV^T += dO^T P,
// dK^T += Q^T dS).  The thresholds and deltas of the tile's 64 query rows vary along the
// accumulator registers, so they cost no arithmetic at all: the accumulators of the two stage-1
// products start from -tau / rho and -delta (read from LDS, four rows per 16-byte read) instead of
// zero.  With the owned keys scaled by kappa the first product is then y / rho, y = (alpha-1) s -
// tau, and the second dP - delta; P = y^r and dS = y^(r-1) (dP - delta) come out in units of
// rho^r and rho^(r-1), which the kernel's epilogue multiplies back in.
template <class E, class E2, int D, int AM, int SPLIT>
EA_DEV void dkdv_tile_staggered(const char* qbuf, const char* gbuf, const float* ntau_s, const float* ndel_s,
                                const Owned<E, D, 1>& kf, const Owned<E, D, 1>& vf, f32x16 (&XV)[D / 32][1],
                                f32x16 (&XK)[D / 32][1], float r, int h, const Frag1<E, D>& f1,
                                const Frag2<E2, D>& f2) {
    constexpr int NS = D / 16, ND = D / 32;
    constexpr int N1 = 2 * NS, N2 = 4 * ND, PF = 4, EPM = 8 / NS;
    static_assert(8 % NS == 0 && 4 % ND == 0 && EPM == 4 / ND, "halves must divide evenly over the MFMAs");
    using frag = typename E::frag;
    using frag2 = typename E2::frag;
    f32x16 S[2], P[2];
    uint32_t pp[2][8], sp[2][8];          // P and dS as fp16 pairs: the stage-2 B operands
    uint32_t pl[2][8], sl[2][8];          // their low halves (SPLIT)
    frag aq[N1], ag[N1];
    frag2 tg[N2], tq[N2];

    // registers 4 g .. 4 g + 3 of half kb are four consecutive tile rows
    auto bias = [&](const float* vec, int kb) {
        f32x16 b;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const f32x4 t = *(const f32x4*)(vec + trow(kb, 4 * g, h));
#pragma unroll
            for (int e = 0; e < 4; ++e) b[4 * g + e] = t[e];
        }
        return b;
    };
    auto score_math = [&](int kb, int e) {
        const float yp = fmaxf(S[kb][e], 0.f);
        float u;
        if constexpr (AM == ALPHA_15) u = yp;
        else u = (yp > 0.f) ? pow_r1<AM>(yp, r) : 0.f;
        S[kb][e] = u * yp;
        P[kb][e] = u * P[kb][e];
        if (e & 1) {
            if constexpr (SPLIT >= SPLIT_ALL) pack_split(S[kb][e - 1], S[kb][e], pp[kb][e >> 1], pl[kb][e >> 1]);
            else pp[kb][e >> 1] = pack_f16x2(S[kb][e - 1], S[kb][e]);
            if constexpr (SPLIT >= SPLIT_SIGNED) pack_split(P[kb][e - 1], P[kb][e], sp[kb][e >> 1], sl[kb][e >> 1]);
            else sp[kb][e >> 1] = pack_f16x2(P[kb][e - 1], P[kb][e]);
        }
    };
    auto read2 = [&](int i2) {
        tg[i2] = f2(gbuf, i2 / (2 * ND), (i2 / ND) & 1, i2 % ND);
        tq[i2] = f2(qbuf, i2 / (2 * ND), (i2 / ND) & 1, i2 % ND);
    };

#pragma unroll
    for (int i = 0; i < PF; ++i) { aq[i] = f1(qbuf, i / NS, i % NS); ag[i] = f1(gbuf, i / NS, i % NS); }
    S[0] = bias(ntau_s, 0); P[0] = bias(ndel_s, 0);
    sched_fence();
#pragma unroll
    for (int i = 0; i < N1; ++i) {
        const int kb = i / NS, s = i % NS;
        if (i + PF < N1) { aq[i + PF] = f1(qbuf, (i + PF) / NS, (i + PF) % NS); ag[i + PF] = f1(gbuf, (i + PF) / NS, (i + PF) % NS); }
        else read2(i + PF - N1);
        if (i == NS - 2) { S[1] = bias(ntau_s, 1); P[1] = bias(ndel_s, 1); }
        S[kb] = E::mma(aq[i], kf.f[0][s], S[kb]);
        sched_fence();
        if (kb == 1) {
#pragma unroll
            for (int k = 0; k < EPM; ++k) score_math(0, 2 * EPM * s + k);
        }
        sched_fence();
        P[kb] = E::mma(ag[i], vf.f[0][s], P[kb]);
        sched_fence();
        if (kb == 1) {
#pragma unroll
            for (int k = 0; k < EPM; ++k) score_math(0, 2 * EPM * s + EPM + k);
        }
        sched_fence();
    }
#pragma unroll
    for (int i = 0; i < N2; ++i) {
        const int kb = i / (2 * ND), s2 = (i / ND) & 1, db = i % ND, j = i % (2 * ND);
        if (i + PF < N2) read2(i + PF);
        E2::template mma_acc<false>(tg[i], frag_of(pp[kb], s2), XV[db][0]);
        sched_fence();
        if (kb == 0) {
#pragma unroll
            for (int k = 0; k < EPM; ++k) score_math(1, 2 * EPM * j + k);
        }
        sched_fence();
        E2::template mma_acc<false>(tq[i], frag_of(sp[kb], s2), XK[db][0]);
        sched_fence();
        if (kb == 0) {
#pragma unroll
            for (int k = 0; k < EPM; ++k) score_math(1, 2 * EPM * j + EPM + k);
        }
        sched_fence();
        if constexpr (SPLIT >= SPLIT_SIGNED) { E2::template mma_acc<false>(tq[i], frag_of(sl[kb], s2), XK[db][0]); sched_fence(); }
        if constexpr (SPLIT >= SPLIT_ALL) { E2::template mma_acc<false>(tg[i], frag_of(pl[kb], s2), XV[db][0]); sched_fence(); }
    }
}

// Which of the MC mask columns jc0.. hold query tile i of head bh (bit c: column jc0 + c); none for
// query tiles of row groups whose supports were listed (those are left to bwd_cols_kernel).
template <int MC>
EA_DEV int column_flags(const Params& p, int bh, int i, int jc0) {
    if (p.gflag && p.gflag[(long)bh * ((p.N + p.grows - 1) / p.grows) + (i * 64) / p.grows]) return 0;
    int flags = 0;
#pragma unroll
    for (int cidx = 0; cidx < MC; ++cidx) {
        const int j = jc0 + cidx;
        if (j >= p.T) continue;
        const uint32_t w = (uint32_t)p.mask[((long)bh * p.T + i) * p.W + (j >> 5)];
        flags |= (int)((w >> (j & 31)) & 1u) << cidx;
    }
    return flags;
}

// Length of every key block's mask column, for dkdv_kernel's launch in parts; a column of more than
// one part has its rows of dK, dV cleared here, since all its parts add to them.
template <int D, int BC>
__global__ __launch_bounds__(128) void col_count_kernel(Params p) {
    constexpr int MC = (BC + 63) / 64;
    __shared__ int total;
    const int tid = threadIdx.x;
    const int GC = (p.N + BC - 1) / BC;
    int bh, J;
    map_block(blockIdx.x, p.BH, GC, bh, J);
    if (p.gflag && *p.nplain == 0) return;
    if (tid == 0) total = 0;
    __syncthreads();
    const int jc0 = J * MC;
    int mine = 0;
    for (int i = (p.causal ? jc0 : 0) + tid; i < p.T; i += 128) mine += column_flags<MC>(p, bh, i, jc0) != 0;
    if (mine) atomicAdd(&total, mine);
    __syncthreads();
    const int cnt = total;
    if (tid == 0) p.colcnt[(long)bh * GC + J] = cnt;
    if (cnt > p.col_part_len) {
        const long k0 = (long)J * BC, nk = min((long)BC, p.N - k0);
        f32x4* const dk = (f32x4*)(p.dK + ((long)bh * p.N + k0) * D);
        f32x4* const dv = (f32x4*)(p.dV + ((long)bh * p.N + k0) * D);
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        for (long e = tid; e < nk * (D / 4); e += 128) { dk[e] = zero; dv[e] = zero; }
    }
}

template <class E, class E2, int D, int QB, int NW, int NBUF>
struct DkdvSmem {
    static constexpr int BC = 32 * QB * NW;
    static constexpr int MC = (BC + 63) / 64;
    static constexpr int RBYTES = RowTile<E, D>::BYTES;
    static constexpr int SET = 2 * RBYTES + 4 * 2 * TILE;    // Q, dO tiles, tau, delta
};

template <class E, class E2, int D, int QB, int AM, int NW, int NBUF>
__global__ __launch_bounds__(NW * 64) void dkdv_kernel(Params p) {
    using SM = DkdvSmem<E, E2, D, QB, NW, NBUF>;
    using elem = typename E::elem;
    constexpr int BC = SM::BC, MC = SM::MC;
    constexpr int THREADS = NW * 64;
    static_assert(NW >= 2, "tau and delta rows are fetched by waves 0 and 1");
    // buffer sets (Q tile, dO tile, tau[64], delta[64]) as separate variables (see stream_tiles)
    __shared__ __align__(1024) char set0[SM::SET];
    __shared__ __align__(1024) char set1[NBUF == 2 ? SM::SET : 1024];
    __shared__ int tl[MAX_T];                // entries: query tile | column flags << 16
    __shared__ int wcnt[16];                 // per-wave counts, [8] = running total
    __shared__ unsigned long long blk_stats[4];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, h = lane >> 5;
    const int N = p.N, T = p.T, W = p.W;
    int bh, J;
    const int GC = (N + BC - 1) / BC, part = (int)blockIdx.x / (p.BH * GC);
    map_block((int)blockIdx.x % (p.BH * GC), p.BH, GC, bh, J);
    J = GC - 1 - J;                           // causal: the first key tiles have the longest columns
    // every row group went by gather: bwd_cols_kernel writes dK, dV itself
    if (p.gflag && *p.nplain == 0) return;
    // launched in parts (col_part_len > 0): a part past the column's end has nothing to do; all
    // parts of a column that has several add to rows that col_count_kernel cleared
    const bool shared_out = p.col_part_len > 0 && p.colcnt[(long)bh * GC + J] > p.col_part_len;
    if (part > 0 && p.colcnt[(long)bh * GC + J] <= part * p.col_part_len) return;
    const long k0 = (long)J * BC, kw0 = k0 + wave * 32 * QB;
    const bool active = kw0 < N;
    const long hoff = (long)bh * N * D;
    const elem* Qh = (const elem*)p.Q + hoff;
    const elem* Gh = (const elem*)p.dO + hoff;
    // dO is used divided by max|dO| throughout (see dq_kernel)
    float go_amax = 1.f;
    if constexpr (E2::SCALED) {
        go_amax = __uint_as_float(p.scal[0]);
        if (!(go_amax > 0.f)) go_amax = 1.f;
    }
    const int mycol = (wave * 32 * QB) / 64;  // my mask column within the group
    const int jc0 = J * MC;                   // first mask column of the group
    const HeadConsts hc = head_consts(p, bh);
    const float c = hc.c, r = hc.r;

    // ---- column walk of the row-packed mask: list of query tiles with a set bit -------------
    const int i_min = p.causal ? jc0 : 0;
    if (tid == 0) wcnt[8] = 0;
    __syncthreads();
    for (int base = i_min; base < T; base += THREADS) {
        const int i = base + tid;
        const int flags = i < T ? column_flags<MC>(p, bh, i, jc0) : 0;
        const unsigned long long bal = __ballot(flags != 0);
        if (lane == 0) wcnt[wave] = __popcll(bal);
        __syncthreads();
        int off = wcnt[8];
        for (int w2 = 0; w2 < wave; ++w2) off += wcnt[w2];
        off += __popcll(bal & ((1ull << lane) - 1ull));
        if (flags != 0) tl[off] = i | (flags << 16);
        __syncthreads();
        if (tid == 0) {
            int tot = wcnt[8];
            for (int w2 = 0; w2 < NW; ++w2) tot += wcnt[w2];
            wcnt[8] = tot;
        }
        __syncthreads();
    }
    int ntl = wcnt[8];
    if (p.col_part_len > 0) {
        // Long columns (a key that every later query tile attends to walks up to T tiles while most
        // columns hold a few) are cut into parts of col_part_len tiles, each worked off by a group
        // of its own: this one keeps its part of the list, moved to the front.
        const int lo = part * p.col_part_len, len = max(0, min(ntl - lo, p.col_part_len));
        if (part > 0) {
            int keep[(MAX_T + THREADS - 1) / THREADS];
#pragma unroll
            for (int q = 0; q < (MAX_T + THREADS - 1) / THREADS; ++q) keep[q] = q * THREADS + tid < len ? tl[lo + q * THREADS + tid] : 0;
            __syncthreads();
#pragma unroll
            for (int q = 0; q < (MAX_T + THREADS - 1) / THREADS; ++q)
                if (q * THREADS + tid < len) tl[q * THREADS + tid] = keep[q];
            __syncthreads();
        }
        ntl = len;
    }
    if (ntl == 0) {
        // no query tile for these keys (none attends to them, or all that do went by gather): their
        // dK, dV are zero, and a part of a shared column has nothing to add
        if (active && !shared_out) {
            f32x4* const dk = (f32x4*)(p.dK + hoff + kw0 * D);
            f32x4* const dv = (f32x4*)(p.dV + hoff + kw0 * D);
            const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
            for (int e = lane; e < 32 * QB * D / 4; e += 64) { dk[e] = zero; dv[e] = zero; }
        }
        return;
    }

    Owned<E, D, QB> kf, vf;
    load_owned<E, D, QB>(kf, (const elem*)p.K + hoff, active ? kw0 : 0, lane);
    // keys scaled by kappa, a power of two: exact, and the scores come out as kappa <q, k>
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int s = 0; s < D / E::KSTEP; ++s) kf.f[qb][s] = kf.f[qb][s] * (elem)hc.kappa;
    load_owned<E, D, QB>(vf, (const elem*)p.V + hoff, active ? kw0 : 0, lane);

    f32x16 XV[D / 32][QB], XK[D / 32][QB];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int v = 0; v < 16; ++v) { XV[db][qb][v] = 0.f; XK[db][qb][v] = 0.f; }

    f32x16 S[2][QB], dP[2][QB];
    unsigned long long ntile_done = 0;
    constexpr int VEC_OFF = 2 * SM::RBYTES;
    auto issue_qg = [&](int it, char* b) {
        const long i = __builtin_amdgcn_readfirstlane(tl[it] & 0xffff);
        issue_rows<E, D, NW>(b, Qh, i * 64, wave, lane);
        issue_rows<E, D, NW>(b + SM::RBYTES, Gh, i * 64, wave, lane);
        // the tile's 64 values of -tau / rho (wave 0) and of -delta (wave 1), one float per lane
        if (wave == 0) load4_to_lds(uniform_address(p.ntau + ((long)bh * N + i * 64)), 4u * lane, lds_address(b + VEC_OFF));
        if (wave == 1) load4_to_lds(uniform_address(p.delta + ((long)bh * N + i * 64)), 4u * lane, lds_address(b + VEC_OFF + 4 * TILE));
    };
    // any tile, statements left to the compiler's order
    auto tile_plain_order = [&](int it, const char* qbuf) {
        const int ent = tl[it];
        const long i = ent & 0xffff;
        if (!((ent >> (16 + mycol)) & 1)) return;
        const char* gbuf = qbuf + SM::RBYTES;
        const float* tau_s = (const float*)(qbuf + VEC_OFF);
        const float* del_s = tau_s + TILE;
        stage1<E, D, QB>(S, qbuf, kf, lane);
        // streamed rows are queries here: hide key > query
        if (p.causal && i * 64 < kw0 + 32 * QB - 1) causal_hide<QB, false>(S, (int)i * 64, (int)kw0, lane);
        stage1<E, D, QB>(dP, gbuf, vf, lane);
        ++ntile_done;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v4 = 0; v4 < 16; v4 += 4) {
                // registers v4..v4+3 are four consecutive tile rows: one 16-byte read each
                const int row = trow(kb, v4, h);
                const f32x4 tq4 = *(const f32x4*)(tau_s + row), dq4 = *(const f32x4*)(del_s + row);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int v = v4 + e;
                    const float tq = tq4[e], dq = dq4[e];
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) {
                        // (same units as the staggered body: y / rho, rho^r, rho^(r-1))
                        const float yp = fmaxf(S[kb][qb][v] + tq, 0.f);
                        float u;
                        if constexpr (AM == ALPHA_15) u = yp;
                        else u = (yp > 0.f) ? pow_r1<AM>(yp, r) : 0.f;
                        S[kb][qb][v] = u * yp;
                        dP[kb][qb][v] = u * (dP[kb][qb][v] + dq);
                    }
                }
            }
        stage2<E2, D, QB, true>(XV, gbuf, S, lane);
        stage2<E2, D, QB, true>(XK, qbuf, dP, lane);
        if constexpr (E2::EPL == 8 && EA_BWD_SPLIT >= SPLIT_SIGNED) { f16_tail<QB>(dP); stage2<E2, D, QB, true>(XK, qbuf, dP, lane); }
        if constexpr (E2::EPL == 8 && EA_BWD_SPLIT >= SPLIT_ALL) { f16_tail<QB>(S); stage2<E2, D, QB, true>(XV, gbuf, S, lane); }
    };
    if constexpr (E::EPL == 8 && QB == 1 && NBUF == 2) {
        // query tiles on the diagonal (the head of the ascending list), and one more when that makes
        // their number even, take the plain body; all tiles wholly below it the staggered one
        int ndiag = 0;
        if (p.causal)
            while (ndiag < ntl && (long)(tl[ndiag] & 0xffff) * 64 < k0 + BC - 1) ++ndiag;
        const Frag1<E, D> frag1(lane);
        const Frag2<E2, D> frag2(lane);
        stream_tiles_split(min(ntl, (ndiag + 1) & ~1), ntl, set0, set1, issue_qg, tile_plain_order,
            [&](int it, const char* qbuf) {
                if (!((tl[it] >> (16 + mycol)) & 1)) return;
                ++ntile_done;
                const float* tau_s = (const float*)(qbuf + VEC_OFF);
                dkdv_tile_staggered<E, E2, D, AM, EA_BWD_SPLIT>(qbuf, qbuf + SM::RBYTES, tau_s, tau_s + TILE, kf, vf, XV, XK, r, h, frag1, frag2);
            });
    } else {
        stream_tiles<NBUF>(ntl, set0, NBUF == 2 ? set1 : set0, issue_qg, tile_plain_order);
    }
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) { settle_acc(XV[db][qb]); settle_acc(XK[db][qb]); }
    if (active) {
        if (!shared_out) {
            store_owned_T<D, QB>(p.dV + hoff, kw0, XV, go_amax * hc.rho_p, lane);
            store_owned_T<D, QB>(p.dK + hoff, kw0, XK, p.inv_sqrt_d * go_amax * hc.rho_u, lane);
        } else {
            add_owned_T<D, QB>(p.dV + hoff, kw0, XV, go_amax * hc.rho_p, lane);
            add_owned_T<D, QB>(p.dK + hoff, kw0, XK, p.inv_sqrt_d * go_amax * hc.rho_u, lane);
        }
    }
    {
        const int slot[1] = {4};
        const unsigned long long val[1] = {ntile_done * QB};
        flush_counters<1>(blk_stats, p.stats, slot, val, tid, lane);
    }
}

// ---- backward of sparse row groups by gather --------------------------------------------------
// Where a row's support is a handful of keys, most tiles the mask marks hold one or two non-zeros,
// and the four matrix products per tile of dq_kernel / dkdv_kernel are spent on zeros.  For such
// row groups the backward of Sec. 3.3 is evaluated entry by entry instead:
//   bwd_list_kernel : one matrix product per marked tile (the scores); every score above the
//                     row's tau goes, with its key index, to a list private to the lane that
//                     computed it (two lists per row, as in tau_list_kernel).  A group whose
//                     lists stay short is flagged; dq_kernel and dkdv_kernel skip flagged groups.
//   bwd_rows_kernel : per row, over its listed support: dP_j = <dO_r, V_j>, delta, and
//                     dQ_r = sum_j dS_j K_j / sqrt(d) (Alg. 3, row by row); every entry is also
//                     filed under its key: (row, u dP, u, P).
//   bwd_cols_kernel : per key, over the entries filed under it, with dS = u dP - u delta_row:
//                     dK_j += sum dS Q_r / sqrt(d), dV_j += sum P dO_r (Alg. 2, column by
//                     column), added to what dkdv_kernel
//                     stored for the other row groups (or, when none was left to it, written as
//                     dK_j, dV_j themselves).
//   bwd_hot_kernel  : the entries of keys with more entries than a key's list holds, added to
//                     dK, dV with atomics after bwd_cols_kernel.
// All three read the caller's Q, K, V, dO (not the 16-bit copies) and work in fp32.
// The gather path pays while a marked 64 x 64 tile holds only a few non-zeros: the group is flagged
// when its lists hold at most BWD_ENTRIES_PER_TILE entries per marked tile (and no list is full);
// or BWD_ENTRIES_PER_ROW per row (and no list is full); the sweep is left early once the entries
// so far run a quarter above that rate.
template <class E, int D, int QB, int AM, int NW>
__global__ __launch_bounds__(NW * 64) void bwd_list_kernel(Params p) {
    using elem = typename E::elem;
    using KT = RowTile<E, D>;
    constexpr int BR = 32 * QB * NW, MR = (BR + 63) / 64, THREADS = NW * 64;
    __shared__ __align__(1024) char set0[KT::BYTES];
    __shared__ __align__(1024) char set1[KT::BYTES];
    __shared__ uint32_t fm[MR * MAX_W];
    __shared__ unsigned short tl[MAX_T];
    __shared__ int tl_count[4];
    __shared__ int gsum[4];                  // [0] support entries so far, [1] marked tiles, [2] a list is full, [3] the group's decision to leave
    __shared__ unsigned long long blk_stats[4];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, h = lane >> 5;
    const int N = p.N, T = p.T, W = p.W;
    int bh, I;
    map_block(blockIdx.x, p.BH, (N + BR - 1) / BR, bh, I);
    const long q0 = (long)I * BR, qw0 = q0 + wave * 32 * QB;
    const bool active = qw0 < N;
    const elem* Qh = (const elem*)p.Q + (long)bh * N * D;
    const elem* Kh = (const elem*)p.K + (long)bh * N * D;
    const int myrow = (wave * 32 * QB) / 64;
    const HeadConsts hc = head_consts(p, bh);
    const float c = hc.c;

    // a mask with few marked tiles altogether: the matrix kernels are done before the gather
    // kernels' passes over dK, dV would be
    if ((long)*p.nmarked * D < (long)BWD_MIN_TILES_PER_BLOCK * 128 * p.BH * T) {
        if (tid == 0) {
            p.gflag[(long)bh * ((N + BR - 1) / BR) + I] = 0;
            atomicAdd(p.nplain, 1);
        }
        return;
    }
    if (tid < 4) gsum[tid] = 0;
    __syncthreads();
    {
        int marked = 0;
        for (int i = tid; i < MR * W; i += THREADS) {
            fm[i] = (I * MR + i / W < T) ? (uint32_t)p.mask[((long)bh * T + (long)I * MR + i / W) * W + (i % W)] : 0u;
            marked += __popc(fm[i]);
        }
        if (marked) atomicAdd(&gsum[1], marked);
    }
    build_tile_list(fm, MR, W, tl, tl_count, tid);
    const int nt = *tl_count;
    // entries the whole group may list (a group with few marked tiles - the first rows of a causal
    // head - still has one entry or more per row, and is cheap either way: it goes with the rest,
    // so that the matrix kernels' input copies are not made for its sake alone)
    // (the matrix kernels' time per tile goes with D, the gather's time per entry hardly does -
    // measured break-even: about 32 entries per tile at D = 128, 8 at D = 64; the power functions
    // of general alpha weigh on every entry)
    constexpr int PER_TILE_X128 = BWD_ENTRIES_PER_TILE * D * D / 128 / (AM == ALPHA_GEN ? 2 : 1);
    constexpr int PER_ROW_X128 = BWD_ENTRIES_PER_ROW * D * D / 128 / (AM == ALPHA_GEN ? 2 : 1);
    const int budget = max(PER_TILE_X128 * gsum[1] / 128,
                           gsum[1] <= BWD_FEW_TILES ? PER_ROW_X128 * min(BR, N - (int)((long)I * BR)) / 128 : 0);

    Owned<E, D, QB> qf;
    load_owned<E, D, QB>(qf, Qh, active ? qw0 : 0, lane);
    float thr[QB], floor_raw[QB];
    char* lptr[QB];
    int cnt[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        thr[qb] = active ? p.tau[(long)bh * N + qw0 + 32 * qb + n] : INFINITY;
        const float thr_raw = thr[qb] / c;   // a score passes only if it is above about this
        floor_raw[qb] = thr_raw - (1e-5f * fabsf(thr_raw) + 1e-30f);
        lptr[qb] = (char*)p.lists + ((size_t)((long)bh * N + (active ? qw0 : 0) + 32 * qb + n) * 2 + h) * (size_t)(BWD_LIST_CAP * 8);
        cnt[qb] = 0;
    }
    unsigned long long ntile = 0;
    f32x16 C[2][QB];
    auto issue = [&](int it, char* buf) { issue_rows<E, D, NW>(buf, Kh, (long)tl[it] * 64, wave, lane); };
    auto compute = [&](int it, const char* buf) {
        const int j = tl[it];
        if (!active || !mask_bit(fm, W, myrow, j)) return;
        stage1<E, D, QB, EA_FENCE, 0>(C, buf, qf, lane);    // rolling fragments (registers of two k-steps): four waves per SIMD fit
        if (p.causal && (long)j * 64 + 63 > qw0) causal_hide<QB, true>(C, j * 64, (int)qw0, lane);
        ++ntile;
        const int key0 = j * 64 + 8 * h;
        bool full = false;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float gm[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                gm[g] = C[g >> 1][qb][8 * (g & 1)];
#pragma unroll
                for (int v = 1; v < 8; ++v) gm[g] = fmaxf(gm[g], C[g >> 1][qb][8 * (g & 1) + v]);
            }
            const float lm = fmaxf(fmaxf(gm[0], gm[1]), fmaxf(gm[2], gm[3]));
            if (!__any(lm > floor_raw[qb])) continue;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                if (!__any(gm[g] > floor_raw[qb])) continue;
#pragma unroll
                for (int v = 0; v < 8; ++v) {
                    const float sc = C[g >> 1][qb][8 * (g & 1) + v];
                    if (fmaf(c, sc, -thr[qb]) > 0.f) {
                        uint2 ent;          // tile row of register v of group g: see causal_hide
                        ent.x = __float_as_uint(sc); ent.y = (uint32_t)(key0 + 32 * (g >> 1) + 16 * (g & 1) + v);
                        *(uint2*)(lptr[qb] + 8 * min(cnt[qb], BWD_LIST_CAP - 1)) = ent;
                        ++cnt[qb];
                        lds_add_u32(&gsum[0], 1u);
                    }
                }
            }
            full |= cnt[qb] > BWD_LIST_CAP;
        }
        if (__any(full) && lane == 0) atomicOr(&gsum[2], 1);
    };
    // the walk of stream_tiles, left as soon as the gather path cannot pay any more.  The counters
    // keep moving while the waves of a group work on a tile, so the group's decision is taken by
    // one thread, from the values it finds right after a barrier, and published in gsum[3]; every
    // wave reads it after the NEXT barrier, before which nobody writes it again: all waves leave
    // at the same tile, or none does.
    auto hopeless = [&](int it) {
        if (*(volatile int*)&gsum[2]) return true;
        const int e = *(volatile int*)&gsum[0];
        return e > budget || (it >= 8 && 4l * e * nt > 5l * budget * it);
    };
    bool gave_up = false;
    if (nt > 0) issue(0, set0);
    for (int it = 0; it < nt; it += 2) {
        wait_loads();
        __syncthreads();
        if ((it & 7) == 0 && tid == 0) gsum[3] = hopeless(it);
        if (it + 1 < nt) issue(it + 1, set1);
        compute(it, set0);
        if (it + 1 >= nt) break;
        wait_loads();
        __syncthreads();
        if ((it & 7) == 0 && *(volatile int*)&gsum[3]) { gave_up = true; break; }
        if (it + 2 < nt) issue(it + 2, set0);
        compute(it + 1, set1);
    }
    lds_settle();            // this wave's counter updates have reached LDS
    wait_loads();
    __syncthreads();
    if (tid == 0) gsum[3] = gave_up || hopeless(nt);
    __syncthreads();
    const int nrows = min(BR, N - (int)q0);
    const bool gather = !*(volatile int*)&gsum[3];
    if (active) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) p.scnt[((long)bh * N + qw0 + 32 * qb + n) * 2 + h] = gather ? cnt[qb] : 0;
    }
    if (tid == 0) {
        p.gflag[(long)bh * ((N + BR - 1) / BR) + I] = gather;
        if (!gather) atomicAdd(p.nplain, 1);
    }
    {
        const int slot[2] = {10, 11};
        const unsigned long long val[2] = {ntile * QB, (tid == 0 && gather) ? (unsigned long long)nrows : 0ull};
        flush_counters<2>(blk_stats, p.stats, slot, val, tid, lane);
    }
}

// When the caller hands the forward's workspace to the backward, the supports need not be found
// again: for the row groups whose output the forward gathered, the front of its candidate lists is
// the support (raw score, key index), with the counts beside it.  This kernel takes the place of
// bwd_list_kernel's sweep: per row group of the backward it applies the same rule - at most so many
// support entries per marked tile, or per row where few tiles are marked - to the forward's counts.
template <int D, int AM>
__global__ __launch_bounds__(128) void bwd_decide_kernel(Params p) {
    __shared__ int gsum[2];
    const int tid = threadIdx.x;
    const int N = p.N, T = p.T, W = p.W, BR = p.grows, G = (N + BR - 1) / BR;
    int bh, I;
    map_block(blockIdx.x, p.BH, G, bh, I);
    const int fwd_grows = (int)p.fwd_scal[2];
    bool gather = (long)*p.nmarked * D >= (long)BWD_MIN_TILES_PER_BLOCK * 128 * p.BH * T && fwd_grows > 0
                  && p.fwd_gflag[(long)bh * ((N + fwd_grows - 1) / fwd_grows) + (I * BR) / fwd_grows] != 0;
    if (tid < 2) gsum[tid] = 0;
    __syncthreads();
    if (gather) {
        const int row = I * BR + tid;
        int ent = 0, marked = 0;
        if (tid < BR && row < N) ent = p.scnt[((long)bh * N + row) * 2] + p.scnt[((long)bh * N + row) * 2 + 1];
        const int MR = (BR + 63) / 64;
        for (int i = tid; i < MR * W; i += 128)
            if (I * MR + i / W < T) marked += __popc((uint32_t)p.mask[((long)bh * T + (long)I * MR + i / W) * W + (i % W)]);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) { ent += __shfl_xor(ent, off); marked += __shfl_xor(marked, off); }
        if ((tid & 63) == 0) { atomicAdd(&gsum[0], ent); atomicAdd(&gsum[1], marked); }
    }
    __syncthreads();
    if (tid == 0) {
        constexpr int PER_TILE_X128 = BWD_ENTRIES_PER_TILE * D * D / 128 / (AM == ALPHA_GEN ? 2 : 1);
        constexpr int PER_ROW_X128 = BWD_ENTRIES_PER_ROW * D * D / 128 / (AM == ALPHA_GEN ? 2 : 1);
        const int budget = max(PER_TILE_X128 * gsum[1] / 128,
                               gsum[1] <= BWD_FEW_TILES ? PER_ROW_X128 * min(BR, N - I * BR) / 128 : 0);
        gather = gather && gsum[0] <= budget;
        p.gflag[(long)bh * G + I] = gather;
        if (!gather) atomicAdd(p.nplain, 1);
        else atomicAdd(&p.stats[(blockIdx.x & (STATS_COPIES - 1)) * STATS_WORDS + 11], (unsigned long long)min(BR, N - I * BR));
    }
}

// Sixteen lanes per row; lane `sub` holds elements [sub * D/16, (sub + 1) * D/16) of the row's
// vectors.  SCALED: dkdv_kernel works on dO / max|dO|, so the delta handed to it is in those units.
template <class E, int D, int AM, bool SCALED>
__global__ __launch_bounds__(256) void bwd_rows_kernel(Params p) {
    using elem = typename E::elem;
    constexpr int EPT = D / 16, CH = 2;      // entries in flight per lane group
    typedef elem vvec __attribute__((ext_vector_type(EPT)));
    typedef float ovec __attribute__((ext_vector_type(4)));
    const int tid = threadIdx.x, sub = tid & 15, rsel = tid >> 4;
    // a work-group takes GATHER_ROWS rows of a row group (one or a few per 16 lanes): the rows are
    // chains of dependent loads, so many short work-groups hide their latency better than few long ones
    const int N = p.N, G = (N + p.grows - 1) / p.grows, parts = p.grows / GATHER_ROWS;
    int bh, I;
    map_block(blockIdx.x, p.BH, G * parts, bh, I);
    const int part = I % parts;
    I /= parts;
    if (!p.gflag[(long)bh * G + I]) return;
    const HeadConsts hc = head_consts(p, bh);
    const float c = hc.c, r = hc.r;
    float amax = 1.f;
    if constexpr (SCALED) {
        amax = __uint_as_float(p.scal[0]);
        if (!(amax > 0.f)) amax = 1.f;
    }
    const long hoff = (long)bh * N * D;
    const elem* Qh = (const elem*)p.Q + hoff;
    const elem* Kh = (const elem*)p.K + hoff + sub * EPT;
    const elem* Vh = (const elem*)p.V + hoff + sub * EPT;
    const elem* Gh = (const elem*)p.dO + hoff;
    const int cap8 = p.list_cap * 8;         // bytes of one lane list
    const char* lists_h = (const char*)p.lists + (size_t)bh * N * (size_t)(2 * cap8);
    const int row_end = min(N, I * p.grows + (part + 1) * GATHER_ROWS);
    for (int row = I * p.grows + part * GATHER_ROWS + rsel; row < row_end; row += 16) {
        const long gi = (long)bh * N + row;
        const float tau = p.tau[gi];
        const int s0 = p.scnt[gi * 2], tot = s0 + p.scnt[gi * 2 + 1];
        const char* l0 = lists_h + (size_t)row * (size_t)(2 * cap8);     // the second list follows the first
        auto entry = [&](int i) { return *(const uint2*)(l0 + (i < s0 ? i * 8 : cap8 + (i - s0) * 8)); };
        const vvec gv = *(const vvec*)(Gh + (long)row * D + sub * EPT);
        float g[EPT];
#pragma unroll
        for (int k = 0; k < EPT; ++k) g[k] = (float)gv[k];
        // One pass over the entries, CH at a time so that their chains of dependent memory
        // operations (entry, rows of V and K, slot in the key's list) overlap:
        //   delta = sum u dP / sum u, and the two sums dQ is made of:
        //   dQ sqrt(d) = sum_j u_j (dP_j - delta) K_j = XA - delta XB;
        // every entry is filed under its key as (row, u dP, u, P): dS = u dP - u delta is formed
        // by bwd_cols_kernel, which reads the row's delta once this kernel has stored it.  An
        // entry whose key's list is full is marked (top bit of its key index) and left to
        // bwd_hot_kernel, which adds it to dK, dV atomically once bwd_cols_kernel has stored them.
        float xa[EPT], xb[EPT], num = 0.f, den = 0.f;
        int ndefer = 0;
#pragma unroll
        for (int k = 0; k < EPT; ++k) { xa[k] = 0.f; xb[k] = 0.f; }
        for (int i0 = 0; i0 < tot; i0 += CH) {
            uint2 e[CH];
            vvec vv[CH], kv[CH];
            int slot[CH];
#pragma unroll
            for (int u = 0; u < CH; ++u) e[u] = i0 + u < tot ? entry(i0 + u) : make_uint2(0u, 0u);
#pragma unroll
            for (int u = 0; u < CH; ++u) {
#pragma unroll
                for (int k = 0; k < EPT; ++k) { vv[u][k] = (elem)0.f; kv[u][k] = (elem)0.f; }
                slot[u] = 0;
                if (i0 + u < tot) {
                    vv[u] = *(const vvec*)(Vh + (long)e[u].y * D);
                    kv[u] = *(const vvec*)(Kh + (long)e[u].y * D);
                    if (sub == 0) slot[u] = atomicAdd(&p.kcnt[(long)bh * N + e[u].y], 1);
                }
            }
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                float dot = 0.f;
#pragma unroll
                for (int k = 0; k < EPT; ++k) dot = fmaf(g[k], (float)vv[u][k], dot);
                const float dP = group_sum<16>(dot);
                const float y = fmaf(c, __uint_as_float(e[u].x), -tau);
                const bool in = i0 + u < tot && y > 0.f;
                const float uu = in ? pow_r1<AM>(y, r) : 0.f;
                const float pr = in ? pow_r<AM>(y, r) : 0.f;
                const float t = uu * dP;
                num += t; den += uu;
#pragma unroll
                for (int k = 0; k < EPT; ++k) { xa[k] = fmaf(t, (float)kv[u][k], xa[k]); xb[k] = fmaf(uu, (float)kv[u][k], xb[k]); }
                const int sl = __shfl(slot[u], (tid & 63) & ~15);
                if (i0 + u < tot) {
                    if (sl < KEY_LIST_CAP) {
                        if (sub == 0)
                            ((uint4*)p.klist)[((long)bh * N + e[u].y) * KEY_LIST_CAP + sl] =
                                make_uint4((uint32_t)row, __float_as_uint(t), __float_as_uint(uu), __float_as_uint(pr));
                    } else {
                        const int i = i0 + u;
                        if (sub == 0)
                            *(uint32_t*)(const_cast<char*>(l0) + (i < s0 ? i * 8 : cap8 + (i - s0) * 8) + 4) = e[u].y | 0x80000000u;
                        ++ndefer;
                    }
                }
            }
        }
        const float delta = den > 0.f ? num / den : 0.f;
        {
            float* out = p.dQ + gi * D + sub * EPT;
#pragma unroll
            for (int k = 0; k < EPT; k += 4)
                *(ovec*)(out + k) = ovec{(xa[k] - delta * xb[k]) * p.inv_sqrt_d, (xa[k + 1] - delta * xb[k + 1]) * p.inv_sqrt_d,
                                         (xa[k + 2] - delta * xb[k + 2]) * p.inv_sqrt_d, (xa[k + 3] - delta * xb[k + 3]) * p.inv_sqrt_d};
        }
        if (sub == 0) {
            p.delta[gi] = -delta / amax;
            p.ntau[gi] = -tau / hc.rho;
        }
        if (sub == 0) p.defer[gi] = ndefer;
    }
}

// The entries bwd_rows_kernel marked: keys that more rows attend to than a key's list holds.  Run
// after bwd_cols_kernel; sixteen lanes per row recompute the entry's dS and P (delta is the row's
// stored one) and add its share to the key's rows of dK, dV with fp32 atomics, lane-interleaved
// (lane `sub` takes elements sub, sub + 16, ...: an instruction then covers whole 64-byte pieces).
template <class E, int D, int AM, bool SCALED>
__global__ __launch_bounds__(256) void bwd_hot_kernel(Params p) {
    using elem = typename E::elem;
    constexpr int EPT = D / 16;
    typedef elem vvec __attribute__((ext_vector_type(EPT)));
    const int tid = threadIdx.x, sub = tid & 15, rsel = tid >> 4;
    // a work-group takes GATHER_ROWS rows of a row group (one or a few per 16 lanes): the rows are
    // chains of dependent loads, so many short work-groups hide their latency better than few long ones
    const int N = p.N, G = (N + p.grows - 1) / p.grows, parts = p.grows / GATHER_ROWS;
    int bh, I;
    map_block(blockIdx.x, p.BH, G * parts, bh, I);
    const int part = I % parts;
    I /= parts;
    if (!p.gflag[(long)bh * G + I]) return;
    const HeadConsts hc = head_consts(p, bh);
    const float c = hc.c, r = hc.r;
    float amax = 1.f;
    if constexpr (SCALED) {
        amax = __uint_as_float(p.scal[0]);
        if (!(amax > 0.f)) amax = 1.f;
    }
    const long hoff = (long)bh * N * D;
    const elem* Qh = (const elem*)p.Q + hoff;
    const elem* Vh = (const elem*)p.V + hoff + sub * EPT;
    const elem* Gh = (const elem*)p.dO + hoff;
    const int cap8 = p.list_cap * 8;
    const char* lists_h = (const char*)p.lists + (size_t)bh * N * (size_t)(2 * cap8);
    const int row_end = min(N, I * p.grows + (part + 1) * GATHER_ROWS);
    for (int row = I * p.grows + part * GATHER_ROWS + rsel; row < row_end; row += 16) {
        const long gi = (long)bh * N + row;
        if (p.defer[gi] == 0) continue;
        const float tau = p.tau[gi], delta = -p.delta[gi] * amax;
        const int s0 = p.scnt[gi * 2], tot = s0 + p.scnt[gi * 2 + 1];
        char* l0 = const_cast<char*>(lists_h) + (size_t)row * (size_t)(2 * cap8);
        const vvec gv = *(const vvec*)(Gh + (long)row * D + sub * EPT);
        for (int i = 0; i < tot; ++i) {
            char* ep = l0 + (i < s0 ? i * 8 : cap8 + (i - s0) * 8);
            const uint2 e = *(const uint2*)ep;
            if (!(e.y >> 31)) continue;
            const uint32_t key = e.y & 0x7fffffffu;
            // the mark comes off again: the lists are left as they were found (they may be the forward's)
            if (sub == 0) *(uint32_t*)(ep + 4) = key;
            const vvec vv = *(const vvec*)(Vh + (long)key * D);
            float dot = 0.f;
#pragma unroll
            for (int k = 0; k < EPT; ++k) dot = fmaf((float)gv[k], (float)vv[k], dot);
            const float dP = group_sum<16>(dot);
            const float y = fmaf(c, __uint_as_float(e.x), -tau);
            const float uu = y > 0.f ? pow_r1<AM>(y, r) : 0.f;
            const float pr = y > 0.f ? pow_r<AM>(y, r) : 0.f;
            const float ds = uu * (dP - delta) * p.inv_sqrt_d;
            float* dk = p.dK + ((long)bh * N + key) * D + sub;
            float* dv = p.dV + ((long)bh * N + key) * D + sub;
#pragma unroll
            for (int k = 0; k < EPT; ++k) {
                unsafeAtomicAdd(dk + 16 * k, ds * (float)Qh[(long)row * D + sub + 16 * k]);
                unsafeAtomicAdd(dv + 16 * k, pr * (float)Gh[(long)row * D + sub + 16 * k]);
            }
        }
    }
}

// Sixteen lanes per key.  Where dkdv_kernel has stored dK, dV for the other row groups, the key's
// rows are read, added to, and written back; when no row group was left to dkdv_kernel (it then
// stores nothing) the sums are the rows, and keys without entries get zeros.
template <class E, int D, bool SCALED>
__global__ __launch_bounds__(256) void bwd_cols_kernel(Params p) {
    using elem = typename E::elem;
    constexpr int EPT = D / 16, CH = 4;      // entries in flight per lane group
    typedef elem vvec __attribute__((ext_vector_type(EPT)));
    typedef float ovec __attribute__((ext_vector_type(4)));
    const int tid = threadIdx.x, sub = tid & 15, rsel = tid >> 4;
    const int N = p.N, G = (N + BWD_COLS_KEYS - 1) / BWD_COLS_KEYS;
    int bh, I;
    map_block(blockIdx.x, p.BH, G, bh, I);
    const long hoff = (long)bh * N * D;
    const elem* Qh = (const elem*)p.Q + hoff + sub * EPT;
    const elem* Gh = (const elem*)p.dO + hoff + sub * EPT;
    const int key_end = min(N, (I + 1) * BWD_COLS_KEYS);
    const bool fresh = *p.nplain == 0;
    float amax = 1.f;                        // the stored deltas are in units of max|dO| (see bwd_rows_kernel)
    if constexpr (SCALED) {
        amax = __uint_as_float(p.scal[0]);
        if (!(amax > 0.f)) amax = 1.f;
    }
    // The entries of a key were filed in the order an integer atomic handed out their slots, which
    // changes from run to run.  They are summed in the order of their query rows instead (a row
    // files at most one entry per key, so the rows are distinct): for a list longer than one batch
    // the rank of every entry among the key's rows, found by the key's 16 lanes through LDS, gives
    // the slot to read at each step (a short list is sorted in registers, below), and
    // dK, dV of a key come out bit-identical in every run (keys with more entries than a list
    // holds get the rest from bwd_hot_kernel's atomic additions and do not).
    __shared__ int rows_s[16][KEY_LIST_CAP];
    __shared__ unsigned char order_s[16][KEY_LIST_CAP];
    constexpr int PER_LANE = KEY_LIST_CAP / 16;      // entries of a key's list per lane of its 16
    static_assert(KEY_LIST_CAP <= 256 && (KEY_LIST_CAP & (KEY_LIST_CAP - 1)) == 0 && KEY_LIST_CAP >= 16, "slot indices are bytes, and masked");
    for (int key = I * BWD_COLS_KEYS + rsel; key < key_end; key += 16) {
        const long kj = (long)bh * N + key;
        const int cnt = min(p.kcnt[kj], KEY_LIST_CAP);
        if (cnt == 0 && !fresh) continue;
        const uint4* el = (const uint4*)p.klist + kj * KEY_LIST_CAP;
        if (cnt > CH) {
            int myrow[PER_LANE], rank[PER_LANE];
#pragma unroll
            for (int q = 0; q < PER_LANE; ++q) {
                const int i = sub + 16 * q;
                myrow[q] = i < cnt ? (int)((const uint32_t*)(el + i))[0] : INT_MAX;
                rank[q] = 0;
                if (i < cnt) rows_s[rsel][i] = myrow[q];
            }
            // (the 16 lanes of a key sit in one wave, whose LDS operations execute in issue order)
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            for (int j = 0; j < cnt; ++j) {
                const int rj = rows_s[rsel][j];
#pragma unroll
                for (int q = 0; q < PER_LANE; ++q) rank[q] += rj < myrow[q];
            }
#pragma unroll
            for (int q = 0; q < PER_LANE; ++q)
                if (sub + 16 * q < cnt) order_s[rsel][rank[q]] = (unsigned char)(sub + 16 * q);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        float ak[EPT], av[EPT];
#pragma unroll
        for (int k = 0; k < EPT; ++k) { ak[k] = 0.f; av[k] = 0.f; }
        for (int i0 = 0; i0 < cnt; i0 += CH) {
            uint4 e[CH];
            vvec qv[CH], gv[CH];
            float nd[CH];                     // -delta / max|dO| of the entry's row
#pragma unroll
            for (int u = 0; u < CH; ++u)
                e[u] = i0 + u < cnt ? el[cnt > CH ? (int)order_s[rsel][i0 + u] & (KEY_LIST_CAP - 1) : u] : make_uint4(0xffffffffu, 0u, 0u, 0u);
            if (cnt <= CH) {
                // a short list is put in row order in registers (no second trip to memory): a
                // sorting network of five exchanges; the unused slots, row 0xffffffff, end up last
                auto exchange = [&](int i, int j) {
                    if (e[j].x < e[i].x) { const uint4 t = e[i]; e[i] = e[j]; e[j] = t; }
                };
                static_assert(CH == 4 || CH == 2, "networks for two and for four entries");
                if constexpr (CH == 4) { exchange(0, 1); exchange(2, 3); exchange(0, 2); exchange(1, 3); exchange(1, 2); }
                else exchange(0, 1);
            }
#pragma unroll
            for (int u = 0; u < CH; ++u)
                if (i0 + u >= cnt) e[u] = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
            for (int u = 0; u < CH; ++u) {
#pragma unroll
                for (int k = 0; k < EPT; ++k) { qv[u][k] = (elem)0.f; gv[u][k] = (elem)0.f; }
                nd[u] = 0.f;
                if (i0 + u < cnt) {
                    qv[u] = *(const vvec*)(Qh + (long)e[u].x * D);
                    gv[u] = *(const vvec*)(Gh + (long)e[u].x * D);
                    nd[u] = p.delta[(long)bh * N + e[u].x];
                }
            }
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                // dS = u dP - u delta; P (all zero past the end)
                const float dS = fmaf(__uint_as_float(e[u].z), nd[u] * amax, __uint_as_float(e[u].y)), pr = __uint_as_float(e[u].w);
#pragma unroll
                for (int k = 0; k < EPT; ++k) { ak[k] = fmaf(dS, (float)qv[u][k], ak[k]); av[k] = fmaf(pr, (float)gv[u][k], av[k]); }
            }
        }
        float* dk = p.dK + kj * D + sub * EPT;
        float* dv = p.dV + kj * D + sub * EPT;
#pragma unroll
        for (int k = 0; k < EPT; k += 4) {
            ovec a = ovec{0.f, 0.f, 0.f, 0.f}, b = a;
            if (!fresh) { a = *(ovec*)(dk + k); b = *(ovec*)(dv + k); }
#pragma unroll
            for (int q = 0; q < 4; ++q) { a[q] = fmaf(ak[k + q], p.inv_sqrt_d, a[q]); b[q] += av[k + q]; }
            *(ovec*)(dk + k) = a;
            *(ovec*)(dv + k) = b;
        }
    }
}

static __global__ void mask_popcount_kernel(const int32_t* mask, long nwords, int32_t* out) {
    int c = 0;
    for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < nwords; i += (long)gridDim.x * blockDim.x) c += __popc((uint32_t)mask[i]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) c += __shfl_xor(c, off);
    if ((threadIdx.x & 63) == 0 && c) atomicAdd(out, c);
}

static __global__ void zero_ints_kernel(int32_t* x, long n) {
    for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) x[i] = 0;
}

}  // namespace ea
