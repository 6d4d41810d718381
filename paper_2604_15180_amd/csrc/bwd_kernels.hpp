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
    const long hoff = (long)bh * N * D;
    const elem* Kh = (const elem*)p.K + hoff;
    const elem* Vh = (const elem*)p.V + hoff;
    const int myrow = (wave * 32 * QB) / 64;
    const float c = p.c, r = p.r;

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
    float num[QB], den[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) num[qb] = den[qb] = 0.f;
    stream_tiles<NBUF>(
        *tl_count, set0, NBUF == 2 ? set1 : set0,
        [&](int it, char* b) {
            const long j = tl[it];
            issue_rows<E, D, NW>(b, Kh, j * 64, wave, lane);
            issue_rows<E, D, NW>(b + SM::RBYTES, Vh, j * 64, wave, lane);
        },
        [&](int it, const char* kbuf) {
            const int j = tl[it];
            if (!mask_bit(fm, W, myrow, j)) return;
            const char* vbuf = kbuf + SM::RBYTES;
            stage1<E, D, QB>(S, kbuf, qf, lane);
            if (p.causal && (long)j * 64 + 63 > qw0) causal_hide<QB, true>(S, j * 64, (int)qw0, lane);
            stage1<E, D, QB>(dP, vbuf, gf, lane);
            ++ntile;
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
        });
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) { settle_acc(XA[db][qb]); settle_acc(XB[db][qb]); }

    // delta (in units of max|dO|) for the dK/dV kernel, and the combination of the two sums
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float dn = xhalf_sum(den[qb]);
        const float drel = dn > 0.f ? xhalf_sum(num[qb]) / dn : 0.f;      // delta - e
        if (h == 0 && active) p.delta[(long)bh * N + qw0 + 32 * qb + n] = drel + ctr[qb];
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
    map_block(blockIdx.x, p.BH, (N + BC - 1) / BC, bh, J);
    J = (N + BC - 1) / BC - 1 - J;            // causal: the first key tiles have the longest columns
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
    const float c = p.c, r = p.r;

    // ---- column walk of the row-packed mask: list of query tiles with a set bit -------------
    const int i_min = p.causal ? jc0 : 0;
    if (tid == 0) wcnt[8] = 0;
    __syncthreads();
    for (int base = i_min; base < T; base += THREADS) {
        const int i = base + tid;
        int flags = 0;
        if (i < T) {
#pragma unroll
            for (int cidx = 0; cidx < MC; ++cidx) {
                const int j = jc0 + cidx;
                if (j >= T) continue;
                const uint32_t w = (uint32_t)p.mask[((long)bh * T + i) * W + (j >> 5)];
                flags |= (int)((w >> (j & 31)) & 1u) << cidx;
            }
        }
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
    const int ntl = wcnt[8];

    Owned<E, D, QB> kf, vf;
    load_owned<E, D, QB>(kf, (const elem*)p.K + hoff, active ? kw0 : 0, lane);
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
    stream_tiles<NBUF>(
        ntl, set0, NBUF == 2 ? set1 : set0,
        [&](int it, char* b) {
            const long i = __builtin_amdgcn_readfirstlane(tl[it] & 0xffff);
            issue_rows<E, D, NW>(b, Qh, i * 64, wave, lane);
            issue_rows<E, D, NW>(b + SM::RBYTES, Gh, i * 64, wave, lane);
            // the tile's 64 thresholds (wave 0) and 64 deltas (wave 1), one float per lane
            if (wave == 0) load4_to_lds(uniform_address(p.tau + ((long)bh * N + i * 64)), 4u * lane, lds_address(b + VEC_OFF));
            if (wave == 1) load4_to_lds(uniform_address(p.delta + ((long)bh * N + i * 64)), 4u * lane, lds_address(b + VEC_OFF + 4 * TILE));
        },
        [&](int it, const char* qbuf) {
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
                            const float yp = fmaxf(fmaf(c, S[kb][qb][v], -tq), 0.f);
                            float u;
                            if constexpr (AM == ALPHA_15) u = yp;
                            else u = (yp > 0.f) ? pow_r1<AM>(yp, r) : 0.f;
                            S[kb][qb][v] = u * yp;
                            dP[kb][qb][v] = u * (dP[kb][qb][v] - dq);
                        }
                    }
                }
            stage2<E2, D, QB, true>(XV, gbuf, S, lane);
            stage2<E2, D, QB, true>(XK, qbuf, dP, lane);
        });
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) { settle_acc(XV[db][qb]); settle_acc(XK[db][qb]); }
    if (active) {
        store_owned_T<D, QB>(p.dV + hoff, kw0, XV, go_amax, lane);
        store_owned_T<D, QB>(p.dK + hoff, kw0, XK, p.inv_sqrt_d * go_amax, lane);
    }
    {
        const int slot[1] = {4};
        const unsigned long long val[1] = {ntile_done * QB};
        flush_counters<1>(blk_stats, p.stats, slot, val, tid, lane);
    }
}

}  // namespace ea
