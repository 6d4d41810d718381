// Forward kernels (Alg. 1 of the AdaSplash-2 paper), re-cut for CDNA4:
//   tau_kernel : Phases 1 and 2 in one dense sweep (row maximum, LDS histogram of the scores within
//                one unit of the running maximum, per-row tile maxima), histogram solve -> tau_0,
//                candidate tiles (those holding a score above tau_0), first Phase-3 sweep over them
//                (f, f', f'' at tau_0, one safeguarded Halley/Newton step, working mask at tau_0)
//   out_kernel : Phase 4 (O = P V over the working mask), which is also the next evaluation of f;
//                further refinement only for rows that fail it; exported mask at the final tau
// One work-group = 32*QB*NW query rows of one head; wave w owns rows 32*QB*w .. of them as MFMA
// B operands in registers; 64-key tiles of K (and V) stream through LDS.
#pragma once
#include <type_traits>

#include "common.hpp"

namespace ea {

// ---- histogram solve (App. C.3), one thread per row ------------------------------------------
// The row's histogram is a window of SLOTS consecutive bins of an absolute grid of width h,
// kept in a circular buffer: bin k of the window (left edge k h above the window's origin) is
// H[(rot + k) % SLOTS].  Returns the root tau_h of f_h(tau) = -1 + sum_k H_k [k h - tau]_+^r
// (Eq. 9) in units above the origin; -h for an empty histogram.
template <int AM, int SLOTS, int BITS>
EA_DEV float solve_histogram(const uint32_t* H, int rot, int shift, float h, float r) {
    // counters of BITS bits at bit `shift` of each word (two rows share a word when BITS == 16)
    auto count = [&](int k) {
        const uint32_t w = H[(rot + k) & (SLOTS - 1)] >> shift;
        return (float)(BITS == 32 ? w : (w & ((1u << (BITS & 31)) - 1u)));
    };
    if constexpr (AM == ALPHA_15 || AM == ALPHA_20) {
        // Descending scan keeping S0, S1, S2 of the bins met so far.  The active set is the largest
        // one whose root lies below the left edge e of its lowest non-empty bin, i.e. (f_h falls
        // with tau) the largest one with f_h(e) < 0; f_h(e) is a polynomial in the three sums, so
        // the scan needs no division, and the root is formed once, from the sums of that set.
        float S0 = 0.f, S1 = 0.f, S2 = 0.f, B0 = 0.f, B1 = 0.f, B2 = 0.f;
#pragma unroll 8
        for (int k = SLOTS - 1; k >= 0; --k) {
            const float cnt = count(k);
            const float e = k * h;
            S0 += cnt; S1 = fmaf(cnt, e, S1); S2 = fmaf(cnt * e, e, S2);
            float fe;
            if constexpr (AM == ALPHA_20) fe = S1 - e * S0 - 1.f;
            else fe = fmaf(e, fmaf(e, S0, -2.f * S1), S2) - 1.f;
            if (cnt > 0.f && fe < 0.f) { B0 = S0; B1 = S1; B2 = S2; }
        }
        if (B0 == 0.f) return -h;
        if constexpr (AM == ALPHA_20) return (B1 - 1.f) / B0;
        const float mean = B1 / B0;
        return mean - sqrtf(fmaxf(mean * mean - (B2 - 1.f) / B0, 0.f));
    } else {
        // general alpha: bisection of f_h on [-h, (SLOTS-1) h]; for alpha <= 2 then Newton from the
        // left end (f_h is convex and decreasing there, so Newton from the left is monotone and
        // stays at or below the root); for alpha > 2 f_h is not convex, so the bisection is run
        // further instead and its left end, where f_h >= 0, is returned
        auto eval = [&](float tau, float& f1) {
            float f = -1.f; f1 = 0.f;
            for (int k = SLOTS - 1; k >= 0; --k) {
                const float y = k * h - tau;
                if (y <= 0.f) break;
                const float cnt = count(k);
                if (cnt == 0.f) continue;
                const float pr1 = pow_r1<AM>(y, r);
                f += cnt * pr1 * y;
                f1 -= cnt * r * pr1;
            }
            return f;
        };
        float lo = -h, hi = (SLOTS - 1) * h, d1;
        const int nbis = r < 1.f ? 22 : 12;
        for (int i = 0; i < nbis; ++i) {
            const float mid = 0.5f * (lo + hi);
            if (eval(mid, d1) >= 0.f) lo = mid; else hi = mid;
        }
        float tau = lo;
        for (int i = 0; i < 4 && !(r < 1.f); ++i) {
            const float f = eval(tau, d1);
            if (d1 >= 0.f) break;
            const float nt = tau - f / d1;
            if (!(nt > tau) || nt > hi) break;
            tau = nt;
        }
        return tau;
    }
}

// ---- pieces of the refinement (Sec. 3.2, Phase 3 of Alg. 1) shared by both forward kernels ----
// Accumulate sum y^r, sum y^(r-1), sum y^(r-2) over the scores of one sub-tile that lie above tau
// (alpha = 1.5: the last one is a count; alpha = 2: the middle one is).  Returns whether any did.
template <int AM, int QB>
EA_DEV bool eval_scores(const f32x16 (&C)[2][QB], const float (&thr)[QB], float c, float r, float (&F)[QB],
                        float (&G)[QB], float (&Hs)[QB], int (&cnt)[QB]) {
    bool hit = false;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        float lmax = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) lmax = fmaxf(lmax, C[kb][qb][v]);
        if (__any(fmaf(c, lmax, -thr[qb]) > 0.f)) {
            hit = true;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float y = fmaf(c, C[kb][qb][v], -thr[qb]);
                    if constexpr (AM == ALPHA_15) {
                        const float yp = fmaxf(y, 0.f);
                        F[qb] = fmaf(yp, yp, F[qb]);
                        G[qb] += yp;
                        cnt[qb] += (y > 0.f);
                    } else if constexpr (AM == ALPHA_20) {
                        F[qb] += fmaxf(y, 0.f);
                        cnt[qb] += (y > 0.f);
                    } else {
                        if (y > 0.f) {
                            const float p2 = pow_r2<AM>(y, r);
                            Hs[qb] += p2;
                            G[qb] = fmaf(p2, y, G[qb]);
                            F[qb] = fmaf(p2 * y, y, F[qb]);
                        }
                    }
                }
        }
    }
    return hit;
}

// Stopping length of the refinement at threshold tau: the caller's tolerance, but no less than four
// units in the last place of tau - fp32 thresholds of large scores (|tau| > 2 at tol = 1e-6) cannot
// move by less, and a row would otherwise iterate until its bracket has collapsed.
EA_DEV float step_tol(float tol, float tau) { return fmaxf(tol, 4.8e-7f * fabsf(tau)); }

// The iterate before the current one and its f, for the secant steps of alpha > 2; t is NaN while
// there is none (at the start of a kernel: the state is not carried from one kernel to the next).
struct SecantPrev { float t = __builtin_nanf(""), f = 0.f; };

// One safeguarded hybrid step from (tau, f = F - 1) with G = sum y^(r-1), Hs = sum y^(r-2):
// Halley for alpha <= 1.5, Newton for 1.5 < alpha <= 2, and for alpha > 2, where f' is unbounded
// next to every score (Prop. 2), a secant step through the last two iterates; the bracket's
// midpoint whenever the proposed point leaves (lo, hi) or does not exist (no earlier iterate, or
// f unchanged).  Updates the bracket; returns the proposed threshold.  tol: the callers' stopping
// length, used by the secant branch only.
template <int AM>
EA_DEV float hybrid_step(float tau, float f, float G, float Hs, float r, float alpha, float& lo, float& hi,
                         SecantPrev& prev, float tol) {
    if (f > 0.f) lo = tau; else hi = tau;
    const float f1 = -r * G;
    float delta;
    if (alpha <= 1.5f) {
        const float f2 = r * (r - 1.f) * Hs;
        delta = -2.f * f * f1 / (2.f * f1 * f1 - f * f2);
    } else {
        delta = -f / f1;
    }
    if constexpr (AM == ALPHA_GEN) {
        if (alpha > 2.f) {
            delta = -f * (tau - prev.t) / (f - prev.f);      // NaN or inf when there is no usable secant
            prev.t = tau; prev.f = f;
            // Callers stop when the step is shorter than tol.  Here a short step is no sign of
            // convergence (f rises vertically at every score, so a secant taken on its flat side
            // can be short far from the root): while the bracket is wider than tol such a step is
            // lengthened to 2 tol - either f changes sign, and the bracket is then no wider than
            // that, or the iterate has moved on by as much.  A step shorter than tol is then left
            // only inside a bracket narrower than tol, or as the half of one narrower than 2 tol.
            if (fabsf(delta) < tol && hi - lo >= tol) delta = f > 0.f ? 2.f * tol : -2.f * tol;
        }
    }
    float cand = tau + delta;
    if (!(cand > lo && cand < hi)) cand = 0.5f * (lo + hi);
    return cand;
}

template <class E, int D, int QB, int NB, int NW, int NBUF>
struct TauSmem {
    static constexpr int BR = 32 * QB * NW;
    static constexpr int MR = (BR + 63) / 64;
    // A row's histogram: NB bins per unit of (alpha-1) s on an absolute grid, of which the NB+1
    // bins that reach from one unit below the running maximum up to it are live, in a circular
    // buffer of SLOTS = NB+1 words (a power of two, so NB = 63).
    static constexpr int SLOTS = NB + 1;
    static_assert((SLOTS & (SLOTS - 1)) == 0 && SLOTS * 4 <= 256, "circular index is taken with a byte mask");
    // QB == 2: the two rows of a lane (n and n + 32 of its wave) share the words of one buffer,
    // 16 bits each, so the histograms of 256 rows take the LDS of 128; a bin then holds up to
    // 65535 keys, which the host guarantees by using this variant only while N < 65536.
    static_assert(QB == 1 || QB == 2, "one or two rows per lane");
    static constexpr int CBITS = 32 / QB;
    static constexpr int HIST_WORDS = 32 * NW * SLOTS;
};

template <class E, int D, int QB, int AM, int NB, int NW, int NBUF>
__global__ __launch_bounds__(NW * 64) void tau_kernel(Params p) {
    using SM = TauSmem<E, D, QB, NB, NW, NBUF>;
    using KT = RowTile<E, D>;
    constexpr int THREADS = NW * 64;
    using elem = typename E::elem;
    constexpr int BR = SM::BR, MR = SM::MR, SLOTS = SM::SLOTS;
    // All LDS is static, and the two K buffers are separate variables (see stream_tiles).
    __shared__ __align__(1024) char kbuf[KT::BYTES];
    __shared__ __align__(1024) char kbuf_b[NBUF == 2 ? KT::BYTES : 1024];
    __shared__ __align__(256) uint32_t hist[SM::HIST_WORDS];
    __shared__ uint32_t wm[MR * MAX_W];
    __shared__ uint32_t cand[MR * MAX_W];
    __shared__ int tl[MAX_T];
    __shared__ int tl_count[4];
    __shared__ unsigned long long blk_stats[4];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, h = lane >> 5;
    const int N = p.N, T = p.T, W = p.W;
    int bh, I;
    map_block(blockIdx.x, p.BH, (N + BR - 1) / BR, bh, I);
    const long q0 = (long)I * BR, qw0 = q0 + wave * 32 * QB;
    const bool active = qw0 < N;          // N is a multiple of 64: the last group may be half empty
    if (p.oflag) {
        // run as the fallback of tau_list_kernel: only groups that hold a flagged 64-row block
        int flagged = 0;
        for (int i = 0; i < MR; ++i)
            if (I * MR + i < T) flagged |= p.oflag[(long)bh * T + (long)I * MR + i];
        if (!flagged) return;
    }
    _Float16* tmax_g = p.tmax + (long)bh * T * N;      // [T][N] per-row tile maxima, rounded up
    const elem* Qh = (const elem*)p.Q + (long)bh * N * D;
    const elem* Kh = (const elem*)p.K + (long)bh * N * D;
    const int njt = p.causal ? min((int)((q0 + BR) / 64), T) : T;          // tiles the group streams
    const int wjt = !active ? 0 : p.causal ? (int)((qw0 + 32 * QB - 1) / 64) + 1 : T;   // tiles this wave needs
    const int myrow = (wave * 32 * QB) / 64;                               // my mask row in the group
    const HeadConsts hc = head_consts(p, bh);
    const float c = hc.c, r = hc.r;

    Owned<E, D, QB> qf;
    load_owned<E, D, QB>(qf, Qh, active ? qw0 : 0, lane);
    for (int i = tid; i < MR * W; i += THREADS) { wm[i] = 0u; cand[i] = 0u; }
    for (int i = tid; i < SM::HIST_WORDS; i += THREADS) hist[i] = 0u;

    f32x16 C[2][QB];
    unsigned long long ntile_done = 0;
    char* const kbuf1 = NBUF == 2 ? kbuf_b : kbuf;
    auto issue_seq = [&](int it, char* buf) { issue_rows<E, D, NW>(buf, Kh, (long)it * 64, wave, lane); };
    auto scores = [&](int j, const char* buf) {
        stage1<E, D, QB>(C, buf, qf, lane);
        if (p.causal && (long)j * 64 + 63 > qw0) causal_hide<QB, true>(C, j * 64, (int)qw0, lane);
        ++ntile_done;
    };

    // ---- Phases 1 and 2 in one dense sweep: row maximum and histogram -------------------------
    // The histogram of Eq. 7-8 is centred on the row maximum, which a single sweep only knows at
    // its end.  Here the bins lie on an absolute grid instead (bin a holds NB x in [a, a+1), x =
    // (alpha-1) s), and a row keeps the window of bins from one unit below its running maximum
    // up to it: every score that can exceed tau* >= max - 1 (Eq. 5) is inside the window when it
    // is met, and stays inside as the maximum grows.  Prop. 1 only uses that a bin's left edge is
    // at most h below its scores, so its bounds hold on this grid as well.  When the maximum
    // moves up by k bins, the k slots that pass from the bottom of the window to its top are
    // cleared (by the row's first lane; LDS operations of one wave execute in program order).
    //
    // A score's slot, times 4, is the integer part of rel = 4 NB c s + k4 taken modulo 256, with
    // k4 = 4 (rot - a_lo): a_lo is the window's lowest bin and rot = a_lo mod SLOTS its slot.
    // The score is inside the window iff rel >= 4 rot.
    const float cb = c * NB, c4 = 4.f * cb;
    float run[QB], k4[QB], thr4[QB];
    int a_top[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) { run[qb] = -INFINITY; k4[qb] = 0.f; thr4[qb] = INFINITY; a_top[qb] = INT_MIN; }
    // Besides the running maximum, every (row, key tile) maximum goes to HBM (fp16, rounded up):
    // once tau_0 is known, only tiles holding a score above it can matter to f or to P.
    stream_tiles<NBUF>(njt, kbuf, kbuf1, issue_seq, [&](int j, const char* buf) {
        if (j >= wjt) return;
        scores(j, buf);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float gm[4];                            // maxima of the four groups of 8 registers
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                gm[g] = C[g >> 1][qb][8 * (g & 1)];
#pragma unroll
                for (int v = 1; v < 8; ++v) gm[g] = fmaxf(gm[g], C[g >> 1][qb][8 * (g & 1) + v]);
            }
            const float lm = fmaxf(fmaxf(gm[0], gm[1]), fmaxf(gm[2], gm[3]));
            const float tm = xhalf_max(lm);
            if (h == 0) tmax_g[(long)j * N + qw0 + 32 * qb + n] = (_Float16)(tm + fabsf(tm) * (1.f / 1024.f) + 1e-7f);
            const int row0 = wave * 32 * QB + 32 * qb;
            char* hrow = (char*)(hist + (wave * 32 + n) * SLOTS);
            const bool rise = tm > run[qb];
            if (__any(rise)) {                      // some row's maximum moves up
                int first = 0, last = -1;           // bins to clear: first..last (none)
                if (rise) {
                    run[qb] = tm;
                    int nt = (int)floorf(fminf(fmaxf(cb * tm, -1e9f), 1e9f));
                    int a_lo = nt - (SLOTS - 1), rot = a_lo & (SLOTS - 1);
                    float kk = 4.f * (float)(rot - a_lo);
                    // the maximum itself must land in the window's top slot, not wrap past it
                    if ((int)fmaf(c4, tm, kk) >= 4 * rot + 4 * SLOTS) {
                        nt += 1; a_lo += 1; rot = a_lo & (SLOTS - 1); kk = 4.f * (float)(rot - a_lo);
                    }
                    if (a_top[qb] != INT_MIN) { first = max(a_top[qb], nt - SLOTS) + 1; last = nt; }
                    a_top[qb] = nt; k4[qb] = kk; thr4[qb] = 4.f * (float)rot;
                }
                // the whole wave clears the slots of one rising row at a time: lane i takes slot i
                unsigned long long todo = __ballot(h == 0 && last >= first);
                while (todo) {
                    const int src = __ffsll((long long)todo) - 1;
                    todo &= todo - 1;
                    const int f0 = __builtin_amdgcn_readlane(first, src);
                    const int cnt = __builtin_amdgcn_readlane(last - first, src);
                    if (((lane - f0) & (SLOTS - 1)) <= cnt) {
                        uint32_t* word = hist + (wave * 32 + src) * SLOTS + lane;
                        if constexpr (QB == 1) *word = 0u;
                        else lds_and_b32(word, qb == 0 ? 0xffff0000u : 0x0000ffffu);
                    }
                }
            }
            if (__any(fmaf(c4, lm, k4[qb]) >= thr4[qb])) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    if (!__any(fmaf(c4, gm[g], k4[qb]) >= thr4[qb])) continue;
#pragma unroll
                    for (int v = 0; v < 8; ++v) {
                        const float rel = fmaf(c4, C[g >> 1][qb][8 * (g & 1) + v], k4[qb]);
                        if (rel >= thr4[qb]) lds_add_u32(hrow + ((int)rel & (4 * SLOTS - 4)), 1u << (SM::CBITS * qb & 31));
                    }
                }
            }
        }
    });
    lds_settle();
    // tau_0 = max(tau_h, max - 1) and the bracket [tau_0, tau_h + 1/NB] (Prop. 1, Eq. 5), raw units.
    // A wave reads only the histograms it filled itself: no barrier.  Lane (n, h) solves row block
    // qb = h of row n (with one row per lane, lane half 0 does), then the two lanes of a row swap.
    float thr[QB], blo[QB], bhi[QB];
    {
        constexpr float hb = 1.f / NB;
        const int sq = (QB == 2) ? h : 0;
        int top = a_top[0];
        float mx = run[0];
        if constexpr (QB == 2) { if (h) { top = a_top[1]; mx = run[1]; } }
        const int a_lo = top == INT_MIN ? 0 : top - (SLOTS - 1);
        const float origin = (float)a_lo * hb;                        // left edge of the window
        const float tau_h = solve_histogram<AM, SLOTS, SM::CBITS>(hist + (wave * 32 + n) * SLOTS, a_lo & (SLOTS - 1),
                                                                  SM::CBITS * sq & 31, hb, r) + origin;
        const float slack = 1e-6f + 2.5e-7f * fabsf(origin);          // fp32 rounding of bins and closed form
        const float my_t0 = fmaxf(tau_h - slack, fmaf(c, mx, -1.f));
        const float my_hi = tau_h + hb + slack;
        const float o_t0 = xhalf_other(my_t0, h), o_hi = xhalf_other(my_hi, h);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const bool mine = (h == (QB == 2 ? qb : 0));
            thr[qb] = mine ? my_t0 : o_t0;
            blo[qb] = thr[qb];
            bhi[qb] = mine ? my_hi : o_hi;
            // right-edge binning moves every bin, and with it the root, up by one bin width: that
            // root, tau_h + h >= tau*, is the bracket's upper end, and it stands as the threshold
            if (active && h == 0) {
                p.rs_t0[(long)bh * N + qw0 + 32 * qb + n] = thr[qb];
                p.rs_up0[(long)bh * N + qw0 + 32 * qb + n] = bhi[qb];
            }
            if (p.right_edge) thr[qb] = bhi[qb];
        }
    }
    // candidate tiles of this wave's rows: those holding a score above tau_0.  64 tiles per
    // round: lane (n, h) looks at tiles j0 + 2u + h, u = 0..31, of row n, with all 32 loads in
    // flight together (one load at a time would string up to T/2 memory round trips).
    {
        float t0[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) t0[qb] = thr[qb];
        // (the tile maxima read below were stored by lanes of this same wave and are read here for
        // the first time: waiting for the wave's stores is enough, see tau_list_kernel)
        wait_loads();
        for (int j0 = 0; j0 < wjt; j0 += 64) {
            _Float16 tm[32][QB];
#pragma unroll
            for (int u = 0; u < 32; ++u) {
                const int j = min(j0 + 2 * u + h, wjt - 1);        // clamped: tested against wjt below
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) tm[u][qb] = tmax_g[(long)j * N + qw0 + 32 * qb + n];
            }
            unsigned long long bits = 0;
#pragma unroll
            for (int u = 0; u < 32; ++u) {
                bool cnd = false;
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) cnd |= fmaf(c, (float)tm[u][qb], -t0[qb]) >= 0.f;
                cnd = cnd && (j0 + 2 * u + h < wjt);
                const unsigned long long bal = __ballot(cnd);
                if (bal & 0xffffffffull) bits |= 1ull << (2 * u);
                if (bal >> 32) bits |= 1ull << (2 * u + 1);
            }
            if (lane == 0) {
                const int w0 = j0 >> 5;
                if ((uint32_t)bits) atomicOr(&cand[myrow * W + w0], (uint32_t)bits);
                if (bits >> 32) atomicOr(&cand[myrow * W + w0 + 1], (uint32_t)(bits >> 32));
            }
        }
    }
    __syncthreads();
    build_tile_list(cand, MR, W, tl, tl_count, tid);
    auto issue_list = [&](int it, char* buf) { issue_rows<E, D, NW>(buf, Kh, (long)tl[it] * 64, wave, lane); };

    // ---- Phase 3: refinement sweeps; the first also records the working mask --------------
    // One evaluation of f, f', f'' at tau_0 over the candidate tiles and one safeguarded step;
    // the tiles that hold a score above tau_0 form the working mask.  Later evaluations ride on
    // Phase 4 (out_kernel).
    {
        float F[QB], G[QB], Hs[QB];
        int cnt[QB];      // number of scores above tau (alpha = 1.5: f'' sum; alpha = 2: f' sum)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) { F[qb] = G[qb] = Hs[qb] = 0.f; cnt[qb] = 0; }
        stream_tiles<NBUF>(*tl_count, kbuf, kbuf1, issue_list, [&](int it, const char* buf) {
            const int j = tl[it];
            if (!mask_bit(cand, W, myrow, j)) return;
            scores(j, buf);
            const bool hit = eval_scores<AM, QB>(C, thr, c, r, F, G, Hs, cnt);
            if (hit && lane == 0) atomicOr(&wm[myrow * W + (j >> 5)], 1u << (j & 31));
        });
        // threshold after this step, its bracket, f' at the point evaluated, and
        // (iterations | done << 16), for the output kernel; both lanes of a row compute the same
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            if constexpr (AM == ALPHA_15) Hs[qb] = (float)cnt[qb];
            if constexpr (AM == ALPHA_20) G[qb] = (float)cnt[qb];
            const float f = xhalf_sum(F[qb]) - 1.f, g = xhalf_sum(G[qb]), hs = xhalf_sum(Hs[qb]);
            bool done = fabsf(f) <= p.tol || p.right_edge;
            float tau = thr[qb];
            if (!done) {
                SecantPrev none;
                const float stol = step_tol(p.tol, tau);
                const float cand_tau = hybrid_step<AM>(tau, f, g, hs, r, hc.alpha, blo[qb], bhi[qb], none, stol);
                done = fabsf(cand_tau - tau) < stol;
                tau = cand_tau;
            }
            if (active && h == 0) {
                const long gi = (long)bh * N + qw0 + 32 * qb + n;
                p.tau[gi] = tau;
                p.rs_lo[gi] = blo[qb];
                p.rs_hi[gi] = bhi[qb];
                p.rs_state[gi] = 1 | ((int)done << 16);
                p.rs_f1[gi] = -r * g;
            }
        }
    }
    __syncthreads();
    for (int i = tid; i < MR * W; i += THREADS)
        if (I * MR + i / W < T) p.wmask[((long)bh * T + (long)I * MR + i / W) * W + (i % W)] = (int32_t)wm[i];
    {
        const int slot[2] = {0, 5};
        const unsigned long long val[2] = {ntile_done * QB, wave == 0 ? 1ull : 0ull};
        flush_counters<2>(blk_stats, p.stats, slot, val, tid, lane);
    }
}

// A cheap lower bound of the histogram's root for general alpha, used while the sweep is under way:
// the largest bin edge e_j with f_h(e_j) >= 0 (f_h falls with tau, so tau_h >= e_j), found by
// bisection over j.  At a bin edge f_h needs no power function: f_h(e_j) = sum_{k>j} H_k pw[k-j] - 1
// with the table pw[m] = (m h)^r.  Returns -h when even the window's bottom edge is too high.
template <int SLOTS, int BITS>
EA_DEV float histogram_edge_bound(const uint32_t* H, int rot, int shift, float h, const float* pw) {
    auto count = [&](int k) {
        const uint32_t w = H[(rot + k) & (SLOTS - 1)] >> shift;
        return (float)(BITS == 32 ? w : (w & ((1u << (BITS & 31)) - 1u)));
    };
    int lo = -1, hi = SLOTS - 1;          // f_h(e_hi) = -1 < 0: no bin lies above the top one
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        float f = -1.f;
        for (int k = mid + 1; k < SLOTS; ++k) f = fmaf(count(k), pw[k - mid], f);
        if (f >= 0.f) lo = mid; else hi = mid;
    }
    return (float)lo * h;
}

// ---- threshold kernel with candidate lists -----------------------------------------------------
// Phases 1-3 of Alg. 1 from ONE dense sweep.  By Eq. 5, tau* >= max - 1 (in units of (alpha-1) s),
// and both the maximum and tau* over a prefix of the keys are at most their values over all keys,
// so a score that lies below a lower bound of the prefix's threshold when it is met can never lie
// above the final one.  Every other score - a handful per row when attention is sparse - is
// (a) counted in the row's LDS histogram (Eq. 6-8; absolute bin grid with a sliding window, as in
// tau_kernel) and (b) appended, with its key tile, to a list private to the lane that computed it
// (each lane sees 16 of every 32 keys of its row, so a row has two lists; no atomics, no ordering
// between lanes).  The lower bound starts as (running maximum - 1); each time a list has grown by
// a fixed number of entries the histogram is solved (Eq. 9) and its root tau_h, a lower bound of the
// prefix's tau* by Prop. 1, becomes the new bound.  Scores that were skipped lie below the bound and
// contribute nothing to f at or above it, so f there, and with it Prop. 1, is that of all scores.
// After the sweep the lists hold a superset of the row's support as exact fp32 scores, and the
// rest happens on them: the refinement iterations of Sec. 3.2 from tau_0 = tau_h, each an
// evaluation of f, f', f'' over the listed true scores instead of another sweep of Q K^T.  The key
// tiles of the entries above tau_0 are the working mask.
// A list that fills up (attention close to uniform: hundreds of non-zeros per row) flags its 64-row
// block; flagged blocks are redone by the sweep-based tau_kernel, which runs right after and exits
// at once everywhere else.
// PAIR (one row per lane only): waves 2w and 2w+1 share the words of one histogram buffer, 16 bits
// each - what two rows per lane do within a wave - so that eight one-row waves need the LDS of
// four and, with half the accumulator and operand registers, four waves fit a SIMD.
template <class E, int D, int QB, int AM, int NB, int NW, int NBUF, int PAIR = 0>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(PAIR ? 4 : 1))) void tau_list_kernel(Params p) {
    static_assert(!PAIR || (QB == 1 && NW % 2 == 0), "paired histograms: one row per lane, an even number of waves");
    using SM = TauSmem<E, D, QB, NB, NW, NBUF>;
    using KT = RowTile<E, D>;
    using elem = typename E::elem;
    constexpr int THREADS = NW * 64, BR = SM::BR, MR = SM::MR, SLOTS = SM::SLOTS;
    constexpr int GROW = 24;              // list growth (entries per lane) between two histogram solves
    __shared__ __align__(1024) char kring[NBUF * KT::BYTES];
    constexpr int HIST_WORDS = PAIR ? SM::HIST_WORDS / 2 : SM::HIST_WORDS;
    constexpr int CB = PAIR ? 16 : SM::CBITS;            // bits per counter
    __shared__ __align__(256) uint32_t hist[HIST_WORDS];
    __shared__ float pw[AM == ALPHA_GEN ? SLOTS : 1];             // (m h)^r, general alpha only
    // used only once the sweep is over: they live in the key-tile ring
    static_assert(2 * MR * MAX_W * 4 + MR * 4 + 96 <= NBUF * KT::BYTES, "post-sweep arrays must fit in the ring");
    uint32_t* const wm = (uint32_t*)kring;                        // working mask (tiles above tau_0)
    uint32_t* const fmk = (uint32_t*)(kring + MR * MAX_W * 4);    // final mask (tiles of the support)
    int* const over_s = (int*)(kring + 2 * MR * MAX_W * 4);
    int* const gsum = (int*)(kring + 2 * MR * MAX_W * 4 + ((MR * 4 + 7) & ~7));   // list entries, support size, obstacles
    unsigned long long* const blk_stats = (unsigned long long*)(kring + 2 * MR * MAX_W * 4 + ((MR * 4 + 7) & ~7) + 16);

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, h = lane >> 5;
    const int N = p.N, T = p.T, W = p.W;
    int bh, I;
    map_block(blockIdx.x, p.BH, (N + BR - 1) / BR, bh, I);
    const long q0 = (long)I * BR, qw0 = q0 + wave * 32 * QB;
    const bool active = qw0 < N;
    const elem* Qh = (const elem*)p.Q + (long)bh * N * D;
    const elem* Kh = (const elem*)p.K + (long)bh * N * D;
    const int njt = p.causal ? min((int)((q0 + BR) / 64), T) : T;
    const int wjt = !active ? 0 : p.causal ? (int)((qw0 + 32 * QB - 1) / 64) + 1 : T;
    const int myrow = (wave * 32 * QB) / 64;
    const HeadConsts hc = head_consts(p, bh);
    const float c = hc.c, r = hc.r;
    constexpr float hb = 1.f / NB;

    Owned<E, D, QB> qf;
    load_owned<E, D, QB>(qf, Qh, active ? qw0 : 0, lane);
    for (int i = tid; i < HIST_WORDS; i += THREADS) hist[i] = 0u;
    if constexpr (AM == ALPHA_GEN) {
        if (tid < SLOTS) pw[tid] = tid == 0 ? 0.f : pow_r<AM>((float)tid * (1.f / NB), r);
    }

    // this lane's lists (per-lane 64-bit addresses: a scalar base would have to be fetched from
    // spilled scalar registers at every append)
    char* const lists_h = (char*)p.lists + (size_t)bh * N * (2 * LIST_CAP * 8);
    char* lptr[QB];
    int cnt[QB], trig[QB], a_top[QB], bottom4[QB];
    float run[QB], lowraw[QB], k4[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        lptr[qb] = lists_h + (size_t)(((active ? qw0 : 0) + 32 * qb + n) * 2 + h) * (size_t)(LIST_CAP * 8);
        cnt[qb] = 0; trig[qb] = GROW;
        run[qb] = -INFINITY; lowraw[qb] = -3.0e38f;
        k4[qb] = 0.f; bottom4[qb] = 0; a_top[qb] = INT_MIN;
    }
    const int hwave = PAIR ? (wave >> 1) : wave;         // whose buffer, and which half of its words
    auto hshift = [&](int qb) { return PAIR ? 16 * (wave & 1) : (CB * qb & 31); };
    char* const hrow = (char*)(hist + (hwave * 32 + n) * SLOTS);

    // Root of the row's histogram (Eq. 9) as it stands: lane (n, h) solves row block qb = h of row n
    // (with one row per lane, both lanes solve the same), then the two lanes of a row swap.  Returns
    // per row block tau_0 = max(tau_h, max - 1) less the fp32 slack, and the bracket's upper end.
    // (coarse: while the sweep runs only a lower bound is wanted; for general alpha, whose exact
    // solve costs hundreds of power functions, the best bin edge then stands in for the root)
    auto histogram_bound = [&](float (&lo)[QB], float (&up)[QB], bool coarse) {
        lds_settle();
        const int sq = (QB == 2) ? h : 0;
        int top = a_top[0];
        float mx = run[0];
        if constexpr (QB == 2) { if (h) { top = a_top[1]; mx = run[1]; } }
        const int a_lo = top == INT_MIN ? 0 : top - (SLOTS - 1);
        const float origin = (float)a_lo * hb;                        // left edge of the window
        float tau_h;
        if (AM == ALPHA_GEN && coarse)
            tau_h = histogram_edge_bound<SLOTS, CB>((const uint32_t*)hrow, a_lo & (SLOTS - 1), hshift(sq), hb, pw) + origin;
        else
            tau_h = solve_histogram<AM, SLOTS, CB>((const uint32_t*)hrow, a_lo & (SLOTS - 1), hshift(sq), hb, r) + origin;
        const float slack = 1e-6f + 2.5e-7f * fabsf(origin);          // fp32 rounding of bins and closed form
        const float my_lo = fmaxf(tau_h - slack, fmaf(c, mx, -1.f)), my_up = tau_h + hb + slack;
        const float o_lo = xhalf_other(my_lo, h), o_up = xhalf_other(my_up, h);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const bool mine = (h == (QB == 2 ? qb : 0));
            lo[qb] = mine ? my_lo : o_lo;
            up[qb] = mine ? my_up : o_up;
        }
    };

    f32x16 C[2][QB];
    unsigned long long ntile_done = 0;
    const float inv_c = 1.f / c, cb = c * NB, c4 = 4.f * cb;
    auto sweep_tile = [&](int j, const char* buf) {
            if (j >= wjt) return;
            stage1<E, D, QB, EA_FENCE, PAIR ? 0 : 8>(C, buf, qf, lane);
            if (p.causal && (long)j * 64 + 63 > qw0) causal_hide<QB, true>(C, j * 64, (int)qw0, lane);
            ++ntile_done;
            // per row block: maxima of the four groups of 8 registers, of the lane, of the row
            float gm[QB][4], lm[QB], tm[QB];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
                for (int g = 0; g < 4; ++g) gm[qb][g] = max8_raw(C[g >> 1][qb], 8 * (g & 1));
                lm[qb] = max2_raw(max3_raw(gm[qb][0], gm[qb][1], gm[qb][2]), gm[qb][3]);
            }
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) tm[qb] = xhalf_max(lm[qb]);
            bool rise_any = false;
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) rise_any |= tm[qb] > run[qb];
            if (__any(rise_any)) {
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    // the window of live bins follows the running maximum (see tau_kernel)
                    const bool rise = tm[qb] > run[qb];
                    int first = 0, last = -1;           // bins to clear: first..last (none)
                    if (rise) {
                        run[qb] = tm[qb];
                        int nt = (int)floorf(fminf(fmaxf(cb * tm[qb], -1e9f), 1e9f));
                        int a_lo = nt - (SLOTS - 1), rot = a_lo & (SLOTS - 1);
                        float kk = 4.f * (float)(rot - a_lo);
                        // the maximum itself must land in the window's top slot, not wrap past it
                        if ((int)fmaf(c4, tm[qb], kk) >= 4 * rot + 4 * SLOTS) {
                            nt += 1; a_lo += 1; rot = a_lo & (SLOTS - 1); kk = 4.f * (float)(rot - a_lo);
                        }
                        if (a_top[qb] != INT_MIN) { first = max(a_top[qb], nt - SLOTS) + 1; last = nt; }
                        a_top[qb] = nt; k4[qb] = kk; bottom4[qb] = 4 * rot;
                    }
                    // the whole wave clears the slots of one rising row at a time: lane i takes slot i
                    unsigned long long todo = __ballot(h == 0 && last >= first);
                    while (todo) {
                        const int src = __ffsll((long long)todo) - 1;
                        todo &= todo - 1;
                        const int f0 = __builtin_amdgcn_readlane(first, src);
                        const int ncl = __builtin_amdgcn_readlane(last - first, src);
                        if (((lane - f0) & (SLOTS - 1)) <= ncl) {
                            uint32_t* word = hist + (hwave * 32 + src) * SLOTS + lane;
                            if constexpr (QB == 1 && !PAIR) *word = 0u;
                            else lds_and_b32(word, hshift(qb) == 0 ? 0xffff0000u : 0x0000ffffu);
                        }
                    }
                }
            }
            // candidates: raw scores at or above the row's current lower bound; most tiles of a
            // sparse row block hold none, and leave here
            float lowv[QB];
            bool maybe = false;
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                lowv[qb] = fmaxf(run[qb] - inv_c, lowraw[qb]);
                maybe |= lm[qb] >= lowv[qb];
            }
            if (!__any(maybe)) return;
            bool grown = false;
            const int key0 = j * 64 + 8 * h;
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                const float low = lowv[qb];
                if (!__any(lm[qb] >= low)) continue;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    if (!__any(gm[qb][g] >= low)) continue;
#pragma unroll
                    for (int v = 0; v < 8; ++v) {
                        const float sc = C[g >> 1][qb][8 * (g & 1) + v];
                        if (sc >= low) {
                            // slot of the score's bin, times 4 (a score that rounding puts a hair
                            // below the window goes to its lowest bin)
                            const int rel = max((int)fmaf(c4, sc, k4[qb]), bottom4[qb]);
                            lds_add_u32(hrow + (rel & (4 * SLOTS - 4)), 1u << hshift(qb));
                            // a full list keeps overwriting its last entry (its block is redone anyway)
                            uint2 ent;          // tile row of register v of group g: see causal_hide
                            ent.x = __float_as_uint(sc); ent.y = (uint32_t)(key0 + 32 * (g >> 1) + 16 * (g & 1) + v);
                            *(uint2*)(lptr[qb] + 8u * (uint32_t)min(cnt[qb], LIST_CAP - 1)) = ent;
                            ++cnt[qb];
                        }
                    }
                }
                grown |= cnt[qb] >= trig[qb];
            }
            if (__any(grown)) {
                // a better lower bound from the histogram so far
                float lo[QB], up[QB];
                histogram_bound(lo, up, true);
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    const float braw = lo[qb] * inv_c;
                    lowraw[qb] = braw - fabsf(braw) * 1e-6f;
                    trig[qb] = cnt[qb] <= LIST_CAP ? cnt[qb] + GROW : INT_MAX;
                }
            }
    };
    stream_tiles_ring<NBUF, KT::NINST / NW>(njt, kring, KT::BYTES,
        [&](int it, char* buf) { issue_rows<E, D, NW>(buf, Kh, (long)it * 64, wave, lane); }, sweep_tile);
    for (int i = tid; i < MR * W; i += THREADS) { wm[i] = 0u; fmk[i] = 0u; }   // (the walk ended with a barrier: the ring is free)
    if (tid < MR) over_s[tid] = 0;
    if (tid < 4) gsum[tid] = 0;
    __syncthreads();
    // The lists are read back below by the lanes that wrote them, for the first time in this kernel
    // (no stale line can sit in the vector cache): it is enough that this wave's stores have
    // completed.  A device-scope fence here writes the whole L2 back once per work-group, which
    // cost 0.1 - 0.4 ms per launch.
    wait_loads();

    // ---- solve and refinement on the lists -----------------------------------------------------
    int any_over = 0;
    float thr[QB];
    int iters[QB], done[QB], mycnt[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) { thr[qb] = 0.f; iters[qb] = 0; done[qb] = 1; mycnt[qb] = 0; }
    if (active) {
        float blo[QB], bhi[QB];
        histogram_bound(thr, bhi, false);
        if (h == 0) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                p.rs_t0[(long)bh * N + qw0 + 32 * qb + n] = thr[qb];
                p.rs_up0[(long)bh * N + qw0 + 32 * qb + n] = bhi[qb];
            }
        }
        float f1_last[QB];
        int nmax = 0;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            any_over |= (cnt[qb] > LIST_CAP);
            mycnt[qb] = min(cnt[qb], LIST_CAP);
            nmax = max(nmax, mycnt[qb]);
            blo[qb] = thr[qb]; iters[qb] = 0; done[qb] = 0; f1_last[qb] = -1.f;
            if (p.right_edge) thr[qb] = bhi[qb];      // tau_h + h >= tau*: the right-edge root, taken as it is
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) nmax = max(nmax, __shfl_xor(nmax, off));
        // refinement (Sec. 3.2): evaluations of f, f', f'' over the listed scores; each lane walks
        // its own lists, sixteen entries per row block at a time with all loads in flight together
        SecantPrev prev[QB];
        // (alpha > 2: a row with a score within the tolerance of its root ends up bisecting, since f
        // rises vertically there; the sweeps over the lists are cheap, those of the output kernel
        // are not, so the limit is doubled here)
        const int nsweeps = r < 1.f ? 2 * p.max_sweeps : p.max_sweeps;
        for (int sweep = 0; sweep < nsweeps; ++sweep) {
            float F[QB], G[QB], Hs[QB];
            uint32_t lastj[QB];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) { F[qb] = G[qb] = Hs[qb] = 0.f; lastj[qb] = 0xffffffffu; }
            for (int i0 = 0; i0 < nmax; i0 += 16) {
                uint4 e[QB][8];
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        e[qb][u] = make_uint4(0u, 0u, 0u, 0u);
                        if (i0 + 2 * u < mycnt[qb]) e[qb][u] = *(const uint4*)(lptr[qb] + (i0 + 2 * u) * 8);
                    }
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                    for (int u = 0; u < 16; ++u) {
                        const uint32_t bits = (u & 1) ? e[qb][u >> 1].z : e[qb][u >> 1].x;
                        const uint32_t j = ((u & 1) ? e[qb][u >> 1].w : e[qb][u >> 1].y) >> 6;      // key tile
                        const float y = fmaf(c, __uint_as_float(bits), -thr[qb]);
                        if (i0 + u < mycnt[qb] && y > 0.f) {
                            if constexpr (AM == ALPHA_15) { F[qb] = fmaf(y, y, F[qb]); G[qb] += y; Hs[qb] += 1.f; }
                            else if constexpr (AM == ALPHA_20) { F[qb] += y; G[qb] += 1.f; }
                            else {
                                const float p2 = pow_r2<AM>(y, r);
                                Hs[qb] += p2; G[qb] = fmaf(p2, y, G[qb]); F[qb] = fmaf(p2 * y, y, F[qb]);
                            }
                            // first evaluation, at tau_0 <= tau*: its tiles are the working mask
                            if (sweep == 0 && j != lastj[qb]) { atomicOr(&wm[myrow * W + (j >> 5)], 1u << (j & 31)); lastj[qb] = j; }
                        }
                    }
            }
            int pending = 0;
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                const float f = xhalf_sum(F[qb]) - 1.f, g = xhalf_sum(G[qb]), hs = xhalf_sum(Hs[qb]);
                if (!done[qb]) {
                    iters[qb] += 1;
                    f1_last[qb] = -r * g;
                    if (fabsf(f) <= p.tol || p.right_edge) done[qb] = 1;
                    else {
                        const float stol = step_tol(p.tol, thr[qb]);
                        const float cand_tau = hybrid_step<AM>(thr[qb], f, g, hs, r, hc.alpha, blo[qb], bhi[qb], prev[qb], stol);
                        if (fabsf(cand_tau - thr[qb]) < stol) done[qb] = 1;
                        thr[qb] = cand_tau;
                    }
                    pending |= !done[qb];
                }
            }
            if (!__any(pending)) break;
        }
        if (h == 0) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                const long gi = (long)bh * N + qw0 + 32 * qb + n;
                p.tau[gi] = thr[qb];
                p.rs_lo[gi] = blo[qb];
                p.rs_hi[gi] = bhi[qb];
                p.rs_state[gi] = iters[qb] | (done[qb] << 16);
                p.rs_f1[gi] = f1_last[qb];
            }
        }
    }
    if (__any(any_over) && lane == 0) atomicOr(&over_s[myrow], 1);

    // ---- sparse row groups: the support itself, for the gather kernel ---------------------------
    // Where the lists are short, the entries above the final tau - the row's support, a handful of
    // keys - are moved to the front of their list, with their key indices; gather_out_kernel then
    // forms O from those rows of V alone, and the block-sparse output kernel skips the row group.
    {
        int len = 0, obstacle = any_over;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) { len += mycnt[qb]; obstacle |= !done[qb]; }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) len += __shfl_xor(len, off);
        if (lane == 0) atomicAdd(&gsum[0], len);
        if (__any(obstacle) && lane == 0) atomicOr(&gsum[2], 1);
    }
    __syncthreads();
    const int nrows = min(BR, N - (int)q0);
    const bool sparse = p.gflag && gsum[2] == 0 && gsum[0] <= GATHER_LIST_MAX * nrows;
    if (sparse) {
        int nsup = 0;
        if (active) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                int w = 0;
                uint32_t lastj = 0xffffffffu;
                for (int i0 = 0; i0 < mycnt[qb]; i0 += 16) {
                    uint4 e[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        e[u] = make_uint4(0u, 0u, 0u, 0u);
                        if (i0 + 2 * u < mycnt[qb]) e[u] = *(const uint4*)(lptr[qb] + (i0 + 2 * u) * 8);
                    }
                    // (all sixteen are in registers before the first is overwritten; w <= i0 + u)
#pragma unroll
                    for (int u = 0; u < 16; ++u) {
                        uint2 ent;
                        ent.x = (u & 1) ? e[u >> 1].z : e[u >> 1].x;
                        ent.y = (u & 1) ? e[u >> 1].w : e[u >> 1].y;
                        if (i0 + u < mycnt[qb] && fmaf(c, __uint_as_float(ent.x), -thr[qb]) > 0.f) {
                            *(uint2*)(lptr[qb] + 8 * w) = ent;
                            ++w;
                            const uint32_t j = ent.y >> 6;
                            if (j != lastj) { atomicOr(&fmk[myrow * W + (j >> 5)], 1u << (j & 31)); lastj = j; }
                        }
                    }
                }
                p.scnt[((long)bh * N + qw0 + 32 * qb + n) * 2 + h] = w;
                nsup += w;
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) nsup += __shfl_xor(nsup, off);
        if (lane == 0) atomicAdd(&gsum[1], nsup);
    }
    __syncthreads();
    const bool gather = sparse && gsum[1] <= GATHER_SUP_MAX * nrows;
    if (blockIdx.x == 0 && tid == 0) p.scal[2] = p.gflag ? (unsigned int)BR : 0u;     // (0: no flags were written)
    if (p.gflag && tid == 0) {
        p.gflag[(long)bh * ((N + BR - 1) / BR) + I] = gather;
        if (!gather) atomicAdd(&p.scal[1], 1u);       // a row group out_kernel will have to serve
    }
    if (gather) {
        if (active && h == 0 && p.iters) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) p.iters[(long)bh * N + qw0 + 32 * qb + n] = iters[qb];
        }
        for (int i = tid; i < MR * W; i += THREADS)
            if (I * MR + i / W < T) p.mask[((long)bh * T + (long)I * MR + i / W) * W + (i % W)] = (int32_t)fmk[i];
    }
    for (int i = tid; i < MR * W; i += THREADS)
        if (I * MR + i / W < T) p.wmask[((long)bh * T + (long)I * MR + i / W) * W + (i % W)] = (int32_t)wm[i];
    if (tid < MR && I * MR + tid < T) p.oflag[(long)bh * T + (long)I * MR + tid] = over_s[tid];
    {
        int nover = 0;
        if (tid == 0)
            for (int i = 0; i < MR; ++i) nover += over_s[i];
        const int slot[3] = {0, 8, 9};
        const unsigned long long val[3] = {ntile_done * QB, (unsigned long long)nover, (tid == 0 && gather) ? (unsigned long long)nrows : 0ull};
        flush_counters<3>(blk_stats, p.stats, slot, val, tid, lane);
    }
}

template <class E, class E2, int D, int QB, bool MASK_ONLY, int NW, int NBUF>
struct OutSmem {
    static constexpr int BR = 32 * QB * NW;
    static constexpr int MR = (BR + 63) / 64;
    static constexpr int KBYTES = RowTile<E, D>::BYTES;
    static constexpr int VBYTES = MASK_ONLY ? 0 : RowTile<E2, D>::BYTES;
    static constexpr int SET = KBYTES + VBYTES;              // one buffer set (static LDS)
};

// Phase 4.  MASK_ONLY: no V, no O - only the mask at the given tau (used by the backward when
// the caller passes no mask).
template <class E, class E2, int D, int QB, int AM, bool MASK_ONLY, int NW, int NBUF>
__global__ __launch_bounds__(NW * 64) void out_kernel(Params p) {
    using SM = OutSmem<E, E2, D, QB, MASK_ONLY, NW, NBUF>;
    using elem = typename E::elem;
    constexpr int BR = SM::BR, MR = SM::MR;
    constexpr int THREADS = NW * 64;
    // buffer sets: K tile, V tile right after it; two separate variables (see stream_tiles)
    __shared__ __align__(1024) char set0[SM::SET];
    __shared__ __align__(1024) char set1[NBUF == 2 ? SM::SET : 1024];
    __shared__ uint32_t wm[MR * MAX_W];
    __shared__ uint32_t fm[MR * MAX_W];
    __shared__ int tl[MAX_T];
    __shared__ int tl_count[4];
    __shared__ unsigned long long blk_stats[4];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31;
    const int N = p.N, T = p.T, W = p.W;
    int bh, I;
    map_block(blockIdx.x, p.BH, (N + BR - 1) / BR, bh, I);
    const long q0 = (long)I * BR, qw0 = q0 + wave * 32 * QB;
    const bool active = qw0 < N;
    if constexpr (!MASK_ONLY) {
        // row groups whose supports were listed get their output from gather_out_kernel
        if (p.gflag && p.gflag[(long)bh * ((N + p.grows - 1) / p.grows) + q0 / p.grows]) return;
    }
    const elem* Qh = (const elem*)p.Q + (long)bh * N * D;
    const elem* Kh = (const elem*)p.K + (long)bh * N * D;
    // V in the stage-2 element type (for bf16 inputs: the fp16 copy made by convert_kernel)
    const typename E2::elem* Vh = MASK_ONLY ? nullptr : (const typename E2::elem*)p.V2 + (long)bh * N * D;
    const int myrow = (wave * 32 * QB) / 64;
    const HeadConsts hc = head_consts(p, bh);
    const float c = hc.c, r = hc.r;

    for (int i = tid; i < MR * W; i += THREADS) {
        wm[i] = (I * MR + i / W < T) ? (uint32_t)p.wmask[((long)bh * T + (long)I * MR + i / W) * W + (i % W)] : 0u;
        fm[i] = 0u;
    }
    build_tile_list(wm, MR, W, tl, tl_count, tid);

    Owned<E, D, QB> qf;
    load_owned<E, D, QB>(qf, Qh, active ? qw0 : 0, lane);
    // per-row solver state, held by both lanes of a row
    constexpr bool REFINE = !MASK_ONLY;
    float thr[QB], lo[QB], hi[QB], f1_prev[QB];
    int done[QB], iters[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const long g = (long)bh * N + qw0 + 32 * qb + n;
        thr[qb] = active ? p.tau[g] : 0.f;
        lo[qb] = hi[qb] = 0.f; done[qb] = 1; iters[qb] = 0; f1_prev[qb] = -1.f;
        if (REFINE && active) {
            lo[qb] = p.rs_lo[g]; hi[qb] = p.rs_hi[g]; f1_prev[qb] = p.rs_f1[g];
            const int st = p.rs_state[g];
            iters[qb] = st & 0xffff; done[qb] = st >> 16;
        }
    }

    f32x16 X[D / 32][QB];
    f32x16 C[2][QB];
    unsigned long long ntile_done = 0, npv_done = 0, nstat_done = 0;
    auto issue_kv = [&](int it, char* buf) {
        const long j = tl[it];
        issue_rows<E, D, NW>(buf, Kh, j * 64, wave, lane);
        if constexpr (!MASK_ONLY) issue_rows<E2, D, NW>(buf + SM::KBYTES, Vh, j * 64, wave, lane);
    };
    auto issue_k = [&](int it, char* buf) { issue_rows<E, D, NW>(buf, Kh, (long)tl[it] * 64, wave, lane); };

    // Phase 4 doubles as the next evaluation of f: the row sums of P are f(tau) + 1.  A row is
    // finished when |f| <= tol, or (alpha <= 2, where f' is bounded) when the step -f / f' (with f'
    // from its previous evaluation: a chord step) is shorter than tol; it then takes that step, and
    // O, computed less than tol away in tau, stands.  Only when some row fails both, a scores-only sweep gathers f', f'' at the
    // same tau, the hybrid step moves those rows, and Phase 4 runs again.
    auto pv_pass = [&](float (&rowsum)[QB]) {
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int v = 0; v < 16; ++v) X[db][qb][v] = 0.f;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) rowsum[qb] = 0.f;
        stream_tiles<NBUF>(*tl_count, set0, NBUF == 2 ? set1 : set0, issue_kv, [&](int it, const char* buf) {
            const int j = tl[it];
            if (!mask_bit(wm, W, myrow, j)) return;
            stage1<E, D, QB>(C, buf, qf, lane);
            if (p.causal && (long)j * 64 + 63 > qw0) causal_hide<QB, true>(C, j * 64, (int)qw0, lane);
            ++ntile_done;
            float ymax = 0.f;
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const float yp = fmaxf(fmaf(c, C[kb][qb][v], -thr[qb]), 0.f);
                        ymax = fmaxf(ymax, yp);
                        float pr;
                        if constexpr (AM == ALPHA_GEN) pr = (yp > 0.f) ? pow_r<AM>(yp, r) : 0.f;
                        else pr = pow_r<AM>(yp, r);
                        if constexpr (REFINE) rowsum[qb] += pr;
                        C[kb][qb][v] = pr;
                    }
            if (!__any(ymax > 0.f)) return;
            if (lane == 0) atomicOr(&fm[myrow * W + (j >> 5)], 1u << (j & 31));
            if constexpr (!MASK_ONLY) { stage2<E2, D, QB>(X, buf + SM::KBYTES, C, lane); ++npv_done; }
        });
    };

    float rowsum[QB];
    pv_pass(rowsum);
    if constexpr (REFINE) {
        int need = 0;
        float fval[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            fval[qb] = xhalf_sum(rowsum[qb]) - 1.f;
            if (!done[qb]) {
                iters[qb] += 1;
                const float chord = -fval[qb] / f1_prev[qb];
                if (fabsf(fval[qb]) <= p.tol) done[qb] = 1;
                else if (fabsf(chord) < step_tol(p.tol, thr[qb]) && f1_prev[qb] < 0.f && hc.alpha <= 2.f) {
                    thr[qb] = fminf(fmaxf(thr[qb] + chord, lo[qb]), hi[qb]);
                    done[qb] = 1;
                } else need = 1;
            }
        }
        if (__syncthreads_count(need) != 0) {
            // rare: finish those rows with scores-only sweeps over the tiles that held some P > 0
            // (a superset of the support at any larger tau), then form O once more.  For alpha > 2
            // the iterates come from both sides of the root, so the next tau may lie below this
            // one: the sweeps then walk the whole working mask, which was taken at tau_0 <= tau*.
            const bool below = hc.alpha > 2.f;
            bool have_f = true;          // the first sweep runs at the tau whose f is already known
            SecantPrev prev[QB];
            for (int sweep = 0; sweep < p.max_sweeps; ++sweep) {
                float F[QB], G[QB], Hs[QB];
                int cnt[QB];
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) { F[qb] = G[qb] = Hs[qb] = 0.f; cnt[qb] = 0; }
                stream_tiles<NBUF>(*tl_count, set0, NBUF == 2 ? set1 : set0, issue_k, [&](int it, const char* buf) {
                    const int j = tl[it];
                    if (!mask_bit(below ? wm : fm, W, myrow, j)) return;
                    stage1<E, D, QB>(C, buf, qf, lane);
                    if (p.causal && (long)j * 64 + 63 > qw0) causal_hide<QB, true>(C, j * 64, (int)qw0, lane);
                    ++nstat_done;
                    eval_scores<AM, QB>(C, thr, c, r, F, G, Hs, cnt);
                });
                int pending = 0;
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    if constexpr (AM == ALPHA_15) Hs[qb] = (float)cnt[qb];
                    if constexpr (AM == ALPHA_20) G[qb] = (float)cnt[qb];
                    const float g = xhalf_sum(G[qb]), hs = xhalf_sum(Hs[qb]);
                    const float f = have_f ? fval[qb] : xhalf_sum(F[qb]) - 1.f;
                    if (!done[qb]) {
                        if (!have_f) iters[qb] += 1;
                        if (!have_f && fabsf(f) <= p.tol) done[qb] = 1;
                        else {
                            const float stol = step_tol(p.tol, thr[qb]);
                            const float cand = hybrid_step<AM>(thr[qb], f, g, hs, r, hc.alpha, lo[qb], hi[qb], prev[qb], stol);
                            if (fabsf(cand - thr[qb]) < stol) done[qb] = 1;
                            thr[qb] = cand;
                        }
                        pending |= !done[qb];
                    }
                }
                have_f = false;
                if (__syncthreads_count(pending) == 0) break;
            }
            __syncthreads();
            for (int i = tid; i < MR * W; i += THREADS) fm[i] = 0u;
            __syncthreads();
            float unused[QB];
            pv_pass(unused);
        }
    }
    if constexpr (REFINE) {
        if (active && (lane >> 5) == 0) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                const long g = (long)bh * N + qw0 + 32 * qb + n;
                p.tau[g] = thr[qb];
                if (p.iters) p.iters[g] = iters[qb];
            }
        }
    }

    if constexpr (!MASK_ONLY)
        if (active) store_owned_T<D, QB>(p.O + (long)bh * N * D, qw0, X, 1.f, lane);
    for (int i = tid; i < MR * W; i += THREADS)
        if (I * MR + i / W < T) p.mask[((long)bh * T + (long)I * MR + i / W) * W + (i % W)] = (int32_t)fm[i];
    {
        const int slot[3] = {MASK_ONLY ? 6 : 1, 7, 0};
        const unsigned long long val[3] = {ntile_done * QB, npv_done * QB, nstat_done * QB};
        flush_counters<3>(blk_stats, p.stats, slot, val, tid, lane);
    }
}

// Phase 4 for sparse row groups: O_r = sum over the row's support of p_j V_j, from the support
// entries (raw score, key index) that tau_list_kernel left at the front of the row's two lists.
// With a handful of non-zeros per row this is a gather of a few rows of V, not a matrix product:
// sixteen lanes per row, each with D / 16 elements of the row of O; four entries, then their rows
// of V, are requested together.  V is read in the caller's element type.
template <class E, int D, int AM>
__global__ __launch_bounds__(256) void gather_out_kernel(Params p) {
    using elem = typename E::elem;
    constexpr int EPT = D / 16, GCH = 2;              // entries in flight per lane group (measured: 2 beats 1, 4 and 8)
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
    const elem* Vh = (const elem*)p.V + (long)bh * N * D + sub * EPT;
    const char* lists_h = (const char*)p.lists + (size_t)bh * N * (2 * LIST_CAP * 8);
    const int row_end = min(N, I * p.grows + (part + 1) * GATHER_ROWS);
    for (int row = I * p.grows + part * GATHER_ROWS + rsel; row < row_end; row += 16) {
        const long gi = (long)bh * N + row;
        const float tau = p.tau[gi];
        const int s0 = p.scnt[gi * 2], tot = s0 + p.scnt[gi * 2 + 1];
        const char* l0 = lists_h + (size_t)row * (2 * LIST_CAP * 8);      // the second list follows the first
        float acc[EPT];
#pragma unroll
        for (int k = 0; k < EPT; ++k) acc[k] = 0.f;
        for (int i0 = 0; i0 < tot; i0 += GCH) {
            uint2 e[GCH];
            vvec v[GCH];
#pragma unroll
            for (int u = 0; u < GCH; ++u) {
                const int i = i0 + u;
                e[u] = make_uint2(0u, 0u);
                if (i < tot) e[u] = *(const uint2*)(l0 + (i < s0 ? i * 8 : LIST_CAP * 8 + (i - s0) * 8));
            }
#pragma unroll
            for (int u = 0; u < GCH; ++u) {
#pragma unroll
                for (int k = 0; k < EPT; ++k) v[u][k] = (elem)0.f;
                if (i0 + u < tot) v[u] = *(const vvec*)(Vh + (long)e[u].y * D);
            }
#pragma unroll
            for (int u = 0; u < GCH; ++u) {
                const float y = fmaf(c, __uint_as_float(e[u].x), -tau);
                const float pr = (i0 + u < tot && y > 0.f) ? pow_r<AM>(y, r) : 0.f;
#pragma unroll
                for (int k = 0; k < EPT; ++k) acc[k] = fmaf(pr, (float)v[u][k], acc[k]);
            }
        }
        float* out = p.O + gi * D + sub * EPT;
#pragma unroll
        for (int k = 0; k < EPT; k += 4) *(ovec*)(out + k) = ovec{acc[k], acc[k + 1], acc[k + 2], acc[k + 3]};
    }
}

// All causally visible tiles set: the working mask handed to out_kernel<MASK_ONLY>.
static __global__ void full_mask_kernel(int32_t* wmask, int BH, int T, int W, int causal) {
    const long total = (long)BH * T * W;
    for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
        const int m = (int)(i % W), row = (int)((i / W) % T);
        const int last = causal ? row : T - 1;       // last visible tile
        uint32_t w = 0;
        const int lo = 32 * m;
        if (last >= lo) {
            const int nb = min(last - lo + 1, 32);
            w = (nb == 32) ? 0xffffffffu : ((1u << nb) - 1u);
        }
        wmask[i] = (int32_t)w;
    }
}

// Element-wise copy into another element type, optionally divided by a (bits of a float a >= 0).
// A value whose magnitude the narrower type cannot hold (fp16: 65504) is copied as the largest finite
// value of its sign and counted in *clamped (so that the caller can see that the result is not the
// one of its inputs: the fp16 copies are the operands of every second-stage product).
template <class Ein, class Eout>
__global__ __launch_bounds__(256) void convert_kernel(const typename Ein::elem* in, typename Eout::elem* out, long n,
                                                      const unsigned int* amax_bits, const int32_t* needed,
                                                      unsigned long long* clamped) {
    if (needed && *needed == 0) return;     // nobody will read the copy
    float mul = 1.f;
    if (amax_bits) {
        const float a = __uint_as_float(*amax_bits);
        if (a > 0.f) mul = 1.f / a;
    }
    constexpr bool NARROW = std::is_same<Eout, F16>::value && !std::is_same<Ein, F16>::value;
    int nclamped = 0;
    for (long i = (blockIdx.x * 256L + threadIdx.x) * 8; i < n; i += (long)gridDim.x * 256 * 8) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float x = (float)in[i + e] * mul;
            if constexpr (NARROW) {
                if (fabsf(x) > 65504.f) { x = copysignf(65504.f, x); ++nclamped; }     // (NaN compares false and stays NaN)
            }
            out[i + e] = Eout::from_float(x);
        }
    }
    if constexpr (NARROW) {
        if (__any(nclamped != 0)) {
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) nclamped += __shfl_xor(nclamped, off);
            if ((threadIdx.x & 63) == 0 && clamped) atomicAdd(clamped, (unsigned long long)nclamped);
        }
    }
}

// The backward's fp16 copies, limited to the rows its matrix kernels will read: one work-group per
// 64 rows of a head and tensor (blockIdx.y picks the tensor).  Query side (Q, dO): the rows of row
// groups that are not served by the gather kernels (gflag = 0).  Key side (K, V): every row such a
// group can see - with a causal mask the rows up to the head's last such group, else all rows when
// the head has one.  gflag null: all rows.
struct ConvertJob { const void* in; void* out; const unsigned int* amax_bits; int query_side; };
struct ConvertJobs { ConvertJob j[4]; };
template <class Ein, class Eout, int D>
__global__ __launch_bounds__(256) void convert_rows_kernel(ConvertJobs jobs, int N, const int32_t* needed,
                                                           const int32_t* gflag, int grows, int causal,
                                                           unsigned long long* clamped) {
    if (needed && *needed == 0) return;     // nobody will read the copies
    __shared__ int last_plain;
    const ConvertJob job = jobs.j[blockIdx.y];
    const typename Ein::elem* in = (const typename Ein::elem*)job.in;
    typename Eout::elem* out = (typename Eout::elem*)job.out;
    const unsigned int* amax_bits = job.amax_bits;
    const int tiles = N / 64, bh = blockIdx.x / tiles, rt = blockIdx.x % tiles;
    if (gflag) {
        const int ng = (N + grows - 1) / grows;
        const int32_t* gf = gflag + (long)bh * ng;
        if (job.query_side) {
            if (gf[(rt * 64) / grows]) return;
        } else {
            if (threadIdx.x == 0) last_plain = -1;
            __syncthreads();
            int mine = -1;
            for (int g = threadIdx.x; g < ng; g += 256)
                if (!gf[g]) mine = g;
            if (mine >= 0) atomicMax(&last_plain, mine);
            __syncthreads();
            if (last_plain < 0 || (causal && rt * 64 >= (last_plain + 1) * grows)) return;
        }
    }
    float mul = 1.f;
    if (amax_bits) {
        const float a = __uint_as_float(*amax_bits);
        if (a > 0.f) mul = 1.f / a;
    }
    constexpr bool NARROW = std::is_same<Eout, F16>::value && !std::is_same<Ein, F16>::value;
    int nclamped = 0;
    const long base = ((long)bh * N + (long)rt * 64) * D;
    for (int i = threadIdx.x * 8; i < 64 * D; i += 256 * 8) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float x = (float)in[base + i + e] * mul;
            if constexpr (NARROW) {
                if (fabsf(x) > 65504.f) { x = copysignf(65504.f, x); ++nclamped; }     // (NaN compares false and stays NaN)
            }
            out[base + i + e] = Eout::from_float(x);
        }
    }
    if constexpr (NARROW) {
        if (__any(nclamped != 0)) {
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) nclamped += __shfl_xor(nclamped, off);
            if ((threadIdx.x & 63) == 0 && clamped) atomicAdd(clamped, (unsigned long long)nclamped);
        }
    }
}

static __global__ void zero_stats_kernel(unsigned long long* stats, int n, unsigned int* scal) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) stats[i] = 0ull;
    if (scal && threadIdx.x < 4) scal[threadIdx.x] = 0u;
}

// max |x| over a tensor, rounded up to a power of two -> atomicMax on the float's bit pattern
// (non-negative floats order as unsigned ints); n is a multiple of 8.  One atomic per block: thousands of them on one word
// would take longer than reading the tensor.
template <class E>
__global__ __launch_bounds__(256) void amax_kernel(const typename E::elem* x, long n, unsigned int* out_bits, const int32_t* needed) {
    __shared__ float part[4];
    if (needed && *needed == 0) return;     // nobody will read the maximum
    float m = 0.f;
    const long stride = (long)gridDim.x * 256 * 8;
    long i = (blockIdx.x * 256L + threadIdx.x) * 8;
    if constexpr (sizeof(typename E::elem) == 2) {
        // four 16-byte loads in flight per thread: one at a time leaves the read latency-bound
        for (; i + 3 * stride < n; i += 4 * stride) {
            u32x4 w[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) w[u] = *(const u32x4*)(x + i + u * stride);
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int e = 0; e < 8; ++e) m = fmaxf(m, fabsf((float)((const typename E::elem*)&w[u])[e]));
        }
    }
    for (; i < n; i += stride) {
#pragma unroll
        for (int e = 0; e < 8; ++e) m = fmaxf(m, fabsf((float)x[i + e]));
    }
    m = wave_max(m);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        // rounded up to a power of two: dividing by it is exact, so the fp16 copy of dO / max|dO|
        // holds the caller's bf16 values exactly (a scale with mantissa bits would round every
        // element, and dP - delta, a difference of nearly equal sums, multiplies that rounding)
        unsigned int bits = __float_as_uint(fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3])));
        if ((bits & 0x007fffffu) && bits < 0x7f000000u) bits = (bits & 0x7f800000u) + 0x00800000u;
        atomicMax(out_bits, bits);
    }
}

}  // namespace ea
