// Kernel sequences of one forward / backward call, templated on the element types, the head
// dim and the alpha mode.  Included by the per-type translation units only.
#pragma once
#include <type_traits>

#include "bwd_kernels.hpp"
#include "fwd_kernels.hpp"
#include "launch.hpp"

namespace ea {

constexpr int QB = 1;        // 32*QB owned rows per wave
// waves per work-group (NW) and LDS buffer sets (NBUF) per kernel; a group owns 32*QB*NW rows
constexpr int NW_TAU = 4, NBUF_TAU = 2, QB_TAU = 2;
// list-based threshold kernel: 8 waves (512 rows with two rows per lane), one group per CU, a ring
// of 4 key tiles so that a tile has three tile times to arrive
constexpr int NW_TAUL = 4, NBUF_TAUL = 3;
// 16-bit inputs, alpha 1.5 or 2: the list kernel runs as 8 waves x 32 rows with the histograms of
// two waves sharing words (four waves per SIMD: 3.3 / 2.0 / 1.7 / 1.6 -> 3.2 / 1.7 / 1.5 / 1.5 ms over
// the benchmark's sigma sweep against 4 waves x 64 rows at two per SIMD)
constexpr bool TAUL_PAIRED = true;
constexpr int NW_OUT = 4, NBUF_OUT = 2;
constexpr int NW_DQ = 2, NBUF_DQ = 2;
constexpr int NW_DKDV = 2, NBUF_DKDV = 2;
constexpr int NW_BLIST = 4;   // waves per row group of the backward's support lists

inline int alpha_mode(float alpha) {
    if (alpha == 1.5f) return ALPHA_15;
    if (alpha == 2.0f) return ALPHA_20;
    return ALPHA_GEN;
}

#define EA_HIP(expr)                                              \
    do {                                                          \
        hipError_t e_ = (expr);                                   \
        if (e_ != hipSuccess) { set_last_hip_error((int)e_); return EA_ERR_HIP; } \
    } while (0)

template <class K>
int launch(K kernel, dim3 grid, int threads, hipStream_t s, Params p) {
    hipLaunchKernelGGL(kernel, grid, dim3(threads), 0, s, p);   // all LDS is static
    EA_HIP(hipGetLastError());
    return EA_OK;
}

template <class Ein, class Eout>
int launch_convert(const void* in, void* out, long n, const unsigned int* amax_bits, const int32_t* needed,
                   unsigned long long* stats, hipStream_t s) {
    // values clamped on the way into the narrower type are counted in the first copy of the counters
    hipLaunchKernelGGL((convert_kernel<Ein, Eout>), dim3(2048), dim3(256), 0, s, (const typename Ein::elem*)in,
                       (typename Eout::elem*)out, n, amax_bits, needed, stats + EA_STAT_F16_CLAMPED);
    EA_HIP(hipGetLastError());
    return EA_OK;
}

// fp16 copies of K, Q, V, dO (in this order in `copies`) in one launch; dO is divided by max|dO|
template <class Ein, class Eout, int D>
int launch_convert_rows(const Params& p, void* const copies[4], const unsigned int* dO_amax_bits, const int32_t* needed,
                        hipStream_t s) {
    ConvertJobs jobs;
    jobs.j[0] = ConvertJob{p.K, copies[0], nullptr, 0};
    jobs.j[1] = ConvertJob{p.Q, copies[1], nullptr, 1};
    jobs.j[2] = ConvertJob{p.V, copies[2], nullptr, 0};
    jobs.j[3] = ConvertJob{p.dO, copies[3], dO_amax_bits, 1};
    hipLaunchKernelGGL((convert_rows_kernel<Ein, Eout, D>), dim3(p.BH * (p.N / 64), 4), dim3(256), 0, s, jobs, p.N, needed,
                       (const int32_t*)p.gflag, p.grows, p.causal, p.stats + EA_STAT_F16_CLAMPED);
    EA_HIP(hipGetLastError());
    return EA_OK;
}

// E: input element type; E2: element type of every second-stage product and of the whole backward
// (for bf16 inputs: fp16; the copies are made by convert_kernel)
template <class E, class E2, int D, int AM>
struct Ops {
    static constexpr bool COPY = !std::is_same<E, E2>::value;
    static int fwd(Params p, hipStream_t s) {
        int rc;
        {
            ScopedKernelTime t(EA_TIMER_TAU, s);
            // one dense sweep that lists each row's candidate scores, then histogram, solve and
            // refinement on the lists
            constexpr int QBL = (E::EPL == 8) ? QB_TAU : 1;
            constexpr int NBL = (E::EPL == 8) ? NBUF_TAUL : 2;       // fp32 tiles are twice as large
            static_assert((32 * QBL * NW_TAUL) % (32 * QB * NW_OUT) == 0, "an output group lies inside one row group of the list kernel");
            p.grows = 32 * QBL * NW_TAUL;
            if constexpr (E::EPL == 8 && TAUL_PAIRED && AM != ALPHA_GEN) {
                // eight one-row waves, paired histograms, two tile buffers: four waves per SIMD
                // (general alpha, with its table of powers and heavier solves, measured slower so)
                p.grows = 32 * 8;
                rc = launch(tau_list_kernel<E, D, 1, AM, NBINS, 8, 2, 1>, groups(p, 8, 1), 8 * 64, s, p);
            } else
            rc = launch(tau_list_kernel<E, D, QBL, AM, NBINS, NW_TAUL, NBL>, groups(p, NW_TAUL, QBL), NW_TAUL * 64, s, p);
            if (rc) return rc;
            // sweep-based fallback for row blocks whose lists overflowed (exits at once elsewhere);
            // two rows per lane (packed 16-bit histogram counters) while a bin cannot overflow
            if (QB_TAU == 2 && E::EPL == 8 && p.N < 65536)
                rc = launch(tau_kernel<E, D, QB_TAU, AM, NBINS, NW_TAU, NBUF_TAU>, groups(p, NW_TAU, QB_TAU), NW_TAU * 64, s, p);
            else
                rc = launch(tau_kernel<E, D, 1, AM, NBINS, NW_TAU, NBUF_TAU>, groups(p, NW_TAU), NW_TAU * 64, s, p);
            if (rc) return rc;
        }
        {
            // the fp16 copy of V is for out_kernel: not made when every row group goes by gather
            // (scal[1] counts the row groups that do not)
            ScopedKernelTime t(EA_TIMER_FWD_PREP, s);
            if (COPY) {
                rc = launch_convert<E, E2>(p.V, const_cast<void*>(p.V2), (long)p.BH * p.N * D, nullptr,
                                           p.gflag ? (const int32_t*)(p.scal + 1) : nullptr, p.stats, s);
                if (rc) return rc;
            }
        }
        ScopedKernelTime t(EA_TIMER_OUT, s);
        // sparse row groups: a gather over each row's support; all others: block-sparse matrix products
        if (p.gflag) {
            rc = launch(gather_out_kernel<E, D, AM>, dim3(p.BH * ((p.N + p.grows - 1) / p.grows) * (p.grows / GATHER_ROWS)), 256, s, p);
            if (rc) return rc;
        }
        return launch(out_kernel<E, E2, D, QB, AM, false, NW_OUT, NBUF_OUT>, groups(p, NW_OUT), NW_OUT * 64, s, p);
    }
    static dim3 groups(const Params& p, int nw, int qb = QB) {
        const int rows = 32 * qb * nw;
        return dim3(p.BH * ((p.N + rows - 1) / rows));
    }
    // `copies`: workspace room for K, Q, V, dO in E2 (used when COPY)
    static int bwd(Params p, bool rebuild_mask, void* const copies[4], hipStream_t s) {
        int rc;
        if (rebuild_mask) {
            ScopedKernelTime t(EA_TIMER_MASK, s);
            hipLaunchKernelGGL(full_mask_kernel, dim3(256), dim3(256), 0, s, p.wmask, p.BH, p.T, p.W, p.causal);
            EA_HIP(hipGetLastError());
            rc = launch(out_kernel<E, E2, D, QB, AM, true, NW_OUT, NBUF_OUT>, groups(p, NW_OUT), NW_OUT * 64, s, p);
            if (rc) return rc;
        }
        // sparse row groups: their supports listed from the caller's Q, K (before the 16-bit copies
        // take their place in p); the flags make dq_kernel and dkdv_kernel skip those groups
        constexpr int QBB = 1;                                   // rows per lane of the list kernel (two were measured: slower)
        p.grows = 32 * QBB * NW_BLIST;
        const Params po = p;
        // the 16-bit copies and max|dO| are made only if some row group stays with the matrix kernels
        const int32_t* needed = p.gflag ? p.nplain : nullptr;
        if (p.gflag) {
            ScopedKernelTime t(EA_TIMER_BWD_LIST, s);
            static_assert((32 * QBB * NW_BLIST) % (32 * QB * NW_DQ) == 0 && (32 * QBB * NW_BLIST) % 64 == 0, "a dQ group and a query tile lie inside one row group");
            hipLaunchKernelGGL(zero_ints_kernel, dim3(256), dim3(256), 0, s, p.kcnt, (long)p.BH * p.N + 2);   // and nplain, nmarked, right behind
            EA_HIP(hipGetLastError());
            hipLaunchKernelGGL(mask_popcount_kernel, dim3(64), dim3(256), 0, s, p.mask, (long)p.BH * p.T * p.W, p.nmarked);
            EA_HIP(hipGetLastError());
            if (p.fwd_gflag) {
                // the forward's lists were handed over: no sweep, only the decision per row group
                static_assert(32 * QBB * NW_BLIST <= 128, "one thread per row of a group");
                rc = launch(bwd_decide_kernel<D, AM>, groups(p, NW_BLIST, QBB), 128, s, po);
            } else {
                rc = launch(bwd_list_kernel<E, D, QBB, AM, NW_BLIST>, groups(p, NW_BLIST, QBB), NW_BLIST * 64, s, po);
            }
            if (rc) return rc;
        }
        {
            ScopedKernelTime t(EA_TIMER_BWD_PREP, s);
            if (E2::SCALED) {
                hipLaunchKernelGGL((amax_kernel<E>), dim3(1024), dim3(256), 0, s, (const typename E::elem*)p.dO,
                                   (long)p.BH * p.N * D, p.scal, needed);
                EA_HIP(hipGetLastError());
            }
            if (COPY) {
                // (only the rows the matrix kernels will read: those of the row groups left to them, and
                // the keys such a group can see)
                if ((rc = launch_convert_rows<E, E2, D>(p, copies, E2::SCALED ? p.scal : nullptr, needed, s))) return rc;
                p.K = copies[0]; p.Q = copies[1]; p.V = copies[2]; p.dO = copies[3];
            }
        }
        {
            ScopedKernelTime t(EA_TIMER_DQ, s);
            rc = launch(dq_kernel<E2, E2, D, QB, AM, NW_DQ, NBUF_DQ>, groups(p, NW_DQ), NW_DQ * 64, s, p);
            if (rc) return rc;
        }
        {
            ScopedKernelTime t(EA_TIMER_DKDV, s);
            constexpr int NB2 = (E2::EPL == 8) ? NBUF_DKDV : 1;     // fp32 tiles are twice as large
            // long mask columns are worked off in parts of `len` query tiles when a column can hold
            // more than four (at 256 tiles the extra work-groups cost more than they gain as soon as
            // most row groups go by gather): a small kernel counts every column first, then one
            // launch holds all parts of all columns (most work-groups past the first part leave at once)
            const int len = p.T >= 8 * COL_PART ? COL_PART : COL_PART / 2;
            const int col_parts = p.T > 4 * len ? (p.T + len - 1) / len : 1;
            p.col_part_len = col_parts > 1 ? len : 0;
            if (col_parts > 1) {
                rc = launch(col_count_kernel<D, 32 * QB * NW_DKDV>, groups(p, NW_DKDV), 128, s, p);
                if (rc) return rc;
            }
            rc = launch(dkdv_kernel<E2, E2, D, QB, AM, NW_DKDV, NB2>, dim3(groups(p, NW_DKDV).x * col_parts), NW_DKDV * 64, s, p);
            if (rc) return rc;
        }
        if (p.gflag) {
            // after dkdv_kernel has stored dK, dV: the listed row groups add their share
            ScopedKernelTime t(EA_TIMER_BWD_GATHER, s);
            rc = launch(bwd_rows_kernel<E, D, AM, E2::SCALED>, dim3(p.BH * ((p.N + p.grows - 1) / p.grows) * (p.grows / GATHER_ROWS)), 256, s, po);
            if (rc) return rc;
            rc = launch(bwd_cols_kernel<E, D, E2::SCALED>, dim3(p.BH * ((p.N + BWD_COLS_KEYS - 1) / BWD_COLS_KEYS)), 256, s, po);
            if (rc) return rc;
            rc = launch(bwd_hot_kernel<E, D, AM, E2::SCALED>, dim3(p.BH * ((p.N + p.grows - 1) / p.grows) * (p.grows / GATHER_ROWS)), 256, s, po);
            if (rc) return rc;
        }
        return EA_OK;
    }
};

template <class E, class E2, int D>
int dispatch_alpha(bool is_bwd, Params p, bool rebuild, void* const copies[4], hipStream_t s) {
    // heads with different alphas all take the general-alpha code
    switch (p.hc_table ? ALPHA_GEN : alpha_mode(p.hc.alpha)) {
        case ALPHA_15: return is_bwd ? Ops<E, E2, D, ALPHA_15>::bwd(p, rebuild, copies, s) : Ops<E, E2, D, ALPHA_15>::fwd(p, s);
        case ALPHA_20: return is_bwd ? Ops<E, E2, D, ALPHA_20>::bwd(p, rebuild, copies, s) : Ops<E, E2, D, ALPHA_20>::fwd(p, s);
        default: return is_bwd ? Ops<E, E2, D, ALPHA_GEN>::bwd(p, rebuild, copies, s) : Ops<E, E2, D, ALPHA_GEN>::fwd(p, s);
    }
}

}  // namespace ea
