// Host side of the C ABI declared in include/entmax_attn.h: argument checks, workspace
// carving, kernel dispatch over (dtype, head dim, alpha mode).  No allocation, no
// synchronisation: every launch goes to the caller's stream.
#include "../../include/entmax_attn.h"

#include <math.h>

#include <type_traits>

#include "bwd_kernels.hpp"
#include "fwd_kernels.hpp"

namespace {

using namespace ea;

constexpr int QB = 1;        // 32*QB owned rows per wave
// waves per work-group (NW) and LDS buffer sets (NBUF) per kernel; a group owns 32*QB*NW rows
constexpr int NW_TAU = 4, NBUF_TAU = 2;
constexpr int NW_OUT = 4, NBUF_OUT = 2;
constexpr int NW_DQ = 2, NBUF_DQ = 2;
constexpr int NW_DKDV = 2, NBUF_DKDV = 2;
constexpr int NBINS = 64;    // histogram bins B (Sec. 3.1): bracket width 1/64 after Phase 2
constexpr int MAX_SWEEPS = 12;

thread_local int g_last_hip_error = 0;

// Optional per-kernel timing with HIP events recorded on the caller's stream around each launch.
// Off by default (then nothing below runs).  Slots name the kernels of one fwd or bwd call.
constexpr int TIMER_SLOTS = EA_TIMER_SLOTS;
constexpr int TIMER_MAX_CALLS = 256;
struct KernelTimer {
    bool enabled = false;
    int ncalls = 0;                                   // calls recorded since the last reset
    hipEvent_t ev[TIMER_MAX_CALLS][TIMER_SLOTS][2];
    unsigned char used[TIMER_MAX_CALLS][TIMER_SLOTS];
    bool created = false;
} g_timer;
int g_timer_call = -1;                                // slot row of the call in flight, -1 = off

struct ScopedKernelTime {
    int slot; hipStream_t s; bool on;
    ScopedKernelTime(int slot_, hipStream_t s_) : slot(slot_), s(s_), on(g_timer_call >= 0) {
        if (on) (void)hipEventRecord(g_timer.ev[g_timer_call][slot][0], s);
    }
    ~ScopedKernelTime() {
        if (on) { (void)hipEventRecord(g_timer.ev[g_timer_call][slot][1], s); g_timer.used[g_timer_call][slot] = 1; }
    }
};
void timer_begin_call() {
    g_timer_call = -1;
    if (g_timer.enabled && g_timer.ncalls < TIMER_MAX_CALLS) {
        g_timer_call = g_timer.ncalls++;
        for (int k = 0; k < TIMER_SLOTS; ++k) g_timer.used[g_timer_call][k] = 0;
    }
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct Layout {
    size_t stats, a, b, c, d, delta, mask, wmask, tmax, rs_lo, rs_hi, rs_f1, rs_state, total;
};

// element size of the stage-2 copies
inline size_t t_elem(ea_dtype t) { return t == EA_BF16 ? 2 : 4; }

Layout fwd_layout(int B, int H, int N, int d, ea_dtype t) {
    Layout L{};
    const size_t BH = (size_t)B * H, T = N / 64, W = (T + 31) / 32;
    size_t off = 0;
    L.stats = off; off += align256(EA_STATS_WORDS * 8);
    L.a = off; off += align256(BH * N * d * t_elem(t));          // V in the stage-2 type
    L.wmask = off; off += align256(BH * T * W * 4);
    L.tmax = off; off += align256(BH * T * (size_t)N * 2);       // per-row key-tile maxima, fp16
    L.rs_lo = off; off += align256(BH * N * 4);                  // solver state between the two kernels
    L.rs_hi = off; off += align256(BH * N * 4);
    L.rs_f1 = off; off += align256(BH * N * 4);
    L.rs_state = off; off += align256(BH * N * 4);
    L.total = off;
    return L;
}
Layout bwd_layout(int B, int H, int N, int d, ea_dtype t) {
    Layout L{};
    const size_t BH = (size_t)B * H, T = N / 64, W = (T + 31) / 32;
    size_t off = 0;
    L.stats = off; off += align256(EA_STATS_WORDS * 8);
    L.a = off; off += align256(BH * N * d * t_elem(t));          // K, Q, V, dO in the stage-2 type
    L.b = off; off += align256(BH * N * d * t_elem(t));
    L.c = off; off += align256(BH * N * d * t_elem(t));
    L.d = off; off += align256(BH * N * d * t_elem(t));
    L.delta = off; off += align256(BH * N * 4);
    L.mask = off; off += align256(BH * T * W * 4);               // rebuilt mask (mask == NULL)
    L.wmask = off; off += align256(BH * T * W * 4);
    L.total = off;
    return L;
}

int check_common(int B, int H, int N, int d, ea_dtype t, float alpha) {
    if (t != EA_F32 && t != EA_BF16) return EA_ERR_DTYPE;
    if (B <= 0 || H <= 0 || N <= 0 || N % 64 != 0 || N > 131072 || (d != 64 && d != 128)) return EA_ERR_SHAPE;
    if ((long)B * H > 65535) return EA_ERR_SHAPE;
    if (!isfinite(alpha) || !(alpha > 1.f) || alpha > 2.f) return EA_ERR_ALPHA;
    return EA_OK;
}

int alpha_mode(float alpha) {
    if (alpha == 1.5f) return ALPHA_15;
    if (alpha == 2.0f) return ALPHA_20;
    return ALPHA_GEN;
}

#define EA_HIP(expr)                                              \
    do {                                                          \
        hipError_t e_ = (expr);                                   \
        if (e_ != hipSuccess) { g_last_hip_error = (int)e_; return EA_ERR_HIP; } \
    } while (0)

template <class K>
int launch(K kernel, dim3 grid, int threads, hipStream_t s, Params p) {
    hipLaunchKernelGGL(kernel, grid, dim3(threads), 0, s, p);   // all LDS is static
    EA_HIP(hipGetLastError());
    return EA_OK;
}

template <class Ein, class Eout>
int launch_convert(const void* in, void* out, long n, const unsigned int* amax_bits, hipStream_t s) {
    hipLaunchKernelGGL((convert_kernel<Ein, Eout>), dim3(2048), dim3(256), 0, s, (const typename Ein::elem*)in,
                       (typename Eout::elem*)out, n, amax_bits);
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
            ScopedKernelTime t(EA_TIMER_FWD_PREP, s);
            if (COPY) {
                rc = launch_convert<E, E2>(p.V, const_cast<void*>(p.V2), (long)p.BH * p.N * D, nullptr, s);
                if (rc) return rc;
            }
        }
        {
            ScopedKernelTime t(EA_TIMER_TAU, s);
            rc = launch(tau_kernel<E, D, QB, AM, NBINS, NW_TAU, NBUF_TAU>, groups(p, NW_TAU), NW_TAU * 64, s, p);
            if (rc) return rc;
        }
        ScopedKernelTime t(EA_TIMER_OUT, s);
        return launch(out_kernel<E, E2, D, QB, AM, false, NW_OUT, NBUF_OUT>, groups(p, NW_OUT), NW_OUT * 64, s, p);
    }
    static dim3 groups(const Params& p, int nw) {
        const int rows = 32 * QB * nw;
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
        {
            ScopedKernelTime t(EA_TIMER_BWD_PREP, s);
            if (E2::SCALED) {
                hipLaunchKernelGGL((amax_kernel<E>), dim3(2048), dim3(256), 0, s, (const typename E::elem*)p.dO,
                                   (long)p.BH * p.N * D, p.scal);
                EA_HIP(hipGetLastError());
            }
            if (COPY) {
                const long n = (long)p.BH * p.N * D;
                if ((rc = launch_convert<E, E2>(p.K, copies[0], n, nullptr, s))) return rc;
                if ((rc = launch_convert<E, E2>(p.Q, copies[1], n, nullptr, s))) return rc;
                if ((rc = launch_convert<E, E2>(p.V, copies[2], n, nullptr, s))) return rc;
                if ((rc = launch_convert<E, E2>(p.dO, copies[3], n, E2::SCALED ? p.scal : nullptr, s))) return rc;
                p.K = copies[0]; p.Q = copies[1]; p.V = copies[2]; p.dO = copies[3];
            }
        }
        {
            ScopedKernelTime t(EA_TIMER_DQ, s);
            rc = launch(dq_kernel<E2, E2, D, QB, AM, NW_DQ, NBUF_DQ>, groups(p, NW_DQ), NW_DQ * 64, s, p);
            if (rc) return rc;
        }
        ScopedKernelTime t(EA_TIMER_DKDV, s);
        constexpr int NB2 = (E2::EPL == 8) ? NBUF_DKDV : 1;     // fp32 tiles are twice as large
        return launch(dkdv_kernel<E2, E2, D, QB, AM, NW_DKDV, NB2>, groups(p, NW_DKDV), NW_DKDV * 64, s, p);
    }
};

template <class E, class E2, int D>
int dispatch_alpha(bool is_bwd, Params p, bool rebuild, void* const copies[4], hipStream_t s) {
    switch (alpha_mode(p.alpha)) {
        case ALPHA_15: return is_bwd ? Ops<E, E2, D, ALPHA_15>::bwd(p, rebuild, copies, s) : Ops<E, E2, D, ALPHA_15>::fwd(p, s);
        case ALPHA_20: return is_bwd ? Ops<E, E2, D, ALPHA_20>::bwd(p, rebuild, copies, s) : Ops<E, E2, D, ALPHA_20>::fwd(p, s);
        default: return is_bwd ? Ops<E, E2, D, ALPHA_GEN>::bwd(p, rebuild, copies, s) : Ops<E, E2, D, ALPHA_GEN>::fwd(p, s);
    }
}

int dispatch(bool is_bwd, ea_dtype t, int d, Params p, bool rebuild, void* const copies[4], hipStream_t s) {
    // bf16 inputs: the forward scores (Q K^T) run on bf16 MFMA straight from the inputs.  Every
    // second-stage product (P V, dS K, P^T dO, dS^T Q) and the whole backward run on fp16 MFMA
    // from fp16 copies: P lies in [0,1] and dS, dO are divided by known bounds first, so fp16's
    // range suffices and its 3 extra mantissa bits keep the rounding of P and dS well inside the
    // tolerances; bf16 values convert to fp16 exactly while 2^-17 <= |x| < 65504 (smaller ones
    // within 2^-25 absolute; larger ones are outside this library's domain).
    if (t == EA_BF16) {
        if (d == 64) return dispatch_alpha<Bf16, F16, 64>(is_bwd, p, rebuild, copies, s);
        return dispatch_alpha<Bf16, F16, 128>(is_bwd, p, rebuild, copies, s);
    }
    if (d == 64) return dispatch_alpha<F32, F32, 64>(is_bwd, p, rebuild, copies, s);
    return dispatch_alpha<F32, F32, 128>(is_bwd, p, rebuild, copies, s);
}

Params base_params(int B, int H, int N, int d, ea_dtype t, float alpha, int causal) {
    Params p{};
    p.BH = B * H; p.N = N; p.T = N / 64; p.W = (p.T + 31) / 32;
    p.causal = causal ? 1 : 0;
    p.alpha = alpha;
    p.inv_sqrt_d = 1.f / sqrtf((float)d);
    p.c = (alpha - 1.f) * p.inv_sqrt_d;
    p.r = 1.f / (alpha - 1.f);
    p.tol = (t == EA_BF16) ? 1e-4f : 1e-6f;
    p.max_sweeps = MAX_SWEEPS;
    return p;
}

}  // namespace

extern "C" {

int entmax_attn_mask_tile(void) { return ea::TILE; }
int entmax_attn_histogram_bins(void) { return NBINS; }
int entmax_attn_last_hip_error(void) { return g_last_hip_error; }

size_t entmax_attn_workspace_bytes(int B, int H, int N, int d, ea_dtype t, int causal, int is_bwd) {
    (void)causal;
    if (check_common(B, H, N, d, t, 1.5f) != EA_OK) return 0;
    return is_bwd ? bwd_layout(B, H, N, d, t).total : fwd_layout(B, H, N, d, t).total;
}

int entmax_attn_fwd(const void* Q, const void* K, const void* V, float* O, float* tau, int32_t* block_mask,
                    int32_t* iters, int B, int H, int N, int d, ea_dtype t, float alpha, int causal,
                    void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!Q || !K || !V || !O || !tau || !block_mask) return EA_ERR_NULL;
    int rc = check_common(B, H, N, d, t, alpha);
    if (rc) return rc;
    const Layout L = fwd_layout(B, H, N, d, t);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < L.total) return EA_ERR_WORKSPACE;
    char* ws = (char*)workspace;
    hipStream_t s = (hipStream_t)hip_stream;
    Params p = base_params(B, H, N, d, t, alpha, causal);
    p.Q = Q; p.K = K; p.V = V;
    p.O = O; p.tau = tau; p.mask = block_mask; p.iters = iters;
    p.stats = (unsigned long long*)(ws + L.stats);
    p.V2 = (t == EA_BF16) ? (const void*)(ws + L.a) : V;
    p.wmask = (int32_t*)(ws + L.wmask);
    p.tmax = (_Float16*)(ws + L.tmax);
    p.rs_lo = (float*)(ws + L.rs_lo); p.rs_hi = (float*)(ws + L.rs_hi); p.rs_f1 = (float*)(ws + L.rs_f1); p.rs_state = (int*)(ws + L.rs_state);
    hipLaunchKernelGGL(zero_stats_kernel, dim3(1), dim3(64), 0, s, p.stats, EA_STATS_WORDS, (unsigned int*)nullptr);
    EA_HIP(hipGetLastError());
    timer_begin_call();
    return dispatch(false, t, d, p, false, nullptr, s);
}

int entmax_attn_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* tau,
                    const int32_t* block_mask, float* dQ, float* dK, float* dV, int B, int H, int N, int d,
                    ea_dtype t, float alpha, int causal, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!Q || !K || !V || !dO || !tau || !dQ || !dK || !dV) return EA_ERR_NULL;
    int rc = check_common(B, H, N, d, t, alpha);
    if (rc) return rc;
    const Layout L = bwd_layout(B, H, N, d, t);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < L.total) return EA_ERR_WORKSPACE;
    char* ws = (char*)workspace;
    hipStream_t s = (hipStream_t)hip_stream;
    Params p = base_params(B, H, N, d, t, alpha, causal);
    p.Q = Q; p.K = K; p.V = V; p.dO = dO;
    p.tau = const_cast<float*>(tau);
    p.O = const_cast<float*>((const float*)O);
    p.dQ = dQ; p.dK = dK; p.dV = dV;
    p.stats = (unsigned long long*)(ws + L.stats);
    void* const copies[4] = {ws + L.a, ws + L.b, ws + L.c, ws + L.d};
    p.delta = (float*)(ws + L.delta);
    p.wmask = (int32_t*)(ws + L.wmask);
    const bool rebuild = (block_mask == nullptr);
    p.mask = rebuild ? (int32_t*)(ws + L.mask) : const_cast<int32_t*>(block_mask);
    p.scal = (unsigned int*)(ws + L.stats + EA_STATS_WORDS * 8);
    hipLaunchKernelGGL(zero_stats_kernel, dim3(1), dim3(64), 0, s, p.stats, EA_STATS_WORDS, p.scal);
    EA_HIP(hipGetLastError());
    timer_begin_call();
    return dispatch(true, t, d, p, rebuild, copies, s);
}

int entmax_attn_timer_enable(int on) {
    if (on && !g_timer.created) {
        for (int c = 0; c < TIMER_MAX_CALLS; ++c)
            for (int k = 0; k < TIMER_SLOTS; ++k)
                for (int e = 0; e < 2; ++e) EA_HIP(hipEventCreate(&g_timer.ev[c][k][e]));
        g_timer.created = true;
    }
    g_timer.enabled = on != 0;
    g_timer.ncalls = 0;
    g_timer_call = -1;
    return EA_OK;
}

int entmax_attn_timer_read(float* ms_sum, int* launches, int slots) {
    if (!ms_sum || !launches || slots < TIMER_SLOTS) return EA_ERR_NULL;
    for (int k = 0; k < TIMER_SLOTS; ++k) { ms_sum[k] = 0.f; launches[k] = 0; }
    for (int c = 0; c < g_timer.ncalls; ++c)
        for (int k = 0; k < TIMER_SLOTS; ++k) {
            if (!g_timer.used[c][k]) continue;
            EA_HIP(hipEventSynchronize(g_timer.ev[c][k][1]));
            float ms = 0.f;
            EA_HIP(hipEventElapsedTime(&ms, g_timer.ev[c][k][0], g_timer.ev[c][k][1]));
            ms_sum[k] += ms;
            launches[k] += 1;
        }
    g_timer.ncalls = 0;
    return EA_OK;
}

const char* entmax_attn_strerror(int code) {
    switch (code) {
        case EA_OK: return "ok";
        case EA_ERR_NULL: return "a required pointer is NULL";
        case EA_ERR_ALPHA: return "alpha must be finite and in (1, 2]";
        case EA_ERR_SHAPE: return "bad shape: need B,H > 0, N a positive multiple of 64 (<= 131072), d in {64, 128}";
        case EA_ERR_DTYPE: return "unknown dtype";
        case EA_ERR_WORKSPACE: return "workspace is NULL, not 256-byte aligned, or too small";
        case EA_ERR_HIP: return "a HIP call failed (see entmax_attn_last_hip_error)";
        default: return "unknown error code";
    }
}

}  // extern "C"
