// Host side of the C ABI declared in include/entmax_attn.h: argument checks, workspace
// carving, dispatch to the per-type kernel sequences (ops.hpp).  No allocation, no
// synchronisation: every launch goes to the caller's stream.
#include <math.h>

#include "fwd_kernels.hpp"
#include "launch.hpp"

namespace {

using namespace ea;

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
    unsigned char created[TIMER_MAX_CALLS][TIMER_SLOTS];    // events exist (made when a slot is first recorded, kept)
} g_timer;
int g_timer_call = -1;                                // slot row of the call in flight, -1 = off

void timer_begin_call() {
    g_timer_call = -1;
    if (g_timer.enabled && g_timer.ncalls < TIMER_MAX_CALLS) {
        g_timer_call = g_timer.ncalls++;
        for (int k = 0; k < TIMER_SLOTS; ++k) g_timer.used[g_timer_call][k] = 0;
    }
}

static_assert(STATS_WORDS == EA_STATS_WORDS && STATS_COPIES == EA_STATS_COPIES, "header and kernels disagree");
constexpr size_t STATS_BYTES = (size_t)EA_STATS_WORDS * EA_STATS_COPIES * 8;

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
thread_local bool g_gather_enabled = true;      // the gather switch of the calling host thread
thread_local bool g_right_edge = false;         // right-edge binning without refinement (approximate forward), same scope

struct Layout {
    size_t stats, hc, a, b, c, d, delta, ntau, mask, wmask, tmax, rs_lo, rs_hi, rs_f1, rs_state, rs_t0, rs_up0, lists, oflag, scnt, gflag, kcnt, klist, defer, colcnt, total;
};

// element size of the stage-2 copies
inline size_t t_elem(int t) { return t == EA_BF16 ? 2 : 4; }

Layout fwd_layout(int B, int H, int N, int d, int t) {
    Layout L{};
    const size_t BH = (size_t)B * H, T = N / 64, W = (T + 31) / 32;
    size_t off = 0;
    L.stats = off; off += align256(STATS_BYTES + 256);   // counters, then the scale words
    L.hc = off; off += align256((size_t)H * sizeof(HeadConsts)); // per-head constants (alpha per head)
    L.a = off; off += align256(BH * N * d * t_elem(t));          // V in the stage-2 type
    L.wmask = off; off += align256(BH * T * W * 4);
    L.tmax = off; off += align256(BH * T * (size_t)N * 2);       // per-row key-tile maxima, fp16
    L.rs_lo = off; off += align256(BH * N * 4);                  // solver state between the two kernels
    L.rs_hi = off; off += align256(BH * N * 4);
    L.rs_f1 = off; off += align256(BH * N * 4);
    L.rs_state = off; off += align256(BH * N * 4);
    L.rs_t0 = off; off += align256(BH * N * 4);                  // tau_0 and bracket end of the histogram stage
    L.rs_up0 = off; off += align256(BH * N * 4);
    L.oflag = off; off += align256(BH * T * 4);                  // 64-row blocks whose candidate lists overflowed
    L.scnt = off; off += align256(BH * N * 2 * 4);               // support entries at the front of each list
    L.gflag = off; off += align256(BH * ((size_t)N / 128 + 1) * 4);   // row groups that take the gather kernel
    L.lists = off; off += align256(BH * N * (size_t)(2 * LIST_CAP * 8));   // candidate lists, two per row
    L.total = off;
    return L;
}
Layout bwd_layout(int B, int H, int N, int d, int t) {
    Layout L{};
    const size_t BH = (size_t)B * H, T = N / 64, W = (T + 31) / 32;
    size_t off = 0;
    L.stats = off; off += align256(STATS_BYTES + 256);   // counters, then the scale words
    L.hc = off; off += align256((size_t)H * sizeof(HeadConsts)); // per-head constants (alpha per head)
    L.a = off; off += align256(BH * N * d * t_elem(t));          // K, Q, V, dO in the stage-2 type
    L.b = off; off += align256(BH * N * d * t_elem(t));
    L.c = off; off += align256(BH * N * d * t_elem(t));
    L.d = off; off += align256(BH * N * d * t_elem(t));
    L.delta = off; off += align256(BH * N * 4);
    L.ntau = off; off += align256(BH * N * 4);
    L.mask = off; off += align256(BH * T * W * 4);               // rebuilt mask (mask == NULL)
    L.wmask = off; off += align256(BH * T * W * 4);
    // sparse row groups: support lists (two per row), their lengths, group flags, lists by key
    L.lists = off; off += align256(BH * N * (size_t)(2 * BWD_LIST_CAP * 8));
    L.scnt = off; off += align256(BH * N * 2 * 4);
    L.gflag = off; off += align256(BH * ((size_t)N / 128 + 1) * 4);
    L.kcnt = off; off += align256(BH * N * 4 + 8);               // and two counters: row groups on the matrix path, set mask bits
    L.klist = off; off += align256(BH * N * (size_t)(KEY_LIST_CAP * 16));
    L.defer = off; off += align256(BH * N * 4);
    L.colcnt = off; off += align256(BH * T * 4);                 // query tiles per key tile's mask column (dkdv_kernel's parts)
    L.total = off;
    return L;
}

bool alpha_ok(float alpha) { return isfinite(alpha) && alpha > 1.f && alpha <= EA_ALPHA_MAX; }

int check_common(int B, int H, int N, int d, int t, float alpha) {
    if (t != EA_F32 && t != EA_BF16) return EA_ERR_DTYPE;
    if (B <= 0 || H <= 0 || N <= 0 || N % 64 != 0 || N > 131072 || (d != 64 && d != 128)) return EA_ERR_SHAPE;
    if ((long)B * H > 65535) return EA_ERR_SHAPE;
    if (!alpha_ok(alpha)) return EA_ERR_ALPHA;
    return EA_OK;
}

#define EA_HIP(expr)                                              \
    do {                                                          \
        hipError_t e_ = (expr);                                   \
        if (e_ != hipSuccess) { g_last_hip_error = (int)e_; return EA_ERR_HIP; } \
    } while (0)

int dispatch(bool is_bwd, int t, int d, const Params& p, bool rebuild, void* const copies[4], hipStream_t s) {
    if (t == EA_BF16) return d == 64 ? run_bf16_d64(is_bwd, p, rebuild, copies, s) : run_bf16_d128(is_bwd, p, rebuild, copies, s);
    return d == 64 ? run_f32_d64(is_bwd, p, rebuild, copies, s) : run_f32_d128(is_bwd, p, rebuild, copies, s);
}

// The alpha-dependent constants (host and device: the per-head table is filled by a kernel).
__host__ __device__ inline HeadConsts head_consts_of(float alpha, float inv_sqrt_d) {
    HeadConsts k;
    k.alpha = alpha;
    k.c = (alpha - 1.f) * inv_sqrt_d;
    k.r = 1.f / (alpha - 1.f);
    int ex = 0;
    const float mant = frexpf(k.c, &ex);          // c = mant * 2^ex, 0.5 <= mant < 1
    k.kappa = ldexpf(1.f, ex - 1);
    k.rho = 2.f * mant;
    k.rho_p = powf(k.rho, k.r);
    k.rho_u = powf(k.rho, k.r - 1.f);
    k.pad = 0.f;
    return k;
}

// Up to 32 alphas travel as kernel arguments (the caller's array is host memory and need not
// outlive the call); thread i writes the constants of head first + i.
struct AlphaChunk { float a[32]; };
__global__ void head_consts_kernel(AlphaChunk chunk, int first, int count, float inv_sqrt_d, HeadConsts* table) {
    const int i = threadIdx.x;
    if (i < count) table[first + i] = head_consts_of(chunk.a[i], inv_sqrt_d);
}

Params base_params(int B, int H, int N, int d, int t, float alpha, int causal) {
    Params p{};
    p.BH = B * H; p.N = N; p.T = N / 64; p.W = (p.T + 31) / 32;
    p.causal = causal ? 1 : 0;
    p.inv_sqrt_d = 1.f / sqrtf((float)d);
    p.hc = head_consts_of(alpha, p.inv_sqrt_d);
    p.hc_table = nullptr;
    p.H = H;
    p.tol = (t == EA_BF16) ? 1e-4f : 1e-6f;
    p.max_sweeps = MAX_SWEEPS;
    return p;
}

}  // namespace

// Matrix-core rate probe: every wave issues `iters` rounds of 32 independent 32x32x16 fp16 MFMAs
// on operands read from `data` (8192 halves, which the caller fills, e.g. with Gaussian values:
// the sustained clock of the chip depends on how many operand bits toggle).  No memory traffic in
// the loop; 4 waves per group, so a grid of 256 (512) groups puts one (two) waves on every SIMD.
__global__ __launch_bounds__(256) void mfma_probe_kernel(const f16x8* data, float* sink, int iters) {
    f32x16 acc[4];
    for (int a = 0; a < 4; ++a)
        for (int v = 0; v < 16; ++v) acc[a][v] = 0.f;
    f16x8 A[8], B[4];
    for (int i = 0; i < 8; ++i) A[i] = data[(threadIdx.x + 97 * i) & 1023];
    for (int i = 0; i < 4; ++i) B[i] = data[(threadIdx.x * 7 + 131 * i + 5) & 1023];
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int a = 0; a < 4; ++a) acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_f16(A[(u + a) & 7], B[a], acc[a], 0, 0, 0);
    }
    float t = 0.f;
    for (int a = 0; a < 4; ++a)
        for (int v = 0; v < 16; ++v) t += acc[a][v];
    sink[blockIdx.x * 256 + threadIdx.x] = t;
}

// How much vector-ALU work hides under the matrix pipe: every wave runs `iters` rounds of 16
// dependent-in-pairs 32x32x16 bf16 MFMAs (MF) followed by NV independent v_add_u32; 8 waves per
// group, and the fixed grid of 512 groups puts four waves on every SIMD of an MI355X, so one
// wave's additions can run while another's MFMAs do.  Registers only, no memory traffic.
template <int NV, bool MF>
__global__ __launch_bounds__(512) void coissue_probe_kernel(float* sink, int iters, float seed) {
    f32x16 c0, c1;
    for (int v = 0; v < 16; ++v) { c0[v] = 0.f; c1[v] = 0.f; }
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(seed + threadIdx.x * 0.001f + i); b[i] = (__bf16)(seed * 0.5f + i); }
    unsigned x0 = threadIdx.x, x1 = 1, x2 = 2, x3 = 3;
    for (int it = 0; it < iters; ++it) {
        if constexpr (MF) {
#pragma unroll
            for (int m = 0; m < 8; ++m) {
                asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c0) : "v"(a), "v"(b));
                asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c1) : "v"(a), "v"(b));
            }
        }
#pragma unroll
        for (int n = 0; n < NV / 2; ++n) {
            asm volatile("v_add_u32 %0, %0, %1" : "+v"(x0) : "v"(x1));
            asm volatile("v_add_u32 %0, %0, %1" : "+v"(x2) : "v"(x3));
        }
    }
    float t = (float)(x0 + x2);
    for (int v = 0; v < 16; ++v) t += c0[v] + c1[v];
    sink[blockIdx.x * 512 + threadIdx.x] = t;
}

namespace ea {
void set_last_hip_error(int e) { g_last_hip_error = e; }
void timer_begin() { timer_begin_call(); }
void timer_mark(int slot, int which, hipStream_t s) {
    if (g_timer_call < 0) return;
    if (!g_timer.created[g_timer_call][slot]) {
        if (hipEventCreate(&g_timer.ev[g_timer_call][slot][0]) != hipSuccess) return;
        if (hipEventCreate(&g_timer.ev[g_timer_call][slot][1]) != hipSuccess) { (void)hipEventDestroy(g_timer.ev[g_timer_call][slot][0]); return; }
        g_timer.created[g_timer_call][slot] = 1;
    }
    (void)hipEventRecord(g_timer.ev[g_timer_call][slot][which], s);
    if (which == 1) g_timer.used[g_timer_call][slot] = 1;
}
}  // namespace ea

extern "C" {

int entmax_attn_mask_tile(void) { return ea::TILE; }
int entmax_attn_histogram_bins(void) { return NBINS; }
int entmax_attn_last_hip_error(void) { return g_last_hip_error; }

size_t entmax_attn_workspace_bytes(int B, int H, int N, int d, int t, int causal, int is_bwd) {
    (void)causal;
    if (check_common(B, H, N, d, t, 1.5f) != EA_OK) return 0;
    return is_bwd ? bwd_layout(B, H, N, d, t).total : fwd_layout(B, H, N, d, t).total;
}

}  // extern "C"

namespace {
// alpha_h: null (one alpha for all heads) or H alphas in host memory
int check_alphas(int H, const float* alpha_h, float& alpha) {
    if (!alpha_h) return EA_OK;
    bool same = true;
    for (int i = 0; i < H; ++i) {
        if (!alpha_ok(alpha_h[i])) return EA_ERR_ALPHA;
        same = same && alpha_h[i] == alpha_h[0];
    }
    alpha = alpha_h[0];
    return same ? 1 : 2;      // 1: all heads alike (the single-alpha path serves), 2: a table is needed
}
int fill_head_table(const float* alpha_h, int H, float inv_sqrt_d, HeadConsts* table, hipStream_t s) {
    for (int first = 0; first < H; first += 32) {
        AlphaChunk chunk{};
        const int count = H - first < 32 ? H - first : 32;
        for (int i = 0; i < count; ++i) chunk.a[i] = alpha_h[first + i];
        hipLaunchKernelGGL(head_consts_kernel, dim3(1), dim3(32), 0, s, chunk, first, count, inv_sqrt_d, table);
        EA_HIP(hipGetLastError());
    }
    return EA_OK;
}

int fwd_impl(const void* Q, const void* K, const void* V, float* O, float* tau, int32_t* block_mask,
             int32_t* iters, int B, int H, int N, int d, int t, float alpha, const float* alpha_h, int causal,
             void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!Q || !K || !V || !O || !tau || !block_mask) return EA_ERR_NULL;
    int rc = check_common(B, H, N, d, t, alpha_h ? 1.5f : alpha);
    if (rc) return rc;
    const int per_head = check_alphas(H, alpha_h, alpha);
    if (per_head < 0) return per_head;
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
    p.lists = ws + L.lists;
    p.oflag = (int32_t*)(ws + L.oflag);
    p.scnt = (int32_t*)(ws + L.scnt);
    p.gflag = g_gather_enabled ? (int32_t*)(ws + L.gflag) : nullptr;
    p.right_edge = g_right_edge ? 1 : 0;
    p.rs_lo = (float*)(ws + L.rs_lo); p.rs_hi = (float*)(ws + L.rs_hi); p.rs_f1 = (float*)(ws + L.rs_f1); p.rs_state = (int*)(ws + L.rs_state);
    p.rs_t0 = (float*)(ws + L.rs_t0); p.rs_up0 = (float*)(ws + L.rs_up0);
    p.scal = (unsigned int*)(ws + L.stats + STATS_BYTES);
    hipLaunchKernelGGL(zero_stats_kernel, dim3(1), dim3(256), 0, s, p.stats, EA_STATS_WORDS * EA_STATS_COPIES, p.scal);
    EA_HIP(hipGetLastError());
    if (per_head == 2) {
        p.hc_table = (const HeadConsts*)(ws + L.hc);
        if ((rc = fill_head_table(alpha_h, H, p.inv_sqrt_d, (HeadConsts*)(ws + L.hc), s))) return rc;
    }
    timer_begin_call();
    return dispatch(false, t, d, p, false, nullptr, s);
}

int bwd_impl(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* tau,
             const int32_t* block_mask, float* dQ, float* dK, float* dV, int B, int H, int N, int d,
             int t, float alpha, const float* alpha_h, int causal, void* workspace, size_t workspace_bytes,
             void* hip_stream, void* fwd_workspace = nullptr, size_t fwd_workspace_bytes = 0) {
    if (!Q || !K || !V || !dO || !tau || !dQ || !dK || !dV) return EA_ERR_NULL;
    int rc = check_common(B, H, N, d, t, alpha_h ? 1.5f : alpha);
    if (rc) return rc;
    const int per_head = check_alphas(H, alpha_h, alpha);
    if (per_head < 0) return per_head;
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
    p.ntau = (float*)(ws + L.ntau);
    p.wmask = (int32_t*)(ws + L.wmask);
    const bool rebuild = (block_mask == nullptr);
    p.mask = rebuild ? (int32_t*)(ws + L.mask) : const_cast<int32_t*>(block_mask);
    p.scal = (unsigned int*)(ws + L.stats + STATS_BYTES);
    p.lists = ws + L.lists;
    p.scnt = (int32_t*)(ws + L.scnt);
    p.gflag = g_gather_enabled ? (int32_t*)(ws + L.gflag) : nullptr;
    p.kcnt = (int32_t*)(ws + L.kcnt);
    p.nplain = p.kcnt + (size_t)B * H * N;
    p.nmarked = p.nplain + 1;
    p.klist = ws + L.klist;
    p.defer = (int32_t*)(ws + L.defer);
    p.colcnt = (int32_t*)(ws + L.colcnt);
    p.list_cap = BWD_LIST_CAP;
    if (fwd_workspace) {
        // the forward's candidate lists (supports at the front), their counts and group flags
        const Layout F = fwd_layout(B, H, N, d, t);
        if (((uintptr_t)fwd_workspace & 255) || fwd_workspace_bytes < F.total || !block_mask) return EA_ERR_WORKSPACE;
        if (p.gflag) {
            char* fw = (char*)fwd_workspace;
            p.lists = fw + F.lists;
            p.scnt = (int32_t*)(fw + F.scnt);
            p.fwd_gflag = (const int32_t*)(fw + F.gflag);
            p.fwd_scal = (const unsigned int*)(fw + F.stats + STATS_BYTES);
            p.list_cap = LIST_CAP;
        }
    }
    hipLaunchKernelGGL(zero_stats_kernel, dim3(1), dim3(256), 0, s, p.stats, EA_STATS_WORDS * EA_STATS_COPIES, p.scal);
    EA_HIP(hipGetLastError());
    if (per_head == 2) {
        p.hc_table = (const HeadConsts*)(ws + L.hc);
        if ((rc = fill_head_table(alpha_h, H, p.inv_sqrt_d, (HeadConsts*)(ws + L.hc), s))) return rc;
    }
    timer_begin_call();
    return dispatch(true, t, d, p, rebuild, copies, s);
}
}  // namespace

extern "C" {

int entmax_attn_fwd(const void* Q, const void* K, const void* V, float* O, float* tau, int32_t* block_mask,
                    int32_t* iters, int B, int H, int N, int d, int t, float alpha, int causal,
                    void* workspace, size_t workspace_bytes, void* hip_stream) {
    return fwd_impl(Q, K, V, O, tau, block_mask, iters, B, H, N, d, t, alpha, nullptr, causal, workspace, workspace_bytes, hip_stream);
}
int entmax_attn_fwd_alpha_per_head(const void* Q, const void* K, const void* V, float* O, float* tau, int32_t* block_mask,
                                   int32_t* iters, int B, int H, int N, int d, int t, const float* alpha_per_head,
                                   int causal, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!alpha_per_head) return EA_ERR_NULL;
    return fwd_impl(Q, K, V, O, tau, block_mask, iters, B, H, N, d, t, 0.f, alpha_per_head, causal, workspace, workspace_bytes, hip_stream);
}
int entmax_attn_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* tau,
                    const int32_t* block_mask, float* dQ, float* dK, float* dV, int B, int H, int N, int d,
                    int t, float alpha, int causal, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return bwd_impl(Q, K, V, O, dO, tau, block_mask, dQ, dK, dV, B, H, N, d, t, alpha, nullptr, causal, workspace, workspace_bytes, hip_stream);
}
int entmax_attn_bwd_with_lists(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* tau,
                               const int32_t* block_mask, void* fwd_workspace, size_t fwd_workspace_bytes,
                               float* dQ, float* dK, float* dV, int B, int H, int N, int d,
                               int t, float alpha, int causal, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!fwd_workspace) return EA_ERR_NULL;
    return bwd_impl(Q, K, V, O, dO, tau, block_mask, dQ, dK, dV, B, H, N, d, t, alpha, nullptr, causal, workspace, workspace_bytes,
                    hip_stream, fwd_workspace, fwd_workspace_bytes);
}
int entmax_attn_bwd_alpha_per_head(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                                   const float* tau, const int32_t* block_mask, float* dQ, float* dK, float* dV, int B,
                                   int H, int N, int d, int t, const float* alpha_per_head, int causal,
                                   void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!alpha_per_head) return EA_ERR_NULL;
    return bwd_impl(Q, K, V, O, dO, tau, block_mask, dQ, dK, dV, B, H, N, d, t, 0.f, alpha_per_head, causal, workspace, workspace_bytes, hip_stream);
}

int entmax_attn_fwd_histogram_bounds(const void* workspace, size_t workspace_bytes, int B, int H, int N, int d, int t,
                                     float* tau0, float* upper, void* hip_stream) {
    if (!workspace || !tau0 || !upper) return EA_ERR_NULL;
    const int rc = check_common(B, H, N, d, t, 1.5f);
    if (rc) return rc;
    const Layout L = fwd_layout(B, H, N, d, t);
    if (((uintptr_t)workspace & 255) || workspace_bytes < L.total) return EA_ERR_WORKSPACE;
    const size_t bytes = (size_t)B * H * N * sizeof(float);
    EA_HIP(hipMemcpyAsync(tau0, (const char*)workspace + L.rs_t0, bytes, hipMemcpyDeviceToDevice, (hipStream_t)hip_stream));
    EA_HIP(hipMemcpyAsync(upper, (const char*)workspace + L.rs_up0, bytes, hipMemcpyDeviceToDevice, (hipStream_t)hip_stream));
    return EA_OK;
}

int entmax_attn_right_edge_enable(int on) {
    g_right_edge = on != 0;
    return EA_OK;
}

int entmax_attn_gather_enable(int on) {
    g_gather_enabled = on != 0;
    return EA_OK;
}

int entmax_attn_timer_enable(int on) {
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

int entmax_attn_mfma_probe(const void* data, float* sink, int groups, int iters, void* hip_stream) {
    if (!data || !sink) return EA_ERR_NULL;
    if (groups <= 0 || groups > 4096 || iters <= 0) return EA_ERR_SHAPE;
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(groups), dim3(256), 0, (hipStream_t)hip_stream, (const f16x8*)data, sink, iters);
    EA_HIP(hipGetLastError());
    return EA_OK;
}

int entmax_attn_coissue_probe(float* sink, int iters, int valu_per_round, int with_mfma, void* hip_stream) {
    if (!sink) return EA_ERR_NULL;
    if (iters <= 0) return EA_ERR_SHAPE;
    hipStream_t s = (hipStream_t)hip_stream;
    const dim3 grid(512), block(512);
    const int key = valu_per_round * 2 + (with_mfma ? 1 : 0);
    switch (key) {
        case 1: hipLaunchKernelGGL((coissue_probe_kernel<0, true>), grid, block, 0, s, sink, iters, 1.f); break;
        case 64 * 2: hipLaunchKernelGGL((coissue_probe_kernel<64, false>), grid, block, 0, s, sink, iters, 1.f); break;
        case 64 * 2 + 1: hipLaunchKernelGGL((coissue_probe_kernel<64, true>), grid, block, 0, s, sink, iters, 1.f); break;
        case 128 * 2: hipLaunchKernelGGL((coissue_probe_kernel<128, false>), grid, block, 0, s, sink, iters, 1.f); break;
        case 128 * 2 + 1: hipLaunchKernelGGL((coissue_probe_kernel<128, true>), grid, block, 0, s, sink, iters, 1.f); break;
        case 256 * 2: hipLaunchKernelGGL((coissue_probe_kernel<256, false>), grid, block, 0, s, sink, iters, 1.f); break;
        case 256 * 2 + 1: hipLaunchKernelGGL((coissue_probe_kernel<256, true>), grid, block, 0, s, sink, iters, 1.f); break;
        default: return EA_ERR_SHAPE;
    }
    EA_HIP(hipGetLastError());
    return EA_OK;
}

const char* entmax_attn_strerror(int code) {
    switch (code) {
        case EA_OK: return "ok";
        case EA_ERR_NULL: return "a required pointer is NULL";
        case EA_ERR_ALPHA: return "alpha must be finite and in (1, 3]";
        case EA_ERR_SHAPE: return "bad shape: need B,H > 0, N a positive multiple of 64 (<= 131072), d in {64, 128}";
        case EA_ERR_DTYPE: return "unknown dtype";
        case EA_ERR_WORKSPACE: return "workspace is NULL, not 256-byte aligned, or too small";
        case EA_ERR_HIP: return "a HIP call failed (see entmax_attn_last_hip_error)";
        case EA_ERR_TOO_LARGE: return "the problem needs more scratch than the allocation-free entry point holds (see entmax_attn_decode_static_max_bytes)";
        default: return "unknown error code";
    }
}

}  // extern "C"
