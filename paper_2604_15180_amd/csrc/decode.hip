// Inference variant on materialised logits (the paper's appendix on language modelling: at
// inference a simplified variant runs on the fully materialised logits z of one query; Sec. 5
// leaves an optimised inference kernel to future work): one query row per head against all N
// cached keys.
//   decode_scores_kernel : z_j = <q, k_j> / sqrt(d) for all keys, written to the workspace, and the
//                          head's maximum logit.  Reads K once: this is the kernel the HBM roofline
//                          prices (N d element bytes per head against 2 N d flops).
//   decode_entmax_kernel : per head, tau from the logits - scores within one unit of the maximum
//                          (Eq. 5) compacted into LDS, histogram (Eq. 6-8) and its root (Eq. 9), then
//                          the safeguarded hybrid refinement (Sec. 3.2) over the compacted scores -
//                          and o = sum_j p_j v_j over the support only (a gather of a few rows of V).
#include <math.h>

#include "fwd_kernels.hpp"
#include "launch.hpp"

namespace ea {

struct DecodeParams {
    const void* q; const void* K; const void* V;
    float* O; float* tau; int32_t* support; int32_t* iters;
    float* logits;            // [BH][N]
    unsigned int* hmax;       // [BH] maximum logit, as unsigned ints that order like the floats
    int BH, N, chunk;         // chunk: keys per work-group of the score kernel
    float inv_sqrt_d, alpha, r, tol;
    int max_iters;
};

EA_DEV unsigned int ordered_bits(float f) {
    const unsigned int u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u ^ 0x80000000u);
}
EA_DEV float from_ordered_bits(unsigned int u) { return __uint_as_float((u & 0x80000000u) ? (u ^ 0x80000000u) : ~u); }

static __global__ void decode_reset_kernel(unsigned int* hmax, int n) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) hmax[i] = 0u;   // below every float
}

// A key row is D elements = LPR lanes x 16 bytes; a wave reads 64 / LPR rows per load, four loads in
// flight; the row's dot product with q is reduced over its LPR lanes.
template <class E, int D>
__global__ __launch_bounds__(256) void decode_scores_kernel(DecodeParams p) {
    using elem = typename E::elem;
    constexpr int EPV = 16 / (int)sizeof(elem), LPR = D / EPV, RPW = 64 / LPR, U = 4;
    typedef elem vec __attribute__((ext_vector_type(EPV)));
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane % LPR, rsel = lane / LPR;
    const int bh = blockIdx.y;
    const long k0 = (long)blockIdx.x * p.chunk, k1 = min((long)p.N, k0 + p.chunk);
    const vec qv = *(const vec*)((const elem*)p.q + (long)bh * D + sub * EPV);
    float qf[EPV];
#pragma unroll
    for (int e = 0; e < EPV; ++e) qf[e] = (float)qv[e];
    const elem* Kh = (const elem*)p.K + (long)bh * p.N * D;
    float* zh = p.logits + (long)bh * p.N;
    float lmax = -INFINITY;
    for (long base = k0 + wave * RPW; base < k1; base += 4 * RPW * U) {
        vec kv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long row = base + (long)u * 4 * RPW + rsel;
#pragma unroll
            for (int e = 0; e < EPV; ++e) kv[u][e] = (elem)0.f;
            if (row < k1) kv[u] = *(const vec*)(Kh + row * D + sub * EPV);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long row = base + (long)u * 4 * RPW + rsel;
            float dot = 0.f;
#pragma unroll
            for (int e = 0; e < EPV; ++e) dot = fmaf(qf[e], (float)kv[u][e], dot);
#pragma unroll
            for (int off = LPR / 2; off >= 1; off >>= 1) dot += __shfl_xor(dot, off);
            const float zval = dot * p.inv_sqrt_d;
            if (row < k1) {
                if (sub == 0) zh[row] = zval;
                lmax = fmaxf(lmax, zval);
            }
        }
    }
    lmax = wave_max(lmax);
    if (lane == 0 && lmax > -INFINITY) atomicMax(&p.hmax[bh], ordered_bits(lmax));
}

template <class E, int D, int AM>
__global__ __launch_bounds__(1024) void decode_entmax_kernel(DecodeParams p) {
    using elem = typename E::elem;
    constexpr int T = 1024, NWV = T / 64, CAP = 4096, NB = 63, SLOTS = NB + 1, CPL = D / 64;
    __shared__ float lx[CAP];               // compacted candidates: (alpha-1) z
    __shared__ int lj[CAP];                 //                       and their key index
    __shared__ uint32_t hist[SLOTS];
    __shared__ int cnt_s;
    __shared__ float red[NWV][4];
    __shared__ float bc[2];
    __shared__ float osum[NWV][D];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int bh = blockIdx.x, N = p.N;
    const float* z = p.logits + (long)bh * N;
    const float c = p.alpha - 1.f, r = p.r;
    constexpr float hb = 1.f / NB;
    const float mx = c * from_ordered_bits(p.hmax[bh]), lower = mx - 1.f;

    if (tid < SLOTS) hist[tid] = 0u;
    if (tid == 0) cnt_s = 0;
    __syncthreads();
    // candidates: scores within one unit of the maximum (Eq. 5), compacted and binned (Eq. 6-8)
    for (int j0 = tid; j0 < N; j0 += 4 * T) {
        float zv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) zv[u] = (j0 + u * T < N) ? z[j0 + u * T] : -INFINITY;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float x = c * zv[u];
            if (x >= lower) {
                const int slot = atomicAdd(&cnt_s, 1);
                if (slot < CAP) { lx[slot] = x; lj[slot] = j0 + u * T; }
                atomicAdd(&hist[min((int)((x - lower) * (float)NB), SLOTS - 1)], 1u);
            }
        }
    }
    __syncthreads();
    const int total = cnt_s;
    const bool over = total > CAP;          // then every evaluation streams the logits instead
    const int nc = min(total, CAP);
    if (tid == 0) {
        const float tau_h = solve_histogram<AM, SLOTS, 32>(hist, 0, 0, hb, r) + lower;
        const float slack = 1e-6f + 2.5e-7f * fabsf(lower);
        bc[0] = fmaxf(tau_h - slack, lower);
        bc[1] = tau_h + hb + slack;
    }
    __syncthreads();
    float thr = bc[0], blo = thr, bhi = bc[1];

    // sums of three per-thread values over the work-group, the same in every thread
    auto block_sum3 = [&](float& a, float& b, float& d3) {
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) { a += __shfl_xor(a, off); b += __shfl_xor(b, off); d3 += __shfl_xor(d3, off); }
        __syncthreads();
        if (lane == 0) { red[wave][0] = a; red[wave][1] = b; red[wave][2] = d3; }
        __syncthreads();
        a = b = d3 = 0.f;
#pragma unroll
        for (int w = 0; w < NWV; ++w) { a += red[w][0]; b += red[w][1]; d3 += red[w][2]; }
    };
    // refinement (Sec. 3.2): f, f', f'' over the candidates, hybrid step, until the step or f is below tol
    int iters = 0;
    for (int it = 0; it < p.max_iters; ++it) {
        float F = 0.f, G = 0.f, Hs = 0.f;
        auto term = [&](float x) {
            const float y = x - thr;
            if (y > 0.f) {
                if constexpr (AM == ALPHA_15) { F = fmaf(y, y, F); G += y; Hs += 1.f; }
                else if constexpr (AM == ALPHA_20) { F += y; G += 1.f; }
                else {
                    const float p2 = pow_r2<AM>(y, r);
                    Hs += p2; G = fmaf(p2, y, G); F = fmaf(p2 * y, y, F);
                }
            }
        };
        if (!over) for (int i = tid; i < nc; i += T) term(lx[i]);
        else for (int j = tid; j < N; j += T) term(c * z[j]);
        block_sum3(F, G, Hs);
        ++iters;
        const float f = F - 1.f;
        if (fabsf(f) <= p.tol) break;
        const float cand = hybrid_step(thr, f, G, Hs, r, p.alpha, blo, bhi);
        const bool small = fabsf(cand - thr) < p.tol;
        thr = cand;
        if (small) break;
    }

    // o = sum over the support of p_j v_j: a wave takes 64 candidates at a time and walks the lanes
    // that hold a non-zero probability; all 64 lanes then read that key's row of V
    float acc[CPL];
#pragma unroll
    for (int k = 0; k < CPL; ++k) acc[k] = 0.f;
    float nsup = 0.f, unused1 = 0.f, unused2 = 0.f;
    const elem* Vh = (const elem*)p.V + (long)bh * N * D;
    const int nsrc = over ? N : nc;
    for (int base = wave * 64; base < nsrc; base += NWV * 64) {
        const int i = base + lane;
        float x = -INFINITY;
        int j = 0;
        if (i < nsrc) { x = over ? c * z[i] : lx[i]; j = over ? i : lj[i]; }
        const float y = x - thr;
        const float pj = y > 0.f ? pow_r<AM>(y, r) : 0.f;
        unsigned long long todo = __ballot(pj > 0.f);
        nsup += (float)__popcll(todo) * (lane == 0 ? 1.f : 0.f);
        while (todo) {
            const int src = __ffsll((long long)todo) - 1;
            todo &= todo - 1;
            const float pv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pj), src));
            const int jv = __builtin_amdgcn_readlane(j, src);
            const elem* vrow = Vh + (long)jv * D + lane * CPL;
#pragma unroll
            for (int k = 0; k < CPL; ++k) acc[k] = fmaf(pv, (float)vrow[k], acc[k]);
        }
    }
#pragma unroll
    for (int k = 0; k < CPL; ++k) osum[wave][lane * CPL + k] = acc[k];
    block_sum3(nsup, unused1, unused2);       // (its barriers also publish osum)
    if (tid < D) {
        float o = 0.f;
#pragma unroll
        for (int w = 0; w < NWV; ++w) o += osum[w][tid];
        p.O[(long)bh * D + tid] = o;
    }
    if (tid == 0) {
        p.tau[bh] = thr;
        if (p.support) p.support[bh] = (int32_t)(nsup + 0.5f);
        if (p.iters) p.iters[bh] = iters;
    }
}

template <class E, int D>
int decode_run(const DecodeParams& p, hipStream_t s) {
    timer_begin();
    hipLaunchKernelGGL(decode_reset_kernel, dim3(1), dim3(256), 0, s, p.hmax, p.BH);
    {
        ScopedKernelTime t(EA_TIMER_DECODE_SCORES, s);
        hipLaunchKernelGGL((decode_scores_kernel<E, D>), dim3((p.N + p.chunk - 1) / p.chunk, p.BH), dim3(256), 0, s, p);
    }
    switch (p.alpha == 1.5f ? ALPHA_15 : p.alpha == 2.0f ? ALPHA_20 : ALPHA_GEN) {
        case ALPHA_15: hipLaunchKernelGGL((decode_entmax_kernel<E, D, ALPHA_15>), dim3(p.BH), dim3(1024), 0, s, p); break;
        case ALPHA_20: hipLaunchKernelGGL((decode_entmax_kernel<E, D, ALPHA_20>), dim3(p.BH), dim3(1024), 0, s, p); break;
        default: hipLaunchKernelGGL((decode_entmax_kernel<E, D, ALPHA_GEN>), dim3(p.BH), dim3(1024), 0, s, p); break;
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_last_hip_error((int)e); return EA_ERR_HIP; }
    return EA_OK;
}

}  // namespace ea

namespace {
inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
bool decode_shape_ok(int B, int H, int N, int d, ea_dtype t) {
    return (t == EA_F32 || t == EA_BF16) && B > 0 && H > 0 && (long)B * H <= 65535 && N > 0 && N <= (1 << 22) && (d == 64 || d == 128);
}
}  // namespace

extern "C" {

size_t entmax_attn_decode_workspace_bytes(int B, int H, int N, int d, ea_dtype t) {
    if (!decode_shape_ok(B, H, N, d, t)) return 0;
    return align256((size_t)B * H * 4) + align256((size_t)B * H * N * 4);
}

int entmax_attn_decode(const void* q, const void* K, const void* V, float* O, float* tau, int32_t* support,
                       int32_t* iters, int B, int H, int N, int d, ea_dtype t, float alpha,
                       void* workspace, size_t workspace_bytes, void* hip_stream) {
    using namespace ea;
    if (!q || !K || !V || !O || !tau) return EA_ERR_NULL;
    if (t != EA_F32 && t != EA_BF16) return EA_ERR_DTYPE;
    if (!decode_shape_ok(B, H, N, d, t)) return EA_ERR_SHAPE;
    if (!isfinite(alpha) || !(alpha > 1.f) || alpha > 2.f) return EA_ERR_ALPHA;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < entmax_attn_decode_workspace_bytes(B, H, N, d, t))
        return EA_ERR_WORKSPACE;
    DecodeParams p{};
    p.q = q; p.K = K; p.V = V; p.O = O; p.tau = tau; p.support = support; p.iters = iters;
    p.hmax = (unsigned int*)workspace;
    p.logits = (float*)((char*)workspace + align256((size_t)B * H * 4));
    p.BH = B * H; p.N = N;
    // about four work-groups of the score kernel per CU, each a multiple of 256 keys
    const int want = (1024 + p.BH - 1) / p.BH;
    int chunk = (N + want - 1) / want;
    chunk = ((chunk + 255) / 256) * 256;
    p.chunk = chunk < 256 ? 256 : chunk;
    p.inv_sqrt_d = 1.f / sqrtf((float)d);
    p.alpha = alpha; p.r = 1.f / (alpha - 1.f);
    p.tol = (t == EA_BF16) ? 1e-4f : 1e-6f;
    p.max_iters = 16;
    hipStream_t s = (hipStream_t)hip_stream;
    if (t == EA_BF16) return d == 64 ? decode_run<Bf16, 64>(p, s) : decode_run<Bf16, 128>(p, s);
    return d == 64 ? decode_run<F32, 64>(p, s) : decode_run<F32, 128>(p, s);
}

}  // extern "C"
