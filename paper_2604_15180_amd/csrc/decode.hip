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

#include <type_traits>

#include "fwd_kernels.hpp"
#include "launch.hpp"

namespace ea {

struct DecodeParams {
    const void* q; const void* K; const void* V;
    float* O; float* tau; int32_t* support; int32_t* iters;
    float* logits;            // [BH][Npad], Npad = N rounded up to 4: every head's logits start 16-byte aligned
    float* gmax;              // [BH][ngrp] maximum logit of each work-group of the score kernel
    int BH, N, Npad, chunk, ngrp;   // chunk: keys per work-group of the score kernel; ngrp of them per head
    float inv_sqrt_d, alpha, r, tol;
    int max_iters;
};

// Sum of v over each aligned group of G lanes (G = 8, 16 or 32), left in all of the group's lanes.
// Within a row of 16 lanes the exchanges are data-parallel-primitive modifiers of the add itself
// (quad permutes, then mirrors: once every lane of a half holds its half's sum, the mirrored lane
// holds the other half's), so a key row's dot product costs four ALU operations and no LDS traffic.
template <int CTRL> EA_DEV float dpp_add(float v) {
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
template <int G> EA_DEV float group_sum(float v) {
    v = dpp_add<0xB1>(v);                       // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);                       // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);                      // row_half_mirror
    if constexpr (G >= 16) v = dpp_add<0x140>(v);   // row_mirror
    if constexpr (G >= 32) v += __shfl_xor(v, 16);
    return v;
}

// A key row is D elements = LPR lanes x 16 bytes; a wave reads RPW = 64 / LPR rows per load and a
// work-group 4 RPW.  U loads per lane form a batch; the next batch is requested before the current
// one is reduced, so a wave always has loads in flight.  K is read once and never again: the loads
// are non-temporal, which keeps the stream out of the way of the cached lines.
template <class E, int D>
__global__ __launch_bounds__(256) void decode_scores_kernel(DecodeParams p) {
    using elem = typename E::elem;
    constexpr int EPV = 16 / (int)sizeof(elem), LPR = D / EPV, RPW = 64 / LPR, U = 4, RPB = 4 * RPW * U;
    typedef elem vec __attribute__((ext_vector_type(EPV)));
    static_assert(LPR == 8 || LPR == 16 || LPR == 32, "a key row spans 8, 16 or 32 lanes");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane % LPR, rsel = lane / LPR;
    const int bh = blockIdx.y;
    const long k0 = (long)blockIdx.x * p.chunk, k1 = min((long)p.N, k0 + p.chunk);
    const vec qv = *(const vec*)((const elem*)p.q + (long)bh * D + sub * EPV);
    float qf[EPV];
#pragma unroll
    for (int e = 0; e < EPV; ++e) qf[e] = (float)qv[e];
    const elem* Kh = (const elem*)p.K + (long)bh * p.N * D;
    float* zh = p.logits + (long)bh * p.Npad;
    __shared__ float wmax[4];
    float lmax = -INFINITY;
    const long nfull = (k1 - k0) / RPB;                     // batches with every row inside the chunk
    const long row_w = k0 + wave * RPW + rsel;              // this lane's row in batch 0, load 0
    auto load = [&](vec (&kv)[U], long it) {
        const elem* src = Kh + (row_w + it * RPB) * D + sub * EPV;
#pragma unroll
        for (int u = 0; u < U; ++u) kv[u] = __builtin_nontemporal_load((const vec*)(src + (long)u * 4 * RPW * D));
    };
    auto reduce = [&](auto guarded, const vec (&kv)[U], long it) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long row = row_w + it * RPB + (long)u * 4 * RPW;
            float dot = 0.f;
#pragma unroll
            for (int e = 0; e < EPV; ++e) dot = fmaf(qf[e], (float)kv[u][e], dot);
            const float zval = group_sum<LPR>(dot) * p.inv_sqrt_d;
            if (!decltype(guarded)::value || row < k1) {
                if (sub == 0) zh[row] = zval;
                lmax = fmaxf(lmax, zval);
            }
        }
    };
    if (nfull > 0) {
        vec ka[U], kb[U];
        load(ka, 0);
        for (long it = 0; it < nfull; it += 2) {
            if (it + 1 < nfull) load(kb, it + 1);
            reduce(std::false_type{}, ka, it);
            if (it + 1 < nfull) {
                if (it + 2 < nfull) load(ka, it + 2);
                reduce(std::false_type{}, kb, it + 1);
            }
        }
    }
    if (k0 + nfull * RPB < k1) {                            // ragged tail: one guarded batch
        vec kt[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long row = row_w + nfull * RPB + (long)u * 4 * RPW;
#pragma unroll
            for (int e = 0; e < EPV; ++e) kt[u][e] = (elem)0.f;
            if (row < k1) kt[u] = *(const vec*)(Kh + row * D + sub * EPV);
        }
        reduce(std::true_type{}, kt, nfull);
    }
    // one maximum per work-group, each in a slot of its own: thousands of atomic maxima on one
    // cache line would queue up behind each other for longer than a short cache takes to read
    lmax = wave_max(lmax);
    if (lane == 0) wmax[wave] = lmax;
    __syncthreads();
    if (tid == 0) p.gmax[(long)bh * p.ngrp + blockIdx.x] = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
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
    const float* z = p.logits + (long)bh * p.Npad;
    const float c = p.alpha - 1.f, r = p.r;
    constexpr float hb = 1.f / NB;

    if (tid < SLOTS) hist[tid] = 0u;
    if (tid == 0) cnt_s = 0;
    float gm = -INFINITY;
    for (int i = tid; i < p.ngrp; i += T) gm = fmaxf(gm, p.gmax[(long)bh * p.ngrp + i]);
    gm = wave_max(gm);
    if (lane == 0) red[wave][0] = gm;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NWV; ++w) gm = fmaxf(gm, red[w][0]);
    const float mx = c * gm, lower = mx - 1.f;
    // candidates: scores within one unit of the maximum (Eq. 5), compacted and binned (Eq. 6-8);
    // four 16-byte loads per thread in flight (the padding of the last four reads as is: tested below)
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    for (int j0 = 4 * tid; j0 < N; j0 += 16 * T) {
        f32x4 zv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            zv[u] = f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
            if (j0 + u * 4 * T < N) zv[u] = *(const f32x4*)(z + j0 + u * 4 * T);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int j = j0 + u * 4 * T + e;
                const float x = c * zv[u][e];
                if (j < N && x >= lower) {
                    const int slot = atomicAdd(&cnt_s, 1);
                    if (slot < CAP) { lx[slot] = x; lj[slot] = j; }
                    atomicAdd(&hist[min((int)((x - lower) * (float)NB), SLOTS - 1)], 1u);
                }
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
    {
        ScopedKernelTime t(EA_TIMER_DECODE_SCORES, s);
        hipLaunchKernelGGL((decode_scores_kernel<E, D>), dim3(p.ngrp, p.BH), dim3(256), 0, s, p);
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
// Keys per work-group of the score kernel: about four work-groups per CU over all heads, each a
// multiple of 256 keys.
int decode_chunk(int BH, int N) {
    const int want = (1024 + BH - 1) / BH;
    int chunk = (N + want - 1) / want;
    chunk = ((chunk + 255) / 256) * 256;
    return chunk < 256 ? 256 : chunk;
}
int decode_groups(int BH, int N) { const int ch = decode_chunk(BH, N); return (N + ch - 1) / ch; }
size_t decode_npad(int N) { return ((size_t)N + 3) & ~(size_t)3; }
bool decode_shape_ok(int B, int H, int N, int d, ea_dtype t) {
    return (t == EA_F32 || t == EA_BF16) && B > 0 && H > 0 && (long)B * H <= 65535 && N > 0 && N <= (1 << 22) && (d == 64 || d == 128);
}
}  // namespace

extern "C" {

size_t entmax_attn_decode_workspace_bytes(int B, int H, int N, int d, ea_dtype t) {
    if (!decode_shape_ok(B, H, N, d, t)) return 0;
    return align256((size_t)B * H * decode_groups(B * H, N) * 4) + align256((size_t)B * H * decode_npad(N) * 4);
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
    p.BH = B * H; p.N = N; p.Npad = (int)decode_npad(N);
    p.chunk = decode_chunk(p.BH, N);
    p.ngrp = decode_groups(p.BH, N);
    p.gmax = (float*)workspace;
    p.logits = (float*)((char*)workspace + align256((size_t)p.BH * p.ngrp * 4));
    p.inv_sqrt_d = 1.f / sqrtf((float)d);
    p.alpha = alpha; p.r = 1.f / (alpha - 1.f);
    p.tol = (t == EA_BF16) ? 1e-4f : 1e-6f;
    p.max_iters = 16;
    hipStream_t s = (hipStream_t)hip_stream;
    if (t == EA_BF16) return d == 64 ? decode_run<Bf16, 64>(p, s) : decode_run<Bf16, 128>(p, s);
    return d == 64 ? decode_run<F32, 64>(p, s) : decode_run<F32, 128>(p, s);
}

}  // extern "C"
