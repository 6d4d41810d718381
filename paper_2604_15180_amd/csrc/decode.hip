// Inference variant on materialised logits (the paper's appendix on language modelling: at
// inference a simplified variant runs on the fully materialised logits z of one query; Sec. 5
// leaves an optimised inference kernel to future work): one query row per head against all N
// cached keys.
//   decode_scores_kernel : z_j = <q, k_j> / sqrt(d) for all keys.  Reads K once: this is the kernel
//                          the HBM roofline prices (N d element bytes per head against 2 N d flops).
//                          By Eq. 5 only logits within 1 / (alpha - 1) of the head's maximum can be
//                          in the support, and a running maximum is a lower bound of the final one,
//                          so a work-group keeps just the logits within that window of the largest
//                          it has met so far (a few per cent of them) and its own maximum: the other
//                          logits are never written.
//   decode_entmax_kernel : per head, tau from the kept logits - those within one unit of the true
//                          maximum compacted into LDS, histogram (Eq. 6-8) and its root (Eq. 9), then
//                          the safeguarded hybrid refinement (Sec. 3.2) over the compacted scores -
//                          and o = sum_j p_j v_j over the support only (a gather of a few rows of V).
#include <math.h>

#include <mutex>
#include <type_traits>

#include "fwd_kernels.hpp"
#include "launch.hpp"

namespace ea {

struct DecodeParams {
    const void* q; const void* K; const void* V;
    float* O; float* tau; int32_t* support; int32_t* iters;
    uint2* cand;              // [BH][ngrp][chunk] kept logits: (bits of z_j, j)
    int* ccnt;                // [BH][ngrp] how many each work-group of the score kernel kept
    float* gmax;              // [BH][ngrp] maximum logit of each work-group
    int BH, N, chunk, ngrp;   // chunk: keys per work-group of the score kernel; ngrp of them per head
    float inv_sqrt_d, alpha, r, tol;
    float zwin;               // 1 / (alpha - 1), slightly widened: the window of Eq. 5 in units of z
    int max_iters;
};

// unsigned integers that order like the floats they come from (for an integer atomic maximum)
EA_DEV unsigned int ordered_bits(float f) {
    const unsigned int u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u ^ 0x80000000u);
}
EA_DEV float from_ordered_bits(unsigned int u) { return __uint_as_float((u & 0x80000000u) ? (u ^ 0x80000000u) : ~u); }

// A key row is D elements = LPR lanes x 16 bytes; a wave reads RPW = 64 / LPR rows per load and a
// work-group 4 RPW.  U loads per lane form a batch; the next batch is requested before the current
// one is reduced, so a wave always has loads in flight.  K is read once and never again: the loads
// are non-temporal, which keeps the stream out of the way of the cached lines.
// A logit is kept when it is within the window of the largest logit known so far: the largest this
// lane has computed, or the one the work-group's waves share through an LDS word.
template <class E, int D>
__global__ __launch_bounds__(256) void decode_scores_kernel(DecodeParams p) {
    using elem = typename E::elem;
    constexpr int EPV = 16 / (int)sizeof(elem), LPR = D / EPV, RPW = 64 / LPR, U = 4, RPB = 4 * RPW * U;
    typedef elem vec __attribute__((ext_vector_type(EPV)));
    static_assert(LPR == 8 || LPR == 16 || LPR == 32, "a key row spans 8, 16 or 32 lanes");
    __shared__ float wmax[4];
    __shared__ unsigned int smax;                           // ordered bits of the shared running maximum
    __shared__ int lcnt;                                    // logits kept so far
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane % LPR, rsel = lane / LPR;
    const int bh = blockIdx.y;
    const long k0 = (long)blockIdx.x * p.chunk, k1 = min((long)p.N, k0 + p.chunk);
    const vec qv = *(const vec*)((const elem*)p.q + (long)bh * D + sub * EPV);
    float qf[EPV];
#pragma unroll
    for (int e = 0; e < EPV; ++e) qf[e] = (float)qv[e];
    const elem* Kh = (const elem*)p.K + (long)bh * p.N * D;
    uint2* const kept = p.cand + ((size_t)bh * p.ngrp + blockIdx.x) * (size_t)p.chunk;
    if (tid == 0) { smax = ordered_bits(-INFINITY); lcnt = 0; }
    __syncthreads();
    float lmax = -INFINITY;
    const long nfull = (k1 - k0) / RPB;                     // batches with every row inside the chunk
    const long row_w = k0 + wave * RPW + rsel;              // this lane's row in batch 0, load 0
    auto load = [&](vec (&kv)[U], long it) {
        const elem* src = Kh + (row_w + it * RPB) * D + sub * EPV;
#pragma unroll
        for (int u = 0; u < U; ++u) kv[u] = __builtin_nontemporal_load((const vec*)(src + (long)u * 4 * RPW * D));
    };
    auto reduce = [&](auto guarded, const vec (&kv)[U], long it) {
        float zval[U];
        float bmax = -INFINITY;
        const long row0 = row_w + it * RPB;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float dot = 0.f;
#pragma unroll
            for (int e = 0; e < EPV; ++e) dot = fmaf(qf[e], (float)kv[u][e], dot);
            zval[u] = group_sum<LPR>(dot) * p.inv_sqrt_d;
            if (decltype(guarded)::value && row0 + (long)u * 4 * RPW >= k1) zval[u] = -INFINITY;
            bmax = fmaxf(bmax, zval[u]);
        }
        lmax = fmaxf(lmax, bmax);
        const float shared_max = from_ordered_bits(*(volatile unsigned int*)&smax);
        const float m = fmaxf(lmax, shared_max);
        // rounding in the comparison made later, (alpha - 1) z >= (alpha - 1) max - 1, is far
        // inside the extra width
        const float keep = m - p.zwin - 1e-6f * fabsf(m);
        if (sub == 0 && bmax >= keep) {                     // -inf (a row past the end) never is
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (zval[u] >= keep) {
                    const int slot = atomicAdd(&lcnt, 1);
                    kept[slot] = make_uint2(__float_as_uint(zval[u]), (unsigned int)(row0 + (long)u * 4 * RPW));
                }
            }
            if (bmax > shared_max) atomicMax(&smax, ordered_bits(bmax));
        }
    };
    if (nfull > 0) {
        vec ka[U], kb[U];
        load(ka, 0);
        long it = 0;
        for (; it + 2 < nfull; it += 2) {
            load(kb, it + 1);
            reduce(std::false_type{}, ka, it);
            load(ka, it + 2);
            reduce(std::false_type{}, kb, it + 1);
        }
        if (it + 1 < nfull) {                               // two batches left, the first one loaded
            load(kb, it + 1);
            reduce(std::false_type{}, ka, it);
            reduce(std::false_type{}, kb, it + 1);
        } else {
            reduce(std::false_type{}, ka, it);
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
    if (tid == 0) {
        p.gmax[(long)bh * p.ngrp + blockIdx.x] = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
        p.ccnt[(long)bh * p.ngrp + blockIdx.x] = lcnt;
    }
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
    __shared__ int pref[T + 1];             // kept logits of the score kernel's work-groups before group g
    __shared__ int wsum[NWV];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int bh = blockIdx.x, N = p.N, ngrp = p.ngrp;
    const uint2* kept = p.cand + (size_t)bh * ngrp * (size_t)p.chunk;
    const float c = p.alpha - 1.f, r = p.r;
    constexpr float hb = 1.f / NB;

    if (tid < SLOTS) hist[tid] = 0u;
    if (tid == 0) cnt_s = 0;
    // the head's maximum, and the running count of kept logits over the score kernel's work-groups
    // (at most T of them): entry i of the head's kept logits is entry i - pref[g] of group g
    float gm = tid < ngrp ? p.gmax[(long)bh * ngrp + tid] : -INFINITY;
    int incl = tid < ngrp ? p.ccnt[(long)bh * ngrp + tid] : 0;
    gm = wave_max(gm);
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
    }
    if (lane == 0) red[wave][0] = gm;
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    int before = 0;
#pragma unroll
    for (int w = 0; w < NWV; ++w) {
        gm = fmaxf(gm, red[w][0]);
        before += w < wave ? wsum[w] : 0;
    }
    pref[tid + 1] = before + incl;
    if (tid == 0) pref[0] = 0;
    __syncthreads();
    const int M = pref[ngrp];
    const float mx = c * gm, lower = mx - 1.f;
    auto kept_at = [&](int i) {             // i < M
        int lo = 0, hi = ngrp;              // pref[lo] <= i < pref[hi]
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (pref[mid] <= i) lo = mid; else hi = mid;
        }
        return kept[(size_t)lo * p.chunk + (i - pref[lo])];
    };
    // candidates: scores within one unit of the maximum (Eq. 5), compacted and binned (Eq. 6-8);
    // four loads per thread in flight
    for (int i0 = tid; i0 < M; i0 += 4 * T) {
        uint2 e[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            e[u] = make_uint2(__float_as_uint(-INFINITY), 0u);
            if (i0 + u * T < M) e[u] = kept_at(i0 + u * T);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float x = c * __uint_as_float(e[u].x);
            if (x >= lower) {
                const int slot = atomicAdd(&cnt_s, 1);
                if (slot < CAP) { lx[slot] = x; lj[slot] = (int)e[u].y; }
                atomicAdd(&hist[min((int)((x - lower) * (float)NB), SLOTS - 1)], 1u);
            }
        }
    }
    __syncthreads();
    const int total = cnt_s;
    const bool over = total > CAP;          // then every evaluation streams the kept logits instead
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
    SecantPrev prev;
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
        else for (int i = tid; i < M; i += T) term(c * __uint_as_float(kept_at(i).x));
        block_sum3(F, G, Hs);
        ++iters;
        const float f = F - 1.f;
        if (fabsf(f) <= p.tol) break;
        const float stol = step_tol(p.tol, thr);
        const float cand = hybrid_step<AM>(thr, f, G, Hs, r, p.alpha, blo, bhi, prev, stol);
        const bool small = fabsf(cand - thr) < stol;
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
    const int nsrc = over ? M : nc;
    for (int base = wave * 64; base < nsrc; base += NWV * 64) {
        const int i = base + lane;
        float x = -INFINITY;
        int j = 0;
        if (i < nsrc) {
            if (over) { const uint2 e = kept_at(i); x = c * __uint_as_float(e.x); j = (int)e.y; }
            else { x = lx[i]; j = lj[i]; }
        }
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
size_t decode_groups_bytes(int BH, int N) { return align256((size_t)BH * decode_groups(BH, N) * 4); }
bool decode_shape_ok(int B, int H, int N, int d, int t) {
    return (t == EA_F32 || t == EA_BF16) && B > 0 && H > 0 && (long)B * H <= 65535 && N > 0 && N <= (1 << 22) && (d == 64 || d == 128);
}

// Scratch of the allocation-free entry point: one array per GPU, in the library's code object, held
// until the process ends.  Host code never uses the array's name as an address: the address on a
// device is asked for once, with that device current, and kept.
constexpr size_t DECODE_SCRATCH_BYTES = (size_t)33 << 20;     // 33 MiB: 4 Mi kept-logit slots of 8 bytes + the per-group words
static __device__ __align__(256) unsigned char scratch[DECODE_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};

int decode_scratch_of_current_device(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { ea::set_last_hip_error((int)e); return EA_ERR_HIP; }
    if (dev < 0 || dev >= MAX_DEVICES) return EA_ERR_SHAPE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) { ea::set_last_hip_error((int)e); return EA_ERR_HIP; }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return EA_OK;
}

int decode_check(const void* q, const void* K, const void* V, const float* O, const float* tau, int B, int H, int N, int d,
                 int t, float alpha) {
    if (!q || !K || !V || !O || !tau) return EA_ERR_NULL;
    if (t != EA_F32 && t != EA_BF16) return EA_ERR_DTYPE;
    if (!decode_shape_ok(B, H, N, d, t)) return EA_ERR_SHAPE;
    if (!isfinite(alpha) || !(alpha > 1.f) || alpha > EA_ALPHA_MAX) return EA_ERR_ALPHA;
    if (decode_groups(B * H, N) > 1024) return EA_ERR_SHAPE;      // decode_entmax_kernel indexes the groups by thread
    return EA_OK;
}

// `workspace`: device memory of at least entmax_attn_decode_workspace_bytes(...) bytes, 256-byte aligned
int decode_enqueue(const void* q, const void* K, const void* V, float* O, float* tau, int32_t* support, int32_t* iters,
                   int B, int H, int N, int d, int t, float alpha, void* workspace, void* hip_stream) {
    using namespace ea;
    DecodeParams p{};
    p.q = q; p.K = K; p.V = V; p.O = O; p.tau = tau; p.support = support; p.iters = iters;
    p.BH = B * H; p.N = N;
    p.chunk = decode_chunk(p.BH, N);
    p.ngrp = decode_groups(p.BH, N);
    p.gmax = (float*)workspace;
    p.ccnt = (int*)((char*)workspace + decode_groups_bytes(p.BH, N));
    p.cand = (uint2*)((char*)workspace + 2 * decode_groups_bytes(p.BH, N));
    p.inv_sqrt_d = 1.f / sqrtf((float)d);
    p.alpha = alpha; p.r = 1.f / (alpha - 1.f);
    p.tol = (t == EA_BF16) ? 1e-4f : 1e-6f;
    p.zwin = p.r * (1.f + 1e-5f);
    p.max_iters = alpha > 2.f ? 32 : 16;      // (alpha > 2: a logit within the tolerance of the root makes the solver bisect)
    hipStream_t s = (hipStream_t)hip_stream;
    if (t == EA_BF16) return d == 64 ? decode_run<Bf16, 64>(p, s) : decode_run<Bf16, 128>(p, s);
    return d == 64 ? decode_run<F32, 64>(p, s) : decode_run<F32, 128>(p, s);
}
}  // namespace

extern "C" {

size_t entmax_attn_decode_workspace_bytes(int B, int H, int N, int d, int t) {
    if (!decode_shape_ok(B, H, N, d, t)) return 0;
    const int BH = B * H;
    return 2 * decode_groups_bytes(BH, N) + align256((size_t)BH * decode_groups(BH, N) * (size_t)decode_chunk(BH, N) * 8);
}

int entmax_attn_decode(const void* q, const void* K, const void* V, float* O, float* tau, int32_t* support,
                       int32_t* iters, int B, int H, int N, int d, int t, float alpha,
                       void* workspace, size_t workspace_bytes, void* hip_stream) {
    const int rc = decode_check(q, K, V, O, tau, B, H, N, d, t, alpha);
    if (rc) return rc;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < entmax_attn_decode_workspace_bytes(B, H, N, d, t))
        return EA_ERR_WORKSPACE;
    return decode_enqueue(q, K, V, O, tau, support, iters, B, H, N, d, t, alpha, workspace, hip_stream);
}

size_t entmax_attn_decode_static_max_bytes(void) { return DECODE_SCRATCH_BYTES; }

int entmax_attn_decode_static(const void* q, const void* K, const void* V, float* O, float* tau, int32_t* support,
                              int32_t* iters, int B, int H, int N, int d, int t, float alpha, void* hip_stream) {
    const int rc = decode_check(q, K, V, O, tau, B, H, N, d, t, alpha);
    if (rc) return rc;
    if (entmax_attn_decode_workspace_bytes(B, H, N, d, t) > DECODE_SCRATCH_BYTES) return EA_ERR_TOO_LARGE;
    void* ws = nullptr;
    const int rs = decode_scratch_of_current_device(&ws);
    if (rs) return rs;
    // the kernels write every word of the scratch they later read (per-group maxima, counts and
    // kept logits): nothing has to start at zero, so what the previous call left needs no clearing
    return decode_enqueue(q, K, V, O, tau, support, iters, B, H, N, d, t, alpha, ws, hip_stream);
}

}  // extern "C"
