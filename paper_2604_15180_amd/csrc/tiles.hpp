// Tile primitives for gfx950 (CDNA4): 32x32 MFMA fragments, LDS tile layouts, global->LDS
// staging.  Everything here is wave64 code for one 256-thread work-group (4 waves).
//
// Shapes.  A work-group streams 64-row tiles (keys in the forward and in the dQ kernel, queries
// in the dK/dV kernel) through LDS; each wave owns 32*QB rows of the other operand in registers.
//   stage 1:  C[kb][qb] = tile rows (32 kb ..) x owned rows (32 qb ..)        (contraction over d)
//   stage 2:  X[db][qb] += tileT rows (32 db ..) x Y[kb][qb]                   (contraction over the
//             64 tile rows), where tileT is the d x 64 transposed tile and Y is a stage-1 shaped
//             result.  This is O^T += V^T P^T, dQ^T += K^T dS^T, dV^T += dO^T P, dK^T += Q^T dS.
// In the 32x32 accumulator layout lane (n, h) (n = lane % 32, h = lane / 32) holds output column n,
// so every owned row lives in two lanes and row reductions are in-lane plus one 32-lane exchange.
//
// Row permutation.  MFMA output register v of lane half h is output row 8(v/4)+4h+v%4.  Stage 1
// feeds tile row perm(m) into MFMA row m so that register v of half h is tile row
// 16(v/8)+8h+v%8: the eight registers 8s..8s+7 are then exactly the eight consecutive contraction
// slots that lane half h supplies to a K=16 MFMA of stage 2, and the matching tileT operand is one
// 16-byte LDS read.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ea {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int THREADS = 256;
constexpr int NWAVES = 4;
constexpr int TILE = 64;        // rows of a streamed tile = mask granularity
constexpr int PAD_BYTES = 16;   // LDS row padding

#define EA_DEV __device__ __forceinline__

// ---- element traits -------------------------------------------------------------------------
struct Bf16 {
    using elem = __bf16;
    using frag = bf16x8;
    static constexpr int KSTEP = 16;   // contraction elements per MFMA
    static constexpr int EPL = 8;      // elements per lane per operand
    static constexpr bool SCALED = false;
    static EA_DEV f32x16 mma(frag a, frag b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    static EA_DEV elem from_float(float x) { return (__bf16)x; }
};
struct F16 {
    using elem = _Float16;
    using frag = f16x8;
    static constexpr int KSTEP = 16;
    static constexpr int EPL = 8;
    // narrow exponent range: gradient-sized operands are divided by a known bound first
    static constexpr bool SCALED = true;
    static EA_DEV f32x16 mma(frag a, frag b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
    static EA_DEV elem from_float(float x) { return (_Float16)x; }
};
struct F32 {
    using elem = float;
    using frag = float;
    static constexpr int KSTEP = 2;
    static constexpr int EPL = 1;
    static constexpr bool SCALED = false;
    static EA_DEV f32x16 mma(frag a, frag b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
    static EA_DEV elem from_float(float x) { return x; }
};

// tile row held by accumulator register v (0..15) of block kb in lane half h
EA_DEV int trow(int kb, int v, int h) { return 32 * kb + 16 * (v >> 3) + 8 * h + (v & 7); }
// tile row fed to MFMA row m (inverse view of the above)
EA_DEV int perm_row(int m) {
    const int a = m >> 3, hh = (m >> 2) & 1, c = m & 3;
    return 16 * (a >> 1) + 8 * hh + 4 * (a & 1) + c;
}

// ---- LDS layouts ---------------------------------------------------------------------------
template <class E, int D> struct RowTile {      // 64 rows x D elements, row-major, padded
    static constexpr int ROW_BYTES = D * (int)sizeof(typename E::elem);
    static constexpr int LD_BYTES = ROW_BYTES + PAD_BYTES;
    static constexpr int BYTES = TILE * LD_BYTES;
    static constexpr int CHUNKS_PER_ROW = ROW_BYTES / 16;
    static constexpr int NCH = TILE * CHUNKS_PER_ROW / THREADS;   // 16-byte chunks per thread
};
template <class E, int D> struct ColTile {      // D rows x 64 elements (the transposed tile), padded
    static constexpr int ROW_BYTES = TILE * (int)sizeof(typename E::elem);
    static constexpr int LD_BYTES = ROW_BYTES + PAD_BYTES;
    static constexpr int BYTES = D * LD_BYTES;
    static constexpr int CHUNKS_PER_ROW = ROW_BYTES / 16;
    static constexpr int NCH = D * CHUNKS_PER_ROW / THREADS;
};

template <int NCH> struct Staged { u32x4 r[NCH]; };

// global [.., D] row-major rows row0..row0+63 -> registers
template <class E, int D>
EA_DEV void gload_rows(Staged<RowTile<E, D>::NCH>& st, const typename E::elem* g, long row0, int tid) {
    using L = RowTile<E, D>;
    const char* base = (const char*)g + row0 * (long)L::ROW_BYTES;
#pragma unroll
    for (int p = 0; p < L::NCH; ++p) {
        const int c = p * THREADS + tid;
        st.r[p] = *(const u32x4*)(base + (long)c * 16);   // rows are contiguous in memory
    }
}
template <class E, int D>
EA_DEV void sstore_rows(const Staged<RowTile<E, D>::NCH>& st, char* lds, int tid) {
    using L = RowTile<E, D>;
#pragma unroll
    for (int p = 0; p < L::NCH; ++p) {
        const int c = p * THREADS + tid;
        const int row = c / L::CHUNKS_PER_ROW, col = c % L::CHUNKS_PER_ROW;
        *(u32x4*)(lds + row * L::LD_BYTES + col * 16) = st.r[p];
    }
}
// global transposed copy [D][N] (elements of E), columns col0..col0+63 -> registers
template <class E, int D>
EA_DEV void gload_cols(Staged<ColTile<E, D>::NCH>& st, const typename E::elem* gT, long N, long col0, int tid) {
    using L = ColTile<E, D>;
#pragma unroll
    for (int p = 0; p < L::NCH; ++p) {
        const int c = p * THREADS + tid;
        const int row = c / L::CHUNKS_PER_ROW, col = c % L::CHUNKS_PER_ROW;
        st.r[p] = *(const u32x4*)((const char*)(gT + (long)row * N + col0) + col * 16);
    }
}
template <class E, int D>
EA_DEV void sstore_cols(const Staged<ColTile<E, D>::NCH>& st, char* lds, int tid) {
    using L = ColTile<E, D>;
#pragma unroll
    for (int p = 0; p < L::NCH; ++p) {
        const int c = p * THREADS + tid;
        const int row = c / L::CHUNKS_PER_ROW, col = c % L::CHUNKS_PER_ROW;
        *(u32x4*)(lds + row * L::LD_BYTES + col * 16) = st.r[p];
    }
}

// ---- owned operand: rows of a row-major [.., D] matrix held in registers as MFMA B fragments --
template <class E, int D, int QB> struct Owned { typename E::frag f[QB][D / E::KSTEP]; };

template <class E, int D, int QB>
EA_DEV void load_owned(Owned<E, D, QB>& o, const typename E::elem* g, long row0, int lane) {
    const int n = lane & 31, h = lane >> 5;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const typename E::elem* rowp = g + (row0 + 32 * qb + n) * (long)D;
#pragma unroll
        for (int s = 0; s < D / E::KSTEP; ++s)
            o.f[qb][s] = *(const typename E::frag*)(rowp + s * E::KSTEP + h * E::EPL);
    }
}

// ---- stage 1: C[kb][qb] = tile(64 x D, LDS row-major) . owned^T -----------------------------
template <class E, int D, int QB>
EA_DEV void stage1(f32x16 (&C)[2][QB], const char* lds_tile, const Owned<E, D, QB>& own, int lane) {
    using L = RowTile<E, D>;
    const int m = lane & 31, h = lane >> 5;
    const char* r0 = lds_tile + perm_row(m) * L::LD_BYTES + h * E::EPL * (int)sizeof(typename E::elem);
    const char* r1 = r0 + 32 * L::LD_BYTES;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int v = 0; v < 16; ++v) C[kb][qb][v] = 0.f;
#pragma unroll
    for (int s = 0; s < D / E::KSTEP; ++s) {
        const int off = s * E::KSTEP * (int)sizeof(typename E::elem);
        const typename E::frag a0 = *(const typename E::frag*)(r0 + off);
        const typename E::frag a1 = *(const typename E::frag*)(r1 + off);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            C[0][qb] = E::mma(a0, own.f[qb][s], C[0][qb]);
            C[1][qb] = E::mma(a1, own.f[qb][s], C[1][qb]);
        }
    }
}

// ---- stage 2: X[db][qb] += tileT(D x 64, LDS) . Y[kb][qb] -----------------------------------
template <class E2, int D, int QB>
EA_DEV void stage2(f32x16 (&X)[D / 32][QB], const char* lds_tileT, const f32x16 (&Y)[2][QB], int lane) {
    using L = ColTile<E2, D>;
    const int m = lane & 31, h = lane >> 5;
    const char* base = lds_tileT + m * L::LD_BYTES;
    if constexpr (E2::EPL == 8) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                typename E2::frag b[QB];
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                    for (int t = 0; t < 8; ++t) b[qb][t] = E2::from_float(Y[kb][qb][8 * s2 + t]);
                const int coff = (32 * kb + 16 * s2 + 8 * h) * (int)sizeof(typename E2::elem);
#pragma unroll
                for (int db = 0; db < D / 32; ++db) {
                    const typename E2::frag a = *(const typename E2::frag*)(base + db * 32 * L::LD_BYTES + coff);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) X[db][qb] = E2::mma(a, b[qb], X[db][qb]);
                }
            }
    } else {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int coff = trow(kb, v, h) * (int)sizeof(typename E2::elem);
#pragma unroll
                for (int db = 0; db < D / 32; ++db) {
                    const typename E2::frag a = *(const typename E2::frag*)(base + db * 32 * L::LD_BYTES + coff);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) X[db][qb] = E2::mma(a, Y[kb][qb][v], X[db][qb]);
                }
            }
    }
}

// Write X^T accumulators (d x owned rows) to a row-major float [.., D] matrix, scaled.
// Register v of block db in lane (n, h) is element (row0 + 32 qb + n, 32 db + 8(v/4) + 4h + v%4).
template <int D, int QB>
EA_DEV void store_owned_T(float* g, long row0, const f32x16 (&X)[D / 32][QB], const float (&scales)[QB], int lane) {
    const int n = lane & 31, h = lane >> 5;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float scale = scales[qb];
        float* rowp = g + (row0 + 32 * qb + n) * (long)D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                f32x4 o;
#pragma unroll
                for (int c = 0; c < 4; ++c) o[c] = X[db][qb][4 * a + c] * scale;
                *(f32x4*)(rowp + 32 * db + 8 * a + 4 * h) = o;
            }
    }
}

template <int D, int QB>
EA_DEV void store_owned_T(float* g, long row0, const f32x16 (&X)[D / 32][QB], float scale, int lane) {
    float scales[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) scales[qb] = scale;
    store_owned_T<D, QB>(g, row0, X, scales, lane);
}

EA_DEV float wave_max(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}
EA_DEV float xhalf_max(float v) { return fmaxf(v, __shfl_xor(v, 32)); }
EA_DEV float xhalf_sum(float v) { return v + __shfl_xor(v, 32); }

}  // namespace ea
