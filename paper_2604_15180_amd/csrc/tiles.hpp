// Tile primitives for gfx950 (CDNA4): 32x32 MFMA fragments, swizzled LDS tile layouts, direct
// global->LDS loads.  Everything here is wave64 code for a work-group of NW waves.
//
// Shapes.  A work-group streams 64-row tiles (keys in the forward and in the dQ kernel, queries
// in the dK/dV kernel) through LDS; each wave owns 32*QB rows of the other operand in registers.
//   stage 1:  C[kb][qb] = tile rows (32 kb ..) x owned rows (32 qb ..)        (contraction over d)
//   stage 2:  X[db][qb] += tile^T rows (32 db ..) x Y[kb][qb]                  (contraction over the
//             64 tile rows), where Y is a stage-1 shaped result.  This is O^T += V^T P^T,
//             dQ^T += K^T dS^T, dV^T += dO^T P, dK^T += Q^T dS.  The tile stays row-major in LDS;
//             its transposed MFMA fragments come from the LDS transpose read ds_read_b64_tr_b16.
// In the 32x32 accumulator layout lane (n, h) (n = lane % 32, h = lane / 32) holds output column n,
// so every owned row lives in two lanes and row reductions are in-lane plus one 32-lane exchange.
//
// Row permutation.  MFMA output register v of lane half h is output row 8(v/4)+4h+v%4.  Stage 1
// feeds tile row perm(m) into MFMA row m so that register v of half h is tile row
// 16(v/8)+8h+v%8: the eight registers 8s..8s+7 are then exactly the eight consecutive contraction
// slots that lane half h supplies to a K=16 MFMA of stage 2.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ea {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int TILE = 64;        // rows of a streamed tile = mask granularity

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
    template <bool FRESH_B = true> static EA_DEV void mma_acc(frag a, frag b, f32x16& c) { c = mma(a, b, c); }
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
    // c += a b with the accumulator pinned to the accumulation registers (AGPRs).  The long-lived
    // stage-2 accumulators are touched by nothing but these MFMAs until the kernel's epilogue;
    // pinned there they cost no vector registers and no copies, which leaves the 256 ordinary
    // registers to the operands the vector ALUs work on.  The compiler does not know that this
    // statement is an MFMA, so what it would otherwise schedule around one is spelled out: two
    // idle cycles ahead of it when its B operand may have been written by the vector ALU just
    // before (FRESH_B), and settle_acc() before anything else reads the accumulator.
    template <bool FRESH_B = true>
    static EA_DEV void mma_acc(frag a, frag b, f32x16& c) {
        if constexpr (FRESH_B) asm("s_nop 1\n\tv_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
        else asm("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
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
    template <bool FRESH_B = true> static EA_DEV void mma_acc(frag a, frag b, f32x16& c) { c = mma(a, b, c); }
    static EA_DEV elem from_float(float x) { return x; }
};

// After the last mma_acc on `c` and before its first other use: outlasts the MFMA pipeline.
EA_DEV void settle_acc(f32x16& c) { asm volatile("s_nop 15\n\ts_nop 7" : "+a"(c)); }

// tile row held by accumulator register v (0..15) of block kb in lane half h
EA_DEV int trow(int kb, int v, int h) { return 32 * kb + 16 * (v >> 3) + 8 * h + (v & 7); }
// tile row fed to MFMA row m (inverse view of the above)
EA_DEV int perm_row(int m) {
    const int a = m >> 3, hh = (m >> 2) & 1, c = m & 3;
    return 16 * (a >> 1) + 8 * hh + 4 * (a & 1) + c;
}

// ---- LDS layouts ---------------------------------------------------------------------------
// Tiles are filled by direct global->LDS loads (global_load_lds_dwordx4): one wave instruction
// writes 64 consecutive 16-byte chunks, so rows cannot be padded.  Bank conflicts are avoided by
// an XOR swizzle instead: chunk c of row r lives at chunk position c ^ swz(r) of that row, where
// swz makes the 16 rows that one ds_read_b128 phase touches land in 16 distinct bank groups.
// The loading lane simply fetches the global chunk that belongs at its LDS position.
template <int CPR> EA_DEV int swz(int row) {   // CPR = 16-byte chunks per row (8, 16 or 32)
    // Two access patterns must both be conflict-free:
    //  (1) stage 1, ds_read_b128: 16 lanes read the same chunk of 16 different rows of a 16-row block;
    //  (2) stage 2, ds_read_b64_tr_b16: 32 lanes read a patch of 4 consecutive rows x 4 chunks.
    // A bit rotation of the row index does both: consecutive rows move by 4 chunks (pattern 2),
    // and the map is still one-to-one over 16 rows (pattern 1).
    if constexpr (CPR == 8) {                  // two rows per 256-byte bank sweep: use row / 2
        const int x = (row >> 1) & 7;
        return ((x & 1) << 2) | (x >> 1);
    } else if constexpr (CPR == 16) {
        return ((row & 3) << 2) | ((row >> 2) & 3);
    } else {
        return row & 15;
    }
}
template <class E, int D> struct RowTile {      // 64 rows x D elements, row-major
    static constexpr int ROW_BYTES = D * (int)sizeof(typename E::elem);
    static constexpr int BYTES = TILE * ROW_BYTES;
    static constexpr int CPR = ROW_BYTES / 16;
    static constexpr int NINST = BYTES / 1024;   // wave-wide load instructions per tile
};

// Direct global->LDS loads, written as instructions of their own: LDS address = M0 (wave-uniform
// base) + lane * 16 (or * 4), global address = scalar base + 32-bit lane offset.  As a compiler
// builtin the load is a "flat access that may touch LDS", and while one is in flight the compiler
// turns every wait into a wait for ALL outstanding LDS reads (and loads) - with a tile always
// being prefetched, no MFMA could start before the last of its sixteen fragments had arrived.
// Hidden from it, the loads cost no such waits; the tile is handed over by an explicit wait
// (wait_loads) followed by a barrier, and the compiler moves no memory access across either.
// (M0 is reserved to the compiler, which uses it for nothing else in these kernels; naming it as
// clobbered is still the honest description of the statement.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
EA_DEV uint64_t uniform_address(const void* p) {      // the same value in scalar registers
    const uint64_t a = (uint64_t)(uintptr_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a), hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
    return ((uint64_t)hi << 32) | lo;
}
EA_DEV uint32_t lds_address(const void* p) {          // LDS byte address of a pointer into LDS, scalar
    return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p);
}
EA_DEV void load16_to_lds(uint64_t base_uniform, uint32_t lane_off, uint32_t lds_wave_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 : : "v"(lane_off), "s"(base_uniform), "s"(lds_wave_base) : "memory", "m0");
}
EA_DEV void load4_to_lds(uint64_t base_uniform, uint32_t lane_off, uint32_t lds_wave_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 : : "v"(lane_off), "s"(base_uniform), "s"(lds_wave_base) : "memory", "m0");
}
#pragma clang diagnostic pop

// rows row0..row0+63 of a row-major [.., D] matrix -> LDS tile; the NW waves share the NINST loads
template <class E, int D, int NW>
EA_DEV void issue_rows(char* lds, const typename E::elem* g, long row0, int wave, int lane) {
    using L = RowTile<E, D>;
    static_assert(L::NINST % NW == 0, "loads must divide evenly over the waves");
    // scalar 64-bit base (the tile's first row is the same for all lanes) + 32-bit lane offset
    const uint64_t base = uniform_address((const char*)g + row0 * (long)L::ROW_BYTES);
    const uint32_t lds0 = lds_address(lds);
#pragma unroll
    for (int i = 0; i < L::NINST / NW; ++i) {
        const int t = i * NW + wave;              // wave is wave-uniform (an SGPR)
        const int p = 64 * t + lane, row = p / L::CPR, pos = p % L::CPR;
        const uint32_t off = (uint32_t)(row * L::ROW_BYTES + ((pos ^ swz<L::CPR>(row)) * 16));
        load16_to_lds(base, off, lds0 + t * 1024);
    }
}
EA_DEV void wait_loads() { __builtin_amdgcn_s_waitcnt(0x0f70); }   // vmcnt(0) only (gfx9 encoding)
// LDS word += v, &= v without a returned value.  Written as instructions of their own because the
// compiler makes an LDS atomic wait for every direct global->LDS load in flight (it cannot tell
// that they target another array), which would stall a histogram update until the next tile has
// landed.  LDS operations of one wave execute in issue order; lds_settle() before other waves
// read the counters.
EA_DEV void lds_add_u32(const void* p, uint32_t v) {
    const uint32_t addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
    asm volatile("ds_add_u32 %0, %1" : : "v"(addr), "v"(v) : "memory");
}
EA_DEV void lds_and_b32(const void* p, uint32_t v) {
    const uint32_t addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
    asm volatile("ds_and_b32 %0, %1" : : "v"(addr), "v"(v) : "memory");
}
EA_DEV void lds_settle() { __builtin_amdgcn_s_waitcnt(0xc07f); }   // lgkmcnt(0) only (gfx9 encoding)

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

// ---- stage 1: C[kb][qb] = tile(64 x D, LDS row-major, swizzled) . owned^T -----------------------
#ifndef EA_FENCE
#define EA_FENCE true
#endif
// PFMAX = 0: rolling - the fragments of k-step s+1 are requested before the MFMAs of k-step s, so
// that their LDS latency passes behind those MFMAs (registers for two k-steps, as with PFMAX = 2).
template <class E, int D, int QB, bool FENCE = EA_FENCE, int PFMAX = 8>
EA_DEV void stage1(f32x16 (&C)[2][QB], const char* lds_tile, const Owned<E, D, QB>& own, int lane) {
    using L = RowTile<E, D>;
    constexpr int ES = (int)sizeof(typename E::elem);
    const int m = lane & 31, h = lane >> 5;
    const int row = perm_row(m);
    const int sw = swz<L::CPR>(row) * 16;        // swz(row + 32) == swz(row)
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int v = 0; v < 16; ++v) C[kb][qb][v] = 0.f;
    if constexpr (E::EPL == 8) {
        // lane half h takes chunk 2s+h of the row: byte (2s+h)*16 ^ sw = ((h*16) ^ sw) ^ (s*32)
        const int lane_off = row * L::ROW_BYTES + ((h * 16) ^ sw);
        // Request the A fragments of PF k-steps at a time and fence the scheduler there: the MFMAs
        // then start as the first fragments land, with the rest of the LDS latency behind them
        // (left alone, the compiler waits for each pair of reads right before its two MFMAs).
        constexpr int NS = D / E::KSTEP;
        if constexpr (PFMAX == 0) {
            typename E::frag a0[2], a1[2];
            a0[0] = *(const typename E::frag*)(lds_tile + lane_off);
            a1[0] = *(const typename E::frag*)(lds_tile + lane_off + 32 * L::ROW_BYTES);
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                if (s + 1 < NS) {
                    const char* a = lds_tile + (lane_off ^ ((s + 1) * 32));
                    a0[(s + 1) & 1] = *(const typename E::frag*)a;
                    a1[(s + 1) & 1] = *(const typename E::frag*)(a + 32 * L::ROW_BYTES);
                }
                if constexpr (FENCE) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    C[0][qb] = E::mma(a0[s & 1], own.f[qb][s], C[0][qb]);
                    C[1][qb] = E::mma(a1[s & 1], own.f[qb][s], C[1][qb]);
                }
                if constexpr (FENCE) __builtin_amdgcn_sched_barrier(0);
            }
            return;
        }
        constexpr int PF = PFMAX == 0 ? 1 : (NS < PFMAX ? NS : PFMAX);
        typename E::frag a0[PF], a1[PF];
#pragma unroll
        for (int s0 = 0; s0 < NS; s0 += PF) {
#pragma unroll
            for (int s = 0; s < PF; ++s) {
                const char* a = lds_tile + (lane_off ^ ((s0 + s) * 32));
                a0[s] = *(const typename E::frag*)a;
                a1[s] = *(const typename E::frag*)(a + 32 * L::ROW_BYTES);
            }
            if constexpr (FENCE) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s = 0; s < PF; ++s) {
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    C[0][qb] = E::mma(a0[s], own.f[qb][s0 + s], C[0][qb]);
                    C[1][qb] = E::mma(a1[s], own.f[qb][s0 + s], C[1][qb]);
                }
            }
            if constexpr (FENCE) __builtin_amdgcn_sched_barrier(0);
        }
    } else {
        // one element 2s+h per lane: chunk s/2, word 2(s%2)+h inside it
        const int lane_off = row * L::ROW_BYTES + sw + h * ES;
#pragma unroll
        for (int s = 0; s < D / E::KSTEP; ++s) {
            const char* a = lds_tile + ((lane_off ^ ((s / 2) * 16)) + 2 * (s % 2) * ES);
            const typename E::frag a0 = *(const typename E::frag*)a;
            const typename E::frag a1 = *(const typename E::frag*)(a + 32 * L::ROW_BYTES);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                C[0][qb] = E::mma(a0, own.f[qb][s], C[0][qb]);
                C[1][qb] = E::mma(a1, own.f[qb][s], C[1][qb]);
            }
        }
    }
}

// ---- stage 2: X[db][qb] += tile^T . Y[kb][qb], tile = 64 x D row-major in LDS (swizzled) ------
// 16-bit types: ds_read_b64_tr_b16 works on groups of 16 lanes.  Lane r of a group passes the
// address of four consecutive 16-bit elements ("row r" of a 16x4 block M); lane i receives
// M[i/4][i%4], M[4+i/4][i%4], M[8+i/4][i%4], M[12+i/4][i%4].  Group g = lane/16 serves MFMA rows
// m = 16(g%2)..+15 (tile columns 32db+m) of lane half h = g/2, whose contraction slots t = 0..7
// are tile rows R+t, R = 32kb+16s2+8h.  Lane r = 4e+q passes &tile[R+e][32db+16(g%2)+4q], so lane
// i receives tile[R+0..3][32db+m]: slots 0..3.  A second read from rows R+4.. gives slots 4..7.
template <class E2, int D, int QB, bool PINNED = false>
EA_DEV void stage2(f32x16 (&X)[D / 32][QB], const char* lds_tile, const f32x16 (&Y)[2][QB], int lane) {
    using L = RowTile<E2, D>;
    constexpr int ES = (int)sizeof(typename E2::elem);
    if constexpr (E2::EPL == 8) {
        typedef short s16x4 __attribute__((ext_vector_type(4)));
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        const int g = lane >> 4, i = lane & 15, e = i >> 2, q = i & 3, h = g >> 1;
        const int r_lo = 8 * h + e, r_hi = r_lo + 4;             // rows within the 16-row step
        const int cc = 2 * (g & 1) + (q >> 1);                     // 16-byte chunk within the 32-column block
        // byte offsets inside the step's first row block; the chunk index is XORed with swz(row),
        // and 4*db chunks / 16*(2kb+s2) rows are added per step (both commute with the XOR)
        const int off_lo = r_lo * L::ROW_BYTES + ((cc ^ swz<L::CPR>(r_lo)) * 16) + (q & 1) * 8;
        const int off_hi = r_hi * L::ROW_BYTES + ((cc ^ swz<L::CPR>(r_hi)) * 16) + (q & 1) * 8;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                typename E2::frag b[QB];
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                    for (int t = 0; t < 8; ++t) b[qb][t] = E2::from_float(Y[kb][qb][8 * s2 + t]);
                const char* rows = lds_tile + (32 * kb + 16 * s2) * L::ROW_BYTES;
#pragma unroll
                for (int db = 0; db < D / 32; ++db) {
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) s16x4*)(rows + (off_lo ^ (db * 64))));
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) s16x4*)(rows + (off_hi ^ (db * 64))));
                    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    const typename E2::frag a = __builtin_bit_cast(typename E2::frag, both);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) {
                        // (every pinned MFMA carries its own idle cycles: the compiler may reorder
                        // these statements, so any of them can end up right behind the conversion
                        // that writes its B fragment)
                        if constexpr (!PINNED) X[db][qb] = E2::mma(a, b[qb], X[db][qb]);
                        else E2::template mma_acc<true>(a, b[qb], X[db][qb]);
                    }
                }
            }
    } else {
        // K=2 MFMA: one tile row per lane half and step, MFMA row m = tile column 32db+m: a plain
        // 4-byte read of tile[trow][32db+m]
        const int m = lane & 31, h = lane >> 5;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = trow(kb, v, h);
                const char* rbase = lds_tile + row * L::ROW_BYTES + (m & 3) * ES;
                const int sw = swz<L::CPR>(row);
#pragma unroll
                for (int db = 0; db < D / 32; ++db) {
                    const int chunk = (32 * db + m) / 4;
                    const typename E2::frag a = *(const typename E2::frag*)(rbase + ((chunk ^ sw) * 16));
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) X[db][qb] = E2::mma(a, Y[kb][qb][v], X[db][qb]);
                }
            }
    }
}

// ---- fragment readers for hand-ordered tile bodies (16-bit types) -----------------------------
// The same fragments stage1/stage2 read, one at a time, so that a kernel can place every LDS read,
// MFMA and vector-ALU statement itself (see sched_fence).
template <class E, int D> struct Frag1 {          // stage-1 A fragment: MFMA rows = permuted tile rows
    using L = RowTile<E, D>;
    int lane_off;
    EA_DEV explicit Frag1(int lane) {
        const int m = lane & 31, h = lane >> 5, row = perm_row(m);
        lane_off = row * L::ROW_BYTES + ((h * 16) ^ (swz<L::CPR>(row) * 16));
    }
    // rows 32 kb .. of the tile, contraction elements 16 s ..
    EA_DEV typename E::frag operator()(const char* tile, int kb, int s) const {
        return *(const typename E::frag*)(tile + (lane_off ^ (s * 32)) + kb * 32 * L::ROW_BYTES);
    }
};
template <class E2, int D> struct Frag2 {         // stage-2 A fragment: tile^T via the LDS transpose read
    using L = RowTile<E2, D>;
    int off_lo, off_hi;
    EA_DEV explicit Frag2(int lane) {
        const int g = lane >> 4, i = lane & 15, e = i >> 2, q = i & 3, h = g >> 1;
        const int r_lo = 8 * h + e, r_hi = r_lo + 4, cc = 2 * (g & 1) + (q >> 1);
        off_lo = r_lo * L::ROW_BYTES + ((cc ^ swz<L::CPR>(r_lo)) * 16) + (q & 1) * 8;
        off_hi = r_hi * L::ROW_BYTES + ((cc ^ swz<L::CPR>(r_hi)) * 16) + (q & 1) * 8;
    }
    // tile columns 32 db .., contraction over tile rows 32 kb + 16 s2 ..
    EA_DEV typename E2::frag operator()(const char* tile, int kb, int s2, int db) const {
        typedef short s16x4 __attribute__((ext_vector_type(4)));
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        const char* rows = tile + (32 * kb + 16 * s2) * L::ROW_BYTES;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(rows + (off_lo ^ (db * 64))));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(rows + (off_hi ^ (db * 64))));
        return __builtin_bit_cast(typename E2::frag, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
};
// Nothing moves across: the statements between two fences are scheduled among themselves only.
EA_DEV void sched_fence() { __builtin_amdgcn_sched_barrier(0); }

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

// The same, added to what is there with fp32 atomics (several work-groups share the rows).
template <int D, int QB>
EA_DEV void add_owned_T(float* g, long row0, const f32x16 (&X)[D / 32][QB], float scale, int lane) {
    const int n = lane & 31, h = lane >> 5;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        float* rowp = g + (row0 + 32 * qb + n) * (long)D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int c = 0; c < 4; ++c) atomicAdd(rowp + 32 * db + 8 * a + 4 * h + c, X[db][qb][4 * a + c] * scale);
    }
}

template <int D, int QB>
EA_DEV void store_owned_T(float* g, long row0, const f32x16 (&X)[D / 32][QB], float scale, int lane) {
    float scales[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) scales[qb] = scale;
    store_owned_T<D, QB>(g, row0, X, scales, lane);
}

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

EA_DEV float wave_max(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}
// Exchange between the two lanes (n, n + 32) of an owned row with v_permlane32_swap, an ALU
// instruction: as an LDS permute the exchange queues behind every tile read of the CU's other waves.
// Swapping a register with a copy of itself leaves (low half, low half) in one and (high half,
// high half) in the other, so any symmetric combination of the two is the row's value in all lanes.
EA_DEV void xhalf_both(float v, float& lo, float& hi) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    lo = __uint_as_float(r[0]); hi = __uint_as_float(r[1]);
}
// Maxima as bare instructions: before an IEEE fmaxf the compiler first copies each operand through
// v_max_f32 x, x (to quiet a signalling NaN), which in the maximum tree of a score tile is a third
// of the instructions.
EA_DEV float max3_raw(float a, float b, float c) { float r; asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c)); return r; }
EA_DEV float max2_raw(float a, float b) { float r; asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b)); return r; }
// maximum of registers off .. off+7 of an accumulator
EA_DEV float max8_raw(const f32x16& C, int off) {
    float m = max3_raw(C[off], C[off + 1], C[off + 2]);
    m = max3_raw(m, C[off + 3], C[off + 4]);
    m = max3_raw(m, C[off + 5], C[off + 6]);
    return max2_raw(m, C[off + 7]);
}
EA_DEV float xhalf_max(float v) { float a, b; xhalf_both(v, a, b); return max2_raw(a, b); }
EA_DEV float xhalf_sum(float v) { float a, b; xhalf_both(v, a, b); return a + b; }
// the value the other lane of the row holds
EA_DEV float xhalf_other(float v, int h) { float a, b; xhalf_both(v, a, b); return h ? a : b; }

}  // namespace ea
