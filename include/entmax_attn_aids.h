/*
 * entmax_attn_aids.h - measurement and test aids of the alpha-entmax attention library.
 *
 * Nothing here is needed to use the library (entmax_attn.h is the whole product interface); these
 * entry points serve the benchmark (per-kernel times, the matrix-core ceiling), A/B measurements
 * (the gather switch) and the tests of the histogram stage.  Same conventions and error codes.
 */
#ifndef ENTMAX_ATTN_AIDS_H
#define ENTMAX_ATTN_AIDS_H

#include "entmax_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Optional per-kernel timing (measurement aid, used by the benchmark; Sec. 4.2 reports forward
 * and backward times separately).  While enabled, every entmax_attn_fwd / entmax_attn_bwd call
 * records HIP events on its stream around each of its kernels, for up to 256 calls between
 * reads.  entmax_attn_timer_read waits for the recorded events, writes per slot the summed
 * kernel time in ms and the number of launches (arrays of at least EA_TIMER_SLOTS entries), and
 * starts a new recording window.  Events are created as they are first needed and kept.  The
 * recording state is one per process: enable, the calls to be timed and the read must come from one
 * host thread at a time.
 */
#define EA_TIMER_SLOTS 10
enum {
    EA_TIMER_FWD_PREP = 0,  /* fp16 copy of V (bf16 inputs; made after the threshold kernel, and only if some row group needs it) */
    EA_TIMER_TAU = 1,       /* dense sweep (maximum, histogram, candidate lists), solve, refinement; fallback kernel */
    EA_TIMER_OUT = 2,       /* phase 4 (gather over listed supports, block-sparse matrix products) and the rest of the refinement */
    EA_TIMER_MASK = 3,      /* mask rebuild of the backward (only when block_mask == NULL) */
    EA_TIMER_BWD_PREP = 4,  /* max |dO| (rounded up to a power of two) and the fp16 copies of K, Q, V, dO (bf16 inputs) */
    EA_TIMER_DQ = 5,        /* delta and dQ, one sweep */
    EA_TIMER_DKDV = 6,      /* dK, dV */
    EA_TIMER_DECODE_SCORES = 7, /* entmax_attn_decode: the kernel that reads K and keeps the logits near the maximum */
    EA_TIMER_BWD_LIST = 8,  /* backward: supports of the sparse row groups listed (one matrix product per marked tile) */
    EA_TIMER_BWD_GATHER = 9 /* backward of the sparse row groups from their lists: rows (dQ, delta), then keys (dK, dV), then the entries of overfull keys */
};
int entmax_attn_timer_enable(int on);
int entmax_attn_timer_read(float* ms_sum, int* launches, int slots);

/*
 * Sparse row groups (a handful of non-zeros per row: the regime Sec. 4 reports at long context)
 * are by default not run through the block-sparse matrix kernels of Alg. 1-3 but evaluated entry by
 * entry from lists of each row's support: forward, O_r as a sum over a few rows of V; backward,
 * dQ row by row and dK, dV key by key (EA_STAT_GATHER_ROWS, EA_STAT_BWD_GATHER_ROWS count the rows
 * that went that way).  Results are the same up to rounding.  entmax_attn_gather_enable(0) keeps
 * every row group on the matrix kernels (measurement and test aid).  The switch is a property of the
 * calling host thread (each thread starts with the gather paths on) and applies to the calls that
 * thread makes after it; returns EA_OK.
 */
int entmax_attn_gather_enable(int on);

/*
 * Matrix-core rate probe (measurement aid: the ceiling the benchmark prices the kernels against
 * besides the published peak).  Launches `groups` work-groups of 4 wavefronts; every wavefront
 * issues iters * 32 independent 32x32x16 fp16 MFMAs (32768 flops each) on operands taken from
 * `data` (device pointer to 8192 fp16 values filled by the caller; the sustained clock depends on
 * the operand values) and writes one float per thread to `sink` (groups * 256 floats).  256 groups
 * put one wavefront on every SIMD of an MI355X, 512 two.  The caller times the launch.
 * Total flops = groups * 4 * iters * 32 * 32768.
 */
int entmax_attn_mfma_probe(const void* data, float* sink, int groups, int iters, void* hip_stream);

/*
 * Co-issue probe (measurement aid: how much vector-ALU work hides under the matrix pipe, the figure
 * behind the distance of the score-handling kernels from the matrix roofline).  Launches 512
 * work-groups of 8 wavefronts (four per SIMD of an MI355X); every wavefront runs `iters` rounds of
 * 16 MFMAs 32x32x16 bf16 (if with_mfma) followed by valu_per_round independent v_add_u32
 * (0 only with with_mfma; else 64, 128 or 256), registers only.  `sink`: device pointer to
 * 512 * 512 floats.  The caller times the launch; time / iters is the time of one round on every
 * SIMD (64 MFMAs and 4 * valu_per_round additions).  EA_ERR_SHAPE for other counts.
 */
int entmax_attn_coissue_probe(float* sink, int iters, int valu_per_round, int with_mfma, void* hip_stream);

/* Histogram bins B per unit of (alpha-1) s used by the threshold kernels (introspection for tests
 * and the benchmark report): the bracket after the histogram solve is 1/B wide (Prop. 1). */
int entmax_attn_histogram_bins(void);

/*
 * What the histogram stage alone produced in the last entmax_attn_fwd call that used `workspace`
 * (Eq. 6-9, App. C.3, before any refinement; for tests of Prop. 1): per row, in the raw convention
 * of `tau`,
 *   tau0   out [B,H,N] float32: max(tau_h, max - 1) less a rounding slack of about 1e-6 - the point
 *                              the refinement starts from, never above the true threshold;
 *   upper  out [B,H,N] float32: tau_h + 1/B plus the same slack - the bracket's upper end.
 * Copies the two arrays out of the workspace on `hip_stream` (device to device, nothing allocated).
 * Shape arguments as in the forward call; error codes as above.
 */
int entmax_attn_fwd_histogram_bounds(const void* workspace, size_t workspace_bytes,
                                     int B, int H, int N, int d, int dtype,
                                     float* tau0, float* upper, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ENTMAX_ATTN_AIDS_H */
