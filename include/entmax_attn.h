/*
 * entmax_attn.h - C ABI of the MI355X (gfx950) alpha-entmax attention library.
 *
 * The library computes, per (batch, head) and per query row r (AdaSplash-2 paper):
 *     S = Q K^T / sqrt(d)                                              (Eq. 2)
 *     P = [(alpha-1) S - tau]_+^{1/(alpha-1)},  sum_j P_rj = 1          (Eq. 3, Eq. 4)
 *     O = P V                                                          (Eq. 2)
 * with tau solved per row from an on-chip histogram of the scores within one unit of the row
 * maximum (Eq. 6-9, Prop. 1) followed by a safeguarded Halley/Newton refinement (Sec. 3.1-3.3,
 * Alg. 1) whose evaluations of f run over the row's candidate scores, listed during the one dense
 * sweep of Q K^T, and the gradient of
 * sum(O * dO) with respect to Q, K, V (Sec. 3.3 "Backward pass", Alg. 2-3).  Key tiles
 * whose probabilities are all zero are recorded in a bit-packed block mask (App. C.4) and
 * skipped in the output phase and in both backward kernels.
 *
 * Conventions common to every entry point
 *   - All tensor arguments are DEVICE pointers owned by the caller.  Tensors are
 *     contiguous [B, H, N, d] with d fastest.  Inputs Q, K, V, dO have the element type
 *     named by `dtype`; O, dQ, dK, dV, tau are always float32.
 *   - N must be a positive multiple of 64 and at most 131072; d must be 64 or 128;
 *     1 < alpha <= EA_ALPHA_MAX.  With bf16 inputs, values of magnitude above 65504 are outside the
 *     library's domain (second-stage products run on fp16 copies): they enter those copies as
 *     +-65504 and are counted in EA_STAT_F16_CLAMPED.
 *   - Causal masking: key j is visible to query r iff j <= r.
 *   - The library allocates nothing and never synchronises: all work is enqueued on
 *     `hip_stream` (a hipStream_t passed as void*; NULL = the default stream).  Scratch
 *     space is the caller's `workspace` (device memory, 256-byte aligned), of at least
 *     entmax_attn_workspace_bytes(...) bytes.
 *   - Return value: EA_OK (0) on success.  On any negative code nothing has been
 *     enqueued, except EA_ERR_HIP where earlier launches of the same call may have been.
 *   - Calls that share a workspace must be ordered on one stream.
 */
#ifndef ENTMAX_ATTN_H
#define ENTMAX_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Element type of Q, K, V, dO.  Entry points take it as a plain int (any other value is answered
 * with EA_ERR_DTYPE, or a size of 0). */
typedef enum { EA_F32 = 0, EA_BF16 = 1 } ea_dtype;

/* Largest alpha accepted.  Sec. 3.2 covers every alpha > 1 (secant steps above 2); the bound keeps
 * the backward's U = P^(2-alpha) = y^(1/(alpha-1) - 1), which grows without limit as a probability
 * approaches zero once alpha > 2, inside the range of the fp16 operands of the second-stage
 * products: with alpha <= 3 the exponent is at least -1/2. */
#define EA_ALPHA_MAX 3.0f

enum {
    EA_OK = 0,
    EA_ERR_NULL = -1,       /* a required pointer is NULL */
    EA_ERR_ALPHA = -2,      /* alpha not finite or outside (1, EA_ALPHA_MAX] */
    EA_ERR_SHAPE = -3,      /* B, H <= 0, N not a positive multiple of 64 or > 131072, d not in {64, 128} */
    EA_ERR_DTYPE = -4,      /* unknown ea_dtype */
    EA_ERR_WORKSPACE = -5,  /* workspace NULL, misaligned or too small */
    EA_ERR_HIP = -6,        /* a HIP call failed; see entmax_attn_last_hip_error() */
    EA_ERR_TOO_LARGE = -7   /* the problem needs more scratch than an allocation-free entry point holds */
};

/* The workspace starts with EA_STATS_COPIES copies of EA_STATS_WORDS 64-bit counters
 * ([copy][counter]); the value of a counter is the sum over the copies (see entmax_attn_fwd). */
#define EA_STATS_WORDS 16
#define EA_STATS_COPIES 64
enum {
    /* units: 64x32 score sub-tiles (64 streamed rows x 32 register-resident rows), the piece one
     * wavefront computes per MFMA block pair; one matmul on a sub-tile is 2*64*32*d flops */
    EA_STAT_TAU_TILES = 0,   /* sub-tiles scored by the dense threshold sweep and by any sweep-based refinement (1 matmul each) */
    EA_STAT_OUT_TILES = 1,   /* sub-tiles scored by the output phase (2 matmuls each where P != 0) */
    EA_STAT_DELTA_TILES = 2, /* unused (delta is found inside the dQ sweep) */
    EA_STAT_DQ_TILES = 3,    /* sub-tiles visited by the dQ kernel (4 matmuls each) */
    EA_STAT_DKDV_TILES = 4,  /* sub-tiles visited by the dK/dV kernel (4 matmuls each) */
    EA_STAT_SWEEPS = 5,      /* work-groups that ran the sweep-based threshold kernel (each runs one refinement sweep) */
    EA_STAT_MASK_TILES = 6,  /* sub-tiles scored when the backward rebuilds the mask (1 matmul each) */
    EA_STAT_OUT_PV_TILES = 7, /* sub-tiles of the output phase whose P V product was issued */
    EA_STAT_LIST_OVERFLOW = 8, /* 64-row blocks whose candidate lists overflowed (redone by the sweep-based kernel) */
    EA_STAT_GATHER_ROWS = 9,  /* rows whose output was gathered from their listed support (no output-phase matmuls) */
    EA_STAT_BWD_LIST_TILES = 10, /* sub-tiles scored when the backward lists the supports of sparse row groups (1 matmul each) */
    EA_STAT_BWD_GATHER_ROWS = 11, /* rows whose gradients were formed entry by entry from their listed support */
    EA_STAT_F16_CLAMPED = 12  /* bf16 input values of magnitude above 65504 that were copied as +-65504 into the fp16 operands of the matrix kernels: non-zero means the inputs were outside the library's domain */
};

/* Edge of the square score tiles that one bit of the block mask stands for (64). */
int entmax_attn_mask_tile(void);

/* Bytes of workspace needed by entmax_attn_fwd (is_bwd == 0) or entmax_attn_bwd
 * (is_bwd != 0) for this problem; 0 if the shape or dtype is invalid. */
size_t entmax_attn_workspace_bytes(int B, int H, int N, int d, int dtype, int causal, int is_bwd);

/*
 * Forward (Alg. 1): row maximum, histogram and candidate lists (one dense sweep) -> histogram
 * solve and refinement on the lists (+ working mask) -> output, whose row sums check f once more.
 * A 64-row block with a row that has more candidates than its two lists hold (256 each, one per
 * half of the lanes that computed its scores) is redone by the sweep-based threshold kernel.
 *   Q, K, V     in   [B,H,N,d] of `dtype`
 *   O           out  [B,H,N,d] float32
 *   tau         out  [B,H,N]   float32, raw convention: P = [(alpha-1) S - tau]_+^{1/(alpha-1)}
 *   block_mask  out  [B,H,N/64,ceil(N/64/32)] int32; bit k of word m of row i is set iff some
 *                    P > 0 (at the returned tau) in the 64x64 tile (i, 32m+k) (App. C.4);
 *                    bits of tiles above the causal diagonal and padding bits are 0
 *   iters       out  [B,H,N] int32, may be NULL: number of refinement iterations the row
 *                    needed; one iteration = one evaluation of f over the true scores followed
 *                    by one update (Sec. 3.3 Phase 3); the check that the output phase gets
 *                    from its row sums counts only where it moved tau
 * The first EA_STATS_COPIES * EA_STATS_WORDS uint64 of `workspace` are zeroed by the call and
 * then hold the executed-tile counters of this call (EA_STAT_*, summed over the copies),
 * readable after the stream has drained.
 */
int entmax_attn_fwd(const void* Q, const void* K, const void* V,
                    float* O, float* tau, int32_t* block_mask, int32_t* iters,
                    int B, int H, int N, int d, int dtype, float alpha, int causal,
                    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Backward (Alg. 2-3): dQ kernel (which also finds delta) over mask rows, dK/dV kernel over mask columns.
 *   Q, K, V, dO in   [B,H,N,d] of `dtype`
 *   O           in   [B,H,N,d] float32, the forward's output; used only to centre the dQ sums
 *                    (<dO_r, O_r> is subtracted from dP before rounding); may be NULL, at the price
 *                    of extra rounding error in dQ when dP is large and nearly constant on a row's support
 *   tau         in   [B,H,N] float32 as returned by the forward
 *   block_mask  in   as returned by the forward, or NULL: then it is rebuilt from tau with one
 *                    dense score sweep
 *   dQ, dK, dV  out  [B,H,N,d] float32, overwritten
 * Counters as for the forward.
 */
int entmax_attn_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                    const float* tau, const int32_t* block_mask,
                    float* dQ, float* dK, float* dV,
                    int B, int H, int N, int d, int dtype, float alpha, int causal,
                    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * entmax_attn_bwd for a caller that still holds the forward call's workspace.  The forward leaves,
 * for every row group whose output it formed from listed supports, each row's support (raw score
 * and key index) at the front of its candidate lists; with them the backward need not find the
 * supports again (one score sweep over the marked tiles less).  Results as entmax_attn_bwd.
 *   fwd_workspace  in  the workspace of the entmax_attn_fwd call (same Q, K, V, shape, dtype, alpha,
 *                      causal) that produced O, tau and block_mask, not written to since; at least
 *                      entmax_attn_workspace_bytes(..., is_bwd = 0) bytes, 256-byte aligned.  The
 *                      backward reads it and leaves it as it found it.
 *   block_mask     in  required here (the forward's).
 * EA_ERR_NULL if fwd_workspace is NULL, EA_ERR_WORKSPACE if it is misaligned or too small or the mask
 * is missing.  Handing over a workspace that does not belong to these tensors gives wrong gradients
 * (or reads of rows that do not exist): the library cannot tell.
 */
int entmax_attn_bwd_with_lists(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                               const float* tau, const int32_t* block_mask,
                               void* fwd_workspace, size_t fwd_workspace_bytes,
                               float* dQ, float* dK, float* dV,
                               int B, int H, int N, int d, int dtype, float alpha, int causal,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Right-edge binning (Sec. 3.2, the paragraph after Prop. 1): an approximate forward.  Rounding
 * every score up to its bin's right edge instead of down to the left one moves the histogram's root
 * up by one bin width h = 1/63, to tau_h + h >= tau*.  With the switch on, entmax_attn_fwd (and the
 * per-head variant) takes that root as the threshold and does no refinement: `tau` holds it
 * (tau* <= tau < tau* + h + 2e-6 (1 + |tau|)), P = [(alpha-1) S - tau]_+^{1/(alpha-1)} has a support
 * inside the exact one and rows that sum to at most 1, O = P V, `block_mask` is P's.  Sparser and
 * cheaper than the exact result, not equal to it.  entmax_attn_bwd on these outputs evaluates the
 * formulas of Sec. 3.3 at that tau; they are the gradient only for the exact threshold.
 * The switch belongs to the calling host thread (off at its start) and applies to the forward calls
 * that thread makes after it; entmax_attn_decode is not affected.  Returns EA_OK.
 */
int entmax_attn_right_edge_enable(int on);

/*
 * The same two operations with one alpha per head (Sec. 3.2 gives the solver for every alpha
 * above 1; heads of one layer may use different values).  `alpha_per_head` is a HOST pointer to H
 * floats, each in (1, 2]; it is read before the call returns.  Head h of every batch entry uses
 * alpha_per_head[h].  When the values differ, all heads run the general-alpha code (power functions
 * through exp2/log2) and a table of per-head constants is written into the workspace first; when
 * they are all equal the call is the single-alpha one.  Everything else as in entmax_attn_fwd /
 * entmax_attn_bwd; EA_ERR_ALPHA if any value is outside (1, EA_ALPHA_MAX].
 */
int entmax_attn_fwd_alpha_per_head(const void* Q, const void* K, const void* V,
                                   float* O, float* tau, int32_t* block_mask, int32_t* iters,
                                   int B, int H, int N, int d, int dtype, const float* alpha_per_head, int causal,
                                   void* workspace, size_t workspace_bytes, void* hip_stream);
int entmax_attn_bwd_alpha_per_head(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                                   const float* tau, const int32_t* block_mask,
                                   float* dQ, float* dK, float* dV,
                                   int B, int H, int N, int d, int dtype, const float* alpha_per_head, int causal,
                                   void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Inference variant on materialised logits (the paper's appendix on language modelling; Sec. 5
 * names an optimised inference kernel as future work): one query row per head against all N
 * cached keys, no causal mask.
 *     z = K q / sqrt(d),  p = [(alpha-1) z - tau]_+^{1/(alpha-1)} with sum p = 1,  o = p V
 *   q           in   [B,H,d] of `dtype`
 *   K, V        in   [B,H,N,d] of `dtype`; any N in 1 .. 4194304, d 64 or 128
 *   O           out  [B,H,d] float32
 *   tau         out  [B,H]   float32, raw convention as in entmax_attn_fwd
 *   support     out  [B,H]   int32, may be NULL: number of keys with p > 0
 *   iters       out  [B,H]   int32, may be NULL: evaluations of f the refinement took
 * A first kernel reads K once and keeps, per work-group, only the logits within the window of Eq. 5
 * below the largest logit it has met so far (value and key index, in per-group lists in the workspace)
 * and its own maximum; a second kernel solves tau per head from the kept logits (histogram of the
 * scores within one unit of the maximum, Eq. 5-9, then the hybrid refinement of Sec. 3.2) and gathers
 * the rows of V in the support.  Conventions, error
 * codes and workspace rules as above; entmax_attn_decode_workspace_bytes returns 0 for a bad shape.
 */
size_t entmax_attn_decode_workspace_bytes(int B, int H, int N, int d, int dtype);
int entmax_attn_decode(const void* q, const void* K, const void* V,
                       float* O, float* tau, int32_t* support, int32_t* iters,
                       int B, int H, int N, int d, int dtype, float alpha,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * entmax_attn_decode for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs,
 * kernels and results as entmax_attn_decode; the scratch (per-group maxima and counts, kept logits)
 * is an array inside the library's code object, entmax_attn_decode_static_max_bytes() bytes
 * (33 MiB) per GPU, held until the process ends; its device address is looked up on the first call
 * on each device.  The call allocates and frees nothing and clears nothing (the kernels write every
 * scratch word before they read it).
 *   - EA_ERR_TOO_LARGE, nothing enqueued, when entmax_attn_decode_workspace_bytes(B, H, N, d, dtype)
 *     exceeds entmax_attn_decode_static_max_bytes() (about B*H*N <= 4 Mi keys, e.g. 32 heads x 128k).
 *   - All calls on one GPU share that GPU's array: calls that overlap on one GPU (different streams
 *     without ordering, or several host threads) race.  Order them on one stream.
 */
size_t entmax_attn_decode_static_max_bytes(void);
int entmax_attn_decode_static(const void* q, const void* K, const void* V,
                              float* O, float* tau, int32_t* support, int32_t* iters,
                              int B, int H, int N, int d, int dtype, float alpha, void* hip_stream);

/* Static, human-readable text for a return code. */
const char* entmax_attn_strerror(int code);

/* hipError_t (as int) of the most recent failing HIP call made by this library on the calling
 * thread, 0 if none. */
int entmax_attn_last_hip_error(void);

/* Measurement and test aids (per-kernel timers, the gather switch, the matrix-core rate probe, the
 * histogram stage's read-out) are declared in entmax_attn_aids.h: none of them is needed to use the
 * library. */

#ifdef __cplusplus
}
#endif
#endif /* ENTMAX_ATTN_H */
