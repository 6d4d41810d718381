// Pieces shared by the forward and backward kernels: parameter block, block->work mapping,
// the entmax power functions, mask-word helpers, the tile streaming loop.
#pragma once
#include "tiles.hpp"

namespace ea {

constexpr int MAX_T = 2048;     // N <= 131072
constexpr int MAX_W = 64;       // mask words per row
// A row group's output comes from the gather kernel when its candidate lists average at most
// GATHER_LIST_MAX entries per row and its supports at most GATHER_SUP_MAX keys per row.
constexpr int GATHER_LIST_MAX = 320, GATHER_SUP_MAX = 48;
// Backward: support entries per lane list (two lists per row), entries per key in the lists by key,
// and the non-zeros per marked 64 x 64 tile up to which a row group takes the gather path.
// Work-group sizes of the gather kernels: each 16 lanes take one row (or key) at a time, a chain of
// dependent loads; 16 rows or keys per work-group (one per 16 lanes) measured 10 - 20 % faster than
// 128 - 256 per work-group, whose lanes walked 8 - 16 such chains one after the other.
// Query tiles per part of a mask column in dkdv_kernel from 65536 tokens on (half that below;
// every part pays the column walk, the owned K, V fragments and atomic adds of its results, and an
// empty part a work-group's launch: parts of 32 or 16 tiles measured slower at every length).
constexpr int COL_PART = 128;
constexpr int GATHER_ROWS = 16;          // rows per work-group of gather_out / bwd_rows / bwd_hot
constexpr int BWD_COLS_KEYS = 16;        // keys per work-group of bwd_cols_kernel
constexpr int BWD_LIST_CAP = 64, KEY_LIST_CAP = 128, BWD_ENTRIES_PER_TILE = 32, BWD_ENTRIES_PER_ROW = 6, BWD_FEW_TILES = 40;
// The gather kernels' fixed cost is a few passes over dK and dV; below this many marked tiles per
// 64-row block (at head dim 128; twice as many at 64) the matrix kernels' whole time is less.
constexpr int BWD_MIN_TILES_PER_BLOCK = 16;

constexpr int ALPHA_15 = 0, ALPHA_20 = 1, ALPHA_GEN = 2;
constexpr int LIST_CAP = 256;   // candidate entries per (row, lane half)

// What depends on alpha, per head when alpha differs between heads (then a table of these, one per
// head, sits in the workspace; otherwise the copy inside Params is used).
struct HeadConsts {
    float alpha;
    float c;              // (alpha-1)/sqrt(d): x = c * <q,k>
    float r;              // 1/(alpha-1)
    // c = kappa * rho with kappa a power of two and 1 <= rho < 2 (dK/dV kernel: keys scaled by kappa,
    // which is exact, scores kept in units of rho); rho_p = rho^r, rho_u = rho^(r-1)
    float kappa, rho, rho_p, rho_u;
    float pad;
};

struct Params {
    const void* Q; const void* K; const void* V; const void* dO;
    const void* V2;       // forward: V in the stage-2 element type (fp16 copy for bf16 inputs)
    float* O;             // forward: output; backward: the forward's output (nullable)
    float* tau; float* delta;
    float* ntau;          // backward scratch [BH][N]: -tau / rho, the bias the dK/dV kernel starts its scores from
    float* dQ; float* dK; float* dV;
    int32_t* mask;        // exported / final mask   [BH][T][W]
    int32_t* wmask;       // working mask (superset) [BH][T][W]
    int32_t* iters;       // nullable
    float* rs_lo; float* rs_hi; float* rs_f1; int* rs_state;   // [BH][N] solver state handed from tau_kernel to out_kernel
    float* rs_t0; float* rs_up0;   // [BH][N] what the histogram stage alone gave: tau_0 and the bracket's upper end (read out by tests)
    _Float16* tmax;       // [BH][T][N] per-row key-tile maxima of the raw scores (forward scratch)
    void* lists;          // [BH][N][2][LIST_CAP] candidate scores (raw score, key index), 8 bytes each
    int32_t* scnt;        // [BH][N][2] entries at the front of each list that are in the support at the final tau
    int32_t* gflag;       // [BH][ceil(N / grows)] 1 = the rows of this row group get their output by the gather kernel
    int grows;            // rows per row group of the candidate-list kernel
    // backward: entries per lane list of p.lists (its own lists, or the forward's when the caller hands
    // them over), and then the forward's group flags and their row-group size
    int right_edge;      // forward: thresholds are the right-edge histogram roots, no refinement (Sec. 3.2)
    // dkdv_kernel: a key block's mask column (its list of query tiles) is worked off in parts of
    // col_part_len tiles: work-group blockIdx takes part blockIdx / (BH * key blocks), leaves at
    // once where colcnt (the columns' lengths, from col_count_kernel) says the list ends before its
    // part, and adds to dK, dV atomically where the column has several parts (col_count_kernel
    // cleared those rows).  col_part_len = 0: whole columns, one work-group each, no counts.
    int col_part_len;
    int32_t* colcnt;
    int list_cap;
    const int32_t* fwd_gflag; const unsigned int* fwd_scal;   // (fwd_scal[2] = rows per row group of the forward's flags)
    int32_t* kcnt;        // backward [BH][N]: entries in each key's list
    int32_t* nplain;      // backward: number of row groups that stay with dq_kernel / dkdv_kernel
    int32_t* nmarked;     // backward: set bits of the whole mask
    int32_t* defer;       // backward [BH][N]: entries of the row left to bwd_hot_kernel
    void* klist;          // backward [BH][N][KEY_LIST_CAP]: (query row, u dP, u, P), 16 bytes each
    int32_t* oflag;       // [BH][T] 1 = some row of this 64-row block has more candidates than its lists hold
    unsigned long long* stats;
    // bits of non-negative floats kept in the workspace (atomicMax on the bit patterns):
    // scal[0] = max |dO| rounded up to a power of two (the backward uses dO divided by it: exact)
    // scal[1] = forward: number of row groups left to out_kernel (a plain counter)
    // scal[2] = forward: rows per row group of its gather flags (for a backward that is handed the forward's lists)
    unsigned int* scal;
    int BH, N, T, W;
    int causal;
    HeadConsts hc;        // the constants of the call's single alpha
    const HeadConsts* hc_table;   // [H] per-head constants, or null
    int H;
    float inv_sqrt_d;
    float tol;
    int max_sweeps;
};

EA_DEV HeadConsts head_consts(const Params& p, int bh) { return p.hc_table ? p.hc_table[bh % p.H] : p.hc; }

// Consecutive block ids are dealt round-robin to the 8 XCDs (each with its own L2).  When the
// number of heads divides by 8 every XCD gets whole heads, so the work-groups that run together
// on one XCD stream the same K/V tiles.  Within a head the longest (causal: last) tiles go first.
EA_DEV void map_block(int bid, int BH, int ntile, int& bh, int& I) {
    int lin = bid;
    if ((BH & 7) == 0) {
        const int per = (BH >> 3) * ntile;
        lin = (bid & 7) * per + (bid >> 3);
    }
    bh = lin / ntile;
    I = ntile - 1 - (lin % ntile);
}

// y > 0:  y^r, y^(r-1), y^(r-2)  with r = 1/(alpha-1)
template <int AM> EA_DEV float pow_r(float y, float r) {
    if constexpr (AM == ALPHA_15) return y * y;
    else if constexpr (AM == ALPHA_20) return y;
    else return __builtin_amdgcn_exp2f(r * __builtin_amdgcn_logf(y));
}
// (alpha > 2: the exponent r - 1 is negative, at least -1/2 for alpha <= 3, and y^(r-1) grows
// without limit as y falls to zero.  y is held at or above 1e-6, about the accuracy to which an fp32
// score difference is known anyway, so that the result stays below 1e3 and its products with dP - delta
// inside the range of the fp16 operands of the backward's second-stage products.)
template <int AM> EA_DEV float pow_r1(float y, float r) {
    if constexpr (AM == ALPHA_15) return y;
    else if constexpr (AM == ALPHA_20) return 1.f;
    else return __builtin_amdgcn_exp2f((r - 1.f) * __builtin_amdgcn_logf(r < 1.f ? fmaxf(y, 1e-6f) : y));
}
template <int AM> EA_DEV float pow_r2(float y, float r) {
    if constexpr (AM == ALPHA_15) return 1.f;
    else if constexpr (AM == ALPHA_20) return 0.f;
    else return __builtin_amdgcn_exp2f((r - 2.f) * __builtin_amdgcn_logf(y));
}

// Walk over `ntiles` streamed tiles.  issue(it, buf) starts the direct global->LDS loads of tile
// `it` into the buffer set at `buf`; compute(it, buf) does the math on it.
// NBUF == 2: the loads of tile it+1 fly under the math of tile it, one barrier per tile.  The two
// buffer sets must be two distinct __shared__ variables: the compiler gives each LDS variable its
// own alias scope, and only then does it refrain from making every LDS read of the tile being
// worked on wait for the loads in flight into the other set.
// NBUF == 1: half the LDS; loads and math alternate (other work-groups on the CU fill the gaps).
template <int NBUF, class IssueF, class ComputeF>
EA_DEV void stream_tiles(int ntiles, char* buf0, char* buf1, IssueF issue, ComputeF compute) {
    if constexpr (NBUF == 2) {
        if (ntiles > 0) issue(0, buf0);
        for (int it = 0; it < ntiles; it += 2) {
            wait_loads();
            __syncthreads();     // tile `it` has landed for every wave; everyone is done with tile it-1
            if (it + 1 < ntiles) issue(it + 1, buf1);
            compute(it, buf0);
            if (it + 1 >= ntiles) break;
            wait_loads();
            __syncthreads();
            if (it + 2 < ntiles) issue(it + 2, buf0);
            compute(it + 1, buf1);
        }
        __syncthreads();
    } else {
        for (int it = 0; it < ntiles; ++it) {
            issue(it, buf0);
            wait_loads();
            __syncthreads();
            compute(it, buf0);
            __syncthreads();
        }
    }
}

// The same walk with two tile bodies: tiles [0, n1) go to compute1, tiles [n1, n) to compute2
// (n1 even, or n1 == n), as two loops one after the other that share the double buffer: the first
// tile of the second loop is loaded under the last tile of the first.  Two loops rather than a
// choice per tile because accumulators pinned to registers by assembly statements must not meet at
// a join inside the loop (the compiler then copies all of them on one of the two paths, every tile).
template <class IssueF, class Compute1, class Compute2>
EA_DEV void stream_tiles_split(int n1, int n, char* buf0, char* buf1, IssueF issue, Compute1 compute1, Compute2 compute2) {
    if (n > 0) issue(0, buf0);
    int it = 0;
    for (; it < n1; it += 2) {
        wait_loads();
        __syncthreads();
        if (it + 1 < n) issue(it + 1, buf1);
        compute1(it, buf0);
        if (it + 1 >= n1) { it = n1; break; }        // only when n1 == n is odd
        wait_loads();
        __syncthreads();
        if (it + 2 < n) issue(it + 2, buf0);
        compute1(it + 1, buf1);
    }
    for (; it < n; it += 2) {
        wait_loads();
        __syncthreads();
        if (it + 1 < n) issue(it + 1, buf1);
        compute2(it, buf0);
        if (it + 1 >= n) break;
        wait_loads();
        __syncthreads();
        if (it + 2 < n) issue(it + 2, buf0);
        compute2(it + 1, buf1);
    }
    __syncthreads();
}

// The walk with NB >= 2 tile buffers in one LDS ring: tiles run NB - 1 ahead of the math, so a tile
// has NB - 1 tile times to arrive.  LPW = direct loads each wave issues per tile.  Vector-memory
// operations complete in issue order, so tile `it` has landed once at most the loads of the tiles
// issued after it are outstanding (other stores a wave issues meanwhile only make the wait longer).
template <int K> EA_DEV void wait_vm_at_most() { asm volatile("s_waitcnt vmcnt(%0)" : : "n"(K) : "memory"); }
template <int NB, int LPW, class IssueF, class ComputeF>
EA_DEV void stream_tiles_ring(int n, char* ring, int tile_bytes, IssueF issue, ComputeF compute) {
    static_assert(NB >= 2 && NB <= 4 && (NB - 2) * LPW < 64, "ring depth");
    for (int i = 0; i < NB - 1 && i < n; ++i) issue(i, ring + i * tile_bytes);
    for (int it = 0; it < n; ++it) {
        const int ahead = min(NB - 2, n - 1 - it);         // tiles issued after tile `it`
        if (NB >= 4 && ahead == 2) wait_vm_at_most<2 * LPW>();
        else if (NB >= 3 && ahead == 1) wait_vm_at_most<LPW>();
        else wait_vm_at_most<0>();
        __syncthreads();     // tile `it` has landed for every wave; everyone is done with tile it-1
        if (it + NB - 1 < n) issue(it + NB - 1, ring + ((it + NB - 1) % NB) * tile_bytes);
        compute(it, ring + (it % NB) * tile_bytes);
    }
    __syncthreads();
}

// Executed-work counters.  The workspace starts with STATS_COPIES copies of the STATS_WORDS
// counters (a counter's value is the sum over the copies).  The waves of a group first add into
// LDS; one thread per counter then issues one global atomic, aimed at the copy picked by the
// block id, so that the atomics of groups finishing together fall on different cache lines
// (tens of thousands of atomics on one line cost more than a small kernel's whole run time).
constexpr int STATS_WORDS = 16, STATS_COPIES = 64;
template <int K>
EA_DEV void flush_counters(unsigned long long* blk, unsigned long long* stats, const int (&slot)[K],
                           const unsigned long long (&val)[K], int tid, int lane) {
    __syncthreads();
    if (tid < K) blk[tid] = 0ull;
    __syncthreads();
    if (lane == 0) {
#pragma unroll
        for (int k = 0; k < K; ++k)
            if (val[k]) atomicAdd(&blk[k], val[k]);
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < K; ++k)
        if (tid == k && blk[k]) atomicAdd(&stats[(blockIdx.x & (STATS_COPIES - 1)) * STATS_WORDS + slot[k]], blk[k]);
}

// Union of `rows` mask rows (LDS, `W` words each) -> ascending list of tile indices in LDS.
// Called by all threads; the first wave does the work.  Uses one wave-wide exclusive scan of
// the per-word popcounts (W <= 64).
template <class ListT>
EA_DEV void build_tile_list(const uint32_t* words, int rows, int W, ListT* list, int* count, int tid) {
    __syncthreads();
    if (tid < 64) {
        uint32_t u = 0;
        if (tid < W)
            for (int r = 0; r < rows; ++r) u |= words[r * W + tid];
        const int cnt = __popc(u);
        int incl = cnt;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int t = __shfl_up(incl, off);
            if (tid >= off) incl += t;
        }
        int pos = incl - cnt;
        while (u) {
            const int b = __ffs(u) - 1;
            u &= u - 1;
            list[pos++] = (ListT)(tid * 32 + b);
        }
        if (tid == 63) *count = incl;
    }
    __syncthreads();
}

EA_DEV bool mask_bit(const uint32_t* words, int W, int row, int j) {
    return (words[row * W + (j >> 5)] >> (j & 31)) & 1u;
}

// Hide keys above the diagonal: element (tile row, owned row) of a stage-1 result with
// streamed index s_idx = s0 + trow and owned index o_idx = o0 + 32 qb + n.
// KEYS_STREAMED: streamed rows are keys (hide when key > query), else streamed rows are queries.
template <int QB, bool KEYS_STREAMED>
EA_DEV void causal_hide(f32x16 (&C)[2][QB], int s0, int o0, int lane) {
    const int n = lane & 31, h = lane >> 5;
    // hide when (s0 + trow) > (o0 + 32 qb + n)   [keys streamed]   i.e. trow > lim
    //        or (o0 + 32 qb + n) > (s0 + trow)   [queries streamed] i.e. trow < lim
    const int lim0 = o0 + n - s0 - 8 * h;      // compare 32 kb + 16 (v/8) + v%8 against lim0 + 32 qb
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int t = 32 * kb + 16 * (v >> 3) + (v & 7) - 32 * qb;   // compile-time constant
                const bool hide = KEYS_STREAMED ? (t > lim0) : (t < lim0);
                if (hide) C[kb][qb][v] = -INFINITY;
            }
}

}  // namespace ea
