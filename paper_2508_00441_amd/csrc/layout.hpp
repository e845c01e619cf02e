// Plan, internal data layouts and kernel-launcher prototypes shared by the libozaki translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace ozaki {

constexpr int MAX_SLICES = 32;
constexpr int MAX_PAIRS = MAX_SLICES * MAX_SLICES;      // all s*s pairs in the full mode
constexpr int64_t MAX_K_BLOCK_IN_REGISTERS = 16384;     // longer blocks are sliced by the streaming kernel (state in work memory)

// ---- tiling of the slice-pair GEMM: one workgroup computes one TILE x TILE block of one pair product ------
constexpr int TILE = 256;
constexpr int CHUNK_BYTES = 64;           // bytes of the inner dimension per row staged per pipeline step (FP8, FP16)
constexpr int CHUNK_BYTES_FP6 = 48;       // the same 64 inner indices as 6-bit codes
constexpr int TILE_ELEMS = TILE * TILE;

// slice formats (values of ozaki_slice_format)
constexpr int FMT_FP8 = 0, FMT_FP16 = 1, FMT_FP6 = 2, FMT_FP6_E3M2 = 3, FMT_INT8 = 4;     // FMT_FP6 is E2M3
__host__ __device__ constexpr bool fmt_is_fp6(int fmt) { return fmt == FMT_FP6 || fmt == FMT_FP6_E3M2; }

// how the slice-pair products of a block are summed (values of the accum_mode / sum_rule arguments)
constexpr int ACC_HW = 0, ACC_EMU = 1, ACC_EXACT = 2;
constexpr int SUM_RUNS = 0, SUM_PLAIN = 1;

// "exact" accumulation: the block sum of an element is a 192-bit two's-complement integer in units of
// 2^(cA_1 + cB_1 - 2b - EXACT_WINDOW_BITS); at most 1024 terms of at most 2^36 units * 2^EXACT_WINDOW_BITS each.
constexpr int EXACT_WINDOW_BITS = 144;
constexpr int SUM_WORDS_MAX = 3;          // 64-bit words of a running block sum kept in work memory between passes

// ---- slice storage ---------------------------------------------------------------------------------------
// One slice matrix (block t, slice p) of an operand is stored as [chunk kc][vector r][CHUNK_BYTES]:
// the 256 vectors a workgroup stages for one pipeline step are 16 KiB of contiguous memory.  The number
// of vectors is padded to a multiple of TILE and every block to whole chunks; the padding holds zero
// codes, which contribute exact zeros to every product.
//
// FP6: a chunk holds 64 inner indices of every vector as 6-bit codes.  The matrix unit wants the 32 codes of a
// vector's k-group g (inner indices 32g .. 32g+31 of the chunk) as one 192-bit little-endian string (code i at
// bits 6i .. 6i+5).  A chunk stores the first 16 bytes and the last 8 bytes of these strings in four planes,
//     [g = 0: rows_pad x 16 B][g = 1: rows_pad x 16 B][g = 0: rows_pad x 8 B][g = 1: rows_pad x 8 B]
// (rows_pad x 48 bytes in all), so that the part of a plane that belongs to a 256-vector tile is contiguous and a
// wave's fragment reads from the staged copy are contiguous, bank-conflict-free 128- and 64-bit accesses.
struct Operand {
    int64_t rows;         // real vectors: m for A (its rows), n for B (its columns)
    int64_t rows_pad;     // multiple of TILE
    uint8_t* slices;      // [T][s][chunks][rows_pad][row_bytes]
    int32_t* exps;        // [T][s][rows_pad]   exponent c of Eq. 4 (0 for padding vectors)
    int32_t* deltas;      // [T][s][rows_pad/LINK_ROWS]  per slice p and group of 32 vectors (one matrix-unit tile edge):
                          //                        c_p - c_(p+1) if that difference is the same for all real vectors of
                          //                        the group, else DELTA_IRREGULAR (always for the last slice)
};

constexpr int LINK_ROWS = 32;             // granularity of the equal-scale decision: one 32 x 32 matrix-unit tile

constexpr int DELTA_IRREGULAR = -2147483647 - 1;

struct Plan {
    int64_t m, n, k;
    int fmt;              // FMT_FP8, FMT_FP16, FMT_FP6, FMT_FP6_E3M2
    int epc;              // inner indices per chunk: 64 (FP8, FP6) or 32 (FP16)
    int row_bytes;        // bytes of one vector in one chunk: 64 (FP8, FP16) or 48 (FP6)
    int p_frac;           // a stored pair product is an integer multiple of 2^-p_frac: 2b, for FP6 (whose codes hold
                          // twice the slice value) 2b - 2; the true product is the stored one times 2^(p_frac - 2b)
    int s;                // slices per operand
    int b;                // magnitude bits of a slice entry (53 - rho)
    int rho;
    int64_t kb;           // block length (elements)
    int64_t T;            // number of blocks
    int64_t chunks;       // chunks per block
    int full;             // 1: all s*s pairs, 0: the pairs with p + q <= s + 1
    int npairs;           // s(s+1)/2 or s*s
    int run_limit;        // floor(window / (kb * 4^b)): equal-scale pair products that may be summed exactly in the
                          // matrix unit's accumulators (window 2^24 for FP32, 2^31 - 1 for INT32)
    int group_len;        // pairs per group of the GEMM kernel, <= run_limit (PairOrder::run_limit of the launches)
    int64_t tiles_m, tiles_n;
    int64_t m_pad, n_pad;
    int p_is_int;         // 1: the stored products are INT32 words (INT8 slices), 0: FP32
};

// The slice pairs (p, q), 1-based, and their accumulation order: anti-diagonals g = p + q from the least
// significant (largest g) down to g = 2, p ascending inside one.  Triangle mode uses the pairs with p + q <= s + 1,
// full mode all s * s.  Consecutive pairs of an anti-diagonal with equal scale are summed exactly before the FP64
// addition; the matrix unit can do that for as many pairs as fit the exact FP32 window (Plan::run_limit), so every
// anti-diagonal is cut into groups of at most run_limit consecutive pairs (Plan::group_len, never more than the
// window), the unit of work of the GEMM kernel; pairs are numbered z = 0, 1, ... in this order.  Everything below
// is a closed form of (s, full, run_limit), evaluated on the host and in the kernels.
struct PairOrder {
    int s;
    int full;
    int run_limit;        // pairs per group
};
__host__ __device__ inline int order_top_diag(const PairOrder& o) { return o.full ? 2 * o.s : o.s + 1; }
__host__ __device__ inline int diag_first_p(const PairOrder& o, int g) { return g - o.s > 1 ? g - o.s : 1; }
__host__ __device__ inline int diag_len(const PairOrder& o, int g) {
    const int hi = g - 1 < o.s ? g - 1 : o.s;
    return hi - diag_first_p(o, g) + 1;
}
__host__ __device__ inline int diag_groups(const PairOrder& o, int g) { return (diag_len(o, g) + o.run_limit - 1) / o.run_limit; }
__host__ __device__ inline int order_num_groups(const PairOrder& o) {
    int n = 0;
    for (int g = order_top_diag(o); g >= 2; --g) n += diag_groups(o, g);
    return n;
}
__host__ __device__ inline int order_num_pairs(const PairOrder& o) { return o.full ? o.s * o.s : o.s * (o.s + 1) / 2; }

// A pass of the accumulation: the anti-diagonals g_hi, g_hi - 1, ..., g_lo; its pair products occupy the slots
// 0 .. npairs-1 of the product buffer in pair order.
struct Pass {
    int g_hi, g_lo;
    int npairs, ngroups;
};

// The gi-th group of a pass: slices (p0 + j, q0 - j), j < len (1-based), first product slot `slot`.
struct Group {
    int p0, q0, len, slot;
};
__host__ __device__ inline Group pass_group(const PairOrder& o, const Pass& ps, int gi) {
    int slot = 0;
    for (int g = ps.g_hi; g >= ps.g_lo; --g) {
        const int len = diag_len(o, g), ng = (len + o.run_limit - 1) / o.run_limit;
        if (gi < ng) {
            const int pos = gi * o.run_limit;
            Group r;
            r.p0 = diag_first_p(o, g) + pos;
            r.q0 = g - r.p0;
            r.len = len - pos < o.run_limit ? len - pos : o.run_limit;
            r.slot = slot + pos;
            return r;
        }
        gi -= ng;
        slot += len;
    }
    return Group{1, 1, 0, 0};
}

// True if, for every element of a 32 x 32 tile, pair (p+1, q-1) carries the same scale factor 2^(cA + cB) as pair
// (p, q) (0-based slice indices): then the two products can be summed in the accumulator of the matrix unit
// (a group has at most run_limit pairs, so the sum stays inside the exact window).  a: the delta of slice p of the
// tile's 32 rows of A, b: the delta of slice q - 1 of its 32 columns of B.
__host__ __device__ inline bool deltas_link(int a, int b) { return a != DELTA_IRREGULAR && a == b; }
// dA / dB: Operand::deltas of the block, advanced to the tile's group of rows of A / columns of B; ga / gb: groups per
// slice (rows_pad / LINK_ROWS) of the two operands.
__host__ __device__ inline bool pair_linked(const int32_t* dA, int64_t ga, const int32_t* dB, int64_t gb, int p, int q) {
    return deltas_link(dA[p * ga], dB[(q - 1) * gb]);
}

// ---- pair-product storage ("accumulator order") ------------------------------------------------------------
// The FP32 product of one pair is stored tile by tile, [tile_n][tile_m][TILE_ELEMS], and inside a tile in
// the order the matrix unit leaves it in the registers of the workgroup's four waves:
//     float index = ((((wave*16 + sub)*4 + a)*64 + lane)*4 + r
//     wave = wn*2 + wm (wn, wm in {0,1});  sub = ti*4 + tj (ti, tj in 0..3)
//     column of C (n) = tile_n*256 + wn*128 + ti*32 + a*8 + (lane/32)*4 + r
//     row    of C (m) = tile_m*256 + wm*128 + tj*32 + lane%32
// Every wave-wide store / load of this buffer is one contiguous kilobyte.
__host__ __device__ inline void acc_order_to_mn(int idx, int& m_in_tile, int& n_in_tile) {
    int r = idx & 3, lane = (idx >> 2) & 63, a = (idx >> 8) & 3, sub = (idx >> 10) & 15, wave = idx >> 14;
    int ti = sub >> 2, tj = sub & 3, wn = wave >> 1, wm = wave & 1;
    n_in_tile = wn * 128 + ti * 32 + a * 8 + (lane >> 5) * 4 + r;
    m_in_tile = wm * 128 + tj * 32 + (lane & 31);
}

// ---- launchers (each enqueues on `st` and returns the launch status) ----------------------------------------
hipError_t launch_transpose(const double* A, int64_t lda, int64_t m, int64_t k, double* At, hipStream_t st);

// Vectors are contiguous: vector r of an operand starts at X + r*ldv and has k entries.  Writes the internal layout of
// up to two operands in one launch (a null Operand, or one without vectors, is skipped).  Blocks longer than
// MAX_K_BLOCK_IN_REGISTERS are sliced by a streaming kernel that keeps its per-element state in `long_state`
// (split_state_bytes(pl) bytes; may be null otherwise).
hipError_t launch_split(const double* X0, int64_t ldv0, const Operand* op0, const double* X1, int64_t ldv1, const Operand* op1,
                        const Plan& pl, int* flags, void* long_state, hipStream_t st);
size_t split_state_bytes(const Plan& pl, int64_t rows_a, int64_t rows_b);

// Slices until every remainder is zero (paragraph before Eq. 4): atomicMax of the per-vector count into flags[1]
// (which the caller has cleared); MAX_SLICES + 1 means that MAX_SLICES slices do not exhaust some vector.
hipError_t launch_count_slices(const double* X, int64_t ldv, const Plan& pl, int64_t rows, int* flags, void* long_state, hipStream_t st);

// Internal layout -> plain vector-major codes (verification export).
hipError_t launch_export_slices(const Plan& pl, const Operand& op, void* out, hipStream_t st);

// Fills Operand::deltas from Operand::exps, for up to two operands in one launch.
hipError_t launch_deltas(const Plan& pl, const Operand* op0, const Operand* op1, hipStream_t st);

// Products of the pairs of pass `ps` of block t into P ([ps.npairs][tiles_n][tiles_m][TILE_ELEMS] floats).  With
// allow_chain, consecutive pairs of a group that are linked for a tile (pair_linked) form a run whose exact sum is
// stored in the slot of the run's first pair; the slots of the other pairs of the run are left untouched.
hipError_t launch_pair_gemm(const Plan& pl, const Operand& A, const Operand& B, const PairOrder& order, const Pass& ps,
                            bool allow_chain, int64_t t, float* P, hipStream_t st);

// Accumulate the pairs of pass `ps` of block t.  S_io: running block sum in accumulator order (read unless the
// pass is the block's first, written unless it is the last): one 64-bit word per element (FP64 bits), three in the
// exact mode, word w of element e at S_io[w * tiles * TILE_ELEMS + e].  On the last pass the block sum is rescaled by
// the first-slice exponents and stored to C (t == 0) or added to C (t > 0).  `chained`: the products were written
// with allow_chain.  sum_rule SUM_PLAIN: every product is added on its own.
hipError_t launch_accumulate(const Plan& pl, const Operand& A, const Operand& B, const PairOrder& order, const Pass& ps,
                             bool first_pass, bool last_pass, int64_t t, const float* P, uint64_t* S_io,
                             double* C, int64_t ldc, int accum_mode, int sum_rule, bool chained, hipStream_t st);

// P in accumulator order -> [nz][n][m] column-major matrices (verification export): FP32 values of Eq. 10-11, or INT32
// integers for INT8 slices.  run_len_out (may be null): for every element and pair slot of the pass, how many pairs'
// products the slot holds summed (1 without chaining; 0: the pair's product is part of an earlier slot's sum, and
// `out` gets 0 there).
hipError_t launch_export_products(const Plan& pl, const Operand& A, const Operand& B, const PairOrder& order, const Pass& ps,
                                  bool chained, int64_t t, const float* P, float* out, uint8_t* run_len_out, hipStream_t st);

// C = alpha * W + beta * C element by element (one rounding per operation, no fused multiply-add; beta == 0: C is not
// read), W and C column-major m x n.
hipError_t launch_axpby(double alpha, double beta, const double* W, int64_t ldw, double* C, int64_t ldc, int64_t m, int64_t n,
                        int accum_mode, hipStream_t st);

hipError_t launch_add_emulated(const double* a, const double* b, double* out, int64_t n, hipStream_t st);
hipError_t launch_fill_zero_f64(double* C, int64_t ldc, int64_t m, int64_t n, hipStream_t st);

}  // namespace ozaki
