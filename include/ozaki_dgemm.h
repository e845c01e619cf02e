/*
 * ozaki_dgemm.h -- C ABI of the MI355X (gfx950) Ozaki-scheme DGEMM library, libozaki.so.
 *
 * The library computes C = A B for FP64 matrices without any FP64 multiply-add in the product,
 * following "DGEMM without FP64 Arithmetic -- Using FP64 Emulation and FP8 Tensor Cores with
 * Ozaki Scheme" (D. Mukunoki): Section 3 (slicing, Eq. 1-8; error-free product expansion,
 * Eq. 9-11), Section 4.1 (FP8 E4M3 and FP16 slices with FP32 accumulation), Section 4.2 (FP64
 * addition emulated with integer instructions) and Section 4.3 (inner-product-wise and
 * outer-product-wise blocking).
 *
 * Conventions common to all entry points
 *   - One GPU, the current HIP device.  Every pointer documented as DEVICE must be device memory
 *     of that GPU; pointers documented as HOST are ordinary host memory.  The library never takes
 *     ownership of caller memory and never frees it.
 *   - Matrices are column-major (BLAS convention): element (i, j) of A is A[i + j*lda].
 *   - State (stream, workspace, profiling, last error) lives in a context.  Every host thread has a
 *     current context, initially the library's built-in default context; ozaki_context_use selects
 *     another one.  All calls below act on the calling thread's current context.  Two contexts with
 *     their own streams and workspaces are independent: their calls may be issued from two host
 *     threads, or interleaved from one, and run concurrently on the GPU.  One context is not
 *     thread-safe: one host thread drives it at a time, and two calls that share a workspace must
 *     be ordered on the same stream.
 *   - Work is enqueued on the context's stream (default: the null stream) and the calls return
 *     without waiting for the GPU unless stated otherwise.
 *   - Return value: 0 on success; a negative value -N means argument number N (1-based, in the
 *     order of the prototype) is invalid and nothing was launched; a positive value is one of the
 *     OZAKI_STATUS_* codes below.
 */
#ifndef OZAKI_DGEMM_H
#define OZAKI_DGEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Type2 of the paper (Section 3): storage format of the slices = input format of the matrix unit. */
enum {
    OZAKI_SLICE_FP8_E4M3 = 0, /* OCP E4M3, 4 significand bits, FP32 accumulation (Section 4.1)        */
    OZAKI_SLICE_FP16 = 1,     /* IEEE binary16, 11 significand bits, FP32 accumulation (Section 4.1)  */
    OZAKI_SLICE_FP6_E2M3 = 2, /* OCP microscaling FP6 E2M3 (bias 1, no Inf/NaN): the 4 significand bits */
                              /* of E4M3, so the same slices and the same C as OZAKI_SLICE_FP8_E4M3,    */
                              /* on the twice as fast FP6 path of the matrix unit that Section 4.1      */
                              /* points to.  E2M3's smallest step is 1/8: a code holds twice the value  */
                              /* of Eq. 8, and the factor 1/4 per product is applied with the exponents */
    OZAKI_SLICE_FP6_E3M2 = 3, /* OCP microscaling FP6 E3M2 (bias 3), 3 significand bits: the FP6 column of    */
                              /* Table 2 (14 slices for a full FP64 significand); same FP6 matrix path        */
    OZAKI_SLICE_INT8 = 4      /* comparison path (the integer-matrix-unit variant of the scheme that Section 2 */
                              /* cites): slice entries are the integers q of Eq. 5-8 with |q| <= 2^6 stored as */
                              /* two's-complement bytes, products accumulate in INT32 (exact while             */
                              /* k_block * 4^b <= 2^31 - 1, which keeps b = 6 up to k_block = 524287)          */
};

/* How the slice-pair products are summed into FP64 (Section 3 after Eq. 11; Section 4.2). */
enum {
    OZAKI_ACCUM_FP64_HW = 0,      /* hardware FP64 additions                                            */
    OZAKI_ACCUM_FP64_INT_EMU = 1, /* FP64 additions emulated with 32/64-bit integer instructions only,  */
                                  /* round-to-nearest-even, bitwise equal to the hardware result        */
    OZAKI_ACCUM_EXACT_FIXED = 2   /* integer-only as well: the terms of a block are summed without any  */
                                  /* rounding in a 192-bit fixed-point integer per element (the sum of  */
                                  /* Eq. 10 free of rounding error, remark after Eq. 11) and rounded   */
                                  /* to FP64 once.  Unit: 2^-144 of the unit of the leading pair's      */
                                  /* product; a term whose scale lies further down is cut to that unit  */
                                  /* towards minus infinity.  Block sums are added to C with the        */
                                  /* emulated FP64 addition.  Not bitwise equal to the other two modes  */
                                  /* (fewer roundings).                                                 */
};

/* Which slice pairs (p, q) are multiplied. */
enum {
    OZAKI_PAIRS_TRIANGLE = 0, /* p + q <= s + 1: s(s+1)/2 products (terms below the last slice's weight are dropped)  */
    OZAKI_PAIRS_ALL = 1       /* all s * s products: the setting of the paper's Table 2 and Section 5.3              */
};

/* Where the FP64 roundings of the block sum happen (OZAKI_ACCUM_FP64_HW and _INT_EMU; Section 4 tunes the order of
 * the accumulation without giving it).  Either way the terms are visited anti-diagonal by anti-diagonal, p + q from
 * the largest (least significant) down to 2, p ascending inside one. */
enum {
    OZAKI_SUM_RUNS = 0,       /* consecutive terms of one anti-diagonal that carry the same power-of-two scale for an    */
                              /* element are summed exactly (matrix-unit accumulators, integer registers) and added      */
                              /* with ONE rounded FP64 addition: fewer roundings, less product traffic                   */
    OZAKI_SUM_PLAIN = 1       /* every term 2^(cA+cB) * product of Eq. 10 is added with its own rounded FP64 addition    */
};

enum {
    OZAKI_STATUS_OK = 0,
    OZAKI_STATUS_INFEASIBLE = 1,   /* no slice width b >= 0 keeps the accumulation of the matrix unit exact for this   */
                                   /* block length (condition after Eq. 8: k_block * 4^0 exceeds the exact window)      */
    OZAKI_STATUS_WORKSPACE = 3,    /* no workspace set, or it is smaller than ozaki_workspace_min_bytes    */
    OZAKI_STATUS_HIP_ERROR = 4,    /* a HIP runtime call failed; see ozaki_last_hip_error                  */
    OZAKI_STATUS_NONFINITE = 5,    /* reported by ozaki_last_device_status: A or B held an Inf or NaN      */
    OZAKI_STATUS_STATIC_LIMIT = 6, /* ozaki_dgemm_static: the problem needs more than OZAKI_STATIC_SCRATCH_BYTES */
    OZAKI_STATUS_SLICE_COUNT = 7   /* num_slices is larger than OZAKI_MAX_SLICES                           */
};

#define OZAKI_MAX_SLICES 32

/* ------------------------------------------------------------------------------------------------
 * Contexts
 * ---------------------------------------------------------------------------------------------- */
typedef struct ozaki_context_s* ozaki_context_t;

/* Creates a context (stream: null stream, no workspace, profiling off).  ctx_out: HOST. */
int ozaki_context_create(ozaki_context_t* ctx_out);
/* Destroys a context created by ozaki_context_create (releases its HIP events; never the caller's stream or
 * workspace).  If it is the calling thread's current context, the thread falls back to the default context.  It
 * must not be current in another thread, and its GPU work should have completed. */
int ozaki_context_destroy(ozaki_context_t ctx);
/* Makes ctx the calling host thread's current context; NULL selects the built-in default context. */
int ozaki_context_use(ozaki_context_t ctx);

/* Stream (a hipStream_t passed as void*; NULL = the null stream) used by all later calls of the current context. */
int ozaki_set_stream(void* hip_stream);

/*
 * ozaki_plan (host only, touches no GPU) -- the constants of Eq. 1-3 for one block length.
 *   k_block       length of the inner-product block the scheme is applied to (Section 4.3); >= 1
 *   slice_format  OZAKI_SLICE_*
 *   rho_out       HOST, may be NULL: rho = max(gamma, xi) of Eq. 3 with Type1 = FP64, Type3 = FP32 (INT32 for
 *                 OZAKI_SLICE_INT8)
 *   bits_out      HOST, may be NULL: b = 53 - rho, the magnitude bits of a slice entry: every entry is
 *                 q * 2^-b with integer |q| <= 2^b, and k_block * 4^b <= 2^24 keeps Eq. 11 exact
 * Returns 0, -1/-2 for invalid arguments, or OZAKI_STATUS_INFEASIBLE when rho > 53.
 */
int ozaki_plan(int64_t k_block, int slice_format, int* rho_out, int* bits_out);

/*
 * ozaki_dgemm -- C := A B by the Ozaki scheme (Section 3; blocking of Section 4.3).
 *   m, n, k       A is m x k, B is k x n, C is m x n; any non-negative sizes (internally zero-padded to
 *                 the tile sizes, which is exact).  m == 0 or n == 0: nothing is done.  k == 0: C := 0.
 *   A, lda        DEVICE, read-only, column-major, lda >= max(1, m)
 *   B, ldb        DEVICE, read-only, column-major, ldb >= max(1, k)
 *   C, ldc        DEVICE, written (every entry of the m x n matrix is overwritten), ldc >= max(1, m);
 *                 must not overlap A, B or the workspace
 *   slice_format  OZAKI_SLICE_*
 *   num_slices    s >= 1: number of slices taken from every row of A and every column of B (Eq. 4-8);
 *                 the slice pairs (p, q) with p + q <= s + 1 are multiplied (OZAKI_PAIRS_TRIANGLE) and summed
 *                 by the rule OZAKI_SUM_RUNS.  0 selects a data-independent default (ceil(61 / (b+1)) slices).
 *                 More than OZAKI_MAX_SLICES: OZAKI_STATUS_SLICE_COUNT.
 *   k_block       inner-product-wise block length (Section 4.3); 0 means k (no blocking).  A last,
 *                 shorter block is allowed.  Any length for which Eq. 1-3 leave b >= 0 is accepted; blocks of
 *                 more than 16384 elements are sliced by a slower streaming kernel that needs 12 more bytes
 *                 of workspace per operand element (included in ozaki_workspace_bytes).
 *   accum_mode    OZAKI_ACCUM_*
 * The slices, exponents and slice-pair products live in the workspace (ozaki_set_workspace).
 * Inputs must be finite; an Inf/NaN raises a device flag readable with ozaki_last_device_status
 * and leaves C unspecified.  Results whose exponent leaves the normal FP64 range are unspecified in
 * the integer-only modes (the emulation omits overflow, underflow and subnormals, Section 4.2).
 */
int ozaki_dgemm(int64_t m, int64_t n, int64_t k,
                const double* A, int64_t lda, const double* B, int64_t ldb,
                double* C, int64_t ldc,
                int slice_format, int num_slices, int64_t k_block, int accum_mode);

/*
 * ozaki_dgemm_ex -- ozaki_dgemm with the pair set and the summation rule as arguments of their own.
 *   pair_set      OZAKI_PAIRS_*.  OZAKI_PAIRS_ALL with num_slices = the count of ozaki_count_slices is the paper's
 *                 error-free setting: the products then sum to the exact product (Eq. 9-10).
 *   sum_rule      OZAKI_SUM_* (ignored by OZAKI_ACCUM_EXACT_FIXED, whose sum has no intermediate rounding)
 *   mem_cap       0, or a cap in bytes on the part of the workspace the call may use: the call then works on
 *                 panels of rows of A and columns of B small enough for the cap (outer-product-wise blocking,
 *                 Section 4.3) and gives the same bits as the uncapped call, since rows of A and columns of B are
 *                 sliced independently of each other.  A cap below the need of one 256 x 256 panel:
 *                 OZAKI_STATUS_WORKSPACE.
 * ozaki_dgemm(...) is ozaki_dgemm_ex(..., OZAKI_PAIRS_TRIANGLE, OZAKI_SUM_RUNS, 0).
 */
int ozaki_dgemm_ex(int64_t m, int64_t n, int64_t k,
                   const double* A, int64_t lda, const double* B, int64_t ldb,
                   double* C, int64_t ldc,
                   int slice_format, int num_slices, int64_t k_block, int accum_mode,
                   int pair_set, int sum_rule, size_t mem_cap);

/*
 * ozaki_dgemm_static -- ozaki_dgemm for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * the same bits in C as ozaki_dgemm, but the slices, exponents and slice-pair products live in a fixed array of
 * OZAKI_STATIC_SCRATCH_BYTES bytes that is part of the library's device code (every GPU the library runs on holds
 * one copy from the first call until the process ends); the workspace of ozaki_set_workspace is neither needed nor
 * touched, and the call allocates and frees nothing.
 *   Limit: ozaki_workspace_min_bytes(m, n, k, slice_format, num_slices, k_block) must not exceed
 *   OZAKI_STATIC_SCRATCH_BYTES, else OZAKI_STATUS_STATIC_LIMIT is returned and nothing is launched (m = n = k = 256
 *   with 12 FP8 slices fits several times over, m = n = 600, k = 1000 with 11 slices just fits, m = n = k = 2048
 *   does not).
 *   Every call on a GPU uses that GPU's one array, which keeps what the previous call left: the kernels overwrite
 *   all they read, so nothing needs clearing between calls, but two calls that overlap in time on one GPU (two
 *   streams, two contexts, two host threads) race on it and give undefined results.  Enqueued on the current
 *   context's stream.  An Inf/NaN input is reported by ozaki_last_device_status as for ozaki_dgemm.
 */
#define OZAKI_STATIC_SCRATCH_BYTES (64u << 20)
int ozaki_dgemm_static(int64_t m, int64_t n, int64_t k,
                       const double* A, int64_t lda, const double* B, int64_t ldb,
                       double* C, int64_t ldc,
                       int slice_format, int num_slices, int64_t k_block, int accum_mode);

/*
 * ozaki_dgemm_scaled -- C := alpha (A B) + beta C, the GEMM of the BLAS that the paper emulates (Section 1), with
 * the FP64 multiplication of Section 4.2 beside the addition.
 *   alpha, beta   HOST values; zeros or normal numbers.
 *   The product P = A B is formed exactly as by ozaki_dgemm (same arguments, same bits), then every entry is
 *   combined as  C = fl(fl(alpha * P) + fl(beta * C))  -- one rounded multiplication per term and one rounded
 *   addition, no fused multiply-add; with beta == 0, C = fl(alpha * P) and the old C is not read (it may hold
 *   anything); with alpha == 1 and beta == 0 the call is ozaki_dgemm.  In the integer-only modes the
 *   multiplications and the addition are integer-only too (same bits; the old C must then hold zeros or
 *   normal numbers).  All other arguments as for ozaki_dgemm.
 *   The workspace must have ozaki_workspace_bytes_scaled bytes (ozaki_workspace_bytes plus the m x n product),
 *   or at least ozaki_workspace_min_bytes plus 8 m n rounded up to 256.
 * Returns as ozaki_dgemm; negative values count positions in THIS argument list.
 */
int ozaki_dgemm_scaled(int64_t m, int64_t n, int64_t k, double alpha,
                       const double* A, int64_t lda, const double* B, int64_t ldb,
                       double beta, double* C, int64_t ldc,
                       int slice_format, int num_slices, int64_t k_block, int accum_mode);
size_t ozaki_workspace_bytes_scaled(int64_t m, int64_t n, int64_t k, int slice_format, int num_slices, int64_t k_block);

/*
 * ozaki_suggest_k_block -- a block length for the inner dimension k (Section 4.3 leaves the choice to the user).
 * A heuristic from measurements on MI355X, not part of the method: FP8 / FP6 slices keep b = 4 up to k = 65536, so
 * they are blocked only above that (into blocks of 16384, the longest the fast slicing kernel takes); FP16 gains a
 * magnitude bit per factor 4 in the block length, and 4096 (b = 6) was the fastest block at k = 16384 (the paper
 * reports the same optimum on its GPU); INT8 keeps b = 6 up to 524287.  Returns the suggested k_block (0 = no
 * blocking), or a negative argument index.  HOST call.
 */
int64_t ozaki_suggest_k_block(int64_t k, int slice_format);

/*
 * Workspace (Section 5.1: work memory is allocated once, outside the timed region).
 *   ozaki_workspace_bytes      size that lets ozaki_dgemm keep all s(s+1)/2 pair products of one block
 *                              resident (capped at 160 GiB of products; more pairs are then processed in
 *                              several passes).  0 if the arguments are invalid or infeasible.
 *   ozaki_workspace_min_bytes  smallest size ozaki_dgemm accepts (the s products of the longest anti-diagonal
 *                              resident at a time).
 *   ozaki_workspace_bytes_ex   either of the two (minimum != 0: the smallest) for a pair set OZAKI_PAIRS_*.
 *   ozaki_set_workspace        dev_ptr: DEVICE memory, 256-byte aligned, owned by the caller, must stay
 *                              valid until replaced; bytes: its size.  (NULL, 0) clears it.
 */
size_t ozaki_workspace_bytes(int64_t m, int64_t n, int64_t k, int slice_format, int num_slices, int64_t k_block);
size_t ozaki_workspace_min_bytes(int64_t m, int64_t n, int64_t k, int slice_format, int num_slices, int64_t k_block);
size_t ozaki_workspace_bytes_ex(int64_t m, int64_t n, int64_t k, int slice_format, int num_slices, int64_t k_block,
                                int pair_set, int minimum);
int ozaki_set_workspace(void* dev_ptr, size_t bytes);

/* Waits for the stream, then returns OZAKI_STATUS_NONFINITE if a kernel since the last call of this
 * function met an Inf/NaN input, OZAKI_STATUS_HIP_ERROR on a HIP failure, else 0. */
int ozaki_last_device_status(void);
/* Numeric hipError_t of the most recent failed HIP call of the current context (0 if none). */
int ozaki_last_hip_error(void);
/* Static, NUL-terminated description of a return value of this library. */
const char* ozaki_status_string(int status);

/*
 * Per-phase GPU time.  ozaki_profile_enable(1) makes ozaki_dgemm bracket its kernels with HIP events
 * on the context's stream; ozaki_profile_read waits for the stream and returns, in HOST arrays of three
 * floats / three ints, the accumulated milliseconds and the number of kernel launches of the phases
 * [0] slicing (Eq. 4-8, includes the transposition of A), [1] slice-pair GEMMs (Eq. 10-11),
 * [2] accumulation and rescaling; then resets the counters.  ozaki_profile_enable(0) turns it off.
 * At most 4096 spans are kept between two reads (later ones are dropped), and nothing is recorded while the
 * stream is being captured into a HIP graph.
 */
int ozaki_profile_enable(int on);
int ozaki_profile_read(float* ms_out, int* launches_out);

/* ------------------------------------------------------------------------------------------------
 * Verification exports: the intermediate results the method defines, in plain layouts, for parity
 * checks against a reference implementation.  Not meant for timed use.  They use the workspace.
 * ---------------------------------------------------------------------------------------------- */

/*
 * ozaki_split -- Eq. 4-8 for one operand.
 *   is_B        0: X is A (rows x k, the vectors are the rows of A, ldx >= rows);
 *               1: X is B (k x rows, the vectors are the columns of B, ldx >= k)
 *   rows, k     number of vectors and their length
 *   X, ldx      DEVICE, column-major
 *   slices_out  DEVICE: T*s matrices in the order [block t][slice p], each `rows` vectors of
 *               kb_t = min(k_block, k - t*k_block) entries, vector-major (entry kk of vector r at
 *               r*kb_t + kk); 1 byte per entry (E4M3 code, E2M3 / E3M2 code in the low six bits, or the INT8
 *               integer) or 2 bytes (binary16 bits).  Blocks are packed back to back (block t starts after
 *               s*rows*kb_u entries of every earlier block u).
 *   exps_out    DEVICE: int32 [T][s][rows], the exponents c of Eq. 4 (32-bit for alignment's sake; every
 *               value fits 16 bits)
 */
int ozaki_split(int is_B, int64_t rows, int64_t k, const double* X, int64_t ldx,
                int slice_format, int num_slices, int64_t k_block,
                void* slices_out, int32_t* exps_out);

/*
 * ozaki_count_slices -- how many slices Eq. 4-8 extract from an operand until its remainder is zero (Section 3, the
 * paragraph before Eq. 4): the largest count over its vectors and k-blocks.  With that many slices (the larger
 * of the two operands' counts) and OZAKI_PAIRS_ALL the sum of the pair products is the exact product, which is
 * the error-free setting of the paper.
 *   is_B, rows, k, X, ldx, slice_format, k_block   as for ozaki_split
 *   count_out   HOST: the count; 0 for an all-zero operand; OZAKI_MAX_SLICES + 1 if OZAKI_MAX_SLICES slices do
 *               not exhaust it (ozaki_dgemm cannot run the error-free setting on it then)
 * Synchronises with the stream.  Workspace: 256 bytes, plus 8 * rows * k bytes (rounded up to 256) for A, plus 12
 * bytes per element of the (64-element padded) operand when the block is longer than 16384.
 */
int ozaki_count_slices(int is_B, int64_t rows, int64_t k, const double* X, int64_t ldx,
                       int slice_format, int64_t k_block, int* count_out);

/*
 * ozaki_pair_products -- the slice-pair products of Eq. 10-11, as the matrix unit produced them.
 *   pair_set    OZAKI_PAIRS_*
 *   chained     0: every pair is multiplied on its own (the kernel's run formation is switched off).
 *               1: the launch configuration of ozaki_dgemm with OZAKI_SUM_RUNS: where all elements of a 32 x 32
 *               tile share the scale of consecutive pairs of an anti-diagonal, the matrix unit keeps accumulating
 *               and ONE slot receives the exact sum of the run.
 *   P_out       DEVICE: [T][pairs][n][m] 4-byte words: for block t and pair index z (pairs in accumulation order:
 *               anti-diagonals g = p+q from the largest down to 2, p ascending within one), an m x n column-major
 *               matrix (leading dimension m).  FP32 value sum_kk sliceA_p(i,kk) * sliceB_q(kk,j), the slices being
 *               the values of Eq. 8 (for FP6 the matrix unit's result times the exact factor 1/4); for
 *               OZAKI_SLICE_INT8 the INT32 integer sum_kk qA qB.  With chained != 0 the slot of a run's first pair
 *               holds the sum over the run and the other slots of the run hold 0.
 *   run_len_out DEVICE, may be NULL: uint8 [T][pairs][n][m]: how many consecutive pairs (starting with this one) the
 *               value in P_out sums; 0 where the pair is part of an earlier pair's run.  All 1 with chained == 0.
 */
int ozaki_pair_products(int64_t m, int64_t n, int64_t k,
                        const double* A, int64_t lda, const double* B, int64_t ldb,
                        int slice_format, int num_slices, int64_t k_block,
                        int pair_set, int chained, void* P_out, uint8_t* run_len_out);

/*
 * ozaki_fp64_add_emulated -- out[i] = a[i] + b[i] with the integer-only FP64 addition used by
 * OZAKI_ACCUM_FP64_INT_EMU (Section 4.2).  a, b, out: DEVICE arrays of n doubles (zeros and normal
 * numbers; out may alias a or b).
 */
int ozaki_fp64_add_emulated(const double* a, const double* b, double* out, int64_t n);

#ifdef __cplusplus
}
#endif
#endif /* OZAKI_DGEMM_H */
