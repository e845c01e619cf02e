/*
 * ozaki_dgemm.h -- C ABI of the MI355X (gfx950) Ozaki-scheme DGEMM library, libozaki.so.
 *
 * The library computes C = A B for FP64 matrices without any FP64 multiply-add in the product,
 * following "DGEMM without FP64 Arithmetic -- Using FP64 Emulation and FP8 Tensor Cores with
 * Ozaki Scheme" (D. Mukunoki): Section 3 (slicing, Eq. 1-8; error-free product expansion,
 * Eq. 9-11), Section 4.1 (FP8 E4M3 and FP16 slices with FP32 accumulation), Section 4.2 (FP64
 * addition emulated with integer instructions) and Section 4.3 (inner-product-wise blocking).
 *
 * Conventions common to all entry points
 *   - One GPU, the current HIP device.  Every pointer documented as DEVICE must be device memory
 *     of that GPU; pointers documented as HOST are ordinary host memory.  The library never takes
 *     ownership of caller memory and never frees it.
 *   - Matrices are column-major (BLAS convention): element (i, j) of A is A[i + j*lda].
 *   - Work is enqueued on the stream given to ozaki_set_stream (default: the null stream) and the
 *     calls return without waiting for the GPU unless stated otherwise.
 *   - Return value: 0 on success; a negative value -N means argument number N (1-based, in the
 *     order of the prototype) is invalid and nothing was launched; a positive value is one of the
 *     OZAKI_STATUS_* codes below.
 *   - Not thread-safe: one host thread drives the library at a time.  Two calls that share the
 *     workspace must be ordered on the same stream.
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
    OZAKI_SLICE_FP6_E3M2 = 3  /* OCP microscaling FP6 E3M2 (bias 3), 3 significand bits: the FP6 column of    */
                              /* Table 2 (14 slices for a full FP64 significand); same FP6 matrix path        */
};

/* How the slice-pair products are summed into FP64 (Section 3 after Eq. 11; Section 4.2). */
enum {
    OZAKI_ACCUM_FP64_HW = 0,     /* hardware FP64 additions                                            */
    OZAKI_ACCUM_FP64_INT_EMU = 1 /* FP64 additions emulated with 32/64-bit integer instructions only,  */
                                 /* round-to-nearest-even, bitwise equal to the hardware result        */
};

enum {
    OZAKI_STATUS_OK = 0,
    OZAKI_STATUS_INFEASIBLE = 1,   /* no slice width b >= 0 keeps the FP32 accumulation exact (condition   */
                                   /* after Eq. 8), or num_slices outside [1, OZAKI_MAX_SLICES], or the    */
                                   /* block length exceeds OZAKI_MAX_K_BLOCK                               */
    OZAKI_STATUS_WORKSPACE = 3,    /* no workspace set, or it is smaller than ozaki_workspace_min_bytes    */
    OZAKI_STATUS_HIP_ERROR = 4,    /* a HIP runtime call failed; see ozaki_last_hip_error                  */
    OZAKI_STATUS_NONFINITE = 5,    /* reported by ozaki_last_device_status: A or B held an Inf or NaN      */
    OZAKI_STATUS_STATIC_LIMIT = 6  /* ozaki_dgemm_static: the problem needs more than OZAKI_STATIC_SCRATCH_BYTES */
};

/* OR-ed into a num_slices argument: multiply all s*s slice pairs (the setting of the paper's Table 2 and
 * Section 5.3) instead of only the s(s+1)/2 pairs with p + q <= s + 1. */
#define OZAKI_PAIRS_ALL 0x100

#define OZAKI_MAX_SLICES 32
#define OZAKI_MAX_K_BLOCK 32768

/*
 * ozaki_plan (host only, touches no GPU) -- the constants of Eq. 1-3 for one block length.
 *   k_block       length of the inner-product block the scheme is applied to (Section 4.3); >= 1
 *   slice_format  OZAKI_SLICE_*
 *   rho_out       HOST, may be NULL: rho = max(gamma, xi) of Eq. 3 with Type1 = FP64, Type3 = FP32
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
 *                 the slice pairs (p, q) with p + q <= s + 1 are multiplied (s(s+1)/2 products) and
 *                 accumulated anti-diagonal by anti-diagonal, least significant first; products of one
 *                 anti-diagonal that carry the same power-of-two scale for an element are summed exactly
 *                 before the (rounded) FP64 addition.
 *                 0 selects a data-independent default (ceil(61 / (b+1)) slices).  OR-ing OZAKI_PAIRS_ALL
 *                 into the value multiplies all s*s pairs (anti-diagonals 2s ... 2, same accumulation rule).
 *   k_block       inner-product-wise block length (Section 4.3); 0 means k (no blocking).  A last,
 *                 shorter block is allowed.  Must not exceed OZAKI_MAX_K_BLOCK elements.
 *   accum_mode    OZAKI_ACCUM_*
 * The slices, exponents and slice-pair products live in the workspace (ozaki_set_workspace).
 * Inputs must be finite; an Inf/NaN raises a device flag readable with ozaki_last_device_status
 * and leaves C unspecified.  Results whose exponent leaves the normal FP64 range are unspecified in
 * INT_EMU mode (the emulation omits overflow, underflow and subnormals, Section 4.2).
 */
int ozaki_dgemm(int64_t m, int64_t n, int64_t k,
                const double* A, int64_t lda, const double* B, int64_t ldb,
                double* C, int64_t ldc,
                int slice_format, int num_slices, int64_t k_block, int accum_mode);

/*
 * ozaki_dgemm_static -- ozaki_dgemm for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * the same bits in C as ozaki_dgemm, but the slices, exponents and slice-pair products live in a fixed array of
 * OZAKI_STATIC_SCRATCH_BYTES bytes that is part of the library's device code (every GPU the library runs on holds
 * one copy from the first call until the process ends); the workspace of ozaki_set_workspace is neither needed nor
 * touched, and the call allocates and frees nothing.
 *   Limit: ozaki_workspace_min_bytes(m, n, k, slice_format, num_slices, k_block) must not exceed
 *   OZAKI_STATIC_SCRATCH_BYTES, else OZAKI_STATUS_STATIC_LIMIT is returned and nothing is launched (for example
 *   m = n = k = 256 with 12 FP8 slices needs 5.6 MiB, m = n = 512, k = 2048 with 13 slices 49.1 MiB).
 *   Every call on a GPU uses that GPU's one array, which keeps what the previous call left: the kernels overwrite
 *   all they read, so nothing needs clearing between calls, but two calls that overlap in time on one GPU (two
 *   streams, two host threads) race on it and give undefined results.  Enqueued on the stream of ozaki_set_stream.
 *   An Inf/NaN input is reported by ozaki_last_device_status as for ozaki_dgemm.
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
 *   anything); with alpha == 1 and beta == 0 the call is ozaki_dgemm.  In OZAKI_ACCUM_FP64_INT_EMU mode the
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
 * they are blocked only as far as the library's OZAKI_MAX_K_BLOCK requires; FP16 gains a magnitude bit per factor 4
 * in the block length, and 4096 (b = 6) was the fastest block at k = 16384 (the paper reports the same optimum on
 * its GPU).  Returns the suggested k_block (0 = no blocking), or a negative argument index.  HOST call.
 */
int64_t ozaki_suggest_k_block(int64_t k, int slice_format);

/* Stream (a hipStream_t passed as void*; NULL = the null stream) used by all later calls. HOST call. */
int ozaki_set_stream(void* hip_stream);

/*
 * Workspace (Section 5.1: work memory is allocated once, outside the timed region).
 *   ozaki_workspace_bytes      size that lets ozaki_dgemm keep all s(s+1)/2 pair products of one block
 *                              resident (capped at 160 GiB of products; more pairs are then processed in
 *                              several passes).  0 if the arguments are invalid or infeasible.
 *   ozaki_workspace_min_bytes  smallest size ozaki_dgemm accepts (the s products of the longest anti-diagonal
 *                              resident at a time).
 *   ozaki_set_workspace        dev_ptr: DEVICE memory, 256-byte aligned, owned by the caller, must stay
 *                              valid until replaced; bytes: its size.  (NULL, 0) clears it.
 */
size_t ozaki_workspace_bytes(int64_t m, int64_t n, int64_t k, int slice_format, int num_slices, int64_t k_block);
size_t ozaki_workspace_min_bytes(int64_t m, int64_t n, int64_t k, int slice_format, int num_slices, int64_t k_block);
int ozaki_set_workspace(void* dev_ptr, size_t bytes);

/* Waits for the stream, then returns OZAKI_STATUS_NONFINITE if a kernel since the last call of this
 * function met an Inf/NaN input, OZAKI_STATUS_HIP_ERROR on a HIP failure, else 0. */
int ozaki_last_device_status(void);
/* Numeric hipError_t of the most recent failed HIP call (0 if none). */
int ozaki_last_hip_error(void);
/* Static, NUL-terminated description of a return value of this library. */
const char* ozaki_status_string(int status);

/*
 * Per-phase GPU time.  ozaki_profile_enable(1) makes ozaki_dgemm bracket its kernels with HIP events
 * on the library stream; ozaki_profile_read waits for the stream and returns, in HOST arrays of three
 * floats / three ints, the accumulated milliseconds and the number of kernel launches of the phases
 * [0] slicing (Eq. 4-8, includes the transposition of A), [1] slice-pair GEMMs (Eq. 10-11),
 * [2] accumulation and rescaling; then resets the counters.  ozaki_profile_enable(0) turns it off.
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
 *               r*kb_t + kk); 1 byte per entry (E4M3 code, or E2M3 code in the low six bits) or 2 bytes
 *               (binary16 bits).  Blocks are packed back to back (block t starts after s*rows*kb_u
 *               entries of every earlier block u).
 *   exps_out    DEVICE: int32 [T][s][rows], the exponents c of Eq. 4
 */
int ozaki_split(int is_B, int64_t rows, int64_t k, const double* X, int64_t ldx,
                int slice_format, int num_slices, int64_t k_block,
                void* slices_out, int32_t* exps_out);

/*
 * ozaki_count_slices -- how many slices Eq. 4-8 extract from an operand "until x^(p) = 0" (Section 3, the
 * paragraph before Eq. 4): the largest count over its vectors and k-blocks.  With that many slices (the larger
 * of the two operands' counts) and OZAKI_PAIRS_ALL the sum of the pair products is the exact product, which is
 * the error-free setting of the paper.
 *   is_B, rows, k, X, ldx, slice_format, k_block   as for ozaki_split
 *   count_out   HOST: the count; 0 for an all-zero operand; OZAKI_MAX_SLICES + 1 if OZAKI_MAX_SLICES slices do
 *               not exhaust it (ozaki_dgemm cannot run the error-free setting on it then)
 * Synchronises with the stream.  Workspace: 256 bytes, plus 8 * rows * k bytes (rounded up to 256) for A.
 */
int ozaki_count_slices(int is_B, int64_t rows, int64_t k, const double* X, int64_t ldx,
                       int slice_format, int64_t k_block, int* count_out);

/*
 * ozaki_pair_products -- the FP32 slice-pair products of Eq. 10-11, as the matrix unit produced them.
 *   P_out  DEVICE: float [T][pairs][n][m]: for block t and pair index z (pairs in accumulation order:
 *          anti-diagonals g = p+q from s+1 down to 2, p ascending within one), an m x n column-major
 *          matrix (leading dimension m) holding sum_kk sliceA_p(i,kk) * sliceB_q(kk,j), the slices
 *          being the values of Eq. 8 (for FP6 the matrix unit's result times the exact factor 1/4).
 */
int ozaki_pair_products(int64_t m, int64_t n, int64_t k,
                        const double* A, int64_t lda, const double* B, int64_t ldb,
                        int slice_format, int num_slices, int64_t k_block, float* P_out);

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
