// Accumulation of the slice-pair products into FP64 and the final rescale (paper Section 3, Eq. 10 and the
// paragraph after Eq. 11; Section 4.2 for the integer-only variants; Section 4.3 for the block sum).
//
// For one k-block, element (i, j), the pairs (p, q) are visited least significant anti-diagonal first, p
// ascending inside one.  The term of a pair is P_pq(i,j) * 2^e with e = (cA_p(i) - cA_1(i)) + (cB_q(j) - cB_1(j)).
// Rule "runs": inside an anti-diagonal, consecutive pairs with the same e form a run.  A run is summed exactly (an
// integer in units of 2^-2b: at most 32 products of at most 2^24, or 2^31 for INT8 slices, units each) and added to
// the block sum S with ONE rounded FP64 addition.  The GEMM kernel has already formed part of these sums in the
// matrix unit's accumulators, as far as the exact window of Eq. 11 reaches (groups of at most run_limit pairs) and
// where a whole 32 x 32 tile shares the scale; the rest is merged here, element by element.  Rule "plain": every
// product is added with its own rounded addition (the GEMM kernel then stores every pair on its own).  Then
//     C   = S * 2^(cA_1(i) + cB_1(j))            first block
//     C  += S * 2^(cA_1(i) + cB_1(j))            later blocks (one more FP64 addition)
// Scaling by a power of two commutes with rounding (inside the normal range), so summing with exponents
// relative to the first slice and rescaling once gives the same bits as scaling every term by
// 2^(cA_p + cB_q) as Eq. 10 writes it.  P_pq is the FP32 value left by the matrix unit; it already
// contains the factor 2^-2b of the two slice entries and is an exact integer multiple of 2^-2b.  (FP6 codes
// hold twice the slice value: the stored product is four times too large, an integer multiple of 2^-(2b-2); it
// is read as that integer and still weighted 2^-2b.  INT8 slices leave the INT32 integer itself.)
//
// Three instantiations of the sum: hardware FP64 (int->double convert, ldexp, add -- no multiply); integer-emulated
// FP64 (fp64_emu.hpp), which executes no FP64 instruction at all and returns the same bits; and the exact mode, a
// 192-bit fixed-point integer per element that takes every run without rounding and is rounded once at the end
// (integer-only as well).
//
// One workgroup handles one 32 x 32 MFMA tile position of a 256 x 256 tile (256 threads x 4 consecutive
// columns of C each), reading the products in the order the GEMM kernel stored them.
#include <string.h>

#include <type_traits>

#include "fp64_emu.hpp"
#include "layout.hpp"

namespace ozaki {

namespace {

struct AccArgs {
    const float* P;          // [nz][tiles_n][tiles_m][TILE_ELEMS] FP32 (or INT32) words
    uint64_t* S;             // running block sum, word w of an element at S[w * plane + element] (may be null when unused)
    double* C;
    int64_t ldc;
    const int32_t* ea;       // exponents of the block: [s][rows_pad_a]
    const int32_t* eb;       // [s][rows_pad_b]
    int64_t rows_pad_a, rows_pad_b;
    int64_t m, n;
    int tiles_m, tiles_n;
    int two_b;               // 2b: a term is (stored product) * 2^(p_frac - two_b) * 2^e
    int p_frac;              // the stored products are integer multiples of 2^-p_frac (2b; 2b - 2 for FP6 codes; 0 for INT32)
    int read_S, write_S, add_to_C;
    int allow_chain;         // the GEMM kernel summed tile-wide runs
    int merge;               // rule "runs": merge equal-scale products of an anti-diagonal element by element
    const int32_t* da;       // deltas of the block: [s][rows_pad_a / 32]
    const int32_t* db;       // [s][rows_pad_b / 32]
    PairOrder order;
    Pass pass;
};

// Is pair `pos` of anti-diagonal g (0-based position) stored on its own, i.e. does it start a run of the GEMM kernel?
// dA / dB: the block's deltas advanced to the group of the 32 rows / 32 columns concerned, ga / gb: groups per slice;
// p, q 0-based slice indices of the pair.
__device__ __forceinline__ bool starts_run(const PairOrder& o, int allow_chain, const int32_t* dA, int64_t ga, const int32_t* dB,
                                           int64_t gb, int pos, int p, int q) {
    return pos % o.run_limit == 0 || !(allow_chain && pair_linked(dA, ga, dB, gb, p - 1, q + 1));
}

template <int MODE, bool PINT>
__global__ void __launch_bounds__(256) accumulate_kernel(const AccArgs a) {
    constexpr bool HW = MODE == ACC_HW, EMU = MODE == ACC_EMU, EXACT = MODE == ACC_EXACT;
    typedef typename std::conditional<PINT, int64_t, int>::type run_t;      // exact sum of a run
    __shared__ int relA[MAX_SLICES][32];
    __shared__ int relB[MAX_SLICES][32];
    __shared__ uint32_t entries[MAX_PAIRS];           // stored runs of this tile: slot | p << 12 | q << 18 | first-of-diagonal << 24
    __shared__ int32_t linkA[MAX_SLICES], linkB[MAX_SLICES];      // deltas of the 32 rows / 32 columns, per slice
    __shared__ int n_entries;

    const int tid = threadIdx.x;
    const int lane = tid & 63, g4 = tid >> 6;
    const int pos = blockIdx.x & 63;                  // wave*16 + sub
    const int tile = blockIdx.x >> 6;
    const int tn = tile / a.tiles_m, tm = tile - tn * a.tiles_m;
    const int wave = pos >> 4, sub = pos & 15;
    const int wn = wave >> 1, wm = wave & 1, ti = sub >> 2, tj = sub & 3;
    const int64_t m0 = (int64_t)tm * TILE + wm * 128 + tj * 32;       // first row of C of this 32 x 32 position
    const int64_t n0 = (int64_t)tn * TILE + wn * 128 + ti * 32;       // first column

    // exponents of the 32 rows and 32 columns: slot 0 keeps the first-slice exponent, slots p >= 1 the difference to it
    for (int idx = tid; idx < a.order.s * 32; idx += 256) {
        const int p = idx >> 5, r = idx & 31;
        const int ca = a.ea[(int64_t)p * a.rows_pad_a + m0 + r], ca1 = a.ea[m0 + r];
        const int cb = a.eb[(int64_t)p * a.rows_pad_b + n0 + r], cb1 = a.eb[n0 + r];
        relA[p][r] = p == 0 ? ca1 : ca - ca1;
        relB[p][r] = p == 0 ? cb1 : cb - cb1;
    }
    // the deltas that decide where the GEMM kernel ended its runs at this position: fetched once, all at the same time
    if (tid < a.order.s) linkA[tid] = a.da[(int64_t)tid * (a.rows_pad_a / LINK_ROWS) + m0 / LINK_ROWS];
    else if (tid >= 64 && tid - 64 < a.order.s) linkB[tid - 64] = a.db[(int64_t)(tid - 64) * (a.rows_pad_b / LINK_ROWS) + n0 / LINK_ROWS];
    __syncthreads();

    const int ml = lane & 31;
    const int nl = g4 * 8 + (lane >> 5) * 4;
    const size_t tile_off = (size_t)tile * TILE_ELEMS + (size_t)pos * 1024 + (size_t)tid * 4;
    const size_t pair_stride = (size_t)a.tiles_m * a.tiles_n * TILE_ELEMS;

    // the block sum of this thread's four elements, in the representation of the mode
    double Sd[4];                                     // HW
    RoundedSum E[4];                                  // EMU: x * 2^ex with an integer significand of at most 53 bits
    Fixed192 X[4];                                    // EXACT
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        if constexpr (HW) Sd[r] = a.read_S ? __longlong_as_double((long long)a.S[tile_off + r]) : 0.0;
        if constexpr (EMU) {
            if (a.read_S) E[r].start_at(a.S[tile_off + r]);
            else E[r].start_at_zero();
        }
        if constexpr (EXACT) {
            if (a.read_S) {
                X[r].w0 = a.S[tile_off + r];
                X[r].w1 = a.S[pair_stride + tile_off + r];
                X[r].w2 = a.S[2 * pair_stride + tile_off + r];
            } else {
                X[r].clear();
            }
        }
    }

    // The stored runs of this 32 x 32 position, in accumulation order: a pair starts a run unless it is linked (for
    // the whole position) to the pair before it inside its group.  Built by the first wave, one anti-diagonal at a time
    // (an anti-diagonal has at most 32 pairs).
    if (tid < 64) {
        int count = 0, slot0 = 0;
        for (int g = a.pass.g_hi; g >= a.pass.g_lo; --g) {
            const int len = diag_len(a.order, g);
            bool start = false;
            uint32_t entry = 0;
            if (tid < len) {
                const int p = diag_first_p(a.order, g) + tid - 1, q = g - p - 2;     // 0-based slice indices
                const bool first = tid == 0;                                        // first pair of the anti-diagonal: ends every run
                start = starts_run(a.order, a.allow_chain, linkA, 1, linkB, 1, tid, p, q);      // stored on its own
                entry = (uint32_t)(slot0 + tid) | ((uint32_t)p << 12) | ((uint32_t)q << 18) | ((uint32_t)first << 24);
            }
            const unsigned long long mask = __ballot(start);
            if (start) entries[count + __popcll(mask & ((1ull << tid) - 1ull))] = entry;
            count += __popcll(mask);
            slot0 += len;
        }
        if (tid == 0) n_entries = count;
    }
    __syncthreads();
    const int n_runs = n_entries;

    auto add_run = [&](int r, run_t run_sum, int run_e) {
        if (run_sum == 0) return;                                     // adding an exact zero changes nothing
        if constexpr (HW) Sd[r] = Sd[r] + ldexp((double)run_sum, run_e - a.two_b);
        if constexpr (EMU) E[r].add(run_sum, run_e - a.two_b);
        if constexpr (EXACT) X[r].add((int64_t)run_sum, EXACT_WINDOW_BITS + run_e);      // unit: 2^(-2b - window) of the leading scale
    };
    // Per element, consecutive stored runs of one anti-diagonal with the same scale are merged further (integer,
    // units of 2^-p_frac) before the FP64 addition: together with the tile-wide runs formed by the GEMM
    // kernel this is the element-wise rule "consecutive pairs of an anti-diagonal with equal scale are summed exactly".
    run_t run_sum[4] = {0, 0, 0, 0};
    int run_e[4] = {0, 0, 0, 0};
    auto process = [&](uint32_t entry, const uint4& v) {
        const int p = (entry >> 12) & 63, q = (entry >> 18) & 63;
        const bool first = (entry >> 24) & 1;
        const int eA = p == 0 ? 0 : relA[p][ml];
        const uint32_t vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int e = eA + (q == 0 ? 0 : relB[q][nl + r]);
            // the product as an integer in units of 2^-p_frac: exact in FP32 (|integer| <= 2^24), no FP64 involved
            const int iv = PINT ? (int)vv[r] : (int)ldexpf(__uint_as_float(vv[r]), a.p_frac);
            if (a.merge && !first && e == run_e[r]) {
                run_sum[r] += iv;
            } else {
                add_run(r, run_sum[r], run_e[r]);
                run_sum[r] = iv;
                run_e[r] = e;
            }
        }
    };
    auto load_run = [&](int i) -> uint4 {
        const uint32_t entry = entries[i < n_runs ? i : n_runs - 1];
        return *reinterpret_cast<const uint4*>(a.P + (size_t)(entry & 0xFFFu) * pair_stride + tile_off);
    };
    // four loads in flight per thread; the loop is unrolled by four so that each load keeps its registers
    if (n_runs > 0) {
        uint4 v0 = load_run(0), v1 = load_run(1), v2 = load_run(2), v3 = load_run(3);
        int i = 0;
        for (; i + 4 <= n_runs; i += 4) {
            const uint4 w0 = v0;
            v0 = load_run(i + 4);
            process(entries[i], w0);
            const uint4 w1 = v1;
            v1 = load_run(i + 5);
            process(entries[i + 1], w1);
            const uint4 w2 = v2;
            v2 = load_run(i + 6);
            process(entries[i + 2], w2);
            const uint4 w3 = v3;
            v3 = load_run(i + 7);
            process(entries[i + 3], w3);
        }
        if (i < n_runs) process(entries[i], v0);
        if (i + 1 < n_runs) process(entries[i + 1], v1);
        if (i + 2 < n_runs) process(entries[i + 2], v2);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) add_run(r, run_sum[r], run_e[r]);

    if (a.write_S) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if constexpr (HW) a.S[tile_off + r] = (uint64_t)__double_as_longlong(Sd[r]);
            if constexpr (EMU) a.S[tile_off + r] = E[r].value();
            if constexpr (EXACT) {
                a.S[tile_off + r] = X[r].w0;
                a.S[pair_stride + tile_off + r] = X[r].w1;
                a.S[2 * pair_stride + tile_off + r] = X[r].w2;
            }
        }
        return;
    }
    const int64_t mi = m0 + ml;
    if (mi >= a.m) return;
    const int baseA = relA[0][ml];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t nj = n0 + nl + r;
        if (nj >= a.n) continue;
        const int base = baseA + relB[0][nl + r];
        if constexpr (HW) {
            double* dst = a.C + mi + nj * a.ldc;
            double v = ldexp(Sd[r], base);
            if (a.add_to_C) v = *dst + v;
            *dst = v;
        } else {
            uint64_t* dst = reinterpret_cast<uint64_t*>(a.C) + mi + nj * a.ldc;
            uint64_t v;
            if constexpr (EMU) v = fp64_scale_pow2_emulated(E[r].value(), base);
            else v = X[r].round_to_fp64(base - a.two_b - EXACT_WINDOW_BITS);
            if (a.add_to_C) v = fp64_add_emulated(*dst, v);
            *dst = v;
        }
    }
}

// Verification export: one thread per stored word; grid.y = pair slot of the pass.  Writes the plain column-major
// matrices and, if asked, the number of pairs each slot sums for the element (see launch_export_products).
struct ExportArgs {
    const float* P;
    float* out;
    uint8_t* run_len;
    int64_t m, n;
    int tiles_m, tiles_n;
    float factor;            // FP32 products: the exact power of two that undoes the FP6 code scaling
    int p_is_int;
    int allow_chain;
    const int32_t* da;
    const int32_t* db;
    int64_t ga, gb;          // groups of 32 vectors per slice in da / db
    PairOrder order;
    Pass pass;
};
__global__ void __launch_bounds__(256) export_products_kernel(const ExportArgs a) {
    const size_t pair_stride = (size_t)a.tiles_m * a.tiles_n * TILE_ELEMS;
    const int z = blockIdx.y;
    // the pair of slot z: anti-diagonal g, position pos in it
    int g = a.pass.g_hi, pos = z;
    for (; g > a.pass.g_lo && pos >= diag_len(a.order, g); --g) pos -= diag_len(a.order, g);
    const int len = diag_len(a.order, g);
    const int p = diag_first_p(a.order, g) + pos - 1, q = g - p - 2;      // 0-based slice indices
    for (size_t gi = (size_t)blockIdx.x * 256 + threadIdx.x; gi < pair_stride; gi += (size_t)gridDim.x * 256) {
        const int tile = (int)(gi / TILE_ELEMS), idx = (int)(gi % TILE_ELEMS);
        const int tn = tile / a.tiles_m, tm = tile - tn * a.tiles_m;
        int ml, nl;
        acc_order_to_mn(idx, ml, nl);
        const int64_t mi = (int64_t)tm * TILE + ml, nj = (int64_t)tn * TILE + nl;
        if (mi >= a.m || nj >= a.n) continue;
        const int32_t* dA = a.da + mi / LINK_ROWS;
        const int32_t* dB = a.db + nj / LINK_ROWS;
        int run = 0;
        if (starts_run(a.order, a.allow_chain, dA, a.ga, dB, a.gb, pos, p, q)) {
            run = 1;
            while (pos + run < len && !starts_run(a.order, a.allow_chain, dA, a.ga, dB, a.gb, pos + run, p + run, q - run)) ++run;
        }
        const size_t o = ((size_t)z * a.n + nj) * a.m + mi;
        const uint32_t w = reinterpret_cast<const uint32_t*>(a.P)[(size_t)z * pair_stride + gi];
        uint32_t* const dst = reinterpret_cast<uint32_t*>(a.out) + o;
        if (run == 0) *dst = 0u;                                                // all-zero bits either way
        else if (a.p_is_int) *dst = w;                                          // the INT32 word, bit for bit
        else *dst = __float_as_uint(__uint_as_float(w) * a.factor);             // power of two: exact
        if (a.run_len) a.run_len[o] = (uint8_t)run;
    }
}

__global__ void __launch_bounds__(256) add_emulated_kernel(const uint64_t* a, const uint64_t* b, uint64_t* out, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
        out[i] = fp64_add_emulated(a[i], b[i]);
}

// C = fl(fl(alpha * W) + fl(beta * C)), or C = fl(alpha * W) without reading C when use_beta == 0: the scaling
// around the product, with the FP64 multiplication and addition in hardware or emulated (Section 4.2).
template <bool EMU>
__global__ void __launch_bounds__(256) axpby_kernel(uint64_t alpha, uint64_t beta, int use_beta, const uint64_t* __restrict__ W,
                                                    int64_t ldw, uint64_t* C, int64_t ldc, int64_t m, int64_t n) {
    const int64_t total = m * n;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
        const int64_t i = idx % m, j = idx / m;
        const uint64_t w = W[i + j * ldw];
        uint64_t* dst = C + i + j * ldc;
        if constexpr (EMU) {
            uint64_t t = fp64_mul_emulated(alpha, w);
            if (use_beta) t = fp64_add_emulated(t, fp64_mul_emulated(beta, *dst));
            *dst = t;
        } else {
            double t = __dmul_rn(__longlong_as_double((long long)alpha), __longlong_as_double((long long)w));
            if (use_beta) t = __dadd_rn(t, __dmul_rn(__longlong_as_double((long long)beta), __longlong_as_double((long long)*dst)));
            *dst = (uint64_t)__double_as_longlong(t);
        }
    }
}

__global__ void __launch_bounds__(256) fill_zero_kernel(uint64_t* C, int64_t ldc, int64_t m, int64_t n) {
    const int64_t total = m * n;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256)
        C[(i % m) + (i / m) * ldc] = 0;
}

unsigned grid_for(int64_t work_items) {
    int64_t blocks = (work_items + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 65536) blocks = 65536;
    return (unsigned)blocks;
}

}  // namespace

hipError_t launch_accumulate(const Plan& pl, const Operand& A, const Operand& B, const PairOrder& order, const Pass& ps,
                             bool first_pass, bool last_pass, int64_t t, const float* P, uint64_t* S_io,
                             double* C, int64_t ldc, int accum_mode, int sum_rule, bool chained, hipStream_t st) {
    if (pl.tiles_m == 0 || pl.tiles_n == 0) return hipSuccess;
    AccArgs a;
    a.P = P; a.S = S_io; a.C = C; a.ldc = ldc;
    a.ea = A.exps + (size_t)t * pl.s * A.rows_pad;
    a.eb = B.exps + (size_t)t * pl.s * B.rows_pad;
    a.rows_pad_a = A.rows_pad; a.rows_pad_b = B.rows_pad;
    a.m = pl.m; a.n = pl.n; a.tiles_m = (int)pl.tiles_m; a.tiles_n = (int)pl.tiles_n;
    a.two_b = 2 * pl.b;
    a.p_frac = pl.p_frac;
    a.allow_chain = chained ? 1 : 0;
    a.merge = (sum_rule == SUM_RUNS || accum_mode == ACC_EXACT) ? 1 : 0;
    a.da = A.deltas + (size_t)t * (A.rows_pad / LINK_ROWS) * pl.s;
    a.db = B.deltas + (size_t)t * (B.rows_pad / LINK_ROWS) * pl.s;
    a.order = order; a.pass = ps;
    a.read_S = !first_pass;
    a.write_S = !last_pass;
    a.add_to_C = t > 0;
    const int64_t blocks = pl.tiles_m * pl.tiles_n * 64;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks), block(256);
    if (pl.p_is_int) {
        if (accum_mode == ACC_EXACT) hipLaunchKernelGGL((accumulate_kernel<ACC_EXACT, true>), grid, block, 0, st, a);
        else if (accum_mode == ACC_EMU) hipLaunchKernelGGL((accumulate_kernel<ACC_EMU, true>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((accumulate_kernel<ACC_HW, true>), grid, block, 0, st, a);
    } else {
        if (accum_mode == ACC_EXACT) hipLaunchKernelGGL((accumulate_kernel<ACC_EXACT, false>), grid, block, 0, st, a);
        else if (accum_mode == ACC_EMU) hipLaunchKernelGGL((accumulate_kernel<ACC_EMU, false>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((accumulate_kernel<ACC_HW, false>), grid, block, 0, st, a);
    }
    return hipGetLastError();
}

hipError_t launch_export_products(const Plan& pl, const Operand& A, const Operand& B, const PairOrder& order, const Pass& ps,
                                  bool chained, int64_t t, const float* P, float* out, uint8_t* run_len_out, hipStream_t st) {
    if (ps.npairs <= 0 || pl.m == 0 || pl.n == 0) return hipSuccess;
    ExportArgs a;
    a.P = P; a.out = out; a.run_len = run_len_out;
    a.m = pl.m; a.n = pl.n; a.tiles_m = (int)pl.tiles_m; a.tiles_n = (int)pl.tiles_n;
    a.factor = ldexpf(1.0f, pl.p_is_int ? 0 : pl.p_frac - 2 * pl.b);
    a.p_is_int = pl.p_is_int;
    a.allow_chain = chained ? 1 : 0;
    a.da = A.deltas + (size_t)t * (A.rows_pad / LINK_ROWS) * pl.s;
    a.db = B.deltas + (size_t)t * (B.rows_pad / LINK_ROWS) * pl.s;
    a.ga = A.rows_pad / LINK_ROWS; a.gb = B.rows_pad / LINK_ROWS;
    a.order = order; a.pass = ps;
    dim3 grid(grid_for(pl.tiles_m * pl.tiles_n * (int64_t)TILE_ELEMS), (unsigned)ps.npairs);
    hipLaunchKernelGGL(export_products_kernel, grid, dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_add_emulated(const double* a, const double* b, double* out, int64_t n, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(add_emulated_kernel, dim3(grid_for(n)), dim3(256), 0, st, reinterpret_cast<const uint64_t*>(a),
                       reinterpret_cast<const uint64_t*>(b), reinterpret_cast<uint64_t*>(out), n);
    return hipGetLastError();
}

hipError_t launch_axpby(double alpha, double beta, const double* W, int64_t ldw, double* C, int64_t ldc, int64_t m, int64_t n,
                        int accum_mode, hipStream_t st) {
    if (m <= 0 || n <= 0) return hipSuccess;
    uint64_t ab, bb;
    memcpy(&ab, &alpha, 8);
    memcpy(&bb, &beta, 8);
    const int use_beta = beta != 0.0;
    if (accum_mode == 1)
        hipLaunchKernelGGL((axpby_kernel<true>), dim3(grid_for(m * n)), dim3(256), 0, st, ab, bb, use_beta,
                           reinterpret_cast<const uint64_t*>(W), ldw, reinterpret_cast<uint64_t*>(C), ldc, m, n);
    else
        hipLaunchKernelGGL((axpby_kernel<false>), dim3(grid_for(m * n)), dim3(256), 0, st, ab, bb, use_beta,
                           reinterpret_cast<const uint64_t*>(W), ldw, reinterpret_cast<uint64_t*>(C), ldc, m, n);
    return hipGetLastError();
}

hipError_t launch_fill_zero_f64(double* C, int64_t ldc, int64_t m, int64_t n, hipStream_t st) {
    if (m <= 0 || n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_zero_kernel, dim3(grid_for(m * n)), dim3(256), 0, st, reinterpret_cast<uint64_t*>(C), ldc, m, n);
    return hipGetLastError();
}

}  // namespace ozaki
