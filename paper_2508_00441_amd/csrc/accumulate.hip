// Accumulation of the slice-pair products into FP64 and the final rescale (paper Section 3, Eq. 10 and the
// paragraph after Eq. 11; Section 4.2 for the integer-emulated variant; Section 4.3 for the block sum).
//
// For one k-block, element (i, j), the pairs (p, q) are visited least significant anti-diagonal first, p
// ascending inside one.  The term of a pair is P_pq(i,j) * 2^e with e = (cA_p(i) - cA_1(i)) + (cB_q(j) - cB_1(j)).
// Inside an anti-diagonal, consecutive pairs with the same e form a run.  A run is summed exactly (a 32-bit
// integer in units of 2^-2b: at most 32 products of at most 2^24 units each) and added to the block sum S with
// ONE rounded FP64 addition.  The GEMM kernel has already formed part of these sums in the matrix unit's
// accumulators, as far as the exact FP32 window of Eq. 11 reaches (groups of at most run_limit pairs) and where a
// whole tile shares the scale; the rest is merged here, element by element.  Then
//     C   = S * 2^(cA_1(i) + cB_1(j))            first block
//     C  += S * 2^(cA_1(i) + cB_1(j))            later blocks (one more FP64 addition)
// Scaling by a power of two commutes with rounding (inside the normal range), so summing with exponents
// relative to the first slice and rescaling once gives the same bits as scaling every term by
// 2^(cA_p + cB_q) as Eq. 10 writes it.  P_pq is the FP32 value left by the matrix unit; it already
// contains the factor 2^-2b of the two slice entries and is an exact integer multiple of 2^-2b.  (FP6 codes
// hold twice the slice value: the stored product is four times too large, an integer multiple of 2^-(2b-2); it
// is read as that integer and still weighted 2^-2b.)
//
// Two instantiations: hardware FP64 (int->double convert, ldexp, add -- no multiply) and integer-only
// (fp64_emu.hpp), which executes no FP64 instruction at all and returns the same bits.
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
    const float* P;          // [nz][tiles_n][tiles_m][TILE_ELEMS]
    double* S;               // [tiles_n][tiles_m][TILE_ELEMS] running block sum (may be null when unused)
    double* C;
    int64_t ldc;
    const int32_t* ea;       // exponents of the block: [s][rows_pad_a]
    const int32_t* eb;       // [s][rows_pad_b]
    int64_t rows_pad_a, rows_pad_b;
    int64_t m, n;
    int tiles_m, tiles_n;
    int two_b;               // 2b: a term is (stored product) * 2^(p_frac - two_b) * 2^e
    int p_frac;              // the stored products are integer multiples of 2^-p_frac (2b; 2b - 2 for FP6 codes)
    int read_S, write_S, add_to_C;
    int allow_chain;
    const int32_t* da;       // deltas of the block: [tiles_m][s]
    const int32_t* db;       // [tiles_n][s]
    PairOrder order;
    Pass pass;
};

template <bool EMU>
__global__ void __launch_bounds__(256) accumulate_kernel(const AccArgs a) {
    __shared__ int relA[MAX_SLICES][32];
    __shared__ int relB[MAX_SLICES][32];
    __shared__ uint32_t entries[MAX_PAIRS];           // stored runs of this tile: slot | p << 12 | q << 18 | first-of-diagonal << 24
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
    __syncthreads();

    const int ml = lane & 31;
    const int nl = g4 * 8 + (lane >> 5) * 4;
    const size_t tile_off = (size_t)tile * TILE_ELEMS + (size_t)pos * 1024 + (size_t)tid * 4;
    const size_t pair_stride = (size_t)a.tiles_m * a.tiles_n * TILE_ELEMS;

    typedef typename std::conditional<EMU, uint64_t, double>::type acc_t;
    acc_t S[4];
    if (a.read_S) {
#pragma unroll
        for (int r = 0; r < 4; ++r) S[r] = reinterpret_cast<const acc_t*>(a.S)[tile_off + r];
    } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) S[r] = 0;
    }

    // The stored runs of this tile, in accumulation order: a pair starts a run unless it is linked (for the whole
    // tile) to the pair before it inside its group.  Built by the first wave, one anti-diagonal at a time (an
    // anti-diagonal has at most 32 pairs).
    if (tid < 64) {
        const int32_t* dA = a.da + (size_t)tm * a.order.s;
        const int32_t* dB = a.db + (size_t)tn * a.order.s;
        int count = 0, slot0 = 0;
        for (int g = a.pass.g_hi; g >= a.pass.g_lo; --g) {
            const int len = diag_len(a.order, g);
            bool start = false;
            uint32_t entry = 0;
            if (tid < len) {
                const int p = diag_first_p(a.order, g) + tid - 1, q = g - p - 2;     // 0-based slice indices
                const bool first = tid == 0;                                        // first pair of the anti-diagonal: ends every run
                start = tid % a.order.run_limit == 0 || !(a.allow_chain && pair_linked(dA, dB, p - 1, q + 1));   // stored on its own
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

    // Integer-only variant: the sum lives in a RoundedSum, which adds exactly in 64-bit integers for as long as no
    // rounding can occur and with the emulated FP64 addition from then on.
    RoundedSum E[4];
    if constexpr (EMU) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (a.read_S) E[r].start_at((uint64_t)S[r]);
            else E[r].start_at_zero();
        }
    }
    auto add_run = [&](int r, int run_sum, int run_e) {
        if (run_sum == 0) return;                                     // adding an exact zero changes nothing
        if constexpr (EMU) {
            E[r].add(run_sum, run_e - a.two_b);
        } else {
            S[r] = (acc_t)((double)S[r] + ldexp((double)run_sum, run_e - a.two_b));
        }
    };
    // Per element, consecutive stored runs of one anti-diagonal with the same scale are merged further (32-bit
    // integer, units of 2^-p_frac) before the FP64 addition: together with the tile-wide runs formed by the GEMM
    // kernel this is the element-wise rule "consecutive pairs of an anti-diagonal with equal scale are summed exactly".
    int run_sum[4] = {0, 0, 0, 0}, run_e[4] = {0, 0, 0, 0};
    auto process = [&](uint32_t entry, const uint4& v) {
        const int p = (entry >> 12) & 63, q = (entry >> 18) & 63;
        const bool first = (entry >> 24) & 1;
        const int eA = p == 0 ? 0 : relA[p][ml];
        const uint32_t vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int e = eA + (q == 0 ? 0 : relB[q][nl + r]);
            // the product as an integer in units of 2^-p_frac: exact in FP32 (|integer| <= 2^24), no FP64 involved
            const int iv = (int)ldexpf(__uint_as_float(vv[r]), a.p_frac);
            if (!first && e == run_e[r]) {
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
    // four loads in flight per thread
    if (n_runs > 0) {
        uint4 v0 = load_run(0), v1 = load_run(1), v2 = load_run(2), v3 = load_run(3);
        for (int i = 0; i < n_runs; ++i) {
            const uint4 w = v0;
            v0 = v1; v1 = v2; v2 = v3;
            v3 = load_run(i + 4);
            process(entries[i], w);
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        add_run(r, run_sum[r], run_e[r]);
        if constexpr (EMU) S[r] = (acc_t)E[r].value();
    }

    if (a.write_S) {
#pragma unroll
        for (int r = 0; r < 4; ++r) reinterpret_cast<acc_t*>(a.S)[tile_off + r] = S[r];
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
        acc_t* dst = reinterpret_cast<acc_t*>(a.C) + mi + nj * a.ldc;
        if constexpr (EMU) {
            uint64_t v = fp64_scale_pow2_emulated((uint64_t)S[r], base);
            if (a.add_to_C) v = fp64_add_emulated((uint64_t)*dst, v);
            *dst = (acc_t)v;
        } else {
            double v = ldexp((double)S[r], base);
            if (a.add_to_C) v = (double)*dst + v;
            *dst = (acc_t)v;
        }
    }
}

__global__ void __launch_bounds__(256) export_products_kernel(const float* __restrict__ P, float* __restrict__ out, int64_t m,
                                                              int64_t n, int tiles_m, int tiles_n, float factor) {
    // one thread per stored float; grid.y = pair
    const size_t pair_stride = (size_t)tiles_m * tiles_n * TILE_ELEMS;
    const int64_t z = blockIdx.y;
    for (size_t g = (size_t)blockIdx.x * 256 + threadIdx.x; g < pair_stride; g += (size_t)gridDim.x * 256) {
        const int tile = (int)(g / TILE_ELEMS), idx = (int)(g % TILE_ELEMS);
        const int tn = tile / tiles_m, tm = tile - tn * tiles_m;
        int ml, nl;
        acc_order_to_mn(idx, ml, nl);
        const int64_t mi = (int64_t)tm * TILE + ml, nj = (int64_t)tn * TILE + nl;
        if (mi < m && nj < n) out[((size_t)z * n + nj) * m + mi] = P[(size_t)z * pair_stride + g] * factor;   // power of two: exact
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
                             bool first_pass, bool last_pass, int64_t t, const float* P, double* S_io,
                             double* C, int64_t ldc, int accum_mode, hipStream_t st) {
    if (pl.tiles_m == 0 || pl.tiles_n == 0) return hipSuccess;
    AccArgs a;
    a.P = P; a.S = S_io; a.C = C; a.ldc = ldc;
    a.ea = A.exps + (size_t)t * pl.s * A.rows_pad;
    a.eb = B.exps + (size_t)t * pl.s * B.rows_pad;
    a.rows_pad_a = A.rows_pad; a.rows_pad_b = B.rows_pad;
    a.m = pl.m; a.n = pl.n; a.tiles_m = (int)pl.tiles_m; a.tiles_n = (int)pl.tiles_n;
    a.two_b = 2 * pl.b;
    a.p_frac = pl.p_frac;
    a.allow_chain = 1;
    a.da = A.deltas + (size_t)t * pl.tiles_m * pl.s;
    a.db = B.deltas + (size_t)t * pl.tiles_n * pl.s;
    a.order = order; a.pass = ps;
    a.read_S = !first_pass;
    a.write_S = !last_pass;
    a.add_to_C = t > 0;
    const int64_t blocks = pl.tiles_m * pl.tiles_n * 64;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    if (accum_mode == 1) hipLaunchKernelGGL((accumulate_kernel<true>), dim3((unsigned)blocks), dim3(256), 0, st, a);
    else hipLaunchKernelGGL((accumulate_kernel<false>), dim3((unsigned)blocks), dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_export_products(const Plan& pl, int nz, const float* P, float* out, hipStream_t st) {
    if (nz <= 0 || pl.m == 0 || pl.n == 0) return hipSuccess;
    dim3 grid(grid_for(pl.tiles_m * pl.tiles_n * (int64_t)TILE_ELEMS), (unsigned)nz);
    const float factor = ldexpf(1.0f, pl.p_frac - 2 * pl.b);
    hipLaunchKernelGGL(export_products_kernel, grid, dim3(256), 0, st, P, out, pl.m, pl.n, (int)pl.tiles_m, (int)pl.tiles_n, factor);
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
